// Pull side of the hash bitmap (section "Hash Bitmap", Algorithm 2).
//
//   server:  hash_bitmap_encode of what the server aggregated.  The aggregated indices ascend and so
//            does the partition's domain II_p, so membership is a merge of two sorted lists: a block
//            takes 8,192 consecutive domain rows, finds the matching slice of the index list with a
//            wave-wide 64-ary search, keeps the slice in LDS and turns ballots into bitmap words.
//            Every word of the partition is written with a plain store: no zero fill, no atomics, no
//            per-row rank table.  The values need no work at all: ascending indices = ascending
//            domain positions = bit order.
//   worker:  hash_bitmap_decode of every server's bitmap and placement of the values in a dense
//            tensor (the outcome of synchronization, section "Elemental Dimensions for
//            Synchronization"): zero fill, per-chunk popcounts, scan, then every set bit j of
//            partition p with running number k puts values[p][k] at row II_p[j].
#include <stdlib.h>
#include <string.h>
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int PULL_THREADS = 256;
static constexpr uint32_t PULL_CHUNK_WORDS = 256;                     // bitmap words per block
static constexpr uint32_t PULL_CHUNK_BITS = PULL_CHUNK_WORDS * 32;    // domain rows per block
static constexpr uint32_t PULL_TILE_ROWS = 8192;                      // element-level placement: rows per block

// One launch group: partitions first_part .. first_part + n - 1, entry i = partition first_part + i.
struct PullSrc {
    const uint32_t *indices[ZEN_MAX_BATCH];
    const uint32_t *bitmap[ZEN_MAX_BATCH];   // first word of the partition
    const float *values[ZEN_MAX_BATCH];
    const uint32_t *count[ZEN_MAX_BATCH];
    uint32_t n, first_part;
};

// Word k of a partition's bitmap with the padding bits of the last word forced to 0, so that a
// malformed bitmap can never name a row outside the domain.
__device__ __forceinline__ uint32_t domain_word(const uint32_t *__restrict__ bm, uint32_t k, uint32_t n_dom)
{
    const uint32_t n_words = (n_dom + 31) >> 5;
    if (!bm || k >= n_words) return 0u;
    uint32_t w = bm[k];
    if (k == n_words - 1 && (n_dom & 31u)) w &= (1u << (n_dom & 31u)) - 1u;
    return w;
}

// First position in the ascending list a[0..n) whose element is >= key (n if none).  Called by all
// 64 lanes of a wave with the same arguments; every step probes 64 evenly spaced elements, so a list
// of 2^24 entries needs four dependent loads instead of twenty-four.
__device__ __forceinline__ uint32_t wave_lower_bound(const uint32_t *__restrict__ a, uint32_t n, uint32_t key)
{
    const uint32_t lane = lane_id();
    uint32_t lo = 0, hi = n;   // the answer lies in [lo, hi]
    while (hi - lo > ZEN_WAVE) {
        const uint32_t step = (hi - lo + ZEN_WAVE - 1) / ZEN_WAVE;
        const uint64_t i = (uint64_t)lo + (uint64_t)lane * step;
        const bool ge = i >= hi || a[i] >= key;
        const uint64_t m = ballot(ge);
        const uint32_t f = m ? (uint32_t)__ffsll((unsigned long long)m) - 1u : (uint32_t)ZEN_WAVE;
        if (f == 0) return lo;
        const uint64_t nh = (uint64_t)lo + (uint64_t)f * step;
        const uint32_t new_lo = lo + (f - 1) * step + 1;
        hi = nh < hi ? (uint32_t)nh : hi;
        lo = new_lo;
    }
    const uint32_t i = lo + lane;
    const bool ge = i >= hi || a[i] >= key;
    const uint64_t m = ballot(ge);
    const uint32_t f = m ? (uint32_t)__ffsll((unsigned long long)m) - 1u : (uint32_t)ZEN_WAVE;
    return lo + f < hi ? lo + f : hi;
}

// ------------------------------------------------------------------------------------------------
// Server side: bitmap words of partition p from its ascending aggregated indices.
// grid = (chunks, servers).  Flag 4 is raised for input that is not an ascending list of distinct
// rows of II_p (a row of another partition, a duplicate, an index out of order).
// ------------------------------------------------------------------------------------------------
// bounds[server][c] = first index of the list that is not below the first domain row of chunk c
// (c = 0: 0; c = number of chunks: the list's length), found by one wave per (chunk, server).
__global__ void __launch_bounds__(PULL_THREADS)
pull_bounds_kernel(PullSrc a, Arr64<uint64_t> cap_rows, const uint32_t *domain, const uint32_t *dom_offsets,
                   uint32_t *bounds, uint32_t n_chunks)
{
    const uint32_t wave_id = blockIdx.x * (PULL_THREADS / ZEN_WAVE) + (threadIdx.x >> 6);
    const uint32_t server = blockIdx.y, p = a.first_part + server;
    if (wave_id > n_chunks) return;
    uint32_t cnt = *a.count[server];
    if ((uint64_t)cnt > cap_rows.v[server]) cnt = (uint32_t)cap_rows.v[server];
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    const uint32_t active = (n_words + PULL_CHUNK_WORDS - 1) / PULL_CHUNK_WORDS;
    uint32_t k;
    if (wave_id == 0) k = 0;
    else if (wave_id >= active) k = cnt;
    else k = wave_lower_bound(a.indices[server], cnt, domain[d0 + wave_id * PULL_CHUNK_BITS]);
    if (lane_id() == 0) bounds[(uint64_t)server * (n_chunks + 1) + wave_id] = k;
}

__global__ void __launch_bounds__(PULL_THREADS)
pull_encode_kernel(PullSrc a, Arr64<uint64_t> cap_rows, Arr64<uint32_t *> out_words, const uint32_t *domain,
                   const uint32_t *dom_offsets, const uint32_t *bounds, uint32_t n_chunks, zen_status_info *status)
{
    __shared__ uint32_t s_idx[PULL_CHUNK_BITS];
    __shared__ uint32_t s_dom[PULL_CHUNK_BITS + PULL_CHUNK_WORDS];   // entry e at e + e/32: a thread's 32 entries
    __shared__ uint32_t s_found;                                     // start in 32 different banks
    const uint32_t chunk = blockIdx.x, server = blockIdx.y, p = a.first_part + server;
    const uint32_t lane = lane_id();
    const uint32_t *__restrict__ idx = a.indices[server];
    uint32_t cnt = *a.count[server];
    if ((uint64_t)cnt > cap_rows.v[server]) cnt = (uint32_t)cap_rows.v[server];
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    const uint32_t active = (n_words + PULL_CHUNK_WORDS - 1) / PULL_CHUNK_WORDS;
    if (chunk >= active) {   // nothing to write; an empty domain cannot hold indices
        if (chunk == 0 && cnt != 0 && threadIdx.x == 0) atomicOr(&status->flags, 4u);
        return;
    }
    // The chunk's slice of the list: everything from this chunk's first row up to the next chunk's.
    // An index that is no row of the domain lands in some slice and is noticed there as unmatched.
    const uint32_t k0 = bounds[(uint64_t)server * (n_chunks + 1) + chunk];
    const uint32_t k1 = min(cnt, bounds[(uint64_t)server * (n_chunks + 1) + chunk + 1]);
    const uint32_t *__restrict__ dom = domain + d0;
    const uint32_t j0 = chunk * PULL_CHUNK_BITS, j1 = min(j0 + PULL_CHUNK_BITS, n_dom);
    const bool bad = k1 < k0 || k1 - k0 > PULL_CHUNK_BITS;   // out of order / more indices than domain rows
    const uint32_t m_all = k1 < k0 ? 0u : k1 - k0;
    const uint32_t m = min(m_all, PULL_CHUNK_BITS);
    // Both lists go to LDS; loads are issued in batches of 16 per list so that 32 are in flight per thread.
    const uint32_t n_here_all = j1 - j0;
    for (uint32_t t0 = 0; t0 < PULL_CHUNK_BITS / PULL_THREADS; t0 += 16) {
        uint32_t rd[16], ri[16];
#pragma unroll
        for (uint32_t u = 0; u < 16; ++u) {
            const uint32_t e = (t0 + u) * PULL_THREADS + threadIdx.x;
            rd[u] = e < n_here_all ? dom[j0 + e] : 0u;
            ri[u] = e < m ? idx[k0 + e] : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < 16; ++u) {
            const uint32_t e = (t0 + u) * PULL_THREADS + threadIdx.x;
            if (e < n_here_all) s_dom[e + (e >> 5)] = rd[u];
            if (e < m) s_idx[e] = ri[u];
        }
    }
    if (threadIdx.x == 0) s_found = 0;
    __syncthreads();
    // One bitmap word per thread: locate the word's first row in the slice, then merge 32 rows.
    const uint32_t e0 = threadIdx.x * 32, word = (j0 >> 5) + threadIdx.x;
    uint32_t bits = 0;
    if (j0 + e0 < j1) {
        const uint32_t n_here = min(32u, j1 - j0 - e0);
        const uint32_t *rows = s_dom + e0 + threadIdx.x;
        const uint32_t first = rows[0];
        uint32_t pos = 0;   // number of slice entries below the word's first row
#pragma unroll
        for (uint32_t step = PULL_CHUNK_BITS / 2; step; step >>= 1) {
            const uint32_t q = pos + step;
            if (q <= m && s_idx[q - 1] < first) pos = q;
        }
        if (pos < m && s_idx[pos] < first) ++pos;   // a full slice (m = 8,192) needs one more step
        for (uint32_t b = 0; b < n_here && pos < m; ++b) {
            const uint32_t row = rows[b];
            uint32_t v = s_idx[pos];
            while (v < row && ++pos < m) v = s_idx[pos];   // entries that are no row of this domain, or repeats
            if (pos < m && v == row) { bits |= 1u << b; ++pos; }
        }
    }
    if (word < n_words) out_words.v[server][word] = bits;
    const uint32_t found = wave_sum(__popc(bits));
    if (lane == 0 && found) atomicAdd(&s_found, found);
    __syncthreads();
    if (threadIdx.x == 0 && (bad || s_found != m_all)) atomicOr(&status->flags, 4u);
}

// ------------------------------------------------------------------------------------------------
// Worker side.
// ------------------------------------------------------------------------------------------------

// dense = 0 (16-byte streaming stores) and a clean status block.
template <bool NT>
__global__ void __launch_bounds__(PULL_THREADS)
pull_zero_kernel(float *dense, uint64_t n_elems, zen_status_info *status)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) { status->flags = 0; status->reserved = 0; status->needed_rows = 0; }
    const uint64_t n_vec = n_elems >> 2;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    f32x4 *d = (f32x4 *)dense;
    const uint64_t stride = (uint64_t)gridDim.x * PULL_THREADS * 4;
    for (uint64_t i = (uint64_t)blockIdx.x * PULL_THREADS * 4 + threadIdx.x; i < n_vec; i += stride) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + (uint64_t)u * PULL_THREADS < n_vec) {
                if (NT) __builtin_nontemporal_store(z, d + i + (uint64_t)u * PULL_THREADS);
                else d[i + (uint64_t)u * PULL_THREADS] = z;
            }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n_elems & 3u)) dense[(n_vec << 2) + threadIdx.x] = 0.f;
}

// cnt[server][chunk] = set bits of the chunk (0 for parts given as index lists).
__global__ void __launch_bounds__(PULL_THREADS)
pull_count_kernel(PullSrc a, const uint32_t *dom_offsets, uint32_t *cnt, uint32_t n_chunks)
{
    __shared__ uint32_t s_c;
    const uint32_t chunk = blockIdx.x, server = blockIdx.y, p = a.first_part + server;
    const uint32_t n_dom = dom_offsets[p + 1] - dom_offsets[p];
    const uint32_t *__restrict__ bm = a.indices[server] ? nullptr : a.bitmap[server];
    const uint32_t k = chunk * PULL_CHUNK_WORDS + threadIdx.x;
    if (threadIdx.x == 0) s_c = 0;
    __syncthreads();
    const uint32_t w = domain_word(bm, k, n_dom);
    const uint32_t s = wave_sum(__popc(w));
    if (lane_id() == 0 && s) atomicAdd(&s_c, s);
    __syncthreads();
    if (threadIdx.x == 0) cnt[(uint64_t)server * (n_chunks + 1) + chunk] = s_c;
}

// Exclusive scan over the chunks of each partition; the total has to equal the part's row count.
// out_count / out_cap (decode to an index list): *out_count = total, capacity flag.
__global__ void __launch_bounds__(PULL_THREADS)
pull_scan_kernel(PullSrc a, uint32_t *cnt, uint32_t n_chunks, uint32_t *out_count, uint64_t out_cap,
                 zen_status_info *status)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t server = blockIdx.x;
    uint32_t *row = cnt + (uint64_t)server * (n_chunks + 1);
    uint32_t run = 0;
    for (uint32_t c0 = 0; c0 < n_chunks; c0 += PULL_THREADS) {
        const uint32_t c = c0 + threadIdx.x;
        const uint32_t v = c < n_chunks ? row[c] : 0u;
        uint32_t total;
        const uint32_t pre = block_exclusive_scan(v, s_tmp, &total);
        if (c < n_chunks) row[c] = run + pre;
        run += total;
    }
    if (threadIdx.x == 0) {
        row[n_chunks] = run;
        if (out_count) {
            *out_count = run;
            if ((uint64_t)run > out_cap) {
                atomicOr(&status->flags, 1u);
                status->needed_rows = run;
            }
        } else if (!a.indices[server] && a.bitmap[server] && run != *a.count[server]) {
            atomicOr(&status->flags, 4u);
        }
    }
}

// hash_bitmap_decode for the bitmap parts of a launch group: out_idx[server][k] = II_p[position of the
// k-th set bit].  1-D grid, block = (chunk, server).
__global__ void __launch_bounds__(PULL_THREADS)
pull_decode_kernel(PullSrc a, const uint32_t *domain, const uint32_t *dom_offsets, const uint32_t *cnt,
                   uint32_t n_chunks, Arr64<uint32_t *> out_idx, Arr64<uint64_t> out_cap)
{
    __shared__ uint32_t s_word[PULL_CHUNK_WORDS], s_pre[PULL_CHUNK_WORDS], s_tmp[32];
    __shared__ uint32_t s_rows[PULL_CHUNK_BITS];
    const uint32_t server = blockIdx.x % a.n, chunk = blockIdx.x / a.n, p = a.first_part + server;
    const uint32_t *__restrict__ bm = a.indices[server] ? nullptr : a.bitmap[server];
    if (!bm) return;
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    if (chunk * PULL_CHUNK_WORDS >= n_words) return;
    const uint32_t w = domain_word(bm, chunk * PULL_CHUNK_WORDS + threadIdx.x, n_dom);
    s_word[threadIdx.x] = w;
    uint32_t total;
    const uint32_t pre = block_exclusive_scan(__popc(w), s_tmp, &total);
    s_pre[threadIdx.x] = pre;
    __syncthreads();
    if (total == 0) return;
    const uint32_t kbase = cnt[(uint64_t)server * (n_chunks + 1) + chunk];
    const uint32_t *__restrict__ dom = domain + d0;
    const uint32_t j0 = chunk * PULL_CHUNK_BITS, b = threadIdx.x & 31u;
#pragma unroll 4
    for (uint32_t t = 0; t < PULL_CHUNK_BITS / PULL_THREADS; ++t) {   // coalesced domain reads, compaction in LDS
        const uint32_t wi = t * (PULL_THREADS / 32) + (threadIdx.x >> 5);
        const uint32_t ww = s_word[wi];
        if ((ww >> b) & 1u) s_rows[s_pre[wi] + __popc(ww & ((1u << b) - 1u))] = dom[j0 + wi * 32 + b];
    }
    __syncthreads();
    uint32_t *__restrict__ out = out_idx.v[server];
    const uint64_t cap = out_cap.v[server];
    for (uint32_t i = threadIdx.x; i < total; i += PULL_THREADS)
        if ((uint64_t)kbase + i < cap) out[kbase + i] = s_rows[i];
}

// dense[indices[k]] = values[k] for index-list parts (given, or decoded by pull_decode_kernel: bit
// `server` of decoded_mask, whose row count is the smaller of *count and the bitmap's set bits).
// grid = (x, parts); one group of `lanes` threads per row, rows spread over the whole grid.
__global__ void __launch_bounds__(PULL_THREADS)
pull_place_rows_kernel(PullSrc a, uint64_t decoded_mask, const uint32_t *cnt, uint32_t n_chunks, uint64_t n_rows,
                       uint32_t D, uint32_t lanes, float *dense, zen_status_info *status)
{
    const uint32_t server = blockIdx.y;
    const uint32_t *__restrict__ idx = a.indices[server];
    if (!idx) return;
    uint32_t count = *a.count[server];
    if ((decoded_mask >> server) & 1ull) count = min(count, cnt[(uint64_t)server * (n_chunks + 1) + n_chunks]);
    const float *__restrict__ vals = a.values[server];
    bool bad = false;
    if (D == 1) {
        for (uint64_t k = (uint64_t)blockIdx.x * PULL_THREADS + threadIdx.x; k < count;
             k += (uint64_t)gridDim.x * PULL_THREADS) {
            const uint32_t r = idx[k];
            if (r < n_rows) dense[r] = vals[k]; else bad = true;
        }
    } else {
        const uint32_t grp = threadIdx.x / lanes, l = threadIdx.x % lanes, n_grp = PULL_THREADS / lanes;
        for (uint64_t k = (uint64_t)blockIdx.x * n_grp + grp; k < count; k += (uint64_t)gridDim.x * n_grp) {
            const uint32_t r = idx[k];
            if (r >= n_rows) { bad = true; continue; }
            if ((D & 3u) == 0) {
                const u32x4 *src = (const u32x4 *)(vals + k * D);
                u32x4 *dst = (u32x4 *)(dense + (uint64_t)r * D);
                const uint32_t V = D >> 2;
                for (uint32_t v = l; v < V; v += lanes * 4) {
                    u32x4 x[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (v + lanes * u < V) x[u] = src[v + lanes * u];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (v + lanes * u < V) dst[v + lanes * u] = x[u];
                }
            } else {
                for (uint32_t v = l; v < D; v += lanes) dense[(uint64_t)r * D + v] = vals[k * D + v];
            }
        }
    }
    if (bad) atomicOr(&status->flags, 4u);
}

// ------------------------------------------------------------------------------------------------
// Element-level tensors (row_dim == 1): placement by tiles of consecutive rows.  The rows of a tile
// that belong to partition p occupy a CONTIGUOUS stretch [base[tile][p], base[tile+1][p]) of II_p, so
// their bits, their domain entries and (set bits being consecutive) their values are all read with
// unit stride; the tile is assembled in LDS and stored once with 16-byte stores -- zeros included,
// so no zero fill and no scattered 4-byte stores to HBM.
// ------------------------------------------------------------------------------------------------

// base[t][p] = number of rows of II_p below row t * step_rows (built once per context).
__global__ void pull_base_kernel(const uint32_t *domain, const uint32_t *dom_offsets, uint32_t n_parts,
                                 uint32_t n_tiles, uint64_t n_rows, uint32_t *base, uint32_t step_rows)
{
    const uint64_t total = ((uint64_t)n_tiles + 1) * n_parts;
    for (uint64_t id = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; id < total;
         id += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t p = (uint32_t)(id % n_parts), t = (uint32_t)(id / n_parts);
        const uint64_t key = min((uint64_t)t * step_rows, n_rows);
        const uint32_t *dom = domain + dom_offsets[p];
        uint32_t lo = 0, hi = dom_offsets[p + 1] - dom_offsets[p];
        while (lo < hi) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if ((uint64_t)dom[mid] < key) lo = mid + 1; else hi = mid;
        }
        base[id] = lo;
    }
}

// cnt[server][tile] = set bits of the part's bitmap inside the tile's stretch of the domain.
__global__ void __launch_bounds__(PULL_THREADS)
pull_tile_count_kernel(PullSrc a, const uint32_t *base, uint32_t n_parts, uint32_t *cnt, uint32_t n_tiles)
{
    const uint64_t total = (uint64_t)n_tiles * a.n;
    for (uint64_t id = (uint64_t)blockIdx.x * PULL_THREADS + threadIdx.x; id < total;
         id += (uint64_t)gridDim.x * PULL_THREADS) {
        const uint32_t server = (uint32_t)(id % a.n), tile = (uint32_t)(id / a.n), p = a.first_part + server;
        const uint32_t b0 = base[(uint64_t)tile * n_parts + p], b1 = base[(uint64_t)(tile + 1) * n_parts + p];
        const uint32_t *__restrict__ bm = a.indices[server] ? nullptr : a.bitmap[server];
        uint32_t c = 0;
        if (bm && b1 > b0) {
            const uint32_t w0 = b0 >> 5, w1 = (b1 - 1) >> 5;
            for (uint32_t w = w0; w <= w1; ++w) {
                uint32_t word = bm[w];
                if (w == w0) word &= 0xFFFFFFFFu << (b0 & 31u);
                if (w == w1 && (b1 & 31u)) word &= (1u << (b1 & 31u)) - 1u;
                c += __popc(word);
            }
        }
        cnt[(uint64_t)server * (n_tiles + 1) + tile] = c;
    }
}

// One block per tile.  Phase 1: the tile's stretch of every partition (start, length, words).  Phase 2:
// the stretches' bitmap words, masked to the stretch, go to LDS with a running popcount.  Phase 3: the
// tile's rows are walked as ONE flat list (partition after partition), so every thread's domain and
// value loads are independent of each other and of all other threads': a handful of dependent memory
// round trips per block instead of one per partition.  Phase 4: the tile is stored.
// direct = 0: the whole tile (zeros where no partition of this launch group holds the row) is stored;
// direct = 1: only the rows this launch group holds are stored (further groups of a context with more
// than ZEN_MAX_BATCH partitions, after the first group has written every tile).
static constexpr uint32_t PULL_TILE_WORDS = PULL_TILE_ROWS / 32 + 2 * ZEN_MAX_BATCH;   // words of all stretches

__device__ __forceinline__ uint32_t stretch_of(const uint32_t *s_off, uint32_t n, uint32_t e)
{
    uint32_t pos = 0;   // largest p with s_off[p] <= e (offsets ascend, s_off[0] = 0)
#pragma unroll
    for (uint32_t step = ZEN_MAX_BATCH; step; step >>= 1) {
        const uint32_t q = pos + step;
        if (q <= n && s_off[q] <= e) pos = q;
    }
    return pos;
}

__global__ void __launch_bounds__(PULL_THREADS)
pull_tile_place_kernel(PullSrc a, const uint32_t *domain, const uint32_t *dom_offsets, const uint32_t *base,
                       uint32_t n_parts, const uint32_t *cnt, uint32_t n_tiles, uint64_t n_rows, float *dense,
                       uint32_t direct)
{
    __shared__ float s_out[PULL_TILE_ROWS];
    __shared__ uint32_t s_b0[ZEN_MAX_BATCH], s_kb[ZEN_MAX_BATCH], s_cn[ZEN_MAX_BATCH], s_d0[ZEN_MAX_BATCH];
    __shared__ uint32_t s_eoff[ZEN_MAX_BATCH + 1], s_woff[ZEN_MAX_BATCH + 1];
    __shared__ const float *s_vals[ZEN_MAX_BATCH];
    __shared__ const uint32_t *s_bm[ZEN_MAX_BATCH];
    __shared__ uint32_t s_w[PULL_TILE_WORDS], s_wpre[PULL_TILE_WORDS], s_tmp[32];
    const uint32_t tile = blockIdx.x;
    const uint64_t row0 = (uint64_t)tile * PULL_TILE_ROWS;
    if (threadIdx.x < ZEN_WAVE) {   // wave 0: one lane per partition of the launch group
        const uint32_t sv = threadIdx.x;
        uint32_t len = 0, nw = 0;
        if (sv < a.n) {
            const uint32_t p = a.first_part + sv;
            const uint32_t b0 = base[(uint64_t)tile * n_parts + p], b1 = base[(uint64_t)(tile + 1) * n_parts + p];
            len = b1 - b0;
            nw = len ? ((b1 - 1) >> 5) - (b0 >> 5) + 1 : 0u;
            s_b0[sv] = b0;
            s_kb[sv] = cnt[(uint64_t)sv * (n_tiles + 1) + tile];
            s_cn[sv] = *a.count[sv];
            s_d0[sv] = dom_offsets[p];
            s_vals[sv] = a.values[sv];
            s_bm[sv] = a.indices[sv] ? nullptr : a.bitmap[sv];
        }
        const uint32_t e_inc = wave_inclusive_scan(len), w_inc = wave_inclusive_scan(nw);
        if (sv == 0) { s_eoff[0] = 0; s_woff[0] = 0; }
        if (sv < a.n) { s_eoff[sv + 1] = e_inc; s_woff[sv + 1] = w_inc; }
    }
    if (!direct && a.n < n_parts)   // rows of partitions outside this launch group: zero for now
        for (uint32_t i = threadIdx.x; i < PULL_TILE_ROWS; i += PULL_THREADS) s_out[i] = 0.f;
    __syncthreads();
    const uint32_t total_e = s_eoff[a.n], total_w = s_woff[a.n];   // <= PULL_TILE_ROWS, <= PULL_TILE_WORDS

    uint32_t run = 0;
    for (uint32_t w0 = 0; w0 < total_w; w0 += PULL_THREADS) {   // uniform trip count
        const uint32_t w = w0 + threadIdx.x;
        uint32_t word = 0;
        if (w < total_w) {
            const uint32_t sv = stretch_of(s_woff, a.n, w);
            const uint32_t b0 = s_b0[sv], b1 = b0 + (s_eoff[sv + 1] - s_eoff[sv]);
            const uint32_t wi = (b0 >> 5) + (w - s_woff[sv]);
            const uint32_t *__restrict__ bm = s_bm[sv];
            word = bm ? bm[wi] : 0u;
            if (wi == (b0 >> 5)) word &= 0xFFFFFFFFu << (b0 & 31u);
            if (wi == ((b1 - 1) >> 5) && (b1 & 31u)) word &= (1u << (b1 & 31u)) - 1u;
            s_w[w] = word;
        }
        uint32_t total;
        const uint32_t pre = block_exclusive_scan(__popc(word), s_tmp, &total);
        if (w < total_w) s_wpre[w] = run + pre;
        run += total;
    }
    __syncthreads();

    // Batches of 16 rows per thread: all positions first (LDS only), then 32 independent global loads.
    for (uint32_t e0 = 0; e0 < total_e; e0 += PULL_THREADS * 16) {
        uint32_t sv[16], k[16], row[16];
        float v[16];
        bool take[16];
#pragma unroll
        for (uint32_t u = 0; u < 16; ++u) {
            const uint32_t e = e0 + u * PULL_THREADS + threadIdx.x;
            sv[u] = stretch_of(s_eoff, a.n, e < total_e ? e : 0u);
            const uint32_t b0 = s_b0[sv[u]], j = b0 + (e - s_eoff[sv[u]]);
            const uint32_t wq0 = s_woff[sv[u]], wq = wq0 + (j >> 5) - (b0 >> 5);
            const uint32_t word = e < total_e ? s_w[wq] : 0u;
            const bool bit = (word >> (j & 31u)) & 1u;
            k[u] = s_kb[sv[u]] + (s_wpre[e < total_e ? wq : 0u] - s_wpre[wq0]) + __popc(word & ((1u << (j & 31u)) - 1u));
            take[u] = bit && k[u] < s_cn[sv[u]];
            row[u] = s_d0[sv[u]] + j;   // position in the domain table for now
        }
#pragma unroll
        for (uint32_t u = 0; u < 16; ++u) {
            const uint32_t e = e0 + u * PULL_THREADS + threadIdx.x;
            row[u] = e < total_e ? domain[row[u]] : 0u;
            v[u] = take[u] ? s_vals[sv[u]][k[u]] : 0.f;
        }
#pragma unroll
        for (uint32_t u = 0; u < 16; ++u) {
            const uint32_t e = e0 + u * PULL_THREADS + threadIdx.x;
            if (e >= total_e) continue;
            if (!direct) s_out[row[u] - row0] = v[u];
            else if (take[u]) dense[row[u]] = v[u];
        }
    }
    if (direct) return;
    __syncthreads();
    const uint32_t here = (uint32_t)min((uint64_t)PULL_TILE_ROWS, n_rows - row0);
    float *__restrict__ out = dense + row0;   // 16-byte aligned: row0 is a multiple of the tile size
    for (uint32_t i = threadIdx.x * 4; i < here; i += PULL_THREADS * 4) {
        if (i + 4 <= here) {
            const f32x4 v = {s_out[i], s_out[i + 1], s_out[i + 2], s_out[i + 3]};
            *(f32x4 *)(out + i) = v;
        } else {
            for (uint32_t e = i; e < here; ++e) out[e] = s_out[e];
        }
    }
}

#define ZEN_LAUNCH_CHECK()                         \
    do {                                           \
        hipError_t e_ = hipGetLastError();         \
        if (e_ != hipSuccess) return e_;           \
    } while (0)

struct PullLayout {
    uint64_t status_off, cnt_off, n_chunks, n_tiles, dec_off, total;
};

static PullLayout pull_layout(const zen_ctx *ctx)
{
    PullLayout L{};
    const Geometry &g = ctx->geo;
    const uint32_t group = g.n_parts < ZEN_MAX_BATCH ? g.n_parts : ZEN_MAX_BATCH;
    L.status_off = 0;
    L.cnt_off = 256;
    L.n_chunks = (ctx->max_dom_words + PULL_CHUNK_WORDS - 1) / PULL_CHUNK_WORDS;
    if (L.n_chunks < 1) L.n_chunks = 1;
    L.n_tiles = (g.n_rows + PULL_TILE_ROWS - 1) / PULL_TILE_ROWS;
    const uint64_t per = (L.n_chunks > L.n_tiles ? L.n_chunks : L.n_tiles) + 1;
    L.dec_off = L.cnt_off + ((uint64_t)group * per * 4 + 255) / 256 * 256;
    // wide rows: bitmap parts are decoded into index lists first (at most one entry per row of the tensor)
    const uint64_t dec_bytes = (ctx->fmt == ZEN_INDEX_BITMAP && g.row_dim > 1) ? g.n_rows * 4 : 0;
    L.total = L.dec_off + (dec_bytes + 255) / 256 * 256;
    return L;
}

// threads that share one row in the row copies: a power of two <= 64 covering the row's 16-byte vectors
static uint32_t lanes_per_row(uint32_t D)
{
    if (D & 3u) return 64;
    uint32_t l = 1;
    while (l < 64 && l < (D >> 2)) l <<= 1;
    return l;
}

hipError_t build_pull_tables(zen_ctx *ctx, hipStream_t s)
{
    const Geometry &g = ctx->geo;
    if (ctx->fmt != ZEN_INDEX_BITMAP || g.row_dim != 1) return hipSuccess;
    const uint64_t n_tiles = (g.n_rows + PULL_TILE_ROWS - 1) / PULL_TILE_ROWS;
    const uint64_t entries = (n_tiles + 1) * g.n_parts;
    hipError_t e = hipMalloc(&ctx->d_pull_base, entries * 4);
    if (e != hipSuccess) return e;
    uint64_t blocks = (entries + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    pull_base_kernel<<<(uint32_t)blocks, 256, 0, s>>>(ctx->d_domain, ctx->d_dom_offsets, g.n_parts, (uint32_t)n_tiles,
                                                      g.n_rows, ctx->d_pull_base, PULL_TILE_ROWS);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // The same table at the granularity the encode's scatter recognises fully non-zero stretches at
    // (n_parts * 4 bytes per ZEN_GROUP_ROWS rows: kept to at most one byte per row).
    if (g.n_parts <= ZEN_GROUP_MAX_PARTS && g.tile_rows % ZEN_GROUP_ROWS == 0) {
        const uint64_t n_groups = (uint64_t)g.n_tiles * (g.tile_rows / ZEN_GROUP_ROWS);
        const uint64_t gentries = (n_groups + 1) * g.n_parts;
        e = hipMalloc(&ctx->d_group_base, gentries * 4);
        if (e != hipSuccess) return e;
        blocks = (gentries + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        pull_base_kernel<<<(uint32_t)blocks, 256, 0, s>>>(ctx->d_domain, ctx->d_dom_offsets, g.n_parts,
                                                          (uint32_t)n_groups, g.n_rows, ctx->d_group_base, ZEN_GROUP_ROWS);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipStreamSynchronize(s);
}

static hipError_t launch_pull_encode(zen_ctx *ctx, const PullSrc &src, const Arr64<uint64_t> &caps,
                                     const Arr64<uint32_t *> &out_words, char *ws, zen_status_info *status,
                                     hipStream_t s)
{
    const PullLayout L = pull_layout(ctx);
    uint32_t *bounds = (uint32_t *)(ws + L.cnt_off);
    const uint32_t n_chunks = (uint32_t)L.n_chunks;
    ProfScope prof(ctx, K_PULL_ENCODE, s);
    pull_bounds_kernel<<<dim3(n_chunks / (PULL_THREADS / ZEN_WAVE) + 1, src.n), PULL_THREADS, 0, s>>>(
        src, caps, ctx->d_domain, ctx->d_dom_offsets, bounds, n_chunks);
    ZEN_LAUNCH_CHECK();
    pull_encode_kernel<<<dim3(n_chunks, src.n), PULL_THREADS, 0, s>>>(
        src, caps, out_words, ctx->d_domain, ctx->d_dom_offsets, bounds, n_chunks, status);
    return hipGetLastError();
}

// count -> scan -> decode for the bitmap parts of one group; out_count / out_cap0: single-part decode
// to a caller's list (capacity flag), else lists without a count of their own.
static hipError_t launch_pull_decode(zen_ctx *ctx, const PullSrc &src, char *ws, const Arr64<uint32_t *> &out_idx,
                                     const Arr64<uint64_t> &out_cap, uint32_t *out_count, hipStream_t s)
{
    const PullLayout L = pull_layout(ctx);
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);
    uint32_t *cnt = (uint32_t *)(ws + L.cnt_off);
    const uint32_t n_chunks = (uint32_t)L.n_chunks;
    {
        ProfScope prof(ctx, K_PULL_COUNT, s);
        pull_count_kernel<<<dim3(n_chunks, src.n), PULL_THREADS, 0, s>>>(src, ctx->d_dom_offsets, cnt, n_chunks);
        ZEN_LAUNCH_CHECK();
    }
    {
        ProfScope prof(ctx, K_PULL_SCAN, s);
        pull_scan_kernel<<<src.n, PULL_THREADS, 0, s>>>(src, cnt, n_chunks, out_count, out_cap.v[0], status);
        ZEN_LAUNCH_CHECK();
    }
    {
        const uint64_t blocks = L.n_chunks * src.n;
        if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
        ProfScope prof(ctx, K_PULL_PLACE, s);
        pull_decode_kernel<<<(uint32_t)blocks, PULL_THREADS, 0, s>>>(src, ctx->d_domain, ctx->d_dom_offsets, cnt,
                                                                     n_chunks, out_idx, out_cap);
        ZEN_LAUNCH_CHECK();
    }
    return hipSuccess;
}

// Element-level tensors: tile counts -> scan -> tile placement for one group.
static hipError_t launch_pull_tiles(zen_ctx *ctx, const PullSrc &src, char *ws, float *dense, bool direct,
                                    hipStream_t s)
{
    const Geometry &g = ctx->geo;
    const PullLayout L = pull_layout(ctx);
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);
    uint32_t *cnt = (uint32_t *)(ws + L.cnt_off);
    const uint32_t n_tiles = (uint32_t)L.n_tiles;
    {
        uint64_t blocks = ((uint64_t)n_tiles * src.n + PULL_THREADS - 1) / PULL_THREADS;
        if (blocks > 65536) blocks = 65536;
        ProfScope prof(ctx, K_PULL_COUNT, s);
        pull_tile_count_kernel<<<(uint32_t)blocks, PULL_THREADS, 0, s>>>(src, ctx->d_pull_base, g.n_parts, cnt, n_tiles);
        ZEN_LAUNCH_CHECK();
    }
    {
        ProfScope prof(ctx, K_PULL_SCAN, s);
        pull_scan_kernel<<<src.n, PULL_THREADS, 0, s>>>(src, cnt, n_tiles, nullptr, 0, status);
        ZEN_LAUNCH_CHECK();
    }
    {
        ProfScope prof(ctx, K_PULL_PLACE, s);
        pull_tile_place_kernel<<<n_tiles, PULL_THREADS, 0, s>>>(src, ctx->d_domain, ctx->d_dom_offsets,
                                                                ctx->d_pull_base, g.n_parts, cnt, n_tiles, g.n_rows,
                                                                dense, direct ? 1u : 0u);
        ZEN_LAUNCH_CHECK();
    }
    return hipSuccess;
}

} // namespace zen

using namespace zen;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return ZEN_ERR_DEVICE;    \
    } while (0)

extern "C" {

zen_status zen_pull_workspace_bytes(const zen_ctx *ctx, uint64_t *host_bytes)
{
    if (!ctx || !host_bytes) return ZEN_ERR_INVALID;
    *host_bytes = pull_layout(ctx).total;
    return ZEN_OK;
}

zen_status zen_pull_encode_batch(zen_ctx *ctx, const zen_aggregated *host_aggs, uint32_t *bitmap, void *workspace,
                                 uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !host_aggs || !bitmap || !workspace || ctx->fmt != ZEN_INDEX_BITMAP) return ZEN_ERR_INVALID;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)bitmap & 3u)) return ZEN_ERR_INVALID;
    const PullLayout L = pull_layout(ctx);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    const uint32_t n = ctx->geo.n_parts;
    for (uint32_t j = 0; j < n; ++j)
        if (!host_aggs[j].indices || !host_aggs[j].count || host_aggs[j].cap_rows > 0xFFFFFFFEull) return ZEN_ERR_INVALID;
    hipStream_t s = (hipStream_t)hip_stream;
    zen_status_info *status = (zen_status_info *)((char *)workspace + L.status_off);
    HIP_TRY(launch_fill_u32((uint32_t *)status, 4, 0u, s));
    for (uint32_t j0 = 0; j0 < n; j0 += ZEN_MAX_BATCH) {
        PullSrc src;
        Arr64<uint64_t> caps;
        Arr64<uint32_t *> words;
        memset(&src, 0, sizeof(src));
        memset(&caps, 0, sizeof(caps));
        memset(&words, 0, sizeof(words));
        src.n = n - j0 < ZEN_MAX_BATCH ? n - j0 : ZEN_MAX_BATCH;
        src.first_part = j0;
        for (uint32_t i = 0; i < src.n; ++i) {
            src.indices[i] = host_aggs[j0 + i].indices;
            src.count[i] = host_aggs[j0 + i].count;
            caps.v[i] = host_aggs[j0 + i].cap_rows;
            words.v[i] = bitmap + ctx->h_bm_word_off[j0 + i];
        }
        HIP_TRY(launch_pull_encode(ctx, src, caps, words, (char *)workspace, status, s));
    }
    return ZEN_OK;
}

zen_status zen_pull_encode(zen_ctx *ctx, const uint32_t *indices, const uint32_t *count, uint64_t cap_rows,
                           uint32_t part_id, uint32_t *bitmap_words, void *workspace, uint64_t workspace_bytes,
                           void *hip_stream)
{
    if (!ctx || !indices || !count || !bitmap_words || !workspace || ctx->fmt != ZEN_INDEX_BITMAP) return ZEN_ERR_INVALID;
    if (part_id >= ctx->geo.n_parts || cap_rows > 0xFFFFFFFEull || ((uintptr_t)workspace & 255u) ||
        ((uintptr_t)bitmap_words & 3u))
        return ZEN_ERR_INVALID;
    const PullLayout L = pull_layout(ctx);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    zen_status_info *status = (zen_status_info *)((char *)workspace + L.status_off);
    HIP_TRY(launch_fill_u32((uint32_t *)status, 4, 0u, s));
    PullSrc src;
    Arr64<uint64_t> caps;
    Arr64<uint32_t *> words;
    memset(&src, 0, sizeof(src));
    memset(&caps, 0, sizeof(caps));
    memset(&words, 0, sizeof(words));
    src.n = 1;
    src.first_part = part_id;
    src.indices[0] = indices;
    src.count[0] = count;
    caps.v[0] = cap_rows;
    words.v[0] = bitmap_words;
    HIP_TRY(launch_pull_encode(ctx, src, caps, words, (char *)workspace, status, s));
    return ZEN_OK;
}

zen_status zen_pull_decode(zen_ctx *ctx, const uint32_t *bitmap_words, uint32_t part_id, uint32_t *out_indices,
                           uint64_t out_cap_rows, uint32_t *out_count, void *workspace, uint64_t workspace_bytes,
                           void *hip_stream)
{
    if (!ctx || !bitmap_words || !out_indices || !out_count || !workspace || ctx->fmt != ZEN_INDEX_BITMAP)
        return ZEN_ERR_INVALID;
    if (part_id >= ctx->geo.n_parts || out_cap_rows > 0xFFFFFFFEull || ((uintptr_t)workspace & 255u) ||
        ((uintptr_t)bitmap_words & 3u))
        return ZEN_ERR_INVALID;
    const PullLayout L = pull_layout(ctx);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(launch_fill_u32((uint32_t *)((char *)workspace + L.status_off), 4, 0u, s));
    PullSrc src;
    Arr64<uint32_t *> oi;
    Arr64<uint64_t> oc;
    memset(&src, 0, sizeof(src));
    memset(&oi, 0, sizeof(oi));
    memset(&oc, 0, sizeof(oc));
    src.n = 1;
    src.first_part = part_id;
    src.bitmap[0] = bitmap_words;
    oi.v[0] = out_indices;
    oc.v[0] = out_cap_rows;
    HIP_TRY(launch_pull_decode(ctx, src, (char *)workspace, oi, oc, out_count, s));
    return ZEN_OK;
}

zen_status zen_pull_apply(zen_ctx *ctx, const zen_part *host_parts, float *dense, void *workspace,
                          uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !host_parts || !dense || !workspace) return ZEN_ERR_INVALID;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)dense & 15u)) return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    const uint32_t n = g.n_parts;
    bool any_bitmap_at_all = false;
    for (uint32_t p = 0; p < n; ++p) {
        const zen_part &q = host_parts[p];
        if (!q.count || !q.values || (!q.indices && !q.bitmap) || ((uintptr_t)q.values & 15u)) return ZEN_ERR_INVALID;
        if (!q.indices && ctx->fmt != ZEN_INDEX_BITMAP) return ZEN_ERR_INVALID;   // no domain tables
        if (!q.indices) any_bitmap_at_all = true;
    }
    const PullLayout L = pull_layout(ctx);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);
    const uint64_t n_elems = g.n_rows * g.row_dim;
    // Element-level tensors with bitmap parts are written tile by tile, zeros included; everything
    // else starts from a zero fill.
    const bool tiles = g.row_dim == 1 && any_bitmap_at_all && ctx->d_pull_base;
    if (tiles) {
        HIP_TRY(launch_fill_u32((uint32_t *)status, 4, 0u, s));
    } else {
        uint64_t blocks = ((n_elems >> 2) + PULL_THREADS * 4 - 1) / (PULL_THREADS * 4);
        if (blocks < 1) blocks = 1;
        if (blocks > (1u << 20)) blocks = 1u << 20;
        ProfScope prof(ctx, K_PULL_ZERO, s);
        pull_zero_kernel<true><<<(uint32_t)blocks, PULL_THREADS, 0, s>>>(dense, n_elems, status);   // streaming stores
        HIP_TRY(hipGetLastError());
    }
    uint32_t *dec = (uint32_t *)(ws + L.dec_off);
    uint64_t dom_start = 0;   // start of partition p's decoded list = start of its domain
    for (uint32_t p0 = 0; p0 < n; p0 += ZEN_MAX_BATCH) {
        PullSrc src;
        memset(&src, 0, sizeof(src));
        src.n = n - p0 < ZEN_MAX_BATCH ? n - p0 : ZEN_MAX_BATCH;
        src.first_part = p0;
        bool any_bitmap = false, any_list = false;
        for (uint32_t i = 0; i < src.n; ++i) {
            const zen_part &q = host_parts[p0 + i];
            src.indices[i] = q.indices;
            src.bitmap[i] = q.bitmap;
            src.values[i] = q.values;
            src.count[i] = q.count;
            if (q.indices) any_list = true; else any_bitmap = true;
        }
        uint64_t decoded_mask = 0;
        if (tiles) {
            // the first group writes every tile in full (also when it holds index lists only)
            if (any_bitmap || p0 == 0) HIP_TRY(launch_pull_tiles(ctx, src, ws, dense, p0 != 0, s));
        } else if (any_bitmap) {
            Arr64<uint32_t *> oi;
            Arr64<uint64_t> oc;
            memset(&oi, 0, sizeof(oi));
            memset(&oc, 0, sizeof(oc));
            uint64_t d = dom_start;
            for (uint32_t i = 0; i < src.n; ++i) {
                oi.v[i] = dec + d;
                oc.v[i] = ctx->h_dom_sizes[p0 + i];
                d += ctx->h_dom_sizes[p0 + i];
            }
            HIP_TRY(launch_pull_decode(ctx, src, ws, oi, oc, nullptr, s));
            for (uint32_t i = 0; i < src.n; ++i)
                if (!src.indices[i]) {
                    src.indices[i] = oi.v[i];
                    decoded_mask |= 1ull << i;
                }
            any_list = true;
        }
        if (ctx->fmt == ZEN_INDEX_BITMAP)
            for (uint32_t i = 0; i < src.n; ++i) dom_start += ctx->h_dom_sizes[p0 + i];
        if (any_list) {
            ProfScope prof(ctx, K_PULL_PLACE_COO, s);
            const uint32_t lanes = lanes_per_row(g.row_dim);
            pull_place_rows_kernel<<<dim3(g.row_dim == 1 ? 512 : 1024, src.n), PULL_THREADS, 0, s>>>(
                src, decoded_mask, (const uint32_t *)(ws + L.cnt_off), (uint32_t)L.n_chunks, g.n_rows, g.row_dim, lanes,
                dense, status);
            HIP_TRY(hipGetLastError());
        }
    }
    return ZEN_OK;
}

} // extern "C"
