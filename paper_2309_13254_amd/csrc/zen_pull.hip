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
#include <string.h>
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int PULL_THREADS = 256;
static constexpr uint32_t PULL_CHUNK_WORDS = 256;                     // bitmap words per block
static constexpr uint32_t PULL_CHUNK_BITS = PULL_CHUNK_WORDS * 32;    // domain rows per block

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

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, ZEN_WAVE);
    return v;
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
__global__ void __launch_bounds__(PULL_THREADS)
pull_encode_kernel(PullSrc a, Arr64<uint64_t> cap_rows, Arr64<uint32_t *> out_words, const uint32_t *domain,
                   const uint32_t *dom_offsets, zen_status_info *status)
{
    __shared__ uint32_t s_idx[PULL_CHUNK_BITS];
    __shared__ uint32_t s_k[3], s_found;
    const uint32_t chunk = blockIdx.x, server = blockIdx.y, p = a.first_part + server;
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t *__restrict__ idx = a.indices[server];
    uint32_t cnt = *a.count[server];
    if ((uint64_t)cnt > cap_rows.v[server]) cnt = (uint32_t)cap_rows.v[server];
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    const uint32_t active = (n_words + PULL_CHUNK_WORDS - 1) / PULL_CHUNK_WORDS;
    if (chunk >= active) {   // nothing to write; an empty domain cannot hold indices
        if (chunk == 0 && cnt != 0 && threadIdx.x == 0) atomicOr(&status->flags, 4u);
        return;
    }
    const uint32_t *__restrict__ dom = domain + d0;
    const uint32_t j0 = chunk * PULL_CHUNK_BITS, j1 = min(j0 + PULL_CHUNK_BITS, n_dom);
    if (wave == 0) {          // first index that can belong to this chunk
        const uint32_t k = wave_lower_bound(idx, cnt, dom[j0]);
        if (lane == 0) s_k[0] = k;
    } else if (wave == 1) {   // first index past this chunk (row ids stay below 2^32 - 1: no wrap)
        const uint32_t k = wave_lower_bound(idx, cnt, dom[j1 - 1] + 1u);
        if (lane == 0) s_k[1] = k;
    } else if (wave == 2) {   // where the previous chunk ended: indices in between belong to no chunk
        const uint32_t k = chunk ? wave_lower_bound(idx, cnt, dom[j0 - 1] + 1u) : 0u;
        if (lane == 0) s_k[2] = k;
    }
    if (threadIdx.x == 0) s_found = 0;
    __syncthreads();
    const uint32_t k0 = s_k[0], k1 = s_k[1];
    bool bad = k1 < k0 || s_k[2] != k0 || (chunk == active - 1 && k1 != cnt);
    const uint32_t m_all = k1 < k0 ? 0u : k1 - k0;
    if (m_all > PULL_CHUNK_BITS) bad = true;   // more indices than domain rows
    const uint32_t m = min(m_all, PULL_CHUNK_BITS);
    for (uint32_t i = threadIdx.x; i < m; i += PULL_THREADS) s_idx[i] = idx[k0 + i];
    __syncthreads();
    uint32_t *__restrict__ bm = out_words.v[server];
    uint32_t found = 0;
#pragma unroll 4
    for (uint32_t t = 0; t < PULL_CHUNK_BITS / PULL_THREADS; ++t) {
        const uint32_t j = j0 + t * PULL_THREADS + threadIdx.x;
        const bool valid = j < j1;
        const uint32_t row = valid ? dom[j] : 0u;
        uint32_t pos = 0;   // number of slice entries below `row`
#pragma unroll
        for (uint32_t step = PULL_CHUNK_BITS / 2; step; step >>= 1) {
            const uint32_t q = pos + step;
            if (q <= m && s_idx[q - 1] < row) pos = q;
        }
        if (pos < m && s_idx[pos] < row) ++pos;   // a full slice (m = 8,192) needs one more step
        const bool member = valid && pos < m && s_idx[pos] == row;
        const uint64_t bal = ballot(member);
        const uint32_t word = (j0 >> 5) + t * (PULL_THREADS / 32) + wave * 2;
        if (lane == 0 && word < n_words) bm[word] = (uint32_t)bal;
        if (lane == 32 && word + 1 < n_words) bm[word + 1] = (uint32_t)(bal >> 32);
        found += (uint32_t)__popcll(bal);
    }
    if (lane == 0) atomicAdd(&s_found, found);
    __syncthreads();
    if (threadIdx.x == 0 && (bad || s_found != m_all)) atomicOr(&status->flags, 4u);
}

// ------------------------------------------------------------------------------------------------
// Worker side.
// ------------------------------------------------------------------------------------------------

// dense = 0 (16-byte streaming stores) and a clean status block.
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
            if (i + (uint64_t)u * PULL_THREADS < n_vec) __builtin_nontemporal_store(z, d + i + (uint64_t)u * PULL_THREADS);
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
    const uint32_t s = wave_sum_u32(__popc(w));
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

// Copies `total` rows src[(kbase + i)] -> dense[s_rows[i]] with groups of `lanes` threads per row.
__device__ __forceinline__ void place_rows(const float *__restrict__ vals, float *__restrict__ dense, uint32_t D,
                                           uint32_t lanes, const uint32_t *s_rows, uint32_t kbase, uint32_t total)
{
    const uint32_t grp = threadIdx.x / lanes, l = threadIdx.x % lanes, n_grp = PULL_THREADS / lanes;
    if ((D & 3u) == 0) {
        const uint32_t V = D >> 2;
        for (uint32_t i = grp; i < total; i += n_grp) {
            const u32x4 *src = (const u32x4 *)(vals + (uint64_t)(kbase + i) * D);
            u32x4 *dst = (u32x4 *)(dense + (uint64_t)s_rows[i] * D);
            for (uint32_t v = l; v < V; v += lanes) dst[v] = src[v];
        }
    } else {
        for (uint32_t i = grp; i < total; i += n_grp) {
            const float *src = vals + (uint64_t)(kbase + i) * D;
            float *dst = dense + (uint64_t)s_rows[i] * D;
            for (uint32_t v = l; v < D; v += lanes) dst[v] = src[v];
        }
    }
}

// Decode + place.  1-D grid; consecutive blocks of one XCD (block id mod 8) take the SAME chunk of
// consecutive partitions: the domains are uniform samples of the row range, so those blocks write
// into the same stretch of the dense tensor and their 4-byte stores meet in that XCD's L2.
//   INDICES: write the decoded row ids (hash_bitmap_decode proper) instead of placing values.
template <bool INDICES>
__global__ void __launch_bounds__(PULL_THREADS)
pull_place_kernel(PullSrc a, const uint32_t *domain, const uint32_t *dom_offsets, const uint32_t *cnt,
                  uint32_t n_chunks, uint32_t D, uint32_t lanes, float *dense, uint32_t *out_idx, uint64_t out_cap)
{
    __shared__ uint32_t s_word[PULL_CHUNK_WORDS], s_pre[PULL_CHUNK_WORDS], s_tmp[32];
    extern __shared__ uint32_t s_rows[];   // [PULL_CHUNK_BITS] unless rows are single elements
    const uint32_t x = blockIdx.x & 7u, t8 = blockIdx.x >> 3;
    const uint32_t server = t8 % a.n, chunk = (t8 / a.n) * 8 + x, p = a.first_part + server;
    const uint32_t *__restrict__ bm = a.indices[server] ? nullptr : a.bitmap[server];
    if (!bm) return;
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    if (chunk * PULL_CHUNK_WORDS >= n_words) return;
    const uint32_t k = chunk * PULL_CHUNK_WORDS + threadIdx.x;
    const uint32_t w = domain_word(bm, k, n_dom);
    s_word[threadIdx.x] = w;
    uint32_t total;
    const uint32_t pre = block_exclusive_scan(__popc(w), s_tmp, &total);
    s_pre[threadIdx.x] = pre;
    __syncthreads();
    if (total == 0) return;
    const uint32_t kbase = cnt[(uint64_t)server * (n_chunks + 1) + chunk];
    const uint32_t count = INDICES ? 0xFFFFFFFFu : *a.count[server];
    const uint32_t *__restrict__ dom = domain + d0;
    const float *__restrict__ vals = a.values[server];
    const uint32_t j0 = chunk * PULL_CHUNK_BITS, b = threadIdx.x & 31u;
    const bool direct = !INDICES && D == 1;
#pragma unroll 4
    for (uint32_t t = 0; t < PULL_CHUNK_BITS / PULL_THREADS; ++t) {
        const uint32_t wi = t * (PULL_THREADS / 32) + (threadIdx.x >> 5);
        const uint32_t ww = s_word[wi];
        if (!((ww >> b) & 1u)) continue;
        const uint32_t j = j0 + wi * 32 + b;
        const uint32_t kl = s_pre[wi] + __popc(ww & ((1u << b) - 1u));
        const uint32_t row = dom[j];
        if (direct) {
            if (kbase + kl < count) dense[row] = vals[kbase + kl];
        } else {
            s_rows[kl] = row;
        }
    }
    if (direct) return;
    __syncthreads();
    if (INDICES) {
        for (uint32_t i = threadIdx.x; i < total; i += PULL_THREADS)
            if ((uint64_t)kbase + i < out_cap) out_idx[kbase + i] = s_rows[i];
    } else {
        const uint32_t usable = kbase >= count ? 0u : min(total, count - kbase);
        place_rows(vals, dense, D, lanes, s_rows, kbase, usable);
    }
}

// Parts given as index lists: dense[indices[k]] = values[k].  grid = (x, parts).
__global__ void __launch_bounds__(PULL_THREADS)
pull_place_coo_kernel(PullSrc a, uint64_t n_rows, uint32_t D, uint32_t lanes, float *dense, zen_status_info *status)
{
    const uint32_t server = blockIdx.y;
    const uint32_t *__restrict__ idx = a.indices[server];
    if (!idx) return;
    const uint32_t count = *a.count[server];
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
                for (uint32_t v = l; v < (D >> 2); v += lanes) dst[v] = src[v];
            } else {
                for (uint32_t v = l; v < D; v += lanes) dense[(uint64_t)r * D + v] = vals[k * D + v];
            }
        }
    }
    if (bad) atomicOr(&status->flags, 4u);
}

#define ZEN_LAUNCH_CHECK()                         \
    do {                                           \
        hipError_t e_ = hipGetLastError();         \
        if (e_ != hipSuccess) return e_;           \
    } while (0)

struct PullLayout {
    uint64_t status_off, cnt_off, n_chunks, total;
};

static PullLayout pull_layout(const zen_ctx *ctx)
{
    PullLayout L{};
    const uint32_t group = ctx->geo.n_parts < ZEN_MAX_BATCH ? ctx->geo.n_parts : ZEN_MAX_BATCH;
    L.status_off = 0;
    L.cnt_off = 256;
    L.n_chunks = (ctx->max_dom_words + PULL_CHUNK_WORDS - 1) / PULL_CHUNK_WORDS;
    if (L.n_chunks < 1) L.n_chunks = 1;
    L.total = L.cnt_off + ((uint64_t)group * (L.n_chunks + 1) * 4 + 255) / 256 * 256;
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

static hipError_t launch_pull_encode(zen_ctx *ctx, const PullSrc &src, const Arr64<uint64_t> &caps,
                                     const Arr64<uint32_t *> &out_words, zen_status_info *status, hipStream_t s)
{
    const PullLayout L = pull_layout(ctx);
    ProfScope prof(ctx, K_PULL_ENCODE, s);
    pull_encode_kernel<<<dim3((uint32_t)L.n_chunks, src.n), PULL_THREADS, 0, s>>>(
        src, caps, out_words, ctx->d_domain, ctx->d_dom_offsets, status);
    return hipGetLastError();
}

// count -> scan -> place for the bitmap parts of one group.
static hipError_t launch_pull_bitmap(zen_ctx *ctx, const PullSrc &src, char *ws, float *dense, uint32_t *out_idx,
                                     uint64_t out_cap, uint32_t *out_count, hipStream_t s)
{
    const Geometry &g = ctx->geo;
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
        pull_scan_kernel<<<src.n, PULL_THREADS, 0, s>>>(src, cnt, n_chunks, out_count, out_cap, status);
        ZEN_LAUNCH_CHECK();
    }
    {
        const uint64_t chunks8 = (L.n_chunks + 7) / 8 * 8;
        const uint64_t blocks = chunks8 * src.n;
        if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
        ProfScope prof(ctx, K_PULL_PLACE, s);
        if (out_idx) {
            pull_place_kernel<true><<<(uint32_t)blocks, PULL_THREADS, PULL_CHUNK_BITS * 4, s>>>(
                src, ctx->d_domain, ctx->d_dom_offsets, cnt, n_chunks, g.row_dim, 1, nullptr, out_idx, out_cap);
        } else {
            const size_t lds = g.row_dim == 1 ? 0 : PULL_CHUNK_BITS * 4;
            pull_place_kernel<false><<<(uint32_t)blocks, PULL_THREADS, lds, s>>>(
                src, ctx->d_domain, ctx->d_dom_offsets, cnt, n_chunks, g.row_dim, lanes_per_row(g.row_dim), dense,
                nullptr, 0);
        }
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
        HIP_TRY(launch_pull_encode(ctx, src, caps, words, status, s));
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
    HIP_TRY(launch_pull_encode(ctx, src, caps, words, status, s));
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
    memset(&src, 0, sizeof(src));
    src.n = 1;
    src.first_part = part_id;
    src.bitmap[0] = bitmap_words;
    HIP_TRY(launch_pull_bitmap(ctx, src, (char *)workspace, nullptr, out_indices, out_cap_rows, out_count, s));
    return ZEN_OK;
}

zen_status zen_pull_apply(zen_ctx *ctx, const zen_part *host_parts, float *dense, void *workspace,
                          uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !host_parts || !dense || !workspace) return ZEN_ERR_INVALID;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)dense & 15u)) return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    const uint32_t n = g.n_parts;
    for (uint32_t p = 0; p < n; ++p) {
        const zen_part &q = host_parts[p];
        if (!q.count || !q.values || (!q.indices && !q.bitmap) || ((uintptr_t)q.values & 15u)) return ZEN_ERR_INVALID;
        if (!q.indices && ctx->fmt != ZEN_INDEX_BITMAP) return ZEN_ERR_INVALID;   // no domain tables
    }
    const PullLayout L = pull_layout(ctx);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);
    const uint64_t n_elems = g.n_rows * g.row_dim;
    {
        uint64_t blocks = ((n_elems >> 2) + PULL_THREADS * 4 - 1) / (PULL_THREADS * 4);
        if (blocks < 1) blocks = 1;
        if (blocks > 16384) blocks = 16384;
        ProfScope prof(ctx, K_PULL_ZERO, s);
        pull_zero_kernel<<<(uint32_t)blocks, PULL_THREADS, 0, s>>>(dense, n_elems, status);
        HIP_TRY(hipGetLastError());
    }
    for (uint32_t p0 = 0; p0 < n; p0 += ZEN_MAX_BATCH) {
        PullSrc src;
        memset(&src, 0, sizeof(src));
        src.n = n - p0 < ZEN_MAX_BATCH ? n - p0 : ZEN_MAX_BATCH;
        src.first_part = p0;
        bool any_bitmap = false, any_coo = false;
        for (uint32_t i = 0; i < src.n; ++i) {
            const zen_part &q = host_parts[p0 + i];
            src.indices[i] = q.indices;
            src.bitmap[i] = q.bitmap;
            src.values[i] = q.values;
            src.count[i] = q.count;
            if (q.indices) any_coo = true; else any_bitmap = true;
        }
        if (any_bitmap) HIP_TRY(launch_pull_bitmap(ctx, src, ws, dense, nullptr, 0, nullptr, s));
        if (any_coo) {
            ProfScope prof(ctx, K_PULL_PLACE_COO, s);
            const uint32_t lanes = lanes_per_row(g.row_dim);
            pull_place_coo_kernel<<<dim3(g.row_dim == 1 ? 512 : 1024, src.n), PULL_THREADS, 0, s>>>(
                src, g.n_rows, g.row_dim, lanes, dense, status);
            HIP_TRY(hipGetLastError());
        }
    }
    return ZEN_OK;
}

} // extern "C"
