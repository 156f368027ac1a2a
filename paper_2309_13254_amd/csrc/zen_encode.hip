// Encode kernels for gfx950: non-zero detection + per-tile owner histogram, the partition scan,
// and the stable scatter with value gather (and hash-bitmap assembly).
//
// One launch covers every worker of a batch: blockIdx.y = worker, blockIdx.x = tile of consecutive
// rows.  The dense gradient is read exactly once, by the detect kernel, with 16-byte loads; all
// later steps work from the 1-bit-per-row mask and touch the dense data only to copy non-zero rows.
#include "zen_device.h"
#include <string.h>
#include "zen_internal.h"

namespace zen {

#ifndef ZEN_DETECT_THREADS
#define ZEN_DETECT_THREADS 256
#endif
#ifndef ZEN_DETECT_NT
#define ZEN_DETECT_NT 1
#endif
#ifndef ZEN_ROW_UNROLL
#define ZEN_ROW_UNROLL 4
#endif
static constexpr int DETECT_THREADS = ZEN_DETECT_THREADS;
static constexpr int SCATTER_THREADS = 256;
static constexpr int SCAN_THREADS = 1024;
static constexpr uint32_t SCAN_FLAG_WORDS = 4096; // partition scan: tile flags kept as bits in LDS up to 131,072 tiles
static constexpr int SEG_WORDS = 64;              // mask words expanded per scatter segment
static constexpr int SEG_ROWS = SEG_WORDS * 32;   // 2048
static constexpr uint32_t SEG_FLAG_WORDS = 32;    // mask words per bit of a tile's flag word (tiles of 1,024 words)
static constexpr int GROUP_WORDS = ZEN_GROUP_ROWS / 32;   // 16 mask words: the unit the element-level scatter counts rows in
static constexpr uint32_t MIN_STRETCH_ROWS = 128;  // shortest stretch of consecutive listed rows placed from the rank tables

__device__ __forceinline__ u32x4 load_stream(const u32x4 *p)
{
#if ZEN_DETECT_NT
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// ----------------------------------------------------------------------------------------------
// E1: detection.  Each variant fills s_mask[tile_words] (bit r%32 of word r/32, tile-relative).
// ----------------------------------------------------------------------------------------------

// row_dim == 1.  A wave-load of 64 x 16 B covers 256 rows = 8 mask words.
template <int UNROLL>
__device__ __forceinline__ void detect_elem(const float *__restrict__ g, uint64_t n_rows, uint64_t row0,
                                            uint32_t tile_rows, uint32_t *s_mask, uint32_t thr)
{   // thr >= 1: smallest magnitude (as an integer) that counts as present; 1 = every non-zero
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint32_t n_chunks = tile_rows >> 8;
    for (uint32_t c0 = wave * UNROLL; c0 < n_chunks; c0 += nw * UNROLL) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t c = c0 + u;
            const uint64_t e = row0 + ((uint64_t)c << 8) + lane * 4;
            v[u] = (u32x4){0u, 0u, 0u, 0u};
            if (c < n_chunks) {
                if (row0 + ((uint64_t)(c + 1) << 8) <= n_rows) {
                    v[u] = load_stream((const u32x4 *)(g + e));
                } else {
                    const uint32_t *gu = (const uint32_t *)g;
                    if (e + 0 < n_rows) v[u].x = gu[e + 0];
                    if (e + 1 < n_rows) v[u].y = gu[e + 1];
                    if (e + 2 < n_rows) v[u].z = gu[e + 2];
                    if (e + 3 < n_rows) v[u].w = gu[e + 3];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t c = c0 + u;
            if (c < n_chunks && ballot(nonzero_mag(v[u]) != 0) != 0) {   // s_mask starts zeroed
                uint32_t nib = ((v[u].x & 0x7fffffffu) >= thr ? 1u : 0u) | ((v[u].y & 0x7fffffffu) >= thr ? 2u : 0u) |
                               ((v[u].z & 0x7fffffffu) >= thr ? 4u : 0u) | ((v[u].w & 0x7fffffffu) >= thr ? 8u : 0u);
                uint32_t word = nib << (4 * (lane & 7));
                word |= __shfl_xor(word, 1, ZEN_WAVE);
                word |= __shfl_xor(word, 2, ZEN_WAVE);
                word |= __shfl_xor(word, 4, ZEN_WAVE);
                if ((lane & 7) == 0) s_mask[c * 8 + (lane >> 3)] = word;
            }
        }
    }
}

// row_dim = 4*L, L a power of two <= 32: L lanes per row, 64/L rows per wave-load, 64 rows per unit.
template <int L>
__device__ __forceinline__ void detect_sub(const float *__restrict__ g, uint64_t n_rows, uint64_t row0,
                                           uint32_t tile_rows, uint32_t *s_mask)
{
    constexpr int RPL = 64 / L;               // rows per wave-load
    constexpr int BATCH = L < 16 ? L : 16;    // loads kept in flight
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint32_t n_units = tile_rows >> 6;
    for (uint32_t unit = wave; unit < n_units; unit += nw) {
        const uint64_t urow = row0 + ((uint64_t)unit << 6);
        const u32x4 *base = (const u32x4 *)(g + urow * (uint64_t)(4 * L));
        uint64_t unit_mask = 0;
#pragma unroll
        for (int j0 = 0; j0 < L; j0 += BATCH) {
            u32x4 v[BATCH];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const uint32_t vi = (uint32_t)(j0 + j) * 64 + lane;   // 16-byte vector inside the unit
                const uint64_t row = urow + vi / L;
                v[j] = (u32x4){0u, 0u, 0u, 0u};
                if (row < n_rows) v[j] = load_stream(base + vi);
            }
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const uint64_t b = ballot(nonzero_mag(v[j]) != 0);
                uint64_t rows_bits;
                if (L == 1) {
                    rows_bits = b;
                } else {
                    const uint64_t lmask = (1ull << L) - 1ull;
                    const bool mine = lane < RPL && ((b >> (lane * L)) & lmask) != 0;
                    rows_bits = ballot(mine);
                }
                unit_mask |= rows_bits << (((j0 + j) * RPL) & 63);
            }
        }
        if (lane == 0) {
            s_mask[unit * 2 + 0] = (uint32_t)unit_mask;
            s_mask[unit * 2 + 1] = (uint32_t)(unit_mask >> 32);
        }
    }
}

// Any row_dim: one wave per row, two rows in flight.  VEC = 4 (16-byte loads) or 1.
template <int VEC>
__device__ __forceinline__ uint32_t row_or(const float *__restrict__ row, uint32_t nvec, uint32_t lane)
{
    constexpr int U = ZEN_ROW_UNROLL;
    uint32_t acc = 0;
    for (uint32_t k = lane; k < nvec; k += 64 * U) {
        if (VEC == 4) {
            u32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                v[u] = (u32x4){0u, 0u, 0u, 0u};
                if (k + 64 * u < nvec) v[u] = load_stream((const u32x4 *)row + k + 64 * u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc |= v[u].x | v[u].y | v[u].z | v[u].w;
        } else {
            uint32_t v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                v[u] = 0;
                if (k + 64 * u < nvec) v[u] = __builtin_nontemporal_load((const uint32_t *)row + k + 64 * u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc |= v[u];
        }
    }
    return acc & 0x7fffffffu;
}

template <int VEC>
__device__ __forceinline__ void detect_row(const float *__restrict__ g, uint64_t n_rows, uint32_t row_dim,
                                           uint64_t row0, uint32_t tile_rows, uint32_t *s_mask)
{
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint32_t nvec = row_dim / VEC;
    // s_mask was zeroed by the caller
    for (uint32_t r = wave; r < tile_rows; r += 2 * nw) {
        const uint32_t r2 = r + nw;
        const uint64_t ga = row0 + r, gb = row0 + r2;
        uint32_t a = 0, b = 0;
        if (ga < n_rows) a = row_or<VEC>(g + ga * (uint64_t)row_dim, nvec, lane);
        if (r2 < tile_rows && gb < n_rows) b = row_or<VEC>(g + gb * (uint64_t)row_dim, nvec, lane);
        const bool nza = ballot(a != 0) != 0, nzb = ballot(b != 0) != 0;
        if (lane == 0) {
            if (nza) atomicOr(&s_mask[r >> 5], 1u << (r & 31));
            if (nzb) atomicOr(&s_mask[r2 >> 5], 1u << (r2 & 31));
        }
    }
}

// E1 + E3: one block per (tile, worker).  Writes the tile's mask words and its owner histogram
// hist[tile][0..n_parts).
// PATH: 0 = row_dim 1; 1..6 = 4*2^(PATH-1) floats per row with 2^(PATH-1) lanes per row;
//       7 = wave per row, 16-byte loads; 8 = wave per row, 4-byte loads.  One kernel per path so
//       that each keeps its own register budget (the widest path would set everyone's occupancy).
template <int PATH>
__global__ void __launch_bounds__(DETECT_THREADS)
detect_kernel(Geometry g, GradPtrs grads, uint32_t *mask_base, uint64_t mask_stride_words,
              uint32_t *hist_base, uint64_t hist_stride_words, uint32_t *tflag_base, uint64_t tflag_stride,
              zen_status_info *reset_status, const uint32_t *min_mag, uint32_t seg_flags, const uint32_t *group_base)
{
    // group_base (element-level hash-bitmap contexts, else NULL): rows of every partition below each 512-row
    // boundary -- the owners of a fully non-zero 512-row group are then two table rows' difference, not 512 hashes
    // seg_flags (element-level tiles of SEG_FLAG_WORDS * 32 mask words only): the tile's flag word says which of its
    // 32 segments hold a non-zero row, and only those segments' mask words are written -- for a consumer that
    // reads the mask through the flag word (the scatter).  Otherwise a non-empty tile's flag is all ones.
    // min_mag (element-level inputs only, may be NULL): per worker, the magnitude threshold of a top-k
    // sparsifier applied on the fly -- elements below it are treated as zeros
    extern __shared__ uint32_t smem[];
    uint32_t *s_mask = smem;                  // [tile_words]
    uint32_t *s_hist = smem + g.tile_words;   // [n_parts]
    const uint32_t tile = blockIdx.x, worker = blockIdx.y;
    const float *__restrict__ grad = grads.p[worker];
    const uint64_t row0 = (uint64_t)tile * g.tile_rows;

    if (reset_status && tile == 0 && worker == 0 && threadIdx.x == 0) {
        reset_status->flags = 0; reset_status->reserved = 0; reset_status->needed_rows = 0;
    }
    for (uint32_t i = threadIdx.x; i < g.n_parts; i += blockDim.x) s_hist[i] = 0;
    if (PATH >= 7 || PATH == 0) {
        for (uint32_t i = threadIdx.x; i < g.tile_words; i += blockDim.x) s_mask[i] = 0;
        __syncthreads();
    }

    if (PATH == 0) detect_elem<8>(grad, g.n_rows, row0, g.tile_rows, s_mask, min_mag ? max(min_mag[worker], 1u) : 1u);
    else if (PATH <= 6) detect_sub<(PATH >= 1 && PATH <= 6) ? (1 << (PATH - 1)) : 1>(grad, g.n_rows, row0, g.tile_rows, s_mask);
    else if (PATH == 7) detect_row<4>(grad, g.n_rows, g.row_dim, row0, g.tile_rows, s_mask);
    else detect_row<1>(grad, g.n_rows, g.row_dim, row0, g.tile_rows, s_mask);
    __syncthreads();

    // Tile flag: non-zero iff the tile holds a non-zero row.  Mask words and histogram rows of empty tiles
    // are NOT written (every consumer looks at the flag first): for sparse inputs that removes most
    // of the write traffic, which costs the streaming read far more than its byte share.
    // Used where a tile has many mask words (element-level inputs); elsewhere the mask itself is
    // as small as a flag array would be and everything is always written.
    uint32_t flag_word = 0xFFFFFFFFu;
    if (g.sparse_mask) {
        __shared__ uint32_t s_segbits;
        const bool by_segment = PATH == 0 && seg_flags && g.tile_words == SEG_FLAG_WORDS * 32 && (blockDim.x & 63u) == 0;
        uint32_t any = 0;
        if (threadIdx.x == 0) s_segbits = 0;
        for (uint32_t i = threadIdx.x; i < g.tile_words; i += blockDim.x) any |= s_mask[i];
        const int flag = __syncthreads_or((int)(any != 0));
        if (flag && by_segment) {
            // a wave's 64 consecutive words are two segments
            for (uint32_t i = threadIdx.x; i < g.tile_words; i += blockDim.x) {
                const uint64_t nzb = ballot(s_mask[i] != 0);
                const uint32_t two = ((uint32_t)nzb ? 1u : 0u) | ((uint32_t)(nzb >> 32) ? 2u : 0u);
                if (lane_id() == 0 && two) atomicOr(&s_segbits, two << ((i / SEG_FLAG_WORDS) & 31u));
            }
            __syncthreads();
            flag_word = s_segbits;
        }
        if (threadIdx.x == 0) tflag_base[worker * tflag_stride + tile] = flag ? flag_word : 0u;
        if (!flag) {
            if (!(g.sparse_mask & 2u) && hist_base) {   // histogram rows are kept valid for every tile: a zero row
                uint32_t *gh = hist_base + worker * hist_stride_words + (uint64_t)tile * g.n_parts;
                for (uint32_t i = threadIdx.x; i < g.n_parts; i += blockDim.x) gh[i] = 0u;
            }
            return;
        }
    }
    uint32_t *gmask = mask_base + worker * mask_stride_words + (uint64_t)tile * g.tile_words;
    for (uint32_t i = threadIdx.x; i < g.tile_words; i += blockDim.x)
        if ((flag_word >> ((i / SEG_FLAG_WORDS) & 31u)) & 1u) gmask[i] = s_mask[i];
    if (!hist_base) return;   // the one-block-per-worker partition path hashes the rows itself
    // owner histogram of the tile's non-zero rows: walk the mask words, most of them are zero
    if (PATH == 0 && group_base && (g.tile_words & 63u) == 0 && g.tile_words <= 1024 && (blockDim.x & 63u) == 0) {
        // (long runs of non-zeros) a wave's 64 consecutive words are four groups of 512 rows; a group whose 16 words
        // are all ones is only marked, and partition p's share of every stretch of marked groups is read off the table
        __shared__ uint32_t s_full[2];                        // one bit per group of the tile (<= 64)
        if (threadIdx.x < 2) s_full[threadIdx.x] = 0;
        __syncthreads();
        for (uint32_t wi = threadIdx.x; wi < g.tile_words; wi += blockDim.x) {
            uint32_t word = s_mask[wi];
            const uint64_t ones = ballot(word == 0xFFFFFFFFu);
            const uint32_t l16 = lane_id() & ~15u;
            if (((ones >> l16) & 0xFFFFull) == 0xFFFFull) {
                const uint32_t gi = wi / GROUP_WORDS;
                if ((lane_id() & 15u) == 0) atomicOr(&s_full[gi >> 5], 1u << (gi & 31u));
                continue;
            }
            while (word) {
                const uint32_t b = __ffs(word) - 1;
                word &= word - 1;
                atomicAdd(&s_hist[owner_of((uint32_t)(row0 + wi * 32 + b), g.seed, g.n_parts, g.pow2_mask)], 1u);
            }
        }
        __syncthreads();
        uint64_t m = ((uint64_t)s_full[1] << 32) | s_full[0];
        const uint64_t G0 = row0 / ZEN_GROUP_ROWS;
        while (m) {                                           // uniform: stretches of marked groups
            const uint32_t g0 = (uint32_t)__ffsll((unsigned long long)m) - 1;
            const uint64_t rest = ~(m >> g0);                 // first unmarked group at or after g0 (bit 64 - g0 and up are ones)
            const uint32_t len = rest ? (uint32_t)__ffsll((unsigned long long)rest) - 1 : 64u - g0;
            for (uint32_t p = threadIdx.x; p < g.n_parts; p += blockDim.x)
                s_hist[p] += group_base[(G0 + g0 + len) * g.n_parts + p] - group_base[(G0 + g0) * g.n_parts + p];
            m = (g0 + len >= 64u) ? 0ull : (m >> (g0 + len)) << (g0 + len);
        }
    } else if (g.tile_words >= blockDim.x) {
        for (uint32_t wi = threadIdx.x; wi < g.tile_words; wi += blockDim.x) {
            uint32_t word = s_mask[wi];
            while (word) {
                const uint32_t b = __ffs(word) - 1;
                word &= word - 1;
                atomicAdd(&s_hist[owner_of((uint32_t)(row0 + wi * 32 + b), g.seed, g.n_parts, g.pow2_mask)], 1u);
            }
        }
    } else {
        for (uint32_t r = threadIdx.x; r < g.tile_rows; r += blockDim.x) {
            if ((s_mask[r >> 5] >> (r & 31)) & 1u) {
                const uint32_t p = owner_of((uint32_t)(row0 + r), g.seed, g.n_parts, g.pow2_mask);
                atomicAdd(&s_hist[p], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t *ghist = hist_base + worker * hist_stride_words + (uint64_t)tile * g.n_parts;
    for (uint32_t i = threadIdx.x; i < g.n_parts; i += blockDim.x) ghist[i] = s_hist[i];
}

// ----------------------------------------------------------------------------------------------
// E4: per worker, turn hist[tile][p] into the output position of the first row of (tile, p):
//     base[tile][p] = offsets[p] + sum_{t < tile} hist[t][p],  offsets = exclusive scan of totals.
// One block per worker; thread (grp, p) walks a contiguous range of tiles.
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(SCAN_THREADS)
partition_scan_kernel(Geometry g, EncodedPtrs outs, uint32_t *hist_base, uint64_t hist_stride_words,
                      const uint32_t *tflag_base, uint64_t tflag_stride, uint32_t *tlist_base, uint64_t tlist_stride,
                      zen_status_info *status)
{
    __shared__ uint32_t s_part[SCAN_THREADS];   // [grp][p] partial sums
    __shared__ uint32_t s_off[ZEN_MAX_PARTS + 1];
    __shared__ uint32_t s_tmp[32];
    const uint32_t worker = blockIdx.x;
    uint32_t *hist = hist_base + worker * hist_stride_words;
    const uint32_t *tflag = tflag_base + worker * tflag_stride;   // rows of empty tiles are undefined
    const uint32_t n = g.n_parts;
    const uint32_t n_groups = SCAN_THREADS / n;   // >= 1 since n <= 1024
    const uint32_t p = threadIdx.x % n, grp = threadIdx.x / n;
    const bool active = grp < n_groups;
    const uint32_t per = (g.n_tiles + n_groups - 1) / n_groups;
    const uint32_t t0 = active ? min(grp * per, g.n_tiles) : 0;
    const uint32_t t1 = active ? min(t0 + per, g.n_tiles) : 0;

    // The tile flags as a bit set in LDS (when there are few enough tiles): the walks below would otherwise wait
    // for a flag before they can ask for the histogram row it gates.  No flags: every tile counts.
    __shared__ uint32_t s_fbits[SCAN_FLAG_WORDS];
    const bool fbits = g.n_tiles <= SCAN_FLAG_WORDS * 32;
    if (fbits) {
        const uint32_t lane = lane_id();
        for (uint32_t tb = 0; tb < g.n_tiles; tb += 8 * SCAN_THREADS) {
            uint32_t f[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t t = tb + u * SCAN_THREADS + threadIdx.x;
                f[u] = t < g.n_tiles ? (g.sparse_mask ? tflag[t] : 1u) : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t first = tb + u * SCAN_THREADS + threadIdx.x - lane;   // the wave's first tile
                const uint64_t m = ballot(f[u] != 0);
                if (first < g.n_tiles && lane < 2) s_fbits[(first >> 5) + lane] = (uint32_t)(m >> (32 * lane));
            }
        }
        __syncthreads();
    }
    auto tile_on = [&](uint32_t t) -> bool {      // does tile t have a histogram row?
        if (!(g.sparse_mask & 2u)) return true;
        if (fbits) return (s_fbits[t >> 5] >> (t & 31u)) & 1u;
        return tflag[t] != 0;
    };

    // Batches of 8 tiles: the loads of a batch are independent and issued together (one at a time,
    // this walk is a chain of memory round trips and the kernel runs one block per worker).
    uint32_t sum = 0;
    for (uint32_t tb = t0; tb < t1; tb += 8) {
        uint32_t h[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) {
            const uint32_t t = tb + u;
            h[u] = (t < t1 && tile_on(t)) ? hist[(uint64_t)t * n + p] : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) sum += h[u];
    }
    if (active) s_part[grp * n + p] = sum;
    __syncthreads();
    // exclusive scan over groups for each p (Hillis-Steele along the group axis, all p at once)
    __shared__ uint32_t s_alt[SCAN_THREADS];
    uint32_t *cur = s_part, *nxt = s_alt;
    for (uint32_t d = 1; d < n_groups; d <<= 1) {
        uint32_t v = 0;
        if (active) v = cur[grp * n + p] + (grp >= d ? cur[(grp - d) * n + p] : 0u);
        if (active) nxt[grp * n + p] = v;
        __syncthreads();
        uint32_t *t = cur; cur = nxt; nxt = t;
    }
    // cur = inclusive prefix over groups; totals per p = last group's value
    uint32_t tot_p = 0;
    if (threadIdx.x < n) tot_p = cur[(n_groups - 1) * n + threadIdx.x];
    uint32_t n_total;
    const uint32_t off_p = block_exclusive_scan(tot_p, s_tmp, &n_total);
    if (threadIdx.x < n) s_off[threadIdx.x] = off_p;
    uint32_t my_prefix = 0;   // rows of partition p in the groups before mine
    if (active) my_prefix = cur[grp * n + p] - sum;
    if (threadIdx.x == 0) {
        s_off[n] = n_total;
        if ((uint64_t)n_total > outs.cap_rows[worker]) {
            atomicOr(&status->flags, 1u);
            atomicMax((unsigned long long *)&status->needed_rows, (unsigned long long)n_total);
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) outs.offsets[worker][i] = s_off[i];
    if (active) {
        uint32_t run = s_off[p] + my_prefix;
        for (uint32_t tb = t0; tb < t1; tb += 8) {
            uint32_t h[8];
            bool on[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t t = tb + u;
                on[u] = t < t1 && tile_on(t);
                h[u] = on[u] ? hist[(uint64_t)t * n + p] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                if (on[u]) hist[(uint64_t)(tb + u) * n + p] = run;
                run += h[u];
            }
        }
    }
    // For the scatter: ascending list of the worker's non-empty tiles (all tiles when the geometry
    // carries no tile flags), its length behind it, and behind that the listed tiles' flag words.
    if (tlist_base) {
        uint32_t *tlist = tlist_base + worker * tlist_stride;
        uint32_t listed = 0;
        if (fbits) {
            const uint32_t n_fw = (g.n_tiles + 31) >> 5;      // a thread lists the tiles of one flag word
            for (uint32_t w0 = 0; w0 < n_fw; w0 += blockDim.x) {
                const uint32_t w = w0 + threadIdx.x;
                uint32_t word = w < n_fw ? s_fbits[w] : 0u, total;
                uint32_t at = listed + block_exclusive_scan(__popc(word), s_tmp, &total);
                while (word) {
                    const uint32_t t = w * 32 + (uint32_t)__ffs((int)word) - 1;
                    tlist[(g.n_tiles + 1) + at] = g.sparse_mask ? tflag[t] : 0xFFFFFFFFu;
                    tlist[at++] = t;
                    word &= word - 1;
                }
                listed += total;
            }
        } else
        for (uint32_t t0b = 0; t0b < g.n_tiles; t0b += blockDim.x) {
            const uint32_t t = t0b + threadIdx.x;
            const uint32_t f = (t < g.n_tiles && (!g.sparse_mask || tflag[t])) ? 1u : 0u;
            uint32_t total;
            const uint32_t pre = block_exclusive_scan(f, s_tmp, &total);
            if (f) {
                tlist[listed + pre] = t;
                tlist[(g.n_tiles + 1) + listed + pre] = g.sparse_mask ? tflag[t] : 0xFFFFFFFFu;
            }
            listed += total;
        }
        if (threadIdx.x == 0) {
            tlist[g.n_tiles] = listed;
            tlist[2 * g.n_tiles + 1] = 0;   // length of a second list a consumer may build in place of the flag words
        }
    }
}

// ----------------------------------------------------------------------------------------------
// E4 over the whole chip, for workers with thousands of tiles: the tiles of a worker are cut into slices of
// SLICE_TILES, a block per (slice, worker).  First launch: every slice's per-partition sums and its number of
// non-empty tiles.  Second launch: every block adds up the sums of the slices before its own (and of all
// slices: the offsets), turns its slice's histogram rows into output positions and lists its non-empty tiles
// behind those of the slices before it.  Same results as partition_scan_kernel.
// ----------------------------------------------------------------------------------------------
static constexpr uint32_t SLICE_TILES = 256;
static constexpr uint32_t SLICE_MIN_TILES = 2048;   // fewer tiles per worker: one block per worker does it in one launch

// MODE 0: sums only (slice_sums[worker][slice][n_parts + 1], the last word = listed tiles of the slice);
// MODE 1: positions, offsets, tile list.
template <int MODE>
__global__ void __launch_bounds__(SCAN_THREADS)
partition_slice_kernel(Geometry g, EncodedPtrs outs, uint32_t *hist_base, uint64_t hist_stride_words,
                       const uint32_t *tflag_base, uint64_t tflag_stride, uint32_t *tlist_base, uint64_t tlist_stride,
                       uint32_t *slice_sums, zen_status_info *status)
{
    __shared__ uint32_t s_part[SCAN_THREADS];   // [grp][p] partial sums
    __shared__ uint32_t s_alt[SCAN_THREADS];
    __shared__ uint32_t s_off[ZEN_MAX_PARTS + 1];
    __shared__ uint32_t s_base[ZEN_MAX_PARTS];  // rows of partition p in the slices before this one
    __shared__ uint32_t s_flag[SLICE_TILES];
    __shared__ uint32_t s_tmp[32];
    const uint32_t slice = blockIdx.x, n_slices = gridDim.x, worker = blockIdx.y;
    uint32_t *hist = hist_base + worker * hist_stride_words;
    const uint32_t *tflag = tflag_base + worker * tflag_stride;   // rows of empty tiles are undefined
    uint32_t *sums = slice_sums + (uint64_t)worker * n_slices * (g.n_parts + 1);
    const uint32_t n = g.n_parts;
    const uint32_t T0 = slice * SLICE_TILES, T1 = min(T0 + SLICE_TILES, g.n_tiles);
    const uint32_t n_groups = min((uint32_t)SCAN_THREADS / n, SLICE_TILES);   // >= 1 since n <= 1024
    const uint32_t p = threadIdx.x % n, grp = threadIdx.x / n;
    const bool active = grp < n_groups;
    const uint32_t per = (SLICE_TILES + n_groups - 1) / n_groups;
    const uint32_t t0 = active ? min(T0 + grp * per, T1) : 0;
    const uint32_t t1 = active ? min(t0 + per, T1) : 0;

    uint32_t listed_here = 0;
    for (uint32_t i = threadIdx.x; i < SLICE_TILES; i += SCAN_THREADS) {
        const uint32_t t = T0 + i;
        const uint32_t f = t < T1 ? (g.sparse_mask ? tflag[t] : 0xFFFFFFFFu) : 0u;
        s_flag[i] = f;
        listed_here += f ? 1u : 0u;
    }
    __syncthreads();
    auto tile_on = [&](uint32_t t) -> bool { return !(g.sparse_mask & 2u) || s_flag[t - T0] != 0; };   // has a histogram row?

    uint32_t sum = 0;
    for (uint32_t tb = t0; tb < t1; tb += 8) {
        uint32_t h[8];
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) {
            const uint32_t t = tb + u;
            h[u] = (t < t1 && tile_on(t)) ? hist[(uint64_t)t * n + p] : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < 8; ++u) sum += h[u];
    }
    if (active) s_part[grp * n + p] = sum;
    __syncthreads();
    // inclusive scan over groups for each p (Hillis-Steele along the group axis, all p at once)
    uint32_t *cur = s_part, *nxt = s_alt;
    for (uint32_t d = 1; d < n_groups; d <<= 1) {
        uint32_t v = 0;
        if (active) v = cur[grp * n + p] + (grp >= d ? cur[(grp - d) * n + p] : 0u);
        if (active) nxt[grp * n + p] = v;
        __syncthreads();
        uint32_t *t = cur; cur = nxt; nxt = t;
    }
    if (MODE == 0) {
        if (threadIdx.x < n) sums[(uint64_t)slice * (n + 1) + threadIdx.x] = cur[(n_groups - 1) * n + threadIdx.x];
        uint32_t total;
        block_exclusive_scan(listed_here, s_tmp, &total);
        if (threadIdx.x == 0) sums[(uint64_t)slice * (n + 1) + n] = total;
        return;
    }
    // totals of all slices and of the slices before this one, per partition (thread p) and for the tile list
    uint32_t tot_p = 0, before_p = 0;
    if (threadIdx.x < n) {
        for (uint32_t s0 = 0; s0 < n_slices; s0 += 8) {
            uint32_t v[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) v[u] = s0 + u < n_slices ? sums[(uint64_t)(s0 + u) * (n + 1) + threadIdx.x] : 0u;
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                tot_p += v[u];
                if (s0 + u < slice) before_p += v[u];
            }
        }
        s_base[threadIdx.x] = before_p;
    }
    uint32_t listed_before = 0, listed_all = 0;    // (uniform: every thread adds up the same few words)
    for (uint32_t s0 = 0; s0 < n_slices; ++s0) {
        const uint32_t v = sums[(uint64_t)s0 * (n + 1) + n];
        listed_all += v;
        if (s0 < slice) listed_before += v;
    }
    uint32_t n_total;
    const uint32_t off_p = block_exclusive_scan(tot_p, s_tmp, &n_total);
    if (threadIdx.x < n) s_off[threadIdx.x] = off_p;
    uint32_t my_prefix = 0;   // rows of partition p in the groups before mine
    if (active) my_prefix = cur[grp * n + p] - sum;
    if (threadIdx.x == 0) {
        s_off[n] = n_total;
        if (slice == 0 && (uint64_t)n_total > outs.cap_rows[worker]) {
            atomicOr(&status->flags, 1u);
            atomicMax((unsigned long long *)&status->needed_rows, (unsigned long long)n_total);
        }
    }
    __syncthreads();
    if (slice == 0)
        for (uint32_t i = threadIdx.x; i <= n; i += blockDim.x) outs.offsets[worker][i] = s_off[i];
    if (active) {
        uint32_t run = s_off[p] + s_base[p] + my_prefix;
        for (uint32_t tb = t0; tb < t1; tb += 8) {
            uint32_t h[8];
            bool on[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t t = tb + u;
                on[u] = t < t1 && tile_on(t);
                h[u] = on[u] ? hist[(uint64_t)t * n + p] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                if (on[u]) hist[(uint64_t)(tb + u) * n + p] = run;
                run += h[u];
            }
        }
    }
    if (tlist_base) {
        uint32_t *tlist = tlist_base + worker * tlist_stride;
        for (uint32_t i0 = 0; i0 < SLICE_TILES; i0 += blockDim.x) {       // one pass: SLICE_TILES <= blockDim.x
            const uint32_t i = i0 + threadIdx.x;
            const uint32_t f = i < SLICE_TILES ? s_flag[i] : 0u;
            uint32_t total;
            const uint32_t at = listed_before + block_exclusive_scan(f ? 1u : 0u, s_tmp, &total);
            if (f) {
                tlist[at] = T0 + i;
                tlist[(g.n_tiles + 1) + at] = f;
            }
            listed_before += total;
        }
        if (slice == 0 && threadIdx.x == 0) {
            tlist[g.n_tiles] = listed_all;
            tlist[2 * g.n_tiles + 1] = 0;   // length of a second list a consumer may build in place of the flag words
        }
    }
}

// ----------------------------------------------------------------------------------------------
// E5 + E6 (+E7): blocks walk (tile, worker) pairs.  For every non-empty tile: expand the mask in
// segments to an ascending row list in LDS, rank every row stably inside its partition, write the
// index, copy the row's values, and (hash-bitmap format) set the row's bit.
//
// Hash bitmap (Algorithm 2, hash_bitmap_encode): bit rank[row] of partition p, where rank[row] is
// the row's position in the sorted domain II_p.  The bits of one (tile, partition) are contiguous
// -- [tile_base[tile][p], tile_base[tile+1][p]) -- so they are assembled in LDS and flushed with
// plain stores; only the first / last word of a range can be shared with a neighbouring tile and
// goes out with atomicOr.  The bitmap must be zero before the kernel runs.
// ----------------------------------------------------------------------------------------------
struct BitmapTables {
    const uint32_t *rank;       // [n_rows]
    const uint32_t *tile_base;  // [n_tiles+1][n_parts]
    const uint32_t *word_off;   // [n_parts+1]
    const uint32_t *group_base; // [n_tiles * tile_rows / ZEN_GROUP_ROWS + 1][n_parts] rows of II_p below each group of
                                // ZEN_GROUP_ROWS rows, or NULL
};

// ELEM = (row_dim == 1): values are single floats fetched ahead of the ranking loop; otherwise rows
// are copied after it.  Two instantiations so that each keeps its own register budget.
#ifndef ZEN_COPY_UNROLL
#define ZEN_COPY_UNROLL 4   // 16-byte vectors a thread of the narrow-row copy keeps in flight (1, 2, 8 measured slower)
#endif
#ifndef ZEN_SCATTER_WAVES
#define ZEN_SCATTER_WAVES 6   // waves per SIMD the register allocation must allow: 6 measured best (8 spills)
#endif
#ifndef ZEN_SCATTER_WAVES_ELEM
#define ZEN_SCATTER_WAVES_ELEM 4   // element-level: the staged output keeps more values in registers (5 spills, and measures slower)
#endif
template <bool ELEM>
__global__ void __launch_bounds__(SCATTER_THREADS, ELEM ? ZEN_SCATTER_WAVES_ELEM : ZEN_SCATTER_WAVES)
scatter_kernel(Geometry g, GradPtrs grads, EncodedPtrs outs, const uint32_t *mask_base,
               uint64_t mask_stride_words, const uint32_t *hist_base, uint64_t hist_stride_words,
               const uint32_t *tlist_base, uint64_t tlist_stride, BitmapTables bt)
{
    extern __shared__ uint32_t smem[];
    const uint32_t n = g.n_parts, D = g.row_dim;
    uint32_t *s_run = smem;                          // [n]
    const uint32_t n_waves = blockDim.x >> 6;
    uint32_t *s_cnt = s_run + n;                     // [n_waves][n]
    uint32_t *s_list = s_cnt + n_waves * n;                // [SEG_ROWS] row ids of the segment, ascending
    uint32_t *s_pos = s_list + SEG_ROWS;             // [SEG_ROWS] output position of each listed row (row copies), or the
                                                     //            values of a fully non-zero stretch in output order
    uint32_t *s_tmp = s_pos + SEG_ROWS;              // [32]
    uint32_t *s_mask = s_tmp + 32;                   // [tile_words] the tile's mask
    uint32_t *s_seg = s_mask + g.tile_words;         // [ceil(tile_words / GROUP_WORDS)] rows of each 16-word group
    uint32_t *s_delta = s_seg + (g.tile_words + GROUP_WORDS - 1) / GROUP_WORDS;   // [n] \ element-level: per-partition terms
    uint32_t *s_goff = s_delta + n;                  // [n] / that turn a rank into an LDS slot and an output position
    uint32_t *s_b0 = s_goff + n;                     // bitmap only: [n] first bit of (tile, p)
    uint32_t *s_b1 = s_b0 + n;                       //              [n] end bit of (tile, p)
    uint32_t *s_boff = s_b1 + n;                     //              [n+1] LDS word offset of p's range
    uint32_t *s_bm = s_boff + n + 1;                 //              [tile_words + 2n] assembled words
    const uint32_t worker = blockIdx.y;
    const float *__restrict__ grad = grads.p[worker];
    uint32_t *__restrict__ out_idx = outs.indices[worker];
    float *__restrict__ out_val = outs.values[worker];
    uint32_t *__restrict__ out_bm = outs.bitmap[worker];
    const uint64_t cap = outs.cap_rows[worker];
    const bool bitmap = g.bitmap && out_bm != nullptr;
    const bool fast_ok = ELEM && bt.group_base != nullptr && bt.rank != nullptr;

    for (uint32_t i = threadIdx.x; i < n_waves * n; i += blockDim.x) s_cnt[i] = 0;

    // Tiles to visit: the ascending list of the worker's non-empty tiles (every tile, each tested here, for the
    // wave-per-row geometry, which carries no tile flags).  Element-level inputs: the mask of the next tile is
    // fetched into registers while the current one is processed, its id one visit earlier still.
    const uint32_t *tlist = tlist_base + worker * tlist_stride;
    const uint32_t n_visit = min(tlist[g.n_tiles], g.n_tiles);
    const uint32_t *wmask = mask_base + worker * mask_stride_words;
    const bool pf_ok = g.tile_words <= 8 * SCATTER_THREADS;   // 8 registers per thread hold a tile's mask
    uint32_t mw[8];
#pragma unroll
    for (uint32_t q = 0; q < 8; ++q) mw[q] = 0;
    uint32_t k = blockIdx.x;
    uint32_t nxt_tile = k < n_visit ? min(tlist[k], g.n_tiles - 1) : 0u;
    uint32_t nxt2_tile = k + gridDim.x < n_visit ? min(tlist[k + gridDim.x], g.n_tiles - 1) : 0u;
    // element-level: the listed tiles' flag words (behind the list) say which 32-word segments of a tile's mask
    // were written; the others read as zero
    const uint32_t *tlflag = tlist + (g.n_tiles + 1);
    uint32_t nxt_flag = (ELEM && k < n_visit) ? tlflag[k] : 0u;
    uint32_t nxt2_flag = (ELEM && k + gridDim.x < n_visit) ? tlflag[k + gridDim.x] : 0u;
    auto seg_written = [](uint32_t flag_word, uint32_t i) -> bool { return (flag_word >> ((i / SEG_FLAG_WORDS) & 31u)) & 1u; };
    if (ELEM && pf_ok && k < n_visit) {
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) {
            const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
            if (i < g.tile_words && seg_written(nxt_flag, i)) mw[q] = wmask[(uint64_t)nxt_tile * g.tile_words + i];
        }
    }
    // element-level, at most one partition per thread: the tile's positions and bit ranges are fetched a tile ahead too
    const bool pf_part = ELEM && n <= SCATTER_THREADS;
    const uint32_t *whist = hist_base + worker * hist_stride_words;
    uint32_t pf_h = 0, pf_b0 = 0, pf_b1 = 0;
    if (pf_part && threadIdx.x < n && k < n_visit) {
        pf_h = whist[(uint64_t)nxt_tile * n + threadIdx.x];
        if (bitmap) {
            pf_b0 = bt.tile_base[(uint64_t)nxt_tile * n + threadIdx.x];
            pf_b1 = bt.tile_base[(uint64_t)(nxt_tile + 1) * n + threadIdx.x];
        }
    }
    for (; k < n_visit; k += gridDim.x) {
        const uint32_t tile = nxt_tile, tile_flag = nxt_flag;
        const uint32_t *gmask = wmask + (uint64_t)tile * g.tile_words;
        const uint32_t cur_h = pf_h, cur_b0 = pf_b0, cur_b1 = pf_b1;
        if (ELEM) {
            __syncthreads();                                   // the barrier between tiles
            // The tile's mask goes to LDS with a row count per 16-word group: empty groups then cost neither a
            // memory access nor a barrier, and sparse neighbours are expanded together.
            for (uint32_t q0 = 0; q0 * SCATTER_THREADS < g.tile_words; q0 += 8) {
                if (!pf_ok) {
#pragma unroll
                    for (uint32_t q = 0; q < 8; ++q) {
                        const uint32_t i = (q0 + q) * SCATTER_THREADS + threadIdx.x;
                        mw[q] = (i < g.tile_words && seg_written(tile_flag, i)) ? gmask[i] : 0u;
                    }
                }
#pragma unroll
                for (uint32_t q = 0; q < 8; ++q) {
                    const uint32_t i = (q0 + q) * SCATTER_THREADS + threadIdx.x;
                    const uint32_t first = i - lane_id();      // the wave's 64 words are four groups
                    if (first >= g.tile_words) continue;       // uniform per wave
                    if (i < g.tile_words) s_mask[i] = mw[q];
                    uint32_t grp_cnt = __popc(mw[q]);   // rows of the 16-word group
#pragma unroll
                    for (int d = GROUP_WORDS / 2; d > 0; d >>= 1) grp_cnt += __shfl_xor(grp_cnt, d, ZEN_WAVE);
                    if ((lane_id() & (GROUP_WORDS - 1)) == 0 && i < g.tile_words) s_seg[i / GROUP_WORDS] = grp_cnt;
                }
            }
            nxt_tile = nxt2_tile;
            nxt_flag = nxt2_flag;
            const uint32_t k2 = k + 2 * gridDim.x;
            nxt2_tile = k2 < n_visit ? min(tlist[k2], g.n_tiles - 1) : 0u;
            nxt2_flag = k2 < n_visit ? tlflag[k2] : 0u;
            if (pf_ok && k + gridDim.x < n_visit) {
#pragma unroll
                for (uint32_t q = 0; q < 8; ++q) {
                    const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                    mw[q] = (i < g.tile_words && seg_written(nxt_flag, i)) ? wmask[(uint64_t)nxt_tile * g.tile_words + i] : 0u;
                }
            }
            if (pf_part && threadIdx.x < n && k + gridDim.x < n_visit) {
                pf_h = whist[(uint64_t)nxt_tile * n + threadIdx.x];
                if (bitmap) {
                    pf_b0 = bt.tile_base[(uint64_t)nxt_tile * n + threadIdx.x];
                    pf_b1 = bt.tile_base[(uint64_t)(nxt_tile + 1) * n + threadIdx.x];
                }
            }
            __syncthreads();
        } else {
            nxt_tile = nxt2_tile;
            const uint32_t k2 = k + 2 * gridDim.x;
            nxt2_tile = k2 < n_visit ? min(tlist[k2], g.n_tiles - 1) : 0u;
            if (g.sparse_mask) {
                __syncthreads();                               // listed tiles hold rows: only the barrier between tiles
            } else {
                uint32_t any = 0;
                for (uint32_t i = threadIdx.x; i < g.tile_words; i += blockDim.x) any |= gmask[i];
                if (!__syncthreads_or((int)(any != 0))) continue;  // empty tile (also the barrier between tiles)
            }
        }

        const uint32_t *ghist = whist + (uint64_t)tile * n;
        const uint64_t row0 = (uint64_t)tile * g.tile_rows;
        if (pf_part) { if (threadIdx.x < n) s_run[threadIdx.x] = cur_h; }
        else for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) s_run[i] = ghist[i];

        if (bitmap) {
            // per-partition bit ranges of this tile and their LDS placement (what follows meets a barrier
            // before it uses them)
            const uint32_t *tb0 = bt.tile_base + (uint64_t)tile * n, *tb1 = tb0 + n;
            if (n <= ZEN_WAVE) {                    // the first wave alone: a scan without block barriers
                if (threadIdx.x < ZEN_WAVE) {
                    const uint32_t p = threadIdx.x;
                    uint32_t b0 = 0, b1 = 0;
                    if (p < n) { b0 = pf_part ? cur_b0 : tb0[p]; b1 = pf_part ? cur_b1 : tb1[p]; }
                    const uint32_t wcnt = b1 > b0 ? ((b1 - 1) >> 5) - (b0 >> 5) + 1 : 0;
                    const uint32_t inc = wave_inclusive_scan(wcnt);
                    if (p < n) { s_b0[p] = b0; s_b1[p] = b1; s_boff[p] = inc - wcnt; }
                    if (p == n - 1) s_boff[n] = inc;
                }
            } else {
            uint32_t bm_words = 0;
            const uint32_t per = (n + blockDim.x - 1) / blockDim.x;   // consecutive partitions per thread
            const uint32_t p0 = min(threadIdx.x * per, n), p1 = min(p0 + per, n);
            uint32_t mine = 0;
            for (uint32_t p = p0; p < p1; ++p) {
                const uint32_t b0 = pf_part ? cur_b0 : tb0[p], b1 = pf_part ? cur_b1 : tb1[p];   // (then per = 1: p = threadIdx.x)
                s_b0[p] = b0;
                s_b1[p] = b1;
                mine += b1 > b0 ? ((b1 - 1) >> 5) - (b0 >> 5) + 1 : 0;
            }
            uint32_t off = block_exclusive_scan(mine, s_tmp, &bm_words);
            for (uint32_t p = p0; p < p1; ++p) {
                const uint32_t b0 = s_b0[p], b1 = s_b1[p];
                s_boff[p] = off;
                off += b1 > b0 ? ((b1 - 1) >> 5) - (b0 >> 5) + 1 : 0;
            }
            if (threadIdx.x == 0) s_boff[n] = bm_words;
            }
            for (uint32_t i = threadIdx.x; i < g.tile_words + 2 * n; i += blockDim.x) s_bm[i] = 0;
        }

        const uint32_t seg_words = ELEM ? GROUP_WORDS : SEG_WORDS;
        const uint32_t n_seg = (g.tile_words + seg_words - 1) / seg_words;
        // element-level: the groups' row counts are held 64 at a time, lane j that of group cur_blk + j, with
        // the non-empty and the fully non-zero ones as wave-uniform bit masks (empty groups cost nothing)
        uint32_t cur_blk = 0xFFFFFFFFu, cnt_l = 0;
        uint64_t nz_m = 0, full_m = 0;
        uint32_t cur = 0;   // element-level: row offset inside the tile below which everything is done
        uint32_t prev_rb = 0xFFFFFFFFu, prev_fb = 0;   // end of the last stretch placed from the rank tables, and (thread p)
                                                       // the rank of partition p's first row at or after it
        for (uint32_t sg = 0; sg < n_seg;) {
            // (a) expand mask words into the ascending row list: 64 words at a time, or -- element-level
            // inputs -- as many consecutive 16-word groups as together hold at most SEG_ROWS rows (a
            // uniformly sparse tile is then one pass instead of sixteen)
            uint32_t w0 = sg * seg_words, w1 = min(w0 + seg_words, g.tile_words), total;
            uint32_t first_mask = 0xFFFFFFFFu;   // element-level: bits of word w0 that belong to this piece
            if (ELEM) {
                sg = cur / ZEN_GROUP_ROWS;
                if (sg >= n_seg) break;
                const uint32_t gblk = sg & ~63u, j = sg & 63u, lane = lane_id();
                if (gblk != cur_blk) {
                    cur_blk = gblk;
                    cnt_l = gblk + lane < n_seg ? s_seg[gblk + lane] : 0u;
                    nz_m = ballot(cnt_l != 0);
                    full_m = fast_ok ? ballot(cnt_l == ZEN_GROUP_ROWS) : 0ull;
                }
                // first listed row at or after cur: in cur's group, else in the next non-empty group
                const uint64_t later = j == 63u ? 0ull : nz_m & (~0ull << (j + 1));
                const uint32_t next_grp_row = (later ? gblk + (uint32_t)__ffsll((unsigned long long)later) - 1 : gblk + 64) * ZEN_GROUP_ROWS;
                if (!((nz_m >> j) & 1ull)) { cur = next_grp_row; continue; }
                uint32_t a;
                {
                    const uint32_t wi = sg * GROUP_WORDS + (lane & (GROUP_WORDS - 1)), cw = cur >> 5;
                    uint32_t wd = (lane < GROUP_WORDS && wi < g.tile_words && wi >= cw) ? s_mask[wi] : 0u;
                    if (wi == cw) wd &= 0xFFFFFFFFu << (cur & 31u);
                    const uint64_t m = ballot(wd != 0);
                    if (m == 0) { cur = next_grp_row; continue; }
                    const uint32_t z = (uint32_t)__ffsll((unsigned long long)m) - 1;
                    a = (sg * GROUP_WORDS + z) * 32 + (uint32_t)__ffs((int)__builtin_amdgcn_readlane((int)wd, (int)z)) - 1;
                }
                // end of the stretch of listed rows that starts at a (looked for in the next 64 words)
                uint32_t b = a;
                if (fast_ok) {
                    const uint32_t aw = a >> 5;
                    uint32_t inv = aw + lane < g.tile_words ? ~s_mask[aw + lane] : 0xFFFFFFFFu;
                    if (lane == 0) inv &= 0xFFFFFFFFu << (a & 31u);
                    const uint64_t zm = ballot(inv != 0);
                    if (zm == 0) {
                        b = (aw + ZEN_WAVE) * 32;
                    } else {
                        const uint32_t z = (uint32_t)__ffsll((unsigned long long)zm) - 1;
                        b = (aw + z) * 32 + (uint32_t)__ffs((int)__builtin_amdgcn_readlane((int)inv, (int)z)) - 1;
                    }
                    if (b - a > SEG_ROWS) b = a + SEG_ROWS;
                }
                if (b - a >= MIN_STRETCH_ROWS) {
                    // (a') A stretch [A, B) of rows that are all listed: the rows of partition p among them are a
                    // contiguous piece of its sorted domain II_p, from the rank of p's first row at or after A to
                    // that at or after B -- the table's value at the 512-row boundary below plus the owners of the
                    // rows from that boundary on, which only have to be hashed.  Output position = running
                    // position + (rank in II_p - first rank); the bits of p are one contiguous range.  No list,
                    // no ranking.  Values are first placed in LDS in output order (partition-major), then
                    // written out: consecutive lanes store to consecutive addresses, not one cache line each.
                    const uint32_t ra = (uint32_t)(row0 + a), rb = (uint32_t)(row0 + b), cnt = b - a;   // cnt <= SEG_ROWS
                    cur = b;
                    constexpr uint32_t FB = SEG_ROWS / SCATTER_THREADS;   // 8 rows per thread
                    float fv[FB];
                    uint32_t fr[FB];
#pragma unroll
                    for (uint32_t q = 0; q < FB; ++q) {
                        const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                        fv[q] = 0.f;
                        fr[q] = 0;
                        if (i < cnt) {
                            fr[q] = bt.rank[ra + i];
                            if (out_val) fv[q] = grad[ra + i];
                        }
                    }
                    // n <= ZEN_GROUP_MAX_PARTS <= blockDim.x: one thread per partition.  A stretch that starts where
                    // the last one ended (a run longer than SEG_ROWS) takes over its end ranks.
                    const bool carry = ra == prev_rb;     // uniform
                    uint32_t fa = prev_fb, fb = 0;
                    if (threadIdx.x < n) {
                        if (!carry) fa = bt.group_base[(uint64_t)(ra / ZEN_GROUP_ROWS) * n + threadIdx.x];
                        fb = bt.group_base[(uint64_t)(rb / ZEN_GROUP_ROWS) * n + threadIdx.x];
                    }
                    uint32_t pp[FB];                      // owners, hashed while the loads are under way
#pragma unroll
                    for (uint32_t q = 0; q < FB; ++q) pp[q] = owner_of(ra + q * SCATTER_THREADS + threadIdx.x, g.seed, n, g.pow2_mask);
                    if (!carry)
                        for (uint32_t r = (ra & ~(ZEN_GROUP_ROWS - 1)) + threadIdx.x; r < ra; r += SCATTER_THREADS)
                            atomicAdd(&s_cnt[owner_of(r, g.seed, n, g.pow2_mask)], 1u);
                    for (uint32_t r = (rb & ~(ZEN_GROUP_ROWS - 1)) + threadIdx.x; r < rb; r += SCATTER_THREADS)
                        atomicAdd(&s_cnt[n + owner_of(r, g.seed, n, g.pow2_mask)], 1u);
                    __syncthreads();
                    if (threadIdx.x < n) {
                        fa += s_cnt[threadIdx.x];        // (zero when the ranks were taken over)
                        fb += s_cnt[n + threadIdx.x];
                        s_cnt[threadIdx.x] = 0;          // the ranking scratch is all zero between its uses
                        s_cnt[n + threadIdx.x] = 0;
                    }
                    prev_rb = rb;
                    prev_fb = fb;
                    uint32_t loff;                       // rows of the partitions before mine in this stretch
                    if (n <= ZEN_WAVE) {                 // the first wave alone, no block barrier
                        loff = threadIdx.x < ZEN_WAVE ? wave_inclusive_scan(fb - fa) - (fb - fa) : 0u;
                    } else {
                        uint32_t stretch_rows;
                        loff = block_exclusive_scan(fb - fa, s_tmp, &stretch_rows);
                    }
                    if (threadIdx.x < n) {
                        const uint32_t p = threadIdx.x, run = s_run[p];
                        s_delta[p] = loff - fa;          // LDS slot   = s_delta[p] + rank
                        s_goff[p] = run - loff;          // output pos = s_goff[p] + slot
                        s_run[p] = run + (fb - fa);
                        if (bitmap && fb > fa) {
                            const uint32_t lw0 = s_boff[p], tw0 = s_b0[p] >> 5;   // LDS word of the tile's first word of p
                            const uint32_t wa = fa >> 5, wb = (fb - 1) >> 5;
                            for (uint32_t w = wa; w <= wb; ++w) {
                                uint32_t m = 0xFFFFFFFFu;
                                if (w == wa) m &= 0xFFFFFFFFu << (fa & 31u);
                                if (w == wb) m &= 0xFFFFFFFFu >> (31u - ((fb - 1) & 31u));
                                s_bm[lw0 + (w - tw0)] |= m;
                            }
                        }
                    }
                    __syncthreads();
#pragma unroll
                    for (uint32_t q = 0; q < FB; ++q) {
                        const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                        if (i < cnt) {
                            const uint32_t row = ra + i;
                            const uint32_t p = pp[q];
                            const uint32_t slot = s_delta[p] + fr[q];
                            const uint32_t pos = s_goff[p] + slot;
                            if (slot < SEG_ROWS) {       // always, for consistent tables
                                s_list[slot] = pos;
                                s_pos[slot] = __float_as_uint(fv[q]);
                            }
                            if (out_idx && pos < cap) out_idx[pos] = row;
                        }
                    }
                    __syncthreads();
                    if (out_val) {
                        for (uint32_t i = threadIdx.x; i < cnt; i += SCATTER_THREADS) {
                            const uint32_t pos = s_list[i];
                            if (pos < cap) out_val[pos] = __uint_as_float(s_pos[i]);
                        }
                    }
                    __syncthreads();   // s_list, s_pos, s_delta, s_goff, s_run are rewritten by what follows
                    continue;
                }
                // scattered rows: the rest of this group and the following non-empty groups, as long as none is
                // fully non-zero and the rows fit (counts of a group partly done already only over-estimate)
                uint32_t merged = (uint32_t)__builtin_amdgcn_readlane((int)cnt_l, (int)j);
                uint32_t e = j + 1;
                uint64_t rest = later;
                while (rest) {
                    const uint32_t j2 = (uint32_t)__ffsll((unsigned long long)rest) - 1;
                    if ((full_m >> j2) & 1ull) break;
                    const uint32_t c2 = (uint32_t)__builtin_amdgcn_readlane((int)cnt_l, (int)j2);
                    if (merged + c2 > SEG_ROWS) break;
                    merged += c2;
                    e = j2 + 1;
                    rest &= rest - 1;
                }
                cur = (gblk + e) * ZEN_GROUP_ROWS;
                w0 = a >> 5;
                first_mask = 0xFFFFFFFFu << (a & 31u);
                w1 = min((gblk + e) * seg_words, g.tile_words);
                const uint32_t wpt = (w1 - w0 + SCATTER_THREADS - 1) / SCATTER_THREADS;   // consecutive words per thread
                const uint32_t wa = min(w0 + threadIdx.x * wpt, w1), wb = min(wa + wpt, w1);
                uint32_t mine = 0;
                for (uint32_t wi = wa; wi < wb; ++wi) mine += __popc(s_mask[wi] & (wi == w0 ? first_mask : 0xFFFFFFFFu));
                uint32_t k = block_exclusive_scan(mine, s_tmp, &total);
                for (uint32_t wi = wa; wi < wb; ++wi) {
                    uint32_t word = s_mask[wi] & (wi == w0 ? first_mask : 0xFFFFFFFFu);
                    const uint32_t rbase = (uint32_t)(row0 + (uint64_t)wi * 32);
                    while (word) {
                        const uint32_t b = __ffs(word) - 1;
                        word &= word - 1;
                        s_list[k++] = rbase + b;
                    }
                }
            } else {
                ++sg;
                uint32_t word = 0;
                if (threadIdx.x < SEG_WORDS && w0 + threadIdx.x < g.tile_words) word = gmask[w0 + threadIdx.x];
                const uint32_t pre = block_exclusive_scan(threadIdx.x < SEG_WORDS ? __popc(word) : 0u, s_tmp, &total);
                if (total == 0) continue;   // uniform: total comes from LDS
                if (threadIdx.x < SEG_WORDS) {
                    uint32_t k = pre;
                    const uint32_t rbase = (uint32_t)(row0 + (uint64_t)(w0 + threadIdx.x) * 32);
                    while (word) {
                        const uint32_t b = __ffs(word) - 1;
                        word &= word - 1;
                        s_list[k++] = rbase + b;
                    }
                }
            }
            if (ELEM)
                for (uint32_t p = threadIdx.x; p < n; p += blockDim.x) s_delta[p] = s_run[p];   // positions at the segment's start
            __syncthreads();
            // (b) rank, write indices, set bitmap bits.  row_dim == 1: the value and the bitmap rank of
            // up to PF chunks are fetched first so the barrier-paced ranking loop does not wait on them.
            constexpr uint32_t PF = SEG_ROWS / SCATTER_THREADS;   // 8
            const bool prefetch = ELEM;
            float pf_val[PF];
            uint32_t pf_bit[PF], pf_pk[PF];
#pragma unroll
            for (uint32_t q = 0; q < PF; ++q) pf_pk[q] = 0;
            if (ELEM) {
#pragma unroll
                for (uint32_t q = 0; q < PF; ++q) {
                    const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                    pf_val[q] = 0.f;
                    pf_bit[q] = 0;
                    if (i < total) {
                        const uint32_t row = s_list[i];
                        if (out_val) pf_val[q] = grad[row];
                        if (bitmap) pf_bit[q] = bt.rank[row];
                    }
                }
            }
            // total <= SEG_ROWS: at most PF chunks when the block has SCATTER_THREADS threads
#pragma unroll
            for (uint32_t q = 0; q < PF; ++q) {
                const uint32_t c = q * blockDim.x;
                if (c >= total) break;                      // uniform
                const uint32_t i = c + threadIdx.x;
                const bool valid = i < total;
                const uint32_t row = valid ? s_list[i] : 0u;
                const uint32_t p = valid ? owner_of(row, g.seed, n, g.pow2_mask) : 0u;
                const uint32_t pos = block_stable_rank(valid, p, g.part_bits, n, s_run, s_cnt);
                if (valid) {
                    if (ELEM) {
                        // partition and position inside the segment's share of it (< SEG_ROWS = 2^11)
                        pf_pk[q] = (p << 11) | (pos - s_delta[p]);
                    } else if (pos < cap) {
                        if (out_idx) out_idx[pos] = row;
                        s_pos[i] = pos;
                    } else {
                        s_pos[i] = 0xFFFFFFFFu;
                    }
                    if (bitmap) {
                        const uint32_t bit = prefetch ? pf_bit[q] : bt.rank[row];
                        atomicOr(&s_bm[s_boff[p] + (bit >> 5) - (s_b0[p] >> 5)], 1u << (bit & 31));
                    }
                }
            }
            if (ELEM) {
                // (b') Indices and values go out in output order: they are first placed in LDS partition-major
                // (slot = start of the partition's share + position inside it), then consecutive lanes store
                // to consecutive addresses -- not one cache line per lane, which is what bounds this kernel.
                __syncthreads();                              // the last chunk's update of s_run
                const uint32_t per = (n + blockDim.x - 1) / blockDim.x;   // consecutive partitions per thread
                const uint32_t p0 = min(threadIdx.x * per, n), p1 = min(p0 + per, n);
                uint32_t mine = 0, seg_total;
                for (uint32_t p = p0; p < p1; ++p) mine += s_run[p] - s_delta[p];
                uint32_t off = block_exclusive_scan(mine, s_tmp, &seg_total);
                for (uint32_t p = p0; p < p1; ++p) { s_goff[p] = off; off += s_run[p] - s_delta[p]; }
                __syncthreads();
                if (out_idx) {
#pragma unroll
                    for (uint32_t q = 0; q < PF; ++q) {
                        const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                        if (i < total) s_pos[s_goff[pf_pk[q] >> 11] + (pf_pk[q] & 2047u)] = s_list[i];
                    }
                    __syncthreads();
                }
#pragma unroll
                for (uint32_t q = 0; q < PF; ++q) {           // the row list is no longer needed: positions replace it
                    const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                    if (i < total) {
                        const uint32_t p = pf_pk[q] >> 11, l = pf_pk[q] & 2047u;
                        s_list[s_goff[p] + l] = s_delta[p] + l;
                    }
                }
                __syncthreads();
                if (out_idx) {
                    for (uint32_t i = threadIdx.x; i < total; i += SCATTER_THREADS) {
                        const uint32_t pos = s_list[i];
                        if (pos < cap) out_idx[pos] = s_pos[i];
                    }
                    __syncthreads();
                }
                if (out_val) {
#pragma unroll
                    for (uint32_t q = 0; q < PF; ++q) {
                        const uint32_t i = q * SCATTER_THREADS + threadIdx.x;
                        if (i < total) s_pos[s_goff[pf_pk[q] >> 11] + (pf_pk[q] & 2047u)] = __float_as_uint(pf_val[q]);
                    }
                    __syncthreads();
                    for (uint32_t i = threadIdx.x; i < total; i += SCATTER_THREADS) {
                        const uint32_t pos = s_list[i];
                        if (pos < cap) out_val[pos] = __uint_as_float(s_pos[i]);
                    }
                }
            }
            // (c) copy rows (row_dim > 1)
            if (!ELEM && out_val) {
                __syncthreads();
                if ((D & 3u) == 0 && D >= 256) {
                    // one wave copies two rows at a time, 8 x 16-byte loads in flight per lane
                    const uint32_t V = D >> 2, lane = lane_id(), nw = blockDim.x >> 6, wv = threadIdx.x >> 6;
                    for (uint32_t i0 = wv * 2; i0 < total; i0 += nw * 2) {
                        const u32x4 *src[2];
                        u32x4 *dst[2];
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            const uint32_t i = i0 + q;
                            const uint32_t pos = i < total ? s_pos[i] : 0xFFFFFFFFu;
                            src[q] = pos != 0xFFFFFFFFu ? (const u32x4 *)(grad + (uint64_t)s_list[i] * D) : nullptr;
                            dst[q] = pos != 0xFFFFFFFFu ? (u32x4 *)(out_val + (uint64_t)pos * D) : nullptr;
                        }
                        for (uint32_t v = lane; v < V; v += 64 * 4) {
                            u32x4 x[2][4];
#pragma unroll
                            for (int q = 0; q < 2; ++q)
#pragma unroll
                                for (int u = 0; u < 4; ++u)
                                    if (src[q] && v + 64 * u < V) x[q][u] = src[q][v + 64 * u];
#pragma unroll
                            for (int q = 0; q < 2; ++q)
#pragma unroll
                                for (int u = 0; u < 4; ++u)
                                    if (dst[q] && v + 64 * u < V) dst[q][v + 64 * u] = x[q][u];
                        }
                    }
                } else if ((D & 3u) == 0) {
                    const uint32_t V = D >> 2;
                    const uint32_t n_vec = total * V;           // total <= 2048, V < 64
                    const uint32_t vsh = (V & (V - 1)) == 0 ? (uint32_t)__ffs((int)V) - 1 : 0xFFFFFFFFu;   // V = 2^vsh
                    // ZEN_COPY_UNROLL vectors per thread in flight; a power-of-two row needs no division to find its row
                    for (uint32_t f0 = threadIdx.x; f0 < n_vec; f0 += ZEN_COPY_UNROLL * blockDim.x) {
                        u32x4 x[ZEN_COPY_UNROLL];
                        u32x4 *dst[ZEN_COPY_UNROLL];
#pragma unroll
                        for (uint32_t u = 0; u < ZEN_COPY_UNROLL; ++u) {
                            const uint32_t f = f0 + u * blockDim.x;
                            dst[u] = nullptr;
                            if (f < n_vec) {
                                const uint32_t i = vsh != 0xFFFFFFFFu ? f >> vsh : f / V, v = f - i * V;
                                const uint32_t pos = s_pos[i];
                                if (pos != 0xFFFFFFFFu) {
                                    x[u] = ((const u32x4 *)(grad + (uint64_t)s_list[i] * D))[v];
                                    dst[u] = (u32x4 *)(out_val + (uint64_t)pos * D) + v;
                                }
                            }
                        }
#pragma unroll
                        for (uint32_t u = 0; u < ZEN_COPY_UNROLL; ++u)
                            if (dst[u]) *dst[u] = x[u];
                    }
                } else {
                    const uint32_t n_el = total * D;            // total <= 2048, row_dim <= 2^20
                    for (uint32_t f = threadIdx.x; f < n_el; f += blockDim.x) {
                        const uint32_t i = f / D, v = f - i * D;
                        const uint32_t pos = s_pos[i];
                        if (pos != 0xFFFFFFFFu) out_val[(uint64_t)pos * D + v] = grad[(uint64_t)s_list[i] * D + v];
                    }
                }
            }
            __syncthreads();   // s_list / s_pos are rewritten by the next segment
        }

        if (bitmap) {
            __syncthreads();
            // a few threads per partition walk its words (no search for the partition a word belongs to)
            const uint32_t tpp = blockDim.x >= n ? blockDim.x / n : 1u, sub = threadIdx.x % tpp;
            for (uint32_t p = threadIdx.x / tpp; p < n; p += blockDim.x / tpp) {
                const uint32_t b0 = s_b0[p], b1 = s_b1[p];
                if (b1 <= b0) continue;
                const uint32_t lw0 = s_boff[p], last = ((b1 - 1) >> 5) - (b0 >> 5);
                uint32_t *dst = out_bm + bt.word_off[p] + (b0 >> 5);
                for (uint32_t k = sub; k <= last; k += tpp) {
                    const uint32_t v = s_bm[lw0 + k];
                    if (!v) continue;
                    const bool shared = (k == 0 && (b0 & 31u)) || (k == last && (b1 & 31u));
                    if (shared) atomicOr(dst + k, v); else dst[k] = v;
                }
            }
        }
    }
}

// E5 for tiles of at most 64 mask words whose rows are a few 16-byte vectors (4 <= row_dim <= 128, a power of
// two of vectors), index-list output, n_parts <= 64: ONE WAVE per listed tile, no block barrier anywhere.  Lane w
// holds mask word w, lane p the running output position of partition p; the tile's rows are listed in the wave's
// own LDS and ranked 64 at a time with wave ballots.  Tiles here hold a handful of rows each (sparse embedding
// rows): a block per tile spent its time at barriers.  Writes the indices only (same as scatter_kernel<false>
// would); the rows are copied by gather_rows_kernel afterwards.
static constexpr uint32_t WAVE_TILE_MAX_ROWS = 2048;
#ifndef ZEN_WAVE_TILE_DENSE_ROWS
#define ZEN_WAVE_TILE_DENSE_ROWS 64
#endif
static constexpr uint32_t WAVE_TILE_DENSE_ROWS = ZEN_WAVE_TILE_DENSE_ROWS;   // tiles with more rows are handed to the block-per-tile kernel
__global__ void __launch_bounds__(SCATTER_THREADS)
scatter_wave_kernel(Geometry g, EncodedPtrs outs, const uint32_t *mask_base,
                    uint64_t mask_stride_words, const uint32_t *hist_base, uint64_t hist_stride_words,
                    uint32_t *tlist_base, uint64_t tlist_stride)
{
    __shared__ uint32_t s_rows[SCATTER_THREADS / ZEN_WAVE][WAVE_TILE_DENSE_ROWS];   // the tile's rows, ascending (fuller tiles are passed on)
    __shared__ uint32_t s_add[SCATTER_THREADS / ZEN_WAVE][ZEN_WAVE];             // rows of a chunk per partition
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6, n = g.n_parts;
    const uint32_t worker = blockIdx.y;
    uint32_t *__restrict__ out_idx = outs.indices[worker];
    const uint64_t cap = outs.cap_rows[worker];
    uint32_t *tlist = tlist_base + worker * tlist_stride;
    uint32_t *dense = tlist + (g.n_tiles + 1);      // tiles left to the block-per-tile kernel: ids, their number at [n_tiles]
    const uint32_t n_visit = min(tlist[g.n_tiles], g.n_tiles);
    const uint32_t *wmask = mask_base + worker * mask_stride_words;
    const uint32_t *whist = hist_base + worker * hist_stride_words;
    uint32_t *rows = s_rows[wave], *add = s_add[wave];
    add[lane] = 0;
    const uint32_t n_waves = gridDim.x * (SCATTER_THREADS / ZEN_WAVE);
    for (uint32_t k = blockIdx.x * (SCATTER_THREADS / ZEN_WAVE) + wave; k < n_visit; k += n_waves) {
        const uint32_t tile = min(tlist[k], g.n_tiles - 1);
        uint32_t word = lane < g.tile_words ? wmask[(uint64_t)tile * g.tile_words + lane] : 0u;
        uint32_t run = lane < n ? whist[(uint64_t)tile * n + lane] : 0u;   // lane p: next output position of partition p
        const uint32_t c = __popc(word);
        const uint32_t inc = wave_inclusive_scan(c);
        const uint32_t total = __shfl(inc, ZEN_WAVE - 1, ZEN_WAVE);
        if (total > WAVE_TILE_DENSE_ROWS) {          // uniform: a well-filled tile (the head of a skewed table) is a
            if (lane == 0) dense[atomicAdd(&dense[g.n_tiles], 1u)] = tile;   // block's work, not one wave's
            continue;
        }
        const uint32_t row0 = tile * g.tile_rows;
        for (uint32_t j = inc - c; word; ++j) {
            rows[j] = row0 + lane * 32 + (uint32_t)__ffs((int)word) - 1;
            word &= word - 1;
        }
        __builtin_amdgcn_wave_barrier();
        for (uint32_t c0 = 0; c0 < total; c0 += ZEN_WAVE) {     // uniform
            const uint32_t i = c0 + lane;
            const bool valid = i < total;
            const uint32_t row = valid ? rows[i] : 0u;
            const uint32_t p = valid ? owner_of(row, g.seed, n, g.pow2_mask) : 0u;
            const uint64_t peers = wave_peers(valid, p, g.part_bits);
            const uint32_t rank = mbcnt(peers);
            const uint32_t pos = __shfl(run, (int)p, ZEN_WAVE) + rank;
            if (valid && rank == 0) add[p] = (uint32_t)__popcll(peers);
            if (valid && pos < cap && out_idx) out_idx[pos] = row;
            __builtin_amdgcn_wave_barrier();
            run += add[lane];
            add[lane] = 0;
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// E2 on its own: ascending list of non-zero rows from the mask (zen_nonzero).  The scan kernel has
// turned hist into bases, so with n_parts = 1 geometry hist[tile][0] is the tile's output position.
__global__ void __launch_bounds__(SCATTER_THREADS)
nonzero_list_kernel(Geometry g, const uint32_t *gmask_base, const uint32_t *tflag, const uint32_t *tile_base,
                    uint32_t *indices, uint64_t cap_rows)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t tile = blockIdx.x;
    if (g.sparse_mask && !tflag[tile]) return;
    const uint32_t *gmask = gmask_base + (uint64_t)tile * g.tile_words;
    uint32_t run = tile_base[tile];
    const uint64_t row0 = (uint64_t)tile * g.tile_rows;
    for (uint32_t w0 = 0; w0 < g.tile_words; w0 += blockDim.x) {
        const uint32_t wi = w0 + threadIdx.x;
        uint32_t word = wi < g.tile_words ? gmask[wi] : 0u;
        uint32_t total;
        const uint32_t pre = block_exclusive_scan(__popc(word), s_tmp, &total);
        uint64_t k = (uint64_t)run + pre;
        const uint32_t rbase = (uint32_t)(row0 + (uint64_t)wi * 32);
        while (word) {
            const uint32_t b = __ffs(word) - 1;
            word &= word - 1;
            if (k < cap_rows) indices[k] = rbase + b;
            ++k;
        }
        run += total;
    }
}

// Sum of per-tile counts for the non-zero list: one block, hist[tile] (n_parts = 1 view) -> bases.
__global__ void __launch_bounds__(SCAN_THREADS)
tile_scan_kernel(uint32_t *tile_cnt, uint32_t n_tiles, uint32_t *count, uint64_t cap_rows,
                 zen_status_info *status)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t per = (n_tiles + blockDim.x - 1) / blockDim.x;
    const uint32_t t0 = min(threadIdx.x * per, n_tiles), t1 = min(t0 + per, n_tiles);
    uint32_t sum = 0;
    for (uint32_t t = t0; t < t1; ++t) sum += tile_cnt[t];
    uint32_t total;
    uint32_t run = block_exclusive_scan(sum, s_tmp, &total);
    for (uint32_t t = t0; t < t1; ++t) { const uint32_t h = tile_cnt[t]; tile_cnt[t] = run; run += h; }
    if (threadIdx.x == 0) {
        *count = total;
        if ((uint64_t)total > cap_rows) {
            atomicOr(&status->flags, 1u);
            atomicMax((unsigned long long *)&status->needed_rows, (unsigned long long)total);
        }
    }
}

// Per-tile popcount of the mask (n_parts-independent), used by zen_nonzero.
__global__ void __launch_bounds__(256)
tile_popcount_kernel(Geometry g, const uint32_t *gmask_base, const uint32_t *tflag, uint32_t *tile_cnt)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t tile = blockIdx.x;
    const uint32_t *gmask = gmask_base + (uint64_t)tile * g.tile_words;
    uint32_t c = 0;
    if (!g.sparse_mask || tflag[tile])
        for (uint32_t i = threadIdx.x; i < g.tile_words; i += blockDim.x) c += __popc(gmask[i]);
    uint32_t total;
    block_exclusive_scan(c, s_tmp, &total);
    if (threadIdx.x == 0) tile_cnt[tile] = total;
}

__global__ void fill_u32_kernel(uint32_t *p, uint64_t n, uint32_t v)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// The hash bitmaps of all workers of a launch group are assembled with OR: cleared first, in one launch (a fill
// kernel, not a memset node), 16 bytes per store where the pointer allows.
__global__ void __launch_bounds__(256) bitmap_clear_kernel(EncodedPtrs outs, uint64_t n_words)
{
    uint32_t *p = outs.bitmap[blockIdx.y];
    if (!p) return;
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (uint64_t)gridDim.x * blockDim.x;
    if (((uintptr_t)p & 15u) == 0) {
        u32x4 *p4 = (u32x4 *)p;
        for (uint64_t i = tid; i < (n_words >> 2); i += nt) p4[i] = (u32x4){0u, 0u, 0u, 0u};
        for (uint64_t i = (n_words & ~3ull) + tid; i < n_words; i += nt) p[i] = 0u;
    } else {
        for (uint64_t i = tid; i < n_words; i += nt) p[i] = 0u;
    }
}

static hipError_t launch_bitmap_clear(const EncodedPtrs &outs, uint32_t batch, uint64_t n_words, hipStream_t s)
{
    bool any = false;
    for (uint32_t w = 0; w < batch; ++w) any |= outs.bitmap[w] != nullptr;
    if (!any || n_words == 0) return hipSuccess;
    uint64_t blocks = (n_words / 4 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    bitmap_clear_kernel<<<dim3((uint32_t)blocks, batch), 256, 0, s>>>(outs, n_words);
    return hipGetLastError();
}

// Plain streaming copy: the reference kernel against which hardware HBM byte counters are scaled.
__global__ void __launch_bounds__(256) copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, uint64_t n_vec)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += (uint64_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

hipError_t launch_copy(const void *src, void *dst, uint64_t bytes, hipStream_t s)
{
    const uint64_t n_vec = bytes / 16;
    if (n_vec == 0) return hipSuccess;
    copy_kernel<<<16384, 256, 0, s>>>((const u32x4 *)src, (u32x4 *)dst, n_vec);
    return hipGetLastError();
}

__global__ void hash_many_kernel(const uint32_t *idx, uint64_t count, uint32_t seed, uint32_t *out)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (uint64_t)gridDim.x * blockDim.x)
        out[i] = murmur3_u32(idx[i], seed);
}

// ----------------------------------------------------------------------------------------------
// launchers
// ----------------------------------------------------------------------------------------------
hipError_t launch_fill_u32(uint32_t *p, uint64_t n, uint32_t v, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + 1023) / 1024;
    fill_u32_kernel<<<(uint32_t)(blocks > 65536 ? 65536 : blocks), 256, 0, s>>>(p, n, v);
    return hipGetLastError();
}

hipError_t launch_hash_many(const uint32_t *idx, uint64_t count, uint32_t seed, uint32_t *out, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    const uint64_t blocks = (count + 255) / 256;
    hash_many_kernel<<<(uint32_t)(blocks > 65536 ? 65536 : blocks), 256, 0, s>>>(idx, count, seed, out);
    return hipGetLastError();
}

hipError_t launch_detect(zen_ctx *ctx, const GradPtrs &grads, uint32_t batch, char *ws,
                         const EncodeLayout &L, bool reset_status, bool want_hist, hipStream_t s,
                         const uint32_t *min_mag, bool seg_flags)
{
    if (min_mag && ctx->geo.mode != MODE_ELEM) return hipErrorInvalidValue;
    const Geometry &g = ctx->geo;
    const size_t lds = (size_t)(g.tile_words + g.n_parts) * 4;
    ProfScope prof(ctx, K_DETECT, s);
    uint32_t *mask = (uint32_t *)(ws + L.mask_off), *hist = want_hist ? (uint32_t *)(ws + L.hist_off) : nullptr;
    zen_status_info *rs = reset_status ? (zen_status_info *)(ws + L.status_off) : nullptr;
    uint32_t *tflag = (uint32_t *)(ws + L.flag_off);
    const dim3 grid(g.n_tiles, batch);
    int path;
    if (g.mode == MODE_ELEM) path = 0;
    else if (g.mode == MODE_SUB) { path = 1; while ((4u << (path - 1)) < g.row_dim) ++path; }
    else path = (g.row_dim & 3u) == 0 ? 7 : 8;
#define ZEN_DETECT_CASE(P)                                                                                 \
    case P:                                                                                                \
        detect_kernel<P><<<grid, DETECT_THREADS, lds, s>>>(g, grads, mask, L.mask_stride / 4, hist,        \
                                                          L.hist_stride / 4, tflag, L.flag_stride / 4, rs, \
                                                          min_mag, seg_flags ? 1u : 0u,                    \
                                                          (want_hist && g.bitmap) ? ctx->d_group_base : nullptr); \
        break;
    switch (path) {
        ZEN_DETECT_CASE(0) ZEN_DETECT_CASE(1) ZEN_DETECT_CASE(2) ZEN_DETECT_CASE(3) ZEN_DETECT_CASE(4)
        ZEN_DETECT_CASE(5) ZEN_DETECT_CASE(6) ZEN_DETECT_CASE(7) ZEN_DETECT_CASE(8)
    }
#undef ZEN_DETECT_CASE
    return hipGetLastError();
}

hipError_t launch_partition_scan(zen_ctx *ctx, const EncodedPtrs &outs, uint32_t batch, char *ws,
                                 const EncodeLayout &L, hipStream_t s)
{
    const Geometry &g = ctx->geo;
    ProfScope prof(ctx, K_PARTITION_SCAN, s);
    if (g.n_tiles >= SLICE_MIN_TILES) {
        // many tiles per worker: slices of tiles over the whole chip, two launches
        const uint32_t n_slices = (g.n_tiles + SLICE_TILES - 1) / SLICE_TILES;
        partition_slice_kernel<0><<<dim3(n_slices, batch), SCAN_THREADS, 0, s>>>(
            g, outs, (uint32_t *)(ws + L.hist_off), L.hist_stride / 4, (const uint32_t *)(ws + L.flag_off), L.flag_stride / 4,
            (uint32_t *)(ws + L.list_off), L.list_stride / 4, (uint32_t *)(ws + L.slice_off), (zen_status_info *)(ws + L.status_off));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        partition_slice_kernel<1><<<dim3(n_slices, batch), SCAN_THREADS, 0, s>>>(
            g, outs, (uint32_t *)(ws + L.hist_off), L.hist_stride / 4, (const uint32_t *)(ws + L.flag_off), L.flag_stride / 4,
            (uint32_t *)(ws + L.list_off), L.list_stride / 4, (uint32_t *)(ws + L.slice_off), (zen_status_info *)(ws + L.status_off));
        return hipGetLastError();
    }
    partition_scan_kernel<<<batch, SCAN_THREADS, 0, s>>>(g, outs, (uint32_t *)(ws + L.hist_off),
                                                         L.hist_stride / 4, (const uint32_t *)(ws + L.flag_off),
                                                         L.flag_stride / 4,
                                                         (uint32_t *)(ws + L.list_off),
                                                         L.list_stride / 4, (zen_status_info *)(ws + L.status_off));
    return hipGetLastError();
}

// Blocks per worker: about 4096 blocks per launch; a block that would get only two or three tiles
// gets one instead (short launches are latency-bound, not block-overhead-bound).
static uint32_t scatter_grid_x(const Geometry &g, uint32_t batch)
{
    uint32_t gx = 4096 / (batch ? batch : 1);
    if (gx < 64) gx = 64;
    if (g.n_tiles <= 3 * gx) gx = g.n_tiles;
    return gx < g.n_tiles ? gx : g.n_tiles;
}

static uint32_t scatter_threads(const Geometry &) { return (uint32_t)SCATTER_THREADS; }

hipError_t launch_scatter(zen_ctx *ctx, const GradPtrs &grads,
                          const EncodedPtrs &outs, uint32_t batch, char *ws, const EncodeLayout &L,
                          hipStream_t s)
{
    const Geometry &g = ctx->geo;
    BitmapTables bt{ctx->d_rank, ctx->d_dom_tile_base, ctx->d_bm_word_off, ctx->d_group_base};
    if (g.bitmap) {
        const hipError_t e = launch_bitmap_clear(outs, batch, ctx->bm_total_words, s);
        if (e != hipSuccess) return e;
    }
    ProfScope prof(ctx, K_SCATTER, s);
    const uint32_t threads = scatter_threads(g);
    size_t words = (3 + threads / 64) * (size_t)g.n_parts + 2 * SEG_ROWS + 32 + g.tile_words +
                   (g.tile_words + GROUP_WORDS - 1) / GROUP_WORDS;
    if (g.bitmap) words += 3 * (size_t)g.n_parts + 1 + g.tile_words + 2 * (size_t)g.n_parts;
    if (words * 4 > 160 * 1024) return hipErrorInvalidValue;
    if (words * 4 > 48 * 1024) {   // beyond the default dynamic LDS limit
        (void)hipFuncSetAttribute((const void *)scatter_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        (void)hipFuncSetAttribute((const void *)scatter_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        (void)hipGetLastError();
    }
    if (g.mode == MODE_SUB && !g.bitmap && g.n_parts <= ZEN_WAVE && g.tile_words <= ZEN_WAVE &&
        g.tile_rows <= WAVE_TILE_MAX_ROWS && g.sparse_mask) {
        // sparse rows of a few vectors: a wave per listed tile
        uint32_t gx = (g.n_tiles + 3) / 4;
        if (gx > 8192) gx = 8192;
        // Both kernels write offsets-ordered indices only; the rows are copied afterwards by one gather over all
        // output positions.  The head tiles of a skewed table hold thousands of rows each: copied by their own
        // block they set the kernel's length, spread over the chip the copy runs at the rate of a plain copy.
        EncodedPtrs outs_idx = outs;
        uint64_t max_cap = 0;
        for (uint32_t w = 0; w < batch; ++w) {
            outs_idx.values[w] = nullptr;
            if (outs.values[w] && outs.cap_rows[w] > max_cap) max_cap = outs.cap_rows[w];
        }
        scatter_wave_kernel<<<dim3(gx, batch), SCATTER_THREADS, 0, s>>>(
            g, outs_idx, (const uint32_t *)(ws + L.mask_off), L.mask_stride / 4,
            (const uint32_t *)(ws + L.hist_off), L.hist_stride / 4, (uint32_t *)(ws + L.list_off),
            L.list_stride / 4);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        // the well-filled tiles it listed: a block each
        scatter_kernel<false><<<dim3(scatter_grid_x(g, batch), batch), threads, words * 4, s>>>(
            g, grads, outs_idx, (const uint32_t *)(ws + L.mask_off), L.mask_stride / 4,
            (const uint32_t *)(ws + L.hist_off), L.hist_stride / 4,
            (const uint32_t *)(ws + L.list_off) + (g.n_tiles + 1), L.list_stride / 4, bt);
        e = hipGetLastError();
        if (e != hipSuccess || max_cap == 0) return e;
        return launch_gather_rows(ctx, grads, outs, batch, max_cap, s);
    }
    if (g.row_dim == 1)
        scatter_kernel<true><<<dim3(scatter_grid_x(g, batch), batch), threads, words * 4, s>>>(
            g, grads, outs, (const uint32_t *)(ws + L.mask_off), L.mask_stride / 4,
            (const uint32_t *)(ws + L.hist_off), L.hist_stride / 4, (const uint32_t *)(ws + L.list_off),
            L.list_stride / 4, bt);
    else
        scatter_kernel<false><<<dim3(scatter_grid_x(g, batch), batch), threads, words * 4, s>>>(
            g, grads, outs, (const uint32_t *)(ws + L.mask_off), L.mask_stride / 4,
            (const uint32_t *)(ws + L.hist_off), L.hist_stride / 4, (const uint32_t *)(ws + L.list_off),
            L.list_stride / 4, bt);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// Few non-zero rows (output capacity <= ESMALL_MAX_ROWS and a mask one block can walk): the whole
// E2-E5 of a worker runs in ONE block -- compact the mask to an ascending row list in LDS, histogram
// the owners, scan, rank stably, write offsets and indices -- and the rows are then copied by a
// separate launch with one wave per output row, so that a run of dense tiles cannot become one
// block's long pole.  Results are identical to the tiled path.
// ----------------------------------------------------------------------------------------------
static constexpr int ESMALL_THREADS = 1024;
static constexpr uint32_t ESMALL_MAX_ROWS = 16384;
static constexpr uint32_t ESMALL_MAX_WORDS = 16384;   // mask words (x32 rows) one block walks in <= 16 rounds

__global__ void __launch_bounds__(ESMALL_THREADS)
encode_small_kernel(Geometry g, GradPtrs grads, EncodedPtrs outs, const uint32_t *mask_base,
                    uint64_t mask_stride_words, const uint32_t *tflag_base, uint64_t tflag_stride,
                    uint32_t list_cap, BitmapTables bt, zen_status_info *status)
{
    extern __shared__ uint32_t smem[];
    const uint32_t n = g.n_parts, n_waves = blockDim.x >> 6;
    uint32_t *s_hist = smem;                     // [n]
    uint32_t *s_run = s_hist + n;                // [n]
    uint32_t *s_cnt = s_run + n;                 // [n_waves][n]
    uint32_t *s_list = s_cnt + n_waves * n;      // [list_cap]
    uint32_t *s_tmp = s_list + list_cap;         // [32]
    const uint32_t worker = blockIdx.x;
    const uint32_t *gmask = mask_base + worker * mask_stride_words;
    const uint32_t *tflag = tflag_base + worker * tflag_stride;   // mask words of empty tiles are undefined
    const uint32_t n_words = g.n_tiles * g.tile_words;
    const float *__restrict__ grad = grads.p[worker];
    uint32_t *__restrict__ out_idx = outs.indices[worker];
    float *__restrict__ out_val = outs.values[worker];
    uint32_t *__restrict__ out_bm = g.bitmap ? outs.bitmap[worker] : nullptr;
    const uint64_t cap = outs.cap_rows[worker];

    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) s_hist[i] = 0;
    for (uint32_t i = threadIdx.x; i < n_waves * n; i += blockDim.x) s_cnt[i] = 0;
    __syncthreads();
    // E2 + E3: ascending row list and owner histogram
    uint32_t total = 0;
    for (uint32_t w0 = 0; w0 < n_words; w0 += blockDim.x) {
        const uint32_t wi = w0 + threadIdx.x;
        uint32_t word = (wi < n_words && (!g.sparse_mask || tflag[wi / g.tile_words])) ? gmask[wi] : 0u;
        uint32_t chunk_total;
        const uint32_t pre = block_exclusive_scan(__popc(word), s_tmp, &chunk_total);
        uint32_t k = total + pre;
        while (word) {
            const uint32_t b = __ffs(word) - 1;
            word &= word - 1;
            const uint32_t row = wi * 32 + b;
            atomicAdd(&s_hist[owner_of(row, g.seed, n, g.pow2_mask)], 1u);
            if (k < list_cap) s_list[k] = row;
            ++k;
        }
        total += chunk_total;
    }
    __syncthreads();
    // E4: offsets
    uint32_t unused;
    const uint32_t off = block_exclusive_scan(threadIdx.x < n ? s_hist[threadIdx.x] : 0u, s_tmp, &unused);
    if (threadIdx.x < n) {
        s_run[threadIdx.x] = off;
        outs.offsets[worker][threadIdx.x] = off;
    }
    if (threadIdx.x == 0) {
        outs.offsets[worker][n] = total;
        if ((uint64_t)total > cap) {
            atomicOr(&status->flags, 1u);
            atomicMax((unsigned long long *)&status->needed_rows, (unsigned long long)total);
        }
    }
    __syncthreads();
    // E5 (+E7): stable rank inside each partition, indices, element values, bitmap bits.  The list
    // holds every row unless the gradient has more non-zero rows than the list (then the output
    // capacity is exceeded too): in that case the mask is walked again in 64-word segments.
    const bool fits = total <= list_cap;
    const uint32_t n_rounds = fits ? 1u : (n_words + SEG_WORDS - 1) / SEG_WORDS;
    for (uint32_t round = 0; round < n_rounds; ++round) {
        uint32_t listed = total;
        if (!fits) {
            const uint32_t wi = round * SEG_WORDS + threadIdx.x;
            uint32_t word = (threadIdx.x < SEG_WORDS && wi < n_words && (!g.sparse_mask || tflag[wi / g.tile_words])) ? gmask[wi] : 0u;
            const uint32_t pre = block_exclusive_scan(__popc(word), s_tmp, &listed);
            uint32_t k = pre;
            while (word) {
                const uint32_t b = __ffs(word) - 1;
                word &= word - 1;
                s_list[k++] = wi * 32 + b;      // list_cap >= SEG_ROWS
            }
            __syncthreads();
        }
        for (uint32_t c = 0; c < listed; c += blockDim.x) {
            const uint32_t i = c + threadIdx.x;
            const bool valid = i < listed;
            const uint32_t row = valid ? s_list[i] : 0u;
            const uint32_t p = valid ? owner_of(row, g.seed, n, g.pow2_mask) : 0u;
            const uint32_t pos = block_stable_rank(valid, p, g.part_bits, n, s_run, s_cnt);
            if (valid) {
                if (pos < cap) {
                    out_idx[pos] = row;
                    if (g.row_dim == 1 && out_val) out_val[pos] = grad[row];
                }
                if (out_bm) {
                    const uint32_t bit = bt.rank[row];
                    atomicOr(out_bm + bt.word_off[p] + (bit >> 5), 1u << (bit & 31));
                }
            }
        }
        __syncthreads();   // the list is rewritten by the next round
    }
}

// E6 on its own: values[pos] = grad[indices[pos]] for pos < min(nnz, capacity); one wave per row
// (wide rows) or one thread per 16 bytes / per element (narrow rows).
__global__ void __launch_bounds__(256)
gather_rows_kernel(Geometry g, GradPtrs grads, EncodedPtrs outs)
{
    const uint32_t worker = blockIdx.y, D = g.row_dim;
    const float *__restrict__ grad = grads.p[worker];
    const uint32_t *__restrict__ idx = outs.indices[worker];
    float *__restrict__ out_val = outs.values[worker];
    if (!out_val || !idx) return;
    const uint32_t nnz = outs.offsets[worker][g.n_parts];
    const uint32_t rows = (uint64_t)nnz < outs.cap_rows[worker] ? nnz : (uint32_t)outs.cap_rows[worker];
    if ((D & 3u) == 0 && D >= 256) {
        const uint32_t V = D >> 2, lane = lane_id(), nw = blockDim.x >> 6;
        for (uint32_t pos = blockIdx.x * nw + (threadIdx.x >> 6); pos < rows; pos += gridDim.x * nw) {
            const u32x4 *src = (const u32x4 *)(grad + (uint64_t)idx[pos] * D);
            u32x4 *dst = (u32x4 *)(out_val + (uint64_t)pos * D);
            for (uint32_t v = lane; v < V; v += 64 * 4) {
                u32x4 x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (v + 64 * u < V) x[u] = src[v + 64 * u];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (v + 64 * u < V) dst[v + 64 * u] = x[u];
            }
        }
    } else if ((D & 3u) == 0) {
        // four vectors per thread in flight (a vector is a chain of two accesses: the row id, then the row)
        const uint32_t V = D >> 2;
        const uint64_t n_vec = (uint64_t)rows * V;
        const uint32_t vsh = (V & (V - 1)) == 0 ? (uint32_t)__ffs((int)V) - 1 : 0xFFFFFFFFu;   // V = 2^vsh
        for (uint64_t f0 = (uint64_t)blockIdx.x * (4 * blockDim.x) + threadIdx.x; f0 < n_vec;
             f0 += (uint64_t)gridDim.x * (4 * blockDim.x)) {
            uint32_t pos[4], v[4], row[4];
            u32x4 x[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint64_t f = f0 + (uint64_t)u * blockDim.x;
                pos[u] = 0xFFFFFFFFu;
                if (f < n_vec) {
                    pos[u] = vsh != 0xFFFFFFFFu ? (uint32_t)(f >> vsh) : (uint32_t)(f / V);
                    v[u] = (uint32_t)(f - (uint64_t)pos[u] * V);
                    row[u] = idx[pos[u]];
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u)
                if (pos[u] != 0xFFFFFFFFu) x[u] = ((const u32x4 *)(grad + (uint64_t)row[u] * D))[v[u]];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u)
                if (pos[u] != 0xFFFFFFFFu) ((u32x4 *)(out_val + (uint64_t)pos[u] * D))[v[u]] = x[u];
        }
    } else {
        const uint64_t n_el = (uint64_t)rows * D;
        for (uint64_t f = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; f < n_el;
             f += (uint64_t)gridDim.x * blockDim.x) {
            const uint32_t pos = (uint32_t)(f / D), v = (uint32_t)(f - (uint64_t)pos * D);
            out_val[(uint64_t)pos * D + v] = grad[(uint64_t)idx[pos] * D + v];
        }
    }
}

bool encode_small_applies(const zen_ctx *ctx, const EncodedPtrs &outs, uint32_t batch)
{
    const Geometry &g = ctx->geo;
    if (!ctx->small_encode || (uint64_t)g.n_tiles * g.tile_words > ESMALL_MAX_WORDS) return false;
    for (uint32_t w = 0; w < batch; ++w)
        if (!outs.indices[w] || outs.cap_rows[w] > ESMALL_MAX_ROWS) return false;
    return true;
}

hipError_t launch_encode_small(zen_ctx *ctx, const GradPtrs &grads, const EncodedPtrs &outs, uint32_t batch,
                               char *ws, const EncodeLayout &L, hipStream_t s)
{
    const Geometry &g = ctx->geo;
    BitmapTables bt{ctx->d_rank, ctx->d_dom_tile_base, ctx->d_bm_word_off, ctx->d_group_base};
    uint64_t max_cap = 1;
    for (uint32_t w = 0; w < batch; ++w)
        if (outs.cap_rows[w] > max_cap) max_cap = outs.cap_rows[w];
    if (g.bitmap) {
        const hipError_t e = launch_bitmap_clear(outs, batch, ctx->bm_total_words, s);
        if (e != hipSuccess) return e;
    }
    uint32_t list_cap = SEG_ROWS;
    while (list_cap < max_cap) list_cap <<= 1;
    const size_t lds = ((size_t)(2 + ESMALL_THREADS / 64) * g.n_parts + list_cap + 32) * 4;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void *)encode_small_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)(((size_t)18 * ZEN_MAX_PARTS + ESMALL_MAX_ROWS + 32) * 4));
        (void)hipGetLastError();
        attr_set = true;
    }
    {
        ProfScope prof(ctx, K_ENCODE_SMALL, s);
        encode_small_kernel<<<batch, ESMALL_THREADS, lds, s>>>(g, grads, outs, (const uint32_t *)(ws + L.mask_off),
                                                              L.mask_stride / 4, (const uint32_t *)(ws + L.flag_off),
                                                              L.flag_stride / 4, list_cap, bt,
                                                              (zen_status_info *)(ws + L.status_off));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (g.row_dim > 1) {
        uint64_t gx;
        if ((g.row_dim & 3u) == 0 && g.row_dim >= 256) gx = (max_cap + 3) / 4;
        else gx = (max_cap * g.row_dim / 4 + 255) / 256;
        if (gx < 1) gx = 1;
        if (gx > 8192) gx = 8192;
        ProfScope prof(ctx, K_GATHER_ROWS, s);
        gather_rows_kernel<<<dim3((uint32_t)gx, batch), 256, 0, s>>>(g, grads, outs);
        return hipGetLastError();
    }
    return hipSuccess;
}

// values[pos] = grad[indices[pos]] for the first min(offsets[n_parts], capacity) rows of every worker.
hipError_t launch_gather_rows(zen_ctx *ctx, const GradPtrs &grads, const EncodedPtrs &outs, uint32_t batch,
                              uint64_t max_cap, hipStream_t s)
{
    const Geometry &g = ctx->geo;
    uint64_t gx;
    if ((g.row_dim & 3u) == 0 && g.row_dim >= 256) gx = (max_cap + 3) / 4;
    else if ((g.row_dim & 3u) == 0) gx = (max_cap * (g.row_dim / 4) + 1023) / 1024;   // four vectors per thread
    else gx = (max_cap * g.row_dim / 4 + 255) / 256;
    if (gx < 1) gx = 1;
    if (gx > 8192) gx = 8192;
    ProfScope prof(ctx, K_GATHER_ROWS, s);
    gather_rows_kernel<<<dim3((uint32_t)gx, batch), 256, 0, s>>>(g, grads, outs);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------------------------
// Hash-domain tables of a BITMAP context ("computed and sorted offline", section "Hash Bitmap"):
// the domains are the partition of ALL rows by h0, i.e. the encode pipeline run on an all-ones mask.
// ----------------------------------------------------------------------------------------------
__global__ void ones_mask_kernel(uint32_t *mask, uint64_t n_words, uint64_t n_rows)
{
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words;
         i += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t r0 = i * 32;
        uint32_t w = 0;
        if (r0 + 32 <= n_rows) w = 0xFFFFFFFFu;
        else if (r0 < n_rows) w = (1u << (uint32_t)(n_rows - r0)) - 1u;
        mask[i] = w;
    }
}

__global__ void __launch_bounds__(DETECT_THREADS)
hist_from_mask_kernel(Geometry g, const uint32_t *mask, uint32_t *hist, uint32_t *tflag)
{
    extern __shared__ uint32_t smem[];
    uint32_t *s_hist = smem;
    const uint32_t tile = blockIdx.x;
    const uint64_t row0 = (uint64_t)tile * g.tile_rows;
    for (uint32_t i = threadIdx.x; i < g.n_parts; i += blockDim.x) s_hist[i] = 0;
    __syncthreads();
    const uint32_t *m = mask + (uint64_t)tile * g.tile_words;
    for (uint32_t r = threadIdx.x; r < g.tile_rows; r += blockDim.x)
        if ((m[r >> 5] >> (r & 31)) & 1u)
            atomicAdd(&s_hist[owner_of((uint32_t)(row0 + r), g.seed, g.n_parts, g.pow2_mask)], 1u);
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < g.n_parts; i += blockDim.x) hist[(uint64_t)tile * g.n_parts + i] = s_hist[i];
    if (threadIdx.x == 0) tflag[tile] = 0xFFFFFFFFu;   // every tile of the all-rows mask holds rows, in every segment
}

// rank[domain[pos]] = pos - dom_offsets[owner]
__global__ void domain_rank_kernel(Geometry g, const uint32_t *domain, const uint32_t *dom_offsets, uint32_t *rank)
{
    for (uint64_t pos = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; pos < g.n_rows;
         pos += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t idx = domain[pos];
        const uint32_t p = owner_of(idx, g.seed, g.n_parts, g.pow2_mask);
        rank[idx] = (uint32_t)pos - dom_offsets[p];
    }
}

// tile_base[t][p]: output position -> position inside the domain; row n_tiles = domain sizes
__global__ void tile_base_fix_kernel(Geometry g, uint32_t *tile_base, const uint32_t *dom_offsets)
{
    const uint64_t total = ((uint64_t)g.n_tiles + 1) * g.n_parts;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t p = (uint32_t)(i % g.n_parts);
        const uint64_t t = i / g.n_parts;
        if (t == g.n_tiles) tile_base[i] = dom_offsets[p + 1] - dom_offsets[p];
        else tile_base[i] -= dom_offsets[p];
    }
}

hipError_t build_domain_tables(zen_ctx *ctx, uint32_t *tmp_mask, zen_status_info *tmp_status, hipStream_t s)
{
    Geometry g = ctx->geo;
    g.row_dim = 1;      // indices only: the scatter copies no values
    g.bitmap = 0;
    const uint64_t n_words = (uint64_t)g.n_tiles * g.tile_words;
    ones_mask_kernel<<<(uint32_t)((n_words + 255) / 256 > 65535 ? 65535 : (n_words + 255) / 256), 256, 0, s>>>(
        tmp_mask, n_words, g.n_rows);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    uint32_t *tflag = tmp_mask + n_words;   // the caller allocates n_tiles flag words behind the mask
    hist_from_mask_kernel<<<g.n_tiles, DETECT_THREADS, g.n_parts * 4, s>>>(g, tmp_mask, ctx->d_dom_tile_base, tflag);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    EncodedPtrs outs;
    memset(&outs, 0, sizeof(outs));
    outs.offsets[0] = ctx->d_dom_offsets;
    outs.indices[0] = ctx->d_domain;
    outs.cap_rows[0] = g.n_rows;
    uint32_t *tlist = tflag + g.n_tiles;    // ... and 2 * (n_tiles + 1) list words (ids, count, flag words) behind the flags
    partition_scan_kernel<<<1, SCAN_THREADS, 0, s>>>(g, outs, ctx->d_dom_tile_base, 0, tflag, 0, tlist, 0, tmp_status);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    GradPtrs grads;
    memset(&grads, 0, sizeof(grads));
    BitmapTables bt{nullptr, nullptr, nullptr, nullptr};
    const size_t words = 7 * (size_t)g.n_parts + 2 * SEG_ROWS + 32 + g.tile_words + (g.tile_words + GROUP_WORDS - 1) / GROUP_WORDS;
    if (words * 4 > 160 * 1024) return hipErrorInvalidValue;
    if (words * 4 > 48 * 1024) {
        (void)hipFuncSetAttribute((const void *)scatter_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        (void)hipGetLastError();
    }
    scatter_kernel<true><<<dim3(scatter_grid_x(g, 1), 1), SCATTER_THREADS, words * 4, s>>>(
        g, grads, outs, tmp_mask, 0, ctx->d_dom_tile_base, 0, tlist, 0, bt);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    domain_rank_kernel<<<4096, 256, 0, s>>>(g, ctx->d_domain, ctx->d_dom_offsets, ctx->d_rank);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tile_base_fix_kernel<<<1024, 256, 0, s>>>(g, ctx->d_dom_tile_base, ctx->d_dom_offsets);
    return hipGetLastError();
}

hipError_t launch_nonzero_list(zen_ctx *ctx, uint32_t *indices, uint64_t cap_rows, uint32_t *count,
                               char *ws, const EncodeLayout &L, hipStream_t s)
{
    const Geometry &g = ctx->geo;
    ProfScope prof(ctx, K_NONZERO_LIST, s);
    uint32_t *mask = (uint32_t *)(ws + L.mask_off);
    uint32_t *tile_cnt = (uint32_t *)(ws + L.hist_off);   // reused: n_tiles words fit (n_parts >= 1)
    const uint32_t *tflag = (const uint32_t *)(ws + L.flag_off);
    tile_popcount_kernel<<<g.n_tiles, 256, 0, s>>>(g, mask, tflag, tile_cnt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    tile_scan_kernel<<<1, SCAN_THREADS, 0, s>>>(tile_cnt, g.n_tiles, count, cap_rows,
                                                (zen_status_info *)(ws + L.status_off));
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    nonzero_list_kernel<<<g.n_tiles, SCATTER_THREADS, 0, s>>>(g, mask, tflag, tile_cnt, indices, cap_rows);
    return hipGetLastError();
}

} // namespace zen
