// Algorithm 1 ("Hierarchical Hashing Algorithm") as the paper runs it: a hash memory of n partitions,
// each with r1 cells of parallel memory and r2 cells of serial memory.  An index goes to partition
// h0(idx); up to k second-level hash functions try to claim a free cell of the parallel memory;
// after k occupied cells the index is appended to the serial memory with an atomic counter; the
// partitions are then extracted with a stream compaction ("nonzero") and the values gathered.
//
// What differs from the listing, and why: a cell is claimed with ONE compare-and-swap (empty ->
// idx) instead of test, plain store and read-back (Technique #4).  The read-back exists because the
// listing's test and store are two steps; a compare-and-swap is the same decision in one step, it
// cannot lose an index, and on this GPU it costs the same memory transaction.  Empty cells hold
// 0xFFFFFFFF (row ids start at 0 here).  The extraction order inside a partition is the memory order,
// which depends on which thread won a contested cell: the SET of indices per partition is fixed.
#include <string.h>
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int HM_THREADS = 256;
static constexpr uint32_t HM_CHUNK = 1024;   // cells per extraction block

struct HashParams {
    uint32_t k, seed2;
    uint32_t r1, r2, cells;   // per partition
};   // device-side copy of zen_hash_params

__global__ void __launch_bounds__(HM_THREADS)
hm_clear_kernel(uint32_t *x, uint64_t n_cells, uint32_t *counters, uint32_t n_parts, uint32_t r1)
{
    const uint64_t tid = (uint64_t)blockIdx.x * HM_THREADS + threadIdx.x, nt = (uint64_t)gridDim.x * HM_THREADS;
    for (uint64_t i = tid; i < n_cells; i += nt) x[i] = ZEN_EMPTY_KEY;
    for (uint64_t i = tid; i < n_parts; i += nt) counters[i] = r1;   // "atomic counters c <- r1^n"
}

// Blocks walk the tiles of the row mask; every set bit is one idx of I, inserted by its own thread.
// Indices that found all k cells taken are parked in LDS and appended to the serial memory in
// batches: the block counts its parked indices per partition and moves each partition's counter ONCE
// per batch (n counters shared by the whole chip are the algorithm's serial bottleneck; the result
// is the same as one atomicAdd per index, the cells handed out are just consecutive per block).
static constexpr uint32_t HM_PARK = 4096;

__device__ __forceinline__ void hm_flush_parked(const HashParams &hp, uint32_t n_parts, uint32_t *x, uint32_t *counters,
                                                uint32_t *s_idx, uint32_t *s_slot, uint32_t *s_n, uint32_t *s_pc,
                                                uint32_t seed, uint32_t pow2_mask)
{
    __syncthreads();
    const uint32_t parked = min(*s_n, HM_PARK);
    for (uint32_t i = threadIdx.x; i < parked; i += HM_THREADS) {   // rank of each parked index inside its partition
        const uint32_t p = owner_of(s_idx[i], seed, n_parts, pow2_mask);
        s_slot[i] = atomicAdd(&s_pc[p], 1u);
    }
    __syncthreads();
    for (uint32_t p = threadIdx.x; p < n_parts; p += HM_THREADS) {   // one counter update per partition
        const uint32_t c = s_pc[p];
        s_pc[p] = c ? atomicAdd(&counters[p], c) : 0u;
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < parked; i += HM_THREADS) {
        const uint32_t idx = s_idx[i], p = owner_of(idx, seed, n_parts, pow2_mask);
        const uint32_t q = s_pc[p] + s_slot[i];
        if (q < hp.cells) x[(uint64_t)p * hp.cells + q] = idx;
    }
    __syncthreads();
    for (uint32_t p = threadIdx.x; p < n_parts; p += HM_THREADS) s_pc[p] = 0;
    if (threadIdx.x == 0) *s_n = 0;
    __syncthreads();
}

__global__ void __launch_bounds__(HM_THREADS)
hm_insert_kernel(Geometry g, HashParams hp, const uint32_t *mask, const uint32_t *tflag, uint32_t *x,
                 uint32_t *counters)
{
    __shared__ uint32_t s_idx[HM_PARK], s_slot[HM_PARK], s_pc[ZEN_MAX_PARTS], s_n;
    for (uint32_t p = threadIdx.x; p < g.n_parts; p += HM_THREADS) s_pc[p] = 0;
    if (threadIdx.x == 0) s_n = 0;
    __syncthreads();
    uint32_t parked = 0;
    for (uint32_t tile = blockIdx.x; tile < g.n_tiles; tile += gridDim.x) {
        if (g.sparse_mask && !tflag[tile]) continue;   // empty tile: its mask words were never written (uniform)
        const uint32_t *m = mask + (uint64_t)tile * g.tile_words;
        const uint64_t row0 = (uint64_t)tile * g.tile_rows;
        for (uint32_t w0 = 0; w0 < g.tile_words; w0 += HM_THREADS) {
            if (parked > HM_PARK / 2) {   // uniform: `parked` was read between two barriers
                hm_flush_parked(hp, g.n_parts, x, counters, s_idx, s_slot, &s_n, s_pc, g.seed, g.pow2_mask);
                parked = 0;
            }
            const uint32_t wi = w0 + threadIdx.x;
            uint32_t word = wi < g.tile_words ? m[wi] : 0u;
            while (word) {
                const uint32_t b = __ffs(word) - 1;
                word &= word - 1;
                const uint32_t idx = (uint32_t)(row0 + wi * 32 + b);
                const uint32_t p = owner_of(idx, g.seed, g.n_parts, g.pow2_mask);
                uint32_t *xp = x + (uint64_t)p * hp.cells;
                bool placed = false;
                for (uint32_t i = 1; i <= hp.k && !placed; ++i) {
                    const uint32_t q = murmur3_u32(idx, hp.seed2 + i) % hp.r1;
                    placed = atomicCAS(&xp[q], ZEN_EMPTY_KEY, idx) == ZEN_EMPTY_KEY;
                }
                if (!placed) {   // serial memory
                    const uint32_t slot = atomicAdd(&s_n, 1u);
                    if (slot < HM_PARK) {
                        s_idx[slot] = idx;
                    } else {     // no room to park: take a cell right away
                        const uint32_t q = atomicAdd(&counters[p], 1u);
                        if (q < hp.cells) xp[q] = idx;
                    }
                }
            }
            __syncthreads();
            parked = s_n;      // the same value in every thread ...
            __syncthreads();   // ... because nobody parks again before all have read it
        }
    }
    hm_flush_parked(hp, g.n_parts, x, counters, s_idx, s_slot, &s_n, s_pc, g.seed, g.pow2_mask);
}

// cnt[p * chunks + c] = occupied cells of chunk c of partition p (flat order = output order).
__global__ void __launch_bounds__(HM_THREADS)
hm_count_kernel(HashParams hp, const uint32_t *x, uint32_t *cnt, uint32_t chunks)
{
    __shared__ uint32_t s_c;
    const uint32_t c = blockIdx.x, p = blockIdx.y;
    if (threadIdx.x == 0) s_c = 0;
    __syncthreads();
    const uint32_t *xp = x + (uint64_t)p * hp.cells;
    uint32_t mine = 0;
#pragma unroll
    for (uint32_t u = 0; u < HM_CHUNK / HM_THREADS; ++u) {
        const uint32_t q = c * HM_CHUNK + u * HM_THREADS + threadIdx.x;
        if (q < hp.cells && xp[q] != ZEN_EMPTY_KEY) ++mine;
    }
    mine = wave_sum(mine);
    if (lane_id() == 0 && mine) atomicAdd(&s_c, mine);
    __syncthreads();
    if (threadIdx.x == 0) cnt[(uint64_t)p * chunks + c] = s_c;
}

// One block: exclusive scan over the flat (partition, chunk) counts, offsets, flags, serial counts.
__global__ void __launch_bounds__(1024)
hm_scan_kernel(HashParams hp, uint32_t *cnt, uint32_t chunks, uint32_t n_parts, const uint32_t *counters,
               uint32_t *offsets, uint64_t cap_rows, uint32_t *serial_counts, zen_status_info *status)
{
    __shared__ uint32_t s_tmp[32];
    __shared__ uint32_t s_worst;
    if (threadIdx.x == 0) s_worst = 0;
    const uint64_t total_entries = (uint64_t)n_parts * chunks;
    uint32_t run = 0;
    for (uint64_t e0 = 0; e0 < total_entries; e0 += 1024) {
        const uint64_t e = e0 + threadIdx.x;
        const uint32_t v = e < total_entries ? cnt[e] : 0u;
        uint32_t total;
        const uint32_t pre = block_exclusive_scan(v, s_tmp, &total);
        if (e < total_entries) {
            cnt[e] = run + pre;
            if (e % chunks == 0) offsets[e / chunks] = run + pre;
        }
        run += total;
    }
    for (uint32_t p = threadIdx.x; p < n_parts; p += 1024) {
        const uint32_t serial = counters[p] - hp.r1;
        if (serial_counts) serial_counts[p] = serial;
        if (serial > hp.r2) atomicMax(&s_worst, serial);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        offsets[n_parts] = run;
        uint32_t flags = 0;
        uint64_t needed = 0;
        if ((uint64_t)run > cap_rows) { flags |= 1u; needed = run; }
        if (s_worst) { flags |= 2u; needed = s_worst; }   // serial memory too small: indices were dropped
        status->flags = flags;
        status->reserved = 0;
        status->needed_rows = needed;
    }
}

// indices = nonzero(x[p]) in memory order, written at the scanned positions.
__global__ void __launch_bounds__(HM_THREADS)
hm_extract_kernel(HashParams hp, const uint32_t *x, const uint32_t *cnt, uint32_t chunks, uint32_t *out_idx,
                  uint64_t cap_rows)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t c = blockIdx.x, p = blockIdx.y;
    const uint32_t *xp = x + (uint64_t)p * hp.cells;
    const uint32_t base = cnt[(uint64_t)p * chunks + c];
    // thread t owns the 4 consecutive cells 4t .. 4t+3 of the chunk: memory order is kept
    uint32_t v[HM_CHUNK / HM_THREADS], mine = 0;
#pragma unroll
    for (uint32_t u = 0; u < HM_CHUNK / HM_THREADS; ++u) {
        const uint32_t q = c * HM_CHUNK + threadIdx.x * (HM_CHUNK / HM_THREADS) + u;
        v[u] = q < hp.cells ? xp[q] : ZEN_EMPTY_KEY;
        mine += v[u] != ZEN_EMPTY_KEY;
    }
    uint32_t total;
    uint32_t pos = base + block_exclusive_scan(mine, s_tmp, &total);
#pragma unroll
    for (uint32_t u = 0; u < HM_CHUNK / HM_THREADS; ++u)
        if (v[u] != ZEN_EMPTY_KEY) {
            if (pos < cap_rows) out_idx[pos] = v[u];
            ++pos;
        }
}

} // namespace zen

using namespace zen;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return ZEN_ERR_DEVICE;    \
    } while (0)

static bool hash_params_ok(const zen_ctx *ctx, const zen_hash_params *hp)
{
    if (!ctx || !hp || hp->k == 0 || hp->k > 8 || hp->r1 == 0) return false;
    if (hp->r1 + hp->r2 > 0x7FFFFFFFull) return false;
    return (hp->r1 + hp->r2) * (uint64_t)ctx->geo.n_parts <= (1ull << 36);
}

static uint64_t hm_chunks(const zen_hash_params *hp) { return (hp->r1 + hp->r2 + HM_CHUNK - 1) / HM_CHUNK; }

extern "C" {

zen_status zen_hash_memory_bytes(const zen_ctx *ctx, const zen_hash_params *host_params, uint64_t *host_bytes)
{
    if (!hash_params_ok(ctx, host_params) || !host_bytes) return ZEN_ERR_INVALID;
    const uint64_t n = ctx->geo.n_parts;
    *host_bytes = (n * (host_params->r1 + host_params->r2) * 4 + 255) / 256 * 256 + (n * 4 + 255) / 256 * 256;
    return ZEN_OK;
}

zen_status zen_encode_hashed_workspace_bytes(const zen_ctx *ctx, const zen_hash_params *host_params,
                                             uint64_t *host_bytes)
{
    if (!hash_params_ok(ctx, host_params) || !host_bytes) return ZEN_ERR_INVALID;
    const uint64_t entries = hm_chunks(host_params) * ctx->geo.n_parts;
    *host_bytes = encode_layout(ctx->geo, 1).total + (entries * 4 + 255) / 256 * 256;
    return ZEN_OK;
}

zen_status zen_encode_hashed(zen_ctx *ctx, const float *grad, const zen_hash_params *host_params, void *hash_memory,
                             uint64_t hash_memory_bytes, const zen_encoded *host_out, uint32_t *serial_counts,
                             void *workspace, uint64_t workspace_bytes, void *hip_stream)
{
    if (!hash_params_ok(ctx, host_params) || !grad || !hash_memory || !host_out || !workspace) return ZEN_ERR_INVALID;
    if (((uintptr_t)grad & 15u) || ((uintptr_t)workspace & 255u) || ((uintptr_t)hash_memory & 255u)) return ZEN_ERR_INVALID;
    if (!host_out->offsets || !host_out->indices || !host_out->values || ((uintptr_t)host_out->values & 15u) ||
        host_out->cap_rows > 0xFFFFFFFEull)
        return ZEN_ERR_INVALID;
    uint64_t need_mem = 0, need_ws = 0;
    (void)zen_hash_memory_bytes(ctx, host_params, &need_mem);
    (void)zen_encode_hashed_workspace_bytes(ctx, host_params, &need_ws);
    if (hash_memory_bytes < need_mem || workspace_bytes < need_ws) return ZEN_ERR_NOMEM;
    const Geometry &g = ctx->geo;
    hipStream_t s = (hipStream_t)hip_stream;
    const EncodeLayout L = encode_layout(g, 1);
    char *ws = (char *)workspace;
    HashParams hp;
    hp.k = host_params->k;
    hp.seed2 = host_params->level2_seed;
    hp.r1 = (uint32_t)host_params->r1;
    hp.r2 = (uint32_t)host_params->r2;
    hp.cells = hp.r1 + hp.r2;
    const uint64_t n_cells = (uint64_t)g.n_parts * hp.cells;
    uint32_t *x = (uint32_t *)hash_memory;
    uint32_t *counters = (uint32_t *)((char *)hash_memory + (n_cells * 4 + 255) / 256 * 256);
    uint32_t *cnt = (uint32_t *)(ws + L.total);
    const uint32_t chunks = (uint32_t)hm_chunks(host_params);
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);

    GradPtrs grads;
    memset(&grads, 0, sizeof(grads));
    grads.p[0] = grad;
    HIP_TRY(launch_detect(ctx, grads, 1, ws, L, true, false, s));   // the row mask = the index set I
    {
        uint64_t blocks = (n_cells + HM_THREADS * 8 - 1) / (HM_THREADS * 8);
        if (blocks < 1) blocks = 1;
        if (blocks > 65536) blocks = 65536;
        ProfScope prof(ctx, K_HM_CLEAR, s);
        hm_clear_kernel<<<(uint32_t)blocks, HM_THREADS, 0, s>>>(x, n_cells, counters, g.n_parts, hp.r1);
        HIP_TRY(hipGetLastError());
    }
    {
        ProfScope prof(ctx, K_HM_INSERT, s);
        const uint32_t blocks = g.n_tiles < 2048 ? g.n_tiles : 2048;
        hm_insert_kernel<<<blocks, HM_THREADS, 0, s>>>(g, hp, (const uint32_t *)(ws + L.mask_off),
                                                         (const uint32_t *)(ws + L.flag_off), x, counters);
        HIP_TRY(hipGetLastError());
    }
    {
        ProfScope prof(ctx, K_HM_EXTRACT, s);
        hm_count_kernel<<<dim3(chunks, g.n_parts), HM_THREADS, 0, s>>>(hp, x, cnt, chunks);
        HIP_TRY(hipGetLastError());
        hm_scan_kernel<<<1, 1024, 0, s>>>(hp, cnt, chunks, g.n_parts, counters, host_out->offsets, host_out->cap_rows,
                                          serial_counts, status);
        HIP_TRY(hipGetLastError());
        hm_extract_kernel<<<dim3(chunks, g.n_parts), HM_THREADS, 0, s>>>(hp, x, cnt, chunks, host_out->indices,
                                                                        host_out->cap_rows);
        HIP_TRY(hipGetLastError());
    }
    EncodedPtrs outs;
    memset(&outs, 0, sizeof(outs));
    outs.offsets[0] = host_out->offsets;
    outs.indices[0] = host_out->indices;
    outs.values[0] = host_out->values;
    outs.cap_rows[0] = host_out->cap_rows;
    HIP_TRY(launch_gather_rows(ctx, grads, outs, 1, host_out->cap_rows, s));   // values = G[indices]
    return ZEN_OK;
}

} // extern "C"
