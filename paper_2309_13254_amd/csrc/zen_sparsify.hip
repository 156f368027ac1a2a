// Top-k threshold of a gradient sparsifier (the paper puts DGC in front of the synchronization:
// section "Implementation" -- sample, take the sample's top-k threshold, apply it to the tensor) and
// the counts behind the sparse-format size comparison (section "Sparse Formats").
//
// Threshold: the keep-th largest magnitude of the sample g[first], g[first + stride], ... found by a
// radix select on the magnitudes taken as integers (bits & 0x7fffffff orders non-NaN floats like
// |x|): four passes of 8 bits, each a histogram over the sample's elements that still match the
// digits chosen so far, then a one-block pick.  Nothing returns to the host; the threshold stays on
// the device, where the dense scan of zen_encode_batch_sparsified applies it on the fly.
#include <string.h>
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int TK_THREADS = 256;

// state[0] = digits chosen so far (in place), state[1] = mask of the bits they cover,
// state[2..3] = rank still wanted inside the matching elements (u64), state[4] = result
__global__ void topk_init_kernel(uint32_t *state, uint32_t *hist, uint64_t keep)
{
    if (threadIdx.x == 0) {
        state[0] = 0;
        state[1] = 0;
        state[2] = (uint32_t)keep;
        state[3] = (uint32_t)(keep >> 32);
    }
    for (uint32_t i = threadIdx.x; i < 4 * 256 * 2; i += blockDim.x) hist[i] = 0;
}

__global__ void __launch_bounds__(TK_THREADS)
topk_hist_kernel(const float *g, uint64_t first, uint64_t stride, uint64_t m, uint32_t pass, const uint32_t *state,
                 unsigned long long *hist_all)
{
    __shared__ uint32_t s_h[256];
    s_h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t prefix = state[0], pmask = state[1], shift = 24 - 8 * pass;
    const uint32_t *gu = (const uint32_t *)g;
    for (uint64_t t = (uint64_t)blockIdx.x * TK_THREADS + threadIdx.x; t < m; t += (uint64_t)gridDim.x * TK_THREADS) {
        const uint32_t mag = gu[first + t * stride] & 0x7fffffffu;
        if ((mag & pmask) == prefix) atomicAdd(&s_h[(mag >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (s_h[threadIdx.x]) atomicAdd(&hist_all[pass * 256 + threadIdx.x], (unsigned long long)s_h[threadIdx.x]);
}

// One thread walks the 256 bins from the top until the wanted rank falls inside one.
__global__ void topk_pick_kernel(uint32_t pass, uint32_t *state, const unsigned long long *hist_all, uint32_t *threshold)
{
    if (threadIdx.x != 0) return;
    const unsigned long long *h = hist_all + pass * 256;
    unsigned long long want = (unsigned long long)state[2] | ((unsigned long long)state[3] << 32);
    const uint32_t shift = 24 - 8 * pass;
    uint32_t digit = 0;
    for (int d = 255; d >= 0; --d) {
        if (h[d] >= want) { digit = (uint32_t)d; break; }
        want -= h[d];
    }
    state[0] |= digit << shift;
    state[1] |= 255u << shift;
    state[2] = (uint32_t)want;
    state[3] = (uint32_t)(want >> 32);
    if (pass == 3) *threshold = state[0];
}

// counts[0] += non-zero rows, counts[1] += blocks of `block_words` mask words holding a non-zero row.
__global__ void __launch_bounds__(TK_THREADS)
format_count_kernel(Geometry g, const uint32_t *mask, const uint32_t *tflag, uint32_t block_words,
                    unsigned long long *counts)
{
    __shared__ uint32_t s_nnz, s_blk;
    const uint32_t tile = blockIdx.x;
    if (g.sparse_mask && !tflag[tile]) return;   // empty tile: no mask words were written
    if (threadIdx.x == 0) { s_nnz = 0; s_blk = 0; }
    __syncthreads();
    const uint32_t *m = mask + (uint64_t)tile * g.tile_words;
    uint32_t nnz = 0, blk = 0;
    for (uint32_t b0 = threadIdx.x * block_words; b0 < g.tile_words; b0 += TK_THREADS * block_words) {
        uint32_t any = 0;
        for (uint32_t q = 0; q < block_words && b0 + q < g.tile_words; ++q) {
            const uint32_t w = m[b0 + q];
            nnz += __popc(w);
            any |= w;
        }
        blk += any != 0;
    }
    if (nnz) atomicAdd(&s_nnz, nnz);
    if (blk) atomicAdd(&s_blk, blk);
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_nnz) atomicAdd(&counts[0], (unsigned long long)s_nnz);
        if (s_blk) atomicAdd(&counts[1], (unsigned long long)s_blk);
    }
}

__global__ void zero_u64_kernel(unsigned long long *p, uint32_t n)
{
    if (threadIdx.x < n) p[threadIdx.x] = 0;
}

} // namespace zen

using namespace zen;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return ZEN_ERR_DEVICE;    \
    } while (0)

extern "C" {

zen_status zen_topk_workspace_bytes(uint64_t *host_bytes)
{
    if (!host_bytes) return ZEN_ERR_INVALID;
    *host_bytes = 256 + 4 * 256 * 8;
    return ZEN_OK;
}

zen_status zen_topk_threshold(const float *g, uint64_t n, uint64_t first, uint64_t stride, uint64_t keep,
                              uint32_t *threshold, void *workspace, uint64_t workspace_bytes, void *hip_stream)
{
    if (!g || !threshold || !workspace || stride == 0 || first >= n) return ZEN_ERR_INVALID;
    if (((uintptr_t)g & 3u) || ((uintptr_t)workspace & 255u) || ((uintptr_t)threshold & 3u)) return ZEN_ERR_INVALID;
    const uint64_t m = (n - first + stride - 1) / stride;
    if (keep == 0 || keep > m) return ZEN_ERR_INVALID;
    if (workspace_bytes < 256 + 4 * 256 * 8) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    uint32_t *state = (uint32_t *)workspace;
    unsigned long long *hist = (unsigned long long *)((char *)workspace + 256);
    topk_init_kernel<<<1, 256, 0, s>>>(state, (uint32_t *)hist, keep);
    HIP_TRY(hipGetLastError());
    uint64_t blocks = (m + TK_THREADS * 8 - 1) / (TK_THREADS * 8);
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    for (uint32_t pass = 0; pass < 4; ++pass) {
        topk_hist_kernel<<<(uint32_t)blocks, TK_THREADS, 0, s>>>(g, first, stride, m, pass, state, hist);
        HIP_TRY(hipGetLastError());
        topk_pick_kernel<<<1, 64, 0, s>>>(pass, state, hist, threshold);
        HIP_TRY(hipGetLastError());
    }
    return ZEN_OK;
}

zen_status zen_format_count(zen_ctx *ctx, const float *grad, uint32_t block, uint64_t *counts, void *workspace,
                            uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !grad || !counts || !workspace || ((uintptr_t)grad & 15u) || ((uintptr_t)workspace & 255u) ||
        ((uintptr_t)counts & 7u))
        return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    if (block < 32 || (block & 31u) || g.tile_rows % block) return ZEN_ERR_INVALID;   // whole mask words, whole blocks per tile
    const EncodeLayout L = encode_layout(g, 1);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    GradPtrs grads;
    memset(&grads, 0, sizeof(grads));
    grads.p[0] = grad;
    HIP_TRY(launch_detect(ctx, grads, 1, ws, L, true, false, s));
    zero_u64_kernel<<<1, 64, 0, s>>>((unsigned long long *)counts, 2);
    HIP_TRY(hipGetLastError());
    format_count_kernel<<<g.n_tiles, TK_THREADS, 0, s>>>(g, (const uint32_t *)(ws + L.mask_off),
                                                        (const uint32_t *)(ws + L.flag_off), block / 32,
                                                        (unsigned long long *)counts);
    HIP_TRY(hipGetLastError());
    return ZEN_OK;
}

zen_status zen_format_bytes(uint64_t n_elems, uint64_t nnz, uint32_t n_servers, uint64_t nonzero_blocks, uint32_t block,
                            double *host_out)
{
    if (!host_out) return ZEN_ERR_INVALID;
    host_out[0] = 4.0 * (double)n_elems;                                       // dense
    host_out[1] = 8.0 * (double)nnz;                                           // COO
    host_out[2] = 4.0 * (double)nnz + (double)n_servers * (double)n_elems / 8.0;   // a |G|-bit bitmap per server
    host_out[3] = 4.0 * (double)nnz + (double)n_elems / 8.0;                   // hash bitmap: |G| bits in all
    host_out[4] = (double)nonzero_blocks * (4.0 * (double)block + 4.0);        // whole blocks + block ids
    return ZEN_OK;
}

} // extern "C"
