// Counts behind the paper's sparsity metrics (section "Characteristics of Sparse Tensors"): per-worker
// non-zero rows, sizes of the running unions (densification), pairwise intersections (overlap ratio)
// and non-zero rows per even consecutive partition (skewness).  Everything is a popcount over the
// 1-bit-per-row masks the dense scan leaves behind, so n workers cost n reads of R/8 bytes after the
// scan.  The two communication-time formulas (Equations 1 and 2) are host arithmetic on the ratios.
#include <math.h>
#include <string.h>
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int ST_THREADS = 256;

struct StatsOut { unsigned long long *nnz, *union_prefix, *overlap, *even_split; };

// One block per tile of the masks; W <= ZEN_MAX_BATCH workers.
__global__ void __launch_bounds__(ST_THREADS)
stats_kernel(Geometry g, uint32_t W, const uint32_t *mask_base, uint64_t mask_stride_words, const uint32_t *tflag_base,
             uint64_t tflag_stride, StatsOut out)
{
    __shared__ uint32_t s_ov[ZEN_MAX_BATCH * ZEN_MAX_BATCH];
    __shared__ uint32_t s_nnz[ZEN_MAX_BATCH], s_uni[ZEN_MAX_BATCH], s_flag[ZEN_MAX_BATCH];
    const uint32_t tile = blockIdx.x, lane = lane_id();
    for (uint32_t i = threadIdx.x; i < W * ZEN_MAX_BATCH; i += ST_THREADS) s_ov[i] = 0;
    if (threadIdx.x < ZEN_MAX_BATCH) {
        s_nnz[threadIdx.x] = 0;
        s_uni[threadIdx.x] = 0;
        // the tile's flag word: bit s says that the s-th stretch of 32 mask words was written (all ones where the
        // scan keeps no flags; mask words of an empty tile, or of an empty stretch, were never written)
        s_flag[threadIdx.x] = threadIdx.x >= W ? 0u : !g.sparse_mask ? 0xFFFFFFFFu : tflag_base[threadIdx.x * tflag_stride + tile];
    }
    __syncthreads();
    const uint64_t row0 = (uint64_t)tile * g.tile_rows;
    const uint64_t part_rows = (g.n_rows + g.n_parts - 1) / g.n_parts;   // even consecutive partitions
    for (uint32_t w0 = 0; w0 < g.tile_words; w0 += ST_THREADS) {          // uniform trip count
        const uint32_t wi = w0 + threadIdx.x;
        uint32_t m[ZEN_MAX_BATCH];
#pragma unroll
        for (uint32_t w = 0; w < ZEN_MAX_BATCH; ++w) {
            m[w] = 0;
            if (w < W && wi < g.tile_words && ((s_flag[w] >> ((wi >> 5) & 31u)) & 1u))
                m[w] = mask_base[w * mask_stride_words + (uint64_t)tile * g.tile_words + wi];
        }
        // the word's rows and the even partition(s) they fall into
        const uint64_t r0 = row0 + (uint64_t)wi * 32;
        const uint32_t i0 = (uint32_t)(r0 / part_rows), i1 = (uint32_t)((r0 + 31) / part_rows);
        const uint32_t i0_first = __shfl(i0, 0, ZEN_WAVE), i1_last = __shfl(i1, ZEN_WAVE - 1, ZEN_WAVE);
        const bool one_part = i0_first == i1_last;   // the whole wave's 2,048 rows lie in one partition
        uint32_t acc = 0;
#pragma unroll
        for (uint32_t w = 0; w < ZEN_MAX_BATCH; ++w) {   // m[] stays in registers: every index is static
            const uint32_t c = __popc(m[w]);
            acc |= m[w];
            const uint32_t cu = __popc(acc);
            if (w < W && ballot(cu != 0) != 0) {          // uniform
                const uint32_t su = wave_sum(cu);
                if (lane == 0) atomicAdd(&s_uni[w], su);
            }
            if (w < W && ballot(c != 0) != 0) {           // uniform
                const uint32_t sc = wave_sum(c);
                if (lane == 0) atomicAdd(&s_nnz[w], sc);
                if (one_part) {
                    if (lane == 0) atomicAdd(&out.even_split[(uint64_t)w * g.n_parts + i0_first], (unsigned long long)sc);
                } else if (c) {
                    if (i0 == i1) {
                        atomicAdd(&out.even_split[(uint64_t)w * g.n_parts + i0], (unsigned long long)c);
                    } else {   // the word straddles one partition boundary, or several when partitions have fewer than 32 rows
                        for (uint32_t i = i0; i <= i1 && i < g.n_parts; ++i) {
                            const uint64_t lo = (uint64_t)i * part_rows, hi = lo + part_rows;   // partition i = rows [lo, hi)
                            const uint32_t b0 = lo > r0 ? (uint32_t)(lo - r0) : 0u;            // its bits of the word: [b0, b1)
                            const uint32_t b1 = hi < r0 + 32 ? (uint32_t)(hi - r0) : 32u;
                            const uint32_t below_b1 = b1 >= 32u ? 0xFFFFFFFFu : (1u << b1) - 1u;
                            const uint32_t ci = __popc(m[w] & below_b1 & ~((1u << b0) - 1u));
                            if (ci) atomicAdd(&out.even_split[(uint64_t)w * g.n_parts + i], (unsigned long long)ci);
                        }
                    }
                }
            }
        }
        // pairwise intersections; pairs with an all-zero word on either side are skipped wave-wide
#pragma unroll
        for (uint32_t a = 0; a + 1 < ZEN_MAX_BATCH; ++a) {
            if (a + 1 >= W || ballot(m[a] != 0) == 0) continue;   // uniform
#pragma unroll
            for (uint32_t b = a + 1; b < ZEN_MAX_BATCH; ++b) {
                const uint32_t c = __popc(m[a] & m[b]);
                if (b < W && ballot(c != 0) != 0) {
                    const uint32_t sc = wave_sum(c);
                    if (lane == 0) atomicAdd(&s_ov[a * ZEN_MAX_BATCH + b], sc);
                }
            }
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < W * ZEN_MAX_BATCH; i += ST_THREADS) {
        const uint32_t a = i / ZEN_MAX_BATCH, b = i % ZEN_MAX_BATCH;
        if (b < W && s_ov[i]) {
            atomicAdd(&out.overlap[(uint64_t)a * W + b], (unsigned long long)s_ov[i]);
            atomicAdd(&out.overlap[(uint64_t)b * W + a], (unsigned long long)s_ov[i]);
        }
    }
    if (threadIdx.x < W) {
        if (s_nnz[threadIdx.x]) {
            atomicAdd(&out.nnz[threadIdx.x], (unsigned long long)s_nnz[threadIdx.x]);
            atomicAdd(&out.overlap[(uint64_t)threadIdx.x * W + threadIdx.x], (unsigned long long)s_nnz[threadIdx.x]);
        }
        if (s_uni[threadIdx.x]) atomicAdd(&out.union_prefix[threadIdx.x], (unsigned long long)s_uni[threadIdx.x]);
    }
}

__global__ void stats_zero_kernel(StatsOut out, uint32_t W, uint32_t n_parts)
{
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = tid; i < W; i += nt) { out.nnz[i] = 0; out.union_prefix[i] = 0; }
    for (uint64_t i = tid; i < (uint64_t)W * W; i += nt) out.overlap[i] = 0;
    for (uint64_t i = tid; i < (uint64_t)W * n_parts; i += nt) out.even_split[i] = 0;
}

} // namespace zen

using namespace zen;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return ZEN_ERR_DEVICE;    \
    } while (0)

extern "C" {

zen_status zen_sparsity_count(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                              const zen_sparsity_counts *host_out, void *workspace, uint64_t workspace_bytes,
                              void *hip_stream)
{
    if (!ctx || !host_grads || !host_out || !workspace || n_workers == 0 || n_workers > ZEN_MAX_BATCH)
        return ZEN_ERR_INVALID;
    if (!host_out->nnz || !host_out->union_prefix || !host_out->overlap || !host_out->even_split) return ZEN_ERR_INVALID;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)host_out->nnz & 7u) || ((uintptr_t)host_out->union_prefix & 7u) ||
        ((uintptr_t)host_out->overlap & 7u) || ((uintptr_t)host_out->even_split & 7u))
        return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    const EncodeLayout L = encode_layout(g, n_workers);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    GradPtrs grads;
    memset(&grads, 0, sizeof(grads));
    for (uint32_t w = 0; w < n_workers; ++w) {
        if (!host_grads[w] || ((uintptr_t)host_grads[w] & 15u)) return ZEN_ERR_INVALID;
        grads.p[w] = host_grads[w];
    }
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    StatsOut out{(unsigned long long *)host_out->nnz, (unsigned long long *)host_out->union_prefix,
                 (unsigned long long *)host_out->overlap, (unsigned long long *)host_out->even_split};
    HIP_TRY(launch_detect(ctx, grads, n_workers, ws, L, true, false, s, nullptr, true));   // masks by stretch: fewer words written
    stats_zero_kernel<<<64, 256, 0, s>>>(out, n_workers, g.n_parts);
    HIP_TRY(hipGetLastError());
    {
        ProfScope prof(ctx, K_STATS, s);
        stats_kernel<<<g.n_tiles, ST_THREADS, 0, s>>>(g, n_workers, (const uint32_t *)(ws + L.mask_off), L.mask_stride / 4,
                                                     (const uint32_t *)(ws + L.flag_off), L.flag_stride / 4, out);
        HIP_TRY(hipGetLastError());
    }
    return ZEN_OK;
}

zen_status zen_scheme_times(uint32_t n, const double *host_gamma_pow2, double d_G, double M, double b,
                            double *host_t_bp, double *host_t_sm)
{
    if (n < 2 || (n & (n - 1)) || !host_gamma_pow2 || !host_t_bp || !host_t_sm || !(b > 0.0)) return ZEN_ERR_INVALID;
    uint32_t stages = 0;
    while ((1u << stages) < n) ++stages;
    double sum = 0.0;
    for (uint32_t i = 0; i < stages; ++i) sum += host_gamma_pow2[i];             // gamma^(2^(i-1)), i = 1..log2 n
    *host_t_sm = sum * 2.0 * M * d_G / b;                                        // Equation (2)
    *host_t_bp = (double)(n - 1) / (double)n * (host_gamma_pow2[stages] + 1.0) * 2.0 * M * d_G / b;   // Equation (1)
    return ZEN_OK;
}

} // extern "C"
