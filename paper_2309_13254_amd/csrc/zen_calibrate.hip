// Read-only streaming kernel of known traffic: what a pure read of HBM reaches on this chip, in the launch
// shapes the dense scan could take.  Not part of the method: it is the yardstick the dense scan is held against
// (same loads, no mask, no histogram, no LDS, no stores) and a second reference for hardware byte counters.
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

// Block b reads the vectors [b * vec_per_block, (b + 1) * vec_per_block) and then strides on by the grid: with one
// block per range that is a tile per block (the dense scan's shape), with fewer blocks a persistent grid.  UNROLL
// 16-byte loads per thread are in flight at a time.  Each lane ORs everything it reads, so that no load can be
// dropped; a wave stores one word only if every lane of it ended at all ones, which data with any bit clear
// throughout never does and other data does at most once per wave.
template <int THREADS, int UNROLL, bool NT>
__global__ void __launch_bounds__(THREADS)
read_kernel(const u32x4 *__restrict__ src, uint64_t n_vec, uint64_t vec_per_block, uint32_t *sink)
{
    uint32_t acc = 0;
    for (uint64_t base = (uint64_t)blockIdx.x * vec_per_block; base < n_vec; base += (uint64_t)gridDim.x * vec_per_block) {
        const uint64_t end = base + vec_per_block < n_vec ? base + vec_per_block : n_vec;
        for (uint64_t i = base + threadIdx.x; i < end; i += (uint64_t)THREADS * UNROLL) {
            u32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint64_t j = i + (uint64_t)u * THREADS;
                v[u] = (u32x4){0u, 0u, 0u, 0u};
                if (j < end) v[u] = NT ? __builtin_nontemporal_load(src + j) : src[j];
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) acc |= v[u].x | v[u].y | v[u].z | v[u].w;
        }
    }
    const uint64_t all_ones = ballot(acc == 0xFFFFFFFFu);
    if (all_ones == ~0ull && lane_id() == 0) sink[blockIdx.x & 63u] = acc;
}

template <int THREADS, int UNROLL>
static hipError_t launch_read_nt(const u32x4 *src, uint64_t n_vec, uint64_t vec_per_block, uint32_t grid, bool nt,
                                 uint32_t *sink, hipStream_t s)
{
    if (nt) read_kernel<THREADS, UNROLL, true><<<grid, THREADS, 0, s>>>(src, n_vec, vec_per_block, sink);
    else read_kernel<THREADS, UNROLL, false><<<grid, THREADS, 0, s>>>(src, n_vec, vec_per_block, sink);
    return hipGetLastError();
}

template <int THREADS>
static hipError_t launch_read_unroll(const u32x4 *src, uint64_t n_vec, uint64_t vec_per_block, uint32_t grid,
                                     uint32_t unroll, bool nt, uint32_t *sink, hipStream_t s)
{
    switch (unroll) {
    case 4: return launch_read_nt<THREADS, 4>(src, n_vec, vec_per_block, grid, nt, sink, s);
    case 8: return launch_read_nt<THREADS, 8>(src, n_vec, vec_per_block, grid, nt, sink, s);
    case 16: return launch_read_nt<THREADS, 16>(src, n_vec, vec_per_block, grid, nt, sink, s);
    }
    return hipErrorInvalidValue;
}

} // namespace zen

using namespace zen;

extern "C" zen_status zen_calibration_read(const void *src, uint64_t bytes, const zen_read_shape *host_shape,
                                           uint32_t *sink, void *hip_stream)
{
    if (!src || !sink || bytes == 0 || (bytes & 15u) || ((uintptr_t)src & 15u) || ((uintptr_t)sink & 3u)) return ZEN_ERR_INVALID;
    zen_read_shape sh = {256u, 8u, 128u * 1024u, 0u, 1u};     // the dense scan's own shape
    if (host_shape) sh = *host_shape;
    if ((sh.threads != 256 && sh.threads != 512 && sh.threads != 1024) || (sh.unroll != 4 && sh.unroll != 8 && sh.unroll != 16) ||
        sh.block_bytes < 4096 || (sh.block_bytes & 15u) || sh.nontemporal > 1u)
        return ZEN_ERR_INVALID;
    const uint64_t n_vec = bytes / 16, vec_per_block = sh.block_bytes / 16;
    uint64_t grid = (n_vec + vec_per_block - 1) / vec_per_block;
    if (sh.max_blocks && grid > sh.max_blocks) grid = sh.max_blocks;
    if (grid > 0x7FFFFFFFull) return ZEN_ERR_INVALID;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e;
    if (sh.threads == 256) e = launch_read_unroll<256>((const u32x4 *)src, n_vec, vec_per_block, (uint32_t)grid, sh.unroll, sh.nontemporal != 0, sink, s);
    else if (sh.threads == 512) e = launch_read_unroll<512>((const u32x4 *)src, n_vec, vec_per_block, (uint32_t)grid, sh.unroll, sh.nontemporal != 0, sink, s);
    else e = launch_read_unroll<1024>((const u32x4 *)src, n_vec, vec_per_block, (uint32_t)grid, sh.unroll, sh.nontemporal != 0, sink, s);
    return e == hipSuccess ? ZEN_OK : ZEN_ERR_DEVICE;
}
