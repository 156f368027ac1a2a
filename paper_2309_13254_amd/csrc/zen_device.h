// Device-side helpers for the gfx950 kernels: the first-level hash h0, wave64 primitives and the
// stable per-bucket ranking shared by the partition scatter and the radix sort.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define ZEN_WAVE 64
#define ZEN_EMPTY_KEY 0xFFFFFFFFu

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace zen {

// MurmurHash3 x86_32 of one 4-byte key (section "Implementation": MurmurHash with a seed).
__device__ __forceinline__ uint32_t murmur3_u32(uint32_t key, uint32_t seed)
{
    uint32_t k = key * 0xcc9e2d51u;
    k = (k << 15) | (k >> 17);
    k *= 0x1b873593u;
    uint32_t h = seed ^ k;
    h = (h << 13) | (h >> 19);
    h = h * 5u + 0xe6546b64u;
    h ^= 4u;
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}

// h0 : idx -> [n]  (Algorithm 1: p <- h0(idx)).  pow2_mask = n-1 when n is a power of two, else 0.
__device__ __forceinline__ uint32_t owner_of(uint32_t idx, uint32_t seed, uint32_t n, uint32_t pow2_mask)
{
    uint32_t h = murmur3_u32(idx, seed);
    return pow2_mask ? (h & pow2_mask) : (n == 1 ? 0u : h % n);
}

// Slot hash of the aggregation table.  Keys that reach one server all share h0 mod n, so the table
// uses a differently seeded mix.
__device__ __forceinline__ uint32_t table_hash(uint32_t key, uint32_t seed)
{
    return murmur3_u32(key, seed ^ 0x5bd1e995u);
}

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (ZEN_WAVE - 1); }

__device__ __forceinline__ uint64_t ballot(bool pred) { return __builtin_amdgcn_ballot_w64(pred); }

// number of set bits of `m` strictly below this lane
__device__ __forceinline__ uint32_t mbcnt(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t nonzero_mag(u32x4 v)
{
    return (v.x | v.y | v.z | v.w) & 0x7fffffffu;
}

// Inclusive scan over the 64 lanes of a wave, in six data-parallel-primitive adds and without the LDS
// crossbar: shifts by 1, 2, 4, 8 inside each row of 16 lanes (a lane shifted in from outside the row
// adds 0), then lane 15 of rows 0 and 2 added to all of rows 1 and 3, then lane 31 added to rows 2 and
// 3.  The active lanes must be lanes [0, n) of the wave for some n (lanes that are off add nothing).
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);   // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

// Sum over the wave, the same in every lane; all 64 lanes must be active.
__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_scan(v), ZEN_WAVE - 1);
}

// Exclusive scan of one value per thread over a block of up to 1024 threads.  `s_tmp` holds at
// least 17 words.  Returns the exclusive prefix; *total receives the block sum.  Contains barriers:
// every thread of the block must call it.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *s_tmp, uint32_t *total)
{
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    uint32_t inc = wave_inclusive_scan(v);
    __syncthreads(); // s_tmp may still be read by a previous call
    if (lane == ZEN_WAVE - 1) s_tmp[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (uint32_t w = 0; w < nw; ++w) { uint32_t t = s_tmp[w]; s_tmp[w] = run; run += t; }
        s_tmp[16] = run;
    }
    __syncthreads();
    *total = s_tmp[16];
    return inc - v + s_tmp[wave];
}

// Lanes of this wave that are valid and hold the same bucket as this lane (bucket < 2^nbits).
__device__ __forceinline__ uint64_t wave_peers(bool valid, uint32_t bucket, uint32_t nbits)
{
    uint64_t peers = ballot(valid);
    for (uint32_t b = 0; b < nbits; ++b) {
        const bool bit = (bucket >> b) & 1u;
        const uint64_t m = ballot(valid && bit);
        peers &= bit ? m : ~m;
    }
    return valid ? peers : 0ull;
}

// Stable position of one item per thread inside its bucket, for a block of NW waves.
//   s_run[b]    running output position of bucket b (persists across calls; advanced here)
//   s_cnt[w][b] per-wave scratch, all zero on entry and on exit
// Items are ordered by thread index; calls are ordered in time, so a sequence of calls over
// ascending data yields ascending data inside every bucket.  Every thread of the block must call.
__device__ __forceinline__ uint32_t block_stable_rank(bool valid, uint32_t bucket, uint32_t nbits,
                                                      uint32_t n_buckets, uint32_t *s_run, uint32_t *s_cnt)
{
    const uint32_t wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const uint64_t peers = wave_peers(valid, bucket, nbits);
    const uint32_t rank_in_wave = mbcnt(peers);
    const uint32_t wave_count = (uint32_t)__popcll(peers);
    const bool leader = valid && rank_in_wave == 0;
    if (leader) s_cnt[wave * n_buckets + bucket] = wave_count;
    __syncthreads();
    uint32_t pos = 0;
    if (valid) {
        pos = s_run[bucket] + rank_in_wave;
        for (uint32_t w = 0; w < wave; ++w) pos += s_cnt[w * n_buckets + bucket];
    }
    __syncthreads();
    if (leader) {
        atomicAdd(&s_run[bucket], wave_count);
        s_cnt[wave * n_buckets + bucket] = 0;
    }
    (void)nw;
    return pos;
}

__device__ __forceinline__ uint32_t ceil_log2(uint32_t n)
{
    uint32_t b = 0;
    while ((1u << b) < n) ++b;
    return b;
}

} // namespace zen
