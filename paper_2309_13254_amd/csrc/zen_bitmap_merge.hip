// Aggregation of parts that all arrive as hash bitmaps (Algorithm 2), done in the bitmaps' own
// domain: bit j of every part means the same row II_p[j], so
//   union of the index sets      = bitwise OR of the bitmaps,
//   output position of a row     = number of union bits before it   (ascending: II_p is sorted),
//   position of a row in part w  = number of part-w bits before it  (the k-th set bit owns value k).
// Three launches for all servers: per-chunk popcounts -> exclusive scans over chunks -> merge.
// No hash table, no sort, no atomics on values; every output element is the sum of its
// contributors in ascending part order, so results are reproducible bit for bit.
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int BM_THREADS = 256;
static constexpr int BM_CHUNK_WORDS = 256;          // bitmap words per block = one per thread
enum : uint32_t { CNT_UNIQUE = 0, CNT_SKIP = 2, CNT_FLAGS = 3, CNT_NEEDED = 4 };

struct BmArgs {
    const uint32_t *bitmap[ZEN_MAX_BATCH];   // per part: whole bitmap (batch) or the partition's words (single)
    const uint32_t *bounds[ZEN_MAX_BATCH];   // per part: offsets array (batch) or count scalar (single)
    uint32_t n_in, single, first_part;
};

__device__ __forceinline__ const uint32_t *part_words(const BmArgs &a, uint32_t w, uint32_t p, const uint32_t *word_off)
{
    return a.bitmap[w] + (a.single ? 0u : word_off[p]);
}

// cnt[server][row][chunk]: row w < n_in = set bits of part w in the chunk, row n_in = union bits.
__global__ void __launch_bounds__(BM_THREADS)
bm_count_kernel(BmArgs a, const uint32_t *dom_offsets, const uint32_t *word_off, uint32_t *cnt, uint32_t n_chunks,
                uint32_t *wave_tot)
{
    // wave_tot (element-level merges, else NULL): the same counts per wave of the block, [server][chunk][row][4]:
    // where each wave of the merge starts in every part's values and in the output
    __shared__ uint32_t s_c[ZEN_MAX_BATCH + 1];
    __shared__ uint32_t s_wt[(ZEN_MAX_BATCH + 1) * 4];   // the same per wave of the block
    const uint32_t chunk = blockIdx.x, server = blockIdx.y, p = a.first_part + server;
    const uint32_t n_dom = dom_offsets[p + 1] - dom_offsets[p], n_words = (n_dom + 31) >> 5;
    const uint32_t k = chunk * BM_CHUNK_WORDS + threadIdx.x;
    uint32_t *wt = wave_tot ? wave_tot + ((uint64_t)server * n_chunks + chunk) * (ZEN_MAX_BATCH + 1) * 4 : nullptr;
    if (threadIdx.x <= a.n_in) s_c[threadIdx.x] = 0;
    __syncthreads();
    uint32_t uni = 0;
    for (uint32_t w0 = 0; w0 < a.n_in; w0 += 8) {
        uint32_t wd[8];
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q)
            wd[q] = (w0 + q < a.n_in && k < n_words) ? part_words(a, w0 + q, p, word_off)[k] : 0u;
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) {
            if (w0 + q >= a.n_in) break;
            uni |= wd[q];
            const uint32_t s = ballot(wd[q] != 0) ? wave_sum(__popc(wd[q])) : 0u;   // (uniform)
            if (lane_id() == 0) {
                if (s) atomicAdd(&s_c[w0 + q], s);
                s_wt[(w0 + q) * 4 + (threadIdx.x >> 6)] = s;
            }
        }
    }
    const uint32_t su = wave_sum(__popc(uni));
    if (lane_id() == 0) {
        if (su) atomicAdd(&s_c[a.n_in], su);
        s_wt[a.n_in * 4 + (threadIdx.x >> 6)] = su;
    }
    __syncthreads();
    if (wt)
        for (uint32_t i = threadIdx.x; i < (a.n_in + 1) * 4; i += BM_THREADS) wt[i] = s_wt[i];
    uint32_t *out = cnt + ((uint64_t)server * (ZEN_MAX_BATCH + 1)) * n_chunks;
    if (threadIdx.x <= a.n_in) out[(uint64_t)threadIdx.x * n_chunks + chunk] = s_c[threadIdx.x];
}

// Exclusive scan over the chunks of every row; one block per server, one wave per row at a time.
// Also: *count = U, per-server flags (a part whose bitmap and row count disagree; output capacity).
__global__ void __launch_bounds__(1024)
bm_scan_kernel(BmArgs a, uint32_t *cnt, uint32_t n_chunks, uint32_t *counters_base, AggOut outs,
               Arr64<const float *> src_values, uint64_t *tabs)
{
    // tabs (element-level merges, else NULL): the parts' bitmap pointers [64] and value pointers [64] as tables in
    // memory for the merge, whose lanes differ in the part they read (thread w copies part w's: one load per
    // thread from the argument buffer, all under way at once)
    if (tabs && blockIdx.x == 0 && threadIdx.x < ZEN_MAX_BATCH) {
        tabs[threadIdx.x] = (uint64_t)(uintptr_t)a.bitmap[threadIdx.x];
        tabs[ZEN_MAX_BATCH + threadIdx.x] = (uint64_t)(uintptr_t)src_values.v[threadIdx.x];
    }
    __shared__ uint32_t s_flags;
    const uint32_t server = blockIdx.x, p = a.first_part + server;
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    uint32_t *base = cnt + ((uint64_t)server * (ZEN_MAX_BATCH + 1)) * n_chunks;
    uint32_t *counters = counters_base + server * 16;
    if (threadIdx.x == 0) s_flags = 0;
    __syncthreads();
    const uint32_t per = (n_chunks + ZEN_WAVE - 1) / ZEN_WAVE;
    for (uint32_t row = wave; row <= a.n_in; row += nw) {
        uint32_t *r = base + (uint64_t)row * n_chunks;
        const uint32_t c0 = min(lane * per, n_chunks), c1 = min(c0 + per, n_chunks);
        uint32_t sum = 0;
        for (uint32_t c = c0; c < c1; ++c) sum += r[c];
        const uint32_t inc = wave_inclusive_scan(sum);
        // a part's prefixes start at the first value of partition p inside the part's value array
        uint32_t run = inc - sum + ((row < a.n_in && !a.single) ? a.bounds[row][p] : 0u);
        for (uint32_t c = c0; c < c1; ++c) { const uint32_t t = r[c]; r[c] = run; run += t; }
        const uint32_t total = __shfl(inc, ZEN_WAVE - 1, ZEN_WAVE);
        if (lane == 0) {
            if (row < a.n_in) {
                const uint32_t expect = a.single ? a.bounds[row][0] : a.bounds[row][p + 1] - a.bounds[row][p];
                if (expect != total) atomicOr(&s_flags, 4u);
            } else {
                const uint64_t cap_rows = outs.cap_rows[server];
                *outs.count[server] = total;
                counters[CNT_UNIQUE] = total;
                counters[CNT_SKIP] = 0;
                counters[CNT_NEEDED] = (uint64_t)total > cap_rows ? total : 0u;
                if ((uint64_t)total > cap_rows) atomicOr(&s_flags, 1u);
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        counters[CNT_FLAGS] = s_flags;
        if (s_flags & 4u) {
            // a part's bitmap and row count disagree: its set bits would index past its values.  The server
            // puts out nothing and the merge does not touch its parts.
            *outs.count[server] = 0;
            counters[CNT_UNIQUE] = 0;
            counters[CNT_SKIP] = 1;
        }
    }
}

// Merge of rows of several floats: one block per (chunk, server), one wave per word, lane w holds part w's
// word, rows are summed column block by column block in registers.  (Element-level parts: bm_merge_lanes_kernel.)
__global__ void __launch_bounds__(BM_THREADS)
bm_merge_kernel(BmArgs a, Arr64<const float *> src_values, uint32_t row_dim, uint32_t n_servers,
                const uint32_t *domain, const uint32_t *dom_offsets, const uint32_t *word_off,
                const uint32_t *cnt, uint32_t n_chunks, uint32_t *counters_base, AggOut outs,
                Arr64<float *> out_values, zen_status_info *status)
{
    extern __shared__ uint32_t smem[];
    const uint32_t chunk = blockIdx.x, server = blockIdx.y, p = a.first_part + server;
    const uint32_t D = row_dim, n_in = a.n_in;
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    if (chunk == 0 && server == 0 && threadIdx.x == 0) {
        uint32_t fl = 0, need = 0;
        for (uint32_t j = 0; j < n_servers; ++j) {
            fl |= counters_base[j * 16 + CNT_FLAGS];
            need = max(need, counters_base[j * 16 + CNT_NEEDED]);
        }
        status->flags = fl;
        status->reserved = 0;
        status->needed_rows = need;
    }
    if (counters_base[server * 16 + CNT_SKIP]) return;   // inconsistent parts (uniform per block)
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    if (chunk * BM_CHUNK_WORDS >= n_words) return;
    const uint32_t *pre = cnt + ((uint64_t)server * (ZEN_MAX_BATCH + 1)) * n_chunks;   // exclusive prefixes (+ value base)
    const uint64_t cap_rows = outs.cap_rows[server];
    uint32_t *__restrict__ out_idx = outs.indices[server];
    float *__restrict__ out_val = out_values.v[server];
    const uint32_t ubase_chunk = pre[(uint64_t)n_in * n_chunks + chunk];

    uint32_t *s_wtot = smem;                       // [n_in + 1][4] per-wave totals of the chunk

    const uint32_t k = chunk * BM_CHUNK_WORDS + threadIdx.x;    // this thread's bitmap word
    {
        // per-part, per-word exclusive positions inside the chunk: s_pre[w][word] (u16, <= 8192)
        uint16_t *s_pre = (uint16_t *)(smem + (ZEN_MAX_BATCH + 1) * 4);     // [n_in + 1][256]
        for (uint32_t w = 0; w <= n_in; ++w) {
            uint32_t word = 0;
            if (k < n_words) {
                if (w < n_in) word = part_words(a, w, p, word_off)[k];
                else for (uint32_t v = 0; v < n_in; ++v) word |= part_words(a, v, p, word_off)[k];
            }
            const uint32_t c = __popc(word);
            const uint32_t inc = wave_inclusive_scan(c);
            if (lane == ZEN_WAVE - 1) s_wtot[w * 4 + wave] = inc;
            s_pre[w * BM_CHUNK_WORDS + threadIdx.x] = (uint16_t)(inc - c);
        }
        __syncthreads();
        // one wave per word; lane w keeps part w's word and its value position
        for (uint32_t wi = wave; wi < BM_CHUNK_WORDS; wi += (BM_THREADS >> 6)) {
            const uint32_t kw = chunk * BM_CHUNK_WORDS + wi;
            if (kw >= n_words) break;
            const uint32_t src_wave = wi >> 6;       // the wave whose scan produced s_pre[..][wi]
            uint32_t myword = 0, mypos = 0;
            if (lane < n_in) {
                myword = part_words(a, lane, p, word_off)[kw];
                mypos = pre[(uint64_t)lane * n_chunks + chunk] + s_pre[lane * BM_CHUNK_WORDS + wi];
                for (uint32_t v = 0; v < src_wave; ++v) mypos += s_wtot[lane * 4 + v];
            }
            uint32_t uni = myword;
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) uni |= __shfl_xor(uni, d, ZEN_WAVE);
            uint32_t urow = ubase_chunk + s_pre[n_in * BM_CHUNK_WORDS + wi];
            for (uint32_t v = 0; v < src_wave; ++v) urow += s_wtot[n_in * 4 + v];
            uint32_t u = uni;
            while (u) {
                const uint32_t b = __ffs(u) - 1;
                u &= u - 1;
                const uint64_t has = ballot(((myword >> b) & 1u) != 0);          // parts that hold this row
                const uint32_t my_src = mypos + __popc(myword & ((1u << b) - 1u));
                if ((uint64_t)urow < cap_rows) {
                    if (lane == 0) out_idx[urow] = domain[d0 + kw * 32 + b];
                    float *o = out_val + (uint64_t)urow * D;
                    for (uint32_t c0 = 0; c0 < D; c0 += ZEN_WAVE) {
                        float acc = 0.f;
                        uint64_t h = has;
                        while (h) {
                            const uint32_t w = (uint32_t)__ffsll((unsigned long long)h) - 1;
                            h &= h - 1;
                            const uint32_t srow = __shfl(my_src, w, ZEN_WAVE);
                            if (c0 + lane < D) acc += src_values.v[w][(uint64_t)srow * D + c0 + lane];
                        }
                        if (c0 + lane < D) o[c0 + lane] = acc;
                    }
                }
                ++urow;
            }
        }
    }
}

// Element-level merge with a LANE PER PART.  Bit j of every part's bitmap is the same row, so a wave that takes
// a span of 64 consecutive bits can let lane b stand for bit b: for every part that has a bit in the span (the
// parts are found by one ballot over the lanes, which each hold their own part's 64 bits), the part's mask is
// broadcast as a scalar, lane b adds that part's value number (values before the span) + (set bits below b),
// a coalesced load; the union is the OR of the scalars and lane b's output position the number of union bits
// below it.  No search, no accumulators in LDS, no atomics; values are added in ascending part order starting
// from -0 (so the first one is copied: -0 + x = x), hence every result is the same on every run and a row with
// one contributor keeps its bits (a signalling NaN comes out quiet).
// A block takes a chunk of 256 words as the count kernel does, a wave 64 words = 32 spans.
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef const __attribute__((address_space(1))) float *gfloat_ptr;   // pointers known to be to global memory (they are
typedef const __attribute__((address_space(1))) uint32_t *gu32_ptr;  // rebuilt from integers, which hides that)
typedef const __attribute__((address_space(1))) u32x4_a4 *gu32x4_ptr;

__device__ __forceinline__ uint64_t readlane64(uint64_t v, uint32_t src)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, (int)src);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), (int)src);
    return ((uint64_t)hi << 32) | lo;
}

__global__ void __launch_bounds__(BM_THREADS)
bm_merge_lanes_kernel(BmArgs a, const uint64_t *tabs, uint32_t n_servers, const uint32_t *domain,
                      const uint32_t *dom_offsets, const uint32_t *word_off, const uint32_t *cnt, uint32_t n_chunks,
                      const uint32_t *counters_base, AggOut outs, Arr64<float *> out_values, zen_status_info *status,
                      const uint32_t *wave_tot)
{
    const uint32_t chunk = blockIdx.x, server = blockIdx.y, p = a.first_part + server;
    const uint32_t n_in = a.n_in, lane = lane_id(), wave = threadIdx.x >> 6;
    if (chunk == 0 && server == 0 && threadIdx.x == 0) {
        uint32_t fl = 0, need = 0;
        for (uint32_t j = 0; j < n_servers; ++j) {
            fl |= counters_base[j * 16 + CNT_FLAGS];
            need = max(need, counters_base[j * 16 + CNT_NEEDED]);
        }
        status->flags = fl;
        status->reserved = 0;
        status->needed_rows = need;
    }
    if (counters_base[server * 16 + CNT_SKIP]) return;   // inconsistent parts (uniform per block)
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0, n_words = (n_dom + 31) >> 5;
    const uint32_t k0 = chunk * BM_CHUNK_WORDS + wave * ZEN_WAVE;   // the wave's first bitmap word
    if (k0 >= n_words) return;                                       // uniform per wave
    const uint32_t *pre = cnt + ((uint64_t)server * (ZEN_MAX_BATCH + 1)) * n_chunks;   // exclusive prefixes (+ value base)
    const uint32_t *wt = wave_tot + ((uint64_t)server * n_chunks + chunk) * (ZEN_MAX_BATCH + 1) * 4;
    const uint64_t cap_rows = outs.cap_rows[server];
    uint32_t *__restrict__ out_idx = outs.indices[server];
    float *__restrict__ out_val = out_values.v[server];

    // lane w: where part w's words and values for this wave start
    uint64_t bmbase = 0;       // part w's first word of the wave (an address: lanes hand it round as two words)
    uint64_t vaddr = 0;        // address of part w's first value at or after the current span
    if (lane < n_in) {
        bmbase = (uint64_t)(uintptr_t)((const uint32_t *)(uintptr_t)tabs[lane] + (a.single ? 0u : word_off[p]) + k0);
        uint32_t voff = pre[(uint64_t)lane * n_chunks + chunk];
        for (uint32_t v = 0; v < wave; ++v) voff += wt[lane * 4 + v];
        vaddr = tabs[ZEN_MAX_BATCH + lane] + 4ull * voff;
    }
    uint32_t ubase = pre[(uint64_t)n_in * n_chunks + chunk];         // first output row of this wave (uniform)
    for (uint32_t v = 0; v < wave; ++v) ubase += wt[n_in * 4 + v];

    // The wave's 64 words of every part, a half (32 words = 16 spans) at a time: read part by part with
    // consecutive lanes on consecutive words (two parts per load: a load whose lanes sit in 64 parts costs 64
    // address translations, and the translation misses of such loads were what bounded this kernel), turned
    // round in LDS so that lane w holds part w's words.
    extern __shared__ uint32_t smem[];
    constexpr uint32_t HW = 32, LSTRIDE = HW + 1;                    // odd stride: the turned reads hit 64 banks
    uint32_t *s_m = smem + wave * (ZEN_WAVE * LSTRIDE);
    uint64_t *s_ptr = (uint64_t *)(smem + (BM_THREADS / ZEN_WAVE) * (ZEN_WAVE * LSTRIDE)) + wave * ZEN_WAVE;   // [64] the parts' word pointers
    s_ptr[lane] = lane < n_in ? bmbase : readlane64(bmbase, 0);     // a valid address for every lane
    __builtin_amdgcn_wave_barrier();
    constexpr uint32_t GS = 4, SLOTS = 8;
    for (uint32_t half = 0; half < ZEN_WAVE / HW; ++half) {
        const uint32_t kw = k0 + half * HW;                          // first word of this half
        if (kw >= n_words) break;                                    // uniform
        {
            const uint32_t q = lane & (HW - 1), hi = lane >> 5;
            const bool inside = kw + q < n_words;
            uint32_t t[ZEN_WAVE / 2];
#pragma unroll
            for (uint32_t it = 0; it < ZEN_WAVE / 2; ++it) {         // parts 2 it and 2 it + 1
                t[it] = 0u;
                if (2 * it < n_in) {                                 // uniform
                    const gu32_ptr src = (gu32_ptr)(uintptr_t)s_ptr[2 * it + hi];
                    if (inside) t[it] = src[half * HW + q];          // (a lane beyond the last part reads part 0's word)
                }
            }
            __builtin_amdgcn_wave_barrier();                         // the last half's reads are done
#pragma unroll
            for (uint32_t it = 0; it < ZEN_WAVE / 2; ++it) s_m[(2 * it + hi) * LSTRIDE + q] = t[it];
            __builtin_amdgcn_wave_barrier();
        }
#pragma unroll 1
        for (uint32_t qt = 0; qt < 2; ++qt) {
        constexpr uint32_t QW = HW / 2;                              // a quarter of the wave's words: eight spans
        uint32_t m[QW];
#pragma unroll
        for (uint32_t q = 0; q < QW; ++q) m[q] = lane < n_in ? s_m[lane * LSTRIDE + qt * QW + q] : 0u;
#pragma unroll
        for (uint32_t grp = 0; grp < QW / (2 * GS); ++grp) {
            // groups of four spans: the value loads of all four are under way before any is consumed
            float v[GS][SLOTS];
            uint32_t row[GS];
            uint64_t mine[GS], uni[GS], rest[GS], vaddr_at[GS];
#pragma unroll
            for (uint32_t sp = 0; sp < GS; ++sp) {
                const uint32_t wq = (grp * GS + sp) * 2;                               // the span's first word of the quarter
                mine[sp] = ((uint64_t)m[wq + 1] << 32) | m[wq];                        // part `lane`'s bits of this span
                uint64_t active = ballot(mine[sp] != 0);                               // parts with a bit in the span
                const uint32_t bitpos = (kw + qt * QW + wq) * 32 + lane;               // this lane's bit = row II_p[bitpos]
                row[sp] = 0;
                if (active != 0 && bitpos < n_dom) row[sp] = domain[d0 + bitpos];
                uni[sp] = 0;
                vaddr_at[sp] = vaddr;
#pragma unroll
                for (uint32_t j = 0; j < SLOTS; ++j) {                                 // the span's first eight parts
                    v[sp][j] = -0.0f;                                                  // x + (-0) = x for every x: an empty slot adds nothing
                    if (active) {                                                      // uniform
                        const uint32_t w = (uint32_t)__ffsll((unsigned long long)active) - 1;
                        active &= active - 1;
                        const uint64_t pm = readlane64(mine[sp], w);                  // part w's bits, a scalar
                        const gfloat_ptr pv = (gfloat_ptr)(uintptr_t)readlane64(vaddr, w);   // its first value of the span
                        uni[sp] |= pm;
                        if (__builtin_amdgcn_inverse_ballot_w64(pm)) v[sp][j] = pv[mbcnt(pm)];   // + set bits below this lane
                    }
                }
                rest[sp] = active;
                vaddr += 4ull * (uint32_t)__popcll(mine[sp]);                          // lanes beyond n_in hold no bits
            }
#pragma unroll
            for (uint32_t sp = 0; sp < GS; ++sp) {
                if (uni[sp] == 0) continue;                                            // uniform
                float acc = -0.0f;                                                     // (-0) + x = x: the first value is copied
#pragma unroll
                for (uint32_t j = 0; j < SLOTS; ++j) acc += v[sp][j];                  // ascending part order
                uint64_t active = rest[sp];
                while (active) {                                                       // a span with more than eight parts
                    const uint32_t w = (uint32_t)__ffsll((unsigned long long)active) - 1;
                    active &= active - 1;
                    const uint64_t pm = readlane64(mine[sp], w);
                    const gfloat_ptr pv = (gfloat_ptr)(uintptr_t)readlane64(vaddr_at[sp], w);
                    uni[sp] |= pm;
                    float x = -0.0f;
                    if (__builtin_amdgcn_inverse_ballot_w64(pm)) x = pv[mbcnt(pm)];
                    acc += x;
                }
                const uint32_t o = ubase + mbcnt(uni[sp]);
                if (__builtin_amdgcn_inverse_ballot_w64(uni[sp]) && (uint64_t)o < cap_rows) {
                    out_idx[o] = row[sp];
                    out_val[o] = acc;
                }
                ubase += (uint32_t)__popcll(uni[sp]);
            }
        }
        }
    }
}

hipError_t launch_bitmap_merge(zen_ctx *ctx, const Arr64<const uint32_t *> &bitmaps,
                               const Arr64<const uint32_t *> &bounds, const Arr64<const float *> &src_values,
                               uint32_t n_in, bool single, uint32_t n_servers, uint32_t first_part,
                               const AggOut &outs, const Arr64<float *> &out_values, char *ws, const AggLayout &L,
                               hipStream_t s)
{
    BmArgs a;
    for (uint32_t w = 0; w < ZEN_MAX_BATCH; ++w) { a.bitmap[w] = bitmaps.v[w]; a.bounds[w] = bounds.v[w]; }
    a.n_in = n_in;
    a.single = single ? 1u : 0u;
    a.first_part = first_part;
    uint32_t *cnt = (uint32_t *)(ws + L.bmcnt_off);
    uint32_t *counters = (uint32_t *)(ws + L.counters_off);
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);
    const uint32_t n_chunks = (uint32_t)L.bm_chunks;
    const bool elem = ctx->geo.row_dim == 1;
    uint32_t *wave_tot = elem ? (uint32_t *)(ws + L.bmwave_off) : nullptr;
    uint64_t *tabs = elem ? (uint64_t *)(ws + L.bmtab_off) : nullptr;
    {
        ProfScope prof(ctx, K_BM_COUNT, s);
        bm_count_kernel<<<dim3(n_chunks, n_servers), BM_THREADS, 0, s>>>(a, ctx->d_dom_offsets, ctx->d_bm_word_off, cnt,
                                                                         n_chunks, wave_tot);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        ProfScope prof(ctx, K_BM_SCAN, s);
        bm_scan_kernel<<<n_servers, 1024, 0, s>>>(a, cnt, n_chunks, counters, outs, src_values, tabs);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        ProfScope prof(ctx, K_BM_MERGE, s);
        if (elem) {
            const size_t lds_lanes = (size_t)(BM_THREADS / ZEN_WAVE) * (ZEN_WAVE * 33 * 4 + ZEN_WAVE * 8);   // a wave's 64 x 32 words, turned; its 64 pointers
            bm_merge_lanes_kernel<<<dim3(n_chunks, n_servers), BM_THREADS, lds_lanes, s>>>(
                a, tabs, n_servers, ctx->d_domain, ctx->d_dom_offsets, ctx->d_bm_word_off, cnt, n_chunks, counters, outs,
                out_values, status, wave_tot);
            return hipGetLastError();
        }
        const size_t lds = (size_t)(ZEN_MAX_BATCH + 1) * 4 * 4 + (size_t)(ZEN_MAX_BATCH + 1) * BM_CHUNK_WORDS * 2;
        bm_merge_kernel<<<dim3(n_chunks, n_servers), BM_THREADS, lds, s>>>(
            a, src_values, ctx->geo.row_dim, n_servers, ctx->d_domain, ctx->d_dom_offsets, ctx->d_bm_word_off, cnt,
            n_chunks, counters, outs, out_values, status);
        return hipGetLastError();
    }
}

uint64_t bitmap_merge_chunks(uint64_t max_dom_words) { return (max_dom_words + BM_CHUNK_WORDS - 1) / BM_CHUNK_WORDS; }

} // namespace zen
