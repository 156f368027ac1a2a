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
                uint32_t *wave_tot, uint32_t *uni_words)
{
    // wave_tot / uni_words (element-level merges, else NULL): the same counts per wave of the block,
    // [server][chunk][row][4], and the union words, [server][chunk][256] -- the merge starts from them
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
    if (uni_words) uni_words[((uint64_t)server * n_chunks + chunk) * BM_CHUNK_WORDS + threadIdx.x] = uni;
    __syncthreads();
    if (wt)
        for (uint32_t i = threadIdx.x; i < (a.n_in + 1) * 4; i += BM_THREADS) wt[i] = s_wt[i];
    uint32_t *out = cnt + ((uint64_t)server * (ZEN_MAX_BATCH + 1)) * n_chunks;
    if (threadIdx.x <= a.n_in) out[(uint64_t)threadIdx.x * n_chunks + chunk] = s_c[threadIdx.x];
}

// Exclusive scan over the chunks of every row; one block per server, one wave per row at a time.
// Also: *count = U, per-server flags (a part whose bitmap and row count disagree; output capacity).
__global__ void __launch_bounds__(1024)
bm_scan_kernel(BmArgs a, uint32_t *cnt, uint32_t n_chunks, uint32_t *counters_base, AggOut outs)
{
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

// Merge: one block per (chunk, server).  D == 1: one thread per bitmap word, private LDS
// accumulators for the word's up-to-32 output elements.  D > 1: one wave per word, lane w holds
// part w's word, rows are summed column block by column block in registers.
__global__ void __launch_bounds__(BM_THREADS)
bm_merge_kernel(BmArgs a, Arr64<const float *> src_values, uint32_t row_dim, uint32_t n_servers,
                const uint32_t *domain, const uint32_t *dom_offsets, const uint32_t *word_off,
                const uint32_t *cnt, uint32_t n_chunks, uint32_t *counters_base, AggOut outs,
                Arr64<float *> out_values, zen_status_info *status, const uint32_t *wave_tot,
                const uint32_t *uni_words)
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
    float *s_acc = (float *)(smem + (ZEN_MAX_BATCH + 1) * 4);   // D == 1: [<= 8192] output elements of the chunk

    const uint32_t k = chunk * BM_CHUNK_WORDS + threadIdx.x;    // this thread's bitmap word
    if (D == 1) {
        // Wave-local tables: each wave owns 64 consecutive bitmap words and the contiguous range of
        // output elements they produce.
        uint32_t *s_word = (uint32_t *)(s_acc + BM_CHUNK_WORDS * 32) + wave * 4 * ZEN_WAVE;   // part's words
        uint32_t *s_ex = s_word + ZEN_WAVE;      // exclusive count of the part's bits before each word
        uint32_t *s_uni = s_ex + ZEN_WAVE;       // union words
        uint32_t *s_uex = s_uni + ZEN_WAVE;      // exclusive count of union bits before each word
        // pass A: the union word and every part's per-wave totals, as the count kernel left them
        const uint32_t uni = uni_words[((uint64_t)server * n_chunks + chunk) * BM_CHUNK_WORDS + threadIdx.x];
        {
            const uint32_t *wt = wave_tot + ((uint64_t)server * n_chunks + chunk) * (ZEN_MAX_BATCH + 1) * 4;
            for (uint32_t i = threadIdx.x; i < n_in * 4; i += BM_THREADS) s_wtot[i] = wt[i];
        }
        const uint32_t uc = __popc(uni);
        const uint32_t uinc = wave_inclusive_scan(uc);
        const uint32_t u_wave = __shfl(uinc, ZEN_WAVE - 1, ZEN_WAVE);      // output elements of this wave
        if (lane == ZEN_WAVE - 1) s_wtot[n_in * 4 + wave] = uinc;
        s_uni[lane] = uni;
        s_uex[lane] = uinc - uc;
        __syncthreads();
        uint32_t ubase_wave = 0;                      // first output element of this wave, chunk-relative
        for (uint32_t v = 0; v < wave; ++v) ubase_wave += s_wtot[n_in * 4 + v];
        float *acc = s_acc + ubase_wave;
        for (uint32_t i = lane; i < u_wave; i += ZEN_WAVE) acc[i] = 0.f;
        // pass B: every part adds its values, in part order; the wave walks the part's values (a
        // contiguous run) and finds each value's (word, bit) by searching the prefix tables
        // lane w works out where part w's values for this wave start (one load for all parts, not one per part
        // on the way)
        uint32_t my_vbase = 0;
        if (lane < n_in) {
            my_vbase = pre[(uint64_t)lane * n_chunks + chunk];
            for (uint32_t v = 0; v < wave; ++v) my_vbase += s_wtot[lane * 4 + v];
        }
        for (uint32_t w0 = 0; w0 < n_in; w0 += 8) {
          uint32_t wd[8];
#pragma unroll
          for (uint32_t q = 0; q < 8; ++q)
              wd[q] = (w0 + q < n_in && k < n_words) ? part_words(a, w0 + q, p, word_off)[k] : 0u;
#pragma unroll
          for (uint32_t q = 0; q < 8; ++q) {
            const uint32_t w = w0 + q;
            if (w >= n_in) break;
            const uint32_t word = wd[q];
            const uint32_t vbase = (uint32_t)__builtin_amdgcn_readlane((int)my_vbase, (int)w);   // every lane is active here
            if (ballot(word != 0) == 0) continue;     // wave-uniform: the part has no row in these 64 words
            const uint32_t c = __popc(word);
            const uint32_t inc = wave_inclusive_scan(c);
            const uint32_t t_wave = __shfl(inc, ZEN_WAVE - 1, ZEN_WAVE);
            s_word[lane] = word;
            s_ex[lane] = inc - c;
            const float *vals = src_values.v[w] + vbase;
            __builtin_amdgcn_wave_barrier();
            for (uint32_t i = lane; i < t_wave; i += ZEN_WAVE) {
                uint32_t lo = 0;
#pragma unroll
                for (uint32_t st = 32; st > 0; st >>= 1)
                    if (s_ex[lo + st] <= i) lo += st;       // last word whose exclusive count <= i ...
                // ... that is non-empty: words with zero bits share their successor's count
                const uint32_t ww = s_word[lo];
                uint32_t r = i - s_ex[lo], pos = 0;
#pragma unroll
                for (uint32_t sh = 16; sh > 0; sh >>= 1) {
                    const uint32_t lowcnt = __popc((ww >> pos) & ((1u << sh) - 1u));
                    if (r >= lowcnt) { r -= lowcnt; pos += sh; }
                }
                acc[s_uex[lo] + __popc(s_uni[lo] & ((1u << pos) - 1u))] += vals[i];
            }
            __builtin_amdgcn_wave_barrier();
          }
        }
        // write out the wave's output range: indices from the sorted domain, values from LDS
        const uint32_t k0 = chunk * BM_CHUNK_WORDS + wave * ZEN_WAVE;
        const uint64_t nzu = ballot(uni != 0);
        if ((uint32_t)__popcll(nzu) < 8 * ((u_wave + ZEN_WAVE - 1) / ZEN_WAVE)) {
            uint64_t todo = nzu;
            while (todo) {   // uniform; as above: two union words per trip, a lane per bit
                const uint32_t wa = (uint32_t)__ffsll((unsigned long long)todo) - 1;
                todo &= todo - 1;
                uint32_t wb = ZEN_WAVE;
                if (todo) { wb = (uint32_t)__ffsll((unsigned long long)todo) - 1; todo &= todo - 1; }
                const uint32_t src = lane < 32 ? wa : wb, bit = lane & 31u;
                if (src < ZEN_WAVE) {
                    const uint32_t ww = s_uni[src];
                    if ((ww >> bit) & 1u) {
                        const uint32_t i = s_uex[src] + __popc(ww & ((1u << bit) - 1u));
                        const uint64_t orow = (uint64_t)ubase_chunk + ubase_wave + i;
                        if (orow < cap_rows) {
                            out_idx[orow] = domain[d0 + (k0 + src) * 32 + bit];
                            out_val[orow] = acc[i];
                        }
                    }
                }
            }
            return;
        }
        for (uint32_t i = lane; i < u_wave; i += ZEN_WAVE) {
            uint32_t lo = 0;
#pragma unroll
            for (uint32_t st = 32; st > 0; st >>= 1)
                if (s_uex[lo + st] <= i) lo += st;
            const uint32_t ww = s_uni[lo];
            uint32_t r = i - s_uex[lo], pos = 0;
#pragma unroll
            for (uint32_t sh = 16; sh > 0; sh >>= 1) {
                const uint32_t lowcnt = __popc((ww >> pos) & ((1u << sh) - 1u));
                if (r >= lowcnt) { r -= lowcnt; pos += sh; }
            }
            const uint64_t orow = (uint64_t)ubase_chunk + ubase_wave + i;
            if (orow < cap_rows) {
                out_idx[orow] = domain[d0 + (k0 + lo) * 32 + pos];
                out_val[orow] = acc[i];
            }
        }
    } else {
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
    uint32_t *wave_tot = ctx->geo.row_dim == 1 ? (uint32_t *)(ws + L.bmwave_off) : nullptr;
    uint32_t *uni_words = ctx->geo.row_dim == 1 ? (uint32_t *)(ws + L.bmuni_off) : nullptr;
    {
        ProfScope prof(ctx, K_BM_COUNT, s);
        bm_count_kernel<<<dim3(n_chunks, n_servers), BM_THREADS, 0, s>>>(a, ctx->d_dom_offsets, ctx->d_bm_word_off, cnt,
                                                                         n_chunks, wave_tot, uni_words);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        ProfScope prof(ctx, K_BM_SCAN, s);
        bm_scan_kernel<<<n_servers, 1024, 0, s>>>(a, cnt, n_chunks, counters, outs);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        ProfScope prof(ctx, K_BM_MERGE, s);
        const size_t lds = (size_t)(ZEN_MAX_BATCH + 1) * 4 * 4 +
                           (ctx->geo.row_dim == 1 ? (size_t)BM_CHUNK_WORDS * 32 * 4 + 4 * 4 * ZEN_WAVE * 4
                                                  : (size_t)(ZEN_MAX_BATCH + 1) * BM_CHUNK_WORDS * 2);
        bm_merge_kernel<<<dim3(n_chunks, n_servers), BM_THREADS, lds, s>>>(
            a, src_values, ctx->geo.row_dim, n_servers, ctx->d_domain, ctx->d_dom_offsets, ctx->d_bm_word_off, cnt,
            n_chunks, counters, outs, out_values, status, wave_tot, uni_words);
        return hipGetLastError();
    }
}

uint64_t bitmap_merge_chunks(uint64_t max_dom_words) { return (max_dom_words + BM_CHUNK_WORDS - 1) / BM_CHUNK_WORDS; }

} // namespace zen
