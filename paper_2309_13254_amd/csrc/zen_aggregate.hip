// Aggregation kernels for gfx950: an open-addressing table of KEYS only (atomicCAS, linear probing), compaction
// and sort of the unique keys, a list of contributing (part, row) pairs per key, and one ordered fp32 sum per
// output row -- plain loads and one store per element, no atomics on values, no zero fill of the output.
//
// One launch covers every server of a batch: blockIdx.z (or .y) = server, blockIdx.y = incoming part.
//   large tables: clear -> insert (keys + repeat counts) -> compact -> segmented LSB radix sort of the unique keys
//                 -> finalize (each key's output rank into its slot, room for its contributor list)
//                 -> fill (every incoming row appends its id to its key's list) -> gather (ordered sums)
//   small tables: one block per server does all of it up to the lists in LDS (or merges ascending parts by
//                 binary searches, no table), then the same gather.
#include "zen_device.h"
#include "zen_internal.h"

namespace zen {

static constexpr int AGG_THREADS = 256;
static constexpr uint32_t GATHER_GROUP_ROWS = 4;   // output rows a lane group of the narrow-row gather keeps in flight
static constexpr int SMALL_THREADS = 1024;
static constexpr uint32_t SMALL_MERGE_MAX_PARTS = 16;   // small tables: parts merged by binary searches when all ascend
static constexpr uint32_t SMALL_MAX_IN = 6500;     // rows into one server that the one-block LDS path takes:
                                                   // table of 8192 slots (load <= 0.8) x 2 arrays + 8192 sorted
                                                   // keys = 96 KB of the 160 KB LDS
static constexpr int RS_ITEMS = 8;                 // radix sort: keys per thread per block
static constexpr int RS_BLOCK_KEYS = AGG_THREADS * RS_ITEMS;

enum : uint32_t { CNT_UNIQUE = 0, CNT_TOTAL_IN = 1, CNT_SKIP = 2, CNT_FLAGS = 3, CNT_NEEDED = 4, CNT_LISTED = 5 };

// rows [begin, begin+count) of idx are the part's indices; its values start at row vbegin
struct PartRange { const uint32_t *idx; uint32_t begin, count, vbegin; };

__device__ __forceinline__ uint32_t part_count(const PartIdx &src, uint32_t w, uint32_t server)
{
    if (src.single) return src.bounds[w][0];
    return src.bounds[w][src.server0 + server + 1] - src.bounds[w][src.server0 + server];
}

__device__ __forceinline__ PartRange part_range(const PartIdx &src, uint32_t w, uint32_t server)
{
    PartRange r;
    r.vbegin = src.single ? 0u : src.bounds[w][src.server0 + server];
    r.count = part_count(src, w, server);
    if (src.indices[w]) {
        r.idx = src.indices[w];
        r.begin = r.vbegin;
    } else {
        // decoded hash-bitmap part: placed after the parts before it in the server's decode area
        uint32_t pre = 0;
        for (uint32_t v = 0; v < w; ++v) pre += part_count(src, v, server);
        r.idx = src.dec_base + (uint64_t)server * src.dec_stride;
        r.begin = pre;
    }
    return r;
}

// A0: hash_bitmap_decode (Algorithm 2) of part (w, server): the k-th set bit j of the partition's
// bitmap is the row domain[dom_offsets[p] + j]; rows come out ascending.  One block per part.
__global__ void __launch_bounds__(1024)
bitmap_decode_kernel(PartIdx src, Arr64<const uint32_t *> src_bitmap, uint32_t first_part,
                     const uint32_t *domain, const uint32_t *dom_offsets, const uint32_t *word_off,
                     uint32_t *dec_base, uint64_t dec_stride, zen_status_info *status, uint32_t *dec_flags)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t w = blockIdx.x, server = blockIdx.y;
    if (src.indices[w] || !src_bitmap.v[w]) {
        if (dec_flags && threadIdx.x == 0) dec_flags[server * ZEN_MAX_BATCH + w] = 0;
        return;
    }
    const uint32_t p = first_part + server;
    const PartRange r = part_range(src, w, server);
    const uint32_t *bm = src_bitmap.v[w] + (src.single ? 0u : word_off[p]);
    const uint32_t d0 = dom_offsets[p], n_dom = dom_offsets[p + 1] - d0;
    const uint32_t n_words = (n_dom + 31) >> 5;
    uint32_t *dec = dec_base + (uint64_t)server * dec_stride;
    uint32_t run = 0;
    for (uint32_t w0 = 0; w0 < n_words; w0 += blockDim.x) {
        const uint32_t wi = w0 + threadIdx.x;
        uint32_t word = wi < n_words ? bm[wi] : 0u;
        uint32_t total;
        const uint32_t pre = block_exclusive_scan(__popc(word), s_tmp, &total);
        uint32_t k = run + pre;
        while (word) {
            const uint32_t b = __ffs(word) - 1;
            word &= word - 1;
            const uint32_t j = wi * 32 + b;
            if (j < n_dom && k < r.count && (uint64_t)r.begin + k < dec_stride) dec[r.begin + k] = domain[d0 + j];
            ++k;
        }
        run += total;
    }
    if (threadIdx.x == 0) {   // bitmap and row count must agree
        if (dec_flags) dec_flags[server * ZEN_MAX_BATCH + w] = run != r.count ? 4u : 0u;
        else if (run != r.count) atomicOr(&status->flags, 4u);
    }
}

__device__ __forceinline__ uint32_t probe_find(const uint32_t *__restrict__ keys, uint32_t cap_mask,
                                               uint32_t key, uint32_t seed)
{
    uint32_t slot = table_hash(key, seed) & cap_mask;
    for (uint32_t i = 0; i <= cap_mask; ++i) {
        const uint32_t k = keys[slot];
        if (k == key) return slot;
        if (k == ZEN_EMPTY_KEY) break;
        slot = (slot + 1) & cap_mask;
    }
    return 0xFFFFFFFFu;
}

// A1: keys = EMPTY and repeat counts = 0 for every server, counters and status zeroed.
__global__ void agg_clear_kernel(uint32_t *keys, uint32_t *occ, uint64_t n_keys, uint32_t *counters, uint32_t n_counters,
                                 zen_status_info *status)
{
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = tid; i < n_keys; i += nt) { keys[i] = ZEN_EMPTY_KEY; occ[i] = 0u; }
    for (uint64_t i = tid; i < n_counters; i += nt) counters[i] = 0;
    if (tid == 0) { status->flags = 0; status->reserved = 0; status->needed_rows = 0; }
}

// A2 (keys): claim a slot for every distinct incoming index.
__global__ void __launch_bounds__(AGG_THREADS)
agg_insert_kernel(PartIdx src, uint32_t n_in, uint32_t seed, uint32_t *keys_base, uint32_t *occ_base, uint64_t table_cap,
                  uint32_t *counters_base, uint64_t max_in_rows, zen_status_info *status)
{
    __shared__ uint32_t s_tmp[32];
    const uint32_t server = blockIdx.z, w = blockIdx.y;
    uint32_t *keys = keys_base + (uint64_t)server * table_cap;
    uint32_t *occ = occ_base + (uint64_t)server * table_cap;   // repeats of the slot's key (the rank table, until finalize)
    uint32_t *counters = counters_base + server * 16;
    const uint32_t cap_mask = (uint32_t)(table_cap - 1);

    // bound check: the table holds at most max_in_rows keys at load factor <= 1/2
    uint32_t mine = 0;
    if (threadIdx.x < n_in) mine = part_count(src, threadIdx.x, server);
    uint32_t total_in;
    block_exclusive_scan(mine, s_tmp, &total_in);
    if ((uint64_t)total_in > max_in_rows) {
        if (blockIdx.x == 0 && w == 0 && threadIdx.x == 0) {
            atomicOr(&status->flags, 2u);
            atomicMax((unsigned long long *)&status->needed_rows, (unsigned long long)total_in);
            counters[CNT_SKIP] = 1;
        }
        return;
    }
    if (blockIdx.x == 0 && w == 0 && threadIdx.x == 0) counters[CNT_TOTAL_IN] = total_in;

    const PartRange r = part_range(src, w, server);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < r.count; i += gridDim.x * blockDim.x) {
        const uint32_t key = r.idx[r.begin + i];
        if (key == ZEN_EMPTY_KEY) { atomicOr(&status->flags, 4u); continue; }
        uint32_t slot = table_hash(key, seed) & cap_mask;
        for (uint32_t t = 0; t <= cap_mask; ++t) {
            const uint32_t prev = atomicCAS(&keys[slot], ZEN_EMPTY_KEY, key);
            if (prev == ZEN_EMPTY_KEY) break;                      // claimed: the first occurrence
            if (prev == key) { atomicAdd(&occ[slot], 1u); break; }  // a repeat
            slot = (slot + 1) & cap_mask;
        }
    }
}

// The parts' value arrays as a table in memory, thread w the pointer of part w: one load per thread from the
// argument buffer, all under way at once (fetched pointer by pointer with constant indices they come one after
// the other, and the argument buffer lies in host memory).
__device__ __forceinline__ void write_src_table(const Arr64<const float *> &src_values, const float **src_tab)
{
    if (threadIdx.x < ZEN_MAX_BATCH) src_tab[threadIdx.x] = src_values.v[threadIdx.x];
}

// ----------------------------------------------------------------------------------------------
// Small tables (max_in_rows <= SMALL_MAX_IN): the whole merge of one server runs in one block with
// the open-addressing table in LDS.
//   insert every incoming index (LDS atomicCAS, linear probing) and count its occurrences
//   -> compact + bitonic-sort the unique keys -> out_indices, *count
//   -> exclusive scan of the occurrence counts in key order = row_start[] (CSR over output rows)
//   -> every incoming row appends its id (part << 32 | row in the part's values) to its key's list
// agg_gather_kernel then sums each output row from its contributor list in ascending (part, row)
// order with plain loads and one store: no value atomics, no zero fill, reproducible bit for bit.
// ----------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lds_probe(const uint32_t *tkeys, uint32_t cap_mask, uint32_t key, uint32_t seed)
{
    uint32_t slot = table_hash(key, seed) & cap_mask;
    while (tkeys[slot] != key) slot = (slot + 1) & cap_mask;   // the key is present: terminates
    return slot;
}

__global__ void __launch_bounds__(SMALL_THREADS)
agg_small_kernel(PartIdx src, uint32_t n_in, uint32_t seed, uint32_t cap, uint32_t max_in_rows,
                 uint32_t *counters_base, AggOut outs, uint32_t *rowstart_base, uint32_t *contrib_base,
                 uint64_t ws_stride, const uint32_t *dec_flags, Arr64<const float *> src_values, const float **src_tab)
{
    if (src_tab && blockIdx.x == 0) write_src_table(src_values, src_tab);   // for the gather of narrow rows
    extern __shared__ uint32_t smem[];
    uint32_t *tkeys = smem;                 // [cap]
    uint32_t *tval = tkeys + cap;           // [cap] occurrences, later the fill cursor
    uint32_t *sorted = tval + cap;          // [power of two >= max_in_rows]
    __shared__ uint32_t s_tmp[32];
    __shared__ uint32_t s_pre[ZEN_MAX_BATCH + 1];
    __shared__ uint32_t s_begin[ZEN_MAX_BATCH];
    __shared__ uint32_t s_vbegin[ZEN_MAX_BATCH];
    __shared__ const uint32_t *s_idx[ZEN_MAX_BATCH];
    __shared__ uint32_t s_n;
    const uint32_t server = blockIdx.x;
    uint32_t *counters = counters_base + server * 16;
    uint32_t *rowstart = rowstart_base + (uint64_t)server * ws_stride;
    uint64_t *contrib = (uint64_t *)(contrib_base + (uint64_t)server * ws_stride);   // ws_stride >= 2*max_in_rows
    const uint32_t cap_mask = cap - 1;

    uint32_t mine = 0, flags = 0;
    if (threadIdx.x < n_in) {
        const PartRange r = part_range(src, threadIdx.x, server);
        mine = r.count;
        s_idx[threadIdx.x] = r.idx;
        s_begin[threadIdx.x] = r.begin;
        s_vbegin[threadIdx.x] = r.vbegin;
        if (dec_flags) flags = dec_flags[server * ZEN_MAX_BATCH + threadIdx.x];
    }
    if (threadIdx.x == 0) s_n = 0;
    uint32_t total_in;
    const uint32_t pre = block_exclusive_scan(mine, s_tmp, &total_in);
    if (threadIdx.x < n_in) s_pre[threadIdx.x] = pre;
    if (threadIdx.x == 0) s_pre[n_in] = total_in;
    flags = __syncthreads_or((int)flags) ? 4u : 0u;
    if (total_in > max_in_rows) {
        if (threadIdx.x == 0) {
            *outs.count[server] = 0;
            counters[CNT_UNIQUE] = 0;
            counters[CNT_SKIP] = 1;
            counters[CNT_FLAGS] = flags | 2u;
            counters[CNT_NEEDED] = total_in;
        }
        return;
    }
    // Parts whose indices ascend strictly (what zen_encode and a decoded hash bitmap produce) need no table and
    // no sort: an element's place in the merged sequence, ordered by (index, part), is its own place in its
    // part plus, for every other part, the number of that part's elements before it -- a binary search each.
    // Heads of equal-index stretches are the output rows, the stretches themselves the contributor lists,
    // already in ascending (part, row) order.  Few parts only (the searches grow with their number).
    if (n_in <= SMALL_MERGE_MAX_PARTS) {
        uint32_t *s_key = smem;                    // [total_in] the parts' indices, part after part
        uint32_t *s_merged = smem + max_in_rows;   // [total_in] the merged sequence
        constexpr uint32_t EPT = (SMALL_MAX_IN + SMALL_THREADS - 1) / SMALL_THREADS;   // elements per thread: 7
        uint32_t key[EPT], part[EPT];
        uint32_t bad = 0;
#pragma unroll
        for (uint32_t q = 0; q < EPT; ++q) {
            const uint32_t e = q * SMALL_THREADS + threadIdx.x;
            key[q] = ZEN_EMPTY_KEY;
            part[q] = 0;
            if (e < total_in) {
                uint32_t lo = 0, hi = n_in;
                while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (s_pre[mid] <= e) lo = mid; else hi = mid; }
                part[q] = lo;
                key[q] = s_idx[lo][s_begin[lo] + (e - s_pre[lo])];
                s_key[e] = key[q];
                bad |= key[q] == ZEN_EMPTY_KEY ? 1u : 0u;
            }
        }
        __syncthreads();
#pragma unroll
        for (uint32_t q = 0; q < EPT; ++q) {
            const uint32_t e = q * SMALL_THREADS + threadIdx.x;
            if (e < total_in && e > s_pre[part[q]]) bad |= s_key[e - 1] >= key[q] ? 1u : 0u;
        }
        if (!__syncthreads_or((int)bad)) {
#pragma unroll
            for (uint32_t q = 0; q < EPT; ++q) {
                const uint32_t e = q * SMALL_THREADS + threadIdx.x;
                if (e >= total_in) continue;
                const uint32_t w = part[q], v = key[q];
                uint32_t pos = e - s_pre[w];
                for (uint32_t o = 0; o < n_in; ++o) {
                    if (o == w) continue;
                    // elements of part o before (v, w): those < v, and an equal one if o < w
                    uint32_t lo = s_pre[o], hi = s_pre[o + 1];
                    const uint32_t limit = o < w ? v + 1u : v;      // count elements < limit (v + 1 wraps only for the reserved key)
                    while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (s_key[mid] < limit) lo = mid + 1; else hi = mid; }
                    pos += lo - s_pre[o];
                }
                s_merged[pos] = v;
                contrib[pos] = ((uint64_t)w << 32) | (uint64_t)(s_vbegin[w] + (e - s_pre[w]));
            }
            __syncthreads();
            // heads -> output rows
            const uint64_t cap_rows = outs.cap_rows[server];
            uint32_t *out_idx = outs.indices[server];
            const uint32_t per = (total_in + blockDim.x - 1) / blockDim.x;
            const uint32_t a0 = min(threadIdx.x * per, total_in), a1 = min(a0 + per, total_in);
            uint32_t heads = 0;
            for (uint32_t a = a0; a < a1; ++a) heads += (a == 0 || s_merged[a] != s_merged[a - 1]) ? 1u : 0u;
            uint32_t U;
            uint32_t u = block_exclusive_scan(heads, s_tmp, &U);
            for (uint32_t a = a0; a < a1; ++a) {
                if (a == 0 || s_merged[a] != s_merged[a - 1]) {
                    rowstart[u] = a;
                    if (u < cap_rows) out_idx[u] = s_merged[a];
                    ++u;
                }
            }
            if (threadIdx.x == 0) {
                rowstart[U] = total_in;
                *outs.count[server] = U;
                counters[CNT_UNIQUE] = U;
                counters[CNT_SKIP] = 0;
                counters[CNT_FLAGS] = flags | ((uint64_t)U > cap_rows ? 1u : 0u);
                counters[CNT_NEEDED] = (uint64_t)U > cap_rows ? U : 0u;
            }
            return;
        }
    }
    for (uint32_t i = threadIdx.x; i < cap; i += blockDim.x) { tkeys[i] = ZEN_EMPTY_KEY; tval[i] = 0; }
    __syncthreads();

    // insert + count
    for (uint32_t e = threadIdx.x; e < total_in; e += blockDim.x) {
        uint32_t lo = 0, hi = n_in;
        while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (s_pre[mid] <= e) lo = mid; else hi = mid; }
        const uint32_t key = s_idx[lo][s_begin[lo] + (e - s_pre[lo])];
        if (key == ZEN_EMPTY_KEY) { flags |= 4u; continue; }
        uint32_t slot = table_hash(key, seed) & cap_mask;
        for (;;) {
            const uint32_t prev = atomicCAS(&tkeys[slot], ZEN_EMPTY_KEY, key);
            if (prev == ZEN_EMPTY_KEY || prev == key) break;
            slot = (slot + 1) & cap_mask;   // load <= 0.8: an empty slot exists
        }
        atomicAdd(&tval[slot], 1u);
    }
    __syncthreads();

    // compact + sort the unique keys
    for (uint32_t i = threadIdx.x; i < cap; i += blockDim.x) {
        const uint32_t k = tkeys[i];
        if (k != ZEN_EMPTY_KEY) sorted[atomicAdd(&s_n, 1u)] = k;
    }
    __syncthreads();
    const uint32_t U = s_n;
    uint32_t P = 1;
    while (P < U) P <<= 1;
    for (uint32_t i = U + threadIdx.x; i < P; i += blockDim.x) sorted[i] = ZEN_EMPTY_KEY;   // pad high
    __syncthreads();
    // Bitonic network.  Pair t of a stage with stride j touches elements inside [128*(t/64), +128)
    // whenever j <= 64, i.e. only data of its own wave: those stages need no block barrier.
    for (uint32_t k = 2; k <= P; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            if (j >= 128) __syncthreads();
            for (uint32_t t = threadIdx.x; t < (P >> 1); t += blockDim.x) {
                const uint32_t lo = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const uint32_t hi = lo | j;
                const bool up = (lo & k) == 0;
                const uint32_t a = sorted[lo], b = sorted[hi];
                if ((a > b) == up) { sorted[lo] = b; sorted[hi] = a; }
            }
            if (j == 128) __syncthreads();
            else __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();

    // row_start = exclusive scan of the occurrence counts in key order; slots get their fill cursor
    const uint64_t cap_rows = outs.cap_rows[server];
    uint32_t *out_idx = outs.indices[server];
    const uint32_t per = (U + blockDim.x - 1) / blockDim.x;
    const uint32_t u0 = min(threadIdx.x * per, U), u1 = min(u0 + per, U);
    uint32_t sum = 0;
    for (uint32_t u = u0; u < u1; ++u) sum += tval[lds_probe(tkeys, cap_mask, sorted[u], seed)];
    uint32_t n_listed;   // incoming rows with a valid key
    uint32_t run = block_exclusive_scan(sum, s_tmp, &n_listed);
    for (uint32_t u = u0; u < u1; ++u) {
        const uint32_t key = sorted[u];
        const uint32_t slot = lds_probe(tkeys, cap_mask, key, seed);
        const uint32_t c = tval[slot];
        tval[slot] = run;
        rowstart[u] = run;
        if (u < cap_rows) out_idx[u] = key;
        run += c;
    }
    if (threadIdx.x == 0) rowstart[U] = n_listed;
    __syncthreads();

    // fill the contributor lists
    for (uint32_t e = threadIdx.x; e < total_in; e += blockDim.x) {
        uint32_t lo = 0, hi = n_in;
        while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (s_pre[mid] <= e) lo = mid; else hi = mid; }
        const uint32_t i = e - s_pre[lo];
        const uint32_t key = s_idx[lo][s_begin[lo] + i];
        if (key == ZEN_EMPTY_KEY) continue;
        const uint32_t at = atomicAdd(&tval[lds_probe(tkeys, cap_mask, key, seed)], 1u);
        contrib[at] = ((uint64_t)lo << 32) | (uint64_t)(s_vbegin[lo] + i);
    }
    flags = __syncthreads_or((int)flags) ? 4u : 0u;
    if (threadIdx.x == 0) {
        *outs.count[server] = U;
        counters[CNT_UNIQUE] = U;
        counters[CNT_SKIP] = 0;
        counters[CNT_FLAGS] = flags | ((uint64_t)U > cap_rows ? 1u : 0u);
        counters[CNT_NEEDED] = (uint64_t)U > cap_rows ? U : 0u;
    }
}

// ----------------------------------------------------------------------------------------------
// Few incoming rows (<= FUSED_MAX_IN per server) of wide rows (a multiple of four floats, >= 256): merge and sums
// in ONE launch.  Every block of a server builds the server's merged (index, part, position) sequence for itself
// in LDS -- it is a few thousand integer operations, far less than a launch of its own and a round trip through
// memory cost -- and then sums its share of the output rows, one wave per row, in ascending (part, position)
// order with plain loads and one store per element.  Strictly ascending parts (what zen_encode sends), at most
// SMALL_MERGE_MAX_PARTS of them, are merged by binary searches; anything else by a bitonic sort of 64-bit
// (index, part, position) words.  Same sums in the same order as the table paths.
// Status: only block (0, 0) writes the status block (zeros and a mark in `reserved`); every server's result
// goes to its counters, which lie behind the status block, and are folded when the status is fetched.
// ----------------------------------------------------------------------------------------------
static constexpr uint32_t FUSED_MAX_IN = 2048;
static constexpr int FUSED_THREADS = 1024;

__global__ void __launch_bounds__(FUSED_THREADS)
agg_fused_kernel(PartIdx src, uint32_t n_in, uint32_t max_in_rows, uint32_t row_dim, uint32_t n_servers,
                 uint32_t *counters_base, AggOut outs, Arr64<const float *> src_values, Arr64<float *> out_values,
                 zen_status_info *status)
{
    __shared__ uint64_t s_sorted[FUSED_MAX_IN];          // the merged sequence: index << 32 | part << 26 | position in the part
    __shared__ uint32_t s_key[FUSED_MAX_IN];             // the parts' indices, part after part
    __shared__ uint32_t s_rowstart[FUSED_MAX_IN + 1];    // first element of every output row's stretch
    __shared__ uint32_t s_tmp[32];
    __shared__ uint32_t s_pre[ZEN_MAX_BATCH + 1];
    __shared__ uint32_t s_begin[ZEN_MAX_BATCH];
    __shared__ uint32_t s_vbegin[ZEN_MAX_BATCH];
    __shared__ const uint32_t *s_idx[ZEN_MAX_BATCH];
    __shared__ const float *s_src[ZEN_MAX_BATCH];
    const uint32_t server = blockIdx.y, D = row_dim;
    uint32_t *counters = counters_base + server * 16;
    if (blockIdx.x == 0 && server == 0 && threadIdx.x == 0) {
        status->flags = 0;
        status->reserved = ZEN_STATUS_IN_COUNTERS | (n_servers << 16);
        status->needed_rows = 0;
    }
    // The parts' pointers go from the kernel arguments to LDS, lane w those of part w: three loads under way at
    // once (the argument buffer lies in host memory; fetched one after the other, pointer by pointer, the
    // arguments cost this kernel 50 us).
    __shared__ const uint32_t *s_bounds[ZEN_MAX_BATCH];
    if (threadIdx.x < ZEN_MAX_BATCH) {
        s_src[threadIdx.x] = src_values.v[threadIdx.x];
        s_idx[threadIdx.x] = src.indices[threadIdx.x];
        s_bounds[threadIdx.x] = src.bounds[threadIdx.x];
    }
    __syncthreads();
    uint32_t mine = 0;
    if (threadIdx.x < n_in) {
        const uint32_t *bnd = s_bounds[threadIdx.x];
        const uint32_t vbegin = src.single ? 0u : bnd[src.server0 + server];
        mine = src.single ? bnd[0] : bnd[src.server0 + server + 1] - vbegin;
        s_begin[threadIdx.x] = vbegin;       // index lists only here: a part's indices and values start at the same row
        s_vbegin[threadIdx.x] = vbegin;
    }
    uint32_t total_in;
    const uint32_t pre = block_exclusive_scan(mine, s_tmp, &total_in);
    if (threadIdx.x < n_in) s_pre[threadIdx.x] = pre;
    if (threadIdx.x == 0) s_pre[n_in] = total_in;
    __syncthreads();
    if (total_in > max_in_rows || total_in > FUSED_MAX_IN) {       // uniform over the server's blocks
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            *outs.count[server] = 0;
            counters[CNT_UNIQUE] = 0;
            counters[CNT_SKIP] = 1;
            counters[CNT_FLAGS] = 2u;
            counters[CNT_NEEDED] = total_in;
        }
        return;
    }
    constexpr uint32_t EPT = FUSED_MAX_IN / FUSED_THREADS;         // elements per thread: 2
    uint32_t key[EPT], part[EPT];
    uint32_t bad = 0, invalid = 0;
#pragma unroll
    for (uint32_t q = 0; q < EPT; ++q) {
        const uint32_t e = q * FUSED_THREADS + threadIdx.x;
        key[q] = ZEN_EMPTY_KEY;
        part[q] = 0;
        if (e < total_in) {
            uint32_t lo = 0, hi = n_in;
            while (hi - lo > 1) { const uint32_t mid = (lo + hi) >> 1; if (s_pre[mid] <= e) lo = mid; else hi = mid; }
            part[q] = lo;
            key[q] = s_idx[lo][s_begin[lo] + (e - s_pre[lo])];
            invalid |= key[q] == ZEN_EMPTY_KEY ? 1u : 0u;
        }
        s_key[e] = key[q];
    }
    __syncthreads();
#pragma unroll
    for (uint32_t q = 0; q < EPT; ++q) {
        const uint32_t e = q * FUSED_THREADS + threadIdx.x;
        if (e < total_in && e > s_pre[part[q]]) bad |= s_key[e - 1] >= key[q] ? 1u : 0u;
    }
    invalid = __syncthreads_or((int)invalid) ? 1u : 0u;
    bad = (__syncthreads_or((int)bad) || invalid || n_in > SMALL_MERGE_MAX_PARTS) ? 1u : 0u;
    uint32_t n_listed = total_in;                                   // elements with a valid index
    if (!bad) {
        // place in the merged sequence = place in the own part + the elements of every other part before it
#pragma unroll
        for (uint32_t q = 0; q < EPT; ++q) {
            const uint32_t e = q * FUSED_THREADS + threadIdx.x;
            if (e >= total_in) continue;
            const uint32_t w = part[q], v = key[q], i = e - s_pre[w];
            uint32_t pos = i;
            for (uint32_t o = 0; o < n_in; ++o) {
                if (o == w) continue;
                uint32_t lo = s_pre[o], hi = s_pre[o + 1];
                const uint32_t limit = o < w ? v + 1u : v;          // elements < v, and an equal one if o < w
                while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (s_key[mid] < limit) lo = mid + 1; else hi = mid; }
                pos += lo - s_pre[o];
            }
            s_sorted[pos] = ((uint64_t)v << 32) | (uint64_t)((w << 26) | i);
        }
        __syncthreads();
    } else {
        // any order, duplicates, many parts: sort the (index, part, position) words; invalid indices go last
        uint32_t valid = 0;
#pragma unroll
        for (uint32_t q = 0; q < EPT; ++q) {
            const uint32_t e = q * FUSED_THREADS + threadIdx.x;
            uint64_t word = ~0ull;
            if (e < total_in && key[q] != ZEN_EMPTY_KEY) {
                word = ((uint64_t)key[q] << 32) | (uint64_t)((part[q] << 26) | (e - s_pre[part[q]]));
                ++valid;
            }
            s_sorted[e] = word;
        }
        block_exclusive_scan(valid, s_tmp, &n_listed);
        __syncthreads();
        // pairs with stride <= 64 touch one wave's own 128 elements only: no block barrier for those stages
        for (uint32_t k = 2; k <= FUSED_MAX_IN; k <<= 1) {
            for (uint32_t j = k >> 1; j > 0; j >>= 1) {
                if (j >= 128) __syncthreads();
                const uint32_t t = threadIdx.x;
                const uint32_t lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
                const bool up = (lo & k) == 0;
                const uint64_t a = s_sorted[lo], b = s_sorted[hi];
                if ((a > b) == up) { s_sorted[lo] = b; s_sorted[hi] = a; }
                if (j == 128) __syncthreads();
                else __builtin_amdgcn_wave_barrier();
            }
        }
        __syncthreads();
    }
    // heads of equal-index stretches = output rows
    const uint64_t cap_rows = outs.cap_rows[server];
    uint32_t *out_idx = outs.indices[server];
    const uint32_t a0 = min(threadIdx.x * EPT, n_listed), a1 = min(a0 + EPT, n_listed);
    uint32_t heads = 0;
    for (uint32_t a = a0; a < a1; ++a)
        heads += (a == 0 || (uint32_t)(s_sorted[a] >> 32) != (uint32_t)(s_sorted[a - 1] >> 32)) ? 1u : 0u;
    uint32_t U;
    uint32_t u = block_exclusive_scan(heads, s_tmp, &U);
    for (uint32_t a = a0; a < a1; ++a)
        if (a == 0 || (uint32_t)(s_sorted[a] >> 32) != (uint32_t)(s_sorted[a - 1] >> 32)) s_rowstart[u++] = a;
    if (threadIdx.x == 0) {
        s_rowstart[U] = n_listed;
        if (blockIdx.x == 0) {
            *outs.count[server] = U;
            counters[CNT_UNIQUE] = U;
            counters[CNT_SKIP] = 0;
            counters[CNT_FLAGS] = (invalid ? 4u : 0u) | ((uint64_t)U > cap_rows ? 1u : 0u);
            counters[CNT_NEEDED] = (uint64_t)U > cap_rows ? U : 0u;
        }
    }
    __syncthreads();
    // sums: one wave per output row
    const uint32_t rows = (uint64_t)U < cap_rows ? U : (uint32_t)cap_rows;
    const uint32_t lane = lane_id(), nw = blockDim.x >> 6, V = D >> 2;
    float *__restrict__ out = out_values.v[server];
    for (uint32_t r = blockIdx.x * nw + (threadIdx.x >> 6); r < rows; r += gridDim.x * nw) {
        const uint32_t r0 = s_rowstart[r], r1 = s_rowstart[r + 1];
        if (lane == 0) out_idx[r] = (uint32_t)(s_sorted[r0] >> 32);
        f32x4 *o4 = (f32x4 *)(out + (uint64_t)r * D);
        for (uint32_t v0 = 0; v0 < V; v0 += 64 * 4) {
            f32x4 acc[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
            for (uint32_t k = r0; k < r1; k += 2) {              // two contributors' loads under way at a time
                const uint32_t e0 = (uint32_t)s_sorted[k], w0 = e0 >> 26, i0 = e0 & 0x3FFFFFFu;
                const bool two = k + 1 < r1;
                const uint32_t e1 = two ? (uint32_t)s_sorted[k + 1] : e0, w1 = e1 >> 26, i1 = e1 & 0x3FFFFFFu;
                const f32x4 *sa = (const f32x4 *)(s_src[w0] + (uint64_t)(s_vbegin[w0] + i0) * D);
                const f32x4 *sb = (const f32x4 *)(s_src[w1] + (uint64_t)(s_vbegin[w1] + i1) * D);
                f32x4 x[4], y[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool in = v0 + 64 * q + lane < V;
                    x[q] = in ? sa[v0 + 64 * q + lane] : (f32x4){0.f, 0.f, 0.f, 0.f};
                    y[q] = (in && two) ? sb[v0 + 64 * q + lane] : (f32x4){0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += x[q];
                if (two) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[q] += y[q];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (v0 + 64 * q + lane < V) o4[v0 + 64 * q + lane] = acc[q];
        }
    }
}

// Smallest contributor id strictly greater than `prev` (ids are distinct); ~0 if none.
__device__ __forceinline__ uint64_t next_contrib(const uint64_t *list, uint32_t len, uint64_t prev, bool first)
{
    uint64_t best = ~0ull;
    for (uint32_t k = 0; k < len; ++k) {
        const uint64_t e = list[k];
        if ((first || e > prev) && e < best) best = e;
    }
    return best;
}

// A2 (values), small tables: out_values[u] = sum of the rows listed for u, in ascending (part, row)
// order.  Wide rows: one wave per output row; otherwise one thread per output element.
__global__ void __launch_bounds__(AGG_THREADS)
agg_gather_kernel(Arr64<const float *> src_values, uint32_t row_dim, uint32_t n_servers,
                  uint32_t *counters_base, const uint32_t *rowstart_base, const uint32_t *rowend_base,
                  uint64_t rowstart_stride, const uint32_t *contrib_base, uint64_t contrib_stride,
                  Arr64<float *> out_values, AggOut outs, zen_status_info *status)
{
    // rowstart / rowend: the contributor list of output row u is contrib[rowstart[u] .. rowend[u]) (a CSR array
    // serves as both, rowend = rowstart + 1); strides in u32 words; status: non-NULL when the servers' results
    // are still to be folded into the call's
    // the parts' base pointers, lane w that of part w, in LDS: indexed by a contributor's part straight from the
    // kernel arguments they would be fetched from the argument buffer in host memory, once per contributor
    __shared__ const float *s_src[ZEN_MAX_BATCH];
    if (threadIdx.x < ZEN_MAX_BATCH) s_src[threadIdx.x] = src_values.v[threadIdx.x];
    __syncthreads();
    const uint32_t server = blockIdx.y;
    const uint32_t D = row_dim;
    if (status && blockIdx.x == 0 && server == 0 && threadIdx.x == 0) {
        // status of the whole call = OR / max over the servers' own results
        uint32_t fl = 0, need = 0;
        for (uint32_t j = 0; j < n_servers; ++j) {
            fl |= counters_base[j * 16 + CNT_FLAGS];
            need = max(need, counters_base[j * 16 + CNT_NEEDED]);
        }
        status->flags = fl;
        status->reserved = 0;
        status->needed_rows = need;
    }
    const uint32_t *counters = counters_base + server * 16;
    if (counters[CNT_SKIP]) return;
    const uint32_t U = counters[CNT_UNIQUE];
    const uint64_t cap_rows = outs.cap_rows[server];
    const uint32_t rows = (uint64_t)U < cap_rows ? U : (uint32_t)cap_rows;
    const uint32_t *rowstart = rowstart_base + (uint64_t)server * rowstart_stride;
    const uint32_t *rowend = rowend_base + (uint64_t)server * rowstart_stride;
    const uint64_t *contrib = (const uint64_t *)(contrib_base + (uint64_t)server * contrib_stride);
    float *__restrict__ out = out_values.v[server];

    if ((D & 3u) == 0 && D >= 256) {
        const uint32_t lane = lane_id(), nw = blockDim.x >> 6, V = D >> 2;
        for (uint32_t u = blockIdx.x * nw + (threadIdx.x >> 6); u < rows; u += gridDim.x * nw) {
            const uint32_t r0 = rowstart[u], len = rowend[u] - r0;
            // the row's contributor list, sorted across the lanes (lists longer than a wave: see below)
            const bool in_wave = len <= ZEN_WAVE;
            uint64_t mine = ~0ull;
            uint32_t my_rank = 0xFFFFFFFFu;
            if (in_wave) {
                if (lane < len) mine = contrib[r0 + lane];
                uint32_t below = 0;
                for (uint32_t j = 0; j < len; ++j) {
                    const uint64_t cj = ((uint64_t)__shfl((uint32_t)(mine >> 32), j, ZEN_WAVE) << 32) |
                                        __shfl((uint32_t)mine, j, ZEN_WAVE);
                    below += cj < mine ? 1u : 0u;
                }
                if (lane < len) my_rank = below;
            }
            f32x4 *o4 = (f32x4 *)(out + (uint64_t)u * D);
            for (uint32_t v0 = 0; v0 < V; v0 += 64 * 4) {
                f32x4 acc[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
                uint64_t prev = 0;
                for (uint32_t k = 0; k < len; ++k) {
                    uint64_t e;
                    if (in_wave) {
                        const uint32_t srcl = (uint32_t)__ffsll((unsigned long long)ballot(my_rank == k)) - 1u;
                        e = ((uint64_t)__shfl((uint32_t)(mine >> 32), srcl, ZEN_WAVE) << 32) |
                            __shfl((uint32_t)mine, srcl, ZEN_WAVE);
                    } else {
                        e = next_contrib(contrib + r0, len, prev, k == 0);   // wave-uniform
                    }
                    prev = e;
                    const f32x4 *s4 = (const f32x4 *)(s_src[(uint32_t)(e >> 32)] + (e & 0xFFFFFFFFull) * D);
                    f32x4 x[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        x[q] = (v0 + 64 * q + lane < V) ? s4[v0 + 64 * q + lane] : (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[q] += x[q];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (v0 + 64 * q + lane < V) o4[v0 + 64 * q + lane] = acc[q];
            }
        }
    } else {
        const uint64_t n_el = (uint64_t)rows * D;
        for (uint64_t f = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; f < n_el;
             f += (uint64_t)gridDim.x * blockDim.x) {
            const uint32_t u = (uint32_t)(f / D), c = (uint32_t)(f - (uint64_t)u * D);
            const uint32_t r0 = rowstart[u], len = rowend[u] - r0;
            float acc = 0.f;
            uint64_t prev = 0;
            for (uint32_t k = 0; k < len; ++k) {
                const uint64_t e = next_contrib(contrib + r0, len, prev, k == 0);
                prev = e;
                acc += s_src[(uint32_t)(e >> 32)][(e & 0xFFFFFFFFull) * D + c];
            }
            out[f] = acc;
        }
    }
}

// The same for rows of 4..252 floats (a multiple of four): a power-of-two group of lanes per output row, 16 bytes
// per lane.  (A kernel of its own: it keeps four rows per group in registers.)
__global__ void __launch_bounds__(AGG_THREADS)
agg_gather_group_kernel(const float *const *__restrict__ src_tab, uint32_t row_dim, uint32_t n_servers,
                        uint32_t *counters_base, const uint32_t *rowstart_base, const uint32_t *rowend_base,
                        uint64_t rowstart_stride, const uint32_t *contrib_base, uint64_t contrib_stride,
                        Arr64<float *> out_values, AggOut outs, zen_status_info *status)
{
    // The parts' base pointers go from their table in memory to LDS, fetched next to the first row bounds: they
    // are then one access less in the chain row bounds -> list entry -> base pointer -> row that every output
    // row is.  (Staged from the kernel arguments instead, 64 constant-index moves per thread, it measured slower.)
    __shared__ const float *s_src[ZEN_MAX_BATCH];
    const float *my_src = threadIdx.x < ZEN_MAX_BATCH ? src_tab[threadIdx.x] : nullptr;
    const uint32_t server = blockIdx.y;
    const uint32_t D = row_dim;
    if (status && blockIdx.x == 0 && server == 0 && threadIdx.x == 0) {
        uint32_t fl = 0, need = 0;
        for (uint32_t j = 0; j < n_servers; ++j) {
            fl |= counters_base[j * 16 + CNT_FLAGS];
            need = max(need, counters_base[j * 16 + CNT_NEEDED]);
        }
        status->flags = fl;
        status->reserved = 0;
        status->needed_rows = need;
    }
    const uint32_t *counters = counters_base + server * 16;
    const uint32_t skip = counters[CNT_SKIP];
    const uint32_t U = counters[CNT_UNIQUE];
    if (threadIdx.x < ZEN_MAX_BATCH) s_src[threadIdx.x] = my_src;
    __syncthreads();
    if (skip) return;
    const uint64_t cap_rows = outs.cap_rows[server];
    const uint32_t rows = (uint64_t)U < cap_rows ? U : (uint32_t)cap_rows;
    const uint32_t *rowstart = rowstart_base + (uint64_t)server * rowstart_stride;
    const uint32_t *rowend = rowend_base + (uint64_t)server * rowstart_stride;
    const uint64_t *contrib = (const uint64_t *)(contrib_base + (uint64_t)server * contrib_stride);
    float *__restrict__ out = out_values.v[server];
    {
        // rows of 4..252 floats: a power-of-two group of lanes per output row, 16 bytes per lane
        const uint32_t V = D >> 2, lane = lane_id();
        uint32_t lanes = 1;
        while (lanes < V) lanes <<= 1;
        const uint32_t per_wave = ZEN_WAVE / lanes, sub = lane / lanes, vl = lane % lanes;
        const uint32_t wave_id = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6), n_wave = gridDim.x * (blockDim.x >> 6);
        const uint32_t g0 = sub * lanes;                 // first lane of my group
        // Four output rows per group at a time: their row bounds, then their lists, then the rows of their first
        // two contributors are fetched together -- a row is a chain of three dependent accesses, and one row at
        // a time leaves the kernel waiting on them.
        constexpr uint32_t R = GATHER_GROUP_ROWS;
        auto rank_holder = [&](uint32_t my_rank, uint32_t k, uint64_t mine) -> uint64_t {
            // the list entry of rank k, from the lane of my group that holds it (every lane of the group calls)
            const uint64_t holders = ballot(my_rank == k) >> g0;
            const uint32_t srcl = g0 + (uint32_t)__ffsll((unsigned long long)holders) - 1u;
            return ((uint64_t)__shfl((uint32_t)(mine >> 32), (int)srcl, ZEN_WAVE) << 32) |
                   __shfl((uint32_t)mine, (int)srcl, ZEN_WAVE);
        };
        auto src_vec = [&](uint64_t e) -> f32x4 {
            // the parts' value arrays come from a table in memory: lanes differ in the part they read
            return ((const f32x4 *)(s_src[(uint32_t)(e >> 32) & (ZEN_MAX_BATCH - 1)] + (e & 0xFFFFFFFFull) * D))[vl];
        };
        for (uint64_t ub = (uint64_t)wave_id * per_wave * R; ub < rows; ub += (uint64_t)n_wave * per_wave * R) {
            uint64_t u[R], mine[R];
            uint32_t r0[R], len[R], my_rank[R];
            bool on[R], held[R];
            f32x4 acc[R], x[R][2];
#pragma unroll
            for (uint32_t r = 0; r < R; ++r) {
                u[r] = ub + (uint64_t)r * per_wave + sub;
                on[r] = u[r] < rows;
                r0[r] = on[r] ? rowstart[u[r]] : 0u;
                len[r] = on[r] ? rowend[u[r]] - r0[r] : 0u;
            }
#pragma unroll
            for (uint32_t r = 0; r < R; ++r) {
                held[r] = on[r] && len[r] <= lanes;           // the list fits across the group's lanes
                mine[r] = (held[r] && vl < len[r]) ? contrib[r0[r] + vl] : ~0ull;
            }
#pragma unroll
            for (uint32_t r = 0; r < R; ++r) {
                my_rank[r] = 0;
                if (held[r]) {
                    for (uint32_t j = 0; j < len[r]; ++j) {
                        const uint64_t cj = ((uint64_t)__shfl((uint32_t)(mine[r] >> 32), (int)(g0 + j), ZEN_WAVE) << 32) |
                                            __shfl((uint32_t)mine[r], (int)(g0 + j), ZEN_WAVE);
                        my_rank[r] += cj < mine[r] ? 1u : 0u;
                    }
                    if (vl >= len[r]) my_rank[r] = 0xFFFFFFFFu;
                }
            }
#pragma unroll
            for (uint32_t r = 0; r < R; ++r)
#pragma unroll
                for (uint32_t q = 0; q < 2; ++q) {
                    x[r][q] = (f32x4){0.f, 0.f, 0.f, 0.f};
                    if (held[r] && q < len[r]) {
                        const uint64_t e = rank_holder(my_rank[r], q, mine[r]);
                        if (vl < V) x[r][q] = src_vec(e);
                    }
                }
#pragma unroll
            for (uint32_t r = 0; r < R; ++r) {
                acc[r] = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (held[r]) {
                    if (len[r] > 0) acc[r] += x[r][0];
                    if (len[r] > 1) acc[r] += x[r][1];
                    for (uint32_t k0 = 2; k0 < len[r]; k0 += 4) {   // longer lists: four rows in flight, added in order
                        f32x4 y[4];
#pragma unroll
                        for (uint32_t q = 0; q < 4; ++q) {
                            y[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
                            if (k0 + q < len[r]) {
                                const uint64_t e = rank_holder(my_rank[r], k0 + q, mine[r]);
                                if (vl < V) y[q] = src_vec(e);
                            }
                        }
#pragma unroll
                        for (uint32_t q = 0; q < 4; ++q)
                            if (k0 + q < len[r]) acc[r] += y[q];
                    }
                } else if (on[r]) {
                    uint64_t prev = 0;
                    for (uint32_t k = 0; k < len[r]; ++k) {
                        const uint64_t e = next_contrib(contrib + r0[r], len[r], prev, k == 0);
                        prev = e;
                        if (vl < V) acc[r] += src_vec(e);
                    }
                }
                if (on[r] && vl < V) ((f32x4 *)(out + u[r] * D))[vl] = acc[r];
            }
        }
    }
}

// A3, large tables, step 1: compact the occupied slots (any order) into uniq[server][0..U).
// A block first counts the occupied slots of all its iterations and moves the server's counter once
// (the counter is one address for the whole chip: one atomic per wave made this kernel atomic-bound),
// then reads its slots again (they are in the L2) and hands out positions through an LDS counter.
__global__ void __launch_bounds__(AGG_THREADS)
agg_compact_kernel(const uint32_t *keys_base, uint64_t table_cap, uint32_t *uniq_base, uint64_t uniq_stride,
                   uint32_t *counters_base)
{
    __shared__ uint32_t s_total, s_base, s_cur;
    const uint32_t server = blockIdx.y;
    const uint32_t *keys = keys_base + (uint64_t)server * table_cap;
    uint32_t *uniq = uniq_base + (uint64_t)server * uniq_stride;
    uint32_t *counters = counters_base + server * 16;
    if (counters[CNT_SKIP]) return;
    if (threadIdx.x == 0) { s_total = 0; s_cur = 0; }
    __syncthreads();
    // table_cap is a multiple of the block size: every wave runs the same number of iterations
    uint32_t mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < table_cap;
         i += (uint64_t)gridDim.x * blockDim.x)
        mine += (uint32_t)__popcll(ballot(keys[i] != ZEN_EMPTY_KEY));   // the same in every lane of the wave
    if (lane_id() == 0 && mine) atomicAdd(&s_total, mine);
    __syncthreads();
    if (threadIdx.x == 0) s_base = s_total ? atomicAdd(&counters[CNT_UNIQUE], s_total) : 0u;
    __syncthreads();
    if (s_total == 0) return;
    const uint32_t block_base = s_base;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < table_cap;
         i += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t k = keys[i];
        const bool occ = k != ZEN_EMPTY_KEY;
        const uint64_t m = ballot(occ);
        uint32_t base = 0;
        if (lane_id() == 0 && m) base = atomicAdd(&s_cur, (uint32_t)__popcll(m));
        base = __shfl(base, 0, ZEN_WAVE);
        if (occ) uniq[block_base + base + mbcnt(m)] = k;
    }
}

// Segmented LSB radix sort, one 8-bit digit per pass.  Segment = server, length = counters[UNIQUE].
__global__ void __launch_bounds__(AGG_THREADS)
rs_hist_kernel(const uint32_t *in_base, uint64_t uniq_stride, const uint32_t *counters_base, uint32_t shift,
               uint32_t *hist_base, uint64_t hist_stride)
{
    __shared__ uint32_t s_h[256];
    const uint32_t server = blockIdx.y;
    const uint32_t U = counters_base[server * 16 + CNT_UNIQUE];
    const uint32_t n_blocks = (U + RS_BLOCK_KEYS - 1) / RS_BLOCK_KEYS;
    uint32_t *hist = hist_base + (uint64_t)server * hist_stride + (uint64_t)blockIdx.x * 256;
    if (blockIdx.x >= n_blocks) return;   // the scan only reads blocks < n_blocks
    const uint32_t *in = in_base + (uint64_t)server * uniq_stride;
    s_h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t k0 = blockIdx.x * RS_BLOCK_KEYS;
#pragma unroll
    for (int it = 0; it < RS_ITEMS; ++it) {
        const uint32_t i = k0 + it * AGG_THREADS + threadIdx.x;
        if (i < U) atomicAdd(&s_h[(in[i] >> shift) & 255u], 1u);
    }
    __syncthreads();
    hist[threadIdx.x] = s_h[threadIdx.x];
}

// hist[block][digit] -> output position of the first key of (block, digit); one block per server.
__global__ void __launch_bounds__(1024)
rs_scan_kernel(const uint32_t *counters_base, uint32_t *hist_base, uint64_t hist_stride)
{
    __shared__ uint32_t s_part[1024];
    __shared__ uint32_t s_off[257];
    const uint32_t server = blockIdx.x;
    const uint32_t U = counters_base[server * 16 + CNT_UNIQUE];
    const uint32_t n_blocks = (U + RS_BLOCK_KEYS - 1) / RS_BLOCK_KEYS;
    uint32_t *hist = hist_base + (uint64_t)server * hist_stride;
    const uint32_t d = threadIdx.x & 255u, grp = threadIdx.x >> 8;   // 4 groups x 256 digits
    const uint32_t per = (n_blocks + 3) / 4;
    const uint32_t b0 = min(grp * per, n_blocks), b1 = min(b0 + per, n_blocks);
    uint32_t sum = 0;
    for (uint32_t b = b0; b < b1; ++b) sum += hist[(uint64_t)b * 256 + d];
    s_part[grp * 256 + d] = sum;
    __syncthreads();
    if (threadIdx.x < 256) {
        uint32_t run = 0;
        for (uint32_t gI = 0; gI < 4; ++gI) {
            const uint32_t t = s_part[gI * 256 + threadIdx.x];
            s_part[gI * 256 + threadIdx.x] = run;
            run += t;
        }
        s_off[threadIdx.x + 1] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        s_off[0] = 0;
        uint32_t run = 0;
        for (uint32_t q = 0; q < 256; ++q) { run += s_off[q + 1]; s_off[q + 1] = run; }
    }
    __syncthreads();
    uint32_t run = s_off[d] + s_part[grp * 256 + d];
    for (uint32_t b = b0; b < b1; ++b) {
        const uint64_t a = (uint64_t)b * 256 + d;
        const uint32_t h = hist[a];
        hist[a] = run;
        run += h;
    }
}

__global__ void __launch_bounds__(AGG_THREADS)
rs_scatter_kernel(const uint32_t *in_base, uint32_t *out_base, uint64_t uniq_stride,
                  const uint32_t *counters_base, uint32_t shift, const uint32_t *hist_base, uint64_t hist_stride)
{
    __shared__ uint32_t s_run[256];
    __shared__ uint32_t s_cnt[4 * 256];
    const uint32_t server = blockIdx.y;
    const uint32_t U = counters_base[server * 16 + CNT_UNIQUE];
    const uint32_t n_blocks = (U + RS_BLOCK_KEYS - 1) / RS_BLOCK_KEYS;
    if (blockIdx.x >= n_blocks) return;
    const uint32_t *in = in_base + (uint64_t)server * uniq_stride;
    uint32_t *out = out_base + (uint64_t)server * uniq_stride;
    const uint32_t *hist = hist_base + (uint64_t)server * hist_stride + (uint64_t)blockIdx.x * 256;
    s_run[threadIdx.x] = hist[threadIdx.x];
    for (uint32_t i = threadIdx.x; i < 4 * 256; i += blockDim.x) s_cnt[i] = 0;
    __syncthreads();
    const uint32_t k0 = blockIdx.x * RS_BLOCK_KEYS;
    for (int it = 0; it < RS_ITEMS; ++it) {
        const uint32_t i = k0 + it * AGG_THREADS + threadIdx.x;
        const bool valid = i < U;
        const uint32_t key = valid ? in[i] : 0u;
        const uint32_t pos = block_stable_rank(valid, (key >> shift) & 255u, 8, 256, s_run, s_cnt);
        if (valid) out[pos] = key;
    }
}

// One radix pass in ONE launch, for servers with few blocks of keys (<= RS_FUSED_MAX_BLOCKS): every block counts the
// digits of all of the server's keys itself (a hundred KB out of the L2) -- the totals per digit and, of the keys
// before its own, the counts per digit -- which is all that the histogram, scan and scatter launches passed
// between them, and then ranks and writes its own keys.  Three launches per sort instead of nine; the launches,
// not the keys, were what the sort of a few ten thousand keys cost.
static constexpr uint32_t RS_FUSED_MAX_BLOCKS = 32;

__global__ void __launch_bounds__(AGG_THREADS)
rs_pass_kernel(const uint32_t *in_base, uint32_t *out_base, uint64_t uniq_stride, const uint32_t *counters_base,
               uint32_t shift)
{
    __shared__ uint32_t s_tot[256];       // keys of the server per digit
    __shared__ uint32_t s_run[256];       // first the keys before this block's per digit, then running output positions
    __shared__ uint32_t s_cnt[4 * 256];
    __shared__ uint32_t s_tmp[32];
    const uint32_t server = blockIdx.y;
    const uint32_t U = counters_base[server * 16 + CNT_UNIQUE];
    const uint32_t n_blocks = (U + RS_BLOCK_KEYS - 1) / RS_BLOCK_KEYS;
    if (blockIdx.x >= n_blocks) return;
    const uint32_t *in = in_base + (uint64_t)server * uniq_stride;
    uint32_t *out = out_base + (uint64_t)server * uniq_stride;
    s_tot[threadIdx.x] = 0;
    s_run[threadIdx.x] = 0;
    for (uint32_t i = threadIdx.x; i < 4 * 256; i += blockDim.x) s_cnt[i] = 0;
    __syncthreads();
    const uint32_t k0 = blockIdx.x * RS_BLOCK_KEYS;
    constexpr uint32_t RD = 24;           // loads under way per thread: the count is a chain of round trips otherwise
    for (uint32_t i0 = 0; i0 < U; i0 += RD * AGG_THREADS) {
        uint32_t key[RD];
#pragma unroll
        for (uint32_t u = 0; u < RD; ++u) {
            const uint32_t i = i0 + u * AGG_THREADS + threadIdx.x;
            key[u] = i < U ? in[i] : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < RD; ++u) {
            const uint32_t i = i0 + u * AGG_THREADS + threadIdx.x;
            if (i < U) {
                const uint32_t d = (key[u] >> shift) & 255u;
                atomicAdd(&s_tot[d], 1u);
                if (i < k0) atomicAdd(&s_run[d], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t total;
    const uint32_t first = block_exclusive_scan(s_tot[threadIdx.x], s_tmp, &total);   // keys with a smaller digit
    s_run[threadIdx.x] += first;
    __syncthreads();
    for (int it = 0; it < RS_ITEMS; ++it) {
        const uint32_t i = k0 + it * AGG_THREADS + threadIdx.x;
        const bool valid = i < U;
        const uint32_t key = valid ? in[i] : 0u;
        const uint32_t pos = block_stable_rank(valid, (key >> shift) & 255u, 8, 256, s_run, s_cnt);
        if (valid) out[pos] = key;
    }
}

// A3, large tables, last step: sorted unique keys -> out_indices, *count, and each key's rank.
__global__ void __launch_bounds__(AGG_THREADS)
agg_finalize_kernel(uint32_t seed, const uint32_t *sorted_base, uint64_t uniq_stride, const uint32_t *keys_base,
                    uint32_t *rank_base, uint64_t table_cap, const uint32_t *counters_base, AggOut outs,
                    uint32_t *rowstart_base, uint32_t *cursor_base, uint64_t row_stride, uint32_t *counters_rw,
                    Arr64<const float *> src_values, const float **src_tab, zen_status_info *status)
{
    // rowstart / cursor: where the contributor list of every output row starts (the fill kernel moves the cursor
    // to the list's end).  A wave takes the room for its 64 rows' lists with one atomic; the lists lie in no
    // particular order, which shows in no result.
    if (src_tab && blockIdx.x == 0 && blockIdx.y == 0) write_src_table(src_values, src_tab);   // for the gather of narrow rows
    const uint32_t server = blockIdx.y;
    const uint32_t *counters = counters_base + server * 16;
    const uint32_t U = counters[CNT_SKIP] ? 0u : counters[CNT_UNIQUE];
    const uint32_t *sorted = sorted_base + (uint64_t)server * uniq_stride;
    const uint32_t *keys = keys_base + (uint64_t)server * table_cap;
    uint32_t *rank = rank_base + (uint64_t)server * table_cap;
    uint32_t *rowstart = rowstart_base + (uint64_t)server * row_stride, *cursor = cursor_base + (uint64_t)server * row_stride;
    const uint32_t cap_mask = (uint32_t)(table_cap - 1);
    const uint64_t cap_rows = outs.cap_rows[server];
    uint32_t *out_idx = outs.indices[server];
    for (uint32_t u0 = blockIdx.x * blockDim.x; u0 < U; u0 += gridDim.x * blockDim.x) {   // whole waves together
        const uint32_t u = u0 + threadIdx.x;
        uint32_t c = 0;
        if (u < U) {
            const uint32_t key = sorted[u];
            if (u < cap_rows) out_idx[u] = key;
            const uint32_t slot = probe_find(keys, cap_mask, key, seed);
            if (slot != 0xFFFFFFFFu) { c = rank[slot] + 1u; rank[slot] = u; }   // the slot counted the key's repeats so far
        }
        const uint32_t inc = wave_inclusive_scan(c);
        uint32_t base = 0;
        if (lane_id() == ZEN_WAVE - 1) base = atomicAdd(&counters_rw[server * 16 + CNT_LISTED], inc);
        base = __shfl(base, ZEN_WAVE - 1, ZEN_WAVE);
        if (u < U) { rowstart[u] = base + inc - c; cursor[u] = base + inc - c; }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *outs.count[server] = U;
        if ((uint64_t)U > cap_rows) {
            atomicOr(&status->flags, 1u);
            atomicMax((unsigned long long *)&status->needed_rows, (unsigned long long)U);
        }
    }
}

// A2 (values), large tables: every incoming row appends its id (part << 32 | row in the part's values) to the
// contributor list of its key's output row.  agg_gather_kernel then sums every output row from its list in
// ascending (part, row) order: no value atomics, no zero fill, reproducible bit for bit.
__global__ void __launch_bounds__(AGG_THREADS)
agg_fill_kernel(PartIdx src, uint32_t seed, const uint32_t *keys_base, const uint32_t *rank_base, uint64_t table_cap,
                const uint32_t *counters_base, uint32_t *cursor_base, uint64_t cursor_stride, uint64_t *contrib_base,
                uint64_t contrib_stride)
{
    const uint32_t server = blockIdx.z, w = blockIdx.y;
    const uint32_t *counters = counters_base + server * 16;
    if (counters[CNT_SKIP]) return;
    const uint32_t *__restrict__ keys = keys_base + (uint64_t)server * table_cap;
    const uint32_t *__restrict__ rank = rank_base + (uint64_t)server * table_cap;
    uint32_t *cursor = cursor_base + (uint64_t)server * cursor_stride;
    uint64_t *contrib = contrib_base + (uint64_t)server * contrib_stride;
    const uint32_t cap_mask = (uint32_t)(table_cap - 1);
    const PartRange r = part_range(src, w, server);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < r.count; i += gridDim.x * blockDim.x) {
        const uint32_t key = r.idx[r.begin + i];
        const uint32_t slot = probe_find(keys, cap_mask, key, seed);
        if (slot == 0xFFFFFFFFu) continue;                      // the reserved key: flagged by the insert
        const uint32_t at = atomicAdd(&cursor[rank[slot]], 1u);
        contrib[at] = ((uint64_t)w << 32) | (uint64_t)(r.vbegin + i);
    }
}

// ----------------------------------------------------------------------------------------------
// layout + launcher
// ----------------------------------------------------------------------------------------------
static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

AggLayout aggregate_layout(const zen_ctx *ctx, uint32_t batch, uint64_t max_in_rows)
{
    const bool decode = ctx->fmt == ZEN_INDEX_BITMAP;
    AggLayout L{};
    uint64_t cap = 1024;
    while (cap < 2 * max_in_rows) cap <<= 1;
    L.table_cap = cap;
    L.small_path = max_in_rows <= SMALL_MAX_IN ? 1u : 0u;
    uint64_t off = 0;
    L.status_off = off; off += 256;
    L.counters_off = off; off += align_up((uint64_t)batch * 16 * 4, 256);
    L.srctab_off = off; off += ZEN_MAX_BATCH * 8;   // the parts' value arrays, for kernels whose lanes differ in the part they read
    L.keys_off = off; off += align_up((uint64_t)batch * cap * 4, 256);
    L.rank_off = off; off += align_up((uint64_t)batch * cap * 4, 256);
    L.uniq_cap = align_up(max_in_rows > 0 ? max_in_rows : 1, 64);
    L.sort_blocks = (L.uniq_cap + RS_BLOCK_KEYS - 1) / RS_BLOCK_KEYS;
    if (!L.small_path) {
        L.uniq_off = off; off += align_up((uint64_t)batch * 2 * L.uniq_cap * 4, 256);
        L.sorthist_off = off; off += align_up((uint64_t)batch * L.sort_blocks * 256 * 4, 256);
        L.rowstart_stride = L.uniq_cap + 64;
        L.rowstart_off = off; off += align_up((uint64_t)batch * 2 * L.rowstart_stride * 4, 256);   // row starts + fill cursors
    }
    L.decode_off = off;
    L.decode_stride = 0;
    if (decode) {
        L.decode_stride = L.uniq_cap;
        off += align_up((uint64_t)batch * L.decode_stride * 4, 256);
        L.decflags_off = off; off += align_up((uint64_t)batch * ZEN_MAX_BATCH * 4, 256);
        L.bm_chunks = bitmap_merge_chunks(ctx->max_dom_words);
        L.bmcnt_off = off; off += align_up((uint64_t)batch * (ZEN_MAX_BATCH + 1) * L.bm_chunks * 4, 256);
        if (ctx->geo.row_dim == 1) {   // element-level merges: per-wave counts of every chunk, the parts' pointer tables
            L.bmwave_off = off; off += align_up((uint64_t)batch * L.bm_chunks * (ZEN_MAX_BATCH + 1) * 4 * 4, 256);
            L.bmtab_off = off; off += align_up(2 * ZEN_MAX_BATCH * 8, 256);
        }
    }
    L.total = off;
    return L;
}

// Blocks per server for the gather kernels: enough for max_in_rows output rows in one sweep, no more (a block
// without a row still waits for the server's counters before it can leave).
static uint32_t gather_grid_x(uint32_t row_dim, uint64_t max_in_rows)
{
    uint64_t gx;
    if ((row_dim & 3u) == 0 && row_dim >= 256) {
        gx = (max_in_rows + 3) / 4;                                   // a wave per row
    } else if ((row_dim & 3u) == 0) {
        uint32_t lanes = 1;
        while (lanes < (row_dim >> 2)) lanes <<= 1;
        const uint64_t rows_per_block = (uint64_t)(AGG_THREADS / lanes) * GATHER_GROUP_ROWS;   // groups x rows per group
        gx = (max_in_rows + rows_per_block - 1) / rows_per_block;
    } else {
        gx = (max_in_rows * row_dim + AGG_THREADS - 1) / AGG_THREADS;
    }
    if (gx < 1) gx = 1;
    if (gx > 8192) gx = 8192;
    return (uint32_t)gx;
}

#define ZEN_LAUNCH_CHECK()                         \
    do {                                           \
        hipError_t e_ = hipGetLastError();         \
        if (e_ != hipSuccess) return e_;           \
    } while (0)

hipError_t launch_aggregate(zen_ctx *ctx, const PartIdx &src,
                            const Arr64<const float *> &src_values, const Arr64<const uint32_t *> &src_bitmap,
                            uint32_t n_in, uint32_t n_servers, uint32_t first_part_id, const AggOut &outs,
                            const Arr64<float *> &out_values, uint64_t max_in_rows, char *ws,
                            const AggLayout &L, hipStream_t s)
{
    const Geometry &g = ctx->geo;
    zen_status_info *status = (zen_status_info *)(ws + L.status_off);
    uint32_t *counters = (uint32_t *)(ws + L.counters_off);
    uint32_t *keys = (uint32_t *)(ws + L.keys_off);
    uint32_t *rank = (uint32_t *)(ws + L.rank_off);
    const uint64_t cap = L.table_cap;
    const uint64_t n_keys = (uint64_t)n_servers * cap;
    const bool narrow_rows = (g.row_dim & 3u) == 0 && g.row_dim < 256;   // summed by agg_gather_group_kernel

    bool any_bitmap = false;
    for (uint32_t w = 0; w < n_in; ++w) any_bitmap |= (src.indices[w] == nullptr);
    if (any_bitmap && (!ctx->d_domain || !L.decode_stride)) return hipErrorInvalidValue;
    bool all_bitmap = n_in > 0;
    for (uint32_t w = 0; w < n_in; ++w) all_bitmap &= (src.indices[w] == nullptr && src_bitmap.v[w] != nullptr);
    if (all_bitmap) {
        // every part is a hash bitmap: merge in the bitmaps' own domain (OR + popcount ranks)
        Arr64<const uint32_t *> bounds;
        for (uint32_t w = 0; w < ZEN_MAX_BATCH; ++w) bounds.v[w] = src.bounds[w];
        return launch_bitmap_merge(ctx, src_bitmap, bounds, src_values, n_in, src.single != 0, n_servers,
                                   first_part_id, outs, out_values, ws, L, s);
    }

    if (L.small_path && !any_bitmap && (g.row_dim & 3u) == 0 && g.row_dim >= 256 && max_in_rows <= FUSED_MAX_IN) {
        // few rows of wide rows: merge and sums in one launch
#ifndef ZEN_FUSED_BLOCKS
#define ZEN_FUSED_BLOCKS 256   // about one block per CU: 64 / 128 / 256 / 512 measured 37 / 33 / 31 / 46 us on the LM workload
#endif
        uint32_t bx = ZEN_FUSED_BLOCKS / n_servers;
        if (bx < 1) bx = 1;
        if (bx > 64) bx = 64;
        ProfScope prof(ctx, K_AGG_SORT_SMALL, s);
        agg_fused_kernel<<<dim3(bx, n_servers), FUSED_THREADS, 0, s>>>(src, n_in, (uint32_t)max_in_rows, g.row_dim, n_servers,
                                                                       counters, outs, src_values, out_values, status);
        return hipGetLastError();
    }
    if (L.small_path) {
        uint32_t *dec_flags = any_bitmap ? (uint32_t *)(ws + L.decflags_off) : nullptr;
        if (any_bitmap) {
            ProfScope prof(ctx, K_BITMAP_DECODE, s);
            bitmap_decode_kernel<<<dim3(n_in, n_servers), 1024, 0, s>>>(
                src, src_bitmap, first_part_id, ctx->d_domain, ctx->d_dom_offsets, ctx->d_bm_word_off,
                (uint32_t *)(ws + L.decode_off), L.decode_stride, status, dec_flags);
            ZEN_LAUNCH_CHECK();
        }
        uint32_t lcap = 1024, sortp = 1;
        while ((uint64_t)lcap * 4 < max_in_rows * 5) lcap <<= 1;   // load <= 0.8
        while (sortp < max_in_rows) sortp <<= 1;
        const size_t lds = ((size_t)2 * lcap + sortp) * 4;
        static bool lds_attr_set = false;
        if (!lds_attr_set) {
            (void)hipFuncSetAttribute((const void *)agg_small_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (2 * 8192 + 8192) * 4);
            (void)hipGetLastError();
            lds_attr_set = true;
        }
        {
            ProfScope prof(ctx, K_AGG_SORT_SMALL, s);
            agg_small_kernel<<<n_servers, SMALL_THREADS, lds, s>>>(src, n_in, g.seed, lcap, (uint32_t)max_in_rows,
                                                                   counters, outs, keys, rank, cap, dec_flags, src_values,
                                                                   narrow_rows ? (const float **)(ws + L.srctab_off) : nullptr);
            ZEN_LAUNCH_CHECK();
        }
        {
            const uint32_t gx = gather_grid_x(g.row_dim, max_in_rows);
            ProfScope prof(ctx, K_AGG_GATHER, s);
            if (narrow_rows)
                agg_gather_group_kernel<<<dim3((uint32_t)gx, n_servers), AGG_THREADS, 0, s>>>(
                    (const float *const *)(ws + L.srctab_off), g.row_dim, n_servers, counters, keys, keys + 1, cap, rank, cap, out_values, outs, status);
            else
                agg_gather_kernel<<<dim3((uint32_t)gx, n_servers), AGG_THREADS, 0, s>>>(
                    src_values, g.row_dim, n_servers, counters, keys, keys + 1, cap, rank, cap, out_values, outs, status);
            ZEN_LAUNCH_CHECK();
        }
        return hipSuccess;
    }

    {
        uint64_t blocks = (n_keys + 1023) / 1024;
        if (blocks > 16384) blocks = 16384;
        {
            ProfScope prof(ctx, K_AGG_CLEAR, s);
            agg_clear_kernel<<<(uint32_t)blocks, 256, 0, s>>>(keys, rank, n_keys, counters, n_servers * 16, status);
            ZEN_LAUNCH_CHECK();
        }
    }
    if (any_bitmap) {
        ProfScope prof(ctx, K_BITMAP_DECODE, s);
        bitmap_decode_kernel<<<dim3(n_in, n_servers), 1024, 0, s>>>(
            src, src_bitmap, first_part_id, ctx->d_domain, ctx->d_dom_offsets, ctx->d_bm_word_off,
            (uint32_t *)(ws + L.decode_off), L.decode_stride, status, nullptr);
        ZEN_LAUNCH_CHECK();
    }
    // rows per (part, server) are unknown on the host; size the x dimension for an even split of
    // max_in_rows over the parts, grid-stride loops cover any skew
    uint64_t per_part = (max_in_rows + n_in - 1) / (n_in ? n_in : 1);
    uint32_t gx = (uint32_t)((per_part + AGG_THREADS - 1) / AGG_THREADS);
    if (gx < 1) gx = 1;
    if (gx > 4096) gx = 4096;
    {
        ProfScope prof(ctx, K_AGG_INSERT, s);
        agg_insert_kernel<<<dim3(gx, n_in, n_servers), AGG_THREADS, 0, s>>>(src, n_in, g.seed, keys, rank, cap, counters,
                                                                            max_in_rows, status);
        ZEN_LAUNCH_CHECK();
    }

    {
        uint32_t *uniq = (uint32_t *)(ws + L.uniq_off);
        uint32_t *hist = (uint32_t *)(ws + L.sorthist_off);
        const uint64_t ustride = 2 * L.uniq_cap, hstride = L.sort_blocks * 256;
        uint64_t cblocks = cap / AGG_THREADS / 8;   // eight iterations per block, one global atomic per block
        if (cblocks < 1) cblocks = 1;
        if (cblocks > 2048) cblocks = 2048;
        {
            ProfScope prof(ctx, K_AGG_COMPACT, s);
            agg_compact_kernel<<<dim3((uint32_t)cblocks, n_servers), AGG_THREADS, 0, s>>>(keys, cap, uniq, ustride,
                                                                                         counters);
            ZEN_LAUNCH_CHECK();
        }
        uint32_t key_bits = 1;
        while (key_bits < 32 && (1ull << key_bits) < g.n_rows) ++key_bits;
        uint32_t *a = uniq, *b = uniq + L.uniq_cap;
        for (uint32_t shift = 0; shift < key_bits; shift += 8) {
            if (L.sort_blocks <= RS_FUSED_MAX_BLOCKS) {
                ProfScope prof(ctx, K_RS_SCATTER, s);
                rs_pass_kernel<<<dim3((uint32_t)L.sort_blocks, n_servers), AGG_THREADS, 0, s>>>(a, b, ustride, counters, shift);
                ZEN_LAUNCH_CHECK();
                uint32_t *t = a; a = b; b = t;
                continue;
            }
            {
                ProfScope prof(ctx, K_RS_HIST, s);
                rs_hist_kernel<<<dim3((uint32_t)L.sort_blocks, n_servers), AGG_THREADS, 0, s>>>(a, ustride, counters, shift,
                                                                                              hist, hstride);
                ZEN_LAUNCH_CHECK();
            }
            {
                ProfScope prof(ctx, K_RS_SCAN, s);
                rs_scan_kernel<<<n_servers, 1024, 0, s>>>(counters, hist, hstride);
                ZEN_LAUNCH_CHECK();
            }
            {
                ProfScope prof(ctx, K_RS_SCATTER, s);
                rs_scatter_kernel<<<dim3((uint32_t)L.sort_blocks, n_servers), AGG_THREADS, 0, s>>>(
                    a, b, ustride, counters, shift, hist, hstride);
                ZEN_LAUNCH_CHECK();
            }
            uint32_t *t = a; a = b; b = t;
        }
        uint64_t fblocks = (L.uniq_cap + AGG_THREADS - 1) / AGG_THREADS;
        if (fblocks > 4096) fblocks = 4096;
        {
            ProfScope prof(ctx, K_AGG_FINALIZE, s);
            uint32_t *rs = (uint32_t *)(ws + L.rowstart_off);
            agg_finalize_kernel<<<dim3((uint32_t)fblocks, n_servers), AGG_THREADS, 0, s>>>(
                g.seed, a, ustride, keys, rank, cap, counters, outs, rs, rs + (uint64_t)n_servers * L.rowstart_stride,
                L.rowstart_stride, counters, src_values, narrow_rows ? (const float **)(ws + L.srctab_off) : nullptr, status);
            ZEN_LAUNCH_CHECK();
        }
    }
    {
        // contributor lists (in the sort's ping-pong buffers, free by now; cursor[u] ends at the end of row u's list), gather
        uint32_t *rowstart = (uint32_t *)(ws + L.rowstart_off), *cursor = rowstart + (uint64_t)n_servers * L.rowstart_stride;
        uint64_t *contrib = (uint64_t *)(ws + L.uniq_off);
        {
            ProfScope prof(ctx, K_AGG_FILL, s);
            agg_fill_kernel<<<dim3(gx, n_in, n_servers), AGG_THREADS, 0, s>>>(src, g.seed, keys, rank, cap, counters, cursor,
                                                                              L.rowstart_stride, contrib, L.uniq_cap);
            ZEN_LAUNCH_CHECK();
        }
        const uint32_t ggx = gather_grid_x(g.row_dim, max_in_rows);
        ProfScope prof(ctx, K_AGG_GATHER, s);
        if (narrow_rows)
            agg_gather_group_kernel<<<dim3((uint32_t)ggx, n_servers), AGG_THREADS, 0, s>>>(
                (const float *const *)(ws + L.srctab_off), g.row_dim, n_servers, counters, rowstart, cursor, L.rowstart_stride,
                (const uint32_t *)contrib, 2 * L.uniq_cap, out_values, outs, nullptr);
        else
            agg_gather_kernel<<<dim3((uint32_t)ggx, n_servers), AGG_THREADS, 0, s>>>(
                src_values, g.row_dim, n_servers, counters, rowstart, cursor, L.rowstart_stride, (const uint32_t *)contrib,
                2 * L.uniq_cap, out_values, outs, nullptr);
        return hipGetLastError();
    }

}

} // namespace zen
