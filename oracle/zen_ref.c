/*
 * zen_ref.c -- CPU oracle for the sparse-gradient encode + aggregate path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * definition of what the GPU library must compute.  It shares no code, header,
 * table or constant generator with the HIP sources, and only the test-suite,
 * the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Every function states the passage of the paper (arXiv 2309.13254, "Zen")
 * it follows.  The paper's hierarchical hashing (Algorithm 1) is lossless: its
 * output is, for each partition, exactly the set of non-zero indices owned by
 * that partition together with their values (Algorithm 1, output loop; section
 * "Data-independent Hierarchical Hashing", paragraph "Negligible extraction
 * overhead").  The oracle is therefore that plain definition written out, not
 * the hash-memory mechanism.
 *
 * Readings taken where the paper is silent (each is pinned by a CPU test):
 *   - indices are 0-based row ids (the paper counts from 1);
 *   - a row is "non-zero" iff any of its D fp32 words has a non-zero magnitude
 *     field, i.e. (bits & 0x7fffffff) != 0, so +0 and -0 are zero while NaN,
 *     Inf and denormals are non-zero;
 *   - inside a partition indices ascend (the paper leaves the order free
 *     because it does not change the aggregate);
 *   - h0(idx) = MurmurHash3_x86_32(4-byte little-endian idx, seed) mod n
 *     (section "Implementation" names MurmurHash with seeds, nothing more);
 *   - hash bitmap: bit j of partition p tells whether the j-th smallest row of
 *     the partition's domain is non-zero; bits are packed LSB-first into
 *     32-bit words and every partition starts on a word boundary;
 *   - aggregation sums every occurrence of an index in fp64, in input order,
 *     and keeps an index even when its sum is exactly zero;
 *   - the hash bitmap a server builds for Pull marks membership in its
 *     aggregated index set (not "value != 0"), so values and set bits stay
 *     paired one to one.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py
 * (published MurmurHash3 vectors and an independent library implementation,
 * the paper's worked hash-bitmap example, closed forms, brute force).  The
 * one thing that cannot be pinned is that h0 equals the hash the paper's own
 * (unpublished) code used: "parity unpinned" for the paper's hash outputs.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ZEN_REF_OK 0
#define ZEN_REF_ERR_INVALID 1
#define ZEN_REF_ERR_CAPACITY 2
#define ZEN_REF_ERR_NOMEM 3

static uint32_t rotl32(uint32_t x, int r) { return (x << r) | (x >> (32 - r)); }

/*
 * MurmurHash3, x86 32-bit variant, of one 4-byte key (the index stored little
 * endian) -- the hash family section "Implementation" names.  One body block,
 * no tail, length 4, then the finaliser.
 */
uint32_t zen_ref_hash(uint32_t idx, uint32_t seed)
{
    uint32_t k = idx;
    uint32_t h = seed;
    k *= 0xcc9e2d51u;
    k = rotl32(k, 15);
    k *= 0x1b873593u;
    h ^= k;
    h = rotl32(h, 13);
    h = h * 5u + 0xe6546b64u;
    h ^= 4u; /* key length in bytes */
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}

void zen_ref_hash_many(const uint32_t *idx, uint64_t count, uint32_t seed, uint32_t *out)
{
    for (uint64_t i = 0; i < count; ++i) out[i] = zen_ref_hash(idx[i], seed);
}

/* h0 : index -> [n]  (Algorithm 1, "p <- h0(idx)"). */
uint32_t zen_ref_owner(uint32_t idx, uint32_t seed, uint32_t n)
{
    return zen_ref_hash(idx, seed) % n;
}

/* owner[r] = h0(r) for every row of the dense tensor; n <= 65535. */
int zen_ref_owner_table(uint64_t n_rows, uint32_t n, uint32_t seed, uint16_t *owner)
{
    if (n == 0 || n > 65535u || n_rows > 0xfffffffeull) return ZEN_REF_ERR_INVALID;
    for (uint64_t r = 0; r < n_rows; ++r) owner[r] = (uint16_t)zen_ref_owner((uint32_t)r, seed, n);
    return ZEN_REF_OK;
}

/*
 * I = ascending indices of the non-zero rows of G (Algorithm 1, input "I is the
 * indices of its non-zero gradients").  Returns |I|; `I` may be NULL to count.
 */
int64_t zen_ref_nonzero(const float *grad, uint64_t n_rows, uint32_t row_dim, uint32_t *I)
{
    int64_t nnz = 0;
    for (uint64_t r = 0; r < n_rows; ++r) {
        const float *row = grad + r * (uint64_t)row_dim;
        int nz = 0;
        for (uint32_t c = 0; c < row_dim; ++c) {
            uint32_t bits;
            memcpy(&bits, &row[c], 4);
            if ((bits & 0x7fffffffu) != 0) { nz = 1; break; }
        }
        if (nz) {
            if (I) I[nnz] = (uint32_t)r;
            ++nnz;
        }
    }
    return nnz;
}

/*
 * Partition an ascending index list by owner (Algorithm 1: every idx goes to
 * partition h0(idx); output loop: one (indices, values) pair per partition).
 * `owner_of_I[k]` is the owner of I[k].  offsets has n+1 entries.
 */
int zen_ref_partition(const uint32_t *I, const uint16_t *owner_of_I, uint64_t nnz, uint32_t n,
                      uint32_t *offsets, uint32_t *indices)
{
    if (n == 0) return ZEN_REF_ERR_INVALID;
    uint64_t pos = 0;
    offsets[0] = 0;
    for (uint32_t p = 0; p < n; ++p) {
        for (uint64_t k = 0; k < nnz; ++k)
            if (owner_of_I[k] == p) indices[pos++] = I[k];
        offsets[p + 1] = (uint32_t)pos;
    }
    return pos == nnz ? ZEN_REF_OK : ZEN_REF_ERR_INVALID; /* an owner >= n would lose an index */
}

/* values = G[indices] (Algorithm 1, output loop), whole rows, bit-exact. */
void zen_ref_gather(const float *grad, uint32_t row_dim, const uint32_t *indices, uint64_t count,
                    float *values)
{
    for (uint64_t k = 0; k < count; ++k)
        memcpy(values + k * (uint64_t)row_dim, grad + (uint64_t)indices[k] * row_dim,
               (size_t)row_dim * 4);
}

/*
 * The whole encode of one worker's gradient: non-zero rows -> owner by h0 ->
 * per-partition ascending indices and their rows, concatenated partition-major
 * with an exclusive prefix `offsets` (Problem 1: worker i sends partition j to
 * server j; Algorithm 1 output).  On ZEN_REF_ERR_CAPACITY *nnz_out still holds
 * the number of rows needed.
 */
int zen_ref_encode(const float *grad, uint64_t n_rows, uint32_t row_dim, uint32_t n, uint32_t seed,
                   uint32_t *offsets, uint32_t *indices, float *values, uint64_t cap_rows,
                   uint64_t *nnz_out)
{
    if (!grad || n == 0 || n > 65535u || row_dim == 0 || n_rows > 0xfffffffeull)
        return ZEN_REF_ERR_INVALID;
    int64_t nnz = zen_ref_nonzero(grad, n_rows, row_dim, NULL);
    if (nnz_out) *nnz_out = (uint64_t)nnz;
    if ((uint64_t)nnz > cap_rows) return ZEN_REF_ERR_CAPACITY;
    uint32_t *I = (uint32_t *)malloc(((size_t)nnz + 1) * 4);
    uint16_t *own = (uint16_t *)malloc(((size_t)nnz + 1) * 2);
    if (!I || !own) { free(I); free(own); return ZEN_REF_ERR_NOMEM; }
    zen_ref_nonzero(grad, n_rows, row_dim, I);
    for (int64_t k = 0; k < nnz; ++k) own[k] = (uint16_t)zen_ref_owner(I[k], seed, n);
    int rc = zen_ref_partition(I, own, (uint64_t)nnz, n, offsets, indices);
    if (rc == ZEN_REF_OK && values) zen_ref_gather(grad, row_dim, indices, (uint64_t)nnz, values);
    free(I);
    free(own);
    return rc;
}

/*
 * Hash-bitmap layout (section "Hash Bitmap"): the domain of partition p is
 * II_p = { r in [0,R) : owner[r] = p } in ascending order; its bitmap has
 * |II_p| bits.  dom_count[p] = |II_p|; word_off[p] = first 32-bit word of
 * partition p when every partition starts on a word boundary; word_off[n] is
 * the total number of words (the appendix "Proof of The Property of Hash
 * Bitmap" gives sum |II_p| = |G| bits, i.e. |G|/32 words before padding).
 */
int zen_ref_bitmap_layout(const uint16_t *owner, uint64_t n_rows, uint32_t n, uint64_t *dom_count,
                          uint64_t *word_off)
{
    if (n == 0) return ZEN_REF_ERR_INVALID;
    for (uint32_t p = 0; p < n; ++p) dom_count[p] = 0;
    for (uint64_t r = 0; r < n_rows; ++r) {
        if (owner[r] >= n) return ZEN_REF_ERR_INVALID;
        dom_count[owner[r]]++;
    }
    word_off[0] = 0;
    for (uint32_t p = 0; p < n; ++p) word_off[p + 1] = word_off[p] + (dom_count[p] + 31) / 32;
    return ZEN_REF_OK;
}

/*
 * hash_bitmap_encode (Algorithm 2): local = G[II_p]; bit j = [local[j] != 0].
 * `nz[r]` is 1 iff row r is non-zero.  All partitions are written, partition p
 * starting at word_off[p]; padding bits are 0.
 */
int zen_ref_bitmap_encode(const uint16_t *owner, uint64_t n_rows, uint32_t n, const uint8_t *nz,
                          const uint64_t *word_off, uint32_t *bitmap)
{
    memset(bitmap, 0, (size_t)word_off[n] * 4);
    for (uint32_t p = 0; p < n; ++p) {
        uint64_t j = 0; /* position inside II_p */
        for (uint64_t r = 0; r < n_rows; ++r) {
            if (owner[r] != p) continue;
            if (nz[r]) bitmap[word_off[p] + (j >> 5)] |= 1u << (j & 31);
            ++j;
        }
    }
    return ZEN_REF_OK;
}

/*
 * hash_bitmap_decode (Algorithm 2): bitmap indices = positions of the 1 bits;
 * indices = II_p[bitmap indices].  `bitmap_p` points at partition p's first
 * word.  Returns the number of indices written (ascending).
 */
int64_t zen_ref_bitmap_decode(const uint16_t *owner, uint64_t n_rows, uint32_t p,
                              const uint32_t *bitmap_p, uint32_t *indices)
{
    int64_t count = 0;
    uint64_t j = 0;
    for (uint64_t r = 0; r < n_rows; ++r) {
        if (owner[r] != p) continue;
        if ((bitmap_p[j >> 5] >> (j & 31)) & 1u) indices[count++] = (uint32_t)r;
        ++j;
    }
    return count;
}

/*
 * Aggregation at a server (section "Elemental Dimensions for Synchronization":
 * gradients with the same indices are aggregated; Definition "imbalance
 * ratio": II_i is the index set at server i after aggregation).
 *
 * Inputs: n_in parts, part w = idx[w][0..counts[w]) with rows val[w][k][0..D).
 * Output: out_idx = ascending union of all indices (kept even if the sum is 0);
 * for every output row u and column c
 *     out_sum[u][c] = sum over every occurrence, in input order (w, then k), fp64
 *     out_abs[u][c] = sum of |x| over the same occurrences (for the test tolerance)
 *     out_val[u][c] = (float)out_sum[u][c]
 * out_ncontrib[u] = number of occurrences.  out_sum/out_abs/out_ncontrib may be
 * NULL.  Returns U (>= 0), or -(needed rows) if U > cap_rows, or INT64_MIN on a
 * bad argument / allocation failure.
 */
int64_t zen_ref_aggregate(uint32_t n_in, const uint32_t *const *idx, const float *const *val,
                          const uint64_t *counts, uint64_t n_rows, uint32_t row_dim,
                          uint32_t *out_idx, float *out_val, double *out_sum, double *out_abs,
                          uint32_t *out_ncontrib, uint64_t cap_rows)
{
    if (row_dim == 0 || n_rows > 0xfffffffeull) return INT64_MIN;
    uint32_t *occ = (uint32_t *)calloc((size_t)n_rows + 1, 4); /* occurrences per row id */
    if (!occ) return INT64_MIN;
    for (uint32_t w = 0; w < n_in; ++w)
        for (uint64_t k = 0; k < counts[w]; ++k) {
            if (idx[w][k] >= n_rows) { free(occ); return INT64_MIN; }
            occ[idx[w][k]]++;
        }
    int64_t U = 0;
    for (uint64_t r = 0; r < n_rows; ++r) if (occ[r]) ++U;
    if ((uint64_t)U > cap_rows) { free(occ); return -U; }

    /* pos[r] = place of row r in the ascending union */
    uint32_t *pos = (uint32_t *)malloc(((size_t)n_rows + 1) * 4);
    double *sum = (double *)calloc((size_t)U * row_dim + 1, 8);
    double *abs_ = (double *)calloc((size_t)U * row_dim + 1, 8);
    if (!pos || !sum || !abs_) { free(occ); free(pos); free(sum); free(abs_); return INT64_MIN; }
    int64_t u = 0;
    for (uint64_t r = 0; r < n_rows; ++r)
        if (occ[r]) {
            out_idx[u] = (uint32_t)r;
            if (out_ncontrib) out_ncontrib[u] = occ[r];
            pos[r] = (uint32_t)u++;
        }
    for (uint32_t w = 0; w < n_in; ++w)
        for (uint64_t k = 0; k < counts[w]; ++k) {
            uint64_t o = (uint64_t)pos[idx[w][k]] * row_dim;
            const float *row = val[w] + k * (uint64_t)row_dim;
            for (uint32_t c = 0; c < row_dim; ++c) {
                sum[o + c] += (double)row[c];
                abs_[o + c] += fabs((double)row[c]);
            }
        }
    for (uint64_t e = 0; e < (uint64_t)U * row_dim; ++e) {
        out_val[e] = (float)sum[e];
        if (out_sum) out_sum[e] = sum[e];
        if (out_abs) out_abs[e] = abs_[e];
    }
    free(occ); free(pos); free(sum); free(abs_);
    return U;
}

/*
 * Pull, server side (section "Hash Bitmap": hash_bitmap_encode is invoked at
 * each server on what it aggregated).  The server's tensor is the aggregated
 * sparse partition; reading taken: a row is "present" iff it belongs to the
 * aggregated index set, so a row whose sum cancelled to zero keeps its bit and
 * the k-th value stays the value of the k-th set bit.  member[r] = 1 iff r is in
 * idx[0..count); the bitmap itself is then zen_ref_bitmap_encode(member).
 */
int zen_ref_member_mask(const uint32_t *idx, uint64_t count, uint64_t n_rows, uint8_t *member)
{
    memset(member, 0, (size_t)n_rows);
    for (uint64_t k = 0; k < count; ++k) {
        if (idx[k] >= n_rows) return ZEN_REF_ERR_INVALID;
        member[idx[k]] = 1;
    }
    return ZEN_REF_OK;
}

/*
 * A sparse tensor given as parts (indices, rows) written out densely: G[idx] =
 * row, zero elsewhere (section "Elemental Dimensions for Synchronization": the
 * outcome of synchronization is the aggregated tensor, identical on all GPUs).
 * An index out of range, or one that occurs twice, is an error: parts of one
 * synchronized tensor are disjoint (Algorithm 1 sends an index to one server).
 */
int zen_ref_densify(uint32_t n_in, const uint32_t *const *idx, const float *const *val,
                    const uint64_t *counts, uint64_t n_rows, uint32_t row_dim, float *dense)
{
    uint8_t *seen = (uint8_t *)calloc((size_t)n_rows + 1, 1);
    if (!seen) return ZEN_REF_ERR_INVALID;
    memset(dense, 0, (size_t)n_rows * row_dim * 4);
    for (uint32_t w = 0; w < n_in; ++w)
        for (uint64_t k = 0; k < counts[w]; ++k) {
            uint32_t r = idx[w][k];
            if (r >= n_rows || seen[r]) { free(seen); return ZEN_REF_ERR_INVALID; }
            seen[r] = 1;
            memcpy(dense + (uint64_t)r * row_dim, val[w] + k * (uint64_t)row_dim, (size_t)row_dim * 4);
        }
    free(seen);
    return ZEN_REF_OK;
}

/*
 * Pull, worker side (section "Hash Bitmap": after a worker has received the
 * hash bitmaps of all servers it calls hash_bitmap_decode with the matching
 * II_p): partition p's bitmap starts at word_off[p]; its k-th set bit names row
 * II_p[bit position], whose values are val[p][k].  The decoded partitions are
 * written out densely.  The number of set bits must equal counts[p].
 */
int zen_ref_pull_apply(const uint16_t *owner, uint64_t n_rows, uint32_t n, uint32_t row_dim,
                       const uint64_t *word_off, const uint32_t *bitmap, const float *const *val,
                       const uint64_t *counts, float *dense)
{
    uint32_t *idx = (uint32_t *)malloc(((size_t)n_rows + 1) * 4);
    if (!idx) return ZEN_REF_ERR_INVALID;
    memset(dense, 0, (size_t)n_rows * row_dim * 4);
    for (uint32_t p = 0; p < n; ++p) {
        int64_t k = zen_ref_bitmap_decode(owner, n_rows, p, bitmap + word_off[p], idx);
        if ((uint64_t)k != counts[p]) { free(idx); return ZEN_REF_ERR_INVALID; }
        for (int64_t i = 0; i < k; ++i)
            memcpy(dense + (uint64_t)idx[i] * row_dim, val[p] + (uint64_t)i * row_dim, (size_t)row_dim * 4);
    }
    free(idx);
    return ZEN_REF_OK;
}

/*
 * Algorithm 1 ("Hierarchical Hashing Algorithm") as a mechanism, step by step,
 * for the indices taken ONE AFTER THE OTHER in the given order (the paper runs
 * them in parallel; any serial order is one of its possible executions).
 *
 *   x      n partitions of r1 + r2 cells, all empty (the paper's zeros; here
 *          0xFFFFFFFF because row ids start at 0)
 *   c      n counters, all r1
 *   for every idx:  p = part[t];  for i = 1..k: q = slot[i-1][t] (in [0, r1));
 *          if x[p][q] is empty, write idx there and stop;  after k occupied
 *          cells: q = c[p]++ and x[p][q] = idx (serial memory).
 *
 * part[t] = h0(I[t]) and slot[i][t] = h_{i+1}(I[t]) are handed in as tables, so
 * that a test can inject the collisions of a worked example; zen_ref_hash_slots
 * fills them with the seeded hash.  The read-after-write check (Technique #4)
 * guards against two threads writing one cell at the same time; with one index
 * at a time it never fires and is left out.
 *
 * Returns 0, or ZEN_REF_ERR_CAPACITY if some partition's serial memory (r2
 * cells) overflows -- the paper does not say what happens then; reading taken:
 * an error, with *needed_r2 = the largest serial count any partition reached.
 * serial_count[p] = indices of partition p that went to serial memory.
 */
int zen_ref_hierarchical_hash(const uint32_t *I, uint64_t nnz, const uint16_t *part, const uint32_t *const *slot,
                              uint32_t k, uint32_t n, uint64_t r1, uint64_t r2, uint32_t *x,
                              uint64_t *serial_count, uint64_t *needed_r2)
{
    const uint64_t cells = r1 + r2;
    uint64_t *c = (uint64_t *)malloc((size_t)n * 8);
    if (!c) return ZEN_REF_ERR_NOMEM;
    for (uint64_t a = 0; a < (uint64_t)n * cells; ++a) x[a] = 0xffffffffu;
    for (uint32_t p = 0; p < n; ++p) c[p] = r1;
    for (uint64_t t = 0; t < nnz; ++t) {
        const uint32_t p = part[t];
        if (p >= n) { free(c); return ZEN_REF_ERR_INVALID; }
        int placed = 0;
        for (uint32_t i = 0; i < k && !placed; ++i) {
            const uint64_t q = slot[i][t];
            if (q >= r1) { free(c); return ZEN_REF_ERR_INVALID; }
            if (x[p * cells + q] == 0xffffffffu) { x[p * cells + q] = I[t]; placed = 1; }
        }
        if (!placed) {
            const uint64_t q = c[p]++;
            if (q < cells) x[p * cells + q] = I[t];
        }
    }
    uint64_t worst = 0;
    for (uint32_t p = 0; p < n; ++p) {
        if (serial_count) serial_count[p] = c[p] - r1;
        if (c[p] - r1 > worst) worst = c[p] - r1;
    }
    free(c);
    if (needed_r2) *needed_r2 = worst;
    return worst > r2 ? ZEN_REF_ERR_CAPACITY : ZEN_REF_OK;
}

/* slot[t] = h_i(I[t]) = MurmurHash3_x86_32(I[t], seed_i) mod r1 -- the second-level hash functions,
 * which a worker may choose freely (Technique #3), here the same seeded family as h0. */
void zen_ref_hash_slots(const uint32_t *I, uint64_t nnz, uint32_t seed_i, uint64_t r1, uint32_t *slot)
{
    for (uint64_t t = 0; t < nnz; ++t) slot[t] = (uint32_t)(zen_ref_hash(I[t], seed_i) % r1);
}

/*
 * Extraction (Algorithm 1, output loop): indices = nonzero(x[p]) in memory
 * order for every partition, concatenated partition-major with an exclusive
 * prefix; the values are then G[indices] (zen_ref_gather).  Returns the number
 * of indices.
 */
int64_t zen_ref_hash_memory_extract(const uint32_t *x, uint32_t n, uint64_t cells, uint32_t *offsets,
                                    uint32_t *indices)
{
    int64_t out = 0;
    for (uint32_t p = 0; p < n; ++p) {
        offsets[p] = (uint32_t)out;
        for (uint64_t q = 0; q < cells; ++q)
            if (x[p * cells + q] != 0xffffffffu) indices[out++] = x[p * cells + q];
    }
    offsets[n] = (uint32_t)out;
    return out;
}

/*
 * Overlap ratio (Definition "The overlap ratio"): |I1 n I2| / min(|I1|, |I2|)
 * for two index sets given as lists without repeats.  0 if either set is empty.
 */
double zen_ref_overlap_ratio(const uint32_t *I1, uint64_t n1, const uint32_t *I2, uint64_t n2, uint64_t n_rows)
{
    if (n1 == 0 || n2 == 0) return 0.0;
    uint8_t *in1 = (uint8_t *)calloc((size_t)n_rows + 1, 1);
    if (!in1) return -1.0;
    for (uint64_t k = 0; k < n1; ++k) in1[I1[k]] = 1;
    uint64_t both = 0;
    for (uint64_t k = 0; k < n2; ++k) both += in1[I2[k]];
    free(in1);
    return (double)both / (double)(n1 < n2 ? n1 : n2);
}

/*
 * Sizes of the unions of the first k index sets, k = 1..n_sets: union_size[k-1]
 * = |I_1 u ... u I_k|.  With |G| rows the density after aggregating k tensors
 * is d_G^k = union_size[k-1] / |G| and the densification ratio (Definition
 * "The densification ratio") gamma_G^k = d_G^k / d_G.
 */
int zen_ref_union_sizes(uint32_t n_sets, const uint32_t *const *idx, const uint64_t *counts, uint64_t n_rows,
                        uint64_t *union_size)
{
    uint8_t *seen = (uint8_t *)calloc((size_t)n_rows + 1, 1);
    if (!seen) return ZEN_REF_ERR_NOMEM;
    uint64_t u = 0;
    for (uint32_t w = 0; w < n_sets; ++w) {
        for (uint64_t k = 0; k < counts[w]; ++k) {
            if (idx[w][k] >= n_rows) { free(seen); return ZEN_REF_ERR_INVALID; }
            if (!seen[idx[w][k]]) { seen[idx[w][k]] = 1; ++u; }
        }
        union_size[w] = u;
    }
    free(seen);
    return ZEN_REF_OK;
}

/*
 * Skewness ratio (Definition "The skewness ratio"): G is split evenly into n
 * consecutive partitions G_1..G_n; the ratio is max_i d_{G_i} / d_G.  Reading
 * taken for |G| not divisible by n: every partition has ceil(|G|/n) rows except
 * the last non-empty one, which has the rest; empty partitions are skipped.
 * part_nnz (may be NULL) receives the non-zero count of every partition.
 */
double zen_ref_skewness(const uint32_t *I, uint64_t nnz, uint64_t n_rows, uint32_t n, uint64_t *part_nnz)
{
    if (n == 0 || n_rows == 0) return 0.0;
    const uint64_t size = (n_rows + n - 1) / n;
    uint64_t *c = (uint64_t *)calloc(n, 8);
    if (!c) return -1.0;
    for (uint64_t k = 0; k < nnz; ++k) c[I[k] / size]++;
    double worst = 0.0;
    for (uint32_t i = 0; i < n; ++i) {
        const uint64_t lo = (uint64_t)i * size;
        if (part_nnz) part_nnz[i] = c[i];
        if (lo >= n_rows) continue;
        const uint64_t rows = (lo + size <= n_rows ? size : n_rows - lo);
        const double d_i = (double)c[i] / (double)rows;
        if (d_i > worst) worst = d_i;
    }
    free(c);
    if (nnz == 0) return 0.0;
    return worst / ((double)nnz / (double)n_rows);
}

/*
 * Theoretical communication time of Balanced Parallelism, Equation (1):
 *     T_bp = (n-1)/n * (gamma_G^n + 1) * 2 M d_G / b
 * (each GPU receives 2(n-1)/n d_G M in Push and gamma_G^n times that in Pull).
 */
double zen_ref_time_balanced_parallelism(uint32_t n, double gamma_n, double d_G, double M, double b)
{
    return (double)(n - 1) / (double)n * (gamma_n + 1.0) * 2.0 * M * d_G / b;
}

/*
 * Theoretical communication time of Hierarchical Centralization, Equation (2):
 *     T_sm = sum_{i=1}^{log2 n} gamma_G^{2^(i-1)} * 2 M d_G / b,   n a power of two;
 * gamma_pow2[i-1] = gamma_G^{2^(i-1)}, so gamma_pow2[0] = gamma_G^1 = 1.
 */
double zen_ref_time_hierarchical_centralization(uint32_t n, const double *gamma_pow2, double d_G, double M, double b)
{
    double sum = 0.0;
    uint32_t stages = 0;
    while ((1u << stages) < n) ++stages;
    for (uint32_t i = 0; i < stages; ++i) sum += gamma_pow2[i];
    return sum * 2.0 * M * d_G / b;
}

/*
 * Top-k threshold of a sparsifier in the style the paper uses in front of the
 * synchronization (section "Implementation": sample the gradients, take the
 * top-k threshold of the sample, apply it to the whole tensor; section
 * "Characteristics": the top 5 % are kept).  The sample is every `stride`-th
 * element starting at `first` (stride 1, first 0 = the whole tensor: exact
 * top-k); magnitudes are compared as integers, mag(x) = bits(x) & 0x7fffffff,
 * which orders non-NaN floats like |x| and puts NaN above Inf.  keep = number of
 * sample elements to keep, 1 <= keep <= sample size; the threshold is the
 * keep-th largest magnitude of the sample.  An element of the tensor is then
 * kept iff mag(x) >= threshold and mag(x) != 0 (zen_ref_threshold_apply).
 * Returns the threshold's bit pattern, or 0xffffffff on a bad argument.
 */
static int cmp_u32_desc(const void *a, const void *b)
{
    const uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return x < y ? 1 : (x > y ? -1 : 0);
}

uint32_t zen_ref_topk_threshold(const float *g, uint64_t n, uint64_t first, uint64_t stride, uint64_t keep)
{
    if (stride == 0 || first >= n) return 0xffffffffu;
    const uint64_t m = (n - first + stride - 1) / stride;
    if (keep == 0 || keep > m) return 0xffffffffu;
    uint32_t *mag = (uint32_t *)malloc((size_t)m * 4);
    if (!mag) return 0xffffffffu;
    for (uint64_t t = 0; t < m; ++t) {
        uint32_t bits;
        memcpy(&bits, g + first + t * stride, 4);
        mag[t] = bits & 0x7fffffffu;
    }
    qsort(mag, (size_t)m, 4, cmp_u32_desc);
    const uint32_t thr = mag[keep - 1];
    free(mag);
    return thr;
}

/* out[i] = g[i] if mag(g[i]) >= max(threshold, 1) else +0.0; returns the number kept. */
uint64_t zen_ref_threshold_apply(const float *g, uint64_t n, uint32_t threshold, float *out)
{
    uint64_t kept = 0;
    const uint32_t thr = threshold ? threshold : 1u;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t bits;
        memcpy(&bits, g + i, 4);
        if ((bits & 0x7fffffffu) >= thr) { out[i] = g[i]; ++kept; } else { out[i] = 0.0f; }
    }
    return kept;
}

/*
 * Bytes needed to send an aggregated fp32 sparse tensor of |G| elements with
 * nnz non-zeros to a worker in each format of section "Sparse Formats" when the
 * tensor is hash-partitioned over n servers (figure "tensor data size with
 * different sparse formats": 16 servers):
 *   dense        4|G|
 *   COO          8 nnz                      (a 4-byte index per 4-byte value)
 *   bitmap       4 nnz + n * |G|/8          (every server's non-zeros are spread over the whole
 *                                            range, so every server sends a |G|-bit bitmap)
 *   hash bitmap  4 nnz + |G|/8              (appendix "Proof of The Property of Hash Bitmap")
 *   tensor block nonzero_blocks * (4*block + 4)   (OmniReduce: whole blocks of `block` gradients,
 *                                            plus a 4-byte block id each)
 * out[0..4] in that order.
 */
void zen_ref_format_bytes(uint64_t G, uint64_t nnz, uint32_t n, uint64_t nonzero_blocks, uint32_t block, double *out)
{
    out[0] = 4.0 * (double)G;
    out[1] = 8.0 * (double)nnz;
    out[2] = 4.0 * (double)nnz + (double)n * (double)G / 8.0;
    out[3] = 4.0 * (double)nnz + (double)G / 8.0;
    out[4] = (double)nonzero_blocks * (4.0 * (double)block + 4.0);
}

/* Number of blocks of `block` consecutive elements that hold at least one non-zero index. */
uint64_t zen_ref_nonzero_blocks(const uint32_t *I, uint64_t nnz, uint64_t n_rows, uint32_t block)
{
    if (block == 0) return 0;
    const uint64_t nb = (n_rows + block - 1) / block;
    uint8_t *hit = (uint8_t *)calloc((size_t)nb + 1, 1);
    if (!hit) return 0;
    uint64_t c = 0;
    for (uint64_t k = 0; k < nnz; ++k) {
        const uint64_t b = I[k] / block;
        if (!hit[b]) { hit[b] = 1; ++c; }
    }
    free(hit);
    return c;
}

/*
 * Imbalance ratio (Definition "The imbalance ratio"): max_j n*|part_j| / total.
 * Push uses one worker's partition sizes; Pull uses the servers' set sizes
 * after aggregation.  Returns 1.0 for an empty input (nothing to balance).
 */
double zen_ref_imbalance(const uint64_t *sizes, uint32_t n)
{
    uint64_t total = 0, mx = 0;
    for (uint32_t j = 0; j < n; ++j) { total += sizes[j]; if (sizes[j] > mx) mx = sizes[j]; }
    if (total == 0) return 1.0;
    return (double)n * (double)mx / (double)total;
}
