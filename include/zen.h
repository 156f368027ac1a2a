/*
 * zen.h -- C ABI of the MI355X (gfx950) sparse-gradient encode + aggregate library.
 *
 * The library implements the per-GPU hot path of Zen's Balanced Parallelism (arXiv 2309.13254):
 *   zen_encode     one worker's dense gradient -> n hash partitions of (indices, values)
 *                  [Algorithm 1 "Hierarchical Hashing Algorithm": input G and its non-zero index set
 *                  I, p <- h0(idx), output one (indices, values) pair per partition; Problem 1]
 *   zen_aggregate  the n incoming partitions of one server -> one summed sparse tensor
 *                  [section "Elemental Dimensions for Synchronization": gradients with the same
 *                  indices are aggregated; Definition "imbalance ratio": index set II_i at server i]
 *   hash bitmap    optional index encoding of a partition over its hash domain
 *                  [section "Hash Bitmap", Algorithm 2 hash_bitmap_encode / hash_bitmap_decode]
 *   zen_pull_*     the way back: a server's aggregated partition as a hash bitmap, and the worker's
 *                  decode of all servers' bitmaps into the synchronized dense tensor
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name starts with host_ or the comment says "host".
 *     Structs (zen_encoded, zen_part, zen_aggregated) live on the host and hold device pointers.
 *   - The caller owns every buffer, including workspaces; the library allocates device memory only
 *     inside zen_ctx_create (immutable hash-domain tables) and frees it in zen_ctx_destroy.
 *   - All work is enqueued on the given HIP stream (hipStream_t passed as void*; NULL = default
 *     stream) and nothing synchronises except zen_ctx_create and zen_status_fetch.  Counts stay on
 *     the device: offsets[n_parts] is a worker's nnz, *count a server's number of unique rows.
 *   - Errors are integer statuses; nothing is thrown across the ABI.  Argument errors are detected
 *     on the host before anything is launched.  Overflow of a caller-given capacity is detected on
 *     the device: nothing is written past a capacity, a flag is raised in the workspace, and
 *     zen_status_fetch turns it into ZEN_ERR_CAPACITY together with the number of rows needed.
 *   - Rows are indexed from 0 with 32-bit ids; 0xFFFFFFFF is reserved, so n_rows <= 2^32 - 2.
 *     A row is non-zero iff any of its row_dim fp32 words has (bits & 0x7fffffff) != 0.
 *   - h0(idx) = MurmurHash3_x86_32(idx as 4 little-endian bytes, hash_seed) mod n_parts -- the same
 *     on every worker, so an index always reaches the same server [Technique #3].
 *   - Inside every partition indices ascend; values follow the same order, whole rows, bit-exact.
 */
#ifndef ZEN_H
#define ZEN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZEN_MAX_PARTS 1024u /* n_parts limit (per-block LDS histograms) */
#define ZEN_MAX_BATCH 64u   /* workers / servers / incoming parts per launch group */

typedef enum {
    ZEN_OK = 0,
    ZEN_ERR_INVALID = 1,  /* bad argument (null, misaligned, out of range, mismatch with the context) */
    ZEN_ERR_CAPACITY = 2, /* an output or table capacity was too small (see zen_status_fetch) */
    ZEN_ERR_NOMEM = 3,    /* device allocation failed / workspace too small */
    ZEN_ERR_DEVICE = 4    /* a HIP call failed */
} zen_status;

typedef enum {
    ZEN_INDEX_COO = 0,   /* indices as a list of row ids (the paper's Push format) */
    ZEN_INDEX_BITMAP = 1 /* indices as a hash bitmap over each partition's domain (Algorithm 2) */
} zen_index_format;

typedef struct zen_ctx zen_ctx; /* immutable function of (n_rows, row_dim, n_parts, hash_seed, fmt) */

/* One encoded gradient = n_parts partitions stored partition-major. */
typedef struct {
    uint32_t *offsets;   /* [n_parts+1] rows; offsets[0]=0, offsets[p+1]-offsets[p] = size of partition p */
    uint32_t *indices;   /* [cap_rows] ascending inside each partition; may be NULL in BITMAP mode */
    float    *values;    /* [cap_rows][row_dim], same order as indices */
    uint32_t *bitmap;    /* BITMAP mode: [zen_bitmap_words()] words, partition p at zen_bitmap_offsets()[p],
                            bit j (LSB-first) = 1 iff the j-th smallest row of partition p's domain is
                            non-zero; padding bits 0.  NULL in COO mode. */
    uint64_t  cap_rows;  /* capacity of indices and values, in rows */
} zen_encoded;

/* One incoming partition at a server (zen_aggregate). */
typedef struct {
    const uint32_t *indices; /* [*count] row ids, any order, duplicates allowed (they are summed);
                                NULL if `bitmap` is given */
    const uint32_t *bitmap;  /* hash bitmap of partition part_id (first word of that partition), or NULL */
    const float    *values;  /* [*count][row_dim]; with a bitmap the k-th row belongs to the k-th set bit */
    const uint32_t *count;   /* device scalar: number of rows */
} zen_part;

/* Aggregated partition of one server. */
typedef struct {
    uint32_t *indices;  /* [cap_rows] ascending union of the incoming indices */
    float    *values;   /* [cap_rows][row_dim] fp32 sums */
    uint32_t *count;    /* device scalar: number of unique rows U */
    uint64_t  cap_rows;
} zen_aggregated;

/* Status block fetched from a workspace. */
typedef struct {
    uint32_t flags;        /* bit 0: output capacity overflow, bit 1: table/bound overflow,
                              bit 2: inconsistent input (bitmap vs row count, foreign or unsorted index) */
    uint32_t reserved;
    uint64_t needed_rows;  /* largest number of rows any overflowing output / table needed */
} zen_status_info;

/*
 * Create a context.  Synchronous.  For ZEN_INDEX_BITMAP it builds, on the device, the sorted hash
 * domains II_p = { r : h0(r) = p } ("computed and sorted offline", section "Hash Bitmap") and their
 * per-tile rank bases: 4*n_rows bytes + small tables.  Limits: 1 <= n_rows <= 2^32-2,
 * row_dim >= 1, 1 <= n_parts <= ZEN_MAX_PARTS.
 */
zen_status zen_ctx_create(zen_ctx **out, uint64_t n_rows, uint32_t row_dim, uint32_t n_parts,
                          uint32_t hash_seed, zen_index_format fmt);
zen_status zen_ctx_destroy(zen_ctx *ctx);

/*
 * zen_ctx_create with explicit tuning (not part of the method; results do not depend on it).  The
 * library reads no environment variable: what can be tuned at run time is tuned here.
 * host_tuning == NULL: the defaults, i.e. zen_ctx_create.
 */
typedef struct {
    uint32_t tile_bytes;    /* dense bytes per tile (the unit of one block of the dense scan and of one
                               histogram row), 4096 .. 8 MiB; 0 = the default, 128 KiB */
    uint32_t tiled_encode;  /* 1 = every encode takes the tiled partition path (per-tile histograms, scan,
                               scatter), also the few-row ones that one block per worker would do; 0 = default */
} zen_tuning;
zen_status zen_ctx_create_tuned(zen_ctx **out, uint64_t n_rows, uint32_t row_dim, uint32_t n_parts,
                                uint32_t hash_seed, zen_index_format fmt, const zen_tuning *host_tuning);

/* Hash-bitmap layout (host outputs).  total words = sum_p ceil(|II_p|/32) <= n_rows/32 + n_parts
 * (appendix "Proof of The Property of Hash Bitmap").  host_word_offsets has n_parts+1 entries and
 * host_domain_sizes n_parts entries; either may be NULL.  ZEN_ERR_INVALID for a COO context. */
zen_status zen_bitmap_layout(const zen_ctx *ctx, uint64_t *host_total_words, uint64_t *host_word_offsets,
                             uint64_t *host_domain_sizes);

/* Workspace sizes in bytes.  `batch` = number of workers (encode) or servers (aggregate) handled by
 * one call; max_in_rows = upper bound on the total rows entering ONE server (sum over its parts). */
zen_status zen_encode_workspace_bytes(const zen_ctx *ctx, uint32_t batch, uint64_t *host_bytes);
zen_status zen_aggregate_workspace_bytes(const zen_ctx *ctx, uint32_t batch, uint64_t max_in_rows,
                                         uint64_t *host_bytes);
/* Both at once: *host_enc_bytes = zen_encode_workspace_bytes(ctx, batch), *host_agg_bytes =
 * zen_aggregate_workspace_bytes(ctx, batch, max_nnz) with max_nnz the bound on the rows entering one
 * server (e.g. the sum over the workers of their largest partition).  Either output may be NULL. */
zen_status zen_workspace_bytes(const zen_ctx *ctx, uint64_t max_nnz, uint32_t batch, uint64_t *host_enc_bytes,
                               uint64_t *host_agg_bytes);

/*
 * Encode one worker's gradient (Algorithm 1's result).  grad: [n_rows][row_dim] fp32 row-major,
 * 16-byte aligned.  n_parts and hash_seed must equal the context's.  Fills out->offsets, and
 * out->indices + out->values (COO) or out->bitmap + out->values (BITMAP; indices also written if
 * out->indices != NULL).  If nnz > out->cap_rows nothing is written past the capacity, offsets are
 * still complete, and the capacity flag is raised with needed_rows = nnz.
 */
zen_status zen_encode(zen_ctx *ctx, const float *grad, uint32_t n_parts, uint32_t hash_seed,
                      const zen_encoded *host_out, void *workspace, uint64_t workspace_bytes,
                      void *hip_stream);

/*
 * zen_encode for callers that cannot allocate device memory or hand in a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same kernels as
 * zen_encode, with the workspace (row mask, per-tile owner histograms, tile flags and lists, the
 * status block) held in a file-scope device array of ZEN_STATIC_SCRATCH_BYTES that every GPU the
 * library runs on keeps until the process ends; its address is looked up once per device
 * (zen_ctx_create does it for the context's device; otherwise the first call on a device does).
 * Nothing is allocated or freed, here or in any routine the call uses.
 *   status (device, 16-byte aligned, may be NULL): receives the call's zen_status_info on the
 *   stream when the encode has finished (flags bit 0: nnz > cap_rows, needed_rows = nnz).
 * A context whose one-worker workspace (zen_encode_workspace_bytes(ctx, 1)) exceeds
 * ZEN_STATIC_SCRATCH_BYTES is refused with ZEN_ERR_NOMEM before anything is launched (element-level
 * tensors: about n_rows <= 5e7; 16-partition tables of 64-float rows: about 4e7 rows).
 * All calls on one GPU share that GPU's array: calls that overlap there (two streams, two threads)
 * race and must be serialised by the caller.  What a call needs cleared it clears itself; nothing is
 * carried from one call to the next.
 */
#define ZEN_STATIC_SCRATCH_BYTES (8u << 20)
zen_status zen_encode_static(zen_ctx *ctx, const float *grad, uint32_t n_parts, uint32_t hash_seed,
                             const zen_encoded *host_out, zen_status_info *status, void *hip_stream);

/* The same for n_workers gradients per launch sequence.  host_grads / host_outs: host arrays. */
zen_status zen_encode_batch(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                            const zen_encoded *host_outs, void *workspace, uint64_t workspace_bytes,
                            void *hip_stream);

/*
 * Ascending list of the non-zero rows of grad (Algorithm 1's input I) -- detection and compaction
 * only.  indices: [cap_rows]; count: device scalar.
 */
zen_status zen_nonzero(zen_ctx *ctx, const float *grad, uint32_t *indices, uint64_t cap_rows,
                       uint32_t *count, void *workspace, uint64_t workspace_bytes, void *hip_stream);

/*
 * Aggregate n_in incoming parts at server part_id: out_indices = ascending union of the parts'
 * indices (kept even if a sum cancels to 0), out_values = fp32 sums over every occurrence, added in
 * ascending (part, position in the part) order with plain loads and one store per element (no value
 * atomics): the same inputs give the same bits on every call, and results agree with an fp64 sum to
 * ~1e-7 relative to sum|x|.  max_in_rows bounds sum of *count over the parts; it sizes the open-addressing table
 * (power of two >= 2*max_in_rows).  A larger actual total raises the table flag and leaves
 * *out_count = 0.  U > out_cap_rows raises the capacity flag, writes the first out_cap_rows rows
 * and sets *out_count = U.
 */
zen_status zen_aggregate(zen_ctx *ctx, const zen_part *host_parts, uint32_t n_in, uint32_t part_id,
                         uint32_t *out_indices, float *out_values, uint64_t out_cap_rows,
                         uint32_t *out_count, uint64_t max_in_rows, void *workspace,
                         uint64_t workspace_bytes, void *hip_stream);

/* All n_parts servers: server j merges partition j of every worker's encoded gradient.
 * host_encs: n_workers <= ZEN_MAX_BATCH entries (as filled by zen_encode*); host_outs: n_parts
 * entries.  Servers are handled in launch groups of ZEN_MAX_BATCH (one group when n_parts <= 64), so
 * the workspace is that of zen_aggregate_workspace_bytes(ctx, min(n_parts, ZEN_MAX_BATCH), max_in_rows);
 * the status block ends up holding the OR / maximum over all groups. */
zen_status zen_aggregate_batch(zen_ctx *ctx, const zen_encoded *host_encs, uint32_t n_workers,
                               const zen_aggregated *host_outs, uint64_t max_in_rows, void *workspace,
                               uint64_t workspace_bytes, void *hip_stream);

/*
 * ---- Pull: what a server sends back and what a worker does with it (section "Hash Bitmap") -----
 *
 * All Pull calls need a ZEN_INDEX_BITMAP context for their bitmap forms (the sorted domains II_p
 * live in the context) and a workspace of zen_pull_workspace_bytes; they keep a status block at the
 * start of the workspace like the other calls (flag bit 2 = inconsistent input, reported by
 * zen_status_fetch as ZEN_ERR_INVALID).
 */
zen_status zen_pull_workspace_bytes(const zen_ctx *ctx, uint64_t *host_bytes);

/*
 * hash_bitmap_encode at server part_id (Algorithm 2; "invoked at each server" on its aggregated
 * partition).  indices: the server's aggregated row ids, ASCENDING and distinct, all owned by
 * part_id (exactly what zen_aggregate writes); count: device scalar, clamped to cap_rows.
 * bitmap_words: the partition's own ceil(|II_p|/32) words; every one of them is written (bit j = 1
 * iff the j-th smallest row of II_p is in `indices`; padding 0).  A row counts as present when it is
 * in the index list, whatever its value, so the k-th value row keeps belonging to the k-th set bit
 * and the values are sent as they are.  Input that is not such a list raises flag bit 2; nothing is
 * read or written out of bounds.
 */
zen_status zen_pull_encode(zen_ctx *ctx, const uint32_t *indices, const uint32_t *count, uint64_t cap_rows,
                           uint32_t part_id, uint32_t *bitmap_words, void *workspace, uint64_t workspace_bytes,
                           void *hip_stream);

/* The same for all n_parts servers: host_aggs[j] = server j's zen_aggregate output, bitmap = the
 * whole layout of zen_bitmap_layout (partition j at word offset j). */
zen_status zen_pull_encode_batch(zen_ctx *ctx, const zen_aggregated *host_aggs, uint32_t *bitmap, void *workspace,
                                 uint64_t workspace_bytes, void *hip_stream);

/*
 * hash_bitmap_decode (Algorithm 2): out_indices = II_p[positions of the 1 bits], ascending;
 * *out_count = number of set bits.  More set bits than out_cap_rows: the first out_cap_rows indices
 * are written and the capacity flag is raised with needed_rows = the number of set bits.  Padding
 * bits of the last word are ignored.
 */
zen_status zen_pull_decode(zen_ctx *ctx, const uint32_t *bitmap_words, uint32_t part_id, uint32_t *out_indices,
                           uint64_t out_cap_rows, uint32_t *out_count, void *workspace, uint64_t workspace_bytes,
                           void *hip_stream);

/*
 * Worker side of Pull: the n_parts aggregated partitions (host_parts[p] = what server p sent: a hash
 * bitmap or an index list, values, count) written out as the synchronized dense tensor
 * dense[n_rows][row_dim] (16-byte aligned): dense[row] = the row's values where some partition holds
 * the row, 0 elsewhere [section "Elemental Dimensions for Synchronization": every GPU ends with the
 * same aggregated result].  Partitions are disjoint by construction; if an index occurs twice one of
 * its rows wins.  A bitmap whose set bits do not number *count, or an index >= n_rows, raises flag
 * bit 2; rows beyond *count are never read.  Index-list parts work with a COO context too.
 */
zen_status zen_pull_apply(zen_ctx *ctx, const zen_part *host_parts, float *dense, void *workspace,
                          uint64_t workspace_bytes, void *hip_stream);

/*
 * ---- Algorithm 1 as the paper runs it: the hash memory ---------------------------------------
 *
 * zen_encode computes Algorithm 1's RESULT with a histogram, a scan and a stable scatter.
 * zen_encode_hashed computes the same partitions with the algorithm's own mechanism [Algorithm 1,
 * Techniques #1-#4]: a memory of n_parts partitions, each with r1 cells of parallel memory and r2 of
 * serial memory; an index goes to partition h0(idx), tries the cells h_1(idx) .. h_k(idx) of the
 * parallel memory and, if all are taken, is appended to the serial memory through an atomic
 * counter; each partition is then extracted (nonzero) and its values gathered.
 *   h_i(idx) = MurmurHash3_x86_32(idx, level2_seed + i) mod r1 -- second-level functions are a
 *   worker's own choice (Technique #3); h0 is the context's.
 *   A cell is claimed with one compare-and-swap, which decides in one step what the listing's test,
 *   store and read-back (Technique #4) decide in three.
 * Output: host_out->offsets / indices / values as zen_encode writes them, except that inside a
 * partition the indices come in memory order (the paper: "random order ... no need to sort"); which
 * index wins a contested cell depends on timing, so only the SET per partition is reproducible.
 * serial_counts (device, [n_parts], may be NULL): indices of each partition that went to serial memory.
 * Errors through the workspace status: bit 0 = nnz > cap_rows (needed_rows = nnz); bit 1 = some
 * partition's serial memory overflowed and indices were dropped (needed_rows = the r2 that would
 * have sufficed).  hash_memory: zen_hash_memory_bytes, 256-byte aligned, overwritten.
 */
typedef struct {
    uint32_t k;           /* second-level hash functions, 1..8 (the paper uses 3) */
    uint32_t level2_seed; /* seeds of h_1..h_k are level2_seed + 1 .. level2_seed + k */
    uint64_t r1;          /* parallel cells per partition, >= 1 (the paper: 2|G|d_G over all partitions) */
    uint64_t r2;          /* serial cells per partition (the paper: r1 / 10) */
} zen_hash_params;

zen_status zen_hash_memory_bytes(const zen_ctx *ctx, const zen_hash_params *host_params, uint64_t *host_bytes);
zen_status zen_encode_hashed_workspace_bytes(const zen_ctx *ctx, const zen_hash_params *host_params,
                                             uint64_t *host_bytes);
zen_status zen_encode_hashed(zen_ctx *ctx, const float *grad, const zen_hash_params *host_params, void *hash_memory,
                             uint64_t hash_memory_bytes, const zen_encoded *host_out, uint32_t *serial_counts,
                             void *workspace, uint64_t workspace_bytes, void *hip_stream);

/*
 * ---- Sparsity metrics and the choice of the scheme ------------------------------------------
 *
 * Counts behind the metrics of section "Characteristics of Sparse Tensors" for n_workers <=
 * ZEN_MAX_BATCH gradients (device arrays of u64, all overwritten):
 *   nnz[w]             |I_w|                          -> density d_G = nnz / n_rows
 *   union_prefix[w]    |I_0 u ... u I_w|              -> d_G^k, densification ratio gamma_G^k = d_G^k / d_G
 *   overlap[a][b]      |I_a n I_b| (diagonal = nnz)   -> overlap ratio = overlap / min(nnz_a, nnz_b)
 *   even_split[w][i]   non-zero rows of worker w in the i-th of n_parts even consecutive partitions of
 *                      ceil(n_rows / n_parts) rows     -> skewness ratio = max_i d_{G_i} / d_G
 * (the hash partitions' sizes, for the imbalance ratio, are the offsets zen_encode writes).
 * workspace: zen_encode_workspace_bytes(ctx, n_workers).
 */
typedef struct {
    uint64_t *nnz;          /* [n_workers] */
    uint64_t *union_prefix; /* [n_workers] */
    uint64_t *overlap;      /* [n_workers][n_workers] */
    uint64_t *even_split;   /* [n_workers][n_parts] */
} zen_sparsity_counts;

zen_status zen_sparsity_count(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                              const zen_sparsity_counts *host_out, void *workspace, uint64_t workspace_bytes,
                              void *hip_stream);

/*
 * Theoretical communication times of the two candidate schemes (host arithmetic, no GPU work):
 *   Balanced Parallelism,        Equation (1): t_bp = (n-1)/n * (gamma^n + 1) * 2 M d_G / b
 *   Hierarchical Centralization, Equation (2): t_sm = sum_{i=1..log2 n} gamma^(2^(i-1)) * 2 M d_G / b
 * host_gamma_pow2 = { gamma^1, gamma^2, gamma^4, ..., gamma^n } (log2 n + 1 entries, gamma^1 = 1);
 * n a power of two >= 2; M = size of the dense tensor, b = bandwidth (same units).  The scheme with the
 * smaller time is the optimal one (Theorem "Optimal schemes").
 */
zen_status zen_scheme_times(uint32_t n, const double *host_gamma_pow2, double d_G, double M, double b,
                            double *host_t_bp, double *host_t_sm);

/*
 * ---- Gradient sparsifier in front of the encode, and the sparse formats' sizes ----------------
 *
 * zen_topk_threshold: the top-k threshold of a sparsifier in the style of DGC as the paper deploys it
 * [section "Implementation": sample the gradients, compute the top-k threshold of the sample, apply
 * it to the tensor; section "Characteristics of Sparse Tensors": the top 5 % are kept].  The sample
 * is g[first], g[first+stride], ... (first = 0, stride = 1: exact top-k of all n elements);
 * *threshold (device) = the keep-th largest magnitude of the sample as a bit pattern
 * (bits & 0x7fffffff; NaN ranks above Inf).  1 <= keep <= sample size.  workspace:
 * zen_topk_workspace_bytes, 256-byte aligned.  Nothing synchronises.
 *
 * zen_encode_batch_sparsified: zen_encode_batch of the tensors with every element whose magnitude is
 * below thresholds[w] (device array, one per worker; 0 and 1 both mean "every non-zero") treated as
 * zero -- the sparsifier is applied inside the dense scan, the tensor is neither copied nor
 * modified.  Element-level contexts (row_dim == 1) only.
 */
zen_status zen_topk_workspace_bytes(uint64_t *host_bytes);
zen_status zen_topk_threshold(const float *g, uint64_t n, uint64_t first, uint64_t stride, uint64_t keep,
                              uint32_t *threshold, void *workspace, uint64_t workspace_bytes, void *hip_stream);
zen_status zen_encode_batch_sparsified(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                                       const uint32_t *thresholds, const zen_encoded *host_outs, void *workspace,
                                       uint64_t workspace_bytes, void *hip_stream);

/*
 * Sizes of the sparse formats of section "Sparse Formats".  zen_format_count: counts[0] = non-zero
 * rows of grad, counts[1] = blocks of `block` consecutive rows holding at least one (device u64[2];
 * block a multiple of 32 that divides the context's tile; workspace: zen_encode_workspace_bytes(ctx, 1)).
 * zen_format_bytes (host arithmetic): bytes to send a tensor of n_elems fp32 elements with nnz
 * non-zeros, hash-partitioned over n_servers, as host_out[0..4] = dense 4|G|, COO 8 nnz, one |G|-bit
 * bitmap per server 4 nnz + n|G|/8, hash bitmap 4 nnz + |G|/8, tensor blocks nonzero_blocks *
 * (4 block + 4).
 */
zen_status zen_format_count(zen_ctx *ctx, const float *grad, uint32_t block, uint64_t *counts, void *workspace,
                            uint64_t workspace_bytes, void *hip_stream);
zen_status zen_format_bytes(uint64_t n_elems, uint64_t nnz, uint32_t n_servers, uint64_t nonzero_blocks, uint32_t block,
                            double *host_out);

/* Synchronous: waits for the stream, reads the status block of a workspace last used by an encode
 * or aggregate call, returns ZEN_OK / ZEN_ERR_CAPACITY and fills *host_info (may be NULL). */
zen_status zen_status_fetch(zen_ctx *ctx, const void *workspace, void *hip_stream,
                            zen_status_info *host_info);

/* After zen_status_fetch on this context returned ZEN_ERR_CAPACITY: *host_needed_rows = the rows the
 * largest overflowing output or table needed (what that fetch read); 0 if the last fetch found no
 * overflow or none was made.  No device work. */
zen_status zen_last_overflow(const zen_ctx *ctx, uint64_t *host_needed_rows);

/* h0's underlying 32-bit hash for `count` indices: out[i] = MurmurHash3_x86_32(idx[i], seed)
 * (section "Implementation").  Exposed so the hash can be checked on its own. */
zen_status zen_hash_many(const uint32_t *idx, uint64_t count, uint32_t seed, uint32_t *out,
                         void *hip_stream);

/* Plain device-to-device streaming copy of `bytes` (multiple of 16, both pointers 16-byte aligned):
 * reads `bytes`, writes `bytes`.  Not part of the method: it is the kernel of known traffic against
 * which hardware HBM byte counters are scaled when the library is profiled. */
zen_status zen_calibration_copy(const void *src, void *dst, uint64_t bytes, void *hip_stream);

/* Plain streaming READ of `bytes` (multiple of 16, src 16-byte aligned) with 16-byte loads: no LDS and next to no stores
 * (sink, a device array of 64 words, gets one word from a wave whose lanes each OR what they read to all ones).  Not part of
 * the method: it measures what a read-only stream reaches in a given launch shape -- the rate the dense scan of
 * zen_encode is held against -- and is a second kernel of known traffic for the byte counters.
 * host_shape == NULL: the dense scan's own shape (256 threads, 8 loads in flight, a 128 KiB tile per block,
 * non-temporal loads). */
typedef struct {
    uint32_t threads;      /* 256, 512 or 1024 per block */
    uint32_t unroll;       /* 4, 8 or 16 16-byte loads in flight per thread */
    uint32_t block_bytes;  /* contiguous bytes a block reads at a time (multiple of 16, >= 4096) */
    uint32_t max_blocks;   /* 0: one block per block_bytes; else at most this many blocks, which stride on */
    uint32_t nontemporal;  /* 1: non-temporal loads, 0: plain loads */
} zen_read_shape;
zen_status zen_calibration_read(const void *src, uint64_t bytes, const zen_read_shape *host_shape, uint32_t *sink,
                                void *hip_stream);

/*
 * Optional kernel timing with HIP events recorded on the launch stream (for benchmarks; not part of
 * the method).  mode 0 = off, 1 = time the dense-scan (detect) kernel only, 2 = time every kernel.
 * max_records event pairs are created up front; launches beyond that are not timed.
 * zen_profile_collect waits for the recorded events, adds up milliseconds and launch counts per
 * kernel into host arrays of at least 32 entries (index = kernel id, name from
 * zen_profile_kernel_name), and empties the record pool.
 */
zen_status zen_profile_enable(zen_ctx *ctx, uint32_t mode, uint32_t max_records);
zen_status zen_profile_collect(zen_ctx *ctx, uint32_t cap, double *host_ms_sum, uint32_t *host_launches,
                               uint32_t *host_n_kernels);
const char *zen_profile_kernel_name(uint32_t kernel);

const char *zen_status_str(zen_status s);

#ifdef __cplusplus
}
#endif
#endif /* ZEN_H */
