// Host-side internals shared by the C-ABI translation units: the context, launch geometry and
// the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/zen.h"

// Element-level hash-bitmap encodes: rows per group in which a fully non-zero stretch is recognised, and the
// most partitions the per-group rank table is kept for.
#define ZEN_GROUP_ROWS 512u
#define ZEN_GROUP_MAX_PARTS 128u

namespace zen {

enum DetectMode : uint32_t {
    MODE_ELEM = 0, // row_dim == 1: one 16-byte load covers four rows
    MODE_SUB = 1,  // row_dim in {4,8,...,128} with row_dim/4 a power of two: row_dim/4 lanes per row
    MODE_ROW = 2   // anything else: one wave per row (16-byte loads if row_dim % 4 == 0)
};

// Everything the kernels need to know about one (n_rows, row_dim, n_parts, seed) problem.
struct Geometry {
    uint64_t n_rows;
    uint32_t row_dim;
    uint32_t n_parts;
    uint32_t seed;
    uint32_t pow2_mask;      // n_parts-1 if power of two else 0
    uint32_t part_bits;      // ceil(log2(n_parts))
    uint32_t mode;           // DetectMode
    uint32_t tile_rows;      // rows per tile (multiple of 256 / 64 / 32 by mode)
    uint32_t tile_words;     // tile_rows / 32
    uint32_t n_tiles;        // ceil(n_rows / tile_rows)
    uint32_t bitmap;         // 1 = hash-bitmap index format
    uint32_t sparse_mask;    // per-tile flags exist and gate: bit 0 the tile's mask words, bit 1 its histogram row
                             // (empty tiles write neither); 0 = no flags, everything is always written
};

// Per-call encode workspace layout (bytes from the workspace base).
struct EncodeLayout {
    uint64_t status_off;     // zen_status_info
    uint64_t mask_off;       // per worker: n_tiles*tile_words u32
    uint64_t mask_stride;
    uint64_t hist_off;       // per worker: n_tiles*n_parts u32 (tile-major)
    uint64_t hist_stride;
    uint64_t flag_off;       // per worker: n_tiles u32, 1 = the tile has a non-zero row (its mask words and
    uint64_t flag_stride;    //             histogram row exist), 0 = empty tile (nothing else was written)
    uint64_t list_off;       // per worker: 2 * (n_tiles + 1) u32: ascending ids of the flagged tiles, their number (at n_tiles),
                             //             then the listed tiles' flag words
    uint64_t list_stride;
    uint64_t slice_off;      // all workers: per (worker, slice of 256 tiles) n_parts + 1 u32, the sliced partition scan's sums
    uint64_t total;
};

struct GradPtrs { const float *p[ZEN_MAX_BATCH]; };
struct EncodedPtrs {
    uint32_t *offsets[ZEN_MAX_BATCH];
    uint32_t *indices[ZEN_MAX_BATCH];
    float *values[ZEN_MAX_BATCH];
    uint32_t *bitmap[ZEN_MAX_BATCH];
    uint64_t cap_rows[ZEN_MAX_BATCH];
};

template <class T> struct Arr64 { T v[ZEN_MAX_BATCH]; };

// Sources of the aggregation: part (w, server j) = rows [bounds[w][j], bounds[w][j+1]) of
// indices[w] / values[w] (batch form), or rows [0, bounds[w][0]) when `single` is set.
struct PartIdx {
    const uint32_t *indices[ZEN_MAX_BATCH];
    const uint32_t *bounds[ZEN_MAX_BATCH];
    uint32_t single;
    uint32_t server0;   // batch form: first server (partition id) handled by this launch group
    // parts given as hash bitmaps (indices[w] == NULL) are decoded into dec_base[server*dec_stride + ...]
    const uint32_t *dec_base;
    uint64_t dec_stride;
};
struct AggOut {
    uint32_t *indices[ZEN_MAX_BATCH];
    uint32_t *count[ZEN_MAX_BATCH];
    uint64_t cap_rows[ZEN_MAX_BATCH];
};

// Mark in the status block's `reserved` word (low 16 bits; the number of servers in the high 16): the call's flags
// and rows needed are the OR / maximum of the servers' counters (words CNT_FLAGS = 3 and CNT_NEEDED = 4 of the 16
// words per server that follow the 256-byte status region), not the status words themselves.
#define ZEN_STATUS_IN_COUNTERS 0xA66Cu

struct AggLayout {
    uint64_t status_off;     // zen_status_info
    uint64_t counters_off;   // per server: 16 u32 (0: unique count, 1: total rows in)
    uint64_t srctab_off;     // ZEN_MAX_BATCH device pointers: the parts' value arrays
    uint64_t keys_off;       // per server: table_cap u32 keys
    uint64_t rank_off;       // per server: table_cap u32 output rank of the slot's key
    uint64_t uniq_off;       // large path: per server 2 x uniq_cap u32 (ping-pong)
    uint64_t uniq_cap;       // = max_in_rows rounded up
    uint64_t sorthist_off;   // large path: per server sort_blocks x 256 u32
    uint64_t sort_blocks;    // radix-sort blocks per server
    uint64_t rowstart_off;   // large path: per server uniq_cap + 64 u32 contributor-list starts, then (all servers) as many fill
                             // cursors, which are the lists' ends once filled
    uint64_t rowstart_stride;
    uint64_t decode_off;     // bitmap parts: per (server, part) decoded indices
    uint64_t decode_stride;
    uint64_t decflags_off;   // small path: per (server, part) decode consistency flag
    uint64_t bmcnt_off;      // bitmap merge: per server (ZEN_MAX_BATCH+1) x bm_chunks u32
    uint64_t bm_chunks;
    uint64_t bmwave_off;     // element-level bitmap merge: per server bm_chunks x (ZEN_MAX_BATCH+1) x 4 per-wave counts
    uint64_t bmtab_off;      //                              the parts' bitmap pointers [64] and value pointers [64]
    uint64_t table_cap;      // slots per server (power of two)
    uint32_t small_path;     // 1: one block per server sorts in LDS
    uint64_t total;
};

} // namespace zen

namespace zen {
enum KernelId : uint32_t {
    K_DETECT = 0, K_PARTITION_SCAN, K_SCATTER, K_AGG_CLEAR, K_AGG_INSERT, K_AGG_SORT_SMALL, K_AGG_COMPACT,
    K_RS_HIST, K_RS_SCAN, K_RS_SCATTER, K_AGG_FINALIZE, K_AGG_FILL, K_NONZERO_LIST, K_BITMAP_DECODE,
    K_AGG_GATHER, K_BM_COUNT, K_BM_SCAN, K_BM_MERGE, K_ENCODE_SMALL, K_GATHER_ROWS,
    K_PULL_ENCODE, K_PULL_ZERO, K_PULL_COUNT, K_PULL_SCAN, K_PULL_PLACE, K_PULL_PLACE_COO,
    K_HM_CLEAR, K_HM_INSERT, K_HM_EXTRACT, K_STATS,
    K_COUNT
};
struct ProfRecord { hipEvent_t start, stop; uint32_t kernel; };
} // namespace zen

struct zen_ctx {
    zen::Geometry geo;
    // optional per-kernel timing with HIP events on the launch stream
    uint32_t prof_mode;               // 0 off, 1 detect kernel only, 2 every kernel
    zen::ProfRecord *prof;            // pool of event pairs
    uint32_t prof_cap, prof_used;
    zen_index_format fmt;
    int device;
    // hash-bitmap tables (BITMAP contexts only)
    uint32_t *d_domain;        // [n_rows] sorted domains, partition-major
    uint32_t *d_dom_offsets;   // [n_parts+1] start of each domain in d_domain
    uint32_t *d_rank;          // [n_rows] position of every row inside its domain
    uint32_t *d_dom_tile_base; // [n_tiles+1][n_parts] rank of the first row of each tile in each domain
    uint32_t *d_bm_word_off;   // [n_parts+1] first bitmap word of each partition
    uint64_t *h_bm_word_off;   // host copy
    uint64_t *h_dom_sizes;     // host copy
    uint64_t bm_total_words;
    uint64_t max_dom_words;    // largest per-partition bitmap, in words
    uint32_t small_encode;     // 1: few-row encodes take the one-block-per-worker partition path
    uint32_t last_flags;       // what the last zen_status_fetch on this context read (zen_last_overflow)
    uint64_t last_needed_rows;
    uint32_t *d_pull_base;     // element-level BITMAP contexts: [ceil(n_rows/8192)+1][n_parts] rows of II_p below each tile
    uint32_t *d_group_base;    // same at ZEN_GROUP_ROWS granularity: [n_tiles * tile_rows / ZEN_GROUP_ROWS + 1][n_parts]
                               // (element-level BITMAP contexts with few partitions; NULL otherwise)
};

namespace zen {

EncodeLayout encode_layout(const Geometry &g, uint32_t batch);
AggLayout aggregate_layout(const zen_ctx *ctx, uint32_t batch, uint64_t max_in_rows);
uint64_t bitmap_merge_chunks(uint64_t max_dom_words);
hipError_t launch_bitmap_merge(zen_ctx *ctx, const Arr64<const uint32_t *> &bitmaps,
                               const Arr64<const uint32_t *> &bounds, const Arr64<const float *> &src_values,
                               uint32_t n_in, bool single, uint32_t n_servers, uint32_t first_part,
                               const AggOut &outs, const Arr64<float *> &out_values, char *ws, const AggLayout &L,
                               hipStream_t s);

// encode launchers (zen_encode.hip)
// Kernel timing: ProfScope records an event pair around a launch when the context asks for it.
struct ProfScope {
    zen_ctx *ctx; hipStream_t s; ProfRecord *rec;
    ProfScope(zen_ctx *c, uint32_t kernel, hipStream_t st) : ctx(c), s(st), rec(nullptr)
    {
        if (!c || !c->prof_mode || (c->prof_mode == 1 && kernel != K_DETECT) || c->prof_used >= c->prof_cap) return;
        rec = &c->prof[c->prof_used++];
        rec->kernel = kernel;
        (void)hipEventRecord(rec->start, s);
    }
    ~ProfScope() { if (rec) (void)hipEventRecord(rec->stop, s); }
};

hipError_t launch_detect(zen_ctx *ctx, const GradPtrs &grads, uint32_t batch, char *ws,
                         const EncodeLayout &L, bool reset_status, bool want_hist, hipStream_t s,
                         const uint32_t *min_mag = nullptr, bool seg_flags = false);
bool encode_small_applies(const zen_ctx *ctx, const EncodedPtrs &outs, uint32_t batch);
hipError_t launch_encode_small(zen_ctx *ctx, const GradPtrs &grads, const EncodedPtrs &outs, uint32_t batch,
                               char *ws, const EncodeLayout &L, hipStream_t s);
hipError_t launch_partition_scan(zen_ctx *ctx, const EncodedPtrs &outs, uint32_t batch, char *ws,
                                 const EncodeLayout &L, hipStream_t s);
hipError_t launch_scatter(zen_ctx *ctx, const GradPtrs &grads, const EncodedPtrs &outs,
                          uint32_t batch, char *ws, const EncodeLayout &L, hipStream_t s);
hipError_t launch_nonzero_list(zen_ctx *ctx, uint32_t *indices, uint64_t cap_rows, uint32_t *count,
                               char *ws, const EncodeLayout &L, hipStream_t s);
hipError_t build_domain_tables(zen_ctx *ctx, uint32_t *tmp_mask, zen_status_info *tmp_status, hipStream_t s);
hipError_t build_pull_tables(zen_ctx *ctx, hipStream_t s);   // zen_pull.hip
hipError_t launch_gather_rows(zen_ctx *ctx, const GradPtrs &grads, const EncodedPtrs &outs, uint32_t batch,
                              uint64_t max_cap, hipStream_t s);
hipError_t launch_copy(const void *src, void *dst, uint64_t bytes, hipStream_t s);
hipError_t launch_fill_u32(uint32_t *p, uint64_t n, uint32_t v, hipStream_t s);
hipError_t launch_hash_many(const uint32_t *idx, uint64_t count, uint32_t seed, uint32_t *out, hipStream_t s);

// aggregate launchers (zen_aggregate.hip)
hipError_t launch_aggregate(zen_ctx *ctx, const PartIdx &src,
                            const Arr64<const float *> &src_values, const Arr64<const uint32_t *> &src_bitmap,
                            uint32_t n_in, uint32_t n_servers, uint32_t first_part_id, const AggOut &outs,
                            const Arr64<float *> &out_values, uint64_t max_in_rows, char *ws,
                            const AggLayout &L, hipStream_t s);

} // namespace zen
