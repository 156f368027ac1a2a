// The C ABI (include/zen.h): argument checks, workspace layouts and launch sequences.
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>
#include "zen_internal.h"

namespace zen {

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

static bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }

// Tile geometry.  A tile is the unit of one detect / scatter block and of the per-partition
// histogram; sized for ~128 KB of dense data so that every launch has far more blocks than CUs.
static void make_geometry(Geometry &g, uint64_t n_rows, uint32_t row_dim, uint32_t n_parts, uint32_t seed,
                          bool bitmap, uint32_t tile_bytes)
{
    memset(&g, 0, sizeof(g));
    g.n_rows = n_rows;
    g.row_dim = row_dim;
    g.n_parts = n_parts;
    g.seed = seed;
    g.pow2_mask = is_pow2(n_parts) ? n_parts - 1 : 0;
    g.part_bits = 0;
    while ((1u << g.part_bits) < n_parts) ++g.part_bits;
    g.bitmap = bitmap ? 1u : 0u;
    const uint64_t target_bytes = tile_bytes ? tile_bytes : 128 * 1024;   // zen_tuning.tile_bytes, checked by the caller
    if (row_dim == 1) {
        g.mode = MODE_ELEM;
        uint64_t t = 2048;
        while (t * 2 * 4 <= target_bytes && t < 65536) t <<= 1;   // 32768 rows = 128 KB
        while (t > 2048 && n_rows / t < 1024) t >>= 1;   // small tensors: keep >= ~1024 tiles
        g.tile_rows = (uint32_t)t;
    } else if ((row_dim & 3u) == 0 && row_dim <= 128 && is_pow2(row_dim / 4)) {
        g.mode = MODE_SUB;
        uint64_t t = 4 * target_bytes / (4ull * row_dim);   // 512 KB: rows are sparse here, and every tile with a row
                                                            // costs the partition scan and the scatter a fixed amount
        while (t > 64 && n_rows / t < 1024) t >>= 1;
        g.tile_rows = (uint32_t)align_up(t < 64 ? 64 : t, 64);
    } else {
        g.mode = MODE_ROW;
        uint64_t t = target_bytes / (4ull * row_dim);
        g.tile_rows = (uint32_t)align_up(t < 32 ? 32 : t, 32);
        if (g.tile_rows > 2048) g.tile_rows = 2048;
    }
    g.tile_words = g.tile_rows / 32;
    // wave-per-row tiles have one or a few mask words: always written; sub-row tiles keep their (short) histogram rows
    g.sparse_mask = g.mode == MODE_ELEM ? 3u : (g.mode == MODE_SUB ? 1u : 0u);
    g.n_tiles = (uint32_t)((n_rows + g.tile_rows - 1) / g.tile_rows);
}

EncodeLayout encode_layout(const Geometry &g, uint32_t batch)
{
    EncodeLayout L{};
    uint64_t off = 0;
    L.status_off = off; off += 256;
    L.mask_stride = align_up((uint64_t)g.n_tiles * g.tile_words * 4, 256);
    L.mask_off = off; off += L.mask_stride * batch;
    L.hist_stride = align_up((uint64_t)g.n_tiles * g.n_parts * 4, 256);
    L.hist_off = off; off += L.hist_stride * batch;
    L.flag_stride = align_up((uint64_t)g.n_tiles * 4, 256);
    L.flag_off = off; off += L.flag_stride * batch;
    L.list_stride = align_up(2 * ((uint64_t)g.n_tiles + 1) * 4, 256);   // ids, their number, the listed tiles' flag words
    L.list_off = off; off += L.list_stride * batch;
    L.slice_off = off; off += align_up((uint64_t)batch * ((g.n_tiles + 255) / 256) * (g.n_parts + 1) * 4, 256);
    L.total = off;
    return L;
}

} // namespace zen

using namespace zen;

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return ZEN_ERR_DEVICE;    \
    } while (0)

static void prof_release(zen_ctx *ctx);

// ---- zen_encode_static: the encode workspace as a file-scope device array ------------------------
// Every GPU the library runs on holds its own copy of the array at its own address.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address that kernels and copies take is
// looked up once per device, with that device current, and kept here.
static __device__ __align__(256) unsigned char scratch[ZEN_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device d, NULL until looked up

// Address of the calling thread's current device's copy of `scratch` (looked up on first use).
static zen_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return ZEN_ERR_DEVICE;
    if (dev < 0 || dev >= kMaxDevices) return ZEN_ERR_INVALID;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return ZEN_ERR_DEVICE;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return ZEN_OK;
}

// Status of a call made of several launch groups: acc = (first ? 0 : acc) folded with the group's status; after
// the last group the status block takes the folded value.
__global__ void status_fold_kernel(zen_status_info *status, zen_status_info *acc, uint32_t first, uint32_t last)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    zen_status_info a = *status;
    if ((a.reserved & 0xFFFFu) == ZEN_STATUS_IN_COUNTERS) {   // the group's result lies in its servers' counters
        const uint32_t n_servers = a.reserved >> 16, *counters = (const uint32_t *)status + 64;
        for (uint32_t j = 0; j < n_servers && j < ZEN_MAX_BATCH; ++j) {
            a.flags |= counters[j * 16 + 3];
            a.needed_rows = a.needed_rows > counters[j * 16 + 4] ? a.needed_rows : counters[j * 16 + 4];
        }
    }
    if (!first) {
        a.flags |= acc->flags;
        a.needed_rows = a.needed_rows > acc->needed_rows ? a.needed_rows : acc->needed_rows;
    }
    a.reserved = 0;
    *acc = a;
    if (last) *status = a;
}

// the status block of a workspace, copied to the caller's device buffer on the stream
__global__ void status_copy_kernel(const zen_status_info *src, zen_status_info *dst)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src;
}

extern "C" {

const char *zen_status_str(zen_status s)
{
    switch (s) {
    case ZEN_OK: return "ok";
    case ZEN_ERR_INVALID: return "invalid argument";
    case ZEN_ERR_CAPACITY: return "capacity exceeded";
    case ZEN_ERR_NOMEM: return "out of memory / workspace too small";
    case ZEN_ERR_DEVICE: return "HIP call failed";
    }
    return "unknown status";
}

zen_status zen_ctx_create(zen_ctx **out, uint64_t n_rows, uint32_t row_dim, uint32_t n_parts,
                          uint32_t hash_seed, zen_index_format fmt)
{
    return zen_ctx_create_tuned(out, n_rows, row_dim, n_parts, hash_seed, fmt, nullptr);
}

zen_status zen_ctx_create_tuned(zen_ctx **out, uint64_t n_rows, uint32_t row_dim, uint32_t n_parts,
                                uint32_t hash_seed, zen_index_format fmt, const zen_tuning *host_tuning)
{
    if (!out) return ZEN_ERR_INVALID;
    *out = nullptr;
    const uint32_t tile_bytes = host_tuning ? host_tuning->tile_bytes : 0u;
    if (tile_bytes && (tile_bytes < 4096u || tile_bytes > (8u << 20))) return ZEN_ERR_INVALID;
    if (host_tuning && host_tuning->tiled_encode > 1u) return ZEN_ERR_INVALID;
    if (n_rows == 0 || n_rows > 0xFFFFFFFEull || row_dim == 0 || row_dim > (1u << 20) || n_parts == 0 ||
        n_parts > ZEN_MAX_PARTS || (fmt != ZEN_INDEX_COO && fmt != ZEN_INDEX_BITMAP))
        return ZEN_ERR_INVALID;
    zen_ctx *ctx = new (std::nothrow) zen_ctx();
    if (!ctx) return ZEN_ERR_NOMEM;
    memset(ctx, 0, sizeof(*ctx));
    make_geometry(ctx->geo, n_rows, row_dim, n_parts, hash_seed, fmt == ZEN_INDEX_BITMAP, tile_bytes);
    ctx->fmt = fmt;
    ctx->small_encode = !(host_tuning && host_tuning->tiled_encode);   // few-row encodes take the one-block-per-worker path
    if (hipGetDevice(&ctx->device) != hipSuccess) { delete ctx; return ZEN_ERR_DEVICE; }
    {   // zen_encode_static's workspace on this device: found here, so that the call itself has no first-use step
        void *unused = nullptr;
        (void)static_scratch(&unused);
    }
    if (fmt == ZEN_INDEX_BITMAP) {
        // sorted hash domains, per-row ranks and per-tile rank bases, built once on the device
        const Geometry &g = ctx->geo;
        const uint32_t n = g.n_parts;
        uint32_t *tmp_mask = nullptr;
        zen_status_info *tmp_status = nullptr;
        uint32_t *h_off = (uint32_t *)malloc((n + 1) * sizeof(uint32_t));
        uint32_t *h_woff32 = (uint32_t *)malloc((n + 1) * sizeof(uint32_t));
        ctx->h_bm_word_off = (uint64_t *)malloc((n + 1) * sizeof(uint64_t));
        ctx->h_dom_sizes = (uint64_t *)malloc(n * sizeof(uint64_t));
        bool ok = h_off && h_woff32 && ctx->h_bm_word_off && ctx->h_dom_sizes;
        ok = ok && hipMalloc(&ctx->d_domain, n_rows * 4) == hipSuccess;
        ok = ok && hipMalloc(&ctx->d_rank, n_rows * 4) == hipSuccess;
        ok = ok && hipMalloc(&ctx->d_dom_offsets, (n + 1) * 4) == hipSuccess;
        ok = ok && hipMalloc(&ctx->d_bm_word_off, (n + 1) * 4) == hipSuccess;
        ok = ok && hipMalloc(&ctx->d_dom_tile_base, ((uint64_t)g.n_tiles + 1) * n * 4) == hipSuccess;
        ok = ok && hipMalloc(&tmp_mask, ((uint64_t)g.n_tiles * g.tile_words + 3 * (uint64_t)g.n_tiles + 2) * 4) == hipSuccess;   // mask + tile flags + tile list (ids, count, flag words)
        ok = ok && hipMalloc(&tmp_status, 256) == hipSuccess;
        zen_status st = ok ? ZEN_OK : ZEN_ERR_NOMEM;
        if (ok) {
            if (build_domain_tables(ctx, tmp_mask, tmp_status, nullptr) != hipSuccess ||
                hipMemcpy(h_off, ctx->d_dom_offsets, (n + 1) * 4, hipMemcpyDeviceToHost) != hipSuccess ||
                build_pull_tables(ctx, nullptr) != hipSuccess)
                st = ZEN_ERR_DEVICE;
        }
        if (st == ZEN_OK) {
            uint64_t w = 0;
            for (uint32_t p = 0; p < n; ++p) {
                ctx->h_bm_word_off[p] = w;
                h_woff32[p] = (uint32_t)w;
                ctx->h_dom_sizes[p] = h_off[p + 1] - h_off[p];
                w += (ctx->h_dom_sizes[p] + 31) / 32;
                if ((ctx->h_dom_sizes[p] + 31) / 32 > ctx->max_dom_words) ctx->max_dom_words = (ctx->h_dom_sizes[p] + 31) / 32;
            }
            ctx->h_bm_word_off[n] = w;
            h_woff32[n] = (uint32_t)w;
            ctx->bm_total_words = w;
            if (h_off[n] != n_rows) st = ZEN_ERR_DEVICE;
            else if (hipMemcpy(ctx->d_bm_word_off, h_woff32, (n + 1) * 4, hipMemcpyHostToDevice) != hipSuccess)
                st = ZEN_ERR_DEVICE;
        }
        if (tmp_mask) (void)hipFree(tmp_mask);
        if (tmp_status) (void)hipFree(tmp_status);
        free(h_off);
        free(h_woff32);
        if (st != ZEN_OK) { zen_ctx_destroy(ctx); return st; }
    }
    *out = ctx;
    return ZEN_OK;
}

zen_status zen_ctx_destroy(zen_ctx *ctx)
{
    if (!ctx) return ZEN_OK;
    prof_release(ctx);
    if (ctx->d_domain) (void)hipFree(ctx->d_domain);
    if (ctx->d_rank) (void)hipFree(ctx->d_rank);
    if (ctx->d_dom_offsets) (void)hipFree(ctx->d_dom_offsets);
    if (ctx->d_dom_tile_base) (void)hipFree(ctx->d_dom_tile_base);
    if (ctx->d_bm_word_off) (void)hipFree(ctx->d_bm_word_off);
    if (ctx->d_pull_base) (void)hipFree(ctx->d_pull_base);
    if (ctx->d_group_base) (void)hipFree(ctx->d_group_base);
    free(ctx->h_bm_word_off);
    free(ctx->h_dom_sizes);
    delete ctx;
    return ZEN_OK;
}

zen_status zen_bitmap_layout(const zen_ctx *ctx, uint64_t *host_total_words, uint64_t *host_word_offsets,
                             uint64_t *host_domain_sizes)
{
    if (!ctx || ctx->fmt != ZEN_INDEX_BITMAP) return ZEN_ERR_INVALID;
    if (host_total_words) *host_total_words = ctx->bm_total_words;
    if (host_word_offsets) memcpy(host_word_offsets, ctx->h_bm_word_off, (ctx->geo.n_parts + 1) * sizeof(uint64_t));
    if (host_domain_sizes) memcpy(host_domain_sizes, ctx->h_dom_sizes, ctx->geo.n_parts * sizeof(uint64_t));
    return ZEN_OK;
}

zen_status zen_encode_workspace_bytes(const zen_ctx *ctx, uint32_t batch, uint64_t *host_bytes)
{
    if (!ctx || !host_bytes || batch == 0) return ZEN_ERR_INVALID;
    const uint32_t b = batch > ZEN_MAX_BATCH ? ZEN_MAX_BATCH : batch;
    *host_bytes = encode_layout(ctx->geo, b).total;
    return ZEN_OK;
}

zen_status zen_aggregate_workspace_bytes(const zen_ctx *ctx, uint32_t batch, uint64_t max_in_rows,
                                         uint64_t *host_bytes)
{
    if (!ctx || !host_bytes || batch == 0 || max_in_rows > 0x7FFFFFFFull) return ZEN_ERR_INVALID;
    const uint32_t b = batch > ZEN_MAX_BATCH ? ZEN_MAX_BATCH : batch;
    *host_bytes = aggregate_layout(ctx, b, max_in_rows).total;
    return ZEN_OK;
}

zen_status zen_workspace_bytes(const zen_ctx *ctx, uint64_t max_nnz, uint32_t batch, uint64_t *host_enc_bytes,
                               uint64_t *host_agg_bytes)
{
    if (!ctx || batch == 0 || (!host_enc_bytes && !host_agg_bytes)) return ZEN_ERR_INVALID;
    if (host_enc_bytes) {
        const zen_status st = zen_encode_workspace_bytes(ctx, batch, host_enc_bytes);
        if (st != ZEN_OK) return st;
    }
    if (host_agg_bytes) return zen_aggregate_workspace_bytes(ctx, batch, max_nnz, host_agg_bytes);
    return ZEN_OK;
}

static zen_status check_encoded(const zen_ctx *ctx, const zen_encoded &e)
{
    if (!e.offsets || !e.values) return ZEN_ERR_INVALID;
    if (ctx->fmt == ZEN_INDEX_COO && !e.indices) return ZEN_ERR_INVALID;
    if (ctx->fmt == ZEN_INDEX_BITMAP && !e.bitmap) return ZEN_ERR_INVALID;
    if (((uintptr_t)e.values & 15u) || ((uintptr_t)e.offsets & 3u) || ((uintptr_t)e.indices & 3u) ||
        ((uintptr_t)e.bitmap & 3u))
        return ZEN_ERR_INVALID;
    if (e.cap_rows > 0xFFFFFFFEull) return ZEN_ERR_INVALID;
    return ZEN_OK;
}

static zen_status encode_batch_impl(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                                    const uint32_t *thresholds, const zen_encoded *host_outs, void *workspace,
                                    uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !host_grads || !host_outs || n_workers == 0 || !workspace) return ZEN_ERR_INVALID;
    if (thresholds && (ctx->geo.row_dim != 1 || ((uintptr_t)thresholds & 3u))) return ZEN_ERR_INVALID;
    if ((uintptr_t)workspace & 255u) return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    for (uint32_t w = 0; w < n_workers; ++w) {
        if (!host_grads[w] || ((uintptr_t)host_grads[w] & 15u)) return ZEN_ERR_INVALID;
        zen_status st = check_encoded(ctx, host_outs[w]);
        if (st != ZEN_OK) return st;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    const uint32_t group = n_workers < ZEN_MAX_BATCH ? n_workers : ZEN_MAX_BATCH;
    const EncodeLayout L = encode_layout(g, group);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    char *ws = (char *)workspace;
    for (uint32_t w0 = 0; w0 < n_workers; w0 += group) {
        const uint32_t nb = n_workers - w0 < group ? n_workers - w0 : group;
        GradPtrs grads;
        EncodedPtrs outs;
        memset(&grads, 0, sizeof(grads));
        memset(&outs, 0, sizeof(outs));
        for (uint32_t i = 0; i < nb; ++i) {
            grads.p[i] = host_grads[w0 + i];
            outs.offsets[i] = host_outs[w0 + i].offsets;
            outs.indices[i] = host_outs[w0 + i].indices;
            outs.values[i] = host_outs[w0 + i].values;
            outs.bitmap[i] = host_outs[w0 + i].bitmap;
            outs.cap_rows[i] = host_outs[w0 + i].cap_rows;
        }
        const uint32_t *thr = thresholds ? thresholds + w0 : nullptr;
        if (encode_small_applies(ctx, outs, nb)) {
            HIP_TRY(launch_detect(ctx, grads, nb, ws, L, w0 == 0, false, s, thr));
            HIP_TRY(launch_encode_small(ctx, grads, outs, nb, ws, L, s));
        } else {
            HIP_TRY(launch_detect(ctx, grads, nb, ws, L, w0 == 0, true, s, thr, true));   // masks by segment: the scatter reads them through the flag words
            HIP_TRY(launch_partition_scan(ctx, outs, nb, ws, L, s));
            HIP_TRY(launch_scatter(ctx, grads, outs, nb, ws, L, s));
        }
    }
    return ZEN_OK;
}

zen_status zen_encode_batch(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                            const zen_encoded *host_outs, void *workspace, uint64_t workspace_bytes,
                            void *hip_stream)
{
    return encode_batch_impl(ctx, host_grads, n_workers, nullptr, host_outs, workspace, workspace_bytes, hip_stream);
}

zen_status zen_encode_batch_sparsified(zen_ctx *ctx, const float *const *host_grads, uint32_t n_workers,
                                       const uint32_t *thresholds, const zen_encoded *host_outs, void *workspace,
                                       uint64_t workspace_bytes, void *hip_stream)
{
    if (!thresholds) return ZEN_ERR_INVALID;
    return encode_batch_impl(ctx, host_grads, n_workers, thresholds, host_outs, workspace, workspace_bytes, hip_stream);
}

zen_status zen_encode(zen_ctx *ctx, const float *grad, uint32_t n_parts, uint32_t hash_seed,
                      const zen_encoded *host_out, void *workspace, uint64_t workspace_bytes,
                      void *hip_stream)
{
    if (!ctx || !host_out) return ZEN_ERR_INVALID;
    if (n_parts != ctx->geo.n_parts || hash_seed != ctx->geo.seed) return ZEN_ERR_INVALID;
    const float *grads[1] = {grad};
    return zen_encode_batch(ctx, grads, 1, host_out, workspace, workspace_bytes, hip_stream);
}

zen_status zen_encode_static(zen_ctx *ctx, const float *grad, uint32_t n_parts, uint32_t hash_seed,
                             const zen_encoded *host_out, zen_status_info *status, void *hip_stream)
{
    if (!ctx || !host_out) return ZEN_ERR_INVALID;
    if (n_parts != ctx->geo.n_parts || hash_seed != ctx->geo.seed) return ZEN_ERR_INVALID;
    if ((uintptr_t)status & 15u) return ZEN_ERR_INVALID;
    if (encode_layout(ctx->geo, 1).total > (uint64_t)ZEN_STATIC_SCRATCH_BYTES) return ZEN_ERR_NOMEM;   // beyond the array
    void *ws = nullptr;
    const zen_status st = static_scratch(&ws);
    if (st != ZEN_OK) return st;
    const float *grads[1] = {grad};
    const zen_status r = encode_batch_impl(ctx, grads, 1, nullptr, host_out, ws, ZEN_STATIC_SCRATCH_BYTES, hip_stream);
    if (r != ZEN_OK || !status) return r;
    status_copy_kernel<<<1, 64, 0, (hipStream_t)hip_stream>>>((const zen_status_info *)ws, status);
    HIP_TRY(hipGetLastError());
    return ZEN_OK;
}

zen_status zen_nonzero(zen_ctx *ctx, const float *grad, uint32_t *indices, uint64_t cap_rows,
                       uint32_t *count, void *workspace, uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !grad || !indices || !count || !workspace) return ZEN_ERR_INVALID;
    if (((uintptr_t)grad & 15u) || ((uintptr_t)workspace & 255u) || cap_rows > 0xFFFFFFFEull) return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    const EncodeLayout L = encode_layout(g, 1);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    GradPtrs grads;
    memset(&grads, 0, sizeof(grads));
    grads.p[0] = grad;
    HIP_TRY(launch_detect(ctx, grads, 1, ws, L, true, true, s));
    HIP_TRY(launch_nonzero_list(ctx, indices, cap_rows, count, ws, L, s));
    return ZEN_OK;
}

static zen_status run_aggregate(zen_ctx *ctx, PartIdx src, const Arr64<const float *> &src_values,
                                const Arr64<const uint32_t *> &src_bitmap, uint32_t n_in, uint32_t n_servers,
                                uint32_t first_part, const AggOut &outs, const Arr64<float *> &out_values,
                                uint64_t max_in_rows, char *ws, const AggLayout &L, hipStream_t s)
{
    src.dec_base = L.decode_stride ? (const uint32_t *)(ws + L.decode_off) : nullptr;
    src.dec_stride = L.decode_stride;
    HIP_TRY(launch_aggregate(ctx, src, src_values, src_bitmap, n_in, n_servers, first_part, outs,
                             out_values, max_in_rows, ws, L, s));
    return ZEN_OK;
}

zen_status zen_aggregate(zen_ctx *ctx, const zen_part *host_parts, uint32_t n_in, uint32_t part_id,
                         uint32_t *out_indices, float *out_values, uint64_t out_cap_rows,
                         uint32_t *out_count, uint64_t max_in_rows, void *workspace,
                         uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || (!host_parts && n_in) || !out_indices || !out_values || !out_count || !workspace)
        return ZEN_ERR_INVALID;
    if (n_in > ZEN_MAX_BATCH || part_id >= ctx->geo.n_parts || max_in_rows > 0x7FFFFFFFull ||
        out_cap_rows > 0xFFFFFFFEull)
        return ZEN_ERR_INVALID;
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)out_values & 15u)) return ZEN_ERR_INVALID;
    PartIdx src;
    Arr64<const float *> sv;
    Arr64<const uint32_t *> sb;
    memset(&src, 0, sizeof(src));
    memset(&sv, 0, sizeof(sv));
    memset(&sb, 0, sizeof(sb));
    src.single = 1;
    bool any_bitmap = false;
    for (uint32_t w = 0; w < n_in; ++w) {
        const zen_part &p = host_parts[w];
        if (!p.count || !p.values || (!p.indices && !p.bitmap)) return ZEN_ERR_INVALID;
        if ((uintptr_t)p.values & 15u) return ZEN_ERR_INVALID;
        if (p.bitmap && !p.indices) any_bitmap = true;
        src.indices[w] = p.indices;
        src.bounds[w] = p.count;
        sv.v[w] = p.values;
        sb.v[w] = p.indices ? nullptr : p.bitmap;
    }
    if (any_bitmap && ctx->fmt != ZEN_INDEX_BITMAP) return ZEN_ERR_INVALID;   // no domain tables
    const AggLayout L = aggregate_layout(ctx, 1, max_in_rows);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    AggOut outs;
    Arr64<float *> ov;
    memset(&outs, 0, sizeof(outs));
    memset(&ov, 0, sizeof(ov));
    outs.indices[0] = out_indices;
    outs.count[0] = out_count;
    outs.cap_rows[0] = out_cap_rows;
    ov.v[0] = out_values;
    return run_aggregate(ctx, src, sv, sb, n_in, 1, part_id, outs, ov, max_in_rows, (char *)workspace, L,
                         (hipStream_t)hip_stream);
}

zen_status zen_aggregate_batch(zen_ctx *ctx, const zen_encoded *host_encs, uint32_t n_workers,
                               const zen_aggregated *host_outs, uint64_t max_in_rows, void *workspace,
                               uint64_t workspace_bytes, void *hip_stream)
{
    if (!ctx || !host_encs || !host_outs || n_workers == 0 || !workspace) return ZEN_ERR_INVALID;
    if (n_workers > ZEN_MAX_BATCH || max_in_rows > 0x7FFFFFFFull || ((uintptr_t)workspace & 255u))
        return ZEN_ERR_INVALID;
    const Geometry &g = ctx->geo;
    PartIdx src;
    Arr64<const float *> sv;
    Arr64<const uint32_t *> sb;
    memset(&src, 0, sizeof(src));
    memset(&sv, 0, sizeof(sv));
    memset(&sb, 0, sizeof(sb));
    for (uint32_t w = 0; w < n_workers; ++w) {
        zen_status st = check_encoded(ctx, host_encs[w]);
        if (st != ZEN_OK) return st;
        src.indices[w] = ctx->fmt == ZEN_INDEX_BITMAP ? nullptr : host_encs[w].indices;   // BITMAP: decode
        src.bounds[w] = host_encs[w].offsets;
        sv.v[w] = host_encs[w].values;
        sb.v[w] = host_encs[w].bitmap;
    }
    for (uint32_t j = 0; j < g.n_parts; ++j) {
        const zen_aggregated &o = host_outs[j];
        if (!o.indices || !o.values || !o.count || ((uintptr_t)o.values & 15u) || o.cap_rows > 0xFFFFFFFEull)
            return ZEN_ERR_INVALID;
    }
    const uint32_t group = g.n_parts < ZEN_MAX_BATCH ? g.n_parts : ZEN_MAX_BATCH;
    const AggLayout L = aggregate_layout(ctx, group, max_in_rows);
    if (workspace_bytes < L.total) return ZEN_ERR_NOMEM;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    src.single = 0;
    // Servers in launch groups of ZEN_MAX_BATCH.  Every group's kernels write the status block anew, so with
    // more than one group the blocks are folded (OR of the flags, maximum of the rows needed) in the spare
    // words behind the status block and the result is put in its place after the last group.
    zen_status_info *status = (zen_status_info *)(ws + L.status_off), *folded = status + 2;
    const bool several = g.n_parts > group;
    for (uint32_t j0 = 0; j0 < g.n_parts; j0 += group) {
        const uint32_t nb = g.n_parts - j0 < group ? g.n_parts - j0 : group;
        AggOut outs;
        Arr64<float *> ov;
        memset(&outs, 0, sizeof(outs));
        memset(&ov, 0, sizeof(ov));
        for (uint32_t j = 0; j < nb; ++j) {
            outs.indices[j] = host_outs[j0 + j].indices;
            outs.count[j] = host_outs[j0 + j].count;
            outs.cap_rows[j] = host_outs[j0 + j].cap_rows;
            ov.v[j] = host_outs[j0 + j].values;
        }
        src.server0 = j0;
        const zen_status st = run_aggregate(ctx, src, sv, sb, n_workers, nb, j0, outs, ov, max_in_rows, ws, L, s);
        if (st != ZEN_OK) return st;
        if (several) {
            status_fold_kernel<<<1, 64, 0, s>>>(status, folded, j0 == 0 ? 1u : 0u, j0 + nb >= g.n_parts ? 1u : 0u);
            HIP_TRY(hipGetLastError());
        }
    }
    return ZEN_OK;
}

zen_status zen_status_fetch(zen_ctx *ctx, const void *workspace, void *hip_stream, zen_status_info *host_info)
{
    if (!ctx || !workspace) return ZEN_ERR_INVALID;
    zen_status_info info;
    hipStream_t s = (hipStream_t)hip_stream;
    HIP_TRY(hipMemcpyAsync(&info, workspace, sizeof(info), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if ((info.reserved & 0xFFFFu) == ZEN_STATUS_IN_COUNTERS) {
        // the one-launch aggregate leaves every server's result in its counters: fold them here
        const uint32_t n_servers = info.reserved >> 16;
        uint32_t counters[ZEN_MAX_BATCH * 16];
        if (n_servers == 0 || n_servers > ZEN_MAX_BATCH) return ZEN_ERR_DEVICE;
        HIP_TRY(hipMemcpyAsync(counters, (const char *)workspace + 256, (size_t)n_servers * 16 * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        info.reserved = 0;
        for (uint32_t j = 0; j < n_servers; ++j) {
            info.flags |= counters[j * 16 + 3];
            if (counters[j * 16 + 4] > info.needed_rows) info.needed_rows = counters[j * 16 + 4];
        }
    }
    if (host_info) *host_info = info;
    ctx->last_flags = info.flags;
    ctx->last_needed_rows = info.needed_rows;
    return (info.flags & 3u) ? ZEN_ERR_CAPACITY : (info.flags ? ZEN_ERR_INVALID : ZEN_OK);
}

zen_status zen_last_overflow(const zen_ctx *ctx, uint64_t *host_needed_rows)
{
    if (!ctx || !host_needed_rows) return ZEN_ERR_INVALID;
    *host_needed_rows = (ctx->last_flags & 3u) ? ctx->last_needed_rows : 0;
    return ZEN_OK;
}

static const char *const kKernelNames[K_COUNT] = {
    "detect_kernel", "partition_scan_kernel", "scatter_kernel", "agg_clear_kernel", "agg_insert_kernel",
    "agg_small_kernel", "agg_compact_kernel", "rs_hist_kernel", "rs_scan_kernel", "rs_scatter_kernel",
    "agg_finalize_kernel", "agg_fill_kernel", "nonzero_list_kernels", "bitmap_decode_kernel",
    "agg_gather_kernel", "bm_count_kernel", "bm_scan_kernel", "bm_merge_kernel", "encode_small_kernel", "gather_rows_kernel",
    "pull_encode_kernel", "pull_zero_kernel", "pull_count_kernel", "pull_scan_kernel", "pull_place_kernel",
    "pull_place_coo_kernel", "hm_clear_kernel", "hm_insert_kernel", "hm_extract_kernels",
    "stats_kernel"};

static void prof_release(zen_ctx *ctx)
{
    for (uint32_t i = 0; i < ctx->prof_cap; ++i) {
        (void)hipEventDestroy(ctx->prof[i].start);
        (void)hipEventDestroy(ctx->prof[i].stop);
    }
    free(ctx->prof);
    ctx->prof = nullptr;
    ctx->prof_cap = ctx->prof_used = 0;
    ctx->prof_mode = 0;
}

zen_status zen_profile_enable(zen_ctx *ctx, uint32_t mode, uint32_t max_records)
{
    if (!ctx || mode > 2) return ZEN_ERR_INVALID;
    prof_release(ctx);
    if (mode == 0) return ZEN_OK;
    if (max_records == 0 || max_records > (1u << 20)) return ZEN_ERR_INVALID;
    ctx->prof = (ProfRecord *)calloc(max_records, sizeof(ProfRecord));
    if (!ctx->prof) return ZEN_ERR_NOMEM;
    for (uint32_t i = 0; i < max_records; ++i) {
        if (hipEventCreate(&ctx->prof[i].start) != hipSuccess || hipEventCreate(&ctx->prof[i].stop) != hipSuccess) {
            ctx->prof_cap = i;
            prof_release(ctx);
            return ZEN_ERR_DEVICE;
        }
        ctx->prof_cap = i + 1;
    }
    ctx->prof_mode = mode;
    return ZEN_OK;
}

zen_status zen_profile_collect(zen_ctx *ctx, uint32_t cap, double *host_ms_sum, uint32_t *host_launches,
                               uint32_t *host_n_kernels)
{
    if (!ctx || !host_ms_sum || !host_launches || cap < K_COUNT) return ZEN_ERR_INVALID;
    for (uint32_t k = 0; k < K_COUNT; ++k) { host_ms_sum[k] = 0.0; host_launches[k] = 0; }
    for (uint32_t i = 0; i < ctx->prof_used; ++i) {
        float ms = 0.f;
        HIP_TRY(hipEventSynchronize(ctx->prof[i].stop));
        HIP_TRY(hipEventElapsedTime(&ms, ctx->prof[i].start, ctx->prof[i].stop));
        host_ms_sum[ctx->prof[i].kernel] += ms;
        host_launches[ctx->prof[i].kernel] += 1;
    }
    ctx->prof_used = 0;
    if (host_n_kernels) *host_n_kernels = K_COUNT;
    return ZEN_OK;
}

const char *zen_profile_kernel_name(uint32_t kernel)
{
    return kernel < K_COUNT ? kKernelNames[kernel] : "";
}

zen_status zen_calibration_copy(const void *src, void *dst, uint64_t bytes, void *hip_stream)
{
    if (!src || !dst || (bytes & 15u) || ((uintptr_t)src & 15u) || ((uintptr_t)dst & 15u)) return ZEN_ERR_INVALID;
    HIP_TRY(launch_copy(src, dst, bytes, (hipStream_t)hip_stream));
    return ZEN_OK;
}

zen_status zen_hash_many(const uint32_t *idx, uint64_t count, uint32_t seed, uint32_t *out, void *hip_stream)
{
    if (count && (!idx || !out)) return ZEN_ERR_INVALID;
    HIP_TRY(launch_hash_many(idx, count, seed, out, (hipStream_t)hip_stream));
    return ZEN_OK;
}

} // extern "C"
