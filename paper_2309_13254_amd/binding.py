"""ctypes binding of include/zen.h: argument marshalling only.

The functions carry the C names.  Tensors are torch CUDA(ROCm) tensors used purely as device
buffers; the HIP stream is torch's current stream unless one is given.  There is no CPU fallback:
loading fails loudly if the HIP library has not been built (`python -m paper_2309_13254_amd.build`).
"""
import ctypes as C
import os

import torch

__all__ = [
    "ZEN_OK", "ZEN_ERR_INVALID", "ZEN_ERR_CAPACITY", "ZEN_ERR_NOMEM", "ZEN_ERR_DEVICE",
    "ZEN_INDEX_COO", "ZEN_INDEX_BITMAP", "ZEN_MAX_BATCH", "ZEN_MAX_PARTS",
    "ZenError", "ZenContext", "Encoded", "Aggregated", "library_path", "load_library",
    "zen_ctx_create", "zen_ctx_create_tuned", "zen_ctx_destroy", "zen_bitmap_layout", "zen_encode_workspace_bytes",
    "zen_workspace_bytes", "zen_last_overflow",
    "zen_aggregate_workspace_bytes", "zen_encode", "zen_encode_static", "ZEN_STATIC_SCRATCH_BYTES", "zen_encode_batch", "zen_nonzero", "zen_aggregate",
    "zen_aggregate_batch", "zen_status_fetch", "zen_hash_many", "zen_status_str",
    "zen_calibration_copy", "zen_calibration_read", "zen_profile_enable", "zen_profile_collect", "zen_profile_kernel_name",
    "zen_pull_workspace_bytes", "zen_pull_encode", "zen_pull_encode_batch", "zen_pull_decode", "zen_pull_apply",
    "zen_hash_memory_bytes", "zen_encode_hashed_workspace_bytes", "zen_encode_hashed",
    "zen_sparsity_count", "zen_scheme_times", "zen_topk_workspace_bytes", "zen_topk_threshold",
    "zen_encode_batch_sparsified", "zen_format_count", "zen_format_bytes",
    "alloc_encoded", "alloc_aggregated", "alloc_workspace",
]

ZEN_OK, ZEN_ERR_INVALID, ZEN_ERR_CAPACITY, ZEN_ERR_NOMEM, ZEN_ERR_DEVICE = 0, 1, 2, 3, 4
ZEN_INDEX_COO, ZEN_INDEX_BITMAP = 0, 1
ZEN_MAX_BATCH, ZEN_MAX_PARTS = 64, 1024
ZEN_STATIC_SCRATCH_BYTES = 8 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libzen_hip.so")
_lib = None


class ZenError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, zen_status_str(status), status))


class _Encoded(C.Structure):
    _fields_ = [("offsets", C.c_void_p), ("indices", C.c_void_p), ("values", C.c_void_p),
                ("bitmap", C.c_void_p), ("cap_rows", C.c_uint64)]


class _Part(C.Structure):
    _fields_ = [("indices", C.c_void_p), ("bitmap", C.c_void_p), ("values", C.c_void_p), ("count", C.c_void_p)]


class _Aggregated(C.Structure):
    _fields_ = [("indices", C.c_void_p), ("values", C.c_void_p), ("count", C.c_void_p), ("cap_rows", C.c_uint64)]


class _HashParams(C.Structure):
    _fields_ = [("k", C.c_uint32), ("level2_seed", C.c_uint32), ("r1", C.c_uint64), ("r2", C.c_uint64)]


class _SparsityCounts(C.Structure):
    _fields_ = [("nnz", C.c_void_p), ("union_prefix", C.c_void_p), ("overlap", C.c_void_p), ("even_split", C.c_void_p)]


class _Tuning(C.Structure):
    _fields_ = [("tile_bytes", C.c_uint32), ("tiled_encode", C.c_uint32)]


class _ReadShape(C.Structure):
    _fields_ = [("threads", C.c_uint32), ("unroll", C.c_uint32), ("block_bytes", C.c_uint32), ("max_blocks", C.c_uint32),
                ("nontemporal", C.c_uint32)]


class _StatusInfo(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("reserved", C.c_uint32), ("needed_rows", C.c_uint64)]


def library_path():
    return _SO


def load_library():
    """Load the C-ABI library; raises if it has not been built (no fallback of any kind)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_SO):
        raise ImportError("HIP library %s is missing: run `python -m paper_2309_13254_amd.build`" % _SO)
    L = C.CDLL(_SO)
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    sig = {
        "zen_ctx_create": [C.POINTER(vp), u64, u32, u32, u32, C.c_int],
        "zen_ctx_create_tuned": [C.POINTER(vp), u64, u32, u32, u32, C.c_int, C.POINTER(_Tuning)],
        "zen_ctx_destroy": [vp],
        "zen_workspace_bytes": [vp, u64, u32, C.POINTER(u64), C.POINTER(u64)],
        "zen_last_overflow": [vp, C.POINTER(u64)],
        "zen_bitmap_layout": [vp, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64)],
        "zen_encode_workspace_bytes": [vp, u32, C.POINTER(u64)],
        "zen_aggregate_workspace_bytes": [vp, u32, u64, C.POINTER(u64)],
        "zen_encode": [vp, vp, u32, u32, C.POINTER(_Encoded), vp, u64, vp],
        "zen_encode_static": [vp, vp, u32, u32, C.POINTER(_Encoded), vp, vp],
        "zen_encode_batch": [vp, C.POINTER(vp), u32, C.POINTER(_Encoded), vp, u64, vp],
        "zen_nonzero": [vp, vp, vp, u64, vp, vp, u64, vp],
        "zen_aggregate": [vp, C.POINTER(_Part), u32, u32, vp, vp, u64, vp, u64, vp, u64, vp],
        "zen_aggregate_batch": [vp, C.POINTER(_Encoded), u32, C.POINTER(_Aggregated), u64, vp, u64, vp],
        "zen_status_fetch": [vp, vp, vp, C.POINTER(_StatusInfo)],
        "zen_hash_many": [vp, u64, u32, vp, vp],
        "zen_calibration_copy": [vp, vp, u64, vp],
        "zen_calibration_read": [vp, u64, C.POINTER(_ReadShape), vp, vp],
        "zen_pull_workspace_bytes": [vp, C.POINTER(u64)],
        "zen_pull_encode": [vp, vp, vp, u64, u32, vp, vp, u64, vp],
        "zen_pull_encode_batch": [vp, C.POINTER(_Aggregated), vp, vp, u64, vp],
        "zen_pull_decode": [vp, vp, u32, vp, u64, vp, vp, u64, vp],
        "zen_pull_apply": [vp, C.POINTER(_Part), vp, vp, u64, vp],
        "zen_hash_memory_bytes": [vp, C.POINTER(_HashParams), C.POINTER(u64)],
        "zen_encode_hashed_workspace_bytes": [vp, C.POINTER(_HashParams), C.POINTER(u64)],
        "zen_encode_hashed": [vp, vp, C.POINTER(_HashParams), vp, u64, C.POINTER(_Encoded), vp, vp, u64, vp],
        "zen_sparsity_count": [vp, C.POINTER(vp), u32, C.POINTER(_SparsityCounts), vp, u64, vp],
        "zen_scheme_times": [u32, C.POINTER(C.c_double), C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double),
                             C.POINTER(C.c_double)],
        "zen_topk_workspace_bytes": [C.POINTER(u64)],
        "zen_topk_threshold": [vp, u64, u64, u64, u64, vp, vp, u64, vp],
        "zen_encode_batch_sparsified": [vp, C.POINTER(vp), u32, vp, C.POINTER(_Encoded), vp, u64, vp],
        "zen_format_count": [vp, vp, u32, vp, vp, u64, vp],
        "zen_format_bytes": [u64, u64, u32, u64, u32, C.POINTER(C.c_double)],
        "zen_profile_enable": [vp, u32, u32],
        "zen_profile_collect": [vp, u32, C.POINTER(C.c_double), C.POINTER(u32), C.POINTER(u32)],
    }
    for name, args in sig.items():
        f = getattr(L, name)
        f.argtypes = args
        f.restype = C.c_int
    L.zen_profile_kernel_name.argtypes = [u32]
    L.zen_profile_kernel_name.restype = C.c_char_p
    L.zen_status_str.argtypes = [C.c_int]
    L.zen_status_str.restype = C.c_char_p
    _lib = L
    return L


def zen_status_str(status):
    try:
        return load_library().zen_status_str(int(status)).decode()
    except ImportError:
        return "status %d" % status


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _check(status, where, allow=()):
    if status != ZEN_OK and status not in allow:
        raise ZenError(status, where)
    return status


class ZenContext:
    """Owns a zen_ctx*: immutable function of (n_rows, row_dim, n_parts, hash_seed, fmt)."""

    def __init__(self, n_rows, row_dim, n_parts, hash_seed, fmt=ZEN_INDEX_COO, tile_bytes=0, tiled_encode=False):
        self.n_rows, self.row_dim, self.n_parts = int(n_rows), int(row_dim), int(n_parts)
        self.hash_seed, self.fmt = int(hash_seed) & 0xFFFFFFFF, int(fmt)
        h = C.c_void_p()
        if tile_bytes or tiled_encode:
            tun = _Tuning(int(tile_bytes), 1 if tiled_encode else 0)
            _check(load_library().zen_ctx_create_tuned(C.byref(h), self.n_rows, self.row_dim, self.n_parts,
                                                       self.hash_seed, self.fmt, C.byref(tun)), "zen_ctx_create_tuned")
        else:
            _check(load_library().zen_ctx_create(C.byref(h), self.n_rows, self.row_dim, self.n_parts,
                                                 self.hash_seed, self.fmt), "zen_ctx_create")
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            load_library().zen_ctx_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def zen_ctx_create(n_rows, row_dim, n_parts, hash_seed, fmt=ZEN_INDEX_COO):
    return ZenContext(n_rows, row_dim, n_parts, hash_seed, fmt)


def zen_ctx_create_tuned(n_rows, row_dim, n_parts, hash_seed, fmt=ZEN_INDEX_COO, tile_bytes=0, tiled_encode=False):
    return ZenContext(n_rows, row_dim, n_parts, hash_seed, fmt, tile_bytes=tile_bytes, tiled_encode=tiled_encode)


def zen_ctx_destroy(ctx):
    ctx.close()


def zen_bitmap_layout(ctx):
    """-> (total_words, word_offsets[n+1], domain_sizes[n]) as Python ints / lists."""
    n = ctx.n_parts
    total = C.c_uint64()
    woff = (C.c_uint64 * (n + 1))()
    dsz = (C.c_uint64 * n)()
    _check(load_library().zen_bitmap_layout(ctx.handle, C.byref(total), woff, dsz), "zen_bitmap_layout")
    return int(total.value), list(woff), list(dsz)


def zen_encode_workspace_bytes(ctx, batch):
    b = C.c_uint64()
    _check(load_library().zen_encode_workspace_bytes(ctx.handle, int(batch), C.byref(b)), "zen_encode_workspace_bytes")
    return int(b.value)


def zen_aggregate_workspace_bytes(ctx, batch, max_in_rows):
    b = C.c_uint64()
    _check(load_library().zen_aggregate_workspace_bytes(ctx.handle, int(batch), int(max_in_rows), C.byref(b)),
           "zen_aggregate_workspace_bytes")
    return int(b.value)


def zen_workspace_bytes(ctx, max_nnz, batch):
    """-> (encode workspace bytes, aggregate workspace bytes) for `batch` workers / servers."""
    e, a = C.c_uint64(), C.c_uint64()
    _check(load_library().zen_workspace_bytes(ctx.handle, int(max_nnz), int(batch), C.byref(e), C.byref(a)),
           "zen_workspace_bytes")
    return int(e.value), int(a.value)


def zen_last_overflow(ctx):
    """-> rows needed by the largest overflow the last zen_status_fetch on this context reported (0: none)."""
    n = C.c_uint64()
    _check(load_library().zen_last_overflow(ctx.handle, C.byref(n)), "zen_last_overflow")
    return int(n.value)


class Encoded:
    """Device buffers of one encoded gradient (a zen_encoded)."""

    def __init__(self, offsets, indices, values, bitmap, cap_rows):
        self.offsets, self.indices, self.values, self.bitmap, self.cap_rows = offsets, indices, values, bitmap, int(cap_rows)

    def struct(self):
        return _Encoded(_ptr(self.offsets), _ptr(self.indices), _ptr(self.values), _ptr(self.bitmap), self.cap_rows)


class Aggregated:
    """Device buffers of one server's aggregated partition (a zen_aggregated)."""

    def __init__(self, indices, values, count, cap_rows):
        self.indices, self.values, self.count, self.cap_rows = indices, values, count, int(cap_rows)

    def struct(self):
        return _Aggregated(_ptr(self.indices), _ptr(self.values), _ptr(self.count), self.cap_rows)


def alloc_encoded(ctx, cap_rows, device="cuda", with_indices=True):
    cap = max(int(cap_rows), 1)
    offsets = torch.empty(ctx.n_parts + 1, dtype=torch.int32, device=device)
    indices = torch.empty(cap, dtype=torch.int32, device=device) if (with_indices or ctx.fmt == ZEN_INDEX_COO) else None
    values = torch.empty((cap, ctx.row_dim), dtype=torch.float32, device=device)
    bitmap = None
    if ctx.fmt == ZEN_INDEX_BITMAP:
        total, _, _ = zen_bitmap_layout(ctx)
        bitmap = torch.empty(max(total, 1), dtype=torch.int32, device=device)
    return Encoded(offsets, indices, values, bitmap, int(cap_rows))


def alloc_aggregated(ctx, cap_rows, device="cuda"):
    cap = max(int(cap_rows), 1)
    return Aggregated(torch.empty(cap, dtype=torch.int32, device=device),
                      torch.empty((cap, ctx.row_dim), dtype=torch.float32, device=device),
                      torch.zeros(1, dtype=torch.int32, device=device), int(cap_rows))


def alloc_workspace(nbytes, device="cuda"):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def zen_encode(ctx, grad, n_parts, hash_seed, out, workspace, stream=None):
    st = out.struct()
    return _check(load_library().zen_encode(ctx.handle, grad.data_ptr(), int(n_parts), int(hash_seed) & 0xFFFFFFFF,
                                            C.byref(st), workspace.data_ptr(), workspace.numel(), _stream(stream)),
                  "zen_encode")


def zen_encode_static(ctx, grad, n_parts, hash_seed, out, status=None, stream=None, allow=()):
    """status: device tensor of 16 bytes (flags u32, reserved u32, needed_rows u64) or None."""
    st = out.struct()
    return _check(load_library().zen_encode_static(ctx.handle, grad.data_ptr(), int(n_parts), int(hash_seed) & 0xFFFFFFFF,
                                                   C.byref(st), _ptr(status), _stream(stream)), "zen_encode_static", allow)


def zen_encode_batch(ctx, grads, outs, workspace, stream=None):
    n = len(grads)
    assert len(outs) == n
    gp = (C.c_void_p * n)(*[g.data_ptr() for g in grads])
    es = (_Encoded * n)(*[o.struct() for o in outs])
    return _check(load_library().zen_encode_batch(ctx.handle, gp, n, es, workspace.data_ptr(), workspace.numel(),
                                                  _stream(stream)), "zen_encode_batch")


def zen_nonzero(ctx, grad, indices, count, workspace, stream=None):
    return _check(load_library().zen_nonzero(ctx.handle, grad.data_ptr(), indices.data_ptr(), indices.numel(),
                                             count.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                             _stream(stream)), "zen_nonzero")


def zen_aggregate(ctx, parts, part_id, out, max_in_rows, workspace, stream=None):
    """parts: list of (indices|None, bitmap|None, values, count) device tensors."""
    n = len(parts)
    ps = (_Part * max(n, 1))(*[_Part(_ptr(p[0]), _ptr(p[1]), _ptr(p[2]), _ptr(p[3])) for p in parts])
    return _check(load_library().zen_aggregate(ctx.handle, ps, n, int(part_id), out.indices.data_ptr(),
                                               out.values.data_ptr(), out.cap_rows, out.count.data_ptr(),
                                               int(max_in_rows), workspace.data_ptr(), workspace.numel(),
                                               _stream(stream)), "zen_aggregate")


def zen_aggregate_batch(ctx, encs, outs, max_in_rows, workspace, stream=None):
    n = len(encs)
    assert len(outs) == ctx.n_parts
    es = (_Encoded * n)(*[e.struct() for e in encs])
    os_ = (_Aggregated * len(outs))(*[o.struct() for o in outs])
    return _check(load_library().zen_aggregate_batch(ctx.handle, es, n, os_, int(max_in_rows), workspace.data_ptr(),
                                                     workspace.numel(), _stream(stream)), "zen_aggregate_batch")


def zen_pull_workspace_bytes(ctx):
    b = C.c_uint64()
    _check(load_library().zen_pull_workspace_bytes(ctx.handle, C.byref(b)), "zen_pull_workspace_bytes")
    return int(b.value)


def zen_pull_encode(ctx, indices, count, cap_rows, part_id, bitmap_words, workspace, stream=None):
    return _check(load_library().zen_pull_encode(ctx.handle, indices.data_ptr(), count.data_ptr(), int(cap_rows),
                                                 int(part_id), bitmap_words.data_ptr(), workspace.data_ptr(),
                                                 workspace.numel(), _stream(stream)), "zen_pull_encode")


def zen_pull_encode_batch(ctx, aggs, bitmap, workspace, stream=None):
    assert len(aggs) == ctx.n_parts
    as_ = (_Aggregated * len(aggs))(*[a.struct() for a in aggs])
    return _check(load_library().zen_pull_encode_batch(ctx.handle, as_, bitmap.data_ptr(), workspace.data_ptr(),
                                                       workspace.numel(), _stream(stream)), "zen_pull_encode_batch")


def zen_pull_decode(ctx, bitmap_words, part_id, out_indices, out_count, workspace, stream=None):
    return _check(load_library().zen_pull_decode(ctx.handle, bitmap_words.data_ptr(), int(part_id),
                                                 out_indices.data_ptr(), out_indices.numel(), out_count.data_ptr(),
                                                 workspace.data_ptr(), workspace.numel(), _stream(stream)),
                  "zen_pull_decode")


def zen_pull_apply(ctx, parts, dense, workspace, stream=None):
    """parts: n_parts entries (indices|None, bitmap|None, values, count), entry p = partition p."""
    assert len(parts) == ctx.n_parts
    ps = (_Part * len(parts))(*[_Part(_ptr(p[0]), _ptr(p[1]), _ptr(p[2]), _ptr(p[3])) for p in parts])
    return _check(load_library().zen_pull_apply(ctx.handle, ps, dense.data_ptr(), workspace.data_ptr(),
                                                workspace.numel(), _stream(stream)), "zen_pull_apply")


def _hash_params(k, level2_seed, r1, r2):
    return _HashParams(int(k), int(level2_seed) & 0xFFFFFFFF, int(r1), int(r2))


def zen_hash_memory_bytes(ctx, k, level2_seed, r1, r2):
    b = C.c_uint64()
    hp = _hash_params(k, level2_seed, r1, r2)
    _check(load_library().zen_hash_memory_bytes(ctx.handle, C.byref(hp), C.byref(b)), "zen_hash_memory_bytes")
    return int(b.value)


def zen_encode_hashed_workspace_bytes(ctx, k, level2_seed, r1, r2):
    b = C.c_uint64()
    hp = _hash_params(k, level2_seed, r1, r2)
    _check(load_library().zen_encode_hashed_workspace_bytes(ctx.handle, C.byref(hp), C.byref(b)),
           "zen_encode_hashed_workspace_bytes")
    return int(b.value)


def zen_encode_hashed(ctx, grad, k, level2_seed, r1, r2, hash_memory, out, serial_counts, workspace, stream=None):
    hp = _hash_params(k, level2_seed, r1, r2)
    st = out.struct()
    return _check(load_library().zen_encode_hashed(ctx.handle, grad.data_ptr(), C.byref(hp), hash_memory.data_ptr(),
                                                   hash_memory.numel(), C.byref(st), _ptr(serial_counts),
                                                   workspace.data_ptr(), workspace.numel(), _stream(stream)),
                  "zen_encode_hashed")


def zen_sparsity_count(ctx, grads, workspace, stream=None):
    """-> dict of int64 device tensors: nnz[W], union_prefix[W], overlap[W, W], even_split[W, n_parts]."""
    W = len(grads)
    out = {"nnz": torch.empty(W, dtype=torch.int64, device=grads[0].device),
           "union_prefix": torch.empty(W, dtype=torch.int64, device=grads[0].device),
           "overlap": torch.empty((W, W), dtype=torch.int64, device=grads[0].device),
           "even_split": torch.empty((W, ctx.n_parts), dtype=torch.int64, device=grads[0].device)}
    st = _SparsityCounts(out["nnz"].data_ptr(), out["union_prefix"].data_ptr(), out["overlap"].data_ptr(),
                         out["even_split"].data_ptr())
    gp = (C.c_void_p * W)(*[g.data_ptr() for g in grads])
    _check(load_library().zen_sparsity_count(ctx.handle, gp, W, C.byref(st), workspace.data_ptr(), workspace.numel(),
                                             _stream(stream)), "zen_sparsity_count")
    return out


def zen_scheme_times(n, gamma_pow2, d_G, M, b):
    """-> (t_bp, t_sm): Equations (1) and (2); gamma_pow2 = [gamma^1, gamma^2, gamma^4, ..., gamma^n]."""
    g = (C.c_double * len(gamma_pow2))(*[float(x) for x in gamma_pow2])
    t_bp, t_sm = C.c_double(), C.c_double()
    if len(gamma_pow2) != int(n).bit_length():
        raise ZenError(ZEN_ERR_INVALID, "zen_scheme_times")
    _check(load_library().zen_scheme_times(int(n), g, float(d_G), float(M), float(b), C.byref(t_bp), C.byref(t_sm)),
           "zen_scheme_times")
    return float(t_bp.value), float(t_sm.value)


def zen_topk_workspace_bytes():
    b = C.c_uint64()
    _check(load_library().zen_topk_workspace_bytes(C.byref(b)), "zen_topk_workspace_bytes")
    return int(b.value)


def zen_topk_threshold(g, keep, threshold, workspace, first=0, stride=1, stream=None):
    """threshold: int32 device tensor with one element (receives the bit pattern)."""
    return _check(load_library().zen_topk_threshold(g.data_ptr(), g.numel(), int(first), int(stride), int(keep),
                                                    threshold.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                                    _stream(stream)), "zen_topk_threshold")


def zen_encode_batch_sparsified(ctx, grads, thresholds, outs, workspace, stream=None):
    n = len(grads)
    assert len(outs) == n and thresholds.numel() >= n
    gp = (C.c_void_p * n)(*[g.data_ptr() for g in grads])
    es = (_Encoded * n)(*[o.struct() for o in outs])
    return _check(load_library().zen_encode_batch_sparsified(ctx.handle, gp, n, thresholds.data_ptr(), es,
                                                             workspace.data_ptr(), workspace.numel(), _stream(stream)),
                  "zen_encode_batch_sparsified")


def zen_format_count(ctx, grad, block, counts, workspace, stream=None):
    """counts: int64 device tensor [2] -> (non-zero rows, non-zero blocks)."""
    return _check(load_library().zen_format_count(ctx.handle, grad.data_ptr(), int(block), counts.data_ptr(),
                                                  workspace.data_ptr(), workspace.numel(), _stream(stream)),
                  "zen_format_count")


def zen_format_bytes(n_elems, nnz, n_servers, nonzero_blocks, block=256):
    out = (C.c_double * 5)()
    _check(load_library().zen_format_bytes(int(n_elems), int(nnz), int(n_servers), int(nonzero_blocks), int(block), out),
           "zen_format_bytes")
    return dict(zip(("dense", "coo", "bitmap", "hash_bitmap", "tensor_block"), list(out)))


def zen_status_fetch(ctx, workspace, stream=None):
    """Synchronous. -> (status, flags, needed_rows)"""
    info = _StatusInfo()
    st = load_library().zen_status_fetch(ctx.handle, workspace.data_ptr(), _stream(stream), C.byref(info))
    return st, int(info.flags), int(info.needed_rows)


def zen_hash_many(idx, seed, out=None, stream=None):
    if out is None:
        out = torch.empty_like(idx)
    _check(load_library().zen_hash_many(idx.data_ptr(), idx.numel(), int(seed) & 0xFFFFFFFF, out.data_ptr(),
                                        _stream(stream)), "zen_hash_many")
    return out


def zen_profile_enable(ctx, mode, max_records=4096):
    return _check(load_library().zen_profile_enable(ctx.handle, int(mode), int(max_records)), "zen_profile_enable")


def zen_profile_kernel_name(kernel):
    return load_library().zen_profile_kernel_name(int(kernel)).decode()


def zen_profile_collect(ctx):
    """-> {kernel name: (total ms, launches)} for the kernels timed since the last collect."""
    ms = (C.c_double * 32)()
    cnt = (C.c_uint32 * 32)()
    n = C.c_uint32()
    _check(load_library().zen_profile_collect(ctx.handle, 32, ms, cnt, C.byref(n)), "zen_profile_collect")
    return {zen_profile_kernel_name(k): (float(ms[k]), int(cnt[k])) for k in range(int(n.value)) if cnt[k]}


def zen_calibration_copy(src, dst, stream=None):
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    return _check(load_library().zen_calibration_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(stream)),
                  "zen_calibration_copy")


def zen_calibration_read(src, sink, nbytes=None, shape=None, stream=None):
    """shape: None (the dense scan's launch shape) or (threads, unroll, block_bytes, max_blocks, nontemporal)."""
    nbytes = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    assert nbytes <= src.numel() * src.element_size() and sink.numel() >= 64
    sh = None if shape is None else C.byref(_ReadShape(*[int(x) for x in shape]))
    return _check(load_library().zen_calibration_read(src.data_ptr(), nbytes, sh, sink.data_ptr(), _stream(stream)),
                  "zen_calibration_read")
