"""ctypes/numpy wrapper around oracle/zen_ref.c (TEST INFRASTRUCTURE ONLY).

Argument marshalling only: every result is computed by the C file.  The shared object is built
with plain gcc (no HIP, no code shared with the GPU library).
"""
import ctypes as C
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zen_ref.c")
_SO = os.path.join(_HERE, "libzen_ref.so")
_lib = None

_u32p = C.POINTER(C.c_uint32)
_u16p = C.POINTER(C.c_uint16)
_u64p = C.POINTER(C.c_uint64)
_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)
_u8p = C.POINTER(C.c_uint8)


def build(force=False):
    """Compile zen_ref.c -> libzen_ref.so with gcc -O2."""
    global _lib
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _SO)
        _lib = None
    return _SO


def use_library(path):
    """Point the wrapper at another build of the oracle (the mutation test loads deliberately broken
    copies to prove that the pins notice); use_library(None) returns to the real one."""
    global _lib, _SO_OVERRIDE
    _SO_OVERRIDE = path
    _lib = None


_SO_OVERRIDE = None


def lib():
    global _lib
    if _lib is None:
        if _SO_OVERRIDE is None:
            build()
        L = C.CDLL(_SO_OVERRIDE or _SO)
        L.zen_ref_hash.restype = C.c_uint32
        L.zen_ref_hash.argtypes = [C.c_uint32, C.c_uint32]
        L.zen_ref_hash_many.restype = None
        L.zen_ref_hash_many.argtypes = [_u32p, C.c_uint64, C.c_uint32, _u32p]
        L.zen_ref_owner.restype = C.c_uint32
        L.zen_ref_owner.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
        L.zen_ref_owner_table.restype = C.c_int
        L.zen_ref_owner_table.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, _u16p]
        L.zen_ref_nonzero.restype = C.c_int64
        L.zen_ref_nonzero.argtypes = [_f32p, C.c_uint64, C.c_uint32, _u32p]
        L.zen_ref_partition.restype = C.c_int
        L.zen_ref_partition.argtypes = [_u32p, _u16p, C.c_uint64, C.c_uint32, _u32p, _u32p]
        L.zen_ref_gather.restype = None
        L.zen_ref_gather.argtypes = [_f32p, C.c_uint32, _u32p, C.c_uint64, _f32p]
        L.zen_ref_encode.restype = C.c_int
        L.zen_ref_encode.argtypes = [_f32p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, _u32p, _u32p,
                                     _f32p, C.c_uint64, _u64p]
        L.zen_ref_bitmap_layout.restype = C.c_int
        L.zen_ref_bitmap_layout.argtypes = [_u16p, C.c_uint64, C.c_uint32, _u64p, _u64p]
        L.zen_ref_bitmap_encode.restype = C.c_int
        L.zen_ref_bitmap_encode.argtypes = [_u16p, C.c_uint64, C.c_uint32, _u8p, _u64p, _u32p]
        L.zen_ref_bitmap_decode.restype = C.c_int64
        L.zen_ref_bitmap_decode.argtypes = [_u16p, C.c_uint64, C.c_uint32, _u32p, _u32p]
        L.zen_ref_aggregate.restype = C.c_int64
        L.zen_ref_aggregate.argtypes = [C.c_uint32, C.POINTER(_u32p), C.POINTER(_f32p), _u64p, C.c_uint64,
                                        C.c_uint32, _u32p, _f32p, _f64p, _f64p, _u32p, C.c_uint64]
        L.zen_ref_member_mask.restype = C.c_int
        L.zen_ref_member_mask.argtypes = [_u32p, C.c_uint64, C.c_uint64, _u8p]
        L.zen_ref_densify.restype = C.c_int
        L.zen_ref_densify.argtypes = [C.c_uint32, C.POINTER(_u32p), C.POINTER(_f32p), _u64p, C.c_uint64,
                                      C.c_uint32, _f32p]
        L.zen_ref_pull_apply.restype = C.c_int
        L.zen_ref_pull_apply.argtypes = [_u16p, C.c_uint64, C.c_uint32, C.c_uint32, _u64p, _u32p,
                                         C.POINTER(_f32p), _u64p, _f32p]
        L.zen_ref_hierarchical_hash.restype = C.c_int
        L.zen_ref_hierarchical_hash.argtypes = [_u32p, C.c_uint64, _u16p, C.POINTER(_u32p), C.c_uint32, C.c_uint32,
                                                C.c_uint64, C.c_uint64, _u32p, _u64p, _u64p]
        L.zen_ref_hash_slots.restype = None
        L.zen_ref_hash_slots.argtypes = [_u32p, C.c_uint64, C.c_uint32, C.c_uint64, _u32p]
        L.zen_ref_hash_memory_extract.restype = C.c_int64
        L.zen_ref_hash_memory_extract.argtypes = [_u32p, C.c_uint32, C.c_uint64, _u32p, _u32p]
        L.zen_ref_overlap_ratio.restype = C.c_double
        L.zen_ref_overlap_ratio.argtypes = [_u32p, C.c_uint64, _u32p, C.c_uint64, C.c_uint64]
        L.zen_ref_union_sizes.restype = C.c_int
        L.zen_ref_union_sizes.argtypes = [C.c_uint32, C.POINTER(_u32p), _u64p, C.c_uint64, _u64p]
        L.zen_ref_skewness.restype = C.c_double
        L.zen_ref_skewness.argtypes = [_u32p, C.c_uint64, C.c_uint64, C.c_uint32, _u64p]
        L.zen_ref_time_balanced_parallelism.restype = C.c_double
        L.zen_ref_time_balanced_parallelism.argtypes = [C.c_uint32, C.c_double, C.c_double, C.c_double, C.c_double]
        L.zen_ref_time_hierarchical_centralization.restype = C.c_double
        L.zen_ref_time_hierarchical_centralization.argtypes = [C.c_uint32, _f64p, C.c_double, C.c_double, C.c_double]
        L.zen_ref_topk_threshold.restype = C.c_uint32
        L.zen_ref_topk_threshold.argtypes = [_f32p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64]
        L.zen_ref_threshold_apply.restype = C.c_uint64
        L.zen_ref_threshold_apply.argtypes = [_f32p, C.c_uint64, C.c_uint32, _f32p]
        L.zen_ref_format_bytes.restype = None
        L.zen_ref_format_bytes.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, _f64p]
        L.zen_ref_nonzero_blocks.restype = C.c_uint64
        L.zen_ref_nonzero_blocks.argtypes = [_u32p, C.c_uint64, C.c_uint64, C.c_uint32]
        L.zen_ref_imbalance.restype = C.c_double
        L.zen_ref_imbalance.argtypes = [_u64p, C.c_uint32]
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def hash32(idx, seed):
    return int(lib().zen_ref_hash(int(idx) & 0xFFFFFFFF, int(seed) & 0xFFFFFFFF))


def hash_many(idx, seed):
    idx = _c(idx, np.uint32)
    out = np.empty(idx.shape, np.uint32)
    lib().zen_ref_hash_many(_p(idx, _u32p), idx.size, int(seed) & 0xFFFFFFFF, _p(out, _u32p))
    return out


def owner_table(n_rows, n, seed):
    out = np.empty(int(n_rows), np.uint16)
    rc = lib().zen_ref_owner_table(int(n_rows), int(n), int(seed) & 0xFFFFFFFF, _p(out, _u16p))
    if rc != 0:
        raise ValueError("zen_ref_owner_table: rc=%d" % rc)
    return out


def nonzero(grad, n_rows, row_dim):
    grad = _c(grad, np.float32).reshape(-1)
    assert grad.size == int(n_rows) * int(row_dim)
    nnz = lib().zen_ref_nonzero(_p(grad, _f32p), int(n_rows), int(row_dim), None)
    I = np.empty(int(nnz), np.uint32)
    lib().zen_ref_nonzero(_p(grad, _f32p), int(n_rows), int(row_dim), _p(I, _u32p) if nnz else None)
    return I


def partition(I, owner_of_I, n):
    I = _c(I, np.uint32)
    owner_of_I = _c(owner_of_I, np.uint16)
    assert I.size == owner_of_I.size
    offsets = np.zeros(int(n) + 1, np.uint32)
    indices = np.empty(I.size, np.uint32)
    rc = lib().zen_ref_partition(_p(I, _u32p), _p(owner_of_I, _u16p), I.size, int(n), _p(offsets, _u32p),
                                 _p(indices, _u32p))
    if rc != 0:
        raise ValueError("zen_ref_partition: rc=%d" % rc)
    return offsets, indices


def gather(grad, row_dim, indices):
    grad = _c(grad, np.float32).reshape(-1)
    indices = _c(indices, np.uint32)
    values = np.empty((indices.size, int(row_dim)), np.float32)
    lib().zen_ref_gather(_p(grad, _f32p), int(row_dim), _p(indices, _u32p), indices.size, _p(values, _f32p))
    return values


def encode(grad, n_rows, row_dim, n, seed, cap_rows=None, want_values=True):
    """Returns SimpleNamespace(rc, nnz, offsets, indices, values)."""
    grad = _c(grad, np.float32).reshape(-1)
    assert grad.size == int(n_rows) * int(row_dim)
    if cap_rows is None:
        cap_rows = int(lib().zen_ref_nonzero(_p(grad, _f32p), int(n_rows), int(row_dim), None))
    offsets = np.zeros(int(n) + 1, np.uint32)
    indices = np.empty(int(cap_rows), np.uint32)
    values = np.empty((int(cap_rows), int(row_dim)), np.float32) if want_values else None
    nnz = C.c_uint64(0)
    rc = lib().zen_ref_encode(_p(grad, _f32p), int(n_rows), int(row_dim), int(n), int(seed) & 0xFFFFFFFF,
                              _p(offsets, _u32p), _p(indices, _u32p),
                              _p(values, _f32p) if want_values else None, int(cap_rows), C.byref(nnz))
    k = int(nnz.value) if rc == 0 else 0
    return SimpleNamespace(rc=rc, nnz=int(nnz.value), offsets=offsets, indices=indices[:k],
                           values=values[:k] if want_values else None)


def bitmap_layout(owner, n):
    owner = _c(owner, np.uint16)
    dom_count = np.zeros(int(n), np.uint64)
    word_off = np.zeros(int(n) + 1, np.uint64)
    rc = lib().zen_ref_bitmap_layout(_p(owner, _u16p), owner.size, int(n), _p(dom_count, _u64p),
                                     _p(word_off, _u64p))
    if rc != 0:
        raise ValueError("zen_ref_bitmap_layout: rc=%d" % rc)
    return dom_count, word_off


def bitmap_encode(owner, n, nz, word_off):
    owner = _c(owner, np.uint16)
    nz = _c(nz, np.uint8)
    word_off = _c(word_off, np.uint64)
    assert nz.size == owner.size and word_off.size == int(n) + 1
    bitmap = np.empty(int(word_off[-1]), np.uint32)
    lib().zen_ref_bitmap_encode(_p(owner, _u16p), owner.size, int(n), _p(nz, _u8p), _p(word_off, _u64p),
                                _p(bitmap, _u32p))
    return bitmap


def bitmap_decode(owner, p, bitmap_p):
    owner = _c(owner, np.uint16)
    bitmap_p = _c(bitmap_p, np.uint32)
    out = np.empty(int((owner == p).sum()), np.uint32)
    need_words = (out.size + 31) // 32
    assert bitmap_p.size >= need_words
    k = lib().zen_ref_bitmap_decode(_p(owner, _u16p), owner.size, int(p), _p(bitmap_p, _u32p), _p(out, _u32p))
    return out[: int(k)]


def aggregate(parts, n_rows, row_dim, cap_rows=None, want_f64=True):
    """parts: list of (indices u32[count], values f32[count, D]).

    Returns SimpleNamespace(U, indices, values, sum64, abs64, ncontrib); U < 0 means capacity
    overflow with -U rows needed.
    """
    n_in = len(parts)
    idx = [_c(p[0], np.uint32).reshape(-1) for p in parts]
    val = [_c(p[1], np.float32).reshape(-1) for p in parts]
    for i, v in zip(idx, val):
        assert v.size == i.size * int(row_dim)
    counts = np.array([i.size for i in idx], np.uint64)
    total = int(counts.sum())
    if cap_rows is None:
        cap_rows = total
    idx_arr = (_u32p * max(n_in, 1))(*[_p(i, _u32p) for i in idx])
    val_arr = (_f32p * max(n_in, 1))(*[_p(v, _f32p) for v in val])
    out_idx = np.empty(int(cap_rows), np.uint32)
    out_val = np.empty((int(cap_rows), int(row_dim)), np.float32)
    out_sum = np.empty((int(cap_rows), int(row_dim)), np.float64) if want_f64 else None
    out_abs = np.empty((int(cap_rows), int(row_dim)), np.float64) if want_f64 else None
    out_nc = np.empty(int(cap_rows), np.uint32)
    U = lib().zen_ref_aggregate(n_in, idx_arr, val_arr, _p(counts, _u64p), int(n_rows), int(row_dim),
                                _p(out_idx, _u32p), _p(out_val, _f32p),
                                _p(out_sum, _f64p) if want_f64 else None,
                                _p(out_abs, _f64p) if want_f64 else None, _p(out_nc, _u32p), int(cap_rows))
    U = int(U)
    if U < 0:
        return SimpleNamespace(U=U, indices=None, values=None, sum64=None, abs64=None, ncontrib=None)
    return SimpleNamespace(U=U, indices=out_idx[:U], values=out_val[:U],
                           sum64=out_sum[:U] if want_f64 else None,
                           abs64=out_abs[:U] if want_f64 else None, ncontrib=out_nc[:U])


def member_mask(indices, n_rows):
    indices = _c(indices, np.uint32).reshape(-1)
    member = np.empty(int(n_rows), np.uint8)
    rc = lib().zen_ref_member_mask(_p(indices, _u32p), indices.size, int(n_rows), _p(member, _u8p))
    if rc != 0:
        raise ValueError("zen_ref_member_mask: rc=%d" % rc)
    return member


def densify(parts, n_rows, row_dim):
    """parts: list of (indices u32[count], values f32[count, D]), pairwise disjoint -> dense f32[R, D]."""
    n_in = len(parts)
    idx = [_c(p[0], np.uint32).reshape(-1) for p in parts]
    val = [_c(p[1], np.float32).reshape(-1) for p in parts]
    for i, v in zip(idx, val):
        assert v.size == i.size * int(row_dim)
    counts = np.array([i.size for i in idx], np.uint64)
    idx_arr = (_u32p * max(n_in, 1))(*[_p(i, _u32p) for i in idx])
    val_arr = (_f32p * max(n_in, 1))(*[_p(v, _f32p) for v in val])
    dense = np.empty((int(n_rows), int(row_dim)), np.float32)
    rc = lib().zen_ref_densify(n_in, idx_arr, val_arr, _p(counts, _u64p), int(n_rows), int(row_dim),
                               _p(dense, _f32p))
    if rc != 0:
        raise ValueError("zen_ref_densify: rc=%d" % rc)
    return dense


def pull_apply(owner, n, row_dim, word_off, bitmap, values):
    """values: list over the n partitions of f32[count_p, D] in bit order -> dense f32[R, D]."""
    owner = _c(owner, np.uint16)
    word_off = _c(word_off, np.uint64)
    bitmap = _c(bitmap, np.uint32)
    assert len(values) == int(n) and word_off.size == int(n) + 1 and bitmap.size >= int(word_off[-1])
    val = [_c(v, np.float32).reshape(-1) for v in values]
    counts = np.array([v.size // int(row_dim) for v in val], np.uint64)
    val_arr = (_f32p * int(n))(*[_p(v, _f32p) for v in val])
    dense = np.empty((owner.size, int(row_dim)), np.float32)
    rc = lib().zen_ref_pull_apply(_p(owner, _u16p), owner.size, int(n), int(row_dim), _p(word_off, _u64p),
                                  _p(bitmap, _u32p), val_arr, _p(counts, _u64p), _p(dense, _f32p))
    if rc != 0:
        raise ValueError("zen_ref_pull_apply: rc=%d" % rc)
    return dense


def hash_slots(I, seed_i, r1):
    I = _c(I, np.uint32).reshape(-1)
    out = np.empty(I.size, np.uint32)
    lib().zen_ref_hash_slots(_p(I, _u32p), I.size, int(seed_i) & 0xFFFFFFFF, int(r1), _p(out, _u32p))
    return out


def hierarchical_hash(I, part, slots, n, r1, r2):
    """Algorithm 1's hash memory for the indices I taken in order.  part: u16[nnz] = h0(I); slots: list
    of k arrays u32[nnz] = h_1(I) .. h_k(I).  -> SimpleNamespace(rc, x[n, r1+r2], serial_count[n],
    needed_r2, offsets, indices) with indices = nonzero(x[p]) in memory order."""
    I = _c(I, np.uint32).reshape(-1)
    part = _c(part, np.uint16).reshape(-1)
    slots = [_c(s, np.uint32).reshape(-1) for s in slots]
    assert part.size == I.size and all(s.size == I.size for s in slots)
    k = len(slots)
    cells = int(r1) + int(r2)
    x = np.empty((int(n), cells), np.uint32)
    serial = np.zeros(int(n), np.uint64)
    needed = C.c_uint64(0)
    slot_arr = (_u32p * max(k, 1))(*[_p(s, _u32p) for s in slots])
    rc = lib().zen_ref_hierarchical_hash(_p(I, _u32p), I.size, _p(part, _u16p), slot_arr, k, int(n), int(r1),
                                         int(r2), _p(x, _u32p), _p(serial, _u64p), C.byref(needed))
    offsets = np.zeros(int(n) + 1, np.uint32)
    indices = np.empty(I.size, np.uint32)
    cnt = 0
    if rc == 0:
        cnt = int(lib().zen_ref_hash_memory_extract(_p(x, _u32p), int(n), cells, _p(offsets, _u32p), _p(indices, _u32p)))
    return SimpleNamespace(rc=rc, x=x, serial_count=serial, needed_r2=int(needed.value), offsets=offsets,
                           indices=indices[:cnt])


def overlap_ratio(I1, I2, n_rows):
    I1, I2 = _c(I1, np.uint32).reshape(-1), _c(I2, np.uint32).reshape(-1)
    return float(lib().zen_ref_overlap_ratio(_p(I1, _u32p), I1.size, _p(I2, _u32p), I2.size, int(n_rows)))


def union_sizes(index_sets, n_rows):
    idx = [_c(i, np.uint32).reshape(-1) for i in index_sets]
    counts = np.array([i.size for i in idx], np.uint64)
    arr = (_u32p * max(len(idx), 1))(*[_p(i, _u32p) for i in idx])
    out = np.zeros(len(idx), np.uint64)
    rc = lib().zen_ref_union_sizes(len(idx), arr, _p(counts, _u64p), int(n_rows), _p(out, _u64p))
    if rc != 0:
        raise ValueError("zen_ref_union_sizes: rc=%d" % rc)
    return out


def skewness(I, n_rows, n):
    """-> (skewness ratio, non-zero count of each of the n even partitions)"""
    I = _c(I, np.uint32).reshape(-1)
    part = np.zeros(int(n), np.uint64)
    r = float(lib().zen_ref_skewness(_p(I, _u32p), I.size, int(n_rows), int(n), _p(part, _u64p)))
    return r, part


def time_balanced_parallelism(n, gamma_n, d_G, M, b):
    return float(lib().zen_ref_time_balanced_parallelism(int(n), float(gamma_n), float(d_G), float(M), float(b)))


def time_hierarchical_centralization(n, gamma_pow2, d_G, M, b):
    g = _c(gamma_pow2, np.float64).reshape(-1)
    assert (1 << g.size) >= int(n)
    return float(lib().zen_ref_time_hierarchical_centralization(int(n), _p(g, _f64p), float(d_G), float(M), float(b)))


def topk_threshold(g, keep, first=0, stride=1):
    """Bit pattern of the keep-th largest magnitude among g[first::stride]."""
    g = _c(g, np.float32).reshape(-1)
    t = int(lib().zen_ref_topk_threshold(_p(g, _f32p), g.size, int(first), int(stride), int(keep)))
    if t == 0xFFFFFFFF:
        raise ValueError("zen_ref_topk_threshold: bad argument")
    return t


def threshold_apply(g, threshold):
    """-> (g with every element of magnitude below the threshold replaced by +0.0, number kept)"""
    g = _c(g, np.float32).reshape(-1)
    out = np.empty_like(g)
    kept = int(lib().zen_ref_threshold_apply(_p(g, _f32p), g.size, int(threshold), _p(out, _f32p)))
    return out, kept


def format_bytes(G, nnz, n, nonzero_blocks, block=256):
    """-> dict of bytes per format: dense, coo, bitmap, hash_bitmap, tensor_block"""
    out = np.zeros(5, np.float64)
    lib().zen_ref_format_bytes(int(G), int(nnz), int(n), int(nonzero_blocks), int(block), _p(out, _f64p))
    return dict(zip(("dense", "coo", "bitmap", "hash_bitmap", "tensor_block"), out.tolist()))


def nonzero_blocks(I, n_rows, block=256):
    I = _c(I, np.uint32).reshape(-1)
    return int(lib().zen_ref_nonzero_blocks(_p(I, _u32p), I.size, int(n_rows), int(block)))


def imbalance(sizes):
    sizes = _c(sizes, np.uint64)
    return float(lib().zen_ref_imbalance(_p(sizes, _u64p), sizes.size))
