"""Helpers for the GPU parity tests: device inputs from the seeded sparse form, run wrappers."""
import numpy as np
import torch

import paper_2309_13254_amd as zen
from workloads import worker_sparse


def dense_device(wl, rows, vals, device="cuda"):
    """Dense fp32 [R, D] device tensor with `vals` planted at `rows` (input plumbing, not the path)."""
    g = torch.zeros((wl.n_rows, wl.row_dim), dtype=torch.float32, device=device)
    if rows.size:
        idx = torch.from_numpy(rows.astype(np.int64)).to(device)
        g.index_copy_(0, idx, torch.from_numpy(np.ascontiguousarray(vals)).to(device))
    return g


def to_dev(a, dtype=None, device="cuda"):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    t = torch.from_numpy(a).to(device)
    return t


def u32(t):
    """torch int32 device tensor -> numpy uint32"""
    return t.detach().cpu().numpy().view(np.uint32)


def run_encode_batch(ctx, grads, caps):
    outs = [zen.alloc_encoded(ctx, c) for c in caps]
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, len(grads)))
    zen.zen_encode_batch(ctx, grads, outs, ws)
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    return outs, (st, flags, needed)


def encoded_to_host(enc, D):
    off = u32(enc.offsets)
    nnz = int(off[-1])
    k = min(nnz, enc.cap_rows)
    idx = u32(enc.indices[:k]) if enc.indices is not None else None
    val = enc.values[:k].detach().cpu().numpy()
    return off, idx, val


def run_aggregate_batch(ctx, encs, out_caps, max_in_rows):
    outs = [zen.alloc_aggregated(ctx, c) for c in out_caps]
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, ctx.n_parts, max_in_rows))
    zen.zen_aggregate_batch(ctx, encs, outs, max_in_rows, ws)
    st = zen.zen_status_fetch(ctx, ws)
    return outs, st


def aggregated_to_host(out):
    U = int(u32(out.count)[0])
    k = min(U, out.cap_rows)
    return U, u32(out.indices[:k]), out.values[:k].detach().cpu().numpy()


def check_sums(gpu_vals, ref, rel=1e-6):
    """|gpu - s| <= rel * sum|x| elementwise; rows with a single contributor bit-exact."""
    err = np.abs(gpu_vals.astype(np.float64) - ref.sum64)
    bound = rel * ref.abs64
    bad = err > bound
    assert not bad.any(), "max err/bound = %g" % float((err[bad] / np.maximum(bound[bad], 1e-300)).max())
    single = ref.ncontrib == 1
    assert np.array_equal(gpu_vals[single].view(np.uint32), ref.values[single].view(np.uint32))


def workload_inputs(wl, n_workers=None):
    n_workers = wl.n_workers if n_workers is None else n_workers
    sparse = [worker_sparse(wl, w) for w in range(n_workers)]
    grads = [dense_device(wl, r, v) for r, v in sparse]
    return sparse, grads


def use_tuning(monkeypatch, tiled_encode=False, tile_bytes=0):
    """Make every zen.ZenContext(...) of the running test a context created with this tuning (the tiled
    partition path for few-row encodes too, another tile size): zen_ctx_create_tuned instead of zen_ctx_create."""
    if not tiled_encode and not tile_bytes:
        return
    plain = zen.ZenContext

    def tuned(*args, **kw):
        kw.setdefault("tiled_encode", tiled_encode)
        kw.setdefault("tile_bytes", tile_bytes)
        return plain(*args, **kw)

    monkeypatch.setattr(zen, "ZenContext", tuned)
