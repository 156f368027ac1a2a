"""GPU parity: zen_encode / zen_encode_batch / zen_nonzero / zen_hash_many against the CPU oracle.

Bit-exact on offsets, indices and values (the values are copies).
"""
import os

import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, Workload, worker_sparse, dense_from_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["small", "tiled"])
def partition_path(request, monkeypatch):
    """Run every test through both partition paths: the one-block-per-worker path that few-row
    encodes take by default, and the tiled histogram / scan / scatter path."""
    import gpu_util as G

    G.use_tuning(monkeypatch, tiled_encode=request.param == "tiled")
    return request.param


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    assert torch.cuda.is_available()
    return z


def _check_encoded(oracle, zen, ctx, wl, g_host, enc, cap=None):
    import gpu_util as G

    ref = oracle.encode(g_host, wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
    off, idx, val = G.encoded_to_host(enc, wl.row_dim)
    assert np.array_equal(off, ref.offsets)
    k = ref.nnz if cap is None else min(ref.nnz, cap)
    if cap is None:
        assert np.array_equal(idx, ref.indices)
        assert np.array_equal(val.view(np.uint32), ref.values.view(np.uint32))
    return ref


def test_hash_matches_oracle(oracle, zen):
    rng = np.random.default_rng(11)
    idx = rng.integers(0, 2**32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    import gpu_util as G

    d_idx = G.to_dev(idx)
    for seed in (0, 1, 0x9E3779B1, 0xFFFFFFFF):
        out = zen.zen_hash_many(d_idx, seed)
        torch.cuda.synchronize()
        assert np.array_equal(G.u32(out), oracle.hash_many(idx, seed))


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_encode_batch_mini_workloads(oracle, zen, cid):
    import gpu_util as G

    wl = MINI_WORKLOADS[cid]
    sparse, grads = G.workload_inputs(wl)
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
    outs, (st, flags, needed) = G.run_encode_batch(ctx, grads, [r.size for r, _ in sparse])
    assert st == 0 and flags == 0
    for w, ((rows, vals), enc) in enumerate(zip(sparse, outs)):
        g_host = dense_from_sparse(wl, rows, vals)
        ref = _check_encoded(oracle, zen, ctx, wl, g_host, enc)
        assert ref.nnz == rows.size
    # determinism: a second run gives identical bits
    outs2, _ = G.run_encode_batch(ctx, grads, [r.size for r, _ in sparse])
    for a, b in zip(outs, outs2):
        assert torch.equal(a.offsets, b.offsets) and torch.equal(a.indices, b.indices)
        assert torch.equal(a.values.view(torch.int32), b.values.view(torch.int32))
    # single-gradient entry point gives the same result as the batch
    one = zen.alloc_encoded(ctx, sparse[0][0].size)
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
    zen.zen_encode(ctx, grads[0], wl.n_parts, wl.hash_seed, one, ws)
    assert zen.zen_status_fetch(ctx, ws)[0] == 0
    assert torch.equal(one.offsets, outs[0].offsets) and torch.equal(one.indices, outs[0].indices)
    assert torch.equal(one.values.view(torch.int32), outs[0].values.view(torch.int32))


@pytest.mark.parametrize("cid", [1, 3, 5])
@pytest.mark.parametrize("fill", [-1, 7, 0x01010101])
def test_encode_ignores_stale_workspace(oracle, zen, cid, fill):
    """The workspace carries over nothing: whatever it held (masks, histogram rows and flags of tiles that
    are empty this time are not rewritten) must not reach the result."""
    import gpu_util as G

    wl = MINI_WORKLOADS[cid]
    sparse, grads = G.workload_inputs(wl, n_workers=min(wl.n_workers, 4))
    fmt = zen.ZEN_INDEX_BITMAP if wl.bitmap else zen.ZEN_INDEX_COO
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed, fmt)
    outs = [zen.alloc_encoded(ctx, r.size) for r, _ in sparse]
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, len(grads)))
    ws.view(torch.int32).fill_(fill)
    zen.zen_encode_batch(ctx, grads, outs, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    for (rows, vals), enc in zip(sparse, outs):
        _check_encoded(oracle, zen, ctx, wl, dense_from_sparse(wl, rows, vals), enc)


SHAPES = [
    # R, D, n
    (1, 1, 1), (5, 1, 3), (255, 1, 2), (256, 1, 4), (257, 1, 5), (70001, 1, 64), (300000, 1, 100),
    (3, 2, 2), (1000, 3, 7), (777, 4, 4), (4099, 8, 16), (513, 16, 3), (2050, 32, 8), (9001, 64, 16),
    (1500, 128, 32), (700, 100, 5), (333, 256, 8), (130, 260, 4), (97, 1024, 8), (70, 4096, 32),
    (40, 1023, 1024), (5000, 1, 1024),
]


@pytest.mark.parametrize("R,D,n", SHAPES)
def test_encode_shapes_and_densities(oracle, zen, R, D, n):
    import gpu_util as G

    rng = np.random.default_rng(R * 31 + D * 7 + n)
    wl = Workload("t", 0, R, D, n, int(rng.integers(0, 2**32)), "uniform")
    ctx = zen.ZenContext(R, D, n, wl.hash_seed)
    hosts = []
    for density in (0.0, 0.03, 0.5, 1.0):
        g = np.zeros((R, D), np.float32)
        rows = np.flatnonzero(rng.random(R) < density)
        if rows.size:
            # a non-zero row may have a single non-zero element anywhere in it
            vals = np.zeros((rows.size, D), np.float32)
            cols = rng.integers(0, D, size=rows.size)
            vals[np.arange(rows.size), cols] = rng.standard_normal(rows.size).astype(np.float32) + 3.0
            dense_rows = rng.random(rows.size) < 0.5
            vals[dense_rows] = rng.standard_normal((int(dense_rows.sum()), D)).astype(np.float32)
            vals[dense_rows, 0] = 1.0
            g[rows] = vals
        hosts.append(g)
    grads = [torch.from_numpy(h).cuda() for h in hosts]
    outs, (st, flags, _) = G.run_encode_batch(ctx, grads, [R] * len(grads))
    assert st == 0 and flags == 0
    for h, enc in zip(hosts, outs):
        _check_encoded(oracle, zen, ctx, wl, h, enc)


def test_special_values_and_signed_zero(oracle, zen):
    import gpu_util as G

    for D in (1, 4, 64, 1024):
        R = 600
        g = np.zeros((R, D), np.float32)
        specials = np.array([-0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 1.17549435e-38, 1.0], np.float32)
        for k, v in enumerate(specials):
            g[10 + 37 * k, (k * 5) % D] = v
        g[500] = -0.0                      # a row of negative zeros is a zero row
        wl = Workload("t", 0, R, D, 4, 77, "uniform")
        ctx = zen.ZenContext(R, D, 4, 77)
        outs, (st, _, _) = G.run_encode_batch(ctx, [torch.from_numpy(g).cuda()], [R])
        assert st == 0
        ref = _check_encoded(oracle, zen, ctx, wl, g, outs[0])
        assert ref.nnz == 7


@pytest.mark.parametrize("cid", [1, 3, 5])
def test_capacity_overflow_is_reported_and_contained(oracle, zen, cid):
    import gpu_util as G

    wl = MINI_WORKLOADS[cid]
    rows, vals = worker_sparse(wl, 0)
    g = G.dense_device(wl, rows, vals)
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
    cap = rows.size // 2
    enc = zen.alloc_encoded(ctx, cap)
    # guard region after the capacity must stay untouched
    big_idx = torch.full((rows.size,), -2, dtype=torch.int32, device="cuda")
    big_val = torch.full((rows.size, wl.row_dim), 7.0, dtype=torch.float32, device="cuda")
    enc.indices, enc.values = big_idx, big_val
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
    zen.zen_encode_batch(ctx, [g], [enc], ws)
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    assert st == zen.ZEN_ERR_CAPACITY and (flags & 1) and needed == rows.size
    ref = oracle.encode(dense_from_sparse(wl, rows, vals), wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
    assert np.array_equal(G.u32(enc.offsets), ref.offsets)            # offsets still complete
    assert np.array_equal(G.u32(big_idx[:cap]), ref.indices[:cap])    # everything below the capacity is right
    assert np.array_equal(big_val[:cap].cpu().numpy().view(np.uint32), ref.values[:cap].view(np.uint32))
    assert torch.all(big_idx[cap:] == -2) and torch.all(big_val[cap:] == 7.0)


def test_nonzero_list(oracle, zen):
    import gpu_util as G

    for cid in (1, 2, 3):
        wl = MINI_WORKLOADS[cid]
        rows, vals = worker_sparse(wl, 1)
        g = G.dense_device(wl, rows, vals)
        ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
        idx = torch.empty(rows.size + 5, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
        zen.zen_nonzero(ctx, g, idx, cnt, ws)
        assert zen.zen_status_fetch(ctx, ws)[0] == 0
        I = oracle.nonzero(dense_from_sparse(wl, rows, vals), wl.n_rows, wl.row_dim)
        assert int(cnt.item()) == I.size
        assert np.array_equal(G.u32(idx[:I.size]), I)


def test_argument_errors(zen):
    with pytest.raises(zen.ZenError):
        zen.ZenContext(0, 1, 4, 1)
    with pytest.raises(zen.ZenError):
        zen.ZenContext(10, 1, 0, 1)
    with pytest.raises(zen.ZenError):
        zen.ZenContext(10, 1, 2000, 1)
    ctx = zen.ZenContext(1000, 4, 4, 1)
    g = torch.zeros((1000, 4), device="cuda")
    enc = zen.alloc_encoded(ctx, 10)
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
    with pytest.raises(zen.ZenError):                       # n_parts / seed must match the context
        zen.zen_encode(ctx, g, 5, 1, enc, ws)
    with pytest.raises(zen.ZenError):                       # misaligned gradient
        zen.zen_encode(ctx, g.view(-1)[1:], 4, 1, enc, ws)
    with pytest.raises(zen.ZenError):                       # workspace too small
        zen.zen_encode(ctx, g, 4, 1, enc, ws[:256])
