"""GPU parity at the benchmark's full sizes for the widened rows: sparsity counts, Algorithm 1's hash
memory, and the top-k threshold sparsifier.  (Pull at full size lives in test_gpu_fullsize.py.)"""
import numpy as np
import pytest
import torch

from workloads import WORKLOADS, worker_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


@pytest.mark.parametrize("cid", [2, 3])
def test_sparsity_counts_full_size(oracle, zen, cid):
    import gpu_util as G

    wl = WORKLOADS[cid]
    R, n, W = wl.n_rows, wl.n_parts, wl.n_workers
    sparse = [worker_sparse(wl, w, want_values=False) for w in range(W)]
    sets = [r for r, _ in sparse]
    ctx = zen.ZenContext(R, wl.row_dim, n, wl.hash_seed, zen.ZEN_INDEX_COO)
    grads = []
    for rows in sets:                                  # any non-zero value marks the row
        g = torch.zeros((R, wl.row_dim), dtype=torch.float32, device="cuda")
        g[torch.from_numpy(rows.astype(np.int64)).cuda(), 0] = 1.0
        grads.append(g)
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, W))
    out = {k: v.cpu().numpy() for k, v in zen.zen_sparsity_count(ctx, grads, ws).items()}
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    assert out["nnz"].tolist() == [s.size for s in sets]
    assert out["union_prefix"].tolist() == oracle.union_sizes(sets, R).tolist()
    for a in range(W):
        assert out["even_split"][a].tolist() == oracle.skewness(sets[a], R, n)[1].tolist()
    rng = np.random.default_rng(cid)
    for a, b in rng.integers(0, W, size=(12, 2)):      # sampled pairs
        m = min(sets[a].size, sets[b].size)
        assert out["overlap"][a][b] / m == oracle.overlap_ratio(sets[a], sets[b], R)


def test_hashed_encode_full_size(oracle, zen):
    """One worker of the recommendation workload through Algorithm 1's hash memory with the paper's
    parameters (k = 3, r1 = 2 nnz over all partitions, r2 = r1 / 10)."""
    import gpu_util as G

    wl = WORKLOADS[3]
    R, D, n = wl.n_rows, wl.row_dim, wl.n_parts
    rows, vals = worker_sparse(wl, 5)
    grad = G.dense_device(wl, rows, vals)
    ctx = zen.ZenContext(R, D, n, wl.hash_seed, zen.ZEN_INDEX_COO)
    r1 = 2 * rows.size // n
    r2 = r1 // 10
    mem = zen.alloc_workspace(zen.zen_hash_memory_bytes(ctx, 3, 4242, r1, r2))
    ws = zen.alloc_workspace(zen.zen_encode_hashed_workspace_bytes(ctx, 3, 4242, r1, r2))
    out = zen.alloc_encoded(ctx, rows.size)
    serial = torch.zeros(n, dtype=torch.int32, device="cuda")
    zen.zen_encode_hashed(ctx, grad, 3, 4242, r1, r2, mem, out, serial, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    part = (oracle.hash_many(rows, wl.hash_seed) % np.uint32(n)).astype(np.uint16)
    ref_off, ref_idx = oracle.partition(rows, part, n)
    off, idx = G.u32(out.offsets), G.u32(out.indices[:rows.size])
    assert np.array_equal(off, ref_off)
    for p in range(n):
        assert np.array_equal(np.sort(idx[off[p]:off[p + 1]]), ref_idx[off[p]:off[p + 1]])
    got = out.values[:rows.size].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), vals[np.searchsorted(rows, idx)].view(np.uint32))
    share = float(serial.sum().item()) / rows.size
    assert 0.01 < share < 0.06                          # ~ 0.5^3 / 4 with three hash functions at load 0.5


def test_topk_threshold_full_size(oracle, zen):
    n = 1 << 26
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    g = torch.randn(n, dtype=torch.float32, device="cuda", generator=gen)
    ws = zen.alloc_workspace(zen.zen_topk_workspace_bytes())
    thr = torch.zeros(2, dtype=torch.int32, device="cuda")
    host = g.cpu().numpy()
    zen.zen_topk_threshold(g, n // 20, thr[0:1], ws)                               # exact top 5 %
    zen.zen_topk_threshold(g, (n // 100) // 20, thr[1:2], ws, first=0, stride=100)  # from a 1 % sample
    t = thr.cpu().numpy().view(np.uint32)
    mag = np.abs(host).view(np.uint32)
    assert int((mag >= t[0]).sum()) == n // 20 and int((mag > t[0]).sum()) < n // 20   # the k-th largest, exactly
    assert int(t[1]) == oracle.topk_threshold(host, (n // 100) // 20, 0, 100)
    ctx = zen.ZenContext(n, 1, 16, 3, zen.ZEN_INDEX_COO)
    out = zen.alloc_encoded(ctx, n // 20)
    ews = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
    zen.zen_encode_batch_sparsified(ctx, [g.view(n, 1)], thr[0:1], [out], ews)
    assert zen.zen_status_fetch(ctx, ews) == (0, 0, 0)
    import gpu_util as G

    off = G.u32(out.offsets)
    kept = np.flatnonzero(mag >= t[0]).astype(np.uint32)
    r_off, r_idx = oracle.partition(kept, (oracle.hash_many(kept, 3) % np.uint32(16)).astype(np.uint16), 16)
    assert np.array_equal(off, r_off) and np.array_equal(G.u32(out.indices[:kept.size]), r_idx)
    assert np.array_equal(out.values[:kept.size].cpu().numpy().reshape(-1).view(np.uint32), host[r_idx].view(np.uint32))
