"""GPU parity of the top-k threshold sparsifier (radix select, threshold applied inside the encode's
dense scan) and of the sparse-format size counts against the CPU oracle: everything bit-exact."""
import numpy as np
import pytest
import torch

from workloads import Workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


@pytest.fixture(params=["small", "tiled"])
def partition_path(request, monkeypatch):
    import gpu_util as G

    G.use_tuning(monkeypatch, tiled_encode=request.param == "tiled")
    return request.param


def _threshold(zen, g, keep, first=0, stride=1):
    ws = zen.alloc_workspace(zen.zen_topk_workspace_bytes())
    thr = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    zen.zen_topk_threshold(g, keep, thr, ws, first=first, stride=stride)
    return int(thr.cpu().numpy().view(np.uint32)[0])


@pytest.mark.parametrize("n", [1, 7, 1000, 65536, 1_000_003])
def test_topk_threshold(oracle, zen, n):
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * np.exp(rng.standard_normal(n) * 3)).astype(np.float32)
    if n >= 1000:
        x[[3, 17, 500]] = [np.nan, np.inf, -np.inf]
        x[10:40] = 0.0
        x[40:50] = -0.0
        x[60:70] = 1.5                                             # ties
    g = torch.from_numpy(x).cuda()
    for keep in sorted(k for k in {1, 2, max(1, n // 20), max(1, n // 2), n} if k <= n):
        assert _threshold(zen, g, keep) == oracle.topk_threshold(x, keep)
    if n >= 1000:                                                  # sampled, as the paper's sparsifier does
        for first, stride in [(0, 100), (7, 13), (n - 1, 5)]:
            m = (n - first + stride - 1) // stride
            for keep in sorted({1, max(1, m // 20), m}):
                assert _threshold(zen, g, keep, first, stride) == oracle.topk_threshold(x, keep, first, stride)
    ws = zen.alloc_workspace(zen.zen_topk_workspace_bytes())
    thr = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(zen.ZenError):
        zen.zen_topk_threshold(g, 0, thr, ws)
    with pytest.raises(zen.ZenError):
        zen.zen_topk_threshold(g, n + 1, thr, ws)


@pytest.mark.parametrize("fmt", ["coo", "bitmap"])
@pytest.mark.parametrize("R,n", [(33, 3), (5000, 4), (70001, 64), (300000, 16), (1 << 20, 7)])
def test_encode_with_threshold_equals_encode_of_thresholded_tensor(oracle, zen, partition_path, R, n, fmt):
    import gpu_util as G

    rng = np.random.default_rng(R + n)
    seed = int(rng.integers(0, 2**32))
    ctx = zen.ZenContext(R, 1, n, seed, zen.ZEN_INDEX_BITMAP if fmt == "bitmap" else zen.ZEN_INDEX_COO)
    hosts = [(rng.standard_normal(R) * (rng.random(R) < d)).astype(np.float32) for d in (1.0, 0.3, 0.01)]
    grads = [torch.from_numpy(h.reshape(R, 1)).cuda() for h in hosts]
    ws_t = zen.alloc_workspace(zen.zen_topk_workspace_bytes())
    thr = torch.zeros(len(grads), dtype=torch.int32, device="cuda")
    keeps = [max(1, R // 20), max(1, R // 100), 1]
    for w, (g, k) in enumerate(zip(grads, keeps)):
        zen.zen_topk_threshold(g, k, thr[w:w + 1], ws_t)
    outs = [zen.alloc_encoded(ctx, R) for _ in grads]
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, len(grads)))
    zen.zen_encode_batch_sparsified(ctx, grads, thr, outs, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    thr_h = thr.cpu().numpy().view(np.uint32)
    for h, k, t, enc, g in zip(hosts, keeps, thr_h, outs, grads):
        assert int(t) == oracle.topk_threshold(h, k)
        sparse, kept = oracle.threshold_apply(h, int(t))
        ref = oracle.encode(sparse, R, 1, n, seed)
        assert ref.nnz == kept
        assert np.array_equal(G.u32(enc.offsets), ref.offsets)
        assert np.array_equal(G.u32(enc.indices[:ref.nnz]), ref.indices)
        assert np.array_equal(enc.values[:ref.nnz].cpu().numpy().view(np.uint32), ref.values.view(np.uint32))
        assert np.array_equal(g.cpu().numpy().reshape(-1).view(np.uint32), h.view(np.uint32))   # the tensor is untouched
    # thresholds 0 and 1 are the plain encode
    thr.fill_(0)
    thr[1] = 1
    zen.zen_encode_batch_sparsified(ctx, grads, thr, outs, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    for h, enc in zip(hosts, outs):
        ref = oracle.encode(h, R, 1, n, seed)
        assert np.array_equal(G.u32(enc.offsets), ref.offsets) and np.array_equal(G.u32(enc.indices[:ref.nnz]), ref.indices)


def test_threshold_needs_an_elementwise_context(zen):
    ctx = zen.ZenContext(1000, 4, 4, 1, zen.ZEN_INDEX_COO)
    g = torch.zeros((1000, 4), dtype=torch.float32, device="cuda")
    out = zen.alloc_encoded(ctx, 10)
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
    with pytest.raises(zen.ZenError):
        zen.zen_encode_batch_sparsified(ctx, [g], torch.zeros(1, dtype=torch.int32, device="cuda"), [out], ws)


@pytest.mark.parametrize("R,D,block", [(1000, 1, 32), (70001, 1, 256), (1 << 20, 1, 256), (9001, 64, 64), (333, 256, 32)])
def test_format_counts_and_sizes(oracle, zen, R, D, block):
    from workloads import dense_from_sparse

    rng = np.random.default_rng(R + D)
    wl = Workload("t", 0, R, D, 16, 5, "uniform")
    ctx = zen.ZenContext(R, D, 16, 5, zen.ZEN_INDEX_COO)
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
    counts = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    for dens in (0.0, 0.003, 0.2, 1.0):
        rows = np.flatnonzero(rng.random(R) < dens).astype(np.uint32)
        vals = rng.standard_normal((rows.size, D)).astype(np.float32) + 4.0
        g = torch.from_numpy(dense_from_sparse(wl, rows, vals)).cuda()
        zen.zen_format_count(ctx, g, block, counts, ws)
        c = counts.cpu().numpy()
        assert int(c[0]) == rows.size and int(c[1]) == oracle.nonzero_blocks(rows, R, block)
        got = zen.zen_format_bytes(R, int(c[0]), 16, int(c[1]), block)
        assert got == oracle.format_bytes(R, rows.size, 16, oracle.nonzero_blocks(rows, R, block), block)
    with pytest.raises(zen.ZenError):
        zen.zen_format_count(ctx, g, 48, counts, ws)               # not whole mask words per block
