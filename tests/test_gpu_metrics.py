"""GPU parity of the sparsity counts (overlap, densification, skewness inputs) and of the two
communication-time formulas against the CPU oracle: integer counts bit-exact, ratios and times to
double rounding."""
import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, Workload, dense_from_sparse, worker_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


def _check(oracle, zen, R, D, n, sets, grads, ctx):
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, len(grads)))
    out = {k: v.cpu().numpy() for k, v in zen.zen_sparsity_count(ctx, grads, ws).items()}
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    W = len(sets)
    assert out["nnz"].tolist() == [s.size for s in sets]
    assert out["union_prefix"].tolist() == oracle.union_sizes(sets, R).tolist()
    for a in range(W):
        skew, part = oracle.skewness(sets[a], R, n)
        assert out["even_split"][a].tolist() == part.tolist()
        if sets[a].size:                                      # the ratio formed from the counts
            size = -(-R // n)
            dens = [out["even_split"][a][i] / min(size, R - i * size) for i in range(n) if i * size < R]
            assert max(dens) / (sets[a].size / R) == pytest.approx(skew, rel=1e-12)
        for b in range(W):
            m = min(sets[a].size, sets[b].size)
            ratio = out["overlap"][a][b] / m if m else 0.0
            assert ratio == oracle.overlap_ratio(sets[a], sets[b], R)
    assert np.array_equal(out["overlap"], out["overlap"].T)


@pytest.mark.parametrize("R,D,n,W", [(1, 1, 1, 1), (1000, 1, 7, 3), (70001, 1, 64, 5), (300000, 1, 1000, 2),
                                     (1 << 20, 1, 3, 64), (9001, 64, 16, 16), (333, 256, 8, 4), (40000, 4, 1000, 2),
                                     # even partitions of fewer than 32 rows: a mask word spans several of them
                                     (100, 1, 10, 3), (333, 1, 64, 4), (1000, 4, 100, 2), (5000, 1, 1000, 3),
                                     (70, 8, 64, 2)])
def test_sparsity_counts_random(oracle, zen, R, D, n, W):
    rng = np.random.default_rng(R + D + n + W)
    wl = Workload("t", 0, R, D, n, 5, "uniform")
    ctx = zen.ZenContext(R, D, n, 5, zen.ZEN_INDEX_COO)
    sets, grads = [], []
    for w in range(W):
        dens = [0.0, 0.01, 0.3, 1.0][w % 4] if W > 1 else 0.2
        rows = np.flatnonzero(rng.random(R) < dens).astype(np.uint32)
        if w % 5 == 4:                                        # a clustered tensor: one long run
            rows = np.arange(R // 3, min(R, R // 3 + 5000), dtype=np.uint32)
        vals = rng.standard_normal((rows.size, D)).astype(np.float32) + 4.0
        sets.append(rows)
        grads.append(torch.from_numpy(dense_from_sparse(wl, rows, vals)).cuda())
    _check(oracle, zen, R, D, n, sets, grads, ctx)


@pytest.mark.parametrize("cid", [1, 2, 3, 5])
def test_sparsity_counts_workloads(oracle, zen, cid):
    import gpu_util as G

    wl = MINI_WORKLOADS[cid]
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed, zen.ZEN_INDEX_COO)
    sparse = [worker_sparse(wl, w) for w in range(wl.n_workers)]
    grads = [G.dense_device(wl, r, v) for r, v in sparse]
    _check(oracle, zen, wl.n_rows, wl.row_dim, wl.n_parts, [r for r, _ in sparse], grads, ctx)


def test_scheme_times_match_the_formulas(oracle, zen):
    rng = np.random.default_rng(3)
    for n in (2, 4, 16, 128):
        stages = n.bit_length() - 1
        gam = np.sort(1.0 + rng.random(stages + 1) * n)
        gam[0] = 1.0
        d, M, b = float(rng.random() * 0.1 + 1e-3), 4e9, 12.5e9
        t_bp, t_sm = zen.zen_scheme_times(n, gam, d, M, b)
        assert t_bp == pytest.approx(oracle.time_balanced_parallelism(n, gam[stages], d, M, b), rel=1e-14)
        assert t_sm == pytest.approx(oracle.time_hierarchical_centralization(n, gam[:stages], d, M, b), rel=1e-14)
    with pytest.raises(zen.ZenError):
        zen.zen_scheme_times(6, [1.0, 2.0, 3.0], 0.1, 1.0, 1.0)          # n not a power of two
    with pytest.raises(zen.ZenError):
        zen.zen_scheme_times(4, [1.0, 2.0], 0.1, 1.0, 1.0)               # gamma^n missing
