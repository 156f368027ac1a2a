"""Pins for the oracle's encode (non-zero detection, owner partition, value gather)."""
import numpy as np
import pytest

import brute
from workloads import MINI_WORKLOADS, worker_sparse, dense_from_sparse


def _tiny(rng, R, D, density):
    g = np.zeros((R, D), np.float32)
    rows = np.flatnonzero(rng.random(R) < density)
    for r in rows:
        cols = rng.choice(D, size=rng.integers(1, D + 1), replace=False)
        g[r, cols] = rng.standard_normal(cols.size).astype(np.float32)
    return g


@pytest.mark.parametrize("R,D,n", [(1, 1, 1), (37, 1, 4), (64, 3, 5), (257, 4, 8), (100, 16, 3), (33, 64, 64)])
def test_encode_matches_brute_force(oracle, R, D, n):
    rng = np.random.default_rng(R * 1000 + D * 10 + n)
    for density in (0.0, 0.1, 0.7, 1.0):
        g = _tiny(rng, R, D, density)
        g[g == 0] = 0.0
        seed = int(rng.integers(0, 2**32))
        own = oracle.owner_table(R, n, seed)
        b_off, b_idx, b_val = brute.encode(g, own, n)
        enc = oracle.encode(g, R, D, n, seed)
        assert enc.rc == 0
        assert enc.offsets.tolist() == b_off
        assert enc.indices.tolist() == b_idx
        assert enc.nnz == len(b_idx)
        if b_idx:
            assert np.array_equal(enc.values.view(np.uint32), np.stack(b_val).view(np.uint32))
        # stepwise entry points agree with the one-shot encode
        I = oracle.nonzero(g, R, D)
        assert I.tolist() == brute.nonzero_rows(g)
        off2, idx2 = oracle.partition(I, own[I], n)
        assert np.array_equal(off2, enc.offsets) and np.array_equal(idx2, enc.indices)
        assert np.array_equal(oracle.gather(g, D, idx2).view(np.uint32), enc.values.view(np.uint32))


def test_special_values(oracle):
    # +0 and -0 are zero; NaN, +-Inf, denormals and the smallest normal are non-zero
    vals = np.array([0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 1.17549435e-38, 1.0, -2.5], np.float32)
    g = vals.reshape(-1, 1)
    I = oracle.nonzero(g, g.shape[0], 1)
    assert I.tolist() == [2, 3, 4, 5, 6, 7, 8, 9]
    # a row is non-zero if ANY element is; the whole row (zeros included) is the value
    g2 = np.zeros((4, 3), np.float32)
    g2[1, 2] = -0.0
    g2[2, 1] = 5.0
    g2[3, 0] = np.float32(1e-45)
    enc = oracle.encode(g2, 4, 3, 1, 0)
    assert enc.indices.tolist() == [2, 3]
    assert np.array_equal(enc.values.view(np.uint32), g2[[2, 3]].view(np.uint32))
    assert enc.offsets.tolist() == [0, 2]


def test_capacity_and_argument_errors(oracle):
    g = np.ones((10, 2), np.float32)
    enc = oracle.encode(g, 10, 2, 4, 1, cap_rows=9)
    assert enc.rc == 2 and enc.nnz == 10
    assert oracle.encode(g, 10, 2, 0, 1, cap_rows=10).rc == 1


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_invariants_on_mini_workloads(oracle, cid):
    wl = MINI_WORKLOADS[cid]
    R, D, n = wl.n_rows, wl.row_dim, wl.n_parts
    owners_by_worker = {}
    for w in range(min(wl.n_workers, 3)):
        rows, vals = worker_sparse(wl, w)
        g = dense_from_sparse(wl, rows, vals)
        enc = oracle.encode(g, R, D, n, wl.hash_seed)
        assert enc.rc == 0
        # the planted rows are exactly the non-zero rows
        assert enc.nnz == rows.size
        off = enc.offsets.astype(np.int64)
        assert off[0] == 0 and off[-1] == rows.size and np.all(np.diff(off) >= 0)   # sizes sum to nnz
        # every non-zero lands in exactly one partition, the one its hash names
        assert np.array_equal(np.sort(enc.indices), rows)
        h = oracle.hash_many(enc.indices, wl.hash_seed) % np.uint32(n)
        for p in range(n):
            seg = enc.indices[off[p]:off[p + 1]]
            assert np.all(h[off[p]:off[p + 1]] == p)
            assert np.all(np.diff(seg.astype(np.int64)) > 0)        # ascending inside a partition
        # values are the rows, bit for bit
        assert np.array_equal(enc.values.view(np.uint32), g[enc.indices.astype(np.int64)].view(np.uint32))
        for r, p in zip(enc.indices.tolist(), h.tolist()):
            assert owners_by_worker.setdefault(r, p) == p            # same idx -> same server on every worker


def test_push_imbalance_obeys_theorem2_shape(oracle):
    # Theorem 2: imbalance of Push <= 1 + Theta(sqrt(n log n / nnz)); we assert the constant <= 3,
    # and the practical "< 1.1" on an index set as large as the paper's examples.
    wl = MINI_WORKLOADS[5]
    rows, _ = worker_sparse(wl, 0, want_values=False)
    for n in (4, 16, 64):
        own = oracle.hash_many(rows, wl.hash_seed) % np.uint32(n)
        sizes = np.bincount(own, minlength=n)
        ratio = oracle.imbalance(sizes)
        assert 1.0 <= ratio <= 1 + 3 * np.sqrt(n * np.log(n) / rows.size)
    idx = np.arange(3_000_000, dtype=np.uint32)     # a clustered (contiguous) index set
    sizes = np.bincount(oracle.hash_many(idx, 7) % np.uint32(128), minlength=128)
    assert oracle.imbalance(sizes) < 1.1
    # the theorem's numeric example: n=128, |G| d = 5e6 -> sqrt(n log n / (|G| d)) < 0.02
    assert np.sqrt(128 * np.log2(128) / 5e6) < 0.02


def test_imbalance_ratio_definition(oracle):
    # section "Balance dimension": 15 gradients, 6 non-zero, 3 GPUs; 4 of them in the middle even
    # partition -> ratio 3*4/6 = 2; balanced (2 each) -> 1
    assert oracle.imbalance([1, 4, 1]) == pytest.approx(2.0)
    assert oracle.imbalance([2, 2, 2]) == pytest.approx(1.0)
    assert oracle.imbalance([0, 0]) == 1.0
