"""Pins for the oracle's aggregation and for encode -> aggregate end to end."""
import numpy as np
import pytest

import brute
from workloads import MINI_WORKLOADS, worker_sparse, dense_from_sparse


def _rand_parts(rng, R, D, n_in, max_count, dup=False):
    parts = []
    for _ in range(n_in):
        c = int(rng.integers(0, max_count + 1))
        idx = rng.choice(R, size=min(c, R), replace=dup).astype(np.uint32)
        rng.shuffle(idx)
        val = rng.standard_normal((idx.size, D)).astype(np.float32)
        parts.append((idx, val))
    return parts


@pytest.mark.parametrize("R,D,n_in", [(10, 1, 1), (50, 1, 4), (64, 3, 5), (200, 8, 8), (17, 64, 3)])
@pytest.mark.parametrize("dup", [False, True])
def test_aggregate_matches_dense_sum(oracle, R, D, n_in, dup):
    rng = np.random.default_rng(R + D + n_in + 17 * dup)
    parts = _rand_parts(rng, R, D, n_in, R // 2 + 1, dup)
    acc, touched = brute.aggregate_dense(parts, R, D)
    out = oracle.aggregate(parts, R, D)
    assert out.U == len(touched)
    assert out.indices.tolist() == touched                           # ascending union
    assert np.array_equal(out.sum64, acc[touched])                   # same fp64 sums, same order
    assert np.array_equal(out.values, acc[touched].astype(np.float32))
    nc = np.zeros(R, np.int64)
    for idx, _ in parts:
        np.add.at(nc, idx.astype(np.int64), 1)
    assert np.array_equal(out.ncontrib, nc[touched])
    absacc, _ = brute.aggregate_dense([(i, np.abs(v)) for i, v in parts], R, D)
    assert np.allclose(out.abs64, absacc[touched], rtol=0, atol=0)
    # U <= sum of counts
    assert out.U <= sum(i.size for i, _ in parts)


def test_disjoint_inputs_give_sorted_concatenation_bit_exact(oracle):
    rng = np.random.default_rng(5)
    perm = rng.permutation(300).astype(np.uint32)
    parts = [(perm[i * 100:(i + 1) * 100], rng.standard_normal((100, 4)).astype(np.float32)) for i in range(3)]
    out = oracle.aggregate(parts, 300, 4)
    all_idx = np.concatenate([p[0] for p in parts])
    all_val = np.concatenate([p[1] for p in parts])
    order = np.argsort(all_idx)
    assert np.array_equal(out.indices, all_idx[order])
    assert np.array_equal(out.values.view(np.uint32), all_val[order].view(np.uint32))
    assert np.all(out.ncontrib == 1)


@pytest.mark.parametrize("m", [2, 3, 8])
def test_identical_inputs_scale_values(oracle, m):
    rng = np.random.default_rng(m)
    idx = rng.choice(1000, 64, replace=False).astype(np.uint32)
    val = rng.standard_normal((64, 2)).astype(np.float32)
    out = oracle.aggregate([(idx, val)] * m, 1000, 2)
    order = np.argsort(idx)
    assert np.array_equal(out.indices, idx[order])
    assert np.array_equal(out.sum64, val[order].astype(np.float64) * m)
    if m in (2, 8):                                                   # power of two: exact in fp32 too
        assert np.array_equal(out.values, val[order] * np.float32(m))


def test_cancelling_sum_keeps_the_index(oracle):
    idx = np.array([3, 9], np.uint32)
    a = np.array([[1.5], [2.0]], np.float32)
    out = oracle.aggregate([(idx, a), (idx[:1], -a[:1])], 16, 1)
    assert out.indices.tolist() == [3, 9]
    assert out.values[:, 0].tolist() == [0.0, 2.0]


def test_capacity_and_bad_index(oracle):
    idx = np.arange(10, dtype=np.uint32)
    val = np.ones((10, 1), np.float32)
    assert oracle.aggregate([(idx, val)], 10, 1, cap_rows=4).U == -10
    assert oracle.aggregate([(idx + 5, val)], 10, 1).U < 0           # index >= R is rejected
    assert oracle.aggregate([], 10, 1).U == 0


@pytest.mark.parametrize("cid", [1, 2, 3, 5])
def test_end_to_end_equals_dense_allreduce(oracle, cid):
    # section "Elemental Dimensions for Synchronization": the outcome of synchronization is that
    # gradients with the same indices are aggregated.  Concatenating the n servers' outputs and
    # densifying must equal the dense fp64 sum of the n workers' gradients.
    wl = MINI_WORKLOADS[cid]
    R, D, n = wl.n_rows, wl.row_dim, wl.n_parts
    n_workers = min(wl.n_workers, 6)
    encs, dense_sum, union = [], np.zeros((R, D), np.float64), set()
    nnzs = []
    for w in range(n_workers):
        rows, vals = worker_sparse(wl, w)
        g = dense_from_sparse(wl, rows, vals)
        dense_sum += g
        union.update(rows.tolist())
        nnzs.append(rows.size)
        encs.append(oracle.encode(g, R, D, n, wl.hash_seed))
    got_rows, got = [], np.zeros((R, D), np.float64)
    sizes = []
    for j in range(n):
        parts = [(e.indices[e.offsets[j]:e.offsets[j + 1]], e.values[e.offsets[j]:e.offsets[j + 1]]) for e in encs]
        out = oracle.aggregate(parts, R, D)
        assert np.all(oracle.hash_many(out.indices, wl.hash_seed) % np.uint32(n) == j)
        got[out.indices.astype(np.int64)] = out.sum64
        got_rows.extend(out.indices.tolist())
        sizes.append(out.U)
    assert sorted(got_rows) == sorted(union) and len(got_rows) == len(union)
    assert np.array_equal(got, dense_sum)        # few addends of fp32 values: fp64 sums are exact
    U = len(union)
    gamma = U / np.mean(nnzs)                     # densification ratio, section C2: 1 <= gamma <= n
    assert 1.0 <= gamma <= n_workers
    if U > 20 * n:
        # Theorem 2, Pull side
        assert oracle.imbalance(sizes) <= 1 + 3 * np.sqrt(n * np.log(n) / U)
