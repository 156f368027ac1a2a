"""Pins for the oracle's sparsity metrics (section "Characteristics of Sparse Tensors") and the two
communication-time formulas that decide the synchronization scheme (Equations 1 and 2)."""
import math

import numpy as np
import pytest

from workloads import WORKLOADS, worker_sparse


def test_overlap_ratio_definition_and_extremes(oracle):
    a = np.array([1, 4, 7, 9], np.uint32)
    assert oracle.overlap_ratio(a, a, 10) == 1.0                       # identical sets
    assert oracle.overlap_ratio(a, [0, 2, 3], 10) == 0.0               # disjoint sets
    assert oracle.overlap_ratio(a, [4, 9, 2, 3, 5, 6], 10) == 2 / 4    # |{4, 9}| / min(4, 6)
    assert oracle.overlap_ratio([4], a, 10) == 1.0                     # a subset overlaps fully
    assert oracle.overlap_ratio([], a, 10) == 0.0
    rng = np.random.default_rng(0)
    for _ in range(20):
        R = int(rng.integers(5, 400))
        s1 = np.flatnonzero(rng.random(R) < rng.random()).astype(np.uint32)
        s2 = np.flatnonzero(rng.random(R) < rng.random()).astype(np.uint32)
        want = len(set(s1.tolist()) & set(s2.tolist())) / min(s1.size, s2.size) if min(s1.size, s2.size) else 0.0
        assert oracle.overlap_ratio(s1, s2, R) == want
        assert oracle.overlap_ratio(s2[::-1].copy(), s1, R) == want    # symmetric, order-free


def test_union_sizes_and_densification(oracle):
    sets = [[0, 1, 2], [2, 3], [0, 3], [9]]
    assert oracle.union_sizes(sets, 10).tolist() == [3, 4, 4, 5]
    # fully overlapped tensors do not get denser; disjoint ones add up ("two extreme cases")
    same = [np.arange(0, 100, 2)] * 8
    assert oracle.union_sizes(same, 100).tolist() == [50] * 8
    disjoint = [np.arange(10 * w, 10 * w + 10) for w in range(8)]
    assert oracle.union_sizes(disjoint, 100).tolist() == [10 * (w + 1) for w in range(8)]
    rng = np.random.default_rng(1)
    R = 5000
    sets = [np.flatnonzero(rng.random(R) < 0.05).astype(np.uint32) for _ in range(16)]
    u = oracle.union_sizes(sets, R)
    acc = set()
    for w, s_ in enumerate(sets):
        acc |= set(s_.tolist())
        assert int(u[w]) == len(acc)
    gamma = u[-1] / R / np.mean([s_.size / R for s_ in sets])
    assert 1.0 < gamma < 16.0                                           # gamma_G^n < n (section C2)
    with pytest.raises(ValueError):
        oracle.union_sizes([[R]], R)


def test_skewness_ratio(oracle):
    # all non-zeros in the first of four even partitions: max density = 4 x the tensor's density
    r, part = oracle.skewness(np.arange(10, dtype=np.uint32), 400, 4)
    assert r == 4.0 and part.tolist() == [10, 0, 0, 0]
    r, _ = oracle.skewness(np.arange(0, 400, 4, dtype=np.uint32), 400, 4)
    assert r == 1.0                                                     # evenly spread
    # |G| not divisible by n: partitions of ceil(|G|/n) rows, the last one shorter
    r, part = oracle.skewness(np.array([0, 9], np.uint32), 10, 3)       # sizes 4, 4, 2
    assert part.tolist() == [1, 0, 1] and r == pytest.approx((1 / 2) / (2 / 10))
    assert oracle.skewness([], 10, 3)[0] == 0.0
    # the language-model workload puts well over 60 % of its non-zero rows into the first of eight
    # even partitions (section C3 observes "over 60%" for the paper's models)
    wl = WORKLOADS[2]
    rows, _ = worker_sparse(wl, 0, want_values=False)
    r, part = oracle.skewness(rows, wl.n_rows, 8)
    assert part[0] / rows.size > 0.6 and r == pytest.approx(8 * part[0] / rows.size)
    brute = np.bincount(rows // (wl.n_rows // 8), minlength=8)
    assert part.tolist() == brute.tolist()


@pytest.mark.parametrize("n", [2, 4, 16, 64, 128])
def test_communication_times_extreme_cases(oracle, n):
    # section "Balanced Parallelism as the practical optimal scheme": with full overlap every gamma is
    # 1 and the two sums are log n and 2(n-1)/n; with no overlap gamma^k = k and they are n-1 and
    # (n-1)(1+1/n)
    d, M, b = 0.01, 4e9, 12.5e9
    unit = 2 * M * d / b
    stages = int(math.log2(n))
    full = [1.0] * stages
    assert oracle.time_hierarchical_centralization(n, full, d, M, b) == pytest.approx(stages * unit)
    assert oracle.time_balanced_parallelism(n, 1.0, d, M, b) == pytest.approx(2 * (n - 1) / n * unit)
    none = [float(2 ** i) for i in range(stages)]
    assert oracle.time_hierarchical_centralization(n, none, d, M, b) == pytest.approx((n - 1) * unit)
    assert oracle.time_balanced_parallelism(n, float(n), d, M, b) == pytest.approx((n - 1) * (1 + 1 / n) * unit)
    # so Balanced Parallelism wins under full overlap for n > 2 and loses, narrowly, with none
    if n > 2:
        assert oracle.time_balanced_parallelism(n, 1.0, d, M, b) < oracle.time_hierarchical_centralization(n, full, d, M, b)
    assert oracle.time_balanced_parallelism(n, float(n), d, M, b) > oracle.time_hierarchical_centralization(n, none, d, M, b)


def test_balanced_parallelism_wins_at_low_overlap_with_16_gpus(oracle):
    # same section: with n = 16, Balanced Parallelism is better "even if the overlap ratio of any two
    # tensors is as low as 0.05".  Independent uniformly random tensors of density 0.05 overlap
    # pairwise by 0.05 (a shared core instead would make the union grow faster and flip the order).
    rng = np.random.default_rng(16)
    R = 1_000_000
    sets = [np.flatnonzero(rng.random(R) < 0.05).astype(np.uint32) for _ in range(16)]
    assert oracle.overlap_ratio(sets[0], sets[9], R) == pytest.approx(0.05, abs=0.003)
    u = oracle.union_sizes(sets, R)
    d = float(np.mean([s_.size for s_ in sets])) / R
    gamma = [u[k - 1] / R / d for k in (1, 2, 4, 8, 16)]
    assert gamma[4] == pytest.approx((1 - 0.95 ** 16) / 0.05, rel=0.01)
    t_bp = oracle.time_balanced_parallelism(16, gamma[4], d, 4.0 * R, 1e9)
    t_sm = oracle.time_hierarchical_centralization(16, gamma[:4], d, 4.0 * R, 1e9)
    assert t_bp < t_sm
