"""Pins for the oracle's Algorithm 1 mechanism (hash memory with parallel and serial regions)."""
import os

import numpy as np
import pytest

import brute

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hier_hash_example.txt")


def _gold():
    d = {}
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            d[k] = int(v)
    return d


def test_figure_example(oracle):
    g = _gold()
    r1, r2 = g["parallel_cells"], g["serial_cells"]
    a, b = g["h1_location_1based"] - 1, g["h2_location_1based"] - 1
    # two earlier indices occupy the first and the fourth location of partition 1; the third index
    # collides with both and must land in the first serial cell
    I = np.array([10, 20, 30], np.uint32)
    part = [1, 1, 1]
    h1 = [a, b, a]
    h2 = [2, 2, b]
    r = oracle.hierarchical_hash(I, part, [h1, h2], 2, r1, r2)
    assert r.rc == 0
    assert int(r.x[1, a]) == 10 and int(r.x[1, b]) == 20
    assert int(r.x[1, g["serial_location_1based"] - 1]) == 30
    assert r.serial_count.tolist() == [0, 1]
    assert (r.x[0] == 0xFFFFFFFF).all() and int((r.x[1] != 0xFFFFFFFF).sum()) == 3
    assert r.offsets.tolist() == [0, 0, 3] and r.indices.tolist() == [10, 20, 30]      # memory order


@pytest.mark.parametrize("R,n,k,load", [(50, 1, 1, 0.5), (3000, 4, 3, 0.5), (3000, 7, 2, 1.0), (20000, 64, 4, 0.5),
                                        (20000, 16, 3, 0.25)])
def test_lossless_and_matches_brute_force(oracle, R, n, k, load):
    rng = np.random.default_rng(R + n + k)
    I = np.flatnonzero(rng.random(R) < 0.3).astype(np.uint32)
    seed0 = int(rng.integers(0, 2**32))
    part = (oracle.hash_many(I, seed0) % np.uint32(n)).astype(np.uint16)
    r1 = max(1, int(np.ceil(I.size / n / load)))
    r2 = I.size                                           # can never overflow
    slots = [oracle.hash_slots(I, 1000 + i, r1) for i in range(k)]
    assert all(int(s.max(initial=0)) < r1 for s in slots)
    r = oracle.hierarchical_hash(I, part, slots, n, r1, r2)
    assert r.rc == 0
    mem, serial = brute.hier_hash(I, part, slots, n, r1, r2)
    assert r.serial_count.tolist() == serial
    for p in range(n):
        assert [None if v == 0xFFFFFFFF else int(v) for v in r.x[p]] == mem[p]
    # lossless: every index exactly once, in the partition h0 names (the result of oracle.partition)
    off, idx = oracle.partition(I, part, n)
    assert np.array_equal(r.offsets, off)
    for p in range(n):
        assert np.array_equal(np.sort(r.indices[off[p]:off[p + 1]]), idx[off[p]:off[p + 1]])
    # with one hash function the split between parallel and serial memory does not depend on the order
    if k == 1:
        for p in range(n):
            mine = slots[0][part == p]
            assert serial[p] == mine.size - np.unique(mine).size
        perm = rng.permutation(I.size)
        r_perm = oracle.hierarchical_hash(I[perm], part[perm], [slots[0][perm]], n, r1, r2)
        assert r_perm.serial_count.tolist() == serial


def test_serial_memory_overflow_is_an_error(oracle):
    I = np.arange(40, dtype=np.uint32)
    part = np.zeros(40, np.uint16)
    slots = [np.zeros(40, np.uint32)]                     # everything collides on cell 0
    ok = oracle.hierarchical_hash(I, part, slots, 1, 4, 39)
    assert ok.rc == 0 and ok.serial_count.tolist() == [39] and np.array_equal(np.sort(ok.indices), I)
    bad = oracle.hierarchical_hash(I, part, slots, 1, 4, 38)
    assert bad.rc == 2 and bad.needed_r2 == 39


def test_more_hash_functions_mean_fewer_serial_writes(oracle):
    # section "Data-independent Hierarchical Hashing", Technique #2, and the parameter study: with a
    # parallel memory of twice the number of indices the share of serial writes falls with k and is
    # around one percent with four hash functions (filling a table to load a, an index fails k probes
    # with probability ~ a^k, averaged over the fill: ~ 0.5^k / (k + 1))
    rng = np.random.default_rng(4)
    nnz, n = 200000, 16
    I = np.sort(rng.choice(10_000_000, nnz, replace=False)).astype(np.uint32)
    part = (oracle.hash_many(I, 9) % np.uint32(n)).astype(np.uint16)
    r1 = 2 * nnz // n
    frac = []
    for k in (1, 2, 3, 4):
        slots = [oracle.hash_slots(I, 77 + i, r1) for i in range(k)]
        r = oracle.hierarchical_hash(I, part, slots, n, r1, nnz)
        assert r.rc == 0
        frac.append(float(r.serial_count.sum()) / nnz)
    assert frac[0] > frac[1] > frac[2] > frac[3]
    for k, f in zip((1, 2, 3, 4), frac):
        assert abs(f - 0.5 ** k / (k + 1)) < 0.35 * 0.5 ** k / (k + 1) + 0.002, (k, f)
    assert frac[3] < 0.015
