"""Pins for the oracle's Pull side: membership bitmap of an aggregated partition (Algorithm 2,
hash_bitmap_encode at the server), decode + dense placement at the worker, and the end-to-end
property that the synchronized tensor is the dense sum of the workers' gradients (section "Elemental
Dimensions for Synchronization")."""
import numpy as np
import pytest

import brute
from workloads import MINI_WORKLOADS, dense_from_sparse, worker_sparse


def test_paper_worked_example_pull(oracle):
    # section "Hash Bitmap", worked example: |G| = 15, three servers, server 0's set holds (1-based)
    # {2, 5, 7, 11, 14}; the aggregated non-zeros {5, 7} are its second and third members.
    owner = np.array([0 if (r + 1) in (2, 5, 7, 11, 14) else 1 + (r % 2) for r in range(15)], np.uint16)
    member = oracle.member_mask([4, 6], 15)
    assert member.tolist() == [0, 0, 0, 0, 1, 0, 1] + [0] * 8
    _, word_off = oracle.bitmap_layout(owner, 3)
    bm = oracle.bitmap_encode(owner, 3, member, word_off)
    assert int(bm[0]) == 0b110
    vals = [np.array([[10.0], [20.0]], np.float32), np.zeros((0, 1), np.float32), np.zeros((0, 1), np.float32)]
    dense = oracle.pull_apply(owner, 3, 1, word_off, bm, vals)
    expect = np.zeros((15, 1), np.float32)
    expect[4], expect[6] = 10.0, 20.0
    assert np.array_equal(dense, expect)


@pytest.mark.parametrize("R,D,n", [(1, 1, 1), (33, 1, 3), (97, 3, 5), (1000, 4, 7), (4099, 2, 64)])
def test_densify_and_pull_apply_match_brute_force(oracle, R, D, n):
    rng = np.random.default_rng(R * 31 + n)
    owner = oracle.owner_table(R, n, int(rng.integers(0, 2**32)))
    for density in (0.0, 0.1, 0.7, 1.0):
        present = np.flatnonzero(rng.random(R) < density).astype(np.uint32)
        vals = rng.standard_normal((present.size, D)).astype(np.float32)
        if present.size:
            vals[0] = 0.0                                   # a cancelled sum: present, value zero
        parts = [(present[owner[present] == p], vals[owner[present] == p]) for p in range(n)]
        expect = brute.densify(parts, R, D)
        assert np.array_equal(oracle.densify(parts, R, D).view(np.uint32), expect.view(np.uint32))
        # shuffled part order and shuffled rows inside a part give the same dense tensor
        perm = rng.permutation(n)
        shuf = []
        for p in perm:
            o = rng.permutation(parts[p][0].size)
            shuf.append((parts[p][0][o], parts[p][1][o]))
        assert np.array_equal(oracle.densify(shuf, R, D).view(np.uint32), expect.view(np.uint32))
        # bitmap form
        _, word_off = oracle.bitmap_layout(owner, n)
        bm = oracle.bitmap_encode(owner, n, oracle.member_mask(present, R), word_off)
        assert sum(bin(int(w)).count("1") for w in bm) == present.size       # zero-valued row kept its bit
        got = oracle.pull_apply(owner, n, D, word_off, bm, [v for _, v in parts])
        assert np.array_equal(got.view(np.uint32), expect.view(np.uint32))


def test_pull_errors(oracle):
    with pytest.raises(ValueError):
        oracle.densify([([1, 1], np.ones((2, 1), np.float32))], 4, 1)                      # duplicate
    with pytest.raises(ValueError):
        oracle.densify([([1], np.ones((1, 1), np.float32)), ([1], np.ones((1, 1), np.float32))], 4, 1)
    with pytest.raises(ValueError):
        oracle.densify([([4], np.ones((1, 1), np.float32))], 4, 1)                         # out of range
    with pytest.raises(ValueError):
        oracle.member_mask([9], 9)
    owner = np.zeros(40, np.uint16)
    _, word_off = oracle.bitmap_layout(owner, 1)
    bm = oracle.bitmap_encode(owner, 1, oracle.member_mask([3, 35], 40), word_off)
    with pytest.raises(ValueError):
        oracle.pull_apply(owner, 1, 1, word_off, bm, [np.ones((3, 1), np.float32)])        # 2 bits, 3 rows


def test_round_trip_of_one_gradient(oracle):
    rng = np.random.default_rng(5)
    R, D, n = 777, 5, 6
    g = np.zeros((R, D), np.float32)
    rows = rng.choice(R, 200, replace=False)
    g[rows] = rng.standard_normal((200, D)).astype(np.float32)
    enc = oracle.encode(g, R, D, n, 11)
    parts = [(enc.indices[enc.offsets[p]:enc.offsets[p + 1]], enc.values[enc.offsets[p]:enc.offsets[p + 1]])
             for p in range(n)]
    assert np.array_equal(oracle.densify(parts, R, D).view(np.uint32), g.view(np.uint32))


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_end_to_end_equals_dense_sum(oracle, cfg):
    """encode on every worker -> aggregate at every server -> bitmap -> decode + place = the dense
    all-reduce of the workers' gradients, computed here by a plain fp64 numpy sum."""
    wl = MINI_WORKLOADS[cfg]
    R, D, n = wl.n_rows, wl.row_dim, wl.n_parts
    total = np.zeros((R, D), np.float64)
    encs = []
    for w in range(wl.n_workers):
        rows, vals = worker_sparse(wl, w)
        g = dense_from_sparse(wl, rows, vals)
        total += g.reshape(R, D).astype(np.float64)
        encs.append(oracle.encode(g, R, D, n, wl.hash_seed))
    aggs = []
    for j in range(n):
        parts = [(e.indices[e.offsets[j]:e.offsets[j + 1]], e.values[e.offsets[j]:e.offsets[j + 1]]) for e in encs]
        aggs.append(oracle.aggregate(parts, R, D, want_f64=False))
    owner = oracle.owner_table(R, n, wl.hash_seed)
    _, word_off = oracle.bitmap_layout(owner, n)
    all_idx = np.concatenate([a.indices for a in aggs])
    bm = oracle.bitmap_encode(owner, n, oracle.member_mask(all_idx, R), word_off)
    for j in range(n):                                                   # decode gives back each server's set
        assert np.array_equal(oracle.bitmap_decode(owner, j, bm[int(word_off[j]):int(word_off[j + 1])]), aggs[j].indices)
    dense = oracle.pull_apply(owner, n, D, word_off, bm, [a.values for a in aggs])
    assert np.array_equal(dense, total.astype(np.float32))
    assert np.array_equal(dense, oracle.densify([(a.indices, a.values) for a in aggs], R, D))
