"""Compact battery of oracle pins, runnable on any build of oracle/zen_ref.c:

    python tests/pins_battery.py /path/to/libzen_ref_variant.so      (exit status 0 = every pin holds)

Used by test_oracle_mutations.py in a child process, because a broken oracle may corrupt memory.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)
sys.path.insert(0, os.path.dirname(HERE))

import brute  # noqa: E402


def battery(oracle):
    """Compact pins; raises AssertionError (or any exception) when the oracle is wrong."""
    from sklearn.utils import murmurhash3_32

    # hash: published vectors + library
    assert oracle.hash32(0x87654321, 0) == 0xF55B516B and oracle.hash32(0x87654321, 0x5082EDEE) == 0x2362F9DE
    assert oracle.hash32(0xFFFFFFFF, 0) == 0x76293B50 and oracle.hash32(0, 0) == 0x2362F9DE
    idx = np.arange(0, 5000, 7, dtype=np.uint32)
    assert np.array_equal(oracle.hash_many(idx, 99), murmurhash3_32(idx.view(np.int32), seed=99, positive=True).astype(np.uint32))
    own = oracle.owner_table(4096, 8, 1)
    assert np.array_equal(own, (murmurhash3_32(np.arange(4096, dtype=np.int32), seed=1, positive=True) % 8).astype(np.uint16))
    # encode vs brute force, special values
    rng = np.random.default_rng(0)
    R, D, n = 97, 3, 5
    g = np.zeros((R, D), np.float32)
    rows = rng.choice(R, 30, replace=False)
    g[rows, rng.integers(0, D, 30)] = rng.standard_normal(30).astype(np.float32)
    g[3] = [0.0, -0.0, 0.0]
    g[4] = [0.0, 0.0, 2.0]
    owner = oracle.owner_table(R, n, 77)
    b_off, b_idx, b_val = brute.encode(g, owner, n)
    enc = oracle.encode(g, R, D, n, 77)
    assert enc.rc == 0 and enc.offsets.tolist() == b_off and enc.indices.tolist() == b_idx
    assert np.array_equal(enc.values.view(np.uint32), np.stack(b_val).view(np.uint32))
    # hash bitmap: the paper's worked example (|G| = 15, 3 servers, non-zeros {5, 7} 1-based are the
    # second and third members of server 0's set) + brute force + round trip
    ex_owner = np.array([0 if (r + 1) in (2, 5, 7, 11, 14) else 1 + (r % 2) for r in range(15)], np.uint16)
    nz = np.zeros(15, np.uint8)
    nz[[4, 6]] = 1
    dom_count, word_off = oracle.bitmap_layout(ex_owner, 3)
    bm = oracle.bitmap_encode(ex_owner, 3, nz, word_off)
    assert int(bm[int(word_off[0])]) == 0b110 and int(dom_count.sum()) == 15
    assert oracle.bitmap_decode(ex_owner, 0, bm[int(word_off[0]):int(word_off[1])]).tolist() == [4, 6]
    # domains whose size is an exact multiple of 32 (and an empty one) need no padding word
    dc3, wo3 = oracle.bitmap_layout(np.array([0] * 64 + [2] * 32, np.uint16), 3)
    assert dc3.tolist() == [64, 0, 32] and wo3.tolist() == [0, 2, 2, 3]
    R2, n2 = 1000, 7
    owner2 = oracle.owner_table(R2, n2, 3)
    nz2 = (rng.random(R2) < 0.3).astype(np.uint8)
    dc2, wo2 = oracle.bitmap_layout(owner2, n2)
    assert np.array_equal(np.diff(wo2), (dc2 + np.uint64(31)) // np.uint64(32))
    bm2 = oracle.bitmap_encode(owner2, n2, nz2, wo2)
    ref2 = brute.bitmap(owner2, n2, np.flatnonzero(nz2))
    for p in range(n2):
        words = bm2[int(wo2[p]):int(wo2[p + 1])]
        assert sum(int(w) << (32 * k) for k, w in enumerate(words)) == ref2[p][0]
        dec = oracle.bitmap_decode(owner2, p, words)
        assert dec.tolist() == [r for r in np.flatnonzero(nz2).tolist() if owner2[r] == p]
    # aggregate vs dense sum (duplicates, cancellation)
    parts = []
    for w in range(4):
        i = rng.integers(0, 60, size=25).astype(np.uint32)
        parts.append((i, rng.standard_normal((25, 2)).astype(np.float32)))
    parts.append((np.array([7], np.uint32), -parts[0][1][:1] * 0 + np.float32(1.5)))
    parts.append((np.array([7, 58], np.uint32), np.array([[-1.5, -1.5], [0.25, 0.5]], np.float32)))
    acc, touched = brute.aggregate_dense(parts, 60, 2)
    out = oracle.aggregate(parts, 60, 2)
    assert out.U == len(touched) and out.indices.tolist() == touched
    assert np.array_equal(out.sum64, acc[touched]) and np.array_equal(out.values, acc[touched].astype(np.float32))
    single = oracle.aggregate([(np.array([9, 2], np.uint32), np.array([[1.0, 2.0], [3.0, 4.0]], np.float32))], 60, 2)
    assert single.indices.tolist() == [2, 9] and single.values.tolist() == [[3.0, 4.0], [1.0, 2.0]]
    cancel = oracle.aggregate([(np.array([5], np.uint32), np.ones((1, 2), np.float32)),
                               (np.array([5], np.uint32), -np.ones((1, 2), np.float32))], 60, 2)
    assert cancel.U == 1 and cancel.indices.tolist() == [5]
    # Pull side: worked example continued (values of the second and third member land at rows 5 and 7,
    # 1-based), brute-force placement, partition p reads its own words
    mem = oracle.member_mask([4, 6], 15)
    assert mem.tolist() == [0, 0, 0, 0, 1, 0, 1] + [0] * 8
    d15 = oracle.pull_apply(ex_owner, 3, 1, word_off, oracle.bitmap_encode(ex_owner, 3, mem, word_off),
                            [np.array([[10.0], [20.0]], np.float32), np.zeros((0, 1), np.float32),
                             np.zeros((0, 1), np.float32)])
    assert d15[:, 0].tolist() == [0, 0, 0, 0, 10.0, 0, 20.0] + [0] * 8
    present = np.flatnonzero(nz2).astype(np.uint32)
    pv = rng.standard_normal((present.size, 2)).astype(np.float32)
    pparts = [(present[owner2[present] == p], pv[owner2[present] == p]) for p in range(n2)]
    want = brute.densify(pparts, R2, 2)
    assert np.array_equal(oracle.densify(pparts, R2, 2), want)
    assert np.array_equal(oracle.pull_apply(owner2, n2, 2, wo2, bm2, [v for _, v in pparts]), want)
    try:                                                   # two set bits, three value rows: refused
        oracle.pull_apply(ex_owner, 3, 1, word_off, oracle.bitmap_encode(ex_owner, 3, mem, word_off),
                          [np.ones((3, 1), np.float32), np.zeros((0, 1), np.float32), np.zeros((0, 1), np.float32)])
        raise AssertionError("count mismatch accepted")
    except ValueError:
        pass
    # Algorithm 1's hash memory: the figure's example (first location taken, re-hash to the fourth, taken
    # too, serial cell right behind the parallel memory), brute force, losslessness
    hh = oracle.hierarchical_hash(np.array([10, 20, 30], np.uint32), [1, 1, 1], [[0, 3, 0], [2, 2, 3]], 2, 4, 2)
    assert hh.rc == 0 and hh.x[1].tolist() == [10, 0xFFFFFFFF, 0xFFFFFFFF, 20, 30, 0xFFFFFFFF]
    assert hh.serial_count.tolist() == [0, 1] and hh.indices.tolist() == [10, 20, 30] and hh.offsets.tolist() == [0, 0, 3]
    Ih = np.flatnonzero(rng.random(3000) < 0.3).astype(np.uint32)
    ph = (oracle.hash_many(Ih, 5) % np.uint32(4)).astype(np.uint16)
    r1h = Ih.size // 4 // 2 + 1
    sl = [oracle.hash_slots(Ih, 100 + i, r1h) for i in range(3)]
    assert np.array_equal(sl[0], oracle.hash_many(Ih, 100) % np.uint32(r1h))
    hh = oracle.hierarchical_hash(Ih, ph, sl, 4, r1h, Ih.size)
    mem, ser = brute.hier_hash(Ih, ph, sl, 4, r1h, Ih.size)
    assert hh.rc == 0 and hh.serial_count.tolist() == ser
    assert all([None if v == 0xFFFFFFFF else int(v) for v in hh.x[q]] == mem[q] for q in range(4))
    offh, idxh = oracle.partition(Ih, ph, 4)
    assert np.array_equal(hh.offsets, offh)
    assert all(np.array_equal(np.sort(hh.indices[offh[q]:offh[q + 1]]), idxh[offh[q]:offh[q + 1]]) for q in range(4))
    assert oracle.hierarchical_hash(np.arange(9, dtype=np.uint32), [0] * 9, [[0] * 9], 1, 2, 7).rc == 2
    # sparsity metrics and the two communication-time formulas: definitions on tiny sets, the extreme
    # cases of section "Balanced Parallelism as the practical optimal scheme"
    assert oracle.overlap_ratio([1, 4, 7, 9], [4, 9, 2, 3, 5, 6], 10) == 0.5 and oracle.overlap_ratio([4], [1, 4], 10) == 1.0
    assert oracle.union_sizes([[0, 1, 2], [2, 3], [0, 3], [9]], 10).tolist() == [3, 4, 4, 5]
    sk, sp = oracle.skewness(np.array([0, 9], np.uint32), 10, 3)
    assert sp.tolist() == [1, 0, 1] and abs(sk - 2.5) < 1e-12
    assert oracle.skewness(np.arange(10, dtype=np.uint32), 400, 4)[0] == 4.0
    unit = 2 * 4e9 * 0.01 / 12.5e9
    assert abs(oracle.time_balanced_parallelism(16, 1.0, 0.01, 4e9, 12.5e9) - 2 * 15 / 16 * unit) < 1e-12
    assert abs(oracle.time_balanced_parallelism(16, 16.0, 0.01, 4e9, 12.5e9) - 15 * (1 + 1 / 16) * unit) < 1e-12
    assert abs(oracle.time_hierarchical_centralization(16, [1, 2, 4, 8], 0.01, 4e9, 12.5e9) - 15 * unit) < 1e-12
    assert abs(oracle.time_hierarchical_centralization(4, [1, 1.5, 99, 99], 0.01, 4e9, 12.5e9) - 2.5 * unit) < 1e-12
    # top-k threshold sparsifier and format sizes
    gt = np.array([0.5, -3.0, 0.0, 2.0, -0.25, 7.0, -7.5, 1.0], np.float32)
    fb = lambda v: int(np.float32(v).view(np.uint32))
    assert oracle.topk_threshold(gt, 1) == fb(7.5) and oracle.topk_threshold(gt, 3) == fb(3.0) and oracle.topk_threshold(gt, 8) == 0
    assert oracle.topk_threshold(gt, 2, first=1, stride=2) == fb(3.0)
    ot, kt = oracle.threshold_apply(gt, fb(2.0))
    assert kt == 4 and ot.tolist() == [0, -3.0, 0, 2.0, 0, 7.0, -7.5, 0] and oracle.threshold_apply(gt, 0)[1] == 7
    fs = oracle.format_bytes(1 << 20, 1 << 19, 16, 10, 256)
    assert fs == {"dense": 4.0 * (1 << 20), "coo": 8.0 * (1 << 19), "bitmap": 4.0 * (1 << 19) + 16 * (1 << 20) / 8,
                  "hash_bitmap": 4.0 * (1 << 19) + (1 << 20) / 8, "tensor_block": 10 * 1028.0}
    assert oracle.nonzero_blocks([0, 1, 255, 256, 1000], 1024, 256) == 3
    # imbalance-ratio example of section "Balance dimension"
    assert abs(oracle.imbalance([1, 4, 1]) - 2.0) < 1e-12




if __name__ == "__main__":
    import oracle

    oracle.use_library(sys.argv[1])
    battery(oracle)
    print("battery ok")
