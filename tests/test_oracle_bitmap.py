"""Pins for the oracle's hash bitmap (Algorithm 2) and its layout."""
import os

import numpy as np
import pytest

import brute
from workloads import MINI_WORKLOADS, worker_sparse

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hash_bitmap_example.txt")


def _gold():
    d = {}
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            d[k] = [int(x) for x in v]
    return d


@pytest.mark.parametrize("first_member_1based", [1, 2, 3, 4])
def test_paper_worked_example(oracle, first_member_1based):
    g = _gold()
    R, n = g["n_gradients"][0], g["n_servers"][0]
    nz_1b = g["nonzero_indices_1based"]
    # injected owner table: server 0 owns (a, 5, 7, 11, 14) in 1-based ids, the rest alternate
    dom0 = [first_member_1based, 5, 7, 11, 14]
    owner = np.array([0 if (r + 1) in dom0 else 1 + (r % 2) for r in range(R)], np.uint16)
    nz = np.zeros(R, np.uint8)
    nz[[i - 1 for i in nz_1b]] = 1
    dom_count, word_off = oracle.bitmap_layout(owner, n)
    assert int(dom_count[0]) == 5 and int(dom_count.sum()) == R
    bm = oracle.bitmap_encode(owner, n, nz, word_off)
    w0 = int(bm[int(word_off[0])])
    assert [j + 1 for j in range(32) if (w0 >> j) & 1] == g["set_bits_1based"]     # second and third bit
    # other servers hold no non-zero gradient
    assert all(int(bm[int(word_off[p])]) == 0 for p in (1, 2))
    dec = oracle.bitmap_decode(owner, 0, bm[int(word_off[0]):int(word_off[1])])
    assert [int(i) + 1 for i in dec] == nz_1b


@pytest.mark.parametrize("R,n", [(1, 1), (31, 2), (32, 1), (33, 3), (1000, 7), (4099, 64)])
def test_bitmap_matches_brute_force_and_roundtrips(oracle, R, n):
    rng = np.random.default_rng(R + n)
    seed = int(rng.integers(0, 2**32))
    owner = oracle.owner_table(R, n, seed)
    for density in (0.0, 0.05, 0.6, 1.0):
        nz = (rng.random(R) < density).astype(np.uint8)
        I = np.flatnonzero(nz).astype(np.uint32)
        dom_count, word_off = oracle.bitmap_layout(owner, n)
        assert int(dom_count.sum()) == R                                  # total bits = |G| (appendix)
        assert np.array_equal(dom_count, np.bincount(owner, minlength=n).astype(np.uint64))
        assert np.array_equal(np.diff(word_off), (dom_count + np.uint64(31)) // np.uint64(32))
        assert R // 32 <= int(word_off[-1]) <= (R + 31) // 32 + n          # |G|/32 words + padding
        bm = oracle.bitmap_encode(owner, n, nz, word_off)
        ref = brute.bitmap(owner, n, I)
        off, idx = oracle.partition(I, owner[I], n)
        for p in range(n):
            words = bm[int(word_off[p]):int(word_off[p + 1])]
            as_int = sum(int(w) << (32 * k) for k, w in enumerate(words))
            assert as_int == ref[p][0]                                     # LSB-first, padding zero
            assert bin(as_int).count("1") == int(off[p + 1]) - int(off[p])  # popcount = partition size
            dec = oracle.bitmap_decode(owner, p, words)
            assert np.array_equal(dec, idx[int(off[p]):int(off[p + 1])])   # k-th set bit <-> k-th index


def test_bitmap_size_closed_forms():
    # section "Existing Sparse Formats": an 856 MB fp32 tensor needs a 27 MB bitmap (|G|/32 words);
    # a plain bitmap per hashed server costs |G|/32 each, 428 MB for 16 servers; the hash bitmap's
    # total stays |G|/32 (appendix "Proof of The Property of Hash Bitmap").
    tensor_mb = 856.0
    assert round(tensor_mb / 32) == 27
    assert round(16 * tensor_mb / 32) == 428


def test_layout_word_boundaries(oracle):
    # |II_p| an exact multiple of 32 needs no padding word; an empty domain takes no word at all
    dom_count, word_off = oracle.bitmap_layout(np.array([0] * 64 + [2] * 32 + [3] * 33, np.uint16), 4)
    assert dom_count.tolist() == [64, 0, 32, 33] and word_off.tolist() == [0, 2, 2, 3, 5]


def test_hash_bitmap_total_is_constant_in_n(oracle):
    R = 1 << 16
    for n in (1, 2, 16, 64, 128):
        owner = oracle.owner_table(R, n, 5)
        dom_count, word_off = oracle.bitmap_layout(owner, n)
        assert int(dom_count.sum()) == R
        assert R // 32 <= int(word_off[-1]) <= R // 32 + n


def test_bitmap_on_mini_config5(oracle):
    wl = MINI_WORKLOADS[5]
    owner = oracle.owner_table(wl.n_rows, wl.n_parts, wl.hash_seed)
    rows, _ = worker_sparse(wl, 1, want_values=False)
    nz = np.zeros(wl.n_rows, np.uint8)
    nz[rows] = 1
    dom_count, word_off = oracle.bitmap_layout(owner, wl.n_parts)
    bm = oracle.bitmap_encode(owner, wl.n_parts, nz, word_off)
    got = np.concatenate([oracle.bitmap_decode(owner, p, bm[int(word_off[p]):int(word_off[p + 1])])
                          for p in range(wl.n_parts)])
    off, idx = oracle.partition(rows, owner[rows], wl.n_parts)
    assert np.array_equal(got, idx)
