"""Pins for the oracle's top-k threshold sparsifier and the sparse-format size accounting."""
import numpy as np
import pytest


def test_topk_threshold_exact_and_sampled(oracle):
    g = np.array([0.5, -3.0, 0.0, 2.0, -0.25, 7.0, -7.5, 1.0], np.float32)
    bits = lambda x: int(np.float32(abs(x)).view(np.uint32))
    assert oracle.topk_threshold(g, 1) == bits(7.5)                 # the largest magnitude, sign ignored
    assert oracle.topk_threshold(g, 3) == bits(3.0)
    assert oracle.topk_threshold(g, 8) == 0                         # keep everything: the zero is the 8th
    assert oracle.topk_threshold(g, 2, first=1, stride=2) == bits(3.0)   # sample = -3, 2, 7, 1 -> 7, 3
    with pytest.raises(ValueError):
        oracle.topk_threshold(g, 0)
    with pytest.raises(ValueError):
        oracle.topk_threshold(g, 5, first=0, stride=2)              # the sample has 4 elements
    out, kept = oracle.threshold_apply(g, bits(2.0))
    assert kept == 4 and out.tolist() == [0, -3.0, 0, 2.0, 0, 7.0, -7.5, 0]
    out, kept = oracle.threshold_apply(g, 0)                        # threshold 0 still drops the zeros
    assert kept == 7 and np.array_equal(out, g)
    # against numpy on random data: exactly k survive when magnitudes are distinct
    rng = np.random.default_rng(0)
    x = rng.standard_normal(10007).astype(np.float32)
    for k in (1, 500, 10007):
        thr = oracle.topk_threshold(x, k)
        assert thr == int(np.sort(np.abs(x))[::-1][k - 1].view(np.uint32))
        out, kept = oracle.threshold_apply(x, thr)
        assert kept == k and np.array_equal(out != 0, np.abs(x).view(np.uint32) >= thr)
    # special values: -0.0 is zero, NaN ranks above Inf
    y = np.array([np.nan, np.inf, -np.inf, 1.0, -0.0], np.float32)
    assert oracle.topk_threshold(y, 1) == int(y[:1].view(np.uint32)[0] & 0x7FFFFFFF)
    assert oracle.topk_threshold(y, 3) == 0x7F800000 and oracle.topk_threshold(y, 5) == 0
    # the sampled threshold keeps about the requested share of the whole tensor (top 5 %, section
    # "Characteristics of Sparse Tensors")
    z = rng.standard_normal(400000).astype(np.float32)
    sample = z[3::100]
    thr = oracle.topk_threshold(z, int(0.05 * sample.size), first=3, stride=100)
    _, kept = oracle.threshold_apply(z, thr)
    assert abs(kept / z.size - 0.05) < 0.01


def test_format_sizes_and_break_even_points(oracle):
    # section "Understanding Zen", paragraph "Hash Bitmap" (16 servers): COO and the plain bitmap stop
    # saving traffic at a density of 50 %, the hash bitmap still saves at 95 %
    G, n = 1 << 20, 16
    for dens, coo_saves, bitmap_saves, hash_saves in [(0.05, True, True, True), (0.49, True, True, True),
                                                      (0.51, False, False, True), (0.95, False, False, True),
                                                      (0.97, False, False, False)]:
        s = oracle.format_bytes(G, int(dens * G), n, G // 256)
        assert (s["coo"] < s["dense"]) == coo_saves
        assert (s["bitmap"] < s["dense"]) == bitmap_saves
        assert (s["hash_bitmap"] < s["dense"]) == hash_saves
        assert s["hash_bitmap"] < s["bitmap"] and s["hash_bitmap"] == 4 * int(dens * G) + G / 8
    # the 856 MB tensor of section "Sparse Formats": 27 MB of hash bitmap, 428 MB of plain bitmaps
    s = oracle.format_bytes(856_000_000 // 4, 0, 16, 0)
    assert round(s["hash_bitmap"] / 1e6) == 27 and round(s["bitmap"] / 1e6) == 428
    # tensor blocks: a block is sent whole, with its id
    assert oracle.format_bytes(1024, 3, 4, 2, 256)["tensor_block"] == 2 * (256 * 4 + 4)
    assert oracle.nonzero_blocks([0, 1, 255, 256, 1000], 1024, 256) == 3
    assert oracle.nonzero_blocks([], 1024, 256) == 0
    rng = np.random.default_rng(1)
    I = np.flatnonzero(rng.random(100000) < 0.01).astype(np.uint32)
    assert oracle.nonzero_blocks(I, 100000, 256) == np.unique(I // 256).size
    # at high density nearly every block is non-zero and blocks cost more than COO at low density ...
    dense_I = np.flatnonzero(rng.random(100000) < 0.5).astype(np.uint32)
    assert oracle.nonzero_blocks(dense_I, 100000, 256) == (100000 + 255) // 256
    sparse = oracle.format_bytes(100000, I.size, 16, oracle.nonzero_blocks(I, 100000, 256))
    assert sparse["tensor_block"] > sparse["coo"]                   # more zeros than non-zeros per block
