"""GPU parity of the Pull side (Algorithm 2 at the server and at the worker) against the CPU oracle:
bitmap of an aggregated partition (bit-exact), decode (bit-exact), dense placement (bit-exact), the
error flags, and encode -> aggregate -> pull on the device = dense sum of the workers' gradients."""
import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, dense_from_sparse, worker_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


def _agg_from_host(zen, ctx, idx, vals, cap=None):
    import gpu_util as G

    cap = idx.size if cap is None else cap
    a = zen.alloc_aggregated(ctx, cap)
    if idx.size:
        a.indices[:idx.size] = G.to_dev(idx)
        a.values[:idx.size] = torch.from_numpy(np.ascontiguousarray(vals)).cuda()
    a.count.fill_(int(idx.size))
    return a


def _status(zen, ctx, ws):
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    return st, flags, needed


SHAPES = [(1, 1, 1), (33, 1, 3), (5000, 1, 4), (70001, 1, 1), (300000, 1, 4), (300000, 1, 100), (4099, 8, 16),
          (9001, 64, 16), (333, 256, 8), (97, 1024, 8), (5000, 3, 1024), (40000, 4, 1000), (100000, 2, 5)]


@pytest.mark.parametrize("R,D,n", SHAPES)
def test_pull_encode_decode_apply(oracle, zen, R, D, n):
    import gpu_util as G

    rng = np.random.default_rng(7 * R + 13 * D + n)
    seed = int(rng.integers(0, 2**32))
    ctx = zen.ZenContext(R, D, n, seed, zen.ZEN_INDEX_BITMAP)
    coo_ctx = zen.ZenContext(R, D, n, seed, zen.ZEN_INDEX_COO)
    total, woff, dsz = zen.zen_bitmap_layout(ctx)
    owner = oracle.owner_table(R, n, seed)
    _, word_off = oracle.bitmap_layout(owner, n)
    ws = zen.alloc_workspace(zen.zen_pull_workspace_bytes(ctx))
    ws_coo = zen.alloc_workspace(zen.zen_pull_workspace_bytes(coo_ctx))
    for density in (0.0, 0.04, 0.6, 1.0):
        present = np.flatnonzero(rng.random(R) < density).astype(np.uint32)
        vals = rng.standard_normal((present.size, D)).astype(np.float32)
        if present.size:
            vals[0] = 0.0                                   # a cancelled sum keeps its bit
        own = owner[present]
        parts = [(present[own == p], vals[own == p]) for p in range(n)]
        aggs = [_agg_from_host(zen, ctx, i, v) for i, v in parts]
        # server side
        bitmap = torch.full((max(total, 1),), -1, dtype=torch.int32, device="cuda")
        zen.zen_pull_encode_batch(ctx, aggs, bitmap, ws)
        assert _status(zen, ctx, ws) == (0, 0, 0)
        ref_bm = oracle.bitmap_encode(owner, n, oracle.member_mask(present, R), word_off)
        assert np.array_equal(G.u32(bitmap[:total]), ref_bm)
        # worker side: decode a few partitions
        for p in sorted(set([0, n // 2, n - 1])):
            out_idx = torch.empty(max(parts[p][0].size, 1), dtype=torch.int32, device="cuda")
            out_cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
            zen.zen_pull_decode(ctx, bitmap[woff[p]:] if woff[p] < bitmap.numel() else bitmap, p, out_idx, out_cnt, ws)
            assert _status(zen, ctx, ws) == (0, 0, 0)
            assert int(out_cnt.item()) == parts[p][0].size
            assert np.array_equal(G.u32(out_idx[:parts[p][0].size]), parts[p][0])
        # worker side: dense placement from bitmaps, from index lists, and from a mix
        expect = oracle.pull_apply(owner, n, D, word_off, ref_bm, [v for _, v in parts])
        dense = torch.full((R, D), 7.0, dtype=torch.float32, device="cuda")
        bm_parts = [(None, bitmap[woff[p]:] if woff[p] < bitmap.numel() else bitmap, aggs[p].values, aggs[p].count)
                    for p in range(n)]
        zen.zen_pull_apply(ctx, bm_parts, dense, ws)
        assert _status(zen, ctx, ws) == (0, 0, 0)
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
        coo_parts = [(aggs[p].indices, None, aggs[p].values, aggs[p].count) for p in range(n)]
        dense.fill_(7.0)
        zen.zen_pull_apply(coo_ctx, coo_parts, dense, ws_coo)
        assert _status(zen, coo_ctx, ws_coo) == (0, 0, 0)
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
        mixed = [bm_parts[p] if p % 2 else coo_parts[p] for p in range(n)]
        dense.fill_(7.0)
        zen.zen_pull_apply(ctx, mixed, dense, ws)
        assert _status(zen, ctx, ws) == (0, 0, 0)
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), expect.view(np.uint32))
        assert np.array_equal(expect, oracle.densify(parts, R, D))


def test_pull_encode_single_partition(oracle, zen):
    import gpu_util as G

    R, D, n, seed = 50000, 1, 6, 99
    ctx = zen.ZenContext(R, D, n, seed, zen.ZEN_INDEX_BITMAP)
    total, woff, dsz = zen.zen_bitmap_layout(ctx)
    owner = oracle.owner_table(R, n, seed)
    _, word_off = oracle.bitmap_layout(owner, n)
    rng = np.random.default_rng(1)
    present = np.flatnonzero(rng.random(R) < 0.3).astype(np.uint32)
    ref_bm = oracle.bitmap_encode(owner, n, oracle.member_mask(present, R), word_off)
    ws = zen.alloc_workspace(zen.zen_pull_workspace_bytes(ctx))
    for p in range(n):
        idx = present[owner[present] == p]
        words = torch.full((woff[p + 1] - woff[p] + 1,), -1, dtype=torch.int32, device="cuda")
        cnt = torch.tensor([idx.size], dtype=torch.int32, device="cuda")
        zen.zen_pull_encode(ctx, G.to_dev(idx), cnt, idx.size, p, words, ws)
        assert _status(zen, ctx, ws) == (0, 0, 0)
        assert np.array_equal(G.u32(words[:-1]), ref_bm[woff[p]:woff[p + 1]])
        assert int(words[-1].item()) == -1                              # nothing past the partition's words
        # count clamped to the capacity: only the first half of the list is encoded
        half = idx.size // 2
        zen.zen_pull_encode(ctx, G.to_dev(idx), cnt, half, p, words, ws)
        assert _status(zen, ctx, ws) == (0, 0, 0)
        ref_half = oracle.bitmap_encode(owner, n, oracle.member_mask(idx[:half], R), word_off)
        assert np.array_equal(G.u32(words[:-1]), ref_half[woff[p]:woff[p + 1]])


def test_pull_flags_inconsistent_input(oracle, zen):
    """Every malformed input is turned into a status flag by the kernels' own bounds checks."""
    import gpu_util as G

    R, D, n, seed = 40000, 2, 3, 5
    ctx = zen.ZenContext(R, D, n, seed, zen.ZEN_INDEX_BITMAP)
    total, woff, dsz = zen.zen_bitmap_layout(ctx)
    owner = oracle.owner_table(R, n, seed)
    ws = zen.alloc_workspace(zen.zen_pull_workspace_bytes(ctx))
    dom0 = np.flatnonzero(owner == 0).astype(np.uint32)
    dom1 = np.flatnonzero(owner == 1).astype(np.uint32)
    words = torch.zeros(woff[1] - woff[0], dtype=torch.int32, device="cuda")

    def encode0(idx):
        idx = np.asarray(idx, np.uint32)
        cnt = torch.tensor([idx.size], dtype=torch.int32, device="cuda")
        zen.zen_pull_encode(ctx, G.to_dev(idx) if idx.size else torch.zeros(1, dtype=torch.int32, device="cuda"), cnt,
                            idx.size, 0, words, ws)
        return _status(zen, ctx, ws)

    good = dom0[::3]
    assert encode0(good) == (0, 0, 0)
    assert encode0(np.sort(np.concatenate([good, dom1[5:6]])))[1] & 4         # a row of another partition
    assert encode0(np.sort(np.concatenate([good, good[10:11]])))[1] & 4       # a duplicate
    assert encode0(good[::-1].copy())[1] & 4                                  # descending
    below = np.flatnonzero(owner != 0)
    below = below[below < dom0[0]]
    if below.size:                                                            # a foreign row before the domain's first
        assert encode0(np.concatenate([below[:1], good]).astype(np.uint32))[1] & 4
    assert encode0(np.concatenate([good, dom1[-1:]]).astype(np.uint32) if dom1[-1] > dom0[-1] else good[::-1].copy())[1] & 4
    st, flags, _ = encode0(np.concatenate([good, [R + 5]]).astype(np.uint32))  # past the last row
    assert st == zen.ZEN_ERR_INVALID and flags & 4
    assert encode0(good) == (0, 0, 0)                                          # the flag does not stick

    # decode: capacity overflow reports the number of set bits
    idx = dom0[::2]
    cnt = torch.tensor([idx.size], dtype=torch.int32, device="cuda")
    zen.zen_pull_encode(ctx, G.to_dev(idx), cnt, idx.size, 0, words, ws)
    out_idx = torch.full((100,), -1, dtype=torch.int32, device="cuda")
    out_cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    zen.zen_pull_decode(ctx, words, 0, out_idx[:99], out_cnt, ws)
    st, flags, needed = _status(zen, ctx, ws)
    assert st == zen.ZEN_ERR_CAPACITY and flags & 1 and needed == idx.size and int(out_cnt.item()) == idx.size
    assert np.array_equal(G.u32(out_idx[:99]), idx[:99]) and int(out_idx[99].item()) == -1

    # apply: a bitmap whose set bits do not number *count; rows beyond *count are never read
    vals = torch.ones((idx.size, D), dtype=torch.float32, device="cuda")
    empty_bm = torch.zeros(max(total, 1), dtype=torch.int32, device="cuda")
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    dense = torch.empty((R, D), dtype=torch.float32, device="cuda")
    short = torch.tensor([idx.size - 7], dtype=torch.int32, device="cuda")
    parts = [(None, words, vals, short), (None, empty_bm[woff[1]:], vals, zero), (None, empty_bm[woff[2]:], vals, zero)]
    zen.zen_pull_apply(ctx, parts, dense, ws)
    st, flags, _ = _status(zen, ctx, ws)
    assert st == zen.ZEN_ERR_INVALID and flags & 4
    host = dense.cpu().numpy()
    assert host[idx[:idx.size - 7]].min() == 1.0 and host.sum() == (idx.size - 7) * D
    # apply: an index list with a row id past the tensor
    bad_idx = G.to_dev(np.array([3, R, 9], np.uint32))
    three = torch.tensor([3], dtype=torch.int32, device="cuda")
    parts = [(bad_idx, None, vals, three), (None, empty_bm[woff[1]:], vals, zero), (None, empty_bm[woff[2]:], vals, zero)]
    zen.zen_pull_apply(ctx, parts, dense, ws)
    st, flags, _ = _status(zen, ctx, ws)
    assert st == zen.ZEN_ERR_INVALID and flags & 4
    assert dense.cpu().numpy().sum() == 2 * D


def test_pull_argument_errors(zen):
    ctx = zen.ZenContext(1000, 4, 4, 1, zen.ZEN_INDEX_COO)
    ws = zen.alloc_workspace(zen.zen_pull_workspace_bytes(ctx))
    a = [zen.alloc_aggregated(ctx, 10) for _ in range(4)]
    bm = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(zen.ZenError):                       # bitmap forms need a BITMAP context
        zen.zen_pull_encode_batch(ctx, a, bm, ws)
    dense = torch.zeros((1000, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(zen.ZenError):
        zen.zen_pull_apply(ctx, [(None, bm, x.values, x.count) for x in a], dense, ws)
    with pytest.raises(zen.ZenError):                       # misaligned dense tensor
        zen.zen_pull_apply(ctx, [(x.indices, None, x.values, x.count) for x in a], dense.view(-1)[1:], ws)
    bctx = zen.ZenContext(1000, 4, 4, 1, zen.ZEN_INDEX_BITMAP)
    with pytest.raises(zen.ZenError):                       # workspace too small
        zen.zen_pull_encode_batch(bctx, a, bm, ws[:256])


@pytest.mark.parametrize("cid", [1, 2, 3, 5])
def test_encode_aggregate_pull_equals_dense_sum(oracle, zen, cid):
    """The whole loop on the device: every worker encodes, every server aggregates and builds its hash
    bitmap, the worker decodes and places -- the result is the dense sum of the workers' gradients."""
    import gpu_util as G
    from dataclasses import replace

    wl = MINI_WORKLOADS[cid]
    R, D, n = wl.n_rows, wl.row_dim, wl.n_parts
    total64 = np.zeros((R, D), np.float64)
    abs64 = np.zeros((R, D), np.float64)
    ncontrib = np.zeros(R, np.int64)
    sparse = []
    for w in range(wl.n_workers):
        rows, vals = worker_sparse(wl, w)
        g = dense_from_sparse(wl, rows, vals).reshape(R, D).astype(np.float64)
        total64 += g
        abs64 += np.abs(g)
        ncontrib[rows] += 1
        sparse.append((rows, vals))
    grads = [G.dense_device(wl, r, v) for r, v in sparse]
    ctx = zen.ZenContext(R, D, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    encs, st = G.run_encode_batch(ctx, grads, [r.size for r, _ in sparse])
    assert st == (0, 0, 0)
    union = np.flatnonzero(ncontrib).astype(np.uint32)
    owner = oracle.owner_table(R, n, wl.hash_seed)
    per_server = np.bincount(owner[union], minlength=n)
    max_in = int(sum(r.size for r, _ in sparse))
    aggs, st = G.run_aggregate_batch(ctx, encs, [int(c) for c in per_server], max_in)
    assert st == (0, 0, 0)
    tot_words, woff, _ = zen.zen_bitmap_layout(ctx)
    ws = zen.alloc_workspace(zen.zen_pull_workspace_bytes(ctx))
    bitmap = torch.empty(max(tot_words, 1), dtype=torch.int32, device="cuda")
    zen.zen_pull_encode_batch(ctx, aggs, bitmap, ws)
    assert _status(zen, ctx, ws) == (0, 0, 0)
    _, word_off = oracle.bitmap_layout(owner, n)
    assert np.array_equal(G.u32(bitmap[:tot_words]), oracle.bitmap_encode(owner, n, oracle.member_mask(union, R), word_off))
    dense = torch.empty((R, D), dtype=torch.float32, device="cuda")
    parts = [(None, bitmap[woff[p]:] if woff[p] < bitmap.numel() else bitmap, aggs[p].values, aggs[p].count)
             for p in range(n)]
    zen.zen_pull_apply(ctx, parts, dense, ws)
    assert _status(zen, ctx, ws) == (0, 0, 0)
    got = dense.cpu().numpy()
    err = np.abs(got.astype(np.float64) - total64)
    assert (err <= 1e-6 * abs64).all()                                   # zero rows are exactly zero
    one = ncontrib == 1
    assert np.array_equal(got[one].view(np.uint32), total64[one].astype(np.float32).view(np.uint32))
