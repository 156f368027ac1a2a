"""GPU parity of the hash-bitmap index format (Algorithm 2) against the CPU oracle: layout, encode
(bit-exact bitmap words), decode inside zen_aggregate, and the clustered-runs workload."""
import os

import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, Workload, worker_sparse, dense_from_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["small", "tiled"])
def partition_path(request, monkeypatch):
    """Run every test through both partition paths: the one-block-per-worker path that few-row
    encodes take by default, and the tiled histogram / scan / scatter path."""
    import gpu_util as G

    G.use_tuning(monkeypatch, tiled_encode=request.param == "tiled")
    return request.param


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


def _ref_bitmap(oracle, wl, rows):
    owner = oracle.owner_table(wl.n_rows, wl.n_parts, wl.hash_seed)
    dom_count, word_off = oracle.bitmap_layout(owner, wl.n_parts)
    nz = np.zeros(wl.n_rows, np.uint8)
    nz[rows] = 1
    return owner, dom_count, word_off, oracle.bitmap_encode(owner, wl.n_parts, nz, word_off)


SHAPES = [(1, 1, 1), (33, 1, 3), (5000, 1, 4), (70001, 1, 64), (300000, 1, 100), (4099, 8, 16), (9001, 64, 16),
          (333, 256, 8), (97, 1024, 8), (5000, 1, 1024), (40000, 4, 1000)]


@pytest.mark.parametrize("R,D,n", SHAPES)
def test_bitmap_layout_and_encode(oracle, zen, R, D, n):
    import gpu_util as G

    rng = np.random.default_rng(R + 13 * D + n)
    wl = Workload("t", 0, R, D, n, int(rng.integers(0, 2**32)), "uniform")
    ctx = zen.ZenContext(R, D, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    total, woff, dsz = zen.zen_bitmap_layout(ctx)
    owner = oracle.owner_table(R, n, wl.hash_seed)
    dom_count, word_off = oracle.bitmap_layout(owner, n)
    assert dsz == dom_count.tolist() and woff == word_off.tolist() and total == int(word_off[-1])
    hosts, rowsets = [], []
    for density in (0.0, 0.04, 0.6, 1.0):
        rows = np.flatnonzero(rng.random(R) < density).astype(np.uint32)
        vals = rng.standard_normal((rows.size, D)).astype(np.float32) + 4.0
        hosts.append(dense_from_sparse(wl, rows, vals))
        rowsets.append(rows)
    grads = [torch.from_numpy(h).cuda() for h in hosts]
    outs, (st, flags, _) = G.run_encode_batch(ctx, grads, [R] * len(grads))
    assert st == 0 and flags == 0
    for h, rows, enc in zip(hosts, rowsets, outs):
        ref = oracle.encode(h, R, D, n, wl.hash_seed)
        nz = np.zeros(R, np.uint8)
        nz[rows] = 1
        ref_bm = oracle.bitmap_encode(owner, n, nz, word_off)
        assert np.array_equal(G.u32(enc.offsets), ref.offsets)
        assert np.array_equal(G.u32(enc.bitmap[:total]), ref_bm)
        assert np.array_equal(G.u32(enc.indices[:ref.nnz]), ref.indices)
        assert np.array_equal(enc.values[:ref.nnz].cpu().numpy().view(np.uint32), ref.values.view(np.uint32))


@pytest.mark.parametrize("cid", [5, 3])
def test_bitmap_encode_then_aggregate(oracle, zen, cid):
    import gpu_util as G
    from dataclasses import replace

    wl = replace(MINI_WORKLOADS[cid], bitmap=True)
    n_workers = min(wl.n_workers, 16)
    sparse = [worker_sparse(wl, w) for w in range(n_workers)]
    grads = [G.dense_device(wl, r, v) for r, v in sparse]
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    # BITMAP encode without an index array at all
    encs = [zen.alloc_encoded(ctx, r.size, with_indices=False) for r, _ in sparse]
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, n_workers))
    zen.zen_encode_batch(ctx, grads, encs, ws)
    assert zen.zen_status_fetch(ctx, ws)[0] == 0
    total, woff, _ = zen.zen_bitmap_layout(ctx)
    refs = []
    for (rows, vals), enc in zip(sparse, encs):
        ref = oracle.encode(dense_from_sparse(wl, rows, vals), wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
        _, _, word_off, ref_bm = _ref_bitmap(oracle, wl, rows)
        assert np.array_equal(G.u32(enc.offsets), ref.offsets)
        assert np.array_equal(G.u32(enc.bitmap[:total]), ref_bm)
        assert np.array_equal(enc.values[:ref.nnz].cpu().numpy().view(np.uint32), ref.values.view(np.uint32))
        refs.append(ref)
    per_server = [sum(int(e.offsets[j + 1]) - int(e.offsets[j]) for e in refs) for j in range(wl.n_parts)]
    max_in = max(per_server)
    outs, (st, flags, _) = G.run_aggregate_batch(ctx, encs, [max(p, 1) for p in per_server], max_in)
    assert st == 0 and flags == 0
    for j in range(wl.n_parts):
        parts = [(e.indices[e.offsets[j]:e.offsets[j + 1]], e.values[e.offsets[j]:e.offsets[j + 1]]) for e in refs]
        ref = oracle.aggregate(parts, wl.n_rows, wl.row_dim)
        U, idx, val = G.aggregated_to_host(outs[j])
        assert U == ref.U and np.array_equal(idx, ref.indices)
        G.check_sums(val, ref)


@pytest.mark.parametrize("mixed", [True, False])
@pytest.mark.parametrize("D", [1, 4, 100])
def test_single_server_bitmap_parts(oracle, zen, mixed, D):
    import gpu_util as G

    # mixed: one COO part among the bitmaps -> decode + table path; else the bitmap-domain merge
    R, n, seed = 20000, 8, 99
    ctx = zen.ZenContext(R, D, n, seed, zen.ZEN_INDEX_BITMAP)
    owner = oracle.owner_table(R, n, seed)
    dom_count, word_off = oracle.bitmap_layout(owner, n)
    rng = np.random.default_rng(8)
    part_id = 5
    dom = np.flatnonzero(owner == part_id).astype(np.uint32)
    parts_h, parts_d = [], []
    for w in range(5):
        rows = np.sort(rng.choice(dom, size=int(rng.integers(0, dom.size // 2)), replace=False)).astype(np.uint32)
        vals = rng.standard_normal((rows.size, D)).astype(np.float32)
        nz = np.zeros(R, np.uint8)
        nz[rows] = 1
        bm = oracle.bitmap_encode(owner, n, nz, word_off)[int(word_off[part_id]):int(word_off[part_id + 1])]
        parts_h.append((rows, vals))
        if w == 2 and mixed:      # one part in COO form, mixed with bitmap parts
            parts_d.append((G.to_dev(rows), None, torch.from_numpy(vals).cuda(),
                            torch.tensor([rows.size], dtype=torch.int32, device="cuda")))
        else:
            parts_d.append((None, G.to_dev(bm) if bm.size else torch.zeros(1, dtype=torch.int32, device="cuda"),
                            torch.from_numpy(vals).cuda() if rows.size else torch.empty((1, D), device="cuda"),
                            torch.tensor([rows.size], dtype=torch.int32, device="cuda")))
    total = sum(r.size for r, _ in parts_h)
    ref = oracle.aggregate(parts_h, R, D)
    out = zen.alloc_aggregated(ctx, total)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, total))
    zen.zen_aggregate(ctx, parts_d, part_id, out, total, ws)
    st, flags, _ = zen.zen_status_fetch(ctx, ws)
    assert st == 0 and flags == 0
    U, idx, val = G.aggregated_to_host(out)
    assert U == ref.U and np.array_equal(idx, ref.indices)
    G.check_sums(val, ref)


@pytest.mark.parametrize("D", [1, 4])
def test_bitmap_part_with_more_bits_than_rows_is_flagged_and_not_merged(oracle, zen, D):
    """A part whose bitmap has more set bits than its row count names: flag bit 2, the server puts out nothing,
    and the merge reads none of the part's values (its value array here is two rows, in the middle of a guard)."""
    import gpu_util as G

    R, n, seed, part_id = 20000, 8, 99, 2
    ctx = zen.ZenContext(R, D, n, seed, zen.ZEN_INDEX_BITMAP)
    owner = oracle.owner_table(R, n, seed)
    dom_count, word_off = oracle.bitmap_layout(owner, n)
    dom = np.flatnonzero(owner == part_id).astype(np.uint32)
    nz = np.zeros(R, np.uint8)
    nz[dom[: dom.size // 2]] = 1                                     # over a thousand set bits ...
    bm = oracle.bitmap_encode(owner, n, nz, word_off)[int(word_off[part_id]):int(word_off[part_id + 1])]
    vals = torch.full((2, D), 3.0, device="cuda")                   # ... and two rows of values
    good_rows = dom[::7]
    nz2 = np.zeros(R, np.uint8)
    nz2[good_rows] = 1
    bm2 = oracle.bitmap_encode(owner, n, nz2, word_off)[int(word_off[part_id]):int(word_off[part_id + 1])]
    cnt = lambda k: torch.tensor([k], dtype=torch.int32, device="cuda")
    parts = [(None, G.to_dev(bm2), torch.ones((good_rows.size, D), device="cuda"), cnt(good_rows.size)),
             (None, G.to_dev(bm), vals, cnt(2))]
    out = zen.alloc_aggregated(ctx, dom.size)
    out.indices.fill_(-7)
    out.values.fill_(-7.0)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, dom.size))
    zen.zen_aggregate(ctx, parts, part_id, out, dom.size, ws)
    st, flags, _ = zen.zen_status_fetch(ctx, ws)
    assert st == zen.ZEN_ERR_INVALID and flags == 4
    assert int(out.count.item()) == 0
    assert torch.all(out.indices == -7) and torch.all(out.values == -7.0)
    # the same parts with the right count for the first and without the bad one: merged as usual
    zen.zen_aggregate(ctx, parts[:1], part_id, out, dom.size, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    U, idx, val = G.aggregated_to_host(out)
    assert U == good_rows.size and np.array_equal(idx, good_rows) and np.all(val == 1.0)


@pytest.mark.parametrize("R,n", [(1, 1), (33, 3), (5000, 4), (70001, 64), (300000, 100), (5000, 1024), (1 << 20, 7)])
def test_elementwise_bitmap_encode_without_index_list(oracle, zen, R, n):
    """Element-level inputs, hash-bitmap output and no index list: the call the clustered-runs benchmark
    makes (uniform densities and long unaligned runs of consecutive non-zeros)."""
    import gpu_util as G

    rng = np.random.default_rng(R + n)
    wl = Workload("t", 0, R, 1, n, int(rng.integers(0, 2**32)), "uniform")
    ctx = zen.ZenContext(R, 1, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    total, woff, _ = zen.zen_bitmap_layout(ctx)
    owner = oracle.owner_table(R, n, wl.hash_seed)
    _, word_off = oracle.bitmap_layout(owner, n)
    hosts, rowsets = [], []
    for density in (0.0, 0.02, 0.5, 1.0, "runs"):
        if density == "runs":      # long runs of consecutive non-zeros at unaligned offsets
            m = np.zeros(R, bool)
            for start in rng.integers(0, max(R - 1, 1), size=5):
                m[int(start):int(start) + 4096 + 37] = True
            rows = np.flatnonzero(m).astype(np.uint32)
        else:
            rows = np.flatnonzero(rng.random(R) < density).astype(np.uint32)
        vals = rng.standard_normal((rows.size, 1)).astype(np.float32) + 4.0
        hosts.append(dense_from_sparse(wl, rows, vals))
        rowsets.append(rows)
    grads = [torch.from_numpy(h).cuda() for h in hosts]
    encs = [zen.alloc_encoded(ctx, r.size, with_indices=False) for r in rowsets]
    for e in encs:
        e.values.fill_(-1.0)
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, len(grads)))
    zen.zen_encode_batch(ctx, grads, encs, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    for h, rows, enc in zip(hosts, rowsets, encs):
        ref = oracle.encode(h, R, 1, n, wl.hash_seed)
        assert np.array_equal(G.u32(enc.offsets), ref.offsets)
        assert np.array_equal(G.u32(enc.bitmap[:total]), oracle.bitmap_encode(owner, n, oracle.member_mask(rows, R), word_off))
        assert np.array_equal(enc.values[:ref.nnz].cpu().numpy().view(np.uint32), ref.values.view(np.uint32))
    # capacity smaller than nnz: offsets complete, flag raised, nothing written past the capacity
    big = max(range(len(rowsets)), key=lambda i: rowsets[i].size)
    nnz = rowsets[big].size
    if nnz >= 4:
        cap = nnz // 2
        small = zen.alloc_encoded(ctx, nnz, with_indices=False)
        small.values.fill_(-1.0)
        small.cap_rows = cap
        zen.zen_encode_batch(ctx, [grads[big]], [small], ws)
        st, flags, needed = zen.zen_status_fetch(ctx, ws)
        assert st == zen.ZEN_ERR_CAPACITY and flags & 1 and needed == nnz
        ref = oracle.encode(hosts[big], R, 1, n, wl.hash_seed)
        assert np.array_equal(G.u32(small.offsets), ref.offsets)
        got = small.values.cpu().numpy()
        assert np.array_equal(got[:cap].view(np.uint32), ref.values[:cap].view(np.uint32))
        assert (got[cap:] == -1.0).all()


@pytest.mark.parametrize("n,with_indices", [(64, False), (5, True), (128, True), (129, False)])
def test_elementwise_stretch_boundaries(oracle, zen, n, with_indices):
    """Stretches of consecutive non-zero rows placed at and around every boundary the element-level scatter
    knows (mask word 32, group 512, the 2,048-row limit of a stretch, tile 32,768, end of the tensor), of
    lengths around the shortest stretch it places from the rank tables (128), next to scattered rows."""
    import gpu_util as G

    R = 3 * 32768 + 1000 + 13                      # three tiles and a ragged tail
    rng = np.random.default_rng(n)
    wl = Workload("t", 0, R, 1, n, int(rng.integers(0, 2**32)), "uniform")
    ctx = zen.ZenContext(R, 1, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    total, _, _ = zen.zen_bitmap_layout(ctx)
    owner = oracle.owner_table(R, n, wl.hash_seed)
    _, word_off = oracle.bitmap_layout(owner, n)
    masks = []
    m = np.zeros(R, bool)                          # runs that start / end on, just before and just after boundaries
    for start, length in [(0, 127), (512 - 1, 128), (1024, 129), (2048 + 31, 2048), (8192 - 5, 2049 + 5),
                          (16384, 4096), (32768 - 100, 300), (2 * 32768 - 2048, 2048), (2 * 32768 + 1, 511),
                          (3 * 32768 - 1, 2), (R - 700, 700)]:
        m[start:start + length] = True
    masks.append(m)
    m = np.zeros(R, bool)                          # scattered rows running into a stretch, a stretch into scattered rows
    m[rng.integers(0, R, size=3000)] = True
    m[5000:5000 + 1500] = True
    m[40000:40000 + 129] = True
    m[70000:70000 + 5000] = True
    m[70000 + 2500] = False                        # one hole inside a long run
    masks.append(m)
    masks.append(np.ones(R, bool))                 # everything
    m = np.ones(R, bool)
    m[::97] = False                                # nearly everything: no stretch reaches 128 rows
    masks.append(m)
    hosts, rowsets = [], []
    for m in masks:
        rows = np.flatnonzero(m).astype(np.uint32)
        vals = rng.standard_normal((rows.size, 1)).astype(np.float32) + 4.0
        hosts.append(dense_from_sparse(wl, rows, vals))
        rowsets.append(rows)
    grads = [torch.from_numpy(h).cuda() for h in hosts]
    encs = [zen.alloc_encoded(ctx, r.size, with_indices=with_indices) for r in rowsets]
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, len(grads)))
    ws.view(torch.int32).fill_(-1)
    zen.zen_encode_batch(ctx, grads, encs, ws)
    assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
    for h, rows, enc in zip(hosts, rowsets, encs):
        ref = oracle.encode(h, R, 1, n, wl.hash_seed)
        assert np.array_equal(G.u32(enc.offsets), ref.offsets)
        assert np.array_equal(G.u32(enc.bitmap[:total]), oracle.bitmap_encode(owner, n, oracle.member_mask(rows, R), word_off))
        assert np.array_equal(enc.values[:ref.nnz].cpu().numpy().view(np.uint32), ref.values.view(np.uint32))
        if with_indices:
            assert np.array_equal(G.u32(enc.indices[:ref.nnz]), ref.indices)
    # capacity short by a few rows in the middle of the output: flag + needed rows, nothing beyond the capacity
    short = [zen.alloc_encoded(ctx, r.size - 7, with_indices=with_indices) for r in rowsets]
    for e in short:
        e.values.fill_(-1.0)
    zen.zen_encode_batch(ctx, grads, short, ws)
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    assert st == 2 and (flags & 1) and needed == max(r.size for r in rowsets)
