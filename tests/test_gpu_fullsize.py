"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(zen_encode_batch over all workers, zen_aggregate_batch over all servers).

The oracle cannot re-derive everything at these sizes in seconds, so: offsets / indices are
checked against the oracle's partition of the planted non-zero rows (every worker, or a sample of
workers for the largest workload), values against the planted rows, bitmaps by decoding sampled
partitions with the oracle and by per-partition popcounts, and the aggregate on all (or sampled)
servers against the oracle's aggregate of the oracle-partitioned inputs.

What is checked on EVERY worker and server of every configuration: the offsets against the oracle's
partition sizes, the per-partition bitmap popcounts, and every server's count U_j against the oracle's
union of the workers' rows per partition.  Indices, values and sums are compared in full on
configurations 1-3, on every worker and eight seeded servers of configuration 4, and on eight seeded
workers and eight seeded servers of configuration 5.
"""
import numpy as np
import pytest
import torch

from workloads import WORKLOADS, worker_sparse

pytestmark = pytest.mark.gpu


def _oracle_partition(oracle, wl, rows):
    own = (oracle.hash_many(rows, wl.hash_seed) % np.uint32(wl.n_parts)).astype(np.uint16)
    return oracle.partition(rows, own, wl.n_parts)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_full_size_workload(oracle, cid):
    import gpu_util as G
    import paper_2309_13254_amd as zen

    wl = WORKLOADS[cid]
    n, D = wl.n_parts, wl.row_dim
    print("workload", wl.name, flush=True)
    sparse = [worker_sparse(wl, w) for w in range(wl.n_workers)]
    grads = [G.dense_device(wl, r, v) for r, v in sparse]
    fmt = zen.ZEN_INDEX_BITMAP if wl.bitmap else zen.ZEN_INDEX_COO
    ctx = zen.ZenContext(wl.n_rows, D, n, wl.hash_seed, fmt)
    nnz = [r.size for r, _ in sparse]
    encs = [zen.alloc_encoded(ctx, c, with_indices=True) for c in nnz]
    ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, wl.n_workers))
    zen.zen_encode_batch(ctx, grads, encs, ws)
    st, flags, _ = zen.zen_status_fetch(ctx, ws)
    assert st == 0 and flags == 0
    offs = np.stack([G.u32(e.offsets).astype(np.int64) for e in encs])
    assert [int(o[-1]) for o in offs] == nnz                          # every planted row found, no other
    assert np.all(np.diff(offs, axis=1) >= 0)

    pick = np.random.default_rng(1000 + cid)
    check_workers = list(range(wl.n_workers)) if cid != 5 else sorted(pick.choice(wl.n_workers, size=8, replace=False).tolist())
    refs = {}
    for w in range(wl.n_workers):                                      # offsets: every worker
        refs[w] = _oracle_partition(oracle, wl, sparse[w][0])
        assert np.array_equal(offs[w], refs[w][0].astype(np.int64)), w
    print("offsets ok; indices and values on workers", check_workers, flush=True)
    for w in check_workers:
        rows, vals = sparse[w]
        r_off, r_idx = refs[w]
        assert np.array_equal(G.u32(encs[w].indices[:rows.size]), r_idx)
        # values = planted rows in output order (sampled rows for the wide tables)
        pos_of_row = np.searchsorted(rows, r_idx)
        if vals.nbytes <= (64 << 20):
            got = encs[w].values[:rows.size].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), vals[pos_of_row].view(np.uint32))
        else:
            sel = np.unique(np.random.default_rng(w).integers(0, rows.size, size=256))
            got = encs[w].values[torch.from_numpy(sel).cuda()].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), vals[pos_of_row[sel]].view(np.uint32))
    # Theorem 2 shape for Push on the large index sets
    sizes = np.diff(offs, axis=1)
    for w in range(wl.n_workers):
        assert sizes[w].max() * n / nnz[w] <= 1 + 3 * np.sqrt(n * np.log(n) / nnz[w])

    if wl.bitmap:
        total, woff, dsz = zen.zen_bitmap_layout(ctx)
        assert sum(dsz) == wl.n_rows and wl.n_rows // 32 <= total <= wl.n_rows // 32 + n
        owner = oracle.owner_table(wl.n_rows, n, wl.hash_seed)
        assert dsz == np.bincount(owner, minlength=n).tolist()
        pop8 = np.array([bin(i).count("1") for i in range(256)], np.uint8)
        for w in range(wl.n_workers):
            bm = G.u32(encs[w].bitmap[:total])
            r_off, r_idx = refs[w]
            for p in range(n):                                         # popcount = partition size, every worker
                words = bm[woff[p]:woff[p + 1]]
                assert int(pop8[words.view(np.uint8)].sum()) == int(r_off[p + 1]) - int(r_off[p])
            if w not in check_workers:
                continue
            for p in (3, int(pick.integers(0, n)), n - 1):             # decode sampled partitions
                dec = oracle.bitmap_decode(owner, p, bm[woff[p]:woff[p + 1]])
                assert np.array_equal(dec, r_idx[int(r_off[p]):int(r_off[p + 1])])
        del owner
        # the benchmark passes no index arrays: same offsets, bitmaps and values
        encs2 = [zen.alloc_encoded(ctx, c, with_indices=False) for c in nnz]
        zen.zen_encode_batch(ctx, grads, encs2, ws)
        assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
        for e1, e2, c in zip(encs, encs2, nnz):
            assert torch.equal(e1.offsets, e2.offsets) and torch.equal(e1.bitmap[:total], e2.bitmap[:total])
            assert torch.equal(e1.values[:c].view(torch.int32), e2.values[:c].view(torch.int32))
        del encs2

    per_server = np.diff(offs, axis=1).sum(axis=0)
    max_in = int(per_server.max() * 1.05) + 16
    aggs = [zen.alloc_aggregated(ctx, max_in) for _ in range(n)]
    ws2 = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, n, max_in))
    zen.zen_aggregate_batch(ctx, encs, aggs, max_in, ws2)
    st, flags, _ = zen.zen_status_fetch(ctx, ws2)
    assert st == 0 and flags == 0
    counts = [int(a.count.item()) for a in aggs]
    union = np.unique(np.concatenate([r for r, _ in sparse]))
    assert sum(counts) == union.size                                   # sum_j U_j = |union|
    assert max(counts) * n / union.size <= 1 + 3 * np.sqrt(n * np.log(n) / union.size)   # Theorem 2, Pull

    # U_j of every server = the oracle's union of the workers' rows, split by owner
    own_u = (oracle.hash_many(union.astype(np.uint32), wl.hash_seed) % np.uint32(n)).astype(np.int64)
    assert counts == np.bincount(own_u, minlength=n).tolist()
    del own_u
    check_servers = list(range(n)) if cid in (1, 2, 3) else sorted(pick.choice(n, size=8, replace=False).tolist())
    print("counts ok; sums on servers", check_servers, flush=True)
    agg_refs = {}
    for j in check_servers:
        parts = []
        for w in range(wl.n_workers):
            rows, vals = sparse[w]
            r_off, r_idx = refs[w]
            seg = r_idx[int(r_off[j]):int(r_off[j + 1])]
            parts.append((seg, vals[np.searchsorted(rows, seg)]))
        ref = oracle.aggregate(parts, wl.n_rows, D)
        U, idx, val = G.aggregated_to_host(aggs[j])
        assert U == ref.U and np.array_equal(idx, ref.indices)
        G.check_sums(val, ref)
        agg_refs[j] = ref
        del parts, val

    # Pull: every server's hash bitmap of what it aggregated, then the worker's decode + placement into
    # the dense synchronized tensor.  Bitmaps: popcount of every partition = its row count, sampled
    # partitions decoded by the oracle.  Dense tensor: rows of the sampled servers against the
    # oracle's sums, sampled rows outside the union exactly zero.
    del grads
    torch.cuda.empty_cache()
    pctx = ctx if wl.bitmap else zen.ZenContext(wl.n_rows, D, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    total, woff, dsz = zen.zen_bitmap_layout(pctx)
    ws3 = zen.alloc_workspace(zen.zen_pull_workspace_bytes(pctx))
    bitmap = torch.empty(max(total, 1), dtype=torch.int32, device="cuda")
    zen.zen_pull_encode_batch(pctx, aggs, bitmap, ws3)
    assert zen.zen_status_fetch(pctx, ws3) == (0, 0, 0)
    bm = G.u32(bitmap[:total])
    pop8 = np.array([bin(i).count("1") for i in range(256)], np.uint8)
    for p in range(n):
        assert int(pop8[bm[woff[p]:woff[p + 1]].view(np.uint8)].sum()) == counts[p]
    owner = oracle.owner_table(wl.n_rows, n, wl.hash_seed)
    for j in check_servers:
        assert np.array_equal(oracle.bitmap_decode(owner, j, bm[woff[j]:woff[j + 1]]), agg_refs[j].indices)
    dense = torch.empty((wl.n_rows, D), dtype=torch.float32, device="cuda")
    parts = [(None, bitmap[woff[p]:], aggs[p].values, aggs[p].count) for p in range(n)]
    zen.zen_pull_apply(pctx, parts, dense, ws3)
    assert zen.zen_status_fetch(pctx, ws3) == (0, 0, 0)
    for j in check_servers:
        ref = agg_refs[j]
        sel = torch.from_numpy(ref.indices.astype(np.int64)).cuda()
        G.check_sums(dense[sel].cpu().numpy(), ref)
    rng = np.random.default_rng(cid)
    probe = np.setdiff1d(np.unique(rng.integers(0, wl.n_rows, size=200000)), union)
    if probe.size:
        assert not dense[torch.from_numpy(probe).cuda()].any().item()
    nz_rows = int((dense != 0).any(dim=1).sum().item())
    assert nz_rows <= union.size and nz_rows >= union.size - 64          # only exact cancellations may be missing
