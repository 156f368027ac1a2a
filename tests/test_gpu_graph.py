"""The stream entry points under HIP graph capture: encode -> aggregate -> pull bitmap -> pull placement
is captured once and replayed with new gradient contents in the same buffers; every replay must give the
dense sum of that replay's gradients (checked against a float64 sum on the host), with eager work and
synchronisations between the replays."""
import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, dense_from_sparse, worker_sparse

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid,fmt_bitmap", [(1, False), (2, False), (3, True), (5, True)])
def test_graph_replays_track_inputs(oracle, cid, fmt_bitmap):
    import gpu_util as G
    import paper_2309_13254_amd as zen

    zen.load_library()
    wl = MINI_WORKLOADS[cid]
    R, D, n, W = wl.n_rows, wl.row_dim, wl.n_parts, min(wl.n_workers, 8)
    reps = 3
    inputs = [[worker_sparse(wl, w + 1000 * rep) for w in range(W)] for rep in range(reps + 1)]
    cap = max(r.size for rep in inputs for r, _ in rep)
    cap_total = max(sum(r.size for r, _ in rep) for rep in inputs)

    ctx = zen.ZenContext(R, D, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP if fmt_bitmap else zen.ZEN_INDEX_COO)
    pctx = ctx if fmt_bitmap else zen.ZenContext(R, D, n, wl.hash_seed, zen.ZEN_INDEX_BITMAP)
    grads = [torch.zeros((R, D), dtype=torch.float32, device="cuda") for _ in range(W)]
    encs = [zen.alloc_encoded(ctx, cap) for _ in range(W)]
    aggs = [zen.alloc_aggregated(ctx, cap_total) for _ in range(n)]
    ws_enc = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, W))
    ws_agg = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, n, cap_total))
    ws_pull = zen.alloc_workspace(zen.zen_pull_workspace_bytes(pctx))
    tot_words, woff, _ = zen.zen_bitmap_layout(pctx)
    bitmap = torch.empty(max(tot_words, 1), dtype=torch.int32, device="cuda")
    dense = torch.empty((R, D), dtype=torch.float32, device="cuda")
    parts = [(None, bitmap[woff[p]:] if woff[p] < bitmap.numel() else bitmap, aggs[p].values, aggs[p].count)
             for p in range(n)]

    def set_inputs(rep):
        for g, (rows, vals) in zip(grads, inputs[rep]):
            g.zero_()
            if rows.size:
                g.index_copy_(0, torch.from_numpy(rows.astype(np.int64)).cuda(),
                              torch.from_numpy(np.ascontiguousarray(vals)).cuda())

    def step():
        zen.zen_encode_batch(ctx, grads, encs, ws_enc)
        zen.zen_aggregate_batch(ctx, encs, aggs, cap_total, ws_agg)
        zen.zen_pull_encode_batch(pctx, aggs, bitmap, ws_pull)
        zen.zen_pull_apply(pctx, parts, dense, ws_pull)

    def check(rep, what):
        for ws, c in ((ws_enc, ctx), (ws_agg, ctx), (ws_pull, pctx)):
            assert zen.zen_status_fetch(c, ws) == (0, 0, 0), what
        total64 = np.zeros((R, D), np.float64)
        abs64 = np.zeros((R, D), np.float64)
        ncontrib = np.zeros(R, np.int64)
        for rows, vals in inputs[rep]:
            g = dense_from_sparse(wl, rows, vals).reshape(R, D).astype(np.float64)
            total64 += g
            abs64 += np.abs(g)
            ncontrib[rows] += 1
        got = dense.cpu().numpy()
        assert (np.abs(got.astype(np.float64) - total64) <= 1e-6 * abs64).all(), what
        one = ncontrib == 1
        assert np.array_equal(got[one].view(np.uint32), total64[one].astype(np.float32).view(np.uint32)), what
        assert sum(int(a.count.item()) for a in aggs) == int(np.count_nonzero(ncontrib)), what

    # eager first (also the first-call set-up of the kernels), on the last input set
    set_inputs(reps)
    step()
    torch.cuda.synchronize()
    check(reps, "eager")

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()

    for rep in range(reps):
        print("replay", rep, flush=True)
        set_inputs(rep)                       # eager work between the replays
        dense.fill_(float("nan"))
        bitmap.fill_(-1)
        for a in aggs:
            a.count.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check(rep, "replay %d" % rep)
