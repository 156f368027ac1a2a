"""GPU parity: zen_aggregate / zen_aggregate_batch against the CPU oracle.

Indices and counts bit-exact; fp32 sums within 1e-6 * sum|x| of the oracle's fp64 sum (the device adds
in fp32, in ascending (part, row) order), bit-exact where a row has a single contributor, and bit-identical
between the device's table paths.
"""
import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, dense_from_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


def _oracle_parts(oracle, wl, sparse):
    encs = []
    for rows, vals in sparse:
        encs.append(oracle.encode(dense_from_sparse(wl, rows, vals), wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed))
    return encs


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
@pytest.mark.parametrize("big_table", [False, True])
def test_encode_then_aggregate_batch(oracle, zen, cid, big_table):
    import gpu_util as G

    wl = MINI_WORKLOADS[cid]
    sparse, grads = G.workload_inputs(wl)
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, wl.n_parts, wl.hash_seed)
    encs, (st, _, _) = G.run_encode_batch(ctx, grads, [r.size for r, _ in sparse])
    assert st == 0
    ref_encs = _oracle_parts(oracle, wl, sparse)
    per_server = [sum(int(e.offsets[j + 1]) - int(e.offsets[j]) for e in ref_encs) for j in range(wl.n_parts)]
    # big_table forces the multi-kernel (radix sort) path, the other the one-block LDS path when it fits
    max_in = max(per_server) if not big_table else max(max(per_server), 20000)
    outs, (st, flags, needed) = G.run_aggregate_batch(ctx, encs, [max(p, 1) for p in per_server], max_in)
    assert st == 0 and flags == 0
    total_u = 0
    for j in range(wl.n_parts):
        parts = [(e.indices[e.offsets[j]:e.offsets[j + 1]], e.values[e.offsets[j]:e.offsets[j + 1]]) for e in ref_encs]
        ref = oracle.aggregate(parts, wl.n_rows, wl.row_dim)
        U, idx, val = G.aggregated_to_host(outs[j])
        assert U == ref.U
        assert np.array_equal(idx, ref.indices)
        G.check_sums(val, ref)
        total_u += U
    union = set()
    for rows, _ in sparse:
        union.update(rows.tolist())
    assert total_u == len(union)


@pytest.mark.parametrize("D", [1, 3, 4, 64, 256, 1024])
@pytest.mark.parametrize("max_in_scale", [1, 40])
def test_single_server_explicit_parts(oracle, zen, D, max_in_scale):
    import gpu_util as G

    rng = np.random.default_rng(D + max_in_scale)
    R, n_in = 50000, 7
    ctx = zen.ZenContext(R, D, 4, 123)
    parts_h = []
    for w in range(n_in):
        c = int(rng.integers(0, 600)) if w != 3 else 0               # one empty part
        idx = rng.integers(0, R, size=c).astype(np.uint32)            # unsorted, duplicates inside a part
        val = rng.standard_normal((c, D)).astype(np.float32)
        parts_h.append((idx, val))
    total = sum(i.size for i, _ in parts_h)
    ref = oracle.aggregate(parts_h, R, D)
    parts_d = []
    for idx, val in parts_h:
        parts_d.append((G.to_dev(idx) if idx.size else torch.empty(1, dtype=torch.int32, device="cuda"), None,
                        torch.from_numpy(val).cuda() if idx.size else torch.empty((1, D), device="cuda"),
                        torch.tensor([idx.size], dtype=torch.int32, device="cuda")))
    max_in = total * max_in_scale
    out = zen.alloc_aggregated(ctx, total)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, max_in))
    zen.zen_aggregate(ctx, parts_d, 2, out, max_in, ws)
    st, flags, _ = zen.zen_status_fetch(ctx, ws)
    assert st == 0 and flags == 0
    U, idx, val = G.aggregated_to_host(out)
    assert U == ref.U and np.array_equal(idx, ref.indices)
    G.check_sums(val, ref)


@pytest.mark.parametrize("ascending", [False, True])
@pytest.mark.parametrize("D", [1, 4, 64, 256])
def test_paths_agree_bit_for_bit(oracle, zen, D, ascending):
    """Both table paths sum every output row from its contributors in ascending (part, row) order: the one-block
    LDS path and the multi-kernel path give the same bits, run after run, whatever the workspace held."""
    import gpu_util as G

    rng = np.random.default_rng(100 + D)
    R, n_in = 30000, 9
    ctx = zen.ZenContext(R, D, 4, 77)
    parts_d, total = [], 0
    for w in range(n_in):
        c = int(rng.integers(100, 600))
        idx = rng.integers(0, 2000, size=c).astype(np.uint32)          # heavy overlap, duplicates inside a part
        if ascending:                                                  # what zen_encode sends: the merge without a table
            idx = np.unique(idx)
            c = idx.size
        val = rng.standard_normal((c, D)).astype(np.float32)
        parts_d.append((G.to_dev(idx), None, torch.from_numpy(val).cuda(),
                        torch.tensor([c], dtype=torch.int32, device="cuda")))
        total += c
    results = []
    for max_in, fill in ((total, 0), (total * 40, 0), (total * 40, -1), (total * 40, 0x3F800000)):
        out = zen.alloc_aggregated(ctx, total)
        ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, max_in))
        ws[: ws.numel() // 4 * 4].view(torch.int32).fill_(fill)
        zen.zen_aggregate(ctx, parts_d, 1, out, max_in, ws)
        assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
        results.append(G.aggregated_to_host(out))
    U0, idx0, val0 = results[0]
    ref = oracle.aggregate([(G.u32(p[0]), p[2].cpu().numpy()) for p in parts_d], R, D)
    assert U0 == ref.U and np.array_equal(idx0, ref.indices)
    G.check_sums(val0, ref)
    for U, idx, val in results[1:]:
        assert U == U0 and np.array_equal(idx, idx0)
        assert np.array_equal(val.view(np.uint32), val0.view(np.uint32))


def test_disjoint_and_identical_inputs(oracle, zen):
    import gpu_util as G

    R, D = 4000, 8
    ctx = zen.ZenContext(R, D, 2, 5)
    rng = np.random.default_rng(3)
    perm = rng.permutation(R).astype(np.uint32)[:900]
    vals = rng.standard_normal((900, D)).astype(np.float32)
    cnt = lambda k: torch.tensor([k], dtype=torch.int32, device="cuda")
    # disjoint: output = sorted concatenation, bit-exact
    parts = [(G.to_dev(perm[i * 300:(i + 1) * 300]), None, torch.from_numpy(vals[i * 300:(i + 1) * 300]).cuda(), cnt(300))
             for i in range(3)]
    out = zen.alloc_aggregated(ctx, 900)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, 900))
    zen.zen_aggregate(ctx, parts, 0, out, 900, ws)
    assert zen.zen_status_fetch(ctx, ws)[0] == 0
    U, idx, val = G.aggregated_to_host(out)
    order = np.argsort(perm)
    assert U == 900 and np.array_equal(idx, perm[order])
    assert np.array_equal(val.view(np.uint32), vals[order].view(np.uint32))
    # the same part four times: values x4 exactly (power of two)
    p0 = (G.to_dev(perm[:300]), None, torch.from_numpy(vals[:300]).cuda(), cnt(300))
    zen.zen_aggregate(ctx, [p0] * 4, 1, out, 1200, zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, 1200)))
    torch.cuda.synchronize()
    U, idx, val = G.aggregated_to_host(out)
    o = np.argsort(perm[:300])
    assert U == 300 and np.array_equal(idx, perm[:300][o])
    assert np.array_equal(val, vals[:300][o] * np.float32(4))
    # cancellation keeps the index
    a = (G.to_dev(np.array([7, 9], np.uint32)), None, torch.tensor([[1.5] * D, [2.0] * D], device="cuda"), cnt(2))
    b = (G.to_dev(np.array([7], np.uint32)), None, torch.tensor([[-1.5] * D], device="cuda"), cnt(1))
    zen.zen_aggregate(ctx, [a, b], 0, out, 900, ws)
    assert zen.zen_status_fetch(ctx, ws)[0] == 0
    U, idx, val = G.aggregated_to_host(out)
    assert U == 2 and idx.tolist() == [7, 9] and np.all(val[0] == 0) and np.all(val[1] == 2.0)


def test_overflow_flags(oracle, zen):
    import gpu_util as G

    R, D = 10000, 4
    ctx = zen.ZenContext(R, D, 2, 5)
    idx = np.arange(0, 3000, 3, dtype=np.uint32)
    val = np.ones((idx.size, D), np.float32)
    part = (G.to_dev(idx), None, torch.from_numpy(val).cuda(), torch.tensor([idx.size], dtype=torch.int32, device="cuda"))
    # bound on incoming rows too small: table flag, count 0, needed = actual total
    out = zen.alloc_aggregated(ctx, 2000)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, 500))
    zen.zen_aggregate(ctx, [part, part], 0, out, 500, ws)
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    assert st == zen.ZEN_ERR_CAPACITY and (flags & 2) and needed == 2 * idx.size
    assert int(out.count.item()) == 0
    # output capacity too small: capacity flag, count = U, first rows correct, nothing past the capacity
    guard_idx = torch.full((1000,), -2, dtype=torch.int32, device="cuda")
    guard_val = torch.full((1000, D), 7.0, device="cuda")
    out2 = zen.Aggregated(guard_idx, guard_val, torch.zeros(1, dtype=torch.int32, device="cuda"), 600)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, 2000))
    zen.zen_aggregate(ctx, [part, part], 0, out2, 2000, ws)
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    assert st == zen.ZEN_ERR_CAPACITY and (flags & 1) and needed == idx.size
    assert int(out2.count.item()) == idx.size
    assert np.array_equal(G.u32(guard_idx[:600]), idx[:600])
    assert torch.all(guard_val[:600] == 2.0)
    assert torch.all(guard_idx[600:] == -2) and torch.all(guard_val[600:] == 7.0)


@pytest.mark.parametrize("fmt_bitmap", [False, True])
@pytest.mark.parametrize("big_table", [False, True])
def test_aggregate_batch_more_servers_than_one_launch_group(oracle, zen, fmt_bitmap, big_table):
    """n_parts = 100: zen_aggregate_batch handles the servers in groups of ZEN_MAX_BATCH; every server's output
    is compared with the oracle, and an output capacity that is too small in the FIRST group only must still
    be reported after the last group."""
    import gpu_util as G
    from workloads import Workload

    wl = Workload("agg100", 0, 300_007, 1 if fmt_bitmap else 8, 6, 0xABCD1234, "uniform", nnz=9_000, sigma=1.0)
    n = 100
    sparse, grads = G.workload_inputs(wl)
    fmt = zen.ZEN_INDEX_BITMAP if fmt_bitmap else zen.ZEN_INDEX_COO
    ctx = zen.ZenContext(wl.n_rows, wl.row_dim, n, wl.hash_seed, fmt)
    encs, (st, _, _) = G.run_encode_batch(ctx, grads, [r.size for r, _ in sparse])
    assert st == 0
    refs = [oracle.encode(dense_from_sparse(wl, r, v), wl.n_rows, wl.row_dim, n, wl.hash_seed) for r, v in sparse]
    per_server = [sum(int(e.offsets[j + 1]) - int(e.offsets[j]) for e in refs) for j in range(n)]
    max_in = max(per_server) if not big_table else max(max(per_server), 20000)
    e_bytes, a_bytes = zen.zen_workspace_bytes(ctx, max_in, n)
    assert e_bytes == zen.zen_encode_workspace_bytes(ctx, n) and a_bytes == zen.zen_aggregate_workspace_bytes(ctx, n, max_in)
    outs, (st, flags, needed) = G.run_aggregate_batch(ctx, encs, [max(p, 1) for p in per_server], max_in)
    assert st == 0 and flags == 0 and zen.zen_last_overflow(ctx) == 0
    ref_out = []
    for j in range(n):
        parts = [(e.indices[e.offsets[j]:e.offsets[j + 1]], e.values[e.offsets[j]:e.offsets[j + 1]]) for e in refs]
        ref = oracle.aggregate(parts, wl.n_rows, wl.row_dim)
        ref_out.append(ref)
        U, idx, val = G.aggregated_to_host(outs[j])
        assert U == ref.U, j
        assert np.array_equal(idx, ref.indices), j
        G.check_sums(val, ref)
    # server 3 (first group) gets room for 5 rows only
    caps = [max(p, 1) for p in per_server]
    caps[3] = 5
    outs, (st, flags, needed) = G.run_aggregate_batch(ctx, encs, caps, max_in)
    assert st == zen.ZEN_ERR_CAPACITY and (flags & 1) and needed == ref_out[3].U
    assert zen.zen_last_overflow(ctx) == ref_out[3].U
    U, idx, _ = G.aggregated_to_host(outs[3])
    assert U == ref_out[3].U and np.array_equal(idx, ref_out[3].indices[:5])
    U, idx, _ = G.aggregated_to_host(outs[99])
    assert U == ref_out[99].U and np.array_equal(idx, ref_out[99].indices)


@pytest.mark.parametrize("ascending", [False, True])
@pytest.mark.parametrize("n_in", [1, 9, 23])
@pytest.mark.parametrize("D", [256, 260, 1024])
def test_one_launch_merge_of_few_wide_rows(oracle, zen, D, n_in, ascending):
    """At most 2,048 incoming rows of wide rows: merge and sums run in one launch (binary-search merge for ascending
    parts, a sort otherwise).  Against the oracle, bit for bit against the multi-kernel table path, and with an
    output capacity and a bound on the incoming rows that are too small."""
    import gpu_util as G

    rng = np.random.default_rng(7 * D + n_in + int(ascending))
    R = 30000
    ctx = zen.ZenContext(R, D, 4, 77)
    parts_d, total = [], 0
    for w in range(n_in):
        c = int(rng.integers(0, 2000 // n_in))
        idx = rng.integers(0, 1500, size=c).astype(np.uint32)          # heavy overlap, duplicates inside a part
        if ascending:
            idx = np.unique(idx)
            c = idx.size
        val = rng.standard_normal((max(c, 1), D)).astype(np.float32)[:c]
        parts_d.append((G.to_dev(idx) if c else torch.empty(1, dtype=torch.int32, device="cuda"), None,
                        torch.from_numpy(val).cuda() if c else torch.empty((1, D), device="cuda"),
                        torch.tensor([c], dtype=torch.int32, device="cuda")))
        total += c
    assert 0 < total <= 2048
    ref = oracle.aggregate([(G.u32(p[0])[:int(p[3].item())], p[2].cpu().numpy()[:int(p[3].item())]) for p in parts_d], R, D)
    results = []
    for max_in in (total, 2048, total * 40):                            # one launch twice, then the table path
        out = zen.alloc_aggregated(ctx, total)
        ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, max_in))
        ws[: ws.numel() // 4 * 4].view(torch.int32).fill_(-1)
        zen.zen_aggregate(ctx, parts_d, 1, out, max_in, ws)
        assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
        results.append(G.aggregated_to_host(out))
    U0, idx0, val0 = results[0]
    assert U0 == ref.U and np.array_equal(idx0, ref.indices)
    G.check_sums(val0, ref)
    for U, idx, val in results[1:]:
        assert U == U0 and np.array_equal(idx, idx0)
        assert np.array_equal(val.view(np.uint32), val0.view(np.uint32))
    if ref.U > 3:
        # output capacity too small: flag, count = U, the first rows correct, nothing past the capacity
        cap = ref.U // 2
        guard_idx = torch.full((ref.U,), -2, dtype=torch.int32, device="cuda")
        guard_val = torch.full((ref.U, D), 7.0, device="cuda")
        out2 = zen.Aggregated(guard_idx, guard_val, torch.zeros(1, dtype=torch.int32, device="cuda"), cap)
        ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, total))
        zen.zen_aggregate(ctx, parts_d, 1, out2, total, ws)
        st, flags, needed = zen.zen_status_fetch(ctx, ws)
        assert st == zen.ZEN_ERR_CAPACITY and flags == 1 and needed == ref.U and zen.zen_last_overflow(ctx) == ref.U
        assert int(out2.count.item()) == ref.U
        assert np.array_equal(G.u32(guard_idx[:cap]), ref.indices[:cap])
        assert np.array_equal(guard_val[:cap].cpu().numpy().view(np.uint32), val0[:cap].view(np.uint32))
        assert torch.all(guard_idx[cap:] == -2) and torch.all(guard_val[cap:] == 7.0)
        # bound on the incoming rows too small: table flag, nothing put out
        out3 = zen.alloc_aggregated(ctx, total)
        ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, total - 1))
        zen.zen_aggregate(ctx, parts_d, 1, out3, total - 1, ws)
        st, flags, needed = zen.zen_status_fetch(ctx, ws)
        assert st == zen.ZEN_ERR_CAPACITY and flags == 2 and needed == total
        assert int(out3.count.item()) == 0


def test_one_launch_merge_flags_a_reserved_index(oracle, zen):
    import gpu_util as G

    D, R = 256, 1000
    ctx = zen.ZenContext(R, D, 2, 5)
    idx = np.array([3, 0xFFFFFFFF, 9], np.uint32)
    part = (G.to_dev(idx), None, torch.ones((3, D), device="cuda"), torch.tensor([3], dtype=torch.int32, device="cuda"))
    out = zen.alloc_aggregated(ctx, 8)
    ws = zen.alloc_workspace(zen.zen_aggregate_workspace_bytes(ctx, 1, 8))
    zen.zen_aggregate(ctx, [part, part], 0, out, 8, ws)
    st, flags, _ = zen.zen_status_fetch(ctx, ws)
    assert st == zen.ZEN_ERR_INVALID and flags == 4
    U, idx_out, val = G.aggregated_to_host(out)
    assert U == 2 and idx_out.tolist() == [3, 9] and np.all(val == 2.0)
