"""GPU parity of Algorithm 1's hash-memory mechanism (zen_encode_hashed) against the CPU oracle.

The order inside a partition depends on which thread wins a contested cell, so what is compared is
what is unique: the offsets, the SET of indices of every partition, the value that travels with each
index, where an index may legally sit in the memory (one of its k cells, or the serial region), and
-- with one hash function, where the split is order-independent -- the exact serial counts."""
import numpy as np
import pytest
import torch

from workloads import MINI_WORKLOADS, Workload, dense_from_sparse, worker_sparse

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


def _run(zen, ctx, grad, k, seed2, r1, r2, cap):
    mem = zen.alloc_workspace(zen.zen_hash_memory_bytes(ctx, k, seed2, r1, r2))
    ws = zen.alloc_workspace(zen.zen_encode_hashed_workspace_bytes(ctx, k, seed2, r1, r2))
    out = zen.alloc_encoded(ctx, cap)
    serial = torch.zeros(ctx.n_parts, dtype=torch.int32, device="cuda")
    zen.zen_encode_hashed(ctx, grad, k, seed2, r1, r2, mem, out, serial, ws)
    st = zen.zen_status_fetch(ctx, ws)
    return out, serial, mem, st


CASES = [(1, 1, 1, 1, 0.5), (33, 1, 3, 2, 0.5), (5000, 1, 4, 3, 0.5), (70001, 1, 64, 1, 0.5), (300000, 1, 16, 3, 0.5),
         (300000, 1, 16, 4, 1.0), (9001, 64, 16, 3, 0.25), (333, 256, 8, 2, 0.5), (97, 1024, 8, 1, 2.0),
         (40000, 4, 1000, 3, 0.5), (100000, 2, 5, 8, 0.5)]


@pytest.mark.parametrize("R,D,n,k,load", CASES)
def test_hashed_encode_matches_oracle(oracle, zen, R, D, n, k, load):
    import gpu_util as G

    rng = np.random.default_rng(R + 7 * D + n + k)
    seed0, seed2 = int(rng.integers(0, 2**32)), int(rng.integers(0, 2**31))
    wl = Workload("t", 0, R, D, n, seed0, "uniform")
    ctx = zen.ZenContext(R, D, n, seed0, zen.ZEN_INDEX_COO)
    for density in (0.0, 0.05, 0.6):
        rows = np.flatnonzero(rng.random(R) < density).astype(np.uint32)
        vals = rng.standard_normal((rows.size, D)).astype(np.float32) + 4.0
        host = dense_from_sparse(wl, rows, vals)
        grad = torch.from_numpy(host).cuda()
        r1 = max(1, int(np.ceil(max(rows.size, 1) / n / load)))
        r2 = rows.size + 1
        out, serial, mem, st = _run(zen, ctx, grad, k, seed2, r1, r2, rows.size)
        assert st == (0, 0, 0)
        part = (oracle.hash_many(rows, seed0) % np.uint32(n)).astype(np.uint16)
        ref_off, ref_idx = oracle.partition(rows, part, n)
        off = G.u32(out.offsets)
        assert np.array_equal(off, ref_off)
        idx = G.u32(out.indices[:rows.size])
        got_vals = out.values[:rows.size].cpu().numpy()
        for p in range(n):
            seg = idx[off[p]:off[p + 1]]
            assert np.array_equal(np.sort(seg), ref_idx[off[p]:off[p + 1]])            # the set, each index once
        if rows.size:                                                                   # values = G[indices]
            assert np.array_equal(got_vals.view(np.uint32), vals[np.searchsorted(rows, idx)].view(np.uint32))
        # where the indices sit in the memory
        slots = [oracle.hash_slots(rows, seed2 + i, r1) for i in range(1, k + 1)]
        x = G.u32(mem.view(torch.int32)[: n * (r1 + r2)]).reshape(n, r1 + r2)
        ser = G.u32(serial)
        ref = oracle.hierarchical_hash(rows, part, slots, n, r1, r2)
        assert ref.rc == 0
        for p in range(n):
            par = x[p, :r1]
            cells = np.flatnonzero(par != 0xFFFFFFFF)
            t = np.searchsorted(rows, par[cells])                                       # position of each index in I
            assert np.array_equal(rows[t], par[cells]) and (part[t] == p).all()
            legal = np.zeros(cells.size, bool)
            for s in slots:
                legal |= s[t] == cells
            assert legal.all()                                                          # one of its k cells
            tail = x[p, r1:]
            assert (tail[:ser[p]] != 0xFFFFFFFF).all() and (tail[ser[p]:] == 0xFFFFFFFF).all()
            assert cells.size + int(ser[p]) == int(off[p + 1]) - int(off[p])
        if k == 1:
            assert np.array_equal(ser.astype(np.uint64), ref.serial_count)              # order-independent
        else:   # the order of insertion moves a few indices between the regions, no more
            one = oracle.hierarchical_hash(rows, part, slots[:1], n, r1, r2).serial_count
            assert (ser.astype(np.uint64) <= one).all()
            assert abs(int(ser.sum()) - int(ref.serial_count.sum())) <= 0.25 * ref.serial_count.sum() + 32


def test_hashed_encode_overflows_are_reported(oracle, zen):
    import gpu_util as G

    R, D, n, seed0, seed2 = 60000, 1, 4, 11, 22
    wl = Workload("t", 0, R, D, n, seed0, "uniform")
    rng = np.random.default_rng(0)
    rows = np.flatnonzero(rng.random(R) < 0.2).astype(np.uint32)
    vals = rng.standard_normal((rows.size, D)).astype(np.float32) + 4.0
    grad = torch.from_numpy(dense_from_sparse(wl, rows, vals)).cuda()
    ctx = zen.ZenContext(R, D, n, seed0, zen.ZEN_INDEX_COO)
    part = (oracle.hash_many(rows, seed0) % np.uint32(n)).astype(np.uint16)
    r1 = rows.size // n // 2
    need = int(oracle.hierarchical_hash(rows, part, [oracle.hash_slots(rows, seed2 + 1, r1)], n, r1, rows.size).serial_count.max())
    out, serial, mem, (st, flags, needed) = _run(zen, ctx, grad, 1, seed2, r1, need, rows.size)     # just enough
    assert st == 0 and int(G.u32(out.offsets)[-1]) == rows.size
    out, serial, mem, (st, flags, needed) = _run(zen, ctx, grad, 1, seed2, r1, need - 1, rows.size)  # one cell short
    assert st == zen.ZEN_ERR_CAPACITY and flags & 2 and needed == need
    assert int(G.u32(out.offsets)[-1]) == rows.size - 1                  # exactly one index was dropped
    # output capacity: nothing written past it, the count is still complete
    out = zen.alloc_encoded(ctx, rows.size)
    out.indices.fill_(-1)
    out.cap_rows = 100
    mem = zen.alloc_workspace(zen.zen_hash_memory_bytes(ctx, 3, seed2, 2 * r1, rows.size))
    ws = zen.alloc_workspace(zen.zen_encode_hashed_workspace_bytes(ctx, 3, seed2, 2 * r1, rows.size))
    zen.zen_encode_hashed(ctx, grad, 3, seed2, 2 * r1, rows.size, mem, out, None, ws)
    st, flags, needed = zen.zen_status_fetch(ctx, ws)
    assert st == zen.ZEN_ERR_CAPACITY and flags & 1 and needed == rows.size
    assert int(G.u32(out.offsets)[-1]) == rows.size and (out.indices[100:] == -1).all().item()
    with pytest.raises(zen.ZenError):                                    # k out of range
        zen.zen_hash_memory_bytes(ctx, 0, 1, 10, 10)
    with pytest.raises(zen.ZenError):
        zen.zen_hash_memory_bytes(ctx, 9, 1, 10, 10)
    with pytest.raises(zen.ZenError):                                    # hash memory too small
        zen.zen_encode_hashed(ctx, grad, 3, seed2, 2 * r1, rows.size, mem[:4096], out, None, ws)


@pytest.mark.parametrize("cid", [2, 3])
def test_hashed_encode_then_aggregate(oracle, zen, cid):
    """Unordered partitions from the hash memory feed zen_aggregate like ordered ones."""
    import gpu_util as G

    wl = MINI_WORKLOADS[cid]
    R, D, n = wl.n_rows, wl.row_dim, wl.n_parts
    ctx = zen.ZenContext(R, D, n, wl.hash_seed, zen.ZEN_INDEX_COO)
    sparse = [worker_sparse(wl, w) for w in range(wl.n_workers)]
    encs, refs = [], []
    for w, (rows, vals) in enumerate(sparse):
        grad = G.dense_device(wl, rows, vals)
        r1 = max(1, 2 * rows.size // n)
        out, serial, mem, st = _run(zen, ctx, grad, 3, 1000 + w, r1, rows.size + 1, rows.size)
        assert st == (0, 0, 0)
        encs.append(out)
        refs.append(oracle.encode(dense_from_sparse(wl, rows, vals), R, D, n, wl.hash_seed))
    per_server = [sum(int(e.offsets[j + 1]) - int(e.offsets[j]) for e in refs) for j in range(n)]
    outs, st = G.run_aggregate_batch(ctx, encs, [max(p, 1) for p in per_server], max(per_server))
    assert st == (0, 0, 0)
    for j in range(n):
        parts = [(e.indices[e.offsets[j]:e.offsets[j + 1]], e.values[e.offsets[j]:e.offsets[j + 1]]) for e in refs]
        ref = oracle.aggregate(parts, R, D)
        U, idx, val = G.aggregated_to_host(outs[j])
        assert U == ref.U and np.array_equal(idx, ref.indices)
        G.check_sums(val, ref)
