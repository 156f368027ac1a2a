"""More tiles than the partition scan keeps flag bits for in LDS (131,072): the scan then reads the tile flags from
memory.  An element-level tensor of 2^28 + 5,000 rows with the smallest tile (2,048 rows) has 131,075 tiles."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_encode_with_more_tiles_than_lds_flag_bits(oracle, monkeypatch):
    import gpu_util as G
    import paper_2309_13254_amd as zen

    zen.load_library()
    G.use_tuning(monkeypatch, tiled_encode=True, tile_bytes=8192)        # 2,048 rows per tile
    R, n, seed = (1 << 28) + 5000, 7, 0x5EED1234
    rng = np.random.default_rng(42)
    rows = np.unique(np.concatenate([
        rng.integers(0, R, size=60000),                  # scattered rows: most tiles stay empty
        np.arange(12345, 12345 + 3000),                  # a run over two tiles
        np.arange(R - 900, R),                           # the ragged last tile
        np.arange((1 << 27) - 70, (1 << 27) + 70),
    ])).astype(np.uint32)
    vals = (rng.standard_normal(rows.size).astype(np.float32) + 3.0).reshape(-1, 1)
    host = np.zeros(R, np.float32)
    host[rows] = vals[:, 0]
    print("oracle encode ...", flush=True)
    ref = oracle.encode(host.reshape(R, 1), R, 1, n, seed)
    assert ref.nnz == rows.size
    grad = torch.from_numpy(host).cuda().reshape(R, 1)
    for fmt in (zen.ZEN_INDEX_COO, zen.ZEN_INDEX_BITMAP):
        print("format", fmt, flush=True)
        ctx = zen.ZenContext(R, 1, n, seed, fmt)
        enc = zen.alloc_encoded(ctx, rows.size)
        ws = zen.alloc_workspace(zen.zen_encode_workspace_bytes(ctx, 1))
        ws.view(torch.int32).fill_(-1)
        zen.zen_encode_batch(ctx, [grad], [enc], ws)
        assert zen.zen_status_fetch(ctx, ws) == (0, 0, 0)
        assert np.array_equal(G.u32(enc.offsets), ref.offsets)
        assert np.array_equal(G.u32(enc.indices[:ref.nnz]), ref.indices)
        assert np.array_equal(enc.values[:ref.nnz].cpu().numpy().view(np.uint32), ref.values.view(np.uint32))
        if fmt == zen.ZEN_INDEX_BITMAP:
            total, woff, _ = zen.zen_bitmap_layout(ctx)
            bm = G.u32(enc.bitmap[:total])
            pop8 = np.array([bin(i).count("1") for i in range(256)], np.uint8)
            for p in range(n):                           # popcount of every partition = its row count
                assert int(pop8[bm[woff[p]:woff[p + 1]].view(np.uint8)].sum()) == int(ref.offsets[p + 1]) - int(ref.offsets[p])
        del ctx, enc, ws
        torch.cuda.empty_cache()
