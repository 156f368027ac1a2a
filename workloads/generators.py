"""Seeded synthetic sparse gradients with the shapes, densities and skew of the paper's workloads.

Every worker's gradient is produced in *sparse form* (ascending unique non-zero row ids + the rows'
values); the dense buffer is materialised from it separately on the host (for the oracle) or on the
device (for the GPU library), so both sides see bit-identical inputs and the large tables never
cross PCIe.

The five full-size workloads follow the benchmark's configuration list; the paper's datasets
(One Billion Word, Criteo, IWSLT'14, RedPajama; section "Experimental Setup") are not available, so
only shapes, densities (Table "model statistics": 1.1-2.8 % for embedding gradients; top-5 % for
DGC) and skew (section "Characteristics of sparse tensors", C3: most non-zeros sit in the first of
eight even partitions) are reproduced.  Zipf rank k maps to row k-1 with no shuffling, which piles
the non-zero rows at low row ids exactly as C3 describes.
"""
from dataclasses import dataclass, replace
from functools import lru_cache

import numpy as np

_BASE_SEED = 20230913


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int          # 1..5 = benchmark configuration number
    n_rows: int             # R
    row_dim: int            # D (1 = element-level sparsity)
    n_workers: int          # n simulated workers = n partitions = n servers
    hash_seed: int
    kind: str               # "uniform" | "zipf" | "runs"
    bitmap: bool = False    # hash-bitmap index encoding
    # kind == "uniform": exactly nnz distinct positions, values N(0, sigma)
    nnz: int = 0
    # kind == "zipf": n_tokens ids drawn iid from finite Zipf(s) over [0, R)
    n_tokens: int = 0
    zipf_s: float = 1.0
    # kind == "runs": n_runs runs of run_len consecutive non-zeros
    n_runs: int = 0
    run_len: int = 0
    sigma: float = 1.0

    @property
    def n_parts(self):
        return self.n_workers

    @property
    def dense_bytes(self):
        return 4 * self.n_rows * self.row_dim


WORKLOADS = {
    1: Workload("cfg1_tiny_uniform", 1, 1 << 20, 1, 4, 0x9E3779B1, "uniform", nnz=10486, sigma=1.0),
    2: Workload("cfg2_lm_embedding", 2, 32000, 1024, 8, 0x85EBCA77, "zipf", n_tokens=8 * 512, zipf_s=1.1,
                sigma=0.01),
    3: Workload("cfg3_recsys_embedding", 3, 10_000_000, 64, 16, 0xC2B2AE3D, "zipf", n_tokens=4096 * 26,
                zipf_s=1.05, sigma=0.01),
    4: Workload("cfg4_large_vocab_lm", 4, 256000, 4096, 32, 0x27D4EB2F, "zipf", n_tokens=16 * 2048,
                zipf_s=1.2, sigma=0.01),
    5: Workload("cfg5_clustered_runs", 5, 1 << 28, 1, 64, 0x165667B1, "runs", bitmap=True, n_runs=3277,
                run_len=4096, sigma=1.0),
}

# Scaled-down versions the CPU oracle finishes in seconds; they keep the structure (kind, skew,
# density class, n) and still span several kernel tiles with a ragged tail.
MINI_WORKLOADS = {
    1: replace(WORKLOADS[1], name="mini1", n_rows=100_003, nnz=1049),
    2: replace(WORKLOADS[2], name="mini2", n_rows=2003, row_dim=1024, n_tokens=300),
    3: replace(WORKLOADS[3], name="mini3", n_rows=300_007, row_dim=64, n_tokens=6000),
    4: replace(WORKLOADS[4], name="mini4", n_rows=1001, row_dim=4096, n_tokens=200, n_workers=32),
    5: replace(WORKLOADS[5], name="mini5", n_rows=(1 << 20) + 77, n_runs=51, run_len=1024, n_workers=64),
}


def get_workload(config_id, mini=False):
    return (MINI_WORKLOADS if mini else WORKLOADS)[int(config_id)]


@lru_cache(maxsize=4)
def zipf_cdf(n_rows, s):
    """CDF of the finite Zipf law P(k) ~ k^-s, k = 1..R (fp64)."""
    w = np.arange(1, n_rows + 1, dtype=np.float64) ** (-float(s))
    c = np.cumsum(w)
    c /= c[-1]
    return c


def _rng(wl, worker):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([_BASE_SEED, wl.config_id, int(worker)])))


def _normal_nonzero(rng, shape, sigma):
    """N(0, sigma) fp32 draws; exact zeros (and draws that round to +-0) are re-drawn."""
    v = (rng.standard_normal(shape, dtype=np.float32) * np.float32(sigma)).astype(np.float32)
    while True:
        z = v == 0
        k = int(z.sum())
        if k == 0:
            return v
        v[z] = (rng.standard_normal(k, dtype=np.float32) * np.float32(sigma)).astype(np.float32)


def _rows_uniform(wl, rng):
    return np.sort(rng.choice(wl.n_rows, size=wl.nnz, replace=False)).astype(np.uint32)


def _rows_zipf(wl, rng):
    cdf = zipf_cdf(wl.n_rows, wl.zipf_s)
    u = rng.random(wl.n_tokens)
    ids = np.searchsorted(cdf, u, side="left")
    ids = np.minimum(ids, wl.n_rows - 1)
    return np.unique(ids).astype(np.uint32)


def _rows_runs(wl, rng):
    n_slots = wl.n_rows // wl.run_len - 1          # last slot left free for the offset
    slots = np.sort(rng.choice(n_slots, size=wl.n_runs, replace=False)).astype(np.int64)
    off = int(rng.integers(0, wl.run_len))
    starts = slots * wl.run_len + off
    rows = (starts[:, None] + np.arange(wl.run_len, dtype=np.int64)[None, :]).reshape(-1)
    return rows.astype(np.uint32)


def worker_sparse(wl, worker, want_values=True):
    """Sparse form of worker `worker`'s gradient: (rows u32 ascending unique, values f32 [nnz, D]).

    Every returned row has at least one non-zero element (for D == 1 every value is non-zero), so
    the number of non-zero rows of the dense tensor equals len(rows) exactly.
    """
    rng = _rng(wl, worker)
    if wl.kind == "uniform":
        rows = _rows_uniform(wl, rng)
    elif wl.kind == "zipf":
        rows = _rows_zipf(wl, rng)
    elif wl.kind == "runs":
        rows = _rows_runs(wl, rng)
    else:
        raise ValueError(wl.kind)
    if not want_values:
        return rows, None
    vals = _normal_nonzero(rng, (rows.size, wl.row_dim), wl.sigma)
    if wl.row_dim > 1:
        # a row of D draws is all-zero with probability 0, but make it certain
        dead = ~np.any(vals != 0, axis=1)
        assert not dead.any()
    return rows, vals


def dense_from_sparse(wl, rows, vals):
    """Host dense fp32 [R, D] tensor holding `vals` at `rows`, zero elsewhere."""
    g = np.zeros((wl.n_rows, wl.row_dim), np.float32)
    g[rows.astype(np.int64)] = vals
    return g
