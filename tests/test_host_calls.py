"""The library's host-only entry points (no GPU work): the two communication-time formulas and the format sizes
against the oracle, and argument errors that are refused before anything touches a device."""
import ctypes as C

import numpy as np
import pytest


@pytest.fixture(scope="module")
def zen():
    import paper_2309_13254_amd as z

    z.load_library()
    return z


def test_scheme_times_match_the_oracle(oracle, zen):
    rng = np.random.default_rng(11)
    for n in (2, 8, 64, 512):
        stages = n.bit_length() - 1
        gam = np.sort(1.0 + rng.random(stages + 1) * n)
        gam[0] = 1.0
        d, M, b = float(rng.random() * 0.05 + 1e-3), 2.5e9, 25e9
        t_bp, t_sm = zen.zen_scheme_times(n, gam, d, M, b)
        assert t_bp == pytest.approx(oracle.time_balanced_parallelism(n, gam[stages], d, M, b), rel=1e-14)
        assert t_sm == pytest.approx(oracle.time_hierarchical_centralization(n, gam[:stages], d, M, b), rel=1e-14)
    # the two extreme cases of the comparison: no overlap (gamma^k = k), full overlap (gamma^k = 1)
    n, d, M, b = 16, 0.01, 1e9, 1e9
    t_bp, t_sm = zen.zen_scheme_times(n, [1, 2, 4, 8, 16], d, M, b)
    assert t_bp == pytest.approx((n - 1) / n * (n + 1) * 2 * M * d / b) and t_sm == pytest.approx((n - 1) * 2 * M * d / b)
    t_bp, t_sm = zen.zen_scheme_times(n, [1, 1, 1, 1, 1], d, M, b)
    assert t_bp == pytest.approx(2 * (n - 1) / n * 2 * M * d / b) and t_sm == pytest.approx(4 * 2 * M * d / b)


def test_format_bytes_match_the_oracle(oracle, zen):
    for G, nnz, n, blocks in ((214_000_000, 6_000_000, 16, 800_000), (1 << 20, 1, 4, 1), (1000, 1000, 16, 4)):
        got = zen.zen_format_bytes(G, nnz, n, blocks, 256)
        ref = oracle.format_bytes(G, nnz, n, blocks, 256)
        assert got == ref


def test_bad_arguments_are_refused_on_the_host(zen):
    L = zen.load_library()
    h = C.c_void_p()
    assert L.zen_ctx_create(C.byref(h), 0, 1, 4, 1, 0) == zen.ZEN_ERR_INVALID and not h.value            # no rows
    assert L.zen_ctx_create(C.byref(h), 10, 1, 2000, 1, 0) == zen.ZEN_ERR_INVALID                        # too many partitions
    assert L.zen_ctx_create(C.byref(h), 10, 1, 4, 1, 7) == zen.ZEN_ERR_INVALID                           # no such format
    assert L.zen_ctx_create(C.byref(h), 1 << 32, 1, 4, 1, 0) == zen.ZEN_ERR_INVALID                      # ids beyond 32 bits
    tun = zen.binding._Tuning(17, 0)
    assert L.zen_ctx_create_tuned(C.byref(h), 10, 1, 4, 1, 0, C.byref(tun)) == zen.ZEN_ERR_INVALID       # tile size out of range
    tun = zen.binding._Tuning(0, 5)
    assert L.zen_ctx_create_tuned(C.byref(h), 10, 1, 4, 1, 0, C.byref(tun)) == zen.ZEN_ERR_INVALID
    b = C.c_uint64()
    assert L.zen_workspace_bytes(None, 10, 1, C.byref(b), C.byref(b)) == zen.ZEN_ERR_INVALID
    assert L.zen_last_overflow(None, C.byref(b)) == zen.ZEN_ERR_INVALID
    assert L.zen_encode_static(None, None, 4, 1, None, None, None) == zen.ZEN_ERR_INVALID
    assert L.zen_calibration_read(None, 16, None, None, None) == zen.ZEN_ERR_INVALID
    with pytest.raises(zen.ZenError):
        zen.zen_scheme_times(6, [1.0, 2.0, 3.0], 0.1, 1.0, 1.0)                                           # n not a power of two
    assert [zen.zen_status_str(s) for s in range(5)] == ["ok", "invalid argument", "capacity exceeded",
                                                         "out of memory / workspace too small", "HIP call failed"]


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU's share; asked for more it says so and exits without touching a GPU."""
    import os
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)
