"""Host-only checks of the C-ABI library: it loads, and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "zen.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zen_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = _declared()
    # the boundary's calls: context, workspace sizing, the encode and the aggregate (single and batched), the
    # overflow report and the status text
    for must in ("zen_ctx_create", "zen_ctx_destroy", "zen_workspace_bytes", "zen_encode", "zen_aggregate",
                 "zen_encode_batch", "zen_aggregate_batch", "zen_last_overflow", "zen_status_str",
                 "zen_status_fetch", "zen_encode_workspace_bytes", "zen_aggregate_workspace_bytes", "zen_bitmap_layout",
                 "zen_nonzero", "zen_encode_static", "zen_ctx_create_tuned", "zen_pull_encode", "zen_pull_decode",
                 "zen_pull_apply", "zen_encode_hashed", "zen_sparsity_count", "zen_scheme_times", "zen_topk_threshold",
                 "zen_format_count", "zen_format_bytes"):
        assert must in names, must


def test_library_reads_no_environment_variable():
    """What can be tuned at run time goes through zen_ctx_create_tuned, not through the environment."""
    csrc = os.path.join(ROOT, "paper_2309_13254_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        assert "getenv" not in open(os.path.join(csrc, f)).read(), f


def test_library_loads_and_exports_every_declared_symbol():
    import paper_2309_13254_amd as zen

    so = zen.library_path()
    if not os.path.exists(so):
        pytest.fail("HIP library not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(so)
    for name in _declared():
        assert hasattr(lib, name), name
    assert zen.zen_status_str(0) == "ok"
    assert zen.zen_status_str(2) == "capacity exceeded"


def test_binding_exposes_the_same_names():
    import paper_2309_13254_amd as zen

    for name in _declared():
        assert hasattr(zen, name), name
