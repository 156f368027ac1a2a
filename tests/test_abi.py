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
    for must in ("zen_encode", "zen_aggregate", "zen_encode_batch", "zen_aggregate_batch", "zen_ctx_create"):
        assert must in names


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
