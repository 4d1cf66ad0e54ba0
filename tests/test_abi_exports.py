"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SO = os.path.join(ROOT, "paper_1704_07355_amd", "libqadc.so")


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(qadc_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_north_star_calls():
    d = _declared()
    for name in ("qadc_build_luts", "qadc_quantize_luts", "qadc_scan_topk"):
        assert name in d


@pytest.mark.parametrize("name", _declared())
def test_symbol_exported(name):
    if not os.path.exists(SO):
        pytest.fail("libqadc.so missing: run __graft_entry__.build() first")
    lib = ctypes.CDLL(SO)
    assert hasattr(lib, name)


def test_binding_lists_every_export():
    import paper_1704_07355_amd as Q
    assert sorted(Q.EXPORTS) == _declared()
    for name in Q.EXPORTS:
        assert callable(getattr(Q, name))


def test_workspace_query_needs_no_gpu():
    import paper_1704_07355_amd as Q
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, 10_000_000, 16, 1, 100) > 0
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, 1000, 7, 1, 100) == 0  # odd m: rejected
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, 1000, 16, 1, 5000) == 0  # R too large
    assert Q.qadc_version().startswith("qadc")
