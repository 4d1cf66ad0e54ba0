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


def test_batch_plans_fit_one_launch(monkeypatch):
    """Host-side planning of the batched scans: a batch's lists stay within the 256 MiB that one
    launch may take (plus the per-query control blocks), small batches get more and shorter chunks
    (a larger share per query), and the kernel choice changes the size, never the validity."""
    import paper_1704_07355_amd as Q
    n, m, R = 100_000_000, 32, 100
    full = Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, n, m, 256, R)
    small = Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, n, m, 32, R)
    assert 0 < full <= (256 << 20) + (1 << 20)
    assert 0 < small < full and small / 32 > full / 256
    monkeypatch.setenv("QADC_TILED_MFMA", "0")
    other = Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, n, m, 32, R)
    assert 0 < other < small
    monkeypatch.delenv("QADC_TILED_MFMA")
    # ten thousand queries in one call are cut into launches: the workspace does not grow with them
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, n, m, 10_000, R) <= (256 << 20) + (4 << 20)


def test_multi_index_workspace_query():
    import paper_1704_07355_amd as Q
    a = Q.qadc_multi_index_workspace_bytes(256, 256, 64)
    assert a >= 256 * 2 * 256 * 4 + 256 * 2 * 64 * 4
    assert Q.qadc_multi_index_workspace_bytes(256, 512, 64) > a
    for bad in ((0, 1, 1), (16385, 1, 1), (16, 0, 1), (16, 1, 0), (16, 1, 257), (16, 70000, 4)):
        assert Q.qadc_multi_index_workspace_bytes(*bad) == 0


def test_multi_index_argument_checks_need_no_gpu():
    """Arguments are checked on the host before anything is launched."""
    import paper_1704_07355_amd as Q
    L = Q.lib()
    assert L.qadc_multi_index_cells(None, 4, 8, None, None) == Q.QADC_EINVAL          # null pointers
    assert L.qadc_multi_index_cells(None, 0, 8, None, None) == Q.QADC_EINVAL          # K < 1
    assert L.qadc_multi_index_cells(None, 4, 7, None, None) == Q.QADC_EINVAL          # odd d
    assert L.qadc_multi_index_assign(None, 4, 8, None, 10, None, None) == Q.QADC_EINVAL
    assert L.qadc_multi_index_assign(None, 4, 8, None, 0, None, None) == Q.QADC_OK    # nothing to do
    assert L.qadc_multi_index_probes(None, 4, 8, None, 0, 4, None, None, 0, None) == Q.QADC_OK
    assert L.qadc_multi_index_probes(None, 4, 8, None, 3, 4, None, None, 0, None) == Q.QADC_EINVAL
    assert b"qadc_multi_index_probes" in L.qadc_last_error()


def test_occupied_cell_entry_points_check_arguments_on_the_host():
    import paper_1704_07355_amd as Q
    L = Q.lib()
    assert Q.qadc_multi_index_group_workspace_bytes(1000, 16384) > 1000 * 4
    assert Q.qadc_multi_index_group_workspace_bytes(1000, 16385) == 0
    assert L.qadc_multi_index_group(None, 10, 8, 5, None, None, None, None, None, 0, None) == Q.QADC_EINVAL   # capacity
    assert b"max_lists" in L.qadc_last_error()
    assert L.qadc_multi_index_group(None, 10, 8, 10, None, None, None, None, None, 0, None) == Q.QADC_EINVAL  # null
    assert L.qadc_multi_index_slots(None, 0, None, 0, None, None) == Q.QADC_OK                                 # nothing to do
    assert L.qadc_multi_index_slots(None, 4, None, 3, None, None) == Q.QADC_EINVAL
    assert L.qadc_multi_index_encode(None, 0, None, 8, 4, None, 0, None, None, 0, None, None) == Q.QADC_EINVAL  # K < 1
    assert L.qadc_multi_index_encode(None, 4, None, 7, 4, None, 0, None, None, 0, None, None) == Q.QADC_EINVAL  # odd d
