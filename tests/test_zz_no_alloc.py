"""qadc_search_static (no allocation, static device scratch) against qadc_search, through the C ABI."""

import ctypes

import numpy as np
import pytest

from gpu_common import config1, to_gpu

pytestmark = pytest.mark.gpu


def _call_both(Q, L, torch, cb, queries, codes, R, init):
    nq, d = queries.shape
    m = cb.shape[0]
    n = codes.shape[0]
    dev = queries.device
    vp = ctypes.c_void_p
    stream = vp(torch.cuda.current_stream().cuda_stream)
    need = L.qadc_workspace_bytes(Q.QADC_WS_SEARCH, n, m, nq, R)
    ws = torch.zeros((max(need, 256),), dtype=torch.uint8, device=dev)
    out = [torch.full((nq, R), -7, dtype=torch.int32, device=dev) for _ in range(2)]
    dist = [torch.full((nq, R), 9, dtype=torch.uint8, device=dev) for _ in range(2)]
    ql = [torch.zeros((nq, m, 16), dtype=torch.uint8, device=dev) for _ in range(2)]
    rc = L.qadc_search(vp(cb.data_ptr()), d, m, vp(queries.data_ptr()), nq, vp(codes.data_ptr()), n, R, init,
                       255, 0, vp(out[0].data_ptr()), vp(dist[0].data_ptr()), vp(ql[0].data_ptr()),
                       vp(ws.data_ptr()), ws.numel(), stream)
    assert rc == 0, L.qadc_last_error()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = L.qadc_search_static(vp(cb.data_ptr()), d, m, vp(queries.data_ptr()), nq, vp(codes.data_ptr()), n, R,
                              init, 255, 0, vp(out[1].data_ptr()), vp(dist[1].data_ptr()), vp(ql[1].data_ptr()),
                              stream)
    assert rc == 0, L.qadc_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(ql[0], ql[1])
    assert torch.equal(out[0], out[1]) and torch.equal(dist[0], dist[1])
    return out[1], dist[1], ql[1]


def test_static_scratch_search_equals_workspace_search():
    import torch
    import paper_1704_07355_amd as Q
    from oracle import qadc_oracle as O
    L = Q.lib()
    assert L.qadc_static_scratch_bytes() == 32 << 20
    c = config1()
    cb, queries = to_gpu(c["codebooks"]), to_gpu(c["queries"])
    # a database long enough for the sampled bound and the barrier-free pass (tiled 4x)
    big = to_gpu(np.tile(c["codes"], (4, 1)))
    R, init = 100, 200
    # first call: one query over the long database; second call: smaller input (fewer codes, three
    # queries) on the same scratch, which the first call must have left clean
    i1, d1, q1 = _call_both(Q, L, torch, cb, queries[:1].contiguous(), big, R, init)
    small = big[:30_001].contiguous()
    i2, d2, q2 = _call_both(Q, L, torch, cb, queries[:3].contiguous(), small, R, init)
    # third call: a larger shape again (a batch over the long database): the array is laid out anew and
    # table data of the calls before must not be taken for control words
    i3, d3, q3 = _call_both(Q, L, torch, cb, queries[:16].contiguous(), big, R, init)
    # and against the oracle on the library's own tables (bit-exact)
    for (idx, dist, ql, codes_np, nq) in ((i1, d1, q1, np.tile(c["codes"], (4, 1)), 1),
                                          (i2, d2, q2, np.tile(c["codes"], (4, 1))[:30_001], 3),
                                          (i3, d3, q3, np.tile(c["codes"], (4, 1)), 16)):
        for iq in range(nq):
            wi, wd = O.top_r(O.scan_saturating(ql[iq].cpu().numpy(), codes_np), R, pad_dist=255)
            assert np.array_equal(idx[iq].cpu().numpy().view(np.uint32), wi)
            assert np.array_equal(dist[iq].cpu().numpy(), wd)


def test_static_scratch_rejects_sizes_beyond_the_array(monkeypatch):
    import paper_1704_07355_amd as Q
    L = Q.lib()
    # a launch shape whose per-query report regions exceed the array (8192 workgroups x 1024 keys x 8
    # bytes): refused before anything is enqueued or dereferenced
    monkeypatch.setenv("QADC_SCAN_WGS", "8192")
    n, m, R = 10_000_000, 16, 1024
    assert L.qadc_workspace_bytes(Q.QADC_WS_SEARCH, n, m, 1, R) > L.qadc_static_scratch_bytes()
    rc = L.qadc_search_static(None, 128, m, None, 1, None, n, R, 200, 255, 0, None, None, None, None)
    assert rc == Q.QADC_ENOMEM
    assert b"static" in L.qadc_last_error()
