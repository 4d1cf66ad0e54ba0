"""GPU parity of the shared-list scan of qadc_ivf_search (large batches: every inverted list is scanned
once for all the queries that probe it) against the CPU oracle and against the per-query scan."""

import numpy as np
import pytest

from gpu_common import to_gpu, idx_np
from test_gpu_ivf import build_ivf, gpu_index

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def Q():
    import torch
    assert torch.cuda.is_available()
    import paper_1704_07355_amd as Q
    Q.lib()
    return Q


@pytest.fixture(scope="module")
def O():
    from oracle import qadc_oracle as O
    return O


def both_routes(Q, monkeypatch, gix, gq, nprobe, R, init, **kw):
    """The search by the shared-list scan and by the per-query scan (the knob is read at every call)."""
    import torch
    monkeypatch.setenv("QADC_IVF_SHARED", "1")
    a = Q.qadc_ivf_search(gix, gq, nprobe, R, init, debug=True, **kw)
    monkeypatch.setenv("QADC_IVF_SHARED", "0")
    b = Q.qadc_ivf_search(gix, gq, nprobe, R, init, debug=True, **kw)
    torch.cuda.synchronize()
    monkeypatch.delenv("QADC_IVF_SHARED")
    return a, b


@pytest.mark.parametrize("m", [8, 16, 32, 64])
@pytest.mark.parametrize("nq,nprobe,R", [(300, 8, 100), (70, 20, 10), (1, 3, 5)])
def test_shared_scan_matches_oracle_and_per_query_scan(Q, O, monkeypatch, m, nq, nprobe, R):
    coarse, cb, x, index = build_ivf(O, n=60_000, K=48, d=64, m=m, seed=100 + m)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(nq)
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    init = 300
    (ids, dist, probes, qluts), (ids2, dist2, _, _) = both_routes(Q, monkeypatch, gix, to_gpu(queries), nprobe, R, init)
    assert np.array_equal(idx_np(ids), idx_np(ids2))
    assert np.array_equal(dist.cpu().numpy(), dist2.cpu().numpy())
    for iq in range(0, nq, max(1, nq // 12)):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_shared_scan_over_long_lists_and_ragged_chunks(Q, O, monkeypatch):
    """Lists far longer than a work item's chunk (several chunks per part, ragged ends), R = 128, and
    cells probed by more pairs than one wavefront takes."""
    coarse, cb, x, index = build_ivf(O, n=400_000, K=6, d=32, m=16, seed=9, zipf=True)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(1)
    nq, nprobe, R, init = 200, 4, 128, 1000
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    (ids, dist, probes, qluts), (ids2, dist2, _, _) = both_routes(Q, monkeypatch, gix, to_gpu(queries), nprobe, R, init)
    assert np.array_equal(idx_np(ids), idx_np(ids2))
    assert np.array_equal(dist.cpu().numpy(), dist2.cpu().numpy())
    for iq in range(0, nq, 40):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_queries_whose_region_overflows_are_redone(Q, O, monkeypatch):
    """A database of identical codes: every sum of a list is the same, so every code passes any bound and
    a query's report region overflows; such queries are redone by the per-query scan.  Mixed in one batch
    with cells of ordinary codes."""
    coarse, cb, x, index = build_ivf(O, n=120_000, K=10, d=32, m=8, seed=5, zipf=False)
    codes = index["codes"].copy()
    off = index["list_off"]
    codes[off[0]:off[2]] = codes[0]          # cells 0 and 1: one code repeated
    ix2 = dict(list_off=off, codes=codes, ids=index["ids"])
    gix = gpu_index(Q, coarse, cb, ix2)
    rng = np.random.default_rng(3)
    nq, nprobe, R, init = 64, 3, 20, 200
    queries = (coarse[rng.integers(0, 10, size=nq)] + rng.normal(scale=10, size=(nq, 32))).astype(np.float32)
    (ids, dist, probes, qluts), (ids2, dist2, _, _) = both_routes(Q, monkeypatch, gix, to_gpu(queries), nprobe, R, init)
    pr = probes.cpu().numpy()
    assert (pr < 2).any(axis=1).sum() > 10 and (pr >= 2).all(axis=1).sum() > 5
    assert np.array_equal(idx_np(ids), idx_np(ids2))
    assert np.array_equal(dist.cpu().numpy(), dist2.cpu().numpy())
    for iq in range(0, nq, 5):
        rep = O.ivf_quick_adc_search(ix2, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=pr[iq], qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_shared_scan_with_given_probes_empty_lists_and_repeats(Q, O, monkeypatch):
    coarse, cb, x, index = build_ivf(O, n=50_000, K=30, d=64, m=16, seed=12)
    K = len(coarse)
    off = index["list_off"].copy()
    for c in (2, 9):
        off[c + 1] = off[c]
    for c in range(K):
        off[c + 1] = max(off[c + 1], off[c])
    off[K] = index["list_off"][K]
    ix2 = dict(list_off=off, codes=index["codes"], ids=index["ids"])
    gix = gpu_index(Q, coarse, cb, ix2)
    rng = np.random.default_rng(2)
    nq, nprobe, R, init = 90, 6, 40, 150
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    probes = rng.integers(0, K, size=(nq, nprobe)).astype(np.int32)
    probes[::4, 1] = -1
    probes[::5, 3] = K + 1
    probes[7] = [2, 9, -1, 2, 9, -1]     # only empty lists
    (ids, dist, pr, qluts), (ids2, dist2, _, _) = both_routes(Q, monkeypatch, gix, to_gpu(queries), nprobe, R, init,
                                                              probes_in=to_gpu(probes))
    assert np.array_equal(idx_np(ids), idx_np(ids2))
    assert np.array_equal(dist.cpu().numpy(), dist2.cpu().numpy())
    assert (idx_np(ids)[7] == 0xFFFFFFFF).all()
    pr = pr.cpu().numpy()
    for iq in range(0, nq, 9):
        mask = pr[iq] >= 0
        rep = O.ivf_quick_adc_search(ix2, coarse, cb, queries[iq], int(mask.sum()), init, R,
                                     probes=pr[iq][mask], qluts=qluts[iq].cpu().numpy()[mask])
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_workspace_is_left_clean_between_routes(Q, O, monkeypatch):
    """One workspace used by calls of different shapes and routes in turn (the layout of the control blocks
    changes every time): each call finds what it needs cleared."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=60_000, K=48, d=64, m=16, seed=44)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(6)
    queries = (x[rng.integers(0, len(x), size=128)] + rng.normal(scale=6, size=(128, x.shape[1]))).astype(np.float32)
    gq = to_gpu(queries)
    monkeypatch.setenv("QADC_IVF_SHARED", "1")
    need = max(Q.qadc_ivf_workspace_bytes(gix, 128, 8, 100), Q.qadc_ivf_workspace_bytes(gix, 50, 12, 30))
    ws = Q.qadc_workspace_init(torch.empty((need,), dtype=torch.uint8, device="cuda"))
    ref = {}
    for route, nq, nprobe, R in [("1", 128, 8, 100), ("0", 50, 12, 30), ("1", 50, 12, 30), ("0", 128, 8, 100),
                                  ("1", 128, 8, 100)]:
        monkeypatch.setenv("QADC_IVF_SHARED", route)
        ids, dist = Q.qadc_ivf_search(gix, gq[:nq].contiguous(), nprobe, R, 300, workspace=ws)
        torch.cuda.synchronize()
        key = (nq, nprobe, R)
        got = (idx_np(ids).copy(), dist.cpu().numpy().copy())
        if key in ref:
            assert np.array_equal(got[0], ref[key][0]) and np.array_equal(got[1], ref[key][1]), (route, key)
        ref[key] = got
    monkeypatch.delenv("QADC_IVF_SHARED")


@pytest.mark.parametrize("min_pairs", [None, "2", "40"])
def test_cells_split_between_the_two_scans(Q, O, monkeypatch, min_pairs):
    """Many cells, Zipf-sized: some are probed by enough queries to be scanned once for all of them, the
    others stay with the per-query kernel; most queries have cells of both kinds and the two reports are
    joined.  (QADC_IVF_SHARED_MIN_PAIRS moves the line between the two.)"""
    coarse, cb, x, index = build_ivf(O, n=150_000, K=400, d=64, m=16, seed=77)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(8)
    nq, nprobe, R, init = 260, 12, 50, 400
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    if min_pairs is not None:
        monkeypatch.setenv("QADC_IVF_SHARED_MIN_PAIRS", min_pairs)
    (ids, dist, probes, qluts), (ids2, dist2, _, _) = both_routes(Q, monkeypatch, gix, to_gpu(queries), nprobe, R, init)
    pr = probes.cpu().numpy()
    per_cell = np.bincount(pr.ravel(), minlength=400)
    line = 8 if min_pairs is None else int(min_pairs)
    shared = per_cell[pr] >= line
    if line == 8:
        assert (shared.any(axis=1) & (~shared).any(axis=1)).sum() > nq // 2   # queries with cells of both kinds
    assert np.array_equal(idx_np(ids), idx_np(ids2))
    assert np.array_equal(dist.cpu().numpy(), dist2.cpu().numpy())
    for iq in range(0, nq, 20):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=pr[iq], qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


@pytest.mark.parametrize("m,nprobe,R", [(16, 64, 128), (64, 100, 30)])
def test_large_batch_takes_the_shared_route_by_itself(Q, O, m, nprobe, R):
    """700 queries (no knob set: calls of 384 queries and more share lists), most cells probed by most
    queries -- many sets of 32 pairs per cell -- with the largest R and nprobe beyond one table chunk of the
    seed kernel; against the oracle and against the same queries sent in calls of 100 (per-query scan)."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=100_000, K=100, d=64, m=m, seed=300 + m)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(17)
    nq, init = 700, 500
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    gq = to_gpu(queries)
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, gq, nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    for s in range(0, nq, 100):
        i2, d2 = Q.qadc_ivf_search(gix, gq[s:s + 100].contiguous(), nprobe, R, init)
        assert np.array_equal(idx_np(i2), idx_np(ids)[s:s + 100]), s
        assert np.array_equal(d2.cpu().numpy(), dist.cpu().numpy()[s:s + 100]), s
    for iq in range(0, nq, 140):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_calls_beyond_one_launch_sequence_and_tiny_indexes(Q, O):
    """4500 queries (more than one launch sequence takes) over a small index, and an index of a single cell:
    both equal the same queries sent in small calls."""
    import torch
    for K, n, nq, nprobe in ((40, 30_000, 4500, 6), (1, 5_000, 700, 1)):
        coarse, cb, x, index = build_ivf(O, n=n, K=K, d=32, m=8, seed=K + 1, zipf=K > 1)
        gix = gpu_index(Q, coarse, cb, index)
        rng = np.random.default_rng(K)
        queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, 32))).astype(np.float32)
        gq = to_gpu(queries)
        R, init = 20, 100
        ids, dist, probes, qluts = Q.qadc_ivf_search(gix, gq, nprobe, R, init, debug=True)
        torch.cuda.synchronize()
        for s in (0, nq // 2, nq - 100):
            i2, d2 = Q.qadc_ivf_search(gix, gq[s:s + 100].contiguous(), nprobe, R, init)
            assert np.array_equal(idx_np(i2), idx_np(ids)[s:s + 100]), (K, s)
            assert np.array_equal(d2.cpu().numpy(), dist.cpu().numpy()[s:s + 100]), (K, s)
        for iq in (0, nq // 2, nq - 1):
            rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                         probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
            assert np.array_equal(idx_np(ids)[iq], rep["ids"]), (K, iq)
            assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), (K, iq)
