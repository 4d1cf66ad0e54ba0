"""GPU parity of qadc_ivf_search against the CPU oracle's non-exhaustive search."""

import numpy as np
import pytest

from gpu_common import to_gpu, idx_np

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


def build_ivf(O, n=60_000, K=48, d=64, m=16, seed=0, zipf=True):
    """Small inverted index with Zipf-skewed lists: vectors around K seeded centres, residual codes."""
    from oracle import cref
    from workloads import zipf_list_sizes
    rng = np.random.default_rng(seed)
    coarse = rng.uniform(0, 255, size=(K, d)).astype(np.float32)
    sizes = zipf_list_sizes(n, K, 0.8, seed) if zipf else np.full(K, n // K)
    cell = np.repeat(np.arange(K), sizes)
    rng.shuffle(cell)
    x = (coarse[cell] + rng.normal(scale=18, size=(len(cell), d))).astype(np.float32)
    dsub = d // m
    resid_sample = (x[:4000] - coarse[cell[:4000]]).astype(np.float32)
    rows = rng.permutation(4000)[:16]
    cb = np.stack([O.kmeans_lloyd(resid_sample[:, j * dsub:(j + 1) * dsub], rows, 3)[0] for j in range(m)])
    # assign + encode residuals with the plain-C twin (same steps as O.ivf_build)
    assign = O.ivf_assign(x, coarse)
    order = np.argsort(assign, kind="stable")
    resid = (x[order] - coarse[assign[order]]).astype(np.float32)
    codes = cref.pq_encode(resid, cb)
    list_off = np.zeros(K + 1, dtype=np.int64)
    np.cumsum(np.bincount(assign, minlength=K), out=list_off[1:])
    index = dict(list_off=list_off, codes=codes, ids=order.astype(np.uint32))
    return coarse, cb, x, index


def gpu_index(Q, coarse, cb, index):
    return Q.IvfIndex(to_gpu(coarse), to_gpu(index["list_off"]), to_gpu(index["codes"]),
                      to_gpu(index["ids"].view(np.int32)), to_gpu(cb))


@pytest.mark.parametrize("m", [16, 32])
@pytest.mark.parametrize("mode", [0, 1])
def test_ivf_search_matches_oracle(Q, O, m, mode):
    import torch
    coarse, cb, x, index = build_ivf(O, m=m, seed=m)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(5)
    queries = (x[rng.integers(0, len(x), size=12)] + rng.normal(scale=6, size=(12, x.shape[1]))).astype(np.float32)
    nprobe, R, init = 8, 100, 300
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, 255, mode, debug=True)
    torch.cuda.synchronize()
    ids, dist, probes, qluts = idx_np(ids), dist.cpu().numpy(), probes.cpu().numpy(), qluts.cpu().numpy()
    for iq in range(len(queries)):
        full = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R, 255, mode)
        # Index step: same cells in the same order (float32 vs float64 distances: allow a swap of
        # cells whose distances agree to 1e-5)
        dq = O.sq_l2(queries[iq][None], coarse)[0]
        if not np.array_equal(probes[iq], full["probes"]):
            np.testing.assert_allclose(dq[probes[iq]], dq[full["probes"]], rtol=1e-5)
        # Tables + quantizer: entries within one step of the oracle's
        if np.array_equal(probes[iq], full["probes"]):
            assert np.abs(qluts[iq].astype(int) - full["qluts"].astype(int)).max() <= 1
        # integer part replayed by the oracle on the GPU's own cells and tables: bit-exact
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R, 255, mode,
                                     probes=probes[iq], qluts=qluts[iq])
        assert np.array_equal(ids[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq], rep["dist"]), iq


def test_ivf_search_given_probes_and_edge_lists(Q, O):
    """Cells given by the caller, including empty lists, an unused slot and a single huge list."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=40_000, K=20, seed=3)
    # empty two lists by moving their boundaries: rebuild offsets with zero-size cells
    gix = gpu_index(Q, coarse, cb, index)
    sizes = np.diff(index["list_off"])
    big = int(np.argmax(sizes))
    small = int(np.argmin(sizes))
    probes_in = np.array([[big, small, 3, -1], [small, 5, big, 7], [big, -1, -1, -1]], dtype=np.int32)
    queries = x[[10, 2000, 30000]] + 1.5
    R, init = 150, 200
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries.astype(np.float32)), 4, R, init,
                                                 probes_in=to_gpu(probes_in), debug=True)
    torch.cuda.synchronize()
    assert np.array_equal(probes.cpu().numpy(), probes_in)
    for iq in range(3):
        cells = probes_in[iq][probes_in[iq] >= 0]
        ql = qluts[iq].cpu().numpy()[:len(cells)]
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq].astype(np.float32), len(cells), init, R,
                                     probes=cells, qluts=ql)
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]) and np.array_equal(dist[iq].cpu().numpy(), rep["dist"])
        # and the GPU's tables are the oracle's within one step
        full = O.ivf_quick_adc_search(index, coarse, cb, queries[iq].astype(np.float32), len(cells), init, R,
                                      probes=cells)
        assert np.abs(ql.astype(int) - full["qluts"].astype(int)).max() <= 1


def test_ivf_all_cells_equals_flat_scan_of_the_lists(Q, O):
    """nprobe = K: every stored code is scanned exactly once, with its own cell's tables."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=30_000, K=9, seed=9)
    gix = gpu_index(Q, coarse, cb, index)
    y = x[123:124].copy()
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(y), 9, 100, 500, debug=True)
    torch.cuda.synchronize()
    probes, qluts = probes.cpu().numpy()[0], qluts.cpu().numpy()[0]
    assert sorted(probes.tolist()) == list(range(9))
    sums = np.empty(len(x), dtype=np.uint8)
    for t, p in enumerate(probes):
        lo, hi = index["list_off"][p], index["list_off"][p + 1]
        sums[lo:hi] = O.scan_saturating(qluts[t], index["codes"][lo:hi])
    pos, d = O.top_r(sums, 100, pad_dist=255)
    assert np.array_equal(idx_np(ids)[0], index["ids"][pos]) and np.array_equal(dist[0].cpu().numpy(), d)
    assert 123 in idx_np(ids)[0]


@pytest.mark.parametrize("seed_kernel", ["1", "0"])
def test_ivf_scan_with_and_without_the_sampled_bound(Q, O, seed_kernel, monkeypatch):
    """The sampled bound only prunes: with it (barrier-free pass) and without it (careful pass)
    the result is the oracle's.  Larger lists, so that workgroups walk several tiles."""
    import torch
    monkeypatch.setenv("QADC_IVF_SEED", seed_kernel)
    coarse, cb, x, index = build_ivf(O, n=400_000, K=12, m=32, seed=21)
    gix = gpu_index(Q, coarse, cb, index)
    queries = (x[[7, 90_000, 399_999]] + 2.0).astype(np.float32)
    nprobe, R, init = 6, 100, 1000
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    for iq in range(len(queries)):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_ivf_bound_without_resolution_falls_back(Q, O):
    """Every stored code identical: all sums tie, the sampled bound lets everything through, the
    barrier-free list overflows and the careful pass decides by storage position."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=120_000, K=6, m=16, seed=4)
    index = dict(index)
    index["codes"] = np.full_like(index["codes"], 0x21)
    gix = gpu_index(Q, coarse, cb, index)
    queries = x[[5, 60_000]].astype(np.float32)
    nprobe, R, init = 3, 100, 200
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    for iq in range(len(queries)):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


def test_ivf_probe_selection_many_cells_with_exact_ties(Q, O):
    """Index step with more cells than selection threads and every centroid stored twice: equal
    distances are ordered by cell id, a pair cut by the nprobe boundary keeps its lower id."""
    import torch
    rng = np.random.default_rng(17)
    K, d, m, nprobe = 3000, 32, 8, 65
    coarse = rng.uniform(0, 255, size=(K, d)).astype(np.float32)
    coarse[K // 2:] = coarse[:K // 2]
    cb = rng.uniform(-20, 20, size=(m, 16, d // m)).astype(np.float32)
    list_off = np.arange(K + 1, dtype=np.int64) * 2
    codes = rng.integers(0, 256, size=(2 * K, m // 2), dtype=np.uint8)
    index = dict(list_off=list_off, codes=codes, ids=np.arange(2 * K, dtype=np.uint32))
    gix = gpu_index(Q, coarse, cb, index)
    queries = rng.uniform(0, 255, size=(5, d)).astype(np.float32)
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, 50, 100, debug=True)
    torch.cuda.synchronize()
    probes = probes.cpu().numpy()
    for iq in range(len(queries)):
        want = O.ivf_probes(queries[iq], coarse, nprobe)
        got = probes[iq]
        if not np.array_equal(got, want):
            dq = O.sq_l2(queries[iq][None], coarse)[0]
            np.testing.assert_allclose(dq[got], dq[want], rtol=1e-5)
        assert len(set(got.tolist())) == nprobe
        where = {int(c): i for i, c in enumerate(got)}
        for c, i in where.items():
            if c >= K // 2:   # the twin with the lower id comes right before
                assert where.get(c - K // 2) == i - 1, (iq, c)


@pytest.mark.parametrize("K,d", [(331, 64), (48, 40)])
def test_ivf_index_step_of_large_batches_equals_small_batches(Q, O, K, d):
    """Batches of 64 queries and more take the tiled distance kernel: same cells, same order, as the
    same queries sent a few at a time (both sum the float32 differences in increasing component
    order), and the oracle's cells up to float32 ties.  K odd, d not a multiple of 16, a ragged batch."""
    import torch
    m = 8
    coarse, cb, x, index = build_ivf(O, n=20_000, K=K, d=d, m=m, seed=K)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(K)
    nq = 203
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, d))).astype(np.float32)
    nprobe, R, init = 7, 20, 100
    gq = to_gpu(queries)
    ids, dist, probes, _ = Q.qadc_ivf_search(gix, gq, nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    probes = probes.cpu().numpy()
    for s in range(0, nq, 29):
        i2, d2, p2, _ = Q.qadc_ivf_search(gix, gq[s:s + 29].contiguous(), nprobe, R, init, debug=True)
        assert np.array_equal(p2.cpu().numpy(), probes[s:s + 29])
        assert np.array_equal(idx_np(i2), idx_np(ids)[s:s + 29])
        assert np.array_equal(d2.cpu().numpy(), dist.cpu().numpy()[s:s + 29])
    for iq in range(0, nq, 17):
        want = O.ivf_probes(queries[iq], coarse, nprobe)
        if not np.array_equal(probes[iq], want):
            dq = O.sq_l2(queries[iq][None], coarse)[0]
            np.testing.assert_allclose(dq[probes[iq]], dq[want], rtol=1e-5)


def test_ivf_large_batch_with_empty_and_huge_lists(Q, O):
    """1500 queries in one call (more than one pass of the workgroup-map kernel's ranking and running
    sums), cells given by the caller: empty lists, unused slots, one list holding most codes.  Same
    results as the same queries sent 50 at a time (a workgroup per unit there), and the oracle's
    replay for a sample."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=60_000, K=24, d=32, m=8, seed=77, zipf=True)
    K = len(coarse)
    # empty three lists by giving their codes to the neighbour list (offsets only move)
    off = index["list_off"].copy()
    for c in (3, 4, 17):
        off[c + 1] = off[c]
    off[K] = index["list_off"][K]
    for c in range(K):
        off[c + 1] = max(off[c + 1], off[c])
    ix2 = dict(list_off=off, codes=index["codes"], ids=index["ids"])
    gix = gpu_index(Q, coarse, cb, ix2)
    rng = np.random.default_rng(7)
    nq, nprobe, R, init = 1500, 5, 30, 120
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    probes = rng.integers(0, K, size=(nq, nprobe)).astype(np.int32)
    probes[::9, 2] = -1            # unused slots
    probes[::13, 4] = K + 3        # a cell that does not exist: an unused slot too
    probes[5] = [3, 4, 17, -1, -1]  # only empty lists
    gq, gp = to_gpu(queries), to_gpu(probes)
    ids, dist, pr, ql = Q.qadc_ivf_search(gix, gq, nprobe, R, init, probes_in=gp, debug=True)
    torch.cuda.synchronize()
    # the draw repeats cells inside many rows: the library scans a list once (first slot wins)
    clean = probes.copy()
    clean[(clean < 0) | (clean >= K)] = -1
    for row in clean:
        for t in range(1, nprobe):
            if row[t] >= 0 and row[t] in row[:t]:
                row[t] = -1
    assert (clean != probes).sum() > 200
    assert np.array_equal(pr.cpu().numpy(), clean)
    probes = clean
    assert (idx_np(ids)[5] == 0xFFFFFFFF).all()
    for s in range(0, nq, 50):
        i2, d2, _, _ = Q.qadc_ivf_search(gix, gq[s:s + 50].contiguous(), nprobe, R, init,
                                         probes_in=gp[s:s + 50].contiguous(), debug=True)
        assert np.array_equal(idx_np(i2), idx_np(ids)[s:s + 50]), s
        assert np.array_equal(d2.cpu().numpy(), dist.cpu().numpy()[s:s + 50]), s
    for iq in range(0, nq, 97):
        mask = probes[iq] >= 0
        rep = O.ivf_quick_adc_search(ix2, coarse, cb, queries[iq], int(mask.sum()), init, R,
                                     probes=probes[iq][mask], qluts=ql[iq].cpu().numpy()[mask])
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


@pytest.mark.parametrize("nprobe,nq", [(40, 3), (17, 1), (64, 15), (9, 2)])
def test_ivf_bound_sampled_by_several_workgroups(Q, O, nprobe, nq):
    """Fewer than 16 queries with more than 8 probed cells: a query's lists are sampled by several
    workgroups that add their histograms in the control block.  The result is the oracle's, and the
    same as when the queries arrive in a batch of 16 (one sampling workgroup per query)."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=150_000, K=80, d=64, m=16, seed=31)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(nprobe)
    queries = (x[rng.integers(0, len(x), size=16)] + rng.normal(scale=6, size=(16, x.shape[1]))).astype(np.float32)
    R, init = 100, 500
    gq = to_gpu(queries)
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, gq[:nq].contiguous(), nprobe, R, init, debug=True)
    ids16, dist16, _, _ = Q.qadc_ivf_search(gix, gq, nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    assert np.array_equal(idx_np(ids), idx_np(ids16)[:nq])
    assert np.array_equal(dist.cpu().numpy(), dist16.cpu().numpy()[:nq])
    for iq in range(nq):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


@pytest.mark.parametrize("R", [600, 1000])
@pytest.mark.parametrize("nq", [3, 70])
def test_ivf_large_R_many_probes(Q, O, R, nq):
    """R above half the candidate list's slack, 32 probed cells: a workgroup's list grows past 512 keys
    while it still holds fewer than R (nothing to cut back yet), for a few queries (a workgroup per
    unit) and for a batch (a workgroup walks many units).  Oracle replay on the GPU's cells and tables."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=300_000, K=40, d=64, m=16, seed=R)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(R + nq)
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    nprobe, init = 32, 1000
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    ids, dist, probes, qluts = idx_np(ids), dist.cpu().numpy(), probes.cpu().numpy(), qluts.cpu().numpy()
    for iq in range(0, nq, max(1, nq // 10)):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq], qluts=qluts[iq])
        assert len(set(ids[iq].tolist())) == R, iq  # every slot written, no neighbour twice
        assert np.array_equal(ids[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq], rep["dist"]), iq


@pytest.mark.parametrize("m", [8, 16, 32, 64])
@pytest.mark.parametrize("wide_q,seed_kernel", [("64", "1"), ("0", "1"), ("64", "0")])
def test_ivf_few_queries_both_workgroup_shapes(Q, O, m, wide_q, seed_kernel, monkeypatch):
    """Calls of a few queries scan with workgroups of 1024 threads, larger calls with 256 (QADC_IVF_WIDE_Q
    moves the limit): both shapes, with the sampled bound and without it (the pass with a barrier per
    tile), give the oracle's result on lists long enough for a workgroup to walk several units."""
    import torch
    monkeypatch.setenv("QADC_IVF_WIDE_Q", wide_q)
    monkeypatch.setenv("QADC_IVF_SEED", seed_kernel)
    monkeypatch.setenv("QADC_IVF_WGS", "3")  # few workgroups per query: several units each
    coarse, cb, x, index = build_ivf(O, n=120_000, K=12, d=64, m=m, seed=100 + m)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(m)
    nq, nprobe, R, init = 5, 6, 100, 300
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, x.shape[1]))).astype(np.float32)
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    for iq in range(nq):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(ids)[iq], rep["ids"]), iq
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"]), iq


@pytest.mark.parametrize("mode", [0, 1])
def test_ivf_few_queries_path_equals_batch_path(Q, O, mode):
    """Calls of up to 32 queries take kernels of their own (centroids staged in one round with the
    minima of runs of 128 cells, Tables and the qmax walk in one launch, tables quantized where they
    are read); a call of 70 takes the batch kernels.  Same cells, tables and neighbours either way, and
    the oracle's on the cells and tables of the few-queries call.  d = 200 (two rounds of components),
    K = 1300 (eleven runs of cells, the last one ragged), and queries that are not 16-byte aligned."""
    import torch
    K, d, m = 1300, 200, 8
    coarse, cb, x, index = build_ivf(O, n=40_000, K=K, d=d, m=m, seed=77)
    gix = gpu_index(Q, coarse, cb, index)
    rng = np.random.default_rng(5)
    nq, nprobe, R, init = 70, 4, 50, 200
    queries = (x[rng.integers(0, len(x), size=nq)] + rng.normal(scale=6, size=(nq, d))).astype(np.float32)
    flat = torch.zeros(nq * d + 1, dtype=torch.float32, device="cuda:0")
    flat[1:] = to_gpu(queries).flatten()
    gq_odd = flat[1:].view(nq, d)  # rows start 4 bytes past a 16-byte boundary
    gq = to_gpu(queries)
    ids, dist, probes, qluts = Q.qadc_ivf_search(gix, gq, nprobe, R, init, qmin_mode=mode, debug=True)
    torch.cuda.synchronize()
    for s, src in ((0, gq), (7, gq), (33, gq_odd), (64, gq_odd)):
        n1 = 1 if s == 7 else 6
        i2, d2, p2, q2 = Q.qadc_ivf_search(gix, src[s:s + n1], nprobe, R, init, qmin_mode=mode, debug=True)
        torch.cuda.synchronize()
        assert np.array_equal(p2.cpu().numpy(), probes.cpu().numpy()[s:s + n1]), s
        assert np.array_equal(q2.cpu().numpy(), qluts.cpu().numpy()[s:s + n1]), s
        assert np.array_equal(idx_np(i2), idx_np(ids)[s:s + n1]), s
        assert np.array_equal(d2.cpu().numpy(), dist.cpu().numpy()[s:s + n1]), s
        for k in range(n1):
            rep = O.ivf_quick_adc_search(index, coarse, cb, queries[s + k], nprobe, init, R, qmin_mode=mode,
                                         probes=p2[k].cpu().numpy(), qluts=q2[k].cpu().numpy())
            assert np.array_equal(idx_np(i2)[k], rep["ids"]), (s, k)
            assert np.array_equal(d2[k].cpu().numpy(), rep["dist"]), (s, k)


@pytest.mark.parametrize("K", [300_000, 530_000])
def test_ivf_few_queries_many_cells(Q, O, K):
    """Hundreds of thousands of cells, most of them empty, a few queries: with 2344 runs of 128 cells the
    selection works from the runs' minima, with 4141 runs (more than fit its LDS list) it walks the
    whole row; either way the oracle's cells (up to float32 ties) and, on those cells and tables, its
    neighbours."""
    import torch
    d, m, n = 8, 8, 30_000
    rng = np.random.default_rng(K)
    coarse = rng.uniform(0, 255, size=(K, d)).astype(np.float32)
    cells = np.sort(rng.integers(0, K, size=n))
    list_off = np.zeros(K + 1, dtype=np.int64)
    np.cumsum(np.bincount(cells, minlength=K), out=list_off[1:])
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    ids = rng.permutation(n).astype(np.uint32)
    cb = rng.normal(scale=20, size=(m, 16, d // m)).astype(np.float32)
    index = dict(list_off=list_off, codes=codes, ids=ids)
    gix = gpu_index(Q, coarse, cb, index)
    nq, nprobe, R, init = 3, 200, 20, 50
    queries = rng.uniform(0, 255, size=(nq, d)).astype(np.float32)
    gi, gd, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    probes = probes.cpu().numpy()
    for iq in range(nq):
        want = O.ivf_probes(queries[iq], coarse, nprobe)
        if not np.array_equal(probes[iq], want):
            dq = O.sq_l2(queries[iq][None], coarse)[0]
            np.testing.assert_allclose(dq[probes[iq]], dq[want], rtol=1e-5)
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq], qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(gi)[iq], rep["ids"]), iq
        assert np.array_equal(gd[iq].cpu().numpy(), rep["dist"]), iq


@pytest.mark.parametrize("seed", [11, 12])
def test_ivf_random_shapes(Q, O, seed):
    """Seeded random indexes and calls: m, d, K, list skew, empty databases, 1 to 650 queries (the kernels
    of a few queries, of batches, and the shared-list route), nprobe up to 200, R up to 600, init from
    1 to 2000, both qmin modes.  Every query: the oracle's neighbours on the GPU's cells and tables, and
    tables within one step of the oracle's own."""
    import torch
    rng = np.random.default_rng(seed)
    for trial in range(20):
        m = int(rng.choice([8, 16, 32, 64]))
        dsub = int(rng.choice([1, 2, 3, 4]))
        d = m * dsub
        K = int(rng.choice([5, 40, 130, 700, 3000]))
        n = int(rng.choice([0, 50, 3000, 40000]))
        nq = int(rng.choice([1, 2, 5, 13, 20, 33, 70, 200, 650]))
        nprobe = int(min(K, rng.choice([1, 3, 8, 33, 64, 200])))
        R = int(rng.choice([1, 10, 100, 600]))
        init = int(rng.choice([1, 30, 300, 2000]))
        mode = int(rng.integers(0, 2))
        coarse = rng.uniform(0, 255, size=(K, d)).astype(np.float32)
        spread = K if rng.random() < 0.7 else max(1, K // 8)   # or: everything in the first eighth of the cells
        cells = np.sort(rng.integers(0, spread, size=n))
        list_off = np.zeros(K + 1, dtype=np.int64)
        np.cumsum(np.bincount(cells, minlength=K), out=list_off[1:])
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        ids = rng.permutation(n).astype(np.uint32)
        cb = rng.normal(scale=20, size=(m, 16, dsub)).astype(np.float32)
        index = dict(list_off=list_off, codes=codes, ids=ids)
        # (an empty database still needs allocations to point at)
        g_codes = to_gpu(codes) if n else torch.zeros((1, m // 2), dtype=torch.uint8, device="cuda:0")
        g_ids = to_gpu(ids.view(np.int32)) if n else torch.zeros((1,), dtype=torch.int32, device="cuda:0")
        gix = Q.IvfIndex(to_gpu(coarse), to_gpu(list_off), g_codes, g_ids, to_gpu(cb))
        gix.c.n = n
        queries = (coarse[rng.integers(0, K, size=nq)] + rng.normal(scale=10, size=(nq, d))).astype(np.float32)
        case = dict(trial=trial, m=m, d=d, K=K, n=n, nq=nq, nprobe=nprobe, R=R, init=init, mode=mode)
        gi, gd, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), nprobe, R, init, qmin_mode=mode, debug=True)
        torch.cuda.synchronize()
        probes, qluts, gi, gd = probes.cpu().numpy(), qluts.cpu().numpy(), idx_np(gi), gd.cpu().numpy()
        for iq in range(0, nq, max(1, nq // 12)):
            rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R, qmin_mode=mode,
                                         probes=probes[iq], qluts=qluts[iq])
            assert np.array_equal(gi[iq], rep["ids"]), (case, iq)
            assert np.array_equal(gd[iq], rep["dist"]), (case, iq)
            own = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R, qmin_mode=mode,
                                         probes=probes[iq])
            assert np.abs(own["qluts"].astype(int) - qluts[iq].astype(int)).max() <= 1, (case, iq)
