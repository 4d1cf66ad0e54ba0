"""GPU parity of the inverted multi-index entry points (Section 5, related work): cell centroids,
assignment, probe order, and a Quick ADC search over an index built on the product cells."""

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


def make_halves(K, dh, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(0, 255, size=(2, K, dh)).astype(np.float32)


@pytest.mark.parametrize("K,dh", [(1, 3), (7, 5), (64, 32), (300, 16)])
def test_cells_are_the_concatenated_half_centroids(Q, O, K, dh):
    halves = make_halves(K, dh, K + dh)
    got = Q.qadc_multi_index_cells(to_gpu(halves)).cpu().numpy()
    assert np.array_equal(got, O.multi_index_cells(halves))


@pytest.mark.parametrize("K,dh,n", [(16, 8, 5003), (256, 64, 3000), (1, 4, 100), (37, 3, 2049)])
def test_assign_matches_oracle(Q, O, K, dh, n):
    rng = np.random.default_rng(K * 7 + dh)
    halves = make_halves(K, dh, K)
    if K > 10:
        halves[0, 7] = halves[0, 2]        # duplicate half-centroids: the lower one must win
        halves[1, K - 1] = halves[1, 5]
    x = rng.uniform(0, 255, size=(n, 2 * dh)).astype(np.float32)
    k = min(n, K)
    x[:k, :dh] = halves[0, :k]             # halves that sit on centroids
    x[:k, dh:] = halves[1, ::-1][:k]
    want = O.multi_index_assign(x, halves)
    got = Q.qadc_multi_index_assign(to_gpu(halves), to_gpu(x)).cpu().numpy()
    assert got.dtype == np.int32 and np.array_equal(got, want)


@pytest.mark.parametrize("K,dh,nprobe,nq", [(64, 16, 64, 40), (256, 64, 64, 20), (300, 8, 256, 9), (5, 4, 7, 6),
                                            (3, 2, 20, 4), (1, 2, 1, 3), (40, 6, 1, 5)])
def test_probes_are_the_smallest_sums_in_order(Q, O, K, dh, nprobe, nq):
    """Against the definition over all K*K sums (float64).  Where float32 rounding orders two nearly
    equal sums the other way, the probed cells' sums must agree to rounding."""
    rng = np.random.default_rng(K + nprobe)
    halves = make_halves(K, dh, K + 1)
    if K > 10:
        halves[0, 3] = halves[0, 1]        # exact ties between cells: lowest cell id first
        halves[1, 4] = halves[1, 0]
    queries = rng.uniform(0, 255, size=(nq, 2 * dh)).astype(np.float32)
    queries[0, :dh] = halves[0, min(1, K - 1)]
    got = Q.qadc_multi_index_probes(to_gpu(halves), to_gpu(queries), nprobe).cpu().numpy()
    cells = K * K
    for iq in range(nq):
        want = O.multi_index_probes(queries[iq], halves, nprobe)
        g = got[iq]
        keep = min(nprobe, cells)
        assert (g[keep:] == -1).all()
        g = g[:keep]
        assert len(set(g.tolist())) == keep and g.min() >= 0 and g.max() < cells
        if not np.array_equal(g, want):
            d1 = O.sq_l2(queries[iq][None, :dh], halves[0])[0]
            d2 = O.sq_l2(queries[iq][None, dh:], halves[1])[0]
            s = (d1[:, None] + d2[None, :]).reshape(-1)
            np.testing.assert_allclose(s[g], s[want], rtol=1e-5)
    if K > 10:   # the planted exact ties, wherever they are probed, come lowest cell first
        for iq in range(nq):
            pos = {int(c): t for t, c in enumerate(got[iq]) if c >= 0}
            for c, t in pos.items():
                i, j = divmod(c, K)
                twin = (1 if i == 3 else i) * K + (0 if j == 4 else j)
                if twin != c and twin in pos:
                    assert pos[twin] < t


def test_probe_errors(Q):
    import torch
    halves = torch.zeros((2, 8, 4), dtype=torch.float32, device="cuda:0")
    y = torch.zeros((3, 8), dtype=torch.float32, device="cuda:0")
    assert Q.qadc_multi_index_workspace_bytes(8, 3, 300) == 0          # nprobe beyond the limit
    assert Q.qadc_multi_index_workspace_bytes(5000, 3, 8) == 0         # K beyond the limit
    with pytest.raises(Q.QadcError):
        Q.qadc_multi_index_probes(halves, y, 300)
    ws = torch.zeros((16,), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(Q.QadcError):
        Q.qadc_multi_index_probes(halves, y, 4, workspace=ws)           # workspace too small


def test_search_over_a_multi_index(Q, O):
    """Index built on the GPU over the K*K product cells (assign -> group -> encode) equals the oracle's
    inverted index over the expanded centroids; a search with the multi-index probes equals the oracle's
    search of that index with the same probes and tables."""
    import torch
    from oracle import cref
    rng = np.random.default_rng(21)
    K, dh, m, n = 12, 16, 16, 40_000
    d = 2 * dh
    halves = make_halves(K, dh, 5)
    coarse = O.multi_index_cells(halves)
    home = rng.integers(0, K * K, size=n)
    x = (coarse[home] + rng.normal(scale=14, size=(n, d))).astype(np.float32)
    dsub = d // m
    cells_h = O.multi_index_assign(x, halves)
    resid_sample = (x[:4000] - coarse[cells_h[:4000]]).astype(np.float32)
    rows = rng.permutation(4000)[:16]
    cb = np.stack([O.kmeans_lloyd(resid_sample[:, j * dsub:(j + 1) * dsub], rows, 3)[0] for j in range(m)])
    order = np.argsort(cells_h, kind="stable")
    want_codes = cref.pq_encode((x[order] - coarse[cells_h[order]]).astype(np.float32), cb)
    want_off = np.zeros(K * K + 1, dtype=np.int64)
    np.cumsum(np.bincount(cells_h, minlength=K * K), out=want_off[1:])
    index = dict(list_off=want_off, codes=want_codes, ids=order.astype(np.uint32))

    gh, gx, gcb = to_gpu(halves), to_gpu(x), to_gpu(cb)
    gco = Q.qadc_multi_index_cells(gh)
    cells = Q.qadc_multi_index_assign(gh, gx)
    assert np.array_equal(cells.cpu().numpy(), cells_h)
    list_off, ids = Q.qadc_ivf_group(cells, K * K)
    codes = Q.qadc_ivf_encode(gco, gcb, gx, cells, ids)
    assert np.array_equal(list_off.cpu().numpy(), want_off)
    assert np.array_equal(idx_np(ids), index["ids"])
    assert np.array_equal(codes.cpu().numpy(), want_codes)

    gix = Q.IvfIndex(gco, list_off, codes, ids, gcb)
    nq, nprobe, R, init = 12, 24, 50, 300
    queries = (x[rng.integers(0, n, size=nq)] + rng.normal(scale=5, size=(nq, d))).astype(np.float32)
    gq = to_gpu(queries)
    probes = Q.qadc_multi_index_probes(gh, gq, nprobe)
    got_ids, dist, pr, qluts = Q.qadc_ivf_search(gix, gq, nprobe, R, init, probes_in=probes, debug=True)
    torch.cuda.synchronize()
    assert np.array_equal(pr.cpu().numpy(), probes.cpu().numpy())
    for iq in range(nq):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], nprobe, init, R,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(got_ids)[iq], rep["ids"])
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"])
