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
    assert Q.qadc_multi_index_workspace_bytes(20000, 3, 8) == 0        # K beyond the limit
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


# ------------------------------------------------------- lists for the occupied cells only

def _group_want(cells, K):
    """Stable sort by cell of the entries inside [0, K*K): (cell_ids, list_off, ids) written with numpy."""
    valid = np.nonzero((cells >= 0) & (cells < K * K))[0]
    order = valid[np.argsort(cells[valid], kind="stable")]
    cell_ids, counts = np.unique(cells[valid], return_counts=True)
    list_off = np.zeros(len(cell_ids) + 1, dtype=np.int64)
    np.cumsum(counts, out=list_off[1:])
    return cell_ids.astype(np.uint32), list_off, order.astype(np.uint32)


@pytest.mark.parametrize("n,K,kind", [
    (0, 8, "uniform"), (1, 8, "uniform"), (5_000, 64, "uniform"), (70_001, 7, "uniform"),
    (300_000, 16384, "uniform"), (300_000, 16384, "clustered"), (40_000, 300, "invalid"),
    (2_000_000, 1000, "clustered"),
])
def test_group_of_occupied_cells(Q, n, K, kind):
    import torch
    rng = np.random.default_rng(n + K)
    if kind == "clustered":   # a few thousand occupied cells with skewed sizes, far apart in cell id
        homes = rng.integers(0, K * K, size=3000)
        cells = homes[np.minimum(rng.zipf(1.3, size=n) - 1, 2999)].astype(np.int32)
    else:
        cells = rng.integers(0, K * K, size=n).astype(np.int32)
    if kind == "invalid":
        cells[::7] = -1
        cells[3::11] = K * K + 5
    want_cells, want_off, want_ids = _group_want(cells, K)
    assert Q.qadc_multi_index_group_workspace_bytes(n, K) > 0
    g = to_gpu(cells) if n else torch.zeros((0,), dtype=torch.int32, device="cuda")
    cell_ids, list_off, ids = Q.qadc_multi_index_group(g, K)
    torch.cuda.synchronize()
    assert np.array_equal(idx_np(cell_ids), want_cells)
    assert np.array_equal(list_off.cpu().numpy(), want_off)
    assert np.array_equal(idx_np(ids), want_ids)


def test_group_rejects_bad_arguments(Q):
    import torch
    assert Q.qadc_multi_index_group_workspace_bytes(10, 16385) == 0
    assert Q.qadc_multi_index_group_workspace_bytes(-1, 16) == 0
    cells = torch.zeros((100,), dtype=torch.int32, device="cuda")
    with pytest.raises(Q.QadcError):
        Q.qadc_multi_index_group(cells, 16385)
    with pytest.raises(Q.QadcError):
        Q.qadc_multi_index_group(cells, 16, workspace=torch.empty((16,), dtype=torch.uint8, device="cuda"))


def test_slots_of_cells(Q, O):
    import torch
    rng = np.random.default_rng(4)
    cell_ids = np.unique(rng.integers(0, 1 << 28, size=50_000)).astype(np.uint32)
    cells = rng.integers(0, 1 << 28, size=(37, 64)).astype(np.int32)
    cells[:, ::3] = rng.choice(cell_ids, size=cells[:, ::3].shape).astype(np.int32)   # present
    cells[5, 7] = -1
    cells[0, 0], cells[0, 1] = int(cell_ids[0]), int(cell_ids[-1])                     # both ends
    got = Q.qadc_multi_index_slots(to_gpu(cell_ids.view(np.int32)), to_gpu(cells)).cpu().numpy()
    assert np.array_equal(got, O.multi_index_slots(cell_ids, cells))
    assert (got >= 0).sum() >= 37 * 22 and (got < 0).any()
    none = Q.qadc_multi_index_slots(torch.zeros((0,), dtype=torch.int32, device="cuda"), to_gpu(cells))
    assert (none.cpu().numpy() == -1).all()                                            # an index without lists


def _sparse_case(O, K, dh, m, n, homes, seed):
    from oracle import cref
    rng = np.random.default_rng(seed)
    d = 2 * dh
    halves = make_halves(K, dh, seed)
    home = rng.choice(K * K, size=homes, replace=False)
    hc = np.concatenate([halves[0][home // K], halves[1][home % K]], axis=1)
    x = (hc[rng.integers(0, homes, size=n)] + rng.normal(scale=10, size=(n, d))).astype(np.float32)
    dsub = d // m
    cells_h = O.multi_index_assign(x, halves)
    cen = np.concatenate([halves[0][cells_h[:4000] // K], halves[1][cells_h[:4000] % K]], axis=1)
    resid_sample = (x[:4000] - cen).astype(np.float32)
    rows = rng.permutation(4000)[:16]
    cb = np.stack([O.kmeans_lloyd(resid_sample[:, j * dsub:(j + 1) * dsub], rows, 3)[0] for j in range(m)])
    # the oracle's index over the occupied cells, its encoding done by the plain-C twin
    cell_ids, list_off, order = _group_want(cells_h, K)
    cen = np.concatenate([halves[0][cells_h[order] // K], halves[1][cells_h[order] % K]], axis=1)
    codes = cref.pq_encode((x[order] - cen).astype(np.float32), cb)
    centroids = np.concatenate([halves[0][cell_ids // K], halves[1][cell_ids % K]], axis=1).astype(np.float32)
    index = dict(cell_ids=cell_ids, centroids=centroids, list_off=list_off, codes=codes, ids=order)
    return halves, x, cb, cells_h, index


@pytest.mark.parametrize("K,m,homes,nq", [(64, 16, 400, 14), (300, 8, 20_000, 14), (64, 16, 400, 80)])
def test_search_over_occupied_cells(Q, O, K, m, homes, nq):
    """The multi-index at its usual shape -- far more product cells than lists: built on the GPU (assign ->
    group -> encode against the half-centroids) it equals the oracle's index over the occupied cells, and a
    search with the multi-index probes mapped to list numbers equals the oracle's search of that index."""
    import torch
    dh, n = 16, 30_000
    d = 2 * dh
    halves, x, cb, cells_h, index = _sparse_case(O, K, dh, m, n, homes, 31 + K)
    small = O.multi_index_build_occupied(x[:3000], halves, cb)   # the oracle's own builder on a part
    gh, gx, gcb = to_gpu(halves), to_gpu(x), to_gpu(cb)
    cells = Q.qadc_multi_index_assign(gh, gx)
    assert np.array_equal(cells.cpu().numpy(), cells_h)
    cell_ids, list_off, ids = Q.qadc_multi_index_group(cells, K)
    codes = Q.qadc_multi_index_encode(gh, gcb, gx, cells, ids)
    torch.cuda.synchronize()
    assert np.array_equal(idx_np(cell_ids), index["cell_ids"])
    assert np.array_equal(list_off.cpu().numpy(), index["list_off"])
    assert np.array_equal(idx_np(ids), index["ids"])
    assert np.array_equal(codes.cpu().numpy(), index["codes"])
    assert len(index["cell_ids"]) < K * K // 4
    # the same builder on the first 3000 vectors against the oracle's builder
    c3 = cells[:3000].contiguous()
    ci3, lo3, id3 = Q.qadc_multi_index_group(c3, K)
    co3 = Q.qadc_multi_index_encode(gh, gcb, gx[:3000].contiguous(), c3, id3)
    assert np.array_equal(idx_np(ci3), small["cell_ids"]) and np.array_equal(lo3.cpu().numpy(), small["list_off"])
    assert np.array_equal(idx_np(id3), small["ids"]) and np.array_equal(co3.cpu().numpy(), small["codes"])

    gix = Q.IvfIndex(None, list_off, codes, ids, gcb, halves=gh, cell_ids=cell_ids)
    rng = np.random.default_rng(2)
    nprobe, R, init = 48, 60, 300   # (64 queries and more: the tables of a query are built by one workgroup)
    queries = (x[rng.integers(0, n, size=nq)] + rng.normal(scale=5, size=(nq, d))).astype(np.float32)
    gq = to_gpu(queries)
    probes = Q.qadc_multi_index_probes(gh, gq, nprobe)
    slots = Q.qadc_multi_index_slots(cell_ids, probes)
    slots_h = slots.cpu().numpy()
    assert np.array_equal(slots_h, O.multi_index_slots(index["cell_ids"], probes.cpu().numpy()))
    assert (slots_h < 0).any() and ((slots_h >= 0).sum(axis=1) >= 1).all() and (slots_h >= 0).sum() >= 3 * nq
    got_ids, dist, pr, qluts = Q.qadc_ivf_search(gix, gq, nprobe, R, init, probes_in=slots, debug=True)
    torch.cuda.synchronize()
    assert np.array_equal(pr.cpu().numpy(), slots_h)
    for iq in range(0, nq, max(1, nq // 14)):
        used = np.nonzero(slots_h[iq] >= 0)[0]
        # whole search by the oracle on the occupied probes: tables within one quantization step
        full = O.ivf_quick_adc_search(index, index["centroids"], cb, queries[iq], len(used), init, R,
                                      probes=slots_h[iq][used])
        ql = qluts[iq].cpu().numpy()
        assert np.abs(ql[used].astype(int) - full["qluts"].astype(int)).max() <= 1
        # integer part replayed on the GPU's tables: bit-exact
        rep = O.ivf_quick_adc_search(index, index["centroids"], cb, queries[iq], len(used), init, R,
                                     probes=slots_h[iq][used], qluts=ql[used])
        assert np.array_equal(idx_np(got_ids)[iq], rep["ids"])
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"])


def test_index_without_centroids_needs_probes(Q, O):
    import torch
    halves, x, cb, cells_h, index = _sparse_case(O, 32, 8, 8, 5000, 50, 3)
    gix = Q.IvfIndex(None, to_gpu(index["list_off"]), to_gpu(index["codes"]), to_gpu(index["ids"].view(np.int32)),
                     to_gpu(cb), halves=to_gpu(halves), cell_ids=to_gpu(index["cell_ids"].view(np.int32)))
    with pytest.raises(Q.QadcError):
        Q.qadc_ivf_search(gix, to_gpu(x[:3]), 4, 10, 100)
