"""GPU parity of the database-side entry points: list layouts (Fig. 2), inverted-index build (Section 2.2)."""

import numpy as np
import pytest

from gpu_common import to_gpu, idx_np
from test_gpu_ivf import build_ivf

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


# ------------------------------------------------------------------ layouts

@pytest.mark.parametrize("m", [8, 16, 32, 64])
@pytest.mark.parametrize("n", [1, 15, 16, 17, 37, 511, 4096, 100_003])
def test_pack_and_unpack_match_oracle(Q, O, m, n):
    rng = np.random.default_rng(m * 1000 + n)
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    want = O.pack_transposed(codes)
    assert Q.qadc_packed_bytes(n, m, Q.QADC_LAYOUT_TRANSPOSED) == len(want) == O.transposed_bytes(n, m)
    assert Q.qadc_packed_bytes(n, m, Q.QADC_LAYOUT_STANDARD) == codes.size
    g = to_gpu(codes)
    packed = Q.qadc_pack_codes(g, Q.QADC_LAYOUT_TRANSPOSED)
    assert np.array_equal(packed.cpu().numpy(), want)          # byte for byte, zero fill included
    import torch
    back = torch.full((n, m // 2), 0xEE, dtype=torch.uint8, device="cuda:0")
    Q.qadc_unpack_codes(packed, n, m, Q.QADC_LAYOUT_TRANSPOSED, out=back)
    assert np.array_equal(back.cpu().numpy(), codes)
    same = Q.qadc_pack_codes(g, Q.QADC_LAYOUT_STANDARD)
    assert np.array_equal(same.cpu().numpy().reshape(n, m // 2), codes)


def test_unpack_does_not_write_past_the_list(Q, O):
    import torch
    n, m = 37, 8   # 37 * 4 = 148 bytes: the list ends inside a 16-byte piece
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    packed = to_gpu(O.pack_transposed(codes))
    buf = torch.full((n + 16, m // 2), 0xEE, dtype=torch.uint8, device="cuda:0")
    Q.qadc_unpack_codes(packed, n, m, Q.QADC_LAYOUT_TRANSPOSED, out=buf[:n])
    got = buf.cpu().numpy()
    assert np.array_equal(got[:n], codes) and (got[n:] == 0xEE).all()


def test_scan_of_an_unpacked_list_equals_block_scan(Q, O):
    """A database kept in the paper's transposed layout: unpack on the GPU, scan, compare with Alg. 2
    run by the oracle over the blocks and rows of the transposed list."""
    rng = np.random.default_rng(9)
    n, m, R = 20_011, 16, 50
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    packed = O.pack_transposed(codes)
    qlut = rng.integers(0, 40, size=(1, m, 16), dtype=np.uint8)
    sums = O.scan_blocks_transposed(qlut[0], packed, n)
    wi, wd = O.top_r(sums, R)
    std = Q.qadc_unpack_codes(to_gpu(packed), n, m, Q.QADC_LAYOUT_TRANSPOSED)
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, std, to_gpu(qlut), R)
    assert np.array_equal(idx_np(idx)[0], wi) and np.array_equal(dist.cpu().numpy()[0], wd)


def test_layout_errors(Q):
    import torch
    g = torch.zeros((64, 8), dtype=torch.uint8, device="cuda:0")
    out = torch.zeros((1024,), dtype=torch.uint8, device="cuda:0")
    L = Q.lib()
    import ctypes
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.qadc_pack_codes(p(g), 64, 16, 7, p(out), None) == Q.QADC_EINVAL          # unknown layout
    assert L.qadc_pack_codes(p(g), 64, 12, 1, p(out), None) == Q.QADC_EINVAL          # unsupported m
    assert L.qadc_pack_codes(p(g), -1, 16, 1, p(out), None) == Q.QADC_EINVAL
    assert L.qadc_pack_codes(p(g), 64, 16, 1, p(g), None) == Q.QADC_EINVAL            # in place
    assert L.qadc_pack_codes(p(g), 64, 16, 1, ctypes.c_void_p(out.data_ptr() + 4), None) == Q.QADC_EINVAL
    assert L.qadc_pack_codes(None, 64, 16, 1, p(out), None) == Q.QADC_EINVAL
    assert L.qadc_pack_codes(None, 0, 16, 1, None, None) == Q.QADC_OK                 # nothing to do
    assert Q.qadc_packed_bytes(10, 12, 1) == 0 and Q.qadc_packed_bytes(10, 16, 5) == 0


# ------------------------------------------------------------------ encode

@pytest.mark.parametrize("shape", [(128, 16, 16), (128, 32, 16), (96, 8, 256), (96, 16, 16), (960, 32, 16)])
def test_pq_encode_is_bit_exact(Q, O, shape):
    from oracle import cref
    d, m, k = shape
    rng = np.random.default_rng(d + m)
    n = 6007
    cb = rng.uniform(0, 255, size=(m, k, d // m)).astype(np.float32)
    x = rng.uniform(0, 255, size=(n, d)).astype(np.float32)
    x[:k] = np.concatenate([cb[j] for j in range(m)], axis=1)[:k]     # vectors that sit on centroids
    cb[:, 3] = cb[:, 1]                                                # a duplicated centroid: ties
    want = cref.pq_encode(x, cb)
    got = Q.qadc_pq_encode(to_gpu(cb), to_gpu(x)).cpu().numpy()
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ inverted index

@pytest.mark.parametrize("K,d,n", [(300, 128, 5003), (64, 20, 1000), (1, 32, 100), (1000, 96, 2049)])
def test_ivf_assign_matches_oracle(Q, O, K, d, n):
    rng = np.random.default_rng(K + d)
    coarse = rng.uniform(0, 255, size=(K, d)).astype(np.float32)
    if K > 10:
        coarse[7] = coarse[2]        # duplicate centroids: the lower cell must win
        coarse[K - 1] = coarse[5]
    x = rng.uniform(0, 255, size=(n, d)).astype(np.float32)
    x[:min(n, K)] = coarse[:min(n, K)]   # vectors that sit on centroids (distance zero)
    x[-1] = coarse[K - 1]
    want = O.ivf_assign(x, coarse)
    got = Q.qadc_ivf_assign(to_gpu(coarse), to_gpu(x)).cpu().numpy()
    assert got.dtype == np.int32 and np.array_equal(got, want)
    if K > 10:
        assert got[7] == 2 and got[-1] == 5


@pytest.mark.parametrize("K,n", [(1000, 100_003), (1, 5000), (65536, 300_000), (48, 63), (7, 0), (300, 4096 * 3 + 1)])
def test_ivf_group_is_the_stable_grouping(Q, O, K, n):
    import torch
    from workloads import zipf_list_sizes
    rng = np.random.default_rng(K + n)
    if n:
        sizes = zipf_list_sizes(n, K, 0.8, 1) if K > 1 else np.array([n])
        cells = np.repeat(np.arange(K), sizes).astype(np.int32)[:n]
        if len(cells) < n:
            cells = np.concatenate([cells, rng.integers(0, K, size=n - len(cells)).astype(np.int32)])
        rng.shuffle(cells)
    else:
        cells = np.zeros(0, dtype=np.int32)
    nbytes = Q.qadc_ivf_group_workspace_bytes(n, K)
    ws = torch.full((max(nbytes, 16),), 0xAB, dtype=torch.uint8, device="cuda:0")   # dirty on purpose
    g = to_gpu(cells) if n else torch.zeros((0,), dtype=torch.int32, device="cuda:0")
    for _ in range(2):   # the workspace is reused as the first call left it
        list_off, ids = Q.qadc_ivf_group(g, K, workspace=ws)
        want_off = np.zeros(K + 1, dtype=np.int64)
        np.cumsum(np.bincount(cells, minlength=K), out=want_off[1:])
        assert np.array_equal(list_off.cpu().numpy(), want_off)
        assert np.array_equal(idx_np(ids), np.argsort(cells, kind="stable").astype(np.uint32))


def test_ivf_group_leaves_out_cells_out_of_range(Q):
    rng = np.random.default_rng(4)
    K, n = 50, 10_000
    cells = rng.integers(0, K, size=n).astype(np.int32)
    cells[::7] = -1
    cells[3::11] = K + 5
    ok = (cells >= 0) & (cells < K)
    list_off, ids = Q.qadc_ivf_group(to_gpu(cells), K)
    want_off = np.zeros(K + 1, dtype=np.int64)
    np.cumsum(np.bincount(cells[ok], minlength=K), out=want_off[1:])
    assert np.array_equal(list_off.cpu().numpy(), want_off)
    kept = np.flatnonzero(ok)
    want = kept[np.argsort(cells[kept], kind="stable")].astype(np.uint32)
    assert np.array_equal(idx_np(ids)[:len(want)], want)


@pytest.mark.parametrize("m", [16, 32])
def test_index_built_on_the_gpu_equals_the_oracles(Q, O, m):
    """assign -> group -> encode on the GPU give the oracle's index byte for byte, and a search of it
    gives the oracle's search of the oracle's index."""
    import torch
    coarse, cb, x, index = build_ivf(O, n=30_000, K=40, m=m, seed=10 + m)
    gx, gco, gcb = to_gpu(x), to_gpu(coarse), to_gpu(cb)
    cells = Q.qadc_ivf_assign(gco, gx)
    list_off, ids = Q.qadc_ivf_group(cells, len(coarse))
    codes = Q.qadc_ivf_encode(gco, gcb, gx, cells, ids)
    assert np.array_equal(list_off.cpu().numpy(), index["list_off"])
    assert np.array_equal(idx_np(ids), index["ids"])
    assert np.array_equal(codes.cpu().numpy(), index["codes"])
    gix = Q.IvfIndex(gco, list_off, codes, ids, gcb)
    rng = np.random.default_rng(1)
    queries = (x[rng.integers(0, len(x), size=6)] + rng.normal(scale=6, size=(6, x.shape[1]))).astype(np.float32)
    got_ids, dist, probes, qluts = Q.qadc_ivf_search(gix, to_gpu(queries), 6, 50, 300, debug=True)
    torch.cuda.synchronize()
    for iq in range(len(queries)):
        rep = O.ivf_quick_adc_search(index, coarse, cb, queries[iq], 6, 300, 50,
                                     probes=probes[iq].cpu().numpy(), qluts=qluts[iq].cpu().numpy())
        assert np.array_equal(idx_np(got_ids)[iq], rep["ids"])
        assert np.array_equal(dist[iq].cpu().numpy(), rep["dist"])


def test_ivf_encode_guards_ids_and_cells(Q, O):
    import torch
    coarse, cb, x, index = build_ivf(O, n=6000, K=8, seed=3)
    cells = O.ivf_assign(x, coarse).astype(np.int32)
    ids = np.arange(len(x), dtype=np.uint32)
    cells_bad = cells.copy()
    cells_bad[5] = 99
    ids_bad = ids.copy()
    ids_bad[9] = 4_000_000_000
    codes = Q.qadc_ivf_encode(to_gpu(coarse), to_gpu(cb), to_gpu(x), to_gpu(cells_bad),
                              to_gpu(ids_bad.view(np.int32))).cpu().numpy()
    from oracle import cref
    want = cref.pq_encode((x - coarse[cells]).astype(np.float32), cb)
    want[5] = 0
    want[9] = 0
    assert np.array_equal(codes, want)
