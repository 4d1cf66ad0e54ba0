"""GPU parity of the OPQ rotation (Section 2.1: opq(x) = pq(R x)) and of a search that uses it."""

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


def random_rotation(rng, d):
    q, r = np.linalg.qr(rng.normal(size=(d, d)))
    return (q * np.sign(np.diag(r))).astype(np.float32)


@pytest.mark.parametrize("shape", [(1, 128), (5, 96), (77, 64), (300, 130), (1000, 960), (3, 7), (64, 16)])
def test_rotate_matches_oracle(Q, O, shape):
    """float64 products and sums, one rounding: equal to the oracle up to the last bit or two of the
    float32 result (the two sides add in different orders), on tiles with ragged edges in both
    directions."""
    n, d = shape
    rng = np.random.default_rng(n * 1000 + d)
    rot = random_rotation(rng, d)
    x = rng.uniform(0, 255, size=(n, d)).astype(np.float32)
    got = Q.qadc_rotate(to_gpu(rot), to_gpu(x)).cpu().numpy()
    want = O.opq_rotate(rot, x)
    scale = np.linalg.norm(x, axis=1, keepdims=True)    # |y_r| <= |x|: tolerance relative to it
    assert np.abs(got - want).max() <= 2e-7 * scale.max()
    np.testing.assert_allclose(got, want, rtol=1e-4, atol=2e-7 * float(scale.max()))


def test_rotate_special_matrices_and_errors(Q):
    import torch
    rng = np.random.default_rng(0)
    x = rng.normal(size=(40, 32)).astype(np.float32)
    g_x = to_gpu(x)
    eye = to_gpu(np.eye(32, dtype=np.float32))
    assert np.array_equal(Q.qadc_rotate(eye, g_x).cpu().numpy(), x)
    perm = rng.permutation(32)
    pm = np.zeros((32, 32), dtype=np.float32)
    pm[np.arange(32), perm] = 1.0                       # y_r = x_perm[r]
    assert np.array_equal(Q.qadc_rotate(to_gpu(pm), g_x).cpu().numpy(), x[:, perm])
    empty = Q.qadc_rotate(eye, g_x[:0])
    assert empty.shape == (0, 32)
    with pytest.raises(Q.QadcError):
        Q.qadc_rotate(eye, g_x, out=g_x)                # in place is refused
    torch.cuda.synchronize()


def test_search_with_an_optimized_product_quantizer(Q, O):
    """An OPQ trained by the oracle (rotation + codebooks); the database is rotated and encoded on
    the host, the query rotated on the GPU and searched with qadc_search: tables within 1e-4 of
    the oracle's on the rotated query, quantized entries within one step, top-R bit-exact on the
    GPU's own tables."""
    import torch
    from oracle import cref
    from workloads import MixtureSpec, mixture_vectors, kmeans_init_rows, SEED_TRAIN, SEED_BASE, SEED_QUERY
    spec = MixtureSpec(d=64)
    train = mixture_vectors(spec, SEED_TRAIN, 0, 3000)
    rot, cb, hist = O.opq_train(train, 16, 16, 3, 2, kmeans_init_rows(3000, 16))
    base = mixture_vectors(spec, SEED_BASE, 0, 50_000)
    codes = cref.pq_encode(O.opq_rotate(rot, base), cb)
    queries = mixture_vectors(spec, SEED_QUERY, 0, 6)
    R, init = 100, 200
    g_yr = Q.qadc_rotate(to_gpu(rot), to_gpu(queries))
    want_yr = O.opq_rotate(rot, queries)
    np.testing.assert_allclose(g_yr.cpu().numpy(), want_yr, rtol=1e-5, atol=1e-3)
    luts = Q.qadc_build_luts(to_gpu(cb), g_yr).cpu().numpy()
    np.testing.assert_allclose(luts, O.build_luts(cb, want_yr), rtol=1e-4, atol=1e-2)
    ql = torch.empty((len(queries), 16, 16), dtype=torch.uint8, device="cuda:0")
    gi, gd = Q.qadc_search(to_gpu(cb), g_yr, to_gpu(codes), R, init, qluts_out=ql)
    torch.cuda.synchronize()
    h_ql = ql.cpu().numpy()
    for iq in range(len(queries)):
        t = O.quick_adc_tables(cb, want_yr[iq], codes, init, R)
        assert np.abs(h_ql[iq].astype(int) - t["qlut"].astype(int)).max() <= 1
        wi, wd = O.top_r(O.scan_saturating(h_ql[iq], codes), R, pad_dist=255)
        assert np.array_equal(idx_np(gi)[iq], wi) and np.array_equal(gd[iq].cpu().numpy(), wd)


@pytest.mark.parametrize("shape", [(960, 32, 400_000), (256, 16, 400_000), (960, 32, 20_000)])
def test_search_on_high_dimensional_descriptors(Q, O, shape):
    """Shapes of the paper's other datasets (Sections 4.5 and 4.6): 960-dimensional descriptors in
    128-bit codes (m = 32, 30 dimensions per sub-space) and 256-dimensional L2-normalized ones in
    64-bit codes.  qadc_search against the three calls and the oracle, on a database long enough
    for the fused prepare kernel and on a short one."""
    import torch
    from oracle import cref
    d, m, n = shape
    rng = np.random.default_rng(d + n)
    cb = rng.normal(size=(m, 16, d // m)).astype(np.float32)
    if d == 256:
        cb /= np.sqrt(d / m) * 4
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    queries = rng.normal(size=(4, d)).astype(np.float32)
    if d == 256:
        queries /= np.linalg.norm(queries, axis=1, keepdims=True)
    R, init = 100, 200
    g_cb, g_q, g_codes = to_gpu(cb), to_gpu(queries), to_gpu(codes)
    ql = torch.empty((4, m, 16), dtype=torch.uint8, device="cuda:0")
    si, sd = Q.qadc_search(g_cb, g_q, g_codes, R, init, qluts_out=ql)
    luts = Q.qadc_build_luts(g_cb, g_q)
    ql3, _, _, _ = Q.qadc_quantize_luts(luts, g_codes[:init], R)
    ci, cd = Q.qadc_scan_topk(Q.QADC_U8_4BIT, g_codes, ql3, R)
    torch.cuda.synchronize()
    assert torch.equal(ql, ql3) and torch.equal(si, ci) and torch.equal(sd, cd)
    np.testing.assert_allclose(luts.cpu().numpy(), O.build_luts(cb, queries), rtol=1e-4)
    h_ql = ql.cpu().numpy()
    for iq in range(4):
        t = O.quick_adc_tables(cb, queries[iq], codes, init, R)
        assert np.abs(h_ql[iq].astype(int) - t["qlut"].astype(int)).max() <= 1
        wi, wd = cref.scan_topk_u8(codes, h_ql[iq][None], R)
        assert np.array_equal(idx_np(si)[iq], wi[0]) and np.array_equal(sd[iq].cpu().numpy(), wd[0])
