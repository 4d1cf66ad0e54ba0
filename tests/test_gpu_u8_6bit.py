"""GPU parity of the 6-bit-component variant (the paper's Conclusion: 6-bit quantizers with wider
registers): qadc_pq_train / qadc_pq_encode with 64 centroids, Eq. (1) on 64-entry tables, Section
3.3's quantizer (qadc_quantize_luts_6bit) and the saturating scan of 6-bit codes (qadc_scan_topk
with QADC_U8_6BIT), against the oracle's chain and its plain-C twin."""

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


def make_db(O, m, n, seed=0, dsub=4):
    """6-bit product quantizer on clustered vectors: codebooks f32 [m][64][dsub], codes u8 [n][3m/4]."""
    rng = np.random.default_rng(seed)
    d = m * dsub
    centres = rng.uniform(0, 255, size=(32, d)).astype(np.float32)
    x = (centres[rng.integers(0, 32, size=n)] + rng.normal(scale=20, size=(n, d))).astype(np.float32)
    learn = (centres[rng.integers(0, 32, size=64)] + rng.normal(scale=20, size=(64, d))).astype(np.float32)
    cb = np.stack([learn[:, j * dsub:(j + 1) * dsub] for j in range(m)]).astype(np.float32)
    queries = (centres[rng.integers(0, 32, size=16)] + rng.normal(scale=20, size=(16, d))).astype(np.float32)
    return cb, x, queries


@pytest.mark.parametrize("m", [8, 16, 32])
def test_encode_and_train_with_64_centroids(Q, O, m):
    import torch
    cb, x, _ = make_db(O, m, 5000, seed=m)
    codes = Q.qadc_pq_encode(to_gpu(cb), to_gpu(x))
    want = O.pack_sixbit(O.pq_encode(x, cb))
    assert codes.shape == (5000, 3 * m // 4)
    assert np.array_equal(codes.cpu().numpy(), want)
    # k-means with 64 centroids: the oracle's Lloyd iterations (float64 on both sides)
    rows = np.random.default_rng(m).permutation(5000)[:64]
    got = Q.qadc_pq_train(to_gpu(x), m, 64, to_gpu(rows.astype(np.int64)), 3).cpu().numpy()
    np.testing.assert_allclose(got, O.pq_train(x, m, 64, 3, rows), rtol=2e-6, atol=1e-4)


@pytest.mark.parametrize("m", [8, 16, 32])
@pytest.mark.parametrize("nbins,mode", [(255, 0), (127, 1)])
def test_quantizer_on_64_entry_tables(Q, O, m, nbins, mode):
    cb, x, queries = make_db(O, m, 3000, seed=10 + m)
    comps = O.pq_encode(x, cb)
    codes = O.pack_sixbit(comps)
    init, R = 500, 100
    luts = Q.qadc_build_luts(to_gpu(cb), to_gpu(queries))
    want_luts = O.build_luts(cb, queries)
    np.testing.assert_allclose(luts.cpu().numpy(), want_luts, rtol=1e-4, atol=1e-3)
    ql, bias, delta, qmax = Q.qadc_quantize_luts_6bit(luts, to_gpu(codes[:init]), R, nbins, mode)
    for q in range(len(queries)):
        wq = O.qmax_from_init(want_luts[q], comps[:init], R)
        wb, wd = O.quantizer_params(want_luts[q], wq, nbins, mode)
        np.testing.assert_allclose(qmax[q].item(), wq, rtol=1e-4)
        np.testing.assert_allclose(bias[q].cpu().numpy(), wb, rtol=1e-4, atol=1e-3)
        np.testing.assert_allclose(delta[q].item(), wd, rtol=1e-4)
        assert np.abs(ql[q].cpu().numpy().astype(int) - O.quantize_luts(want_luts[q], wb, wd, nbins).astype(int)).max() <= 1
    # the oracle's float tables fed in: bit-exact
    ql2, bias2, delta2, qmax2 = Q.qadc_quantize_luts_6bit(to_gpu(want_luts), to_gpu(codes[:init]), R, nbins, mode)
    for q in range(len(queries)):
        wq = O.qmax_from_init(want_luts[q], comps[:init], R)
        wb, wd = O.quantizer_params(want_luts[q], wq, nbins, mode)
        assert qmax2[q].item() == wq and delta2[q].item() == wd
        assert np.array_equal(bias2[q].cpu().numpy(), wb)
        assert np.array_equal(ql2[q].cpu().numpy(), O.quantize_luts(want_luts[q], wb, wd, nbins))


@pytest.mark.parametrize("m,n,nq", [(8, 20_011, 3), (8, 600_007, 1), (16, 300_007, 2), (16, 1_100_003, 1),
                                    (32, 300_001, 9), (16, 57, 2), (8, 0, 1), (32, 1_000_000, 1)])
@pytest.mark.parametrize("nbins", [255, 127])
def test_scan_of_6bit_codes_matches_oracle(Q, O, m, n, nq, nbins):
    """Short databases (no sampled bound), long ones (sampled bound, barrier-free pass, several tiles
    per workgroup, ragged tails), one and several queries; sums and top-R bit-exact against the
    plain-C chain on the oracle's quantized tables."""
    from oracle import cref
    cb, x, queries = make_db(O, m, max(n, 300), seed=m + n)
    comps = O.pq_encode(x[:max(n, 300)], cb) if n <= 50_000 else None
    if comps is None:  # long databases: codes drawn directly (the encoder is tested above)
        rng = np.random.default_rng(n)
        base = O.pq_encode(x[:20_000], cb)
        comps = base[rng.integers(0, len(base), size=n)]
    R, init = 100, 200
    codes_all = O.pack_sixbit(comps)
    qluts = np.stack([O.quick_adc_sixbit_search(cb, y, codes_all[:init], init, R, nbins)["qlut"] for y in queries[:nq]])
    codes = codes_all[:n]
    wi, wd = cref.scan_topk_u8_sixbit(codes, qluts, R, nbins)
    gi, gd = Q.qadc_scan_topk(Q.QADC_U8_6BIT, to_gpu(codes) if n else to_gpu(np.zeros((0, 3 * m // 4), np.uint8)),
                              to_gpu(qluts), R, nbins)
    assert np.array_equal(idx_np(gi), wi)
    assert np.array_equal(gd.cpu().numpy(), wd)


def test_6bit_scan_ties_and_useless_bound(Q, O):
    """Every code identical: all sums tie, the sampled bound lets everything through, the list
    overflows and the careful pass decides by index; then codes in decreasing order of their sum."""
    from oracle import cref
    m, n, R = 16, 400_000, 100
    rng = np.random.default_rng(3)
    qlut = rng.integers(0, 30, size=(1, m, 64)).astype(np.uint8)
    comps = np.tile(rng.integers(0, 64, size=(1, m)).astype(np.uint8), (n, 1))
    codes = O.pack_sixbit(comps)
    wi, wd = cref.scan_topk_u8_sixbit(codes, qlut, R)
    gi, gd = Q.qadc_scan_topk(Q.QADC_U8_6BIT, to_gpu(codes), to_gpu(qlut), R)
    assert np.array_equal(idx_np(gi), wi) and np.array_equal(gd.cpu().numpy(), wd)
    assert wi[0].tolist() == list(range(R))
    # decreasing sums: component 0 falls from 63 to 0 along the database, its table rises with the index
    qlut2 = np.zeros((1, m, 64), dtype=np.uint8)
    qlut2[0, 0] = np.arange(64) * 3
    comps2 = np.zeros((n, m), dtype=np.uint8)
    comps2[:, 0] = 63 - (np.arange(n) * 64 // n)
    codes2 = O.pack_sixbit(comps2)
    wi, wd = cref.scan_topk_u8_sixbit(codes2, qlut2, R)
    gi, gd = Q.qadc_scan_topk(Q.QADC_U8_6BIT, to_gpu(codes2), to_gpu(qlut2), R)
    assert np.array_equal(idx_np(gi), wi) and np.array_equal(gd.cpu().numpy(), wd)


def test_6bit_variant_errors(Q):
    import torch
    L = Q.lib()
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_U8_6BIT, 1000, 16, 1, 100) > 0
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_U8_6BIT, 1000, 12, 1, 100) == 0   # m not in {8, 16, 32}
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_U8_6BIT, 1000, 64, 1, 100) == 0
    cb = torch.zeros((6, 64, 2), device="cuda:0")
    x = torch.zeros((4, 12), device="cuda:0")
    with pytest.raises(Q.QadcError):
        Q.qadc_pq_encode(cb, x)   # m not a multiple of 4
