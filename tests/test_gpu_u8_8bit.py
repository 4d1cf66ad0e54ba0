"""GPU parity of the 8-bit-component variant: Section 3.3's quantizer on 256-entry tables and the
saturating scan of 8-bit codes (qadc_quantize_luts_8bit, qadc_scan_topk with QADC_U8_8BIT)."""

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


def make_db(m, n, d=None, seed=0):
    """8-bit product quantizer on clustered vectors: codebooks f32 [m][256][dsub], codes u8 [n][m]."""
    from oracle import cref
    rng = np.random.default_rng(seed)
    dsub = 4
    d = m * dsub
    centres = rng.uniform(0, 255, size=(32, d)).astype(np.float32)
    x = (centres[rng.integers(0, 32, size=n)] + rng.normal(scale=20, size=(n, d))).astype(np.float32)
    learn = (centres[rng.integers(0, 32, size=256)] + rng.normal(scale=20, size=(256, d))).astype(np.float32)
    cb = np.stack([learn[:, j * dsub:(j + 1) * dsub] for j in range(m)]).astype(np.float32)
    codes = cref.pq_encode(x, cb)
    queries = (centres[rng.integers(0, 32, size=16)] + rng.normal(scale=20, size=(16, d))).astype(np.float32)
    return cb, codes, queries


@pytest.mark.parametrize("m", [4, 8, 16, 32])
@pytest.mark.parametrize("nbins,mode", [(255, 0), (127, 1)])
def test_quantizer_on_256_entry_tables(Q, O, m, nbins, mode):
    cb, codes, queries = make_db(m, 3000, seed=m)
    init, R = 500, 100
    luts = Q.qadc_build_luts(to_gpu(cb), to_gpu(queries))
    ql, bias, delta, qmax = Q.qadc_quantize_luts(luts, to_gpu(codes[:init]), R, nbins, mode)
    want_luts = O.build_luts(cb, queries)
    np.testing.assert_allclose(luts.cpu().numpy(), want_luts, rtol=1e-4, atol=1e-3)
    # whole GPU chain within tolerance
    for q in range(len(queries)):
        wq = O.qmax_from_init(want_luts[q], codes[:init], R)
        wb, wd = O.quantizer_params(want_luts[q], wq, nbins, mode)
        wl = O.quantize_luts(want_luts[q], wb, wd, nbins)
        np.testing.assert_allclose(qmax[q].item(), wq, rtol=1e-4)
        np.testing.assert_allclose(bias[q].cpu().numpy(), wb, rtol=1e-4, atol=1e-3)
        np.testing.assert_allclose(delta[q].item(), wd, rtol=1e-4)
        assert np.abs(ql[q].cpu().numpy().astype(int) - wl.astype(int)).max() <= 1
    # the oracle's float tables fed in: bit-exact
    ql2, bias2, delta2, qmax2 = Q.qadc_quantize_luts(to_gpu(want_luts), to_gpu(codes[:init]), R, nbins, mode)
    for q in range(len(queries)):
        wq = O.qmax_from_init(want_luts[q], codes[:init], R)
        wb, wd = O.quantizer_params(want_luts[q], wq, nbins, mode)
        assert qmax2[q].item() == wq and delta2[q].item() == wd
        assert np.array_equal(bias2[q].cpu().numpy(), wb)
        assert np.array_equal(ql2[q].cpu().numpy(), O.quantize_luts(want_luts[q], wb, wd, nbins))


@pytest.mark.parametrize("m,n,nq", [(8, 20_011, 3), (8, 300_007, 1), (8, 300_007, 16), (4, 600_000, 2),
                                    (16, 150_000, 9), (32, 70_001, 16), (8, 57, 2)])
@pytest.mark.parametrize("nbins", [255, 127])
def test_scan_of_8bit_codes_matches_oracle(Q, O, m, n, nq, nbins):
    """Unseeded, seeded and query-tiled launches; the full path of the oracle per query."""
    from oracle import cref
    cb, codes, queries = make_db(m, n, seed=m + n)
    R, init = 100, 200
    qluts = np.stack([O.quick_adc_bytes_search(cb, y, codes[:max(init, 1)], init, R, nbins)["qlut"]
                      for y in queries[:nq]])
    wi, wd = cref.scan_topk_u8_bytes(codes, qluts, R, nbins)
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_8BIT, to_gpu(codes), to_gpu(qluts), R, nbins)
    assert np.array_equal(idx_np(idx), wi)
    assert np.array_equal(dist.cpu().numpy(), wd)
    if n < 30_000:  # the NumPy oracle end to end (its own sums and top-R)
        for q in range(nq):
            r = O.quick_adc_bytes_search(cb, queries[q], codes, init, R, nbins)
            keep = min(R, n)
            assert np.array_equal(idx_np(idx)[q][:keep], r["idx"][:keep])
            assert np.array_equal(dist.cpu().numpy()[q][:keep], r["dist"][:keep])


def test_scan_of_8bit_codes_massive_ties_and_large_entries(Q, O):
    """Tables of tiny values (every sum ties) and tables whose entries exceed nbins (clamped)."""
    from oracle import cref
    rng = np.random.default_rng(3)
    m, n, R = 8, 280_000, 100
    codes = rng.integers(0, 256, size=(n, m), dtype=np.uint8)
    for hi, nbins in ((2, 255), (256, 100)):
        qluts = rng.integers(0, hi, size=(2, m, 256)).astype(np.uint8)
        wi, wd = cref.scan_topk_u8_bytes(codes, qluts, R, nbins)
        idx, dist = Q.qadc_scan_topk(Q.QADC_U8_8BIT, to_gpu(codes), to_gpu(qluts), R, nbins)
        assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd)


def test_8bit_variant_errors(Q):
    import torch
    codes = torch.zeros((1000, 6), dtype=torch.uint8, device="cuda:0")
    qluts = torch.zeros((1, 6, 256), dtype=torch.uint8, device="cuda:0")
    assert Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_U8_8BIT, 1000, 6, 1, 10) == 0      # m = 6 unsupported
    with pytest.raises(Q.QadcError):
        Q.qadc_scan_topk(Q.QADC_U8_8BIT, codes, qluts, 10)
    luts = torch.zeros((1, 6, 256), dtype=torch.float32, device="cuda:0")
    with pytest.raises(Q.QadcError):
        Q.qadc_quantize_luts(luts, codes[:100], 10)
