"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs."""

import os

import numpy as np
import pytest

from gpu_common import config1, to_gpu, idx_np

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


def oracle_topk(codes, qlut, R, nbins=255):
    from oracle import cref
    i, d = cref.scan_topk_u8(codes, qlut[None], R, nbins)
    return i[0], d[0]


def gpu_topk(Q, codes_gpu, qluts, R, nbins=255, n=None):
    import torch
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, codes_gpu, to_gpu(qluts), R, nbins, n=n)
    torch.cuda.synchronize()
    return idx_np(idx), dist.cpu().numpy()


# ------------------------------------------------------------------ tables

@pytest.mark.parametrize("with_base", [False, True])
def test_build_luts_matches_oracle(Q, O, with_base):
    c = config1()
    base = c["base"][:len(c["queries"])] if with_base else None
    want = O.build_luts(c["codebooks"], c["queries"], base)
    got = Q.qadc_build_luts(to_gpu(c["codebooks"]), to_gpu(c["queries"]),
                            to_gpu(base) if with_base else None).cpu().numpy()
    np.testing.assert_allclose(got, want, rtol=1e-4, atol=0)


def test_build_luts_8bit_tables(Q, O):
    rng = np.random.default_rng(0)
    cb = rng.normal(scale=30, size=(8, 256, 12)).astype(np.float32)
    y = rng.normal(scale=30, size=(5, 96)).astype(np.float32)
    got = Q.qadc_build_luts(to_gpu(cb), to_gpu(y)).cpu().numpy()
    np.testing.assert_allclose(got, O.build_luts(cb, y), rtol=1e-4)


@pytest.mark.parametrize("nbins", [255, 127])
@pytest.mark.parametrize("mode", [0, 1])
def test_quantize_luts_matches_oracle(Q, O, nbins, mode):
    c = config1()
    cb, codes, queries = c["codebooks"], c["codes"], c["queries"]
    R, init = 100, 200
    # (a) the whole GPU chain: float tables within 1e-4, quantized entries within +-1
    luts = Q.qadc_build_luts(to_gpu(cb), to_gpu(queries))
    ql, bias, delta, qmax = Q.qadc_quantize_luts(luts, to_gpu(codes[:init]), R, nbins, mode)
    ql, bias, delta, qmax = (t.cpu().numpy() for t in (ql, bias, delta, qmax))
    for iq in range(len(queries)):
        t = O.quick_adc_tables(cb, queries[iq], codes, init, R, nbins, mode)
        np.testing.assert_allclose(qmax[iq], t["qmax"], rtol=1e-4)
        np.testing.assert_allclose(bias[iq], t["bias"], rtol=1e-4)
        np.testing.assert_allclose(delta[iq], t["delta"], rtol=1e-4)
        assert np.abs(ql[iq].astype(int) - t["qlut"].astype(int)).max() <= 1
        assert ql[iq].max() <= nbins
    # (b) identical float tables in -> identical float32 arithmetic -> identical bytes out
    o_luts = O.build_luts(cb, queries)
    ql, bias, delta, qmax = Q.qadc_quantize_luts(to_gpu(o_luts), to_gpu(codes[:init]), R, nbins, mode)
    ql, bias, delta, qmax = (t.cpu().numpy() for t in (ql, bias, delta, qmax))
    for iq in range(len(queries)):
        t = O.quick_adc_tables(cb, queries[iq], codes, init, R, nbins, mode, lut=o_luts[iq])
        assert qmax[iq] == t["qmax"] and delta[iq] == t["delta"]
        assert np.array_equal(bias[iq], t["bias"])
        assert np.array_equal(ql[iq], t["qlut"])


def test_quantize_edge_cases(Q, O):
    c = config1()
    cb, codes, queries = c["codebooks"], c["codes"], c["queries"][:3]
    o_luts = O.build_luts(cb, queries)
    # init smaller than R, init = 1, init larger than usual
    for init, R in [(50, 100), (1, 100), (1000, 100), (8192, 1000), (200, 1)]:
        ql, bias, delta, qmax = Q.qadc_quantize_luts(to_gpu(o_luts), to_gpu(codes[:init]), R)
        for iq in range(len(queries)):
            t = O.quick_adc_tables(cb, queries[iq], codes, init, R, lut=o_luts[iq])
            assert qmax[iq].item() == t["qmax"], (init, R)
            assert np.array_equal(ql[iq].cpu().numpy(), t["qlut"])
    # qmax given instead of init codes; degenerate delta (qmax <= qmin)
    import torch
    for qm in (1e9, 0.0):
        qmax_in = torch.full((len(queries),), qm, dtype=torch.float32, device="cuda:0")
        ql, bias, delta, qmax = Q.qadc_quantize_luts(to_gpu(o_luts), None, 100, qmax_in=qmax_in)
        for iq in range(len(queries)):
            b, dl = O.quantizer_params(o_luts[iq], np.float32(qm), 255, 0)
            assert delta[iq].item() == dl
            assert np.array_equal(ql[iq].cpu().numpy(), O.quantize_luts(o_luts[iq], b, dl, 255))
    # several table sets per query share one quantizer
    rng = np.random.default_rng(1)
    luts = rng.uniform(5, 3000, size=(4, 6, 16, 16)).astype(np.float32)
    qmax_in = to_gpu(np.array([20000, 30000, 1000, 50000], dtype=np.float32))
    for mode in (0, 1):
        ql, bias, delta, _ = Q.qadc_quantize_luts(to_gpu(luts), None, 100, 255, mode, qmax_in=qmax_in)
        for iq in range(4):
            b, dl = O.quantizer_params(luts[iq], qmax_in[iq].item(), 255, mode)
            assert np.array_equal(bias[iq].cpu().numpy(), b) and delta[iq].item() == dl
            want = np.stack([O.quantize_luts(l, b, dl, 255) for l in luts[iq]])
            assert np.array_equal(ql[iq].cpu().numpy(), want)


def test_bad_arguments_are_errors(Q):
    import torch
    c = config1()
    codes = to_gpu(c["codes"][:1000])
    ql = torch.zeros((1, 16, 16), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(Q.QadcError) as e:
        Q.qadc_scan_topk(Q.QADC_U8_4BIT, codes, ql, 5000)
    assert e.value.code == Q.QADC_EINVAL
    with pytest.raises(Q.QadcError) as e:
        Q.qadc_scan_topk(Q.QADC_U8_4BIT, codes, ql, 100,
                         workspace=torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert e.value.code == Q.QADC_ENOMEM
    with pytest.raises(Q.QadcError):
        Q.qadc_scan_topk(Q.QADC_U8_4BIT, codes, ql, 100, nbins=300)
    luts = torch.zeros((1, 16, 16), dtype=torch.float32, device="cuda:0")
    with pytest.raises(Q.QadcError):
        Q.qadc_quantize_luts(luts, None, 100)  # neither init codes nor qmax


# -------------------------------------------------------------------- scan

@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("nbins", [255, 127])
def test_scan_topk_config1_bit_exact(Q, O, nbins, mode):
    """Config 1: N=100k, 16 queries, oracle-quantized tables in -> identical indices and sums out."""
    c = config1()
    cb, codes, queries = c["codebooks"], c["codes"], c["queries"]
    R = 100
    qluts = np.stack([O.quick_adc_tables(cb, y, codes, 200, R, nbins, mode)["qlut"] for y in queries])
    gi, gd = gpu_topk(Q, to_gpu(codes), qluts, R, nbins)
    for iq in range(len(queries)):
        wi, wd = oracle_topk(codes, qluts[iq], R, nbins)
        assert np.array_equal(gi[iq], wi), f"query {iq}"
        assert np.array_equal(gd[iq], wd), f"query {iq}"


def test_full_chain_config1(Q, O):
    """GPU tables -> GPU quantization -> GPU scan; the oracle replays the integer part on the GPU's tables."""
    c = config1()
    cb, codes, queries = c["codebooks"], c["codes"], c["queries"]
    R, init = 100, 200
    g_codes = to_gpu(codes)
    luts = Q.qadc_build_luts(to_gpu(cb), to_gpu(queries))
    ql, _, _, _ = Q.qadc_quantize_luts(luts, g_codes[:init], R)
    import torch
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, g_codes, ql, R)
    torch.cuda.synchronize()
    h_ql = ql.cpu().numpy()
    fidx = []
    for iq in range(len(queries)):
        wi, wd = oracle_topk(codes, h_ql[iq], R)
        assert np.array_equal(idx_np(idx)[iq], wi) and np.array_equal(dist[iq].cpu().numpy(), wd)
        fi, _ = O.adc_search(cb, queries[iq], O.unpack_nibbles(codes), R)
        fidx.append(fi)
    # Section 4.2: quantized tables barely change what float ADC returns (ordering check only)
    assert O.overlap_at_r(idx_np(idx), np.stack(fidx)) > 0.6


@pytest.mark.parametrize("m", [8, 16, 32, 64])
@pytest.mark.parametrize("n", [0, 1, 99, 100, 4097, 100_003])
def test_scan_topk_shapes_and_ragged_tails(Q, m, n):
    rng = np.random.default_rng(m * 1000003 + n)
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    qluts = rng.integers(0, 40, size=(3, m, 16)).astype(np.uint8)
    R = 100
    g = to_gpu(codes) if n else to_gpu(np.zeros((1, m // 2), dtype=np.uint8))
    gi, gd = gpu_topk(Q, g, qluts, R, n=n)
    for iq in range(3):
        wi, wd = oracle_topk(codes, qluts[iq], R)
        assert np.array_equal(gi[iq], wi), (m, n, iq)
        assert np.array_equal(gd[iq], wd), (m, n, iq)


@pytest.mark.parametrize("kind", ["zeros", "saturated", "binary", "wide", "one_hot_far"])
@pytest.mark.parametrize("R", [1, 100, 1024])
def test_scan_topk_ties_and_saturation(Q, kind, R):
    """Degenerate tables: every sum equal, every sum saturated, two-valued sums, sums that overflow a byte."""
    rng = np.random.default_rng(42)
    n, m = 50_021, 16
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    codes[1000:1200] = codes[7]  # duplicate codes: equal sums at distinct indices
    if kind == "zeros":
        ql = np.zeros((m, 16), dtype=np.uint8)
    elif kind == "saturated":
        ql = np.full((m, 16), 255, dtype=np.uint8)
    elif kind == "binary":
        ql = rng.integers(0, 2, size=(m, 16)).astype(np.uint8)
    elif kind == "wide":
        ql = rng.integers(0, 256, size=(m, 16)).astype(np.uint8)
    else:
        ql = np.full((m, 16), 200, dtype=np.uint8)
        ql[:, 3] = 0
    gi, gd = gpu_topk(Q, to_gpu(codes), ql[None], R)
    wi, wd = oracle_topk(codes, ql, R)
    assert np.array_equal(gi[0], wi) and np.array_equal(gd[0], wd)


def test_scan_topk_adversarial_order(Q):
    """Sums strictly decreasing with the index: every code beats all earlier ones."""
    n, m = 70_000, 16
    codes = np.zeros((n, m // 2), dtype=np.uint8)
    lvl = (np.arange(n)[::-1] * 240 // n).astype(np.int64)  # 239 .. 0
    # component 0 carries lvl % 16, component 1 carries lvl // 16
    codes[:, 0] = (lvl % 16) | ((lvl // 16) << 4)
    ql = np.zeros((m, 16), dtype=np.uint8)
    ql[0] = np.arange(16)
    ql[1] = np.arange(16) * 16
    gi, gd = gpu_topk(Q, to_gpu(codes), ql[None], 100)
    wi, wd = oracle_topk(codes, ql, 100)
    assert np.array_equal(gi[0], wi) and np.array_equal(gd[0], wd)


def test_scan_topk_is_deterministic_and_launch_shape_free(Q, O):
    c = config1()
    codes, cb = c["codes"], c["codebooks"]
    qlut = O.quick_adc_tables(cb, c["queries"][0], codes, 200, 100)["qlut"]
    g = to_gpu(codes)
    ref = gpu_topk(Q, g, qlut[None], 100)
    saved = {k: os.environ.get(k) for k in ("QADC_SCAN_NT", "QADC_SCAN_WGS")}
    try:
        for nt, wgs in [("256", "1"), ("512", "7"), ("1024", "256"), ("1024", "3"), ("256", "4096"),
                        ("512", "1024")]:
            os.environ["QADC_SCAN_NT"], os.environ["QADC_SCAN_WGS"] = nt, wgs
            for _ in range(2):
                got = gpu_topk(Q, g, qlut[None], 100)
                assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1]), (nt, wgs)
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
    wi, wd = oracle_topk(codes, qlut, 100)
    assert np.array_equal(ref[0][0], wi) and np.array_equal(ref[1][0], wd)


# ------------------------------------------------------------------ encode

@pytest.mark.parametrize("shape", [(128, 16, 16), (128, 32, 16), (96, 8, 256), (96, 16, 16)])
def test_pq_encode_matches_oracle(Q, O, shape):
    """GPU encode (float32 distances) against the oracle (float64): identical except where the two
    best centroids are closer than float32 rounding can tell apart."""
    from oracle import cref
    from workloads import MixtureSpec, mixture_vectors, SEED_BASE, SEED_TRAIN
    d, m, k = shape
    spec = MixtureSpec(d=d)
    x = mixture_vectors(spec, SEED_BASE, 0, 20_011)
    rng = np.random.default_rng(d + m + k)
    train = mixture_vectors(spec, SEED_TRAIN, 0, 4000)
    rows = rng.permutation(4000)[:k]
    dsub = d // m
    cb = np.stack([train[rows, j * dsub:(j + 1) * dsub] for j in range(m)]).astype(np.float32)
    x[:k] = train[rows]  # vectors that sit exactly on centroids
    want = cref.pq_encode(x, cb)
    got = Q.qadc_pq_encode(to_gpu(cb), to_gpu(x)).cpu().numpy()
    assert got.shape == want.shape
    wc = O.unpack_nibbles(want) if k == 16 else want
    gc = O.unpack_nibbles(got) if k == 16 else got
    bad = np.argwhere(wc != gc)
    assert len(bad) < 1e-4 * wc.size
    for r, j in bad:
        dist = O.sq_l2(x[r:r + 1, j * dsub:(j + 1) * dsub], cb[j])[0]
        assert abs(dist[wc[r, j]] - dist[gc[r, j]]) <= 1e-5 * dist[wc[r, j]]


def test_workspace_is_left_clean_between_calls(Q, O):
    """One workspace, cleared once, then reused by calls of different sizes and tables."""
    import torch
    c = config1()
    codes, cb = c["codes"], c["codebooks"]
    g = to_gpu(codes)
    R = 100
    nbytes = Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, len(codes), 16, 4, R)
    ws = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device="cuda:0")  # dirty on purpose
    Q.qadc_workspace_init(ws)
    rng = np.random.default_rng(8)
    for it, (n, nq) in enumerate([(100_000, 4), (5_000, 1), (100_000, 2), (77, 3), (60_001, 4)]):
        if it % 2 == 0:
            ql = np.stack([O.quick_adc_tables(cb, y, codes, 200, R)["qlut"] for y in c["queries"][:nq]])
        else:
            ql = rng.integers(0, 30, size=(nq, 16, 16)).astype(np.uint8)
        idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, g, to_gpu(ql), R, workspace=ws, n=n)
        torch.cuda.synchronize()
        for iq in range(nq):
            wi, wd = oracle_topk(codes[:n], ql[iq], R)
            assert np.array_equal(idx_np(idx)[iq], wi), (it, iq)
            assert np.array_equal(dist[iq].cpu().numpy(), wd), (it, iq)


@pytest.mark.parametrize("kind", ["mixture", "zeros", "decreasing", "binary", "global_offset"])
def test_scan_topk_large_enough_for_the_seed_kernel(Q, O, kind):
    """Databases long enough for the sampling kernel: good bound, useless bound (every code ties:
    the barrier-free pass overflows and the careful pass takes over), adversarial order."""
    rng = np.random.default_rng(77)
    n, m, R = 700_003, 16, 100
    if kind == "mixture":
        c = config1()
        reps = -(-n // len(c["codes"]))
        codes = np.tile(c["codes"], (reps, 1))[:n].copy()
        codes[::7] = rng.integers(0, 256, size=codes[::7].shape, dtype=np.uint8)
        ql = O.quick_adc_tables(c["codebooks"], c["queries"][3], codes, 200, R)["qlut"]
    elif kind == "zeros":
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        ql = np.zeros((m, 16), dtype=np.uint8)
    elif kind == "binary":
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        ql = rng.integers(0, 2, size=(m, 16)).astype(np.uint8)
    elif kind == "global_offset":  # every sum >= 16 * 9: the low bins of the histogram stay empty
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        ql = (9 + rng.integers(0, 6, size=(m, 16))).astype(np.uint8)
    else:
        codes = np.zeros((n, m // 2), dtype=np.uint8)
        lvl = (np.arange(n)[::-1] * 240 // n).astype(np.int64)
        codes[:, 0] = (lvl % 16) | ((lvl // 16) << 4)
        ql = np.zeros((m, 16), dtype=np.uint8)
        ql[0] = np.arange(16)
        ql[1] = np.arange(16) * 16
    gi, gd = gpu_topk(Q, to_gpu(codes), ql[None], R)
    wi, wd = oracle_topk(codes, ql, R)
    assert np.array_equal(gi[0], wi) and np.array_equal(gd[0], wd)


# ------------------------------------------------------- float ADC (Alg. 1)

def gpu_topk_f32(Q, variant, codes_gpu, luts, R, n=None):
    import torch
    idx, dist = Q.qadc_scan_topk(variant, codes_gpu, to_gpu(luts), R, n=n)
    torch.cuda.synchronize()
    return idx_np(idx), dist.cpu().numpy()


def test_float_adc_scan_config1_bit_exact(Q, O):
    """Alg. 1 on 4-bit codes: float32 sums in increasing j on both sides -> identical bits."""
    from oracle import cref
    c = config1()
    luts = O.build_luts(c["codebooks"], c["queries"])
    gi, gd = gpu_topk_f32(Q, Q.QADC_F32_4BIT, to_gpu(c["codes"]), luts, 100)
    wi, wd = cref.scan_topk_f32(c["codes"], luts, 100)
    assert np.array_equal(gi, wi)
    assert np.array_equal(gd.view(np.uint32), wd.view(np.uint32))


def test_float_adc_scan_8bit_codes(Q, O):
    """Config-5-shaped baseline: d=96, m=8 x 256 centroids, float tables of 8 KiB."""
    from oracle import cref
    from workloads import MixtureSpec, mixture_vectors, SEED_BASE, SEED_TRAIN, SEED_QUERY
    spec = MixtureSpec(d=96)
    train = mixture_vectors(spec, SEED_TRAIN, 0, 3000)
    rows = np.random.default_rng(0).permutation(3000)[:256]
    cb = np.stack([O.kmeans_lloyd(train[:, j * 12:(j + 1) * 12], rows, 2)[0] for j in range(8)])
    base = mixture_vectors(spec, SEED_BASE, 0, 60_007)
    codes = cref.pq_encode(base, cb)
    queries = mixture_vectors(spec, SEED_QUERY, 0, 5)
    luts = O.build_luts(cb, queries)
    assert luts.shape == (5, 8, 256)
    g_luts = Q.qadc_build_luts(to_gpu(cb), to_gpu(queries)).cpu().numpy()
    np.testing.assert_allclose(g_luts, luts, rtol=1e-4)
    gi, gd = gpu_topk_f32(Q, Q.QADC_F32_8BIT, to_gpu(codes), luts, 100)
    wi, wd = cref.scan_topk_f32(codes, luts, 100)
    assert np.array_equal(gi, wi)
    assert np.array_equal(gd.view(np.uint32), wd.view(np.uint32))


@pytest.mark.parametrize("variant_m", [("4", 8), ("4", 16), ("4", 32), ("4", 64),
                                       ("8", 4), ("8", 8), ("8", 16), ("8", 32)])
@pytest.mark.parametrize("n", [0, 37, 2049, 30_011])
def test_float_adc_scan_shapes(Q, variant_m, n):
    from oracle import cref
    bits, m = variant_m
    k = 16 if bits == "4" else 256
    variant = Q.QADC_F32_4BIT if bits == "4" else Q.QADC_F32_8BIT
    row = m // 2 if k == 16 else m
    rng = np.random.default_rng(m * 131 + n + k)
    codes = rng.integers(0, 256, size=(n, row), dtype=np.uint8)
    luts = rng.uniform(0, 1000, size=(2, m, k)).astype(np.float32)
    luts[1] = np.floor(luts[1] / 250)  # few distinct values: many exact ties
    g = to_gpu(codes) if n else to_gpu(np.zeros((1, row), dtype=np.uint8))
    gi, gd = gpu_topk_f32(Q, variant, g, luts, 64, n=n)
    wi, wd = cref.scan_topk_f32(codes, luts, 64)
    assert np.array_equal(gi, wi), (bits, m, n)
    assert np.array_equal(gd.view(np.uint32), wd.view(np.uint32)), (bits, m, n)


@pytest.mark.parametrize("bits", ["4", "8"])
@pytest.mark.parametrize("kind", ["mixture", "constant", "far_head", "decreasing", "ties"])
def test_float_adc_scan_large_enough_for_the_seed_kernel(Q, O, bits, kind):
    """Float scan with the sampled bound: a good bound, a bound with no resolution (every distance
    equal), a bound placed by an unrepresentative head (the barrier-free pass overflows and the
    careful pass takes over), decreasing distances, and many exact ties at the R-th place."""
    from oracle import cref
    rng = np.random.default_rng(5 + len(kind))
    n, R = 700_003, 100
    m, k = (16, 16) if bits == "4" else (8, 256)
    row = m // 2 if k == 16 else m
    variant = Q.QADC_F32_4BIT if bits == "4" else Q.QADC_F32_8BIT
    codes = rng.integers(0, 256, size=(n, row), dtype=np.uint8)
    if kind == "mixture":
        luts = rng.gamma(2.0, 50.0, size=(2, m, k)).astype(np.float32)
    elif kind == "constant":
        luts = np.full((2, m, k), 3.25, dtype=np.float32)
    elif kind == "far_head":
        luts = rng.uniform(0, 100, size=(2, m, k)).astype(np.float32)
        luts[:, 0, :] += np.linspace(0, 5000, k, dtype=np.float32)
        hi = 255 if k == 256 else 0xff
        codes[:1024, 0] = hi   # the head only holds the largest entry of table 0 (and 1)
        codes[1024:, 0] = 0
    elif kind == "decreasing":
        luts = np.zeros((2, m, k), dtype=np.float32)
        luts[:, 0, :] = np.arange(k, dtype=np.float32) * (1.0 if k == 256 else 16.0)
        if k == 16:
            luts[:, 1, :] = np.arange(k, dtype=np.float32)
        codes[:] = 0
        codes[:, 0] = (np.arange(n)[::-1] * 250 // n).astype(np.uint8)
    else:
        luts = rng.integers(0, 3, size=(2, m, k)).astype(np.float32)
    gi, gd = gpu_topk_f32(Q, variant, to_gpu(codes), luts, R)
    wi, wd = cref.scan_topk_f32(codes, luts, R)
    assert np.array_equal(gi, wi), (bits, kind)
    assert np.array_equal(gd.view(np.uint32), wd.view(np.uint32)), (bits, kind)


@pytest.mark.parametrize("shape", [(128, 16, 16, 6000, 4), (96, 8, 256, 3000, 2)])
def test_pq_train_matches_oracle(Q, O, shape):
    """GPU k-means (float64 assignment, deterministic float64 means) against the oracle's Lloyd."""
    from workloads import MixtureSpec, mixture_vectors, kmeans_init_rows, SEED_TRAIN
    d, m, k, n, iters = shape
    train = mixture_vectors(MixtureSpec(d=d), SEED_TRAIN, 0, n)
    rows = kmeans_init_rows(n, k)
    want = O.pq_train(train, m, k, iters, rows)
    got = Q.qadc_pq_train(to_gpu(train), m, k, to_gpu(rows), iters).cpu().numpy()
    np.testing.assert_allclose(got, want, rtol=2e-6, atol=1e-5)
    again = Q.qadc_pq_train(to_gpu(train), m, k, to_gpu(rows), iters).cpu().numpy()
    assert np.array_equal(got, again)


# ------------------------------------------------------------- qadc_search

@pytest.mark.parametrize("n", [100_000, 700_003])
@pytest.mark.parametrize("mode_nbins", [(0, 255), (1, 255), (0, 127)])
def test_search_equals_the_three_call_chain_and_the_oracle(Q, O, n, mode_nbins):
    """qadc_search = build_luts + quantize_luts + scan_topk, bit for bit (small databases take the
    separate kernels, large ones the fused prepare kernel), and the oracle replays its integer part."""
    import torch
    mode, nbins = mode_nbins
    c = config1()
    cb, queries = c["codebooks"], c["queries"][:6]
    reps = -(-n // len(c["codes"]))
    codes = np.tile(c["codes"], (reps, 1))[:n].copy()
    if reps > 1:
        rng = np.random.default_rng(n)
        codes[100_000:] ^= rng.integers(0, 256, size=codes[100_000:].shape, dtype=np.uint8) & 0x11
    R, init = 100, 200
    g_codes, g_cb, g_q = to_gpu(codes), to_gpu(cb), to_gpu(queries)
    ql_out = torch.empty((len(queries), 16, 16), dtype=torch.uint8, device="cuda:0")
    si, sd = Q.qadc_search(g_cb, g_q, g_codes, R, init, nbins, mode, qluts_out=ql_out)
    luts = Q.qadc_build_luts(g_cb, g_q)
    ql, _, _, _ = Q.qadc_quantize_luts(luts, g_codes[:init], R, nbins, mode)
    ci, cd = Q.qadc_scan_topk(Q.QADC_U8_4BIT, g_codes, ql, R, nbins)
    torch.cuda.synchronize()
    assert torch.equal(ql_out, ql)
    assert torch.equal(si, ci) and torch.equal(sd, cd)
    h_ql = ql_out.cpu().numpy()
    for iq in range(len(queries)):
        wi, wd = oracle_topk(codes, h_ql[iq], R, nbins)
        assert np.array_equal(idx_np(si)[iq], wi) and np.array_equal(sd[iq].cpu().numpy(), wd)
        t = O.quick_adc_tables(cb, queries[iq], codes, init, R, nbins, mode)
        assert np.abs(h_ql[iq].astype(int) - t["qlut"].astype(int)).max() <= 1


def test_search_large_init_and_other_code_sizes(Q, O):
    """init above 1024 (radix select instead of rank counting) and m = 8 / 32 in the fused kernel."""
    import torch
    from workloads import MixtureSpec, mixture_vectors, SEED_QUERY
    rng = np.random.default_rng(31)
    for m, init in [(8, 1500), (32, 1000), (16, 3000)]:
        d = 128
        cb = rng.uniform(0, 255, size=(m, 16, d // m)).astype(np.float32)
        n = 600_011
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        queries = mixture_vectors(MixtureSpec(d=d), SEED_QUERY, 0, 3)
        g_codes, g_cb, g_q = to_gpu(codes), to_gpu(cb), to_gpu(queries)
        ql_out = torch.empty((3, m, 16), dtype=torch.uint8, device="cuda:0")
        si, sd = Q.qadc_search(g_cb, g_q, g_codes, 100, init, qluts_out=ql_out)
        luts = Q.qadc_build_luts(g_cb, g_q)
        ql, _, _, _ = Q.qadc_quantize_luts(luts, g_codes[:init], 100)
        torch.cuda.synchronize()
        assert torch.equal(ql_out, ql), (m, init)
        h_ql = ql_out.cpu().numpy()
        for iq in range(3):
            wi, wd = oracle_topk(codes, h_ql[iq], 100)
            assert np.array_equal(idx_np(si)[iq], wi) and np.array_equal(sd[iq].cpu().numpy(), wd), (m, init)


# ----------------------------------------------------- query-tiled scan

@pytest.mark.parametrize("m", [8, 16, 32, 64])
def test_scan_topk_query_batches_share_code_reads(Q, O, m):
    """Batches of >= 8 queries on a long database go through the query-tiled kernel (8 queries per
    workgroup); queries whose bound is useless (all sums tie) fall back to the single-query kernel."""
    rng = np.random.default_rng(m)
    n, R, nq = 500_009, 100, 21
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    codes[::5] = codes[3]  # duplicates: ties at distinct indices
    qluts = rng.integers(0, 1 + 255 // m, size=(nq, m, 16)).astype(np.uint8)
    qluts[4] = 0                                   # every sum ties: redo path
    qluts[9] = rng.integers(0, 2, size=(m, 16))    # two-valued entries: heavy ties
    qluts[13] = 255                                # everything saturates
    qluts[17, :, :8] = 0                           # many zero sums
    gi, gd = gpu_topk(Q, to_gpu(codes), qluts, R)
    for iq in range(nq):
        wi, wd = oracle_topk(codes, qluts[iq], R)
        assert np.array_equal(gi[iq], wi), (m, iq)
        assert np.array_equal(gd[iq], wd), (m, iq)


@pytest.mark.parametrize("m", [8, 16, 32, 64])
def test_scan_topk_query_groups_by_bound(Q, O, m):
    """Groups of 16 queries are scanned by one of two kernels according to the largest bound in
    the group (byte lanes for bounds up to 126, else 16-bit lanes): a batch with groups of each
    kind, bounds right at the limit, mixed groups and a partial last group."""
    rng = np.random.default_rng(100 + m)
    n, R = 300_007, 100
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    groups = []
    for base in (0, 60, 62, 63, 100, 126, 127, 200):   # smallest possible sum of each query
        ql = rng.integers(0, 3, size=(m, 16)).astype(np.uint8)
        ql[0] += base                                   # every sum of this query is >= base
        groups.append(ql)
    qluts = []
    for gsel in ([0, 0, 1, 1], [2, 2, 3, 3], [4, 4, 5, 5], [6, 7, 7, 6], [0, 3, 5, 7]):
        for i in range(16 if len(qluts) < 64 else 5):
            qluts.append(groups[gsel[i % 4]].copy())
    qluts = np.stack(qluts)                             # 64 + 5 queries
    gi, gd = gpu_topk(Q, to_gpu(codes), qluts, R)
    checked = {}
    for iq in range(len(qluts)):
        key = qluts[iq].tobytes()
        if key not in checked:
            checked[key] = oracle_topk(codes, qluts[iq], R)
        wi, wd = checked[key]
        assert np.array_equal(gi[iq], wi), (m, iq)
        assert np.array_equal(gd[iq], wd), (m, iq)


@pytest.mark.parametrize("m", [8, 16, 32, 64])
@pytest.mark.parametrize("nq,R,nbins", [(130, 100, 255), (97, 1000, 127), (256, 10, 255), (40, 100, 255)])
def test_scan_topk_large_batches_on_the_matrix_cores(Q, O, m, nq, R, nbins):
    """Batches of 4-bit codes from 16 queries up (32 for the shortest codes) are scanned as one-hot matrix
    products, 32 or 64 queries per wavefront: full and partial sets of queries, a ragged database
    tail, tables that tie heavily, saturate, exceed nbins or are all zero (those queries overflow
    their lists and are redone one by one).  Indices and sums equal the plain-C scan bit for bit."""
    from oracle import cref
    rng = np.random.default_rng(m * 1000 + nq)
    n = 600_011
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    codes[::7] = codes[5]                               # duplicates: ties at distinct indices
    qluts = rng.integers(0, 1 + 255 // m, size=(nq, m, 16)).astype(np.uint8)
    qluts[3] = 0                                        # every sum ties
    qluts[11] = rng.integers(0, 2, size=(m, 16))        # two-valued entries
    qluts[33] = 255                                     # everything saturates
    qluts[64 % nq] = rng.integers(100, 256, size=(m, 16))    # entries beyond nbins = 127
    qluts[70 % nq, :, :8] = 0                           # many zero sums
    qluts[nq - 1] = rng.integers(0, 4, size=(m, 16))
    wi, wd = cref.scan_topk_u8(codes, qluts, R, nbins)
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, to_gpu(codes), to_gpu(qluts), R, nbins)
    assert np.array_equal(idx_np(idx), wi)
    assert np.array_equal(dist.cpu().numpy(), wd)


def test_scan_topk_random_large_batches_against_c_twin(Q, O):
    """Twenty-four seeded draws of (n, m, queries, R, nbins, table range) with 33 to 300 queries over
    databases long enough for the sampled bound: every form of the matrix-core kernel (32, 64, 128
    queries per wavefront), partial last sets, sizes that end inside a 32-code step, tables that
    saturate always, sometimes or never.  Indices and sums equal the plain-C scan bit for bit."""
    from oracle import cref
    rng = np.random.default_rng(4242)
    for it in range(24):
        m = int(rng.choice([8, 16, 32, 64]))
        n = int(rng.integers(540_000, 700_000))
        nq = int(rng.choice([33, 64, 65, 100, 128, 150, 257, 300]))
        R = int(rng.choice([1, 10, 100, 500]))
        nbins = int(rng.choice([255, 127, 31]))
        hi = int(rng.choice([3, 20, 90, 256]))
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        qluts = rng.integers(0, hi, size=(nq, m, 16)).astype(np.uint8)
        wi, wd = cref.scan_topk_u8(codes, qluts, R, nbins)
        idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, to_gpu(codes), to_gpu(qluts), R, nbins)
        assert np.array_equal(idx_np(idx), wi), (it, n, m, nq, R, nbins, hi)
        assert np.array_equal(dist.cpu().numpy(), wd), (it, n, m, nq, R, nbins, hi)


@pytest.mark.parametrize("knobs", [{"QADC_TILED_MFMA": "0"}, {"QADC_MFMA_MIN_Q2": "100000", "QADC_MFMA_MIN_Q4": "100000"},
                                   {"QADC_MFMA_MIN_Q": "8", "QADC_MFMA_MIN_Q2": "8", "QADC_MFMA_MIN_Q4": "8"},
                                   {"QADC_MFMA_WAVES": "300"}, {"QADC_TILED_SEED": "0"}, {"QADC_TILED": "0"}])
def test_kernel_choice_knobs_never_change_results(Q, O, monkeypatch, knobs):
    """The tuning variables pick among equivalent kernels and launch shapes: the vector-ALU kernels
    instead of the matrix-core one, each of its forms (32, 64, 128 queries per wavefront) forced on
    batches that would not take it, few long chunks, the per-query sample, no query tiling at all."""
    from oracle import cref
    for k, v in knobs.items():
        monkeypatch.setenv(k, v)
    rng = np.random.default_rng(99)
    for m, nq in ((16, 130), (8, 300), (64, 40)):
        n, R = 560_003, 100
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        qluts = rng.integers(0, 1 + 255 // m, size=(nq, m, 16)).astype(np.uint8)
        qluts[1] = 0
        wi, wd = cref.scan_topk_u8(codes, qluts, R, 255)
        idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, to_gpu(codes), to_gpu(qluts), R)
        assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd), (knobs, m, nq)


def test_scan_topk_a_thousand_queries_in_one_call(Q, O):
    """A call with far more queries than one launch takes (the workspace bounds the queries per
    launch): full sub-batches and a last short one."""
    from oracle import cref
    rng = np.random.default_rng(5)
    n, m, nq, R = 600_011, 16, 1003, 10
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    qluts = rng.integers(0, 17, size=(nq, m, 16)).astype(np.uint8)
    wi, wd = cref.scan_topk_u8(codes, qluts, R, 255)
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, to_gpu(codes), to_gpu(qluts), R)
    assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd)


def test_scan_topk_batch_with_tables_at_a_4_byte_offset(Q, O):
    """Tables that are only 4-byte aligned (the documented minimum) in a batch large enough for the
    matrix-core kernel, whose operands are 16-byte loads: the batch takes the other kernels."""
    import torch
    from oracle import cref
    rng = np.random.default_rng(77)
    n, m, nq, R = 300_011, 32, 70, 100
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    qluts = rng.integers(0, 9, size=(nq, m, 16)).astype(np.uint8)
    buf = torch.zeros((qluts.size + 64,), dtype=torch.uint8, device="cuda:0")
    off = 4 + (-buf.data_ptr()) % 16            # address = 4 mod 16
    g = buf[off:off + qluts.size].view(nq, m, 16)
    g.copy_(to_gpu(qluts))
    assert g.data_ptr() % 16 == 4
    wi, wd = cref.scan_topk_u8(codes, qluts, R, 255)
    idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, to_gpu(codes), g, R)
    assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd)


def test_search_batch_config1_shaped(Q, O):
    """qadc_search on a batch of 16 mixture queries over a long database (fused prepare kernel +
    query-tiled scan) against the oracle's replay of the integer part and its own tables."""
    import torch
    c = config1()
    n = 800_000
    reps = -(-n // len(c["codes"]))
    rng = np.random.default_rng(3)
    codes = np.tile(c["codes"], (reps, 1))[:n].copy()
    codes[100_000:] ^= rng.integers(0, 256, size=codes[100_000:].shape, dtype=np.uint8) & 0x33
    ql_out = torch.empty((16, 16, 16), dtype=torch.uint8, device="cuda:0")
    si, sd = Q.qadc_search(to_gpu(c["codebooks"]), to_gpu(c["queries"]), to_gpu(codes), 100, 200,
                           qluts_out=ql_out)
    torch.cuda.synchronize()
    h_ql = ql_out.cpu().numpy()
    for iq in range(16):
        t = O.quick_adc_tables(c["codebooks"], c["queries"][iq], codes, 200, 100)
        assert np.abs(h_ql[iq].astype(int) - t["qlut"].astype(int)).max() <= 1
        wi, wd = oracle_topk(codes, h_ql[iq], 100)
        assert np.array_equal(idx_np(si)[iq], wi) and np.array_equal(sd[iq].cpu().numpy(), wd)


def test_scan_topk_random_shapes_against_c_twin(Q, O):
    """Forty seeded draws of (n, m, queries, R, nbins, table range): sizes that end inside a tile, a
    16-byte piece or below R; tables that saturate always, sometimes or never; unseeded, seeded and
    query-tiled launches.  Indices and sums equal the plain-C scan bit for bit."""
    from oracle import cref
    rng = np.random.default_rng(2024)
    for it in range(40):
        m = int(rng.choice([8, 16, 32, 64]))
        big = it % 4 == 0
        n = int(rng.integers(260_000, 420_000)) if big else int(rng.integers(1, 40_000))
        nq = int(rng.choice([1, 2, 5, 8, 11, 17])) if not big else int(rng.choice([1, 3, 8, 16]))
        R = int(rng.choice([1, 7, 100, 257, 1024]))
        nbins = int(rng.choice([255, 127, 31]))
        hi = int(rng.choice([3, 20, 90, 256]))
        codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
        qluts = rng.integers(0, hi, size=(nq, m, 16)).astype(np.uint8)
        wi, wd = cref.scan_topk_u8(codes, qluts, R, nbins)
        idx, dist = Q.qadc_scan_topk(Q.QADC_U8_4BIT, to_gpu(codes), to_gpu(qluts), R, nbins)
        assert np.array_equal(idx_np(idx), wi), (it, n, m, nq, R, nbins, hi)
        assert np.array_equal(dist.cpu().numpy(), wd), (it, n, m, nq, R, nbins, hi)


@pytest.mark.parametrize("m,n,nq", [(8, 300_007, 8), (8, 300_007, 19), (4, 700_000, 16), (16, 280_000, 9)])
def test_float_scan_of_8bit_codes_in_query_batches(Q, O, m, n, nq):
    """Batches of eight queries and more over 8-bit codes take the query-tiled float kernel: indices
    and float32 distances equal the plain-C scan bit for bit (same order of additions)."""
    from oracle import cref
    rng = np.random.default_rng(m + n + nq)
    codes = rng.integers(0, 256, size=(n, m), dtype=np.uint8)
    luts = (rng.gamma(2.0, 50.0, size=(nq, m, 256))).astype(np.float32)
    R = 100
    wi, wd = cref.scan_topk_f32(codes, luts, R)
    idx, dist = Q.qadc_scan_topk(Q.QADC_F32_8BIT, to_gpu(codes), to_gpu(luts), R)
    assert np.array_equal(idx_np(idx), wi)
    assert np.array_equal(dist.cpu().numpy(), wd)


def test_float_scan_batches_with_ties_and_useless_bounds(Q, O):
    """All codes equal (every distance ties: the bound lets everything through, the lists of the
    tiled kernel overflow and each query is redone alone) and tables with a few huge entries."""
    from oracle import cref
    rng = np.random.default_rng(12)
    m, n, nq, R = 8, 290_000, 10, 100
    luts = rng.gamma(2.0, 50.0, size=(nq, m, 256)).astype(np.float32)
    codes = np.full((n, m), 7, dtype=np.uint8)
    wi, wd = cref.scan_topk_f32(codes, luts, R)
    idx, dist = Q.qadc_scan_topk(Q.QADC_F32_8BIT, to_gpu(codes), to_gpu(luts), R)
    assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd)
    codes = rng.integers(0, 256, size=(n, m), dtype=np.uint8)
    luts[:, :, ::17] = 1e30
    wi, wd = cref.scan_topk_f32(codes, luts, R)
    idx, dist = Q.qadc_scan_topk(Q.QADC_F32_8BIT, to_gpu(codes), to_gpu(luts), R)
    assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd)


@pytest.mark.parametrize("m,n,nq", [(16, 300_007, 8), (16, 300_007, 19), (8, 700_000, 16), (32, 280_000, 9)])
def test_float_scan_of_4bit_codes_in_query_batches(Q, O, m, n, nq):
    """Batches of eight queries and more over 4-bit codes take the query-tiled float kernel too (two
    table entries per code byte, added in increasing component order): indices and float32
    distances equal the plain-C scan of Alg. 1 bit for bit."""
    from oracle import cref
    rng = np.random.default_rng(m + n + nq)
    codes = rng.integers(0, 256, size=(n, m // 2), dtype=np.uint8)
    luts = (rng.gamma(2.0, 50.0, size=(nq, m, 16))).astype(np.float32)
    R = 100
    wi, wd = cref.scan_topk_f32(codes, luts, R)
    idx, dist = Q.qadc_scan_topk(Q.QADC_F32_4BIT, to_gpu(codes), to_gpu(luts), R)
    assert np.array_equal(idx_np(idx), wi)
    assert np.array_equal(dist.cpu().numpy(), wd)
    # ties: every code equal, every list of the tiled kernel overflows, each query is redone alone
    codes[:] = 0x5a
    wi, wd = cref.scan_topk_f32(codes, luts, R)
    idx, dist = Q.qadc_scan_topk(Q.QADC_F32_4BIT, to_gpu(codes), to_gpu(luts), R)
    assert np.array_equal(idx_np(idx), wi) and np.array_equal(dist.cpu().numpy(), wd)
