"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the GPU or the HIP library.  Each test is chosen so that
a plausible slip in the oracle (dropped term, wrong nibble, transposed operand,
off-by-one rank, wrong tie order) makes it fail.
"""

import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist

from oracle import qadc_oracle as O
from oracle import cref

HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------ printed sizes

def _golden_rows():
    rows = []
    with open(os.path.join(HERE, "golden", "paper_sizes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                w = line.split()
                rows.append((w[0], int(w[1]), int(w[2]), int(w[3])))
    return rows


@pytest.mark.parametrize("what,m,b,value", _golden_rows())
def test_sizes_printed_in_paper(what, m, b, value):
    fn = {"table_bytes": O.table_bytes, "code_bits": O.code_bits}[what]
    assert fn(m, 2 ** b) == value


def test_ivf_memory_128bit_billion():
    # Section 2.2: 4 bytes of index overhead per vector; Section 4.6: 128-bit
    # codes of 10^9 vectors occupy 20 GB.
    per_vec = O.code_bits(32, 16) // 8 + 4
    assert per_vec * 10 ** 9 == 20 * 10 ** 9


# ------------------------------------------------------------------ Eq. (1)

def test_luts_match_cdist(tiny_pq):
    cb, q = tiny_pq["codebooks"], tiny_pq["queries"]
    luts = O.build_luts(cb, q)
    m, k, dsub = cb.shape
    assert luts.shape == (len(q), m, k) and luts.dtype == np.float32
    for j in range(m):
        ref = cdist(q[:, j * dsub:(j + 1) * dsub].astype(np.float64),
                    cb[j].astype(np.float64), "sqeuclidean")
        np.testing.assert_allclose(luts[:, j, :], ref, rtol=1e-6)
    # a query equal to a centroid tuple has a zero in every table, at that centroid
    y = O.pq_decode(np.arange(16, dtype=np.uint8)[None, :] % 16, cb)
    l0 = O.build_luts(cb, y)[0]
    assert np.all(l0[np.arange(16), np.arange(16) % 16] == 0)


def test_luts_residual_is_shifted_query(tiny_pq):
    cb, q = tiny_pq["codebooks"], tiny_pq["queries"]
    base = tiny_pq["base"][:len(q)]
    a = O.build_luts(cb, q, base)
    b = O.build_luts(cb, (q.astype(np.float64) - base).astype(np.float64))
    np.testing.assert_allclose(a, b, rtol=1e-6)
    assert not np.allclose(a, O.build_luts(cb, q))


# ----------------------------------------------------------- encode / layout

def test_encode_is_argmin_of_cdist(tiny_pq):
    cb, x = tiny_pq["codebooks"], tiny_pq["base"][:3000]
    comps = O.pq_encode(x, cb)
    m, k, dsub = cb.shape
    for j in range(m):
        ref = np.argmin(cdist(x[:, j * dsub:(j + 1) * dsub].astype(np.float64),
                              cb[j].astype(np.float64), "sqeuclidean"), axis=1)
        assert np.array_equal(comps[:, j], ref)


def test_nibble_layout():
    # Fig. 2 / Alg. 2: low nibble = component 2j (reached by the 0x0f mask),
    # high nibble = component 2j+1 (reached after the 4-bit right shift).
    comps = np.array([[1, 2, 3, 4], [15, 0, 0, 15]], dtype=np.uint8)
    codes = O.pack_nibbles(comps)
    assert codes.tolist() == [[0x21, 0x43], [0x0F, 0xF0]]
    rng = np.random.default_rng(5)
    c = rng.integers(0, 16, size=(1000, 32), dtype=np.uint8)
    assert np.array_equal(O.unpack_nibbles(O.pack_nibbles(c)), c)
    assert O.pack_nibbles(c).shape == (1000, 16)


def test_transposed_layout_by_hand_and_block_scan():
    # Fig. 2b: a block of 16 codes a..p becomes m/2 rows; row j = byte j of a, b, .. p.
    # Hand-made block, m = 4: code c has bytes (0x10 + c, 0xA0 + c).
    codes = np.array([[0x10 + c, 0xA0 + c] for c in range(16)], dtype=np.uint8)
    packed = O.pack_transposed(codes)
    assert packed.tolist() == [0x10 + c for c in range(16)] + [0xA0 + c for c in range(16)]
    # a ragged list: 37 codes of m = 16 -> three blocks of 16 * 8 bytes, zero filled
    rng = np.random.default_rng(11)
    codes = rng.integers(0, 256, size=(37, 8), dtype=np.uint8)
    packed = O.pack_transposed(codes)
    assert len(packed) == O.transposed_bytes(37, 16) == 3 * 128
    assert packed[2 * 128 + 0 * 16 + 4] == codes[36, 0] and packed[2 * 128 + 7 * 16 + 4] == codes[36, 7]
    assert not packed.reshape(3, 8, 16)[2, :, 5:].any()
    assert packed[1 * 128 + 3 * 16 + 9] == codes[25, 3]        # block 1, row 3, column 9
    assert np.array_equal(O.unpack_transposed(packed, 37, 16), codes)
    # Alg. 2 run over blocks and rows gives the sums of the scan over the standard layout,
    # and the plain definition min(n, sum of the 16 looked-up entries)
    qlut = rng.integers(0, 90, size=(16, 16), dtype=np.uint8)
    for nbins in (255, 127):
        got = O.scan_blocks_transposed(qlut, packed, 37, nbins)
        assert np.array_equal(got, O.scan_saturating(qlut, codes, nbins))
        comps = O.unpack_nibbles(codes)
        brute = [min(nbins, sum(int(qlut[j][comps[i, j]]) for j in range(16))) for i in range(37)]
        assert got.tolist() == brute


def test_c_encode_matches_numpy(tiny_pq):
    cb, x = tiny_pq["codebooks"], tiny_pq["base"][:5000]
    assert np.array_equal(cref.pq_encode(x, cb), O.pack_nibbles(O.pq_encode(x, cb)))
    # 8-bit sub-quantizers: 8 x 256 on d=96 shaped data
    rng = np.random.default_rng(1)
    cb8 = rng.normal(size=(8, 256, 12)).astype(np.float32)
    x8 = rng.normal(size=(500, 96)).astype(np.float32)
    assert np.array_equal(cref.pq_encode(x8, cb8), O.pq_encode(x8, cb8))


# ------------------------------------------------------- Eq. (2) == Eq. (3)

def test_adc_equals_distance_to_decoded_code(tiny_pq):
    cb, comps, q = tiny_pq["codebooks"], tiny_pq["comps"][:2000], tiny_pq["queries"]
    dec = O.pq_decode(comps, cb).astype(np.float64)
    luts = O.build_luts(cb, q)
    for iq in range(len(q)):
        brute = ((q[iq].astype(np.float64)[None, :] - dec) ** 2).sum(axis=1)
        np.testing.assert_allclose(O.adc_float(luts[iq], comps), brute, rtol=1e-5)


def test_adc_exact_on_centroid_tuple_database():
    # Database vectors that ARE centroid tuples are encoded without error, so
    # ADC is the exact squared distance and ADC top-R is exact k-NN.
    rng = np.random.default_rng(11)
    m, k, dsub = 8, 16, 4
    cb = rng.normal(scale=10, size=(m, k, dsub)).astype(np.float32)
    comps = rng.integers(0, k, size=(3000, m), dtype=np.uint8)
    comps = np.unique(comps, axis=0)
    base = O.pq_decode(comps, cb)
    assert np.array_equal(O.pq_encode(base, cb), comps)
    q = rng.normal(scale=10, size=(5, m * dsub)).astype(np.float32)
    for y in q:
        idx, dist = O.adc_search(cb, y, comps, 20)
        exact = ((y.astype(np.float64)[None, :] - base.astype(np.float64)) ** 2).sum(axis=1)
        order = np.argsort(exact, kind="stable")[:20]
        assert np.array_equal(idx, order.astype(np.uint32))
        np.testing.assert_allclose(dist, exact[order], rtol=1e-5)


def test_adc_uses_table_j_for_component_j():
    # tables that differ only in which j they belong to: a transposed or
    # shifted lookup changes the sum
    m, k = 4, 16
    lut = (np.arange(m)[:, None] * 1000 + np.arange(k)[None, :]).astype(np.float32)
    comps = np.array([[1, 2, 3, 4]], dtype=np.uint8)
    assert O.adc_float(lut, comps)[0] == (0 + 1) + (1000 + 2) + (2000 + 3) + (3000 + 4)
    codes = O.pack_nibbles(comps)
    assert cref.adc_f32(codes, lut)[0] == O.adc_float(lut, comps)[0]
    q = lut.astype(np.uint8)  # wraps mod 256: entries still distinct per (j, i)
    s = int(q[0, 1]) + int(q[1, 2]) + int(q[2, 3]) + int(q[3, 4])
    assert O.scan_saturating(q, codes)[0] == min(255, s)
    assert O.scan_clamped(q, codes)[0] == min(255, s)
    assert cref.scan_u8(codes, q)[0] == min(255, s)


# ------------------------------------------------------------- Section 3.3

def test_qmax_is_rth_smallest_of_init(tiny_pq):
    cb, comps, q = tiny_pq["codebooks"], tiny_pq["comps"], tiny_pq["queries"]
    lut = O.build_luts(cb, q[:1])[0]
    for init, R in [(200, 100), (1000, 100), (50, 100), (200, 1), (200, 200)]:
        cand = sorted(float(v) for v in O.adc_float(lut, comps[:init]))
        want = cand[min(R, len(cand)) - 1]
        assert float(O.qmax_from_init(lut, comps[:init], R)) == want
    # qmax bounds the true R-th distance from above (Section 3.3: later
    # candidates must be closer)
    full = np.sort(O.adc_float(lut, comps))
    assert O.qmax_from_init(lut, comps[:200], 100) >= full[99]


@pytest.mark.parametrize("nbins", [255, 127])
@pytest.mark.parametrize("mode", [O.QMIN_PER_TABLE, O.QMIN_GLOBAL])
def test_quantizer_properties(tiny_pq, nbins, mode):
    cb, comps, q = tiny_pq["codebooks"], tiny_pq["comps"], tiny_pq["queries"]
    for y in q[:4]:
        lut = O.build_luts(cb, y[None])[0]
        qmax = O.qmax_from_init(lut, comps[:200], 100)
        bias, delta = O.quantizer_params(lut, qmax, nbins, mode)
        ql = O.quantize_luts(lut, bias, delta, nbins)
        assert ql.dtype == np.uint8 and ql.max() <= nbins
        if mode == O.QMIN_PER_TABLE:
            assert np.all(bias == lut.min(axis=1))
            assert np.all(ql.min(axis=1) == 0)
            qmin = np.float32(0)
            for b in bias:
                qmin = np.float32(qmin + b)
        else:
            assert np.all(bias == lut.min())
            qmin = lut.min()
            assert ql.min() == 0
        assert delta == np.float32((qmax - qmin) / np.float32(nbins))
        # monotone in the table value
        for j in range(lut.shape[0]):
            o = np.argsort(lut[j], kind="stable")
            assert np.all(np.diff(ql[j][o].astype(int)) >= 0)
        # bin index: floor((D - bias)/Delta) in exact arithmetic, within float32 rounding
        t = (lut.astype(np.float64) - bias[:, None]) / float(delta)
        exact = np.minimum(np.floor(t), nbins)
        near_edge = np.abs(t - np.round(t)) < 1e-4 * np.maximum(1, t)
        assert np.all((ql == exact) | near_edge)
        # an entry at or beyond the range saturates alone
        assert np.all(ql[(lut - bias[:, None]) >= np.float32(nbins + 1) * delta] == nbins)


def test_quantizer_degenerate_delta():
    lut = np.full((4, 16), 7.0, dtype=np.float32)
    bias, delta = O.quantizer_params(lut, np.float32(28.0), 255, O.QMIN_PER_TABLE)
    assert delta == 1.0  # qmax == qmin
    assert np.all(O.quantize_luts(lut, bias, delta) == 0)
    bias, delta = O.quantizer_params(lut, np.float32(1.0), 255, O.QMIN_GLOBAL)
    assert delta == 1.0  # qmax < qmin
    lut2 = lut.copy()
    lut2[0, 3] = 7.0 + 300.0
    assert O.quantize_luts(lut2, bias, delta)[0, 3] == 255
    assert O.quantize_luts(lut2, bias, delta, 127)[0, 3] == 127


def test_shared_quantizer_over_probe_tables():
    rng = np.random.default_rng(3)
    luts = rng.uniform(10, 1000, size=(5, 8, 16)).astype(np.float32)
    bias, delta = O.quantizer_params(luts, np.float32(5000), 255, O.QMIN_PER_TABLE)
    assert np.all(bias == luts.min(axis=(0, 2)))
    bias_g, _ = O.quantizer_params(luts, np.float32(5000), 255, O.QMIN_GLOBAL)
    assert np.all(bias_g == luts.min())


# ------------------------------------------------------------- Alg. 2 scan

@pytest.mark.parametrize("nbins", [255, 127])
def test_saturating_chain_equals_clamped_sum(nbins):
    rng = np.random.default_rng(7)
    for m in (8, 16, 32):
        codes = rng.integers(0, 256, size=(5000, m // 2), dtype=np.uint8)
        for hi in (nbins + 1, 40, 12):  # saturating often / sometimes / never
            qlut = rng.integers(0, hi, size=(m, 16)).astype(np.uint8)
            a = O.scan_saturating(qlut, codes, nbins)
            b = O.scan_clamped(qlut, codes, nbins)
            c = cref.scan_u8(codes, qlut, nbins)
            assert np.array_equal(a, b) and np.array_equal(a, c)
    # brute force, pure Python, tiny
    qlut = rng.integers(0, 90, size=(8, 16)).astype(np.uint8)
    codes = rng.integers(0, 256, size=(50, 4), dtype=np.uint8)
    want = []
    for code in codes:
        acc = 0
        for j, byte in enumerate(code):
            acc = min(nbins, acc + int(qlut[2 * j][byte & 15]))
            acc = min(nbins, acc + int(qlut[2 * j + 1][byte >> 4]))
        want.append(acc)
    assert O.scan_saturating(qlut, codes, nbins).tolist() == want


@pytest.mark.parametrize("nbins", [255, 127])
@pytest.mark.parametrize("mode", [O.QMIN_PER_TABLE, O.QMIN_GLOBAL])
def test_quantized_sum_brackets_float_adc(tiny_pq, nbins, mode):
    # floor quantization: B + Delta*s <= adc < B + Delta*(s+m) when s < n,
    # adc >= qmax when s == n; so no member of the float top-R saturates.
    cb, comps, codes, q = (tiny_pq[k] for k in ("codebooks", "comps", "codes", "queries"))
    m = cb.shape[0]
    for y in q[:4]:
        t = O.quick_adc_tables(cb, y, codes, 200, 100, nbins, mode)
        s = O.scan_saturating(t["qlut"], codes, nbins).astype(np.float64)
        adc = np.zeros(len(comps))
        for j in range(m):
            adc += t["lut"][j][comps[:, j]].astype(np.float64)
        B = float(t["bias"].astype(np.float64).sum())
        d = float(t["delta"])
        slack = 1e-5 * np.maximum(adc, 1.0)
        unsat = s < nbins
        assert unsat.any() and (~unsat).any()
        assert np.all(B + d * s[unsat] <= adc[unsat] + slack[unsat])
        assert np.all(adc[unsat] < B + d * (s[unsat] + m) + slack[unsat])
        assert np.all(adc[~unsat] >= float(t["qmax"]) - slack[~unsat])
        top = np.argsort(adc, kind="stable")[:100]
        assert np.all(s[top] < nbins)


# ------------------------------------------------------------------ top-R

def test_byte_component_variant_chain_bounds_and_c_twin():
    # 8-bit sub-quantizers with quantized tables: the chain equals min(n, sum); an unsaturated sum
    # s brackets the float ADC distance, B + Delta*s <= adc < B + Delta*(s+m); the plain-C twin
    # returns the R best of the NumPy sums.
    from oracle import cref
    rng = np.random.default_rng(21)
    m, k, dsub, n = 8, 256, 4, 3000
    cb = rng.normal(scale=20, size=(m, k, dsub)).astype(np.float32)
    x = rng.normal(scale=20, size=(n, m * dsub)).astype(np.float32)
    comps = O.pq_encode(x, cb)
    assert comps.shape == (n, m) and comps.max() > 15
    y = rng.normal(scale=20, size=m * dsub).astype(np.float32)
    for nbins, mode in ((255, O.QMIN_PER_TABLE), (127, O.QMIN_GLOBAL)):
        r = O.quick_adc_bytes_search(cb, y, comps, 200, 50, nbins, mode)
        sums = O.scan_saturating_bytes(r["qlut"], comps, nbins)
        brute = np.array([min(nbins, sum(int(r["qlut"][j][comps[i, j]]) for j in range(m))) for i in range(n)])
        assert np.array_equal(sums, brute)
        adc = O.adc_float(r["lut"], comps).astype(np.float64)
        B = float(r["bias"].astype(np.float64).sum())
        D = float(r["delta"])
        free = sums < nbins
        assert free.any()
        sf = sums[free].astype(np.int64)
        lo, hi = B + D * sf, B + D * (sf + m)
        tol = 1e-4 * np.abs(adc[free]) + 1e-3
        assert (adc[free] >= lo - tol).all() and (adc[free] < hi + tol).all()
        order = np.lexsort((np.arange(n), sums))[:50]
        assert np.array_equal(r["idx"], order.astype(np.uint32)) and np.array_equal(r["dist"], sums[order])
        ci, cd = cref.scan_topk_u8_bytes(comps, r["qlut"][None], 50, nbins)
        assert np.array_equal(ci[0], r["idx"]) and np.array_equal(cd[0], r["dist"])


def test_top_r_order_and_ties():
    rng = np.random.default_rng(9)
    s = rng.integers(0, 6, size=500).astype(np.uint8)  # massive ties
    idx, dist = O.top_r(s, 100, pad_dist=255)
    pairs = sorted((int(v), i) for i, v in enumerate(s))[:100]
    assert idx.tolist() == [p[1] for p in pairs]
    assert dist.tolist() == [p[0] for p in pairs]
    # all equal -> the first R indices
    idx, dist = O.top_r(np.zeros(300, dtype=np.uint8), 100, pad_dist=255)
    assert idx.tolist() == list(range(100)) and not dist.any()
    # fewer than R inputs -> padding
    idx, dist = O.top_r(np.array([3, 1, 2], dtype=np.uint8), 5, pad_dist=255)
    assert idx.tolist() == [1, 2, 0, 0xFFFFFFFF, 0xFFFFFFFF]
    assert dist.tolist() == [1, 2, 3, 255, 255]


def test_c_scan_topk_matches_numpy(tiny_pq):
    cb, codes, q = tiny_pq["codebooks"], tiny_pq["codes"], tiny_pq["queries"]
    qluts = np.stack([O.quick_adc_tables(cb, y, codes, 200, 100)["qlut"] for y in q])
    idx, dist = cref.scan_topk_u8(codes, qluts, 100)
    for iq in range(len(q)):
        wi, wd = O.top_r(O.scan_saturating(qluts[iq], codes), 100, pad_dist=255)
        assert np.array_equal(idx[iq], wi) and np.array_equal(dist[iq], wd)
    # heavy ties + N < R padding
    rng = np.random.default_rng(2)
    ql = rng.integers(0, 2, size=(1, 16, 16)).astype(np.uint8)
    idx, dist = cref.scan_topk_u8(codes[:3000], ql, 100)
    wi, wd = O.top_r(O.scan_saturating(ql[0], codes[:3000]), 100, pad_dist=255)
    assert np.array_equal(idx[0], wi) and np.array_equal(dist[0], wd)
    idx, dist = cref.scan_topk_u8(codes[:30], ql, 100)
    wi, wd = O.top_r(O.scan_saturating(ql[0], codes[:30]), 100, pad_dist=255)
    assert np.array_equal(idx[0], wi) and np.array_equal(dist[0], wd)
    # float scan
    luts = O.build_luts(cb, q)
    fi, fd = cref.scan_topk_f32(codes, luts, 100)
    for iq in range(len(q)):
        wi, wd = O.top_r(O.adc_float(luts[iq], tiny_pq["comps"]), 100, pad_dist=np.inf)
        assert np.array_equal(fi[iq], wi) and np.array_equal(fd[iq], wd)


# ---------------------------------------------------------------- k-means

def test_kmeans_distortion_and_recovery():
    rng = np.random.default_rng(4)
    centres = np.array([[0, 0], [100, 0], [0, 100], [100, 100]], dtype=np.float32)
    lab = rng.integers(0, 4, size=2000)
    x = (centres[lab] + rng.normal(scale=2.0, size=(2000, 2))).astype(np.float32)
    first = [int(np.flatnonzero(lab == c)[0]) for c in range(4)]
    c, hist = O.kmeans_lloyd(x, np.array(first), 6)
    assert all(b <= a + 1e-9 for a, b in zip(hist, hist[1:]))
    for t in range(4):
        assert np.abs(c[t] - x[lab == t].mean(axis=0)).max() < 1e-3
    # k = 1: the mean, after one iteration
    c1, _ = O.kmeans_lloyd(x, np.array([17]), 1)
    np.testing.assert_allclose(c1[0], x.astype(np.float64).mean(axis=0), rtol=1e-6)


def test_pq_train_distortion_decreases(tiny_pq):
    x = tiny_pq["train"][:, :8]
    from workloads import kmeans_init_rows
    _, hist = O.kmeans_lloyd(x, kmeans_init_rows(len(x), 16), 8)
    assert all(b <= a + 1e-9 for a, b in zip(hist, hist[1:])) and hist[-1] < hist[0]


# ------------------------------------------------------------------- IVF

def _small_ivf(seed=0, n=6000, K=12, d=32, m=8):
    rng = np.random.default_rng(seed)
    coarse = rng.uniform(0, 255, size=(K, d)).astype(np.float32)
    x = (coarse[rng.integers(0, K, size=n)] + rng.normal(scale=20, size=(n, d))).astype(np.float32)
    cb = rng.normal(scale=15, size=(m, 16, d // m)).astype(np.float32)
    return coarse, x, cb, rng


def test_ivf_build_groups_by_cell():
    coarse, x, cb, _ = _small_ivf()
    ix = O.ivf_build(x, coarse, cb)
    cell = np.argmin(cdist(x.astype(np.float64), coarse.astype(np.float64), "sqeuclidean"), axis=1)
    assert ix["list_off"][-1] == len(x)
    for c in range(len(coarse)):
        ids = ix["ids"][ix["list_off"][c]:ix["list_off"][c + 1]]
        assert np.array_equal(ids, np.flatnonzero(cell == c).astype(np.uint32))
    # codes are those of the residuals
    p = 1234
    i = int(ix["ids"][p])
    r = (x[i] - coarse[cell[i]])[None, :]
    assert np.array_equal(ix["codes"][p], O.pack_nibbles(O.pq_encode(r, cb))[0])


def test_ivf_single_list_equals_flat_search():
    # one cell with a zero centroid: residual == vector, the index is the flat database
    _, x, cb, rng = _small_ivf(1)
    coarse = np.zeros((1, x.shape[1]), dtype=np.float32)
    ix = O.ivf_build(x, coarse, cb)
    y = x[5] + 3
    a = O.ivf_quick_adc_search(ix, coarse, cb, y, 1, 200, 50)
    b = O.quick_adc_search(cb, y, ix["codes"], 200, 50)
    assert np.array_equal(a["ids"], b["idx"]) and np.array_equal(a["dist"], b["dist"])
    assert np.array_equal(a["qluts"][0], b["qlut"])


def test_ivf_probes_and_all_cells():
    coarse, x, cb, rng = _small_ivf(2)
    ix = O.ivf_build(x, coarse, cb)
    y = x[77]
    dist = cdist(y[None].astype(np.float64), coarse.astype(np.float64), "sqeuclidean")[0]
    assert O.ivf_probes(y, coarse, 5).tolist() == np.argsort(dist, kind="stable")[:5].tolist()
    # probing every cell scans every stored code exactly once, each with its cell's tables
    K = len(coarse)
    res = O.ivf_quick_adc_search(ix, coarse, cb, y, K, 500, 40)
    sums = np.empty(len(x), dtype=np.uint8)
    for t, p in enumerate(res["probes"]):
        lo, hi = ix["list_off"][p], ix["list_off"][p + 1]
        sums[lo:hi] = O.scan_saturating(res["qluts"][t], ix["codes"][lo:hi])
    pos, d = O.top_r(sums, 40, pad_dist=255)
    assert np.array_equal(res["pos"], pos.astype(np.int64)) and np.array_equal(res["dist"], d)
    assert np.array_equal(res["ids"], ix["ids"][pos])
    # the query's own vector (distance ~ quantization error) is found
    assert 77 in res["ids"]


# ------------------------------------------------------------------ optimized product quantizer

def test_opq_rotate_against_hand_worked_matrices():
    """y = R x (Section 2.1): a permutation matrix permutes components, a plane rotation by 90
    degrees maps (a, b) to (-b, a), the identity changes nothing."""
    from oracle import qadc_oracle as O
    x = np.array([[1.0, 2.0, 3.0, 4.0], [-5.0, 0.5, 7.0, 8.0]], dtype=np.float32)
    assert np.array_equal(O.opq_rotate(np.eye(4, dtype=np.float32), x), x)
    perm = np.zeros((4, 4), dtype=np.float32)
    perm[0, 2] = perm[1, 0] = perm[2, 3] = perm[3, 1] = 1.0     # y0 = x2, y1 = x0, y2 = x3, y3 = x1
    assert np.array_equal(O.opq_rotate(perm, x), x[:, [2, 0, 3, 1]])
    quarter = np.eye(4, dtype=np.float32)
    quarter[:2, :2] = [[0.0, -1.0], [1.0, 0.0]]
    assert np.array_equal(O.opq_rotate(quarter, x), np.stack([-x[:, 1], x[:, 0], x[:, 2], x[:, 3]], axis=1))


def test_opq_train_is_orthonormal_monotone_and_finds_a_hidden_rotation():
    """Data made of two independent 2-d cluster sets (one per sub-space) and then rotated by a
    known orthonormal Q: a plain product quantizer on the rotated data mixes the sub-spaces and
    pays for it; OPQ must return an orthonormal R, never increase its distortion from round to
    round, and end far below the plain product quantizer."""
    from oracle import qadc_oracle as O
    rng = np.random.default_rng(42)
    n, k = 3000, 16
    grid = np.array([[a, b] for a in range(4) for b in range(4)], dtype=np.float64) * 10.0
    parts = [grid[rng.integers(0, 16, size=n)] + rng.normal(scale=0.3, size=(n, 2)) for _ in range(2)]
    clean = np.concatenate(parts, axis=1)
    q, _ = np.linalg.qr(rng.normal(size=(4, 4)))
    mixed = (clean @ q.T).astype(np.float32)
    rows = rng.permutation(n)[:k]
    plain = O.pq_distortion(mixed, O.pq_train(mixed, 2, k, 8, rows))
    ideal = O.pq_distortion(clean.astype(np.float32), O.pq_train(clean.astype(np.float32), 2, k, 8, rows))
    rot, cb, hist = O.opq_train(mixed, 2, k, 12, 4, rows)
    np.testing.assert_allclose(rot.astype(np.float64).T @ rot.astype(np.float64), np.eye(4), atol=1e-5)
    assert all(b <= a * (1 + 1e-6) for a, b in zip(hist, hist[1:]))
    got = O.pq_distortion(O.opq_rotate(rot, mixed), cb)
    assert got <= hist[0] * (1 + 1e-6)
    assert plain > 1.5 * ideal          # the hidden rotation matters on this data
    assert got < 0.5 * plain            # and OPQ undoes most of the damage


def test_opq_with_identity_rotation_is_the_product_quantizer():
    """outer = 0 rounds: R = I and the codebooks of pq_train."""
    from oracle import qadc_oracle as O
    rng = np.random.default_rng(1)
    x = rng.normal(size=(500, 8)).astype(np.float32)
    rows = np.arange(16)
    rot, cb, hist = O.opq_train(x, 4, 16, 0, 3, rows)
    assert np.array_equal(rot, np.eye(8, dtype=np.float32)) and hist == []
    assert np.array_equal(cb, O.pq_train(x, 4, 16, 3, rows))


# ------------------------------------------------------------------ inverted multi-index (Section 5)

def test_multi_index_probe_order_on_a_worked_example():
    """One component per half, query at the origin: d1 = (0, 1, 4), d2 = (0, 4, 9).  The nine sums in
    order, equal sums by cell id: 0 (0,0); 1 (1,0); 4 (0,1) then (2,0); 5 (1,1); 8 (2,1); 9 (0,2);
    10 (1,2); 13 (2,2)."""
    from oracle import qadc_oracle as O
    halves = np.array([[[0.0], [1.0], [2.0]], [[0.0], [2.0], [3.0]]], dtype=np.float32)
    got = O.multi_index_probes(np.zeros(2, dtype=np.float32), halves, 9)
    assert got.tolist() == [0, 3, 1, 6, 4, 7, 2, 5, 8]
    cells = O.multi_index_cells(halves)
    assert cells.shape == (9, 2) and cells[5].tolist() == [1.0, 3.0] and cells[6].tolist() == [2.0, 0.0]


def test_multi_index_is_the_inverted_index_over_the_product_cells():
    """The product structure: the closest cell is the pair of closest half-centroids, and the cells
    by increasing d1 + d2 are the cells by increasing distance to the concatenated centroids; the
    multi-sequence walk (which never forms the K*K sums) outputs the same order."""
    from oracle import qadc_oracle as O
    rng = np.random.default_rng(8)
    K, dh, n = 23, 5, 400
    halves = rng.normal(size=(2, K, dh)).astype(np.float32)
    x = rng.normal(size=(n, 2 * dh)).astype(np.float32)
    coarse = O.multi_index_cells(halves)
    assert np.array_equal(O.multi_index_assign(x, halves), O.ivf_assign(x, coarse))
    for y in x[:20]:
        want = O.ivf_probes(y, coarse, 60)
        assert np.array_equal(O.multi_index_probes(y, halves, 60), want)
        d1 = O.sq_l2(y[None, :dh], halves[0])[0]
        d2 = O.sq_l2(y[None, dh:], halves[1])[0]
        walk = [i * K + j for i, j in O.multi_sequence(d1, d2, 60)]
        assert walk == want.tolist()
