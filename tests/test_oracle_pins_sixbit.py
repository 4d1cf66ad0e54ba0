"""Pins of the oracle's 6-bit sub-quantizer path (the paper's Conclusion names 6-bit quantizers as
what wider registers buy; the layout is this repository's reading: components back to back,
least significant bit first).  CPU only; expected values are written out by hand, taken from
brute force in pure Python, or from the 4-bit path they must reduce to."""

from __future__ import annotations

import numpy as np

from oracle import qadc_oracle as O
from oracle import cref


def test_sixbit_layout_on_bytes_written_by_hand():
    # 1 | 2 << 6 | 3 << 12 | 4 << 18 = 0x103081 -> bytes 81 30 10; 63 | 0 << 6 | 63 << 12 | 0 << 18 = 0x03F03F
    comps = np.array([[1, 2, 3, 4, 63, 0, 63, 0], [0, 0, 0, 32, 33, 21, 42, 7]], dtype=np.uint8)
    codes = O.pack_sixbit(comps)
    assert codes.shape == (2, 6)
    assert codes[0].tolist() == [0x81, 0x30, 0x10, 0x3F, 0xF0, 0x03]
    # 32 << 18 = 0x800000 -> bytes 00 00 80; 33 | 21 << 6 | 42 << 12 | 7 << 18 = 0x1EA561
    assert codes[1].tolist() == [0x00, 0x00, 0x80, 0x61, 0xA5, 0x1E]
    assert np.array_equal(O.unpack_sixbit(codes), comps)
    rng = np.random.default_rng(1)
    big = rng.integers(0, 64, size=(500, 32), dtype=np.uint8)
    assert np.array_equal(O.unpack_sixbit(O.pack_sixbit(big)), big)
    # code i as a little-endian number
    for row, c in zip(O.pack_sixbit(big)[:20], big[:20]):
        assert int.from_bytes(row.tobytes(), "little") == sum(int(v) << (6 * j) for j, v in enumerate(c))
    assert O.code_bits(16, 64) == 96 and O.table_bytes(16, 64) == 4096


def test_sixbit_chain_brackets_float_adc_and_matches_brute_force_and_c_twin():
    rng = np.random.default_rng(31)
    m, k, dsub, n = 8, 64, 4, 2500
    cb = rng.normal(scale=20, size=(m, k, dsub)).astype(np.float32)
    x = rng.normal(scale=20, size=(n, m * dsub)).astype(np.float32)
    comps = O.pq_encode(x, cb)
    assert comps.max() > 15 and comps.max() < 64
    codes = O.pack_sixbit(comps)
    y = rng.normal(scale=20, size=m * dsub).astype(np.float32)
    # Eq. (2) equals Eq. (3): the distance to the decoded vector
    lut = O.build_luts(cb, y[None])[0]
    adc = O.adc_float(lut, comps).astype(np.float64)
    brute_d = ((y.astype(np.float64)[None, :] - O.pq_decode(comps, cb).astype(np.float64)) ** 2).sum(axis=1)
    np.testing.assert_allclose(adc, brute_d, rtol=1e-5)
    for nbins, mode in ((255, O.QMIN_PER_TABLE), (127, O.QMIN_GLOBAL)):
        r = O.quick_adc_sixbit_search(cb, y, codes, 200, 50, nbins, mode)
        sums = O.scan_saturating_sixbit(r["qlut"], codes, nbins)
        brute = np.array([min(nbins, sum(int(r["qlut"][j][comps[i, j]]) for j in range(m))) for i in range(n)])
        assert np.array_equal(sums, brute)
        # sequential saturation, written out for a few codes
        for i in range(0, n, 97):
            acc = 0
            for j in range(m):
                acc = min(nbins, acc + int(r["qlut"][j][comps[i, j]]))
            assert acc == sums[i]
        B = float(r["bias"].astype(np.float64).sum())
        D = float(r["delta"])
        free = sums < nbins
        assert free.any()
        sf = sums[free].astype(np.int64)
        tol = 1e-4 * np.abs(adc[free]) + 1e-3
        assert (adc[free] >= B + D * sf - tol).all() and (adc[free] < B + D * (sf + m) + tol).all()
        assert (adc[~free] >= float(r["qmax"]) - 1e-3).all()
        order = sorted(range(n), key=lambda i: (int(sums[i]), i))[:50]
        assert r["idx"].tolist() == order and r["dist"].tolist() == [int(sums[i]) for i in order]
        ci, cd = cref.scan_topk_u8_sixbit(codes, r["qlut"][None], 50, nbins)
        assert np.array_equal(ci[0], r["idx"]) and np.array_equal(cd[0], r["dist"])


def test_sixbit_reduces_to_the_4bit_path_when_codebooks_repeat():
    """Codebooks of 64 centroids whose entries 16..63 repeat entry i mod 16... would tie; instead the
    extra 48 centroids are placed far away, so that every vector encodes to an index below 16 and
    the 6-bit search must return what the 4-bit search returns on the first 16 centroids."""
    rng = np.random.default_rng(5)
    m, dsub, n = 8, 4, 1500
    cb16 = rng.normal(scale=20, size=(m, 16, dsub)).astype(np.float32)
    far = (1e4 + rng.normal(scale=20, size=(m, 48, dsub))).astype(np.float32)
    cb64 = np.concatenate([cb16, far], axis=1)
    x = rng.normal(scale=20, size=(n, m * dsub)).astype(np.float32)
    c16, c64 = O.pq_encode(x, cb16), O.pq_encode(x, cb64)
    assert np.array_equal(c16, c64)
    y = rng.normal(scale=20, size=m * dsub).astype(np.float32)
    a = O.quick_adc_search(cb16, y, O.pack_nibbles(c16), 300, 40)
    b = O.quick_adc_sixbit_search(cb64, y, O.pack_sixbit(c64), 300, 40)
    # same qmax and same minima per table (the far centroids never hold a table's minimum)
    assert a["qmax"] == b["qmax"] and np.array_equal(a["bias"], b["bias"]) and a["delta"] == b["delta"]
    assert np.array_equal(a["qlut"], b["qlut"][:, :16])
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["dist"], b["dist"])
