"""Pins of the oracle's inverted-index search and accuracy measures (CPU only).

Each expected value here is worked out without the function under test: distances by brute force
on decoded vectors (Section 2.2: a stored vector is approximated by its cell's centroid plus the
reproduction of its residual; Eq. (3): ADC is the distance to that approximation), orders by
Python's sort of (sum, position) tuples, accuracy measures on rows written by hand.  Every test
also asserts that the plausible wrong reading gives a different value on its data, so that the
pin cannot pass by coincidence.
"""

from __future__ import annotations

import numpy as np

from oracle import qadc_oracle as O


def _hand_index(list_lens, m, rng):
    """An index whose lists hold random codes; ids are a permutation, so ids != positions."""
    n = int(sum(list_lens))
    list_off = np.zeros(len(list_lens) + 1, dtype=np.int64)
    np.cumsum(list_lens, out=list_off[1:])
    comps = rng.integers(0, 16, size=(n, m), dtype=np.uint8)
    ids = rng.permutation(n).astype(np.uint32)
    return dict(list_off=list_off, codes=O.pack_nibbles(comps), ids=ids), comps


def _brute_candidates(y, coarse, cb, comps, list_off, probes, init, own_tables=True, stop=True):
    """Float64 squared distances from y to centroid + decode(code) of the first `init` codes met
    walking the probed lists in probe order.  own_tables=False / stop=False are the two wrong
    readings (first cell's centroid for every list; no limit on the walk)."""
    out = []
    left = init
    for t, p in enumerate(probes):
        for pos in range(int(list_off[p]), int(list_off[p + 1])):
            if stop and left <= 0:
                break
            cen = coarse[p] if own_tables else coarse[probes[0]]
            approx = cen.astype(np.float64) + O.pq_decode(comps[pos:pos + 1], cb)[0].astype(np.float64)
            out.append(float(((y.astype(np.float64) - approx) ** 2).sum()))
            left -= 1
    return np.array(out)


def test_ivf_qmax_walks_lists_in_probe_order_with_each_cells_tables():
    """Section 3.3 (qmax from the first `init` codes) on an inverted index (Section 2.3: one set of
    tables per probed cell): three short lists, the walk ends inside the second probed list."""
    rng = np.random.default_rng(11)
    d, m = 16, 4
    coarse = rng.uniform(0, 200, size=(3, d)).astype(np.float32)
    cb = rng.normal(scale=20, size=(m, 16, d // m)).astype(np.float32)
    ix, comps = _hand_index([5, 7, 6], m, rng)
    y = (coarse[1] + rng.normal(scale=30, size=d)).astype(np.float32)
    probes = np.array([2, 0, 1], dtype=np.int32)  # probe order differs from storage order
    init, R = 9, 4                                  # 6 codes of list 2, then 3 of the 5 of list 0
    want = _brute_candidates(y, coarse, cb, comps, ix["list_off"], probes, init)
    assert len(want) == init
    qmax = np.sort(want)[R - 1]
    res = O.ivf_quick_adc_search(ix, coarse, cb, y, 3, init, R, probes=probes)
    assert abs(float(res["qmax"]) - qmax) <= 1e-5 * qmax
    # the wrong readings give another value on this data
    wrong_tables = np.sort(_brute_candidates(y, coarse, cb, comps, ix["list_off"], probes, init, own_tables=False))[R - 1]
    wrong_walk = np.sort(_brute_candidates(y, coarse, cb, comps, ix["list_off"], probes, init, stop=False))[R - 1]
    storage_order = np.sort(_brute_candidates(y, coarse, cb, comps, ix["list_off"], np.array([0, 1, 2]), init))[R - 1]
    for w in (wrong_tables, wrong_walk, storage_order):
        assert abs(w - qmax) > 1e-3 * qmax
    # one quantizer for the query: bias_j is the minimum of table j over all probed cells
    for j in range(m):
        dsub = d // m
        lo = min(float(((y[j * dsub:(j + 1) * dsub].astype(np.float64) - coarse[p, j * dsub:(j + 1) * dsub]
                         - cb[j, i].astype(np.float64)) ** 2).sum()) for p in probes for i in range(16))
        assert abs(float(res["bias"][j]) - lo) <= 1e-5 * max(lo, 1.0)


def test_ivf_walk_takes_whole_lists_when_init_exceeds_them():
    """init beyond the probed lists: every code is a candidate; fewer than R: the largest."""
    rng = np.random.default_rng(12)
    d, m = 8, 2
    coarse = rng.uniform(0, 100, size=(3, d)).astype(np.float32)
    cb = rng.normal(scale=10, size=(m, 16, d // m)).astype(np.float32)
    ix, comps = _hand_index([2, 0, 3], m, rng)
    y = rng.uniform(0, 100, size=d).astype(np.float32)
    probes = np.array([2, 1, 0], dtype=np.int32)
    want = _brute_candidates(y, coarse, cb, comps, ix["list_off"], probes, 1000)
    assert len(want) == 5
    res = O.ivf_quick_adc_search(ix, coarse, cb, y, 3, 1000, 50, probes=probes)
    assert abs(float(res["qmax"]) - want.max()) <= 1e-5 * want.max()


def test_ivf_ties_are_broken_by_storage_position_across_lists():
    """Equal sums across the R boundary, lists probed in the reverse of their storage order: the
    R smallest (sum, storage position) pairs, whatever the probe order."""
    m = 4
    qluts = np.zeros((2, m, 16), dtype=np.uint8)
    qluts[:, 0, :] = np.arange(16, dtype=np.uint8)  # sum = component 0 of the code, in both cells
    comp0 = {0: [3, 1, 3, 2], 1: [3, 0, 3, 3, 2, 3]}  # cell -> component 0 of its codes
    comps = np.zeros((10, m), dtype=np.uint8)
    comps[:4, 0] = comp0[0]
    comps[4:, 0] = comp0[1]
    ix = dict(list_off=np.array([0, 4, 10], dtype=np.int64), codes=O.pack_nibbles(comps),
              ids=np.array([90, 80, 70, 60, 50, 40, 30, 20, 10, 0], dtype=np.uint32))
    coarse = np.zeros((2, 8), dtype=np.float32)
    cb = np.zeros((m, 16, 2), dtype=np.float32)
    y = np.zeros(8, dtype=np.float32)
    pairs = sorted((int(comps[p, 0]), p) for p in range(10))
    for R in (5, 7):
        want = pairs[:R]  # R = 5: (0,5) (1,1) (2,3) (2,8) (3,0); the sum-3 codes 2, 4, 6, 7, 9 stay out
        res = O.ivf_quick_adc_search(ix, coarse, cb, y, 2, 100, R, probes=np.array([1, 0]), qluts=qluts)
        assert res["pos"].tolist() == [p for _, p in want]
        assert res["dist"].tolist() == [s for s, _ in want]
        assert res["ids"].tolist() == [int(ix["ids"][p]) for _, p in want]
        # probe order would have put position 4 (list 1, probed first) before position 0
        probe_order = sorted((int(comps[p, 0]), (0 if p >= 4 else 1), p) for p in range(10))[:R]
        assert [p for _, _, p in probe_order] != [p for _, p in want]
    assert pairs[4] == (3, 0) and pairs[5] == (3, 2) and pairs[6] == (3, 4)


def test_ivf_probes_equal_distances_go_to_the_lowest_cell():
    """Index step with repeated centroids: equal distances are ordered by cell id."""
    rng = np.random.default_rng(13)
    d = 6
    distinct = rng.uniform(0, 10, size=(4, d)).astype(np.float32)
    which = rng.integers(0, 4, size=96)          # 96 cells, only 4 distinct centroids
    coarse = distinct[which]
    y = rng.uniform(0, 10, size=d).astype(np.float32)
    dist = [float(((y.astype(np.float64) - c.astype(np.float64)) ** 2).sum()) for c in distinct]
    want = [cell for _, cell in sorted((dist[which[cell]], cell) for cell in range(96))]
    for nprobe in (1, 7, 40, 96):
        assert O.ivf_probes(y, coarse, nprobe).tolist() == want[:nprobe]
    assert len(set(dist)) == 4


def test_accuracy_measures_on_rows_written_by_hand():
    pad = 0xFFFFFFFF
    a = np.array([[1, 2, 3, 4], [5, 6, 7, pad]], dtype=np.uint32)
    b = np.array([[4, 9, 1, 8], [pad, 7, 5, 6]], dtype=np.uint32)
    # row 0 shares {1, 4}: 2/4; row 1 shares {5, 6, 7}, the padding is no neighbour: 3/4
    assert O.overlap_at_r(a, b) == (2 / 4 + 3 / 4) / 2
    assert O.overlap_at_r(a[0], a[0]) == 1.0
    assert O.overlap_at_r(a[0], np.array([10, 11, 12, 13], dtype=np.uint32)) == 0.0
    # exact neighbour of query 0 is 3 (returned), of query 1 is 9 (not returned)
    assert O.nn_recall_at_r(a, np.array([3, 9])) == 0.5
    assert O.nn_recall_at_r(a, np.array([9, 9])) == 0.0
    assert O.nn_recall_at_r(a, np.array([4, 5])) == 1.0


def test_exact_nn_on_a_grid_worked_by_hand():
    base = np.array([[0, 0], [3, 0], [0, 4], [3, 4], [3, 0]], dtype=np.float32)  # row 4 repeats row 1
    queries = np.array([[2.9, 0.1],    # next to (3, 0): rows 1 and 4 tie, the lower index wins
                        [0.2, 3.0],    # 1.04 from (0, 4), 9.04 from (0, 0)
                        [1.5, 2.0],    # the centre: all four corners at 6.25, row 0 wins
                        [10, 10]],     # closest corner (3, 4)
                       dtype=np.float32)
    want = [1, 2, 0, 3]
    for chunk in (1, 2, 3, 100):       # the answer does not depend on how the base is cut
        assert O.exact_nn(queries, base, chunk=chunk).tolist() == want
