"""Pins of the oracle's multi-index over occupied cells (CPU only).

The related-work section combines Quick ADC with the fine partition of an inverted multi-index;
at its usual size most of the K*K cells are empty and only occupied cells carry a list.  Expected
values are written by hand (cells, list boundaries, centroids) or come from brute force over all
codes (a stored code must be the one whose reproduction, added to the cell's centroid, is closest
to the vector: Section 2.2), or from the inverted index over all K*K cells, pinned on its own.
"""

from __future__ import annotations

import itertools

import numpy as np

from oracle import qadc_oracle as O


def _tiny():
    # d = 2: first half-quantizer {0, 10, 20}, second {0, 100, 200}; cell (i, j) = 3 i + j
    halves = np.array([[[0.0], [10.0], [20.0]], [[0.0], [100.0], [200.0]]], dtype=np.float32)
    x = np.array([[11, 190],    # (1, 2) -> 5
                  [1, 96],      # (0, 1) -> 1
                  [19, 3],      # (2, 0) -> 6
                  [9, 204],     # (1, 2) -> 5
                  [-2, 110],    # (0, 1) -> 1
                  [12, 170]],   # (1, 2) -> 5
                 dtype=np.float32)
    return halves, x


def test_occupied_cells_lists_and_centroids_by_hand():
    halves, x = _tiny()
    rng = np.random.default_rng(3)
    cb = rng.normal(scale=6, size=(2, 16, 1)).astype(np.float32)
    ix = O.multi_index_build_occupied(x, halves, cb)
    assert ix["cell_ids"].tolist() == [1, 5, 6]                   # 6 of the 9 cells have no list
    assert ix["list_off"].tolist() == [0, 2, 5, 6]
    assert ix["ids"].tolist() == [1, 4, 0, 3, 5, 2]               # input order inside a list
    assert ix["centroids"].tolist() == [[0, 100], [10, 200], [20, 0]]
    # every stored code is the best of all 16^2 codes for centroid + reproduction (Section 2.2)
    comps = O.unpack_nibbles(ix["codes"])
    for pos, v in enumerate(ix["ids"]):
        s = int(np.searchsorted(ix["list_off"], pos, side="right")) - 1
        best, best_err = None, np.inf
        for a, b in itertools.product(range(16), repeat=2):
            approx = ix["centroids"][s].astype(np.float64) + np.array([cb[0, a, 0], cb[1, b, 0]], dtype=np.float64)
            err = float(((x[v].astype(np.float64) - approx) ** 2).sum())
            if err < best_err:
                best, best_err = (a, b), err
        assert tuple(comps[pos]) == best
    # the wrong reading (residual against the swapped halves) would store other codes
    swapped = np.concatenate([halves[0][ix["cell_ids"] % 3], halves[1][ix["cell_ids"] // 3]], axis=1)
    assert not np.array_equal(swapped, ix["centroids"])


def test_slots_of_cells_by_hand():
    cell_ids = np.array([1, 5, 6], dtype=np.uint32)
    cells = np.array([[5, 0, 6], [8, 1, 1]], dtype=np.int32)
    assert O.multi_index_slots(cell_ids, cells).tolist() == [[1, -1, 2], [-1, 0, 0]]


def test_occupied_index_is_the_dense_index_without_its_empty_lists():
    """Same lists, codes and search results as the inverted index over all K*K cells (pinned by the
    inverted-index pins), the empty cells left out."""
    rng = np.random.default_rng(8)
    K, dh, m, n = 9, 4, 4, 150          # 81 cells, most of them empty
    d = 2 * dh
    halves = rng.uniform(0, 255, size=(2, K, dh)).astype(np.float32)
    cells_all = O.multi_index_cells(halves)
    home = rng.choice(K * K, size=20, replace=False)
    x = (cells_all[rng.choice(home, size=n)] + rng.normal(scale=6, size=(n, d))).astype(np.float32)
    cb = rng.normal(scale=5, size=(m, 16, d // m)).astype(np.float32)
    dense = O.ivf_build(x, cells_all, cb)
    ix = O.multi_index_build_occupied(x, halves, cb)
    sizes = np.diff(dense["list_off"])
    assert np.array_equal(ix["cell_ids"], np.nonzero(sizes)[0])
    assert 1 < len(ix["cell_ids"]) < K * K // 2
    assert np.array_equal(np.diff(ix["list_off"]), sizes[sizes > 0])
    assert np.array_equal(ix["codes"], dense["codes"]) and np.array_equal(ix["ids"], dense["ids"])
    assert np.array_equal(ix["centroids"], cells_all[ix["cell_ids"]])
    for seed in range(5):
        y = (x[rng.integers(n)] + rng.normal(scale=4, size=d)).astype(np.float32)
        probes = O.multi_index_probes(y, halves, 30)
        slots = O.multi_index_slots(ix["cell_ids"], probes)
        assert (slots < 0).any() and (slots >= 0).sum() >= 2
        # an empty cell contributes no code and, having no list, no tables: both searches see the
        # same candidates for qmax only when the quantizer is built from the occupied cells' tables
        occupied = probes[slots >= 0]
        a = O.ivf_quick_adc_search(dense, cells_all, cb, y, len(occupied), 40, 10, probes=occupied)
        b = O.ivf_quick_adc_search(ix, ix["centroids"], cb, y, len(occupied), 40, 10, probes=slots[slots >= 0])
        assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["dist"], b["dist"])
        assert np.array_equal(a["qluts"], b["qluts"]) and np.array_equal(a["pos"], b["pos"])
