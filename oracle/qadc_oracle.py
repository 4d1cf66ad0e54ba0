"""CPU oracle for the Quick ADC query path -- TEST INFRASTRUCTURE, not product.

Only tests, the smoke check and the bench's CPU-baseline leg may import this
module.  It shares no code with the HIP library and imports nothing from it.

Everything here follows the paper (Andre, Kermarrec, Le Scouarnec, "Accelerated
Nearest Neighbor Search with Quick ADC", ICMR'17) step by step in plain NumPy,
slow and unblocked, so that it can be checked against the text by eye:

  Section 2.1          vector / product quantizers, codes of m*b bits; optimized product
                       quantizers opq(x) = pq(R x), R orthonormal
  Section 2.2          inverted index, residual encoding
  Section 5 (related)  inverted multi-index as the coarse partition
  Section 2.3, Alg. 1  Index / Tables / Scan, Eq. (1) tables, Eq. (2) ADC
  Section 3.2, Fig. 2  two 4-bit components per byte, low nibble = even one;
                       lists transposed by blocks of 16 codes
  Section 3.3          8-bit quantization of the tables, qmin / qmax / Delta
  Section 3.4, Alg. 2  lookup, saturating add, top-R

Readings taken where the text is silent, garbled or ambiguous (each is also
listed in the design notes of the repository):

  * loop bounds "0 to m" in Alg. 1 are read as j = 0 .. m-1; `adc(p, ...)`
    is read as adc(c, ...).
  * Alg. 2 `lookup_add` shuffles with the masked nibbles (Fig. 5), not the
    unmasked register.
  * Fig. 2: byte j of a code holds component 2j in its low nibble and
    component 2j+1 in its high nibble.
  * Section 3.3 rounding: floor (a bin index).  The overflow test applies to
    the offset value: q = min(n, floor((D - bias) / Delta)).
  * Section 3.3 qmin: two modes.  GLOBAL is the literal text (one scalar, the
    minimum over all tables, subtracted from every entry).  PER_TABLE
    subtracts each table's own minimum and starts the range at the sum of
    those minima (the smallest ADC sum that can occur).
  * Section 3.3 n: 127 in the paper (signed bytes, x86 limitation); any
    1 <= n <= 255 is accepted, the saturation cap is n.
  * The `init` codes only fix qmax; all N codes (the first `init` included)
    are then scanned with the quantized tables, and top-R is over quantized
    sums only.
  * init > N: the first min(init, N) codes are used; fewer than R of them:
    the largest.  Delta <= 0 (or NaN): Delta = 1.
  * `extract_matches` / the heap are unspecified about ties: the R smallest
    under the total order (sum, index) are returned, ascending.
  * Inverted index with several probed cells: one quantizer per query, shared
    by all probed cells; ties are broken by storage position in the
    concatenated lists.
  * 6-bit sub-quantizers (named in the Conclusion as what wider registers buy,
    without a layout): the m six-bit components of a code are stored back to
    back, least significant bit first -- component j is bits 6j .. 6j+5 of the
    code read as one little-endian number, so four components fill three
    bytes; tables have 64 entries; quantization and saturating sums as for
    4-bit components.

Pins (tests/test_oracle_*.py): Eq. (1) against scipy cdist; encode against the
argmin of the same; Eq. (2) against Eq. (3) by brute force; centroid-tuple
databases where ADC is the exact distance; the sequential saturating chain
against min(n, sum); the bound  B + Delta*s <= adc < B + Delta*(s+m)  for
unsaturated sums; stable-argsort and brute-force top-R; the table sizes
printed in the paper's Table 1.  Recall figures of the paper need its datasets
and are unpinned (ordering checks only).  k-means is pinned only by
non-increasing distortion and recovery of well-separated clusters.  The OPQ
trainer is pinned by the orthonormality of R, by a distortion that does not grow
from round to round, and by data that a known rotation makes separable per
sub-space (it must get close to the distortion reached with that rotation);
opq_rotate by permutation and block-rotation matrices worked by hand.  The
transposed layout of Fig. 2b is pinned by a block written out by hand, the
positions of single bytes of a ragged list, and by Alg. 2 run over its blocks
and rows giving the sums of the standard-layout scan and of the plain definition.
The inverted-index search is pinned by hand-built indexes: the qmax walk (first
`init` codes in probe order, each with its own cell's tables) against brute-force
distances to centroid + decoded residual, the (sum, storage position) order
against sorted tuples on lists probed in reverse storage order, the Index step
on repeated centroids; overlap, NN-recall and exact_nn on rows worked by hand.
The multi-index over occupied cells is pinned by a six-vector example whose cells,
list boundaries and centroids are written by hand, its codes by brute force over
all codes, and by equality with the inverted index over all K*K cells.
"""

from __future__ import annotations

import numpy as np

QMIN_PER_TABLE = 0
QMIN_GLOBAL = 1

PAD_IDX = np.uint32(0xFFFFFFFF)


# --------------------------------------------------------------------------
# Section 2.1: quantizers
# --------------------------------------------------------------------------

def sq_l2(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Squared Euclidean distances ||a_r - b_i||^2, float64 [len(a)][len(b)]."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    diff = a[:, None, :] - b[None, :, :]
    return np.einsum("rit,rit->ri", diff, diff)


def vq_encode(x: np.ndarray, centroids: np.ndarray, chunk: int | None = None) -> np.ndarray:
    """enc(x) = index of the closest centroid (Section 2.1); ties -> lowest index."""
    out = np.empty(len(x), dtype=np.int64)
    if chunk is None:  # bound the [chunk][k][dim] float64 temporary to ~64 MiB
        chunk = max(1, (1 << 23) // max(1, centroids.shape[0] * centroids.shape[1]))
    for s in range(0, len(x), chunk):
        out[s:s + chunk] = np.argmin(sq_l2(x[s:s + chunk], centroids), axis=1)
    return out


def kmeans_lloyd(x: np.ndarray, init_rows: np.ndarray, iters: int):
    """Lloyd's k-means.  x float32 [n][dsub]; start = rows `init_rows` of x.

    One iteration = assign every row to its closest centroid (float64
    distances, ties -> lowest index), then replace each centroid by the mean
    of its rows (float64 sum, stored as float32).  A centroid that owns no row
    keeps its value.  Returns (centroids float32 [k][dsub], distortion list),
    distortion[t] = mean squared distance at the assignment of iteration t.
    """
    x = np.asarray(x, dtype=np.float32)
    c = x[np.asarray(init_rows)].copy()
    k = len(c)
    history = []
    for _ in range(iters):
        dist = sq_l2(x, c)
        a = np.argmin(dist, axis=1)
        history.append(float(dist[np.arange(len(x)), a].mean()))
        for i in range(k):
            own = x[a == i]
            if len(own):
                c[i] = own.astype(np.float64).sum(axis=0) / len(own)
    return c, history


def pq_train(train: np.ndarray, m: int, k: int, iters: int, init_rows: np.ndarray):
    """Product quantizer (Section 2.1): one k-centroid codebook per sub-space.

    Returns codebooks float32 [m][k][d/m].
    """
    n, d = train.shape
    assert d % m == 0
    dsub = d // m
    cb = np.empty((m, k, dsub), dtype=np.float32)
    for j in range(m):
        cb[j], _ = kmeans_lloyd(train[:, j * dsub:(j + 1) * dsub], init_rows, iters)
    return cb


def pq_encode(x: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """enc(x) = (i_0, ..., i_{m-1}) (Section 2.1).  Returns uint8 [n][m]."""
    m, k, dsub = codebooks.shape
    comps = np.empty((len(x), m), dtype=np.uint8)
    for j in range(m):
        comps[:, j] = vq_encode(x[:, j * dsub:(j + 1) * dsub], codebooks[j])
    return comps


def pq_decode(comps: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """pq(x): concatenation of the selected centroids, float32 [n][d]."""
    m = codebooks.shape[0]
    return np.concatenate([codebooks[j][comps[:, j]] for j in range(m)], axis=1)


def opq_rotate(rot: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y = R x for every row x (Section 2.1, opq(x) = pq(R x)): float64 products and sums,
    one rounding to float32.  rot float32 [d][d], x float32 [n][d] -> float32 [n][d]."""
    return (np.asarray(x, dtype=np.float64) @ np.asarray(rot, dtype=np.float64).T).astype(np.float32)


def kmeans_refine(x: np.ndarray, centroids: np.ndarray, iters: int):
    """`iters` Lloyd iterations (as kmeans_lloyd) started from the given centroids."""
    x = np.asarray(x, dtype=np.float32)
    c = np.asarray(centroids, dtype=np.float32).copy()
    for _ in range(iters):
        a = np.argmin(sq_l2(x, c), axis=1)
        for i in range(len(c)):
            own = x[a == i]
            if len(own):
                c[i] = own.astype(np.float64).sum(axis=0) / len(own)
    return c


def pq_distortion(x: np.ndarray, codebooks: np.ndarray) -> float:
    """Mean squared distance between the rows of x and their reproductions pq(x)."""
    y = pq_decode(pq_encode(x, codebooks), codebooks)
    return float(((np.asarray(x, dtype=np.float64) - y) ** 2).sum(axis=1).mean())


def opq_train(train: np.ndarray, m: int, k: int, outer: int, inner: int, init_rows: np.ndarray):
    """Optimized product quantizer (Section 2.1): an orthonormal R (R^T R = I) and the codebooks
    of pq, so that opq(x) = pq(R x).  The paper takes R from the cited OPQ method; this is
    its non-parametric form written out: starting from R = I and a product quantizer of the
    unrotated data, alternate
      (1) codebooks: `inner` Lloyd iterations per sub-space on the rotated learning set R x,
          continued from the current codebooks;
      (2) rotation: with Y the reproductions pq(R x) of the learning set, the orthonormal R
          minimising sum ||R x - y||^2, i.e. the orthogonal Procrustes solution
          R = V U^T for the SVD  X^T Y = U S V^T.
    Neither step increases the distortion sum ||R x - pq(R x)||^2.
    Returns (R float32 [d][d], codebooks float32 [m][k][d/m], distortion after each round).
    """
    x = np.asarray(train, dtype=np.float32)
    n, d = x.shape
    dsub = d // m
    rot = np.eye(d, dtype=np.float64)
    cb = pq_train(x, m, k, inner, init_rows)
    history = []
    for _ in range(outer):
        xr = (x.astype(np.float64) @ rot.T).astype(np.float32)
        for j in range(m):
            cb[j] = kmeans_refine(xr[:, j * dsub:(j + 1) * dsub], cb[j], inner)
        y = pq_decode(pq_encode(xr, cb), cb).astype(np.float64)
        history.append(float(((xr.astype(np.float64) - y) ** 2).sum(axis=1).mean()))
        u, _, vt = np.linalg.svd(x.astype(np.float64).T @ y)
        rot = (u @ vt).T
    return rot.astype(np.float32), cb, history


def code_bits(m: int, k: int) -> int:
    """Size of a code: m * ceil(log2 k) bits (Section 2.1)."""
    return m * int(np.ceil(np.log2(k)))


def table_bytes(m: int, k: int) -> int:
    """Size of the float tables of one query: m * k * sizeof(float) (Section 2.4)."""
    return m * k * 4


# --------------------------------------------------------------------------
# Section 3.2 / Fig. 2: standard layout, two 4-bit components per byte
# --------------------------------------------------------------------------

def pack_nibbles(comps: np.ndarray) -> np.ndarray:
    """uint8 [n][m] (values < 16) -> uint8 [n][m/2]; byte j = c[2j] | c[2j+1] << 4."""
    comps = np.asarray(comps, dtype=np.uint8)
    assert comps.shape[1] % 2 == 0 and comps.max(initial=0) < 16
    return (comps[:, 0::2] | (comps[:, 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(codes: np.ndarray) -> np.ndarray:
    """Inverse of pack_nibbles: the mask (0x0f) and the 4-bit right shift of Alg. 2."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, half = codes.shape
    comps = np.empty((n, 2 * half), dtype=np.uint8)
    comps[:, 0::2] = codes & 0x0F
    comps[:, 1::2] = codes >> 4
    return comps


# --------------------------------------------------------------------------
# 6-bit components (Conclusion): four components per three bytes
# --------------------------------------------------------------------------

def pack_sixbit(comps: np.ndarray) -> np.ndarray:
    """uint8 [n][m] (values < 64, m a multiple of 4) -> uint8 [n][3m/4].

    The code is the number sum_j c[j] << 6j written in little-endian bytes.
    """
    comps = np.asarray(comps, dtype=np.uint8)
    n, m = comps.shape
    assert m % 4 == 0 and comps.max(initial=0) < 64
    out = np.zeros((n, 3 * m // 4), dtype=np.uint8)
    for j in range(m):
        for b in range(6):  # bit b of component j is bit 6j + b of the code
            bit = 6 * j + b
            out[:, bit // 8] |= (((comps[:, j] >> b) & 1) << (bit % 8)).astype(np.uint8)
    return out


def unpack_sixbit(codes: np.ndarray) -> np.ndarray:
    """Inverse of pack_sixbit: uint8 [n][3m/4] -> uint8 [n][m]."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, nbytes = codes.shape
    assert nbytes % 3 == 0
    m = nbytes * 4 // 3
    comps = np.zeros((n, m), dtype=np.uint8)
    for j in range(m):
        for b in range(6):
            bit = 6 * j + b
            comps[:, j] |= (((codes[:, bit // 8] >> (bit % 8)) & 1) << b).astype(np.uint8)
    return comps


def scan_saturating_sixbit(qlut: np.ndarray, codes: np.ndarray, nbins: int = 255) -> np.ndarray:
    """The chain of Alg. 2 for 6-bit components: component j -> 64-entry table j, saturating add.
    qlut uint8 [m][64], codes uint8 [n][3m/4] (pack_sixbit)."""
    comps = unpack_sixbit(codes)
    acc = np.zeros(len(codes), dtype=np.int64)
    for j in range(qlut.shape[0]):
        acc = np.minimum(nbins, acc + qlut[j][comps[:, j]])
    return acc.astype(np.uint8)


def quick_adc_sixbit_search(codebooks, query, codes, init, R, nbins=255, qmin_mode=QMIN_PER_TABLE):
    """Quick ADC with 6-bit sub-quantizers: Tables (Eq. 1, [m][64]), qmax from the first `init`
    codes (Section 3.3), the quantizer, saturating scan, top-R.  codes uint8 [n][3m/4]."""
    lut = build_luts(codebooks, query[None, :])[0]
    comps = unpack_sixbit(codes)
    qmax = qmax_from_init(lut, comps[:min(init, len(comps))], R)
    bias, delta = quantizer_params(lut, qmax, nbins, qmin_mode)
    qlut = quantize_luts(lut, bias, delta, nbins)
    sums = scan_saturating_sixbit(qlut, codes, nbins)
    idx, dist = top_r(sums, R, pad_dist=nbins)
    return dict(lut=lut, qmax=qmax, bias=bias, delta=delta, qlut=qlut, idx=idx, dist=dist)


# --------------------------------------------------------------------------
# Section 3.2 / Fig. 2b: lists transposed by blocks of 16 codes
# --------------------------------------------------------------------------

BLOCK = 16  # codes per block: one byte of 16 codes fills a 128-bit register


def transposed_bytes(n: int, m: int) -> int:
    """Size of a list of n codes in the transposed layout: whole blocks of 16 * m/2 bytes."""
    return -(-n // BLOCK) * BLOCK * (m // 2)


def pack_transposed(codes: np.ndarray) -> np.ndarray:
    """Standard layout uint8 [n][m/2] -> transposed layout, flat uint8.

    Each block of 16 codes (a .. p) is stored as m/2 rows of 16 bytes; row j holds
    byte j (components 2j and 2j+1) of a, b, .. p in this order.  The last block
    is filled up with zero bytes.
    """
    codes = np.asarray(codes, dtype=np.uint8)
    n, half = codes.shape
    nblk = -(-n // BLOCK)
    out = np.zeros((nblk, half, BLOCK), dtype=np.uint8)
    for i in range(n):  # code i is column i % 16 of block i // 16
        out[i // BLOCK, :, i % BLOCK] = codes[i]
    return out.reshape(-1)


def unpack_transposed(packed: np.ndarray, n: int, m: int) -> np.ndarray:
    """Inverse of pack_transposed for a list of n codes."""
    half = m // 2
    blocks = np.asarray(packed, dtype=np.uint8).reshape(-1, half, BLOCK)
    out = np.empty((n, half), dtype=np.uint8)
    for i in range(n):
        out[i] = blocks[i // BLOCK, :, i % BLOCK]
    return out


def scan_blocks_transposed(qlut: np.ndarray, packed: np.ndarray, n: int, nbins: int = 255) -> np.ndarray:
    """Alg. 2 quick_adc_scan over a block-transposed list: block by block, row by row.

    A row is one "register" of 16 bytes; the accumulator holds the 16 sums of the
    block.  Low nibbles -> table 2j, saturating add; shift by four; -> table 2j+1,
    saturating add.  Returns the sums of the n codes of the list.
    """
    m = qlut.shape[0]
    half = m // 2
    blocks = np.asarray(packed, dtype=np.uint8).reshape(-1, half, BLOCK)
    out = np.empty(len(blocks) * BLOCK, dtype=np.uint8)
    for b, blk in enumerate(blocks):
        acc = np.zeros(BLOCK, dtype=np.int64)
        for j in range(half):
            comps = blk[j]
            acc = np.minimum(nbins, acc + qlut[2 * j][comps & 0x0F])
            comps = comps >> 4
            acc = np.minimum(nbins, acc + qlut[2 * j + 1][comps & 0x0F])
        out[b * BLOCK:(b + 1) * BLOCK] = acc
    return out[:n]


# --------------------------------------------------------------------------
# Section 2.3: Tables (Eq. 1) and ADC (Eq. 2)
# --------------------------------------------------------------------------

def build_luts(codebooks: np.ndarray, queries: np.ndarray, base: np.ndarray | None = None):
    """Eq. (1): D^j[i] = || y'^j - C^j[i] ||^2, float32 [nq][m][k].

    y' = y for exhaustive search, y' = y - base for a probed cell whose
    centroid is `base` (Section 2.3, Index).  Float64 accumulation, one
    rounding to float32.
    """
    m, k, dsub = codebooks.shape
    y = np.asarray(queries, dtype=np.float64)
    if base is not None:
        y = y - np.asarray(base, dtype=np.float64)
    out = np.empty((len(y), m, k), dtype=np.float32)
    for j in range(m):
        out[:, j, :] = sq_l2(y[:, j * dsub:(j + 1) * dsub], codebooks[j])
    return out


def adc_float(lut: np.ndarray, comps: np.ndarray) -> np.ndarray:
    """Eq. (2): adc(y, c) = sum_j D^j[c[j]], float32, added in increasing j.

    lut float32 [m][k], comps uint8 [n][m]  ->  float32 [n].
    """
    m = lut.shape[0]
    acc = np.zeros(len(comps), dtype=np.float32)
    for j in range(m):
        acc = acc + lut[j][comps[:, j]]  # float32 + float32
    return acc


# --------------------------------------------------------------------------
# Section 3.3: quantization of the tables
# --------------------------------------------------------------------------

def qmax_from_init(lut: np.ndarray, comps_init: np.ndarray, R: int) -> np.float32:
    """qmax: float ADC distance of the R-th best among the `init` first codes."""
    cand = adc_float(lut, comps_init)
    return qmax_from_candidates(cand, R)


def qmax_from_candidates(cand: np.ndarray, R: int) -> np.float32:
    cand = np.sort(np.asarray(cand, dtype=np.float32))
    return np.float32(cand[min(R, len(cand)) - 1])


def quantizer_params(luts: np.ndarray, qmax, nbins: int = 255, qmin_mode: int = QMIN_PER_TABLE):
    """bias float32 [m] and Delta float32 for one query.

    luts float32 [..., m, k]: every leading entry is one set of m tables of the
    same query (one set for exhaustive search, one per probed cell otherwise);
    they share the quantizer.

    GLOBAL    bias_j = g = min over everything, qmin = g           (Section 3.3)
    PER_TABLE bias_j = min over table j (all sets), qmin = sum_j bias_j
    Delta = (qmax - qmin) / n, replaced by 1 when not positive.
    """
    luts = np.asarray(luts, dtype=np.float32)
    m, k = luts.shape[-2:]
    flat = luts.reshape(-1, m, k)
    if qmin_mode == QMIN_GLOBAL:
        g = flat.min()
        bias = np.full(m, g, dtype=np.float32)
        qmin = np.float32(g)
    elif qmin_mode == QMIN_PER_TABLE:
        bias = flat.min(axis=(0, 2)).astype(np.float32)
        qmin = np.float32(0)
        for j in range(m):
            qmin = np.float32(qmin + bias[j])  # float32, increasing j
    else:
        raise ValueError("qmin_mode")
    delta = np.float32((np.float32(qmax) - qmin) / np.float32(nbins))
    if not (delta > 0):
        delta = np.float32(1.0)
    return bias, delta


def quantize_luts(luts: np.ndarray, bias: np.ndarray, delta, nbins: int = 255) -> np.ndarray:
    """q^j[i] = min(n, floor(max(0, D^j[i] - bias_j) / Delta)), float32 arithmetic, uint8."""
    luts = np.asarray(luts, dtype=np.float32)
    off = np.maximum(np.float32(0), luts - bias[:, None].astype(np.float32))
    t = np.floor(off / np.float32(delta))
    return np.minimum(t, np.float32(nbins)).astype(np.uint8)


# --------------------------------------------------------------------------
# Section 3.4 / Alg. 2: lookups and saturating adds
# --------------------------------------------------------------------------

def scan_saturating(qlut: np.ndarray, codes: np.ndarray, nbins: int = 255) -> np.ndarray:
    """Alg. 2 quick_adc_block on the standard layout, one code per "lane".

    For each byte row j: low nibble -> table 2j, saturating add; shift right by
    four; -> table 2j+1, saturating add.  qlut uint8 [m][16], codes uint8
    [n][m/2].  Saturating add with cap n: min(n, acc + partial).
    """
    n, half = codes.shape
    acc = np.zeros(n, dtype=np.int64)
    for j in range(half):
        comps = codes[:, j]
        masked = comps & 0x0F
        acc = np.minimum(nbins, acc + qlut[2 * j][masked])
        comps = comps >> 4
        masked = comps & 0x0F
        acc = np.minimum(nbins, acc + qlut[2 * j + 1][masked])
    return acc.astype(np.uint8)


def scan_clamped(qlut: np.ndarray, codes: np.ndarray, nbins: int = 255) -> np.ndarray:
    """min(n, sum_j q^j[c[j]]): equal to the saturating chain for entries >= 0."""
    comps = unpack_nibbles(codes)
    total = np.zeros(len(codes), dtype=np.int64)
    for j in range(qlut.shape[0]):
        total += qlut[j][comps[:, j]]
    return np.minimum(total, nbins).astype(np.uint8)


def scan_saturating_bytes(qlut: np.ndarray, comps: np.ndarray, nbins: int = 255) -> np.ndarray:
    """The chain of Alg. 2 for 8-bit components: one byte and one 256-entry table per component.

    The paper keeps 16-entry tables because a table has to fit a 128-bit register
    (Section 3.1); where the tables live in a memory that takes 256 entries, the
    quantization of Section 3.3 and the saturating sums apply unchanged to the
    8-bit sub-quantizers of Section 2.1.  qlut uint8 [m][256], comps uint8 [n][m].
    """
    acc = np.zeros(len(comps), dtype=np.int64)
    for j in range(qlut.shape[0]):
        acc = np.minimum(nbins, acc + qlut[j][comps[:, j]])
    return acc.astype(np.uint8)


def top_r(dist: np.ndarray, R: int, pad_dist=None):
    """The R smallest under the order (dist, index), ascending.

    Returns (idx uint32 [R], dist [R]); missing entries (fewer than R inputs)
    hold index 0xFFFFFFFF and `pad_dist`.
    """
    dist = np.asarray(dist)
    order = np.argsort(dist, kind="stable")[:R]
    idx = np.full(R, PAD_IDX, dtype=np.uint32)
    out = np.full(R, pad_dist if pad_dist is not None else 0, dtype=dist.dtype)
    idx[:len(order)] = order.astype(np.uint32)
    out[:len(order)] = dist[order]
    return idx, out


# --------------------------------------------------------------------------
# Whole query paths
# --------------------------------------------------------------------------

def quick_adc_tables(codebooks, query, codes, init, R, nbins=255, qmin_mode=QMIN_PER_TABLE,
                     lut=None):
    """Tables step of a Quick ADC query on a flat database (Sections 2.3, 3.3).

    Returns dict(lut, qmax, bias, delta, qlut).  `lut` may be supplied (float32
    [m][16]) to quantize tables obtained elsewhere.
    """
    if lut is None:
        lut = build_luts(codebooks, query[None, :])[0]
    n_init = min(init, len(codes))
    qmax = qmax_from_init(lut, unpack_nibbles(codes[:n_init]), R)
    bias, delta = quantizer_params(lut, qmax, nbins, qmin_mode)
    qlut = quantize_luts(lut, bias, delta, nbins)
    return dict(lut=lut, qmax=qmax, bias=bias, delta=delta, qlut=qlut)


def quick_adc_search(codebooks, query, codes, init, R, nbins=255, qmin_mode=QMIN_PER_TABLE):
    """Exhaustive Quick ADC search for one query: Tables, quantize, scan, top-R."""
    t = quick_adc_tables(codebooks, query, codes, init, R, nbins, qmin_mode)
    sums = scan_saturating(t["qlut"], codes, nbins)
    idx, dist = top_r(sums, R, pad_dist=nbins)
    t.update(idx=idx, dist=dist)
    return t


def quick_adc_bytes_search(codebooks, query, comps, init, R, nbins=255, qmin_mode=QMIN_PER_TABLE):
    """Quick ADC with 8-bit sub-quantizers: Tables (Eq. 1, [m][256]), qmax from the first
    `init` codes, the quantizer of Section 3.3, saturating scan, top-R.  comps uint8 [n][m]."""
    lut = build_luts(codebooks, query[None, :])[0]
    qmax = qmax_from_init(lut, comps[:min(init, len(comps))], R)
    bias, delta = quantizer_params(lut, qmax, nbins, qmin_mode)
    qlut = quantize_luts(lut, bias, delta, nbins)
    sums = scan_saturating_bytes(qlut, comps, nbins)
    idx, dist = top_r(sums, R, pad_dist=nbins)
    return dict(lut=lut, qmax=qmax, bias=bias, delta=delta, qlut=qlut, idx=idx, dist=dist)


def adc_search(codebooks, query, comps, R):
    """Alg. 1: float ADC scan of a flat database + R best by (distance, index)."""
    lut = build_luts(codebooks, query[None, :])[0]
    d = adc_float(lut, comps)
    return top_r(d, R, pad_dist=np.float32(np.inf))


# --------------------------------------------------------------------------
# Section 2.2 / 2.3: inverted index
# --------------------------------------------------------------------------

def ivf_assign(x: np.ndarray, coarse: np.ndarray) -> np.ndarray:
    """q_i(x): closest coarse centroid (ties -> lowest cell id)."""
    return vq_encode(x, coarse)


def ivf_build(x: np.ndarray, coarse: np.ndarray, codebooks: np.ndarray):
    """Section 2.2: assign, encode the residual r(x) = x - q_i(x), group by cell.

    Returns dict(list_off int64 [K+1], codes uint8 [n][m/2] in list order,
    ids uint32 [n]); inside a list, vectors keep their input order.
    """
    K = len(coarse)
    cell = ivf_assign(x, coarse)
    order = np.argsort(cell, kind="stable")
    resid = x[order] - coarse[cell[order]]
    comps = pq_encode(resid.astype(np.float32), codebooks)
    list_off = np.zeros(K + 1, dtype=np.int64)
    np.cumsum(np.bincount(cell, minlength=K), out=list_off[1:])
    return dict(list_off=list_off, codes=pack_nibbles(comps), ids=order.astype(np.uint32))


def ivf_probes(query: np.ndarray, coarse: np.ndarray, nprobe: int) -> np.ndarray:
    """Index step: the nprobe closest cells, closest first (ties -> lowest id)."""
    dist = sq_l2(query[None, :], coarse)[0]
    return np.argsort(dist, kind="stable")[:nprobe].astype(np.int32)


# --------------------------------------------------------------------------
# Related work: inverted multi-index as the coarse partition
# --------------------------------------------------------------------------
#
# The paper's related-work section notes that Quick ADC, needing no minimum
# list size, combines with the finer partition of an inverted multi-index.
# There the coarse quantizer is a product of two quantizers over the two
# halves of the vector: cell (i, j), id i*K + j, has the centroid
# (halves[0][i], halves[1][j]).  Everything after the Index step is the
# inverted-index search over those K*K cells.

def multi_index_cells(halves: np.ndarray) -> np.ndarray:
    """halves float32 [2][K][d/2] -> the K*K cell centroids float32 [K*K][d], cell id = i*K + j."""
    K, dh = halves.shape[1], halves.shape[2]
    out = np.empty((K, K, 2 * dh), dtype=np.float32)
    out[:, :, :dh] = halves[0][:, None, :]
    out[:, :, dh:] = halves[1][None, :, :]
    return out.reshape(K * K, 2 * dh)


def multi_index_assign(x: np.ndarray, halves: np.ndarray) -> np.ndarray:
    """Cell of every vector: each half goes to its closest half-centroid (ties -> lowest)."""
    K, dh = halves.shape[1], halves.shape[2]
    return vq_encode(x[:, :dh], halves[0]) * K + vq_encode(x[:, dh:], halves[1])


def multi_index_probes(query: np.ndarray, halves: np.ndarray, nprobe: int) -> np.ndarray:
    """The nprobe cells with the smallest d1[i] + d2[j], smallest first (ties -> lowest cell id):
    the definition, written out over all K*K cells."""
    K, dh = halves.shape[1], halves.shape[2]
    d1 = sq_l2(query[None, :dh], halves[0])[0]
    d2 = sq_l2(query[None, dh:], halves[1])[0]
    sums = (d1[:, None] + d2[None, :]).reshape(K * K)
    return np.argsort(sums, kind="stable")[:nprobe].astype(np.int32)


def multi_sequence(d1: np.ndarray, d2: np.ndarray, count: int):
    """Cells (i, j) by increasing d1[i] + d2[j] without forming the K*K sums: walk the two sorted
    lists from their heads; a pair enters the queue once both its predecessors (one rank lower in
    either list) have been output.  Returns the first `count` (i, j)."""
    import heapq
    o1, o2 = np.argsort(d1, kind="stable"), np.argsort(d2, kind="stable")
    K1, K2 = len(d1), len(d2)
    done = set()
    heap = [(d1[o1[0]] + d2[o2[0]], 0, 0)]
    pushed = {(0, 0)}
    out = []
    while heap and len(out) < count:
        _, r1, r2 = heapq.heappop(heap)
        out.append((int(o1[r1]), int(o2[r2])))
        done.add((r1, r2))
        for a, b in ((r1 + 1, r2), (r1, r2 + 1)):
            if a < K1 and b < K2 and (a, b) not in pushed:
                if (a == 0 or (a - 1, b) in done) and (b == 0 or (a, b - 1) in done):
                    heapq.heappush(heap, (d1[o1[a]] + d2[o2[b]], a, b))
                    pushed.add((a, b))
    return out


def multi_index_build_occupied(x: np.ndarray, halves: np.ndarray, codebooks: np.ndarray):
    """The multi-index at its usual size (K*K far above the number of vectors): only the cells that
    hold a vector get an inverted list.  Lists are in increasing cell id; inside a list vectors keep
    their input order; the residual is taken against (halves[0][i], halves[1][j]).

    Returns dict(cell_ids uint32 [L] ascending, centroids float32 [L][d], list_off int64 [L+1],
    codes uint8 [n][m/2], ids uint32 [n]): an inverted index over L lists, list s being cell
    cell_ids[s]; ivf_quick_adc_search takes it with coarse = centroids and probes = list numbers.
    """
    K = halves.shape[1]
    cell = multi_index_assign(x, halves)
    cell_ids = np.unique(cell)
    order = np.argsort(cell, kind="stable")
    i, j = cell[order] // K, cell[order] % K
    resid = x[order] - np.concatenate([halves[0][i], halves[1][j]], axis=1)
    comps = pq_encode(resid.astype(np.float32), codebooks)
    list_off = np.zeros(len(cell_ids) + 1, dtype=np.int64)
    list_off[1:] = np.cumsum([np.count_nonzero(cell == c) for c in cell_ids])
    centroids = np.concatenate([halves[0][cell_ids // K], halves[1][cell_ids % K]], axis=1)
    return dict(cell_ids=cell_ids.astype(np.uint32), centroids=centroids.astype(np.float32),
                list_off=list_off, codes=pack_nibbles(comps), ids=order.astype(np.uint32))


def multi_index_slots(cell_ids: np.ndarray, cells: np.ndarray) -> np.ndarray:
    """List number of every cell id in `cells` (its place in the ascending `cell_ids`), -1 for a
    cell that holds no vector."""
    where = {int(c): s for s, c in enumerate(cell_ids)}
    return np.array([where.get(int(c), -1) for c in np.asarray(cells).ravel()],
                    dtype=np.int32).reshape(np.shape(cells))


def ivf_quick_adc_search(index, coarse, codebooks, query, nprobe, init, R, nbins=255,
                         qmin_mode=QMIN_PER_TABLE, probes=None, qluts=None):
    """Non-exhaustive Quick ADC search for one query.

    Index: nprobe cells.  Tables: one set per probed cell with y' = y - centroid.
    qmax: float ADC of the first `init` codes met walking the probed lists in
    probe order, each code with its own cell's tables; R-th best.  One
    quantizer for the query.  Scan: every code of every probed list, quantized
    sums; top-R by (sum, storage position); ids[position] returned.

    `probes` / `qluts` (uint8 [nprobe][m][16]) may be supplied to replay the
    integer part on tables obtained elsewhere.
    """
    list_off, codes, ids = index["list_off"], index["codes"], index["ids"]
    if probes is None:
        probes = ivf_probes(query, coarse, nprobe)
    probes = np.asarray(probes)
    luts = np.stack([build_luts(codebooks, query[None, :], coarse[p][None, :])[0] for p in probes])
    out = dict(probes=probes, luts=luts)
    if qluts is None:
        cand = []
        left = init
        for t, p in enumerate(probes):
            if left <= 0:
                break
            lo, hi = int(list_off[p]), int(list_off[p + 1])
            take = min(left, hi - lo)
            cand.append(adc_float(luts[t], unpack_nibbles(codes[lo:lo + take])))
            left -= take
        cand = np.concatenate(cand) if cand else np.zeros(0, dtype=np.float32)
        if len(cand):
            qmax = qmax_from_candidates(cand, R)
        else:
            qmax = np.float32(0)
        bias, delta = quantizer_params(luts, qmax, nbins, qmin_mode)
        qluts = np.stack([quantize_luts(l, bias, delta, nbins) for l in luts])
        out.update(qmax=qmax, bias=bias, delta=delta)
    out["qluts"] = qluts
    pos_all, sum_all = [], []
    for t, p in enumerate(probes):
        lo, hi = int(list_off[p]), int(list_off[p + 1])
        sum_all.append(scan_saturating(qluts[t], codes[lo:hi], nbins))
        pos_all.append(np.arange(lo, hi, dtype=np.int64))
    pos_all = np.concatenate(pos_all) if pos_all else np.zeros(0, dtype=np.int64)
    sum_all = np.concatenate(sum_all) if sum_all else np.zeros(0, dtype=np.uint8)
    order = np.lexsort((pos_all, sum_all))[:R]
    out_ids = np.full(R, PAD_IDX, dtype=np.uint32)
    out_pos = np.full(R, -1, dtype=np.int64)
    out_dist = np.full(R, nbins, dtype=np.uint8)
    out_ids[:len(order)] = ids[pos_all[order]]
    out_pos[:len(order)] = pos_all[order]
    out_dist[:len(order)] = sum_all[order]
    out.update(ids=out_ids, pos=out_pos, dist=out_dist)
    return out


# --------------------------------------------------------------------------
# Accuracy measures
# --------------------------------------------------------------------------

def overlap_at_r(idx_a: np.ndarray, idx_b: np.ndarray) -> float:
    """|A & B| / R averaged over queries; rows are top-R index lists."""
    idx_a, idx_b = np.atleast_2d(idx_a), np.atleast_2d(idx_b)
    tot = 0.0
    for a, b in zip(idx_a, idx_b):
        tot += len(np.intersect1d(a[a != PAD_IDX], b[b != PAD_IDX])) / a.shape[0]
    return tot / len(idx_a)


def nn_recall_at_r(idx: np.ndarray, true_nn: np.ndarray) -> float:
    """Fraction of queries whose exact nearest neighbour is among the R returned."""
    idx = np.atleast_2d(idx)
    return float(np.mean([true_nn[q] in idx[q] for q in range(len(idx))]))


def exact_nn(queries: np.ndarray, base: np.ndarray, chunk: int = 65536) -> np.ndarray:
    """Index of the exact nearest base vector of each query (lowest index on ties)."""
    q = np.asarray(queries, dtype=np.float64)
    best = np.full(len(q), np.inf)
    arg = np.zeros(len(q), dtype=np.int64)
    qq = (q * q).sum(axis=1)
    for s in range(0, len(base), chunk):
        b = np.asarray(base[s:s + chunk], dtype=np.float64)
        dist = qq[:, None] - 2.0 * q @ b.T + (b * b).sum(axis=1)[None, :]
        a = np.argmin(dist, axis=1)
        v = dist[np.arange(len(q)), a]
        upd = v < best
        best[upd] = v[upd]
        arg[upd] = a[upd] + s
    return arg
