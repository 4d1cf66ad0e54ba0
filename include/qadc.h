/*
 * qadc.h -- C ABI of the Quick ADC hot path for AMD MI355X (gfx950).
 *
 * Quick ADC (Andre, Kermarrec, Le Scouarnec, ICMR'17): nearest-neighbour search
 * over product-quantization codes with m sub-quantizers of 16 centroids each
 * (4-bit components), per-query lookup tables whose float distances are
 * quantized to 8-bit integers, saturating integer sums and top-R selection.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every array argument is a CALLER-OWNED DEVICE pointer (HBM), dense, in the
 *    row-major shape written beside it.  The library keeps no pointer after a
 *    call returns and frees nothing of the caller's.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue kernels on it and return without synchronizing; outputs are
 *    valid once the stream has reached that point.
 *  - Scratch memory comes from the caller: `workspace` (device, 256-byte
 *    aligned) of at least qadc_workspace_bytes(...) bytes.  The library never
 *    allocates device memory.  A workspace holds control words that every call
 *    expects to be zero and leaves zero: clear it with qadc_workspace_init before
 *    its first use, after a call on it failed or was aborted, and before a call
 *    whose entry point or sizes (n, m, nq, R, nprobe) differ from those of the
 *    call before it on that workspace -- another shape lays the workspace out
 *    differently, and table data of the earlier call may lie where the new one
 *    keeps its control words.  Calls of one shape need no clearing in between.
 *    (qadc_ivf_search clears its own control words at every call.)
 *    Calls that share a workspace must be ordered on one stream.
 *  - Return value: QADC_OK, or a negative error.  On QADC_EINVAL / QADC_ENOMEM
 *    nothing was enqueued and the outputs are untouched.  qadc_last_error()
 *    gives a thread-local message for the last failing call.
 *  - Standard code layout (Fig. 2a of the paper): code i is m/2 consecutive
 *    bytes; byte j holds component 2j in its low nibble and component 2j+1 in
 *    its high nibble (the 0x0f mask and the 4-bit shift of Alg. 2).  8-bit
 *    codes (ksub = 256) are m consecutive bytes.
 *  - Environment variables named QADC_* (QADC_SCAN_WGS, QADC_SCAN_NT, QADC_TILED,
 *    QADC_SEED_MIN_TILES, QADC_SEED_WGS, QADC_SCAN_F32_WGS, QADC_IVF_WGS, QADC_IVF_UNITS,
 *    QADC_IVF_SEED, QADC_TILED_SEED, QADC_TILED_MFMA, QADC_MFMA_MIN_Q, QADC_MFMA_MIN_Q2, QADC_MFMA_MIN_Q4,
 *    QADC_MFMA_WAVES, QADC_IVF_SEED_PARTS, QADC_IVF_SEED_PROBES, QADC_IVF_SHARED, QADC_IVF_SHARED_WGS,
 *    QADC_IVF_SHARED_MIN_PAIRS, QADC_IVF_WIDE_Q)
 *    change launch shapes, which of the equivalent kernels scans a batch and whether a
 *    sampled bound is used -- never a result.
 *    They are read once per call of an entry point and exist for tuning and for tests.
 *  - Top-R outputs: row q holds the R best of query q, ascending under the
 *    total order (distance, index) -- lowest index first among equal
 *    distances.  When fewer than R codes exist the tail is padded with index
 *    0xFFFFFFFF and distance `nbins` (u8) or +inf (f32).
 */
#ifndef QADC_H
#define QADC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QADC_OK       0
#define QADC_EINVAL  (-1)  /* bad argument: null pointer, unsupported m / ksub / R / n ... */
#define QADC_ENOMEM  (-2)  /* workspace too small */
#define QADC_EHIP    (-3)  /* a HIP runtime call failed */

#define QADC_MAX_R     1024  /* largest R accepted by the scans */
#define QADC_MAX_INIT  8192  /* largest n_init accepted by qadc_quantize_luts */

/* qmin_mode of qadc_quantize_luts */
#define QADC_QMIN_PER_TABLE 0 /* bias_j = min of table j; range starts at sum_j bias_j */
#define QADC_QMIN_GLOBAL    1 /* bias_j = min over all tables (Section 3.3, literal)  */

/* variant of qadc_scan_topk */
#define QADC_U8_4BIT    0 /* Alg. 2: 4-bit codes, uint8 tables, saturating sums      */
#define QADC_F32_4BIT   1 /* Alg. 1: 4-bit codes, float tables, float32 sums         */
#define QADC_F32_8BIT   2 /* Alg. 1: 8-bit codes (ksub = 256), float tables          */
#define QADC_U8_8BIT    3 /* Alg. 2's sums with 8-bit codes: uint8 tables of 256 entries */
#define QADC_U8_6BIT    4 /* Alg. 2's sums with 6-bit codes: uint8 tables of 64 entries  */

/* which call a workspace is for (qadc_workspace_bytes) */
#define QADC_WS_SCAN_TOPK      0 /* qadc_scan_topk, variant QADC_U8_4BIT  */
#define QADC_WS_SCAN_F32_4BIT  1 /* qadc_scan_topk, variant QADC_F32_4BIT */
#define QADC_WS_SCAN_F32_8BIT  2 /* qadc_scan_topk, variant QADC_F32_8BIT */
#define QADC_WS_SEARCH         3 /* qadc_search */
#define QADC_WS_SCAN_U8_8BIT   4 /* qadc_scan_topk, variant QADC_U8_8BIT  */
#define QADC_WS_SCAN_U8_6BIT   5 /* qadc_scan_topk, variant QADC_U8_6BIT  */

/*
 * Tables step, Eq. (1) of the paper:
 *     luts[q][j][i] = || y'_q^j - codebooks[j][i] ||^2 ,  y'_q = queries[q] - base[q]
 * for j < m sub-spaces of d/m dimensions and i < ksub centroids.  Differences and
 * their squares are summed in float64 (no norm expansion) and rounded once to float32.
 *   codebooks [m][ksub][d/m] f32   ksub in {16, 64, 256}; d % m == 0
 *   queries   [nq][d] f32
 *   base      [nq][d] f32 or NULL   (NULL: exhaustive search, y' = y;  else the
 *             centroid of the probed cell, Section 2.3 "Index")
 *   luts      [nq][m][ksub] f32     (output)
 */
int qadc_build_luts(const float *codebooks, int d, int m, int ksub,
                    const float *queries, const float *base, int nq,
                    float *luts, void *stream);

/*
 * Quantization of the tables, Section 3.3.  For each query q:
 *   qmax   = the min(R, n_init)-th smallest float ADC distance (Eq. (2), float32,
 *            increasing j) of the n_init codes `init_codes`, or qmax_in[q] when
 *            init_codes is NULL;
 *   bias_j = min_i,g luts[q][g][j][i]  (PER_TABLE)  or  min over all j too (GLOBAL);
 *   qmin   = sum_j bias_j in increasing j (PER_TABLE)  or  the global minimum (GLOBAL);
 *   delta  = (qmax - qmin) / nbins, replaced by 1 when not > 0;
 *   qluts[q][g][j][i] = min(nbins, floor(max(0, luts[q][g][j][i] - bias_j) / delta))
 * all in float32 with a correctly rounded division.
 *   luts       [nq][ngroup][m][16] f32   ngroup table sets per query share one
 *              quantizer (1 for exhaustive search; one per probed cell otherwise)
 *   init_codes [n_init][m/2] u8, standard layout, scanned with table set 0 of each
 *              query; nullable.  n_init <= QADC_MAX_INIT.
 *   qmax_in    [nq] f32, read only when init_codes is NULL (then required)
 *   nbins      1..255: number of bins n; also the saturation value (255 for
 *              unsigned bytes, 127 for the paper's signed bytes)
 *   qluts      [nq][ngroup][m][16] u8    (output)
 *   bias       [nq][m] f32               (output, nullable)
 *   delta      [nq] f32                  (output, nullable)
 *   qmax_out   [nq] f32                  (output, nullable)
 */
int qadc_quantize_luts(const float *luts, int nq, int ngroup, int m,
                       const uint8_t *init_codes, int64_t n_init, const float *qmax_in,
                       int R, int nbins, int qmin_mode,
                       uint8_t *qluts, float *bias, float *delta, float *qmax_out,
                       void *stream);

/*
 * The same quantizer for 8-bit components (the standard product quantizer of Section 2.1,
 * 256 centroids per sub-quantizer).  The paper keeps 16-entry tables because a table must fit
 * a 128-bit register (Section 3.1); here tables live in LDS, where a 256-entry table costs one
 * lookup per code byte as a pair of 16-entry tables does, so Section 3.3's quantization and
 * Alg. 2's saturating sums apply unchanged to 8-bit codes (scan variant QADC_U8_8BIT).
 *   luts [nq][ngroup][m][256] f32;  init_codes [n_init][m] u8;  m in {4, 8, 16, 32}
 *   qluts [nq][ngroup][m][256] u8 (output);  everything else as qadc_quantize_luts
 */
int qadc_quantize_luts_8bit(const float *luts, int nq, int ngroup, int m,
                            const uint8_t *init_codes, int64_t n_init, const float *qmax_in,
                            int R, int nbins, int qmin_mode,
                            uint8_t *qluts, float *bias, float *delta, float *qmax_out,
                            void *stream);

/*
 * The same quantizer for 6-bit components: 64 centroids per sub-quantizer, which the paper's
 * Conclusion names as what registers of 512 bits would allow (a 64-entry table of bytes fills
 * one).  The paper gives no layout; here the m components of a code are stored back to back,
 * least significant bit first: component j is bits 6j .. 6j+5 of the code read as one
 * little-endian number, so four components fill three bytes and a code has 3m/4 bytes.
 * Section 3.3's quantization and Alg. 2's saturating sums apply unchanged (scan variant
 * QADC_U8_6BIT); codes come from qadc_pq_encode with ksub = 64, tables from qadc_build_luts.
 *   luts [nq][ngroup][m][64] f32;  init_codes [n_init][3m/4] u8;  m in {8, 16, 32}
 *   qluts [nq][ngroup][m][64] u8 (output);  everything else as qadc_quantize_luts
 */
int qadc_quantize_luts_6bit(const float *luts, int nq, int ngroup, int m,
                            const uint8_t *init_codes, int64_t n_init, const float *qmax_in,
                            int R, int nbins, int qmin_mode,
                            uint8_t *qluts, float *bias, float *delta, float *qmax_out,
                            void *stream);

/*
 * Scan step + top-R (Alg. 1 / Alg. 2).  For every query q and code i < n:
 *   QADC_U8_4BIT   dist = min(nbins, sum_j luts_u8[q][j][c_i[j]])   (equal to the chain of
 *                  saturating adds of Alg. 2, entries being non-negative)
 *   QADC_F32_4BIT  dist = sum_j luts_f32[q][j][c_i[j]], float32, increasing j (Eq. (2))
 *   QADC_F32_8BIT  same with one byte per component and 256-entry tables
 *   QADC_U8_8BIT   dist = min(nbins, sum_j luts_u8[q][j][c_i[j]]) with one byte per component
 *                  and 256-entry uint8 tables (see qadc_quantize_luts_8bit)
 *   QADC_U8_6BIT   the same with 6-bit components, four per three bytes, and 64-entry uint8
 *                  tables (see qadc_quantize_luts_6bit); m in {8, 16, 32}; one scan per query
 * and the R smallest (dist, i) are written in ascending order.
 *   codes    [n][m/2] u8 (4-bit variants), [n][m] u8 (8-bit) or [n][3m/4] u8 (6-bit), standard layout
 *   m        4-bit variants: 8, 16, 32 or 64;  8-bit variants: 4, 8, 16 or 32
 *   luts     [nq][m][16] u8, [nq][m][16] f32, [nq][m][256] f32, [nq][m][256] u8 or [nq][m][64] u8 by variant
 *            (4-byte aligned; batches of 16-entry u8 tables that are 16-byte aligned can be
 *            scanned by the matrix-core kernel, others take the vector kernels -- same results;
 *            float tables are expected non-negative, as squared distances are)
 *   nbins    saturation value of the u8 variant (1..255); ignored otherwise
 *   R        1..QADC_MAX_R
 *   out_idx  [nq][R] u32   position i of the code in `codes`
 *   out_dist [nq][R] u8 or f32 by variant
 *   workspace  >= qadc_workspace_bytes(QADC_WS_SCAN_TOPK | _F32_4BIT | _F32_8BIT | _U8_8BIT, n, m,
 *              nq, R), by variant
 */
int qadc_scan_topk(int variant, const void *codes, int64_t n, int m,
                   const void *luts, int nq, int R, int nbins,
                   uint32_t *out_idx, void *out_dist,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Exhaustive Quick ADC search in one call: Tables (Eq. (1)), quantization of the tables
 * (Section 3.3, qmax from the first min(init, n) codes of `codes`), scan with saturating sums
 * and top-R (Alg. 2) -- the same arithmetic, operation for operation, as qadc_build_luts +
 * qadc_quantize_luts(ngroup = 1) + qadc_scan_topk(QADC_U8_4BIT), in fewer kernel launches:
 * for large databases the tables are recomputed inside the kernel that samples the codes.
 *   codebooks [m][16][d/m] f32;  queries [nq][d] f32;  codes [n][m/2] u8 (n >= 1)
 *   out_idx [nq][R] u32, out_dist [nq][R] u8 as qadc_scan_topk
 *   qluts_out [nq][m][16] u8 or NULL: the quantized tables used (output, for replay/tests)
 *   workspace >= qadc_workspace_bytes(QADC_WS_SEARCH, n, m, nq, R), cleared once as above
 */
int qadc_search(const float *codebooks, int d, int m, const float *queries, int nq,
                const uint8_t *codes, int64_t n, int R, int init, int nbins, int qmin_mode,
                uint32_t *out_idx, uint8_t *out_dist, uint8_t *qluts_out,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * qadc_search for callers that cannot allocate device memory or own no workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results as qadc_search, without the workspace: the scratch of the scan is a static device array
 * of QADC_STATIC_SCRATCH_BYTES inside the library (each GPU the entry point is used on holds its
 * own copy until the process ends).  The call allocates nothing and frees nothing.
 *   - Limit: the scratch of ONE query (qadc_workspace_bytes(QADC_WS_SEARCH, n, m, 1, R)) must fit
 *     the array, else QADC_ENOMEM and nothing is enqueued; batches larger than the array holds are
 *     cut into several launch sequences on `stream` (same results).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU -- from two
 *     streams or two threads -- race; order them on one stream.  The array is cleared by a kernel
 *     on `stream` at the first call on a GPU, at a call whose sizes (n, m, nq, R) differ from the
 *     previous call's on that GPU, and after a call that failed with QADC_EHIP; calls of one shape
 *     leave it cleared for the next.
 */
#define QADC_STATIC_SCRATCH_BYTES (32u << 20)
int qadc_search_static(const float *codebooks, int d, int m, const float *queries, int nq,
                       const uint8_t *codes, int64_t n, int R, int init, int nbins, int qmin_mode,
                       uint32_t *out_idx, uint8_t *out_dist, uint8_t *qluts_out, void *stream);
size_t qadc_static_scratch_bytes(void);

/*
 * Inverted index (Section 2.2): K cells around the coarse centroids; the codes of the
 * RESIDUALS x - centroid of a cell's vectors are stored contiguously (one inverted list per
 * cell, cell c holding storage positions list_off[c] .. list_off[c+1]-1), with the vector
 * id of every position.  The struct itself lives in HOST memory; its pointers are device
 * pointers.
 *
 * A multi-index at its usual size (far more product cells than vectors, see
 * qadc_multi_index_group) keeps lists for its occupied cells only and no table of K centroids:
 * then coarse is NULL, the K lists are the occupied cells in increasing cell id, cell_ids[s] is
 * the product cell of list s and its centroid is (halves[0][cell_ids[s] / Kh],
 * halves[1][cell_ids[s] % Kh]).  Such an index is searched with probes_in given as list numbers
 * (qadc_multi_index_probes, then qadc_multi_index_slots).  With coarse set, halves, cell_ids and Kh
 * are not read.
 */
typedef struct qadc_ivf_index {
    const float *coarse;      /* [K][d] f32 coarse centroids, or NULL (see above)    */
    const int64_t *list_off;  /* [K+1] i64, list_off[0] = 0, list_off[K] = n         */
    const uint8_t *codes;     /* [n][m/2] u8, standard layout, in list order, 16-byte aligned */
    const uint32_t *ids;      /* [n] u32 vector id of each storage position          */
    const float *codebooks;   /* [m][16][d/m] f32 product quantizer of the residuals */
    int d, m, K;
    int64_t n;
    const float *halves;      /* [2][Kh][d/2] f32 half-centroids, read when coarse is NULL */
    const uint32_t *cell_ids; /* [K] u32 ascending product cell of every list, same      */
    int Kh;                   /* half-centroids per half, same                           */
} qadc_ivf_index;

/*
 * Non-exhaustive Quick ADC search, Section 2.3 with the tables quantized as in Section 3.3.
 * For each query: Index (the nprobe closest cells by squared distance to the coarse
 * centroids, float32, closest first, ties to the lowest cell id; or the cells given in
 * probes_in), Tables (Eq. (1) on the residual y - centroid, one set of m tables per cell),
 * qmax (the min(R, n_walk)-th smallest float ADC distance of the first n_walk = min(init,
 * codes in the probed lists) codes met walking the lists in probe order, each with its own
 * cell's tables), ONE quantizer for the query shared by its nprobe table sets (as
 * qadc_quantize_luts with ngroup = nprobe), Scan of every code of every probed list with
 * saturating sums, and the R smallest under the order (sum, storage position).
 *   queries    [nq][d] f32
 *   nprobe     1..256 (the paper's `ma`); init 1..QADC_MAX_INIT; nbins 1..255; R 1..QADC_MAX_R
 *   probes_in  [nq][nprobe] i32 or NULL; a negative entry is an unused slot, and so is an entry
 *              >= K or one that repeats an earlier cell of the same query (a list is scanned once).
 *              Required (QADC_EINVAL without) when the index has no coarse centroids.
 *   out_ids    [nq][R] u32   ids[position] of the neighbours (0xFFFFFFFF padding)
 *   out_dist   [nq][R] u8    their quantized sums (nbins padding)
 *   dbg_probes [nq][nprobe] i32 or NULL: the cells scanned      (output, for replay/tests)
 *   dbg_qluts  [nq][nprobe][m][16] u8 or NULL: the tables used  (output, for replay/tests)
 *   workspace  >= qadc_ivf_workspace_bytes(ix, nq, nprobe, R), cleared once as above
 */
int qadc_ivf_search(const qadc_ivf_index *ix, const float *queries, int nq, int nprobe, int R,
                    int init, int nbins, int qmin_mode, const int32_t *probes_in,
                    uint32_t *out_ids, uint8_t *out_dist, int32_t *dbg_probes, uint8_t *dbg_qluts,
                    void *workspace, size_t workspace_bytes, void *stream);

size_t qadc_ivf_workspace_bytes(const qadc_ivf_index *ix, int nq, int nprobe, int R);

/*
 * Database side, Section 2.1: enc(x) = (i_0 .. i_{m-1}), i_j = index of the centroid of
 * sub-quantizer j closest to sub-vector x^j (float64 distances from the differences, summed in
 * increasing component order; ties to the lowest index), written in the standard layout.  Not on the query
 * path; it exists to build large databases directly in HBM.
 *   codebooks [m][ksub][d/m] f32, ksub in {16, 64, 256} (m even when ksub == 16, a multiple of 4
 *             when ksub == 64)
 *   x         [n][d] f32
 *   codes     [n][m/2] u8 (ksub 16), [n][3m/4] u8 (ksub 64: components back to back, least
 *             significant bit first) or [n][m] u8 (ksub 256)   (output)
 */
int qadc_pq_encode(const float *codebooks, int d, int m, int ksub, const float *x, int64_t n,
                   uint8_t *codes, void *stream);

/*
 * List layouts, Section 3.2 and Fig. 2.  QADC_LAYOUT_STANDARD is the layout every scan of this
 * library reads (Fig. 2a).  QADC_LAYOUT_TRANSPOSED is the paper's offline re-layout (Fig. 2b):
 * the list is cut into blocks of 16 codes and each block is stored as m/2 rows of 16 bytes, row
 * j holding byte j (components 2j and 2j+1) of the block's 16 codes in order; the last block is
 * filled with zero bytes.  qadc_pack_codes writes a list in `layout` from the standard one,
 * qadc_unpack_codes restores the standard list (a database kept in the transposed layout is
 * converted once before it is scanned here); with QADC_LAYOUT_STANDARD both are a copy.
 * qadc_packed_bytes is the size of a list of n codes in `layout` (0 on bad arguments).
 *   std_codes [n][m/2] u8;  packed [qadc_packed_bytes(n, m, layout)] u8; m in {8, 16, 32, 64};
 *   both 16-byte aligned and distinct.
 */
#define QADC_LAYOUT_STANDARD   0
#define QADC_LAYOUT_TRANSPOSED 1
size_t qadc_packed_bytes(int64_t n, int m, int layout);
int qadc_pack_codes(const uint8_t *std_codes, int64_t n, int m, int layout, uint8_t *packed,
                    void *stream);
int qadc_unpack_codes(const uint8_t *packed, int64_t n, int m, int layout, uint8_t *std_codes,
                      void *stream);

/*
 * Building an inverted index, Section 2.2 (database side, not on the query path).
 *
 * qadc_ivf_assign: cells[i] = index of the coarse centroid closest to x[i] (the vector
 * quantizer q_i; float64 distances from the differences, ties to the lowest cell).
 *   coarse [K][d] f32;  x [n][d] f32;  cells [n] i32 (output)
 *
 * qadc_ivf_group: the list order of the database, a stable grouping by cell:
 * list_off[c] = number of vectors in cells below c (list_off[K] = n) and
 * ids[list_off[c] + r] = the r-th vector of cell c in input order -- the `list_off` and `ids`
 * of qadc_ivf_index.  An entry of `cells` outside [0, K) is left out (list_off[K] < n then).
 *   cells [n] i32, n <= 2^32;  K <= 2^24;  list_off [K+1] i64 (output);  ids [n] u32 (output)
 *   workspace >= qadc_ivf_group_workspace_bytes(n, K), 16-byte aligned; it need not be cleared
 *   and is not left cleared.
 *
 * qadc_ivf_encode: the codes of the index in list order: row p encodes the residual
 * x[ids[p]] - coarse[cells[ids[p]]] (float32 subtraction) with the product quantizer
 * `codebooks` as qadc_pq_encode does (ksub = 16).  A row whose id or cell is out of range is
 * written as zero bytes.
 *   x [n][d] f32;  cells [n] i32;  ids [n_list] u32;  codes [n_list][m/2] u8 (output)
 */
int qadc_ivf_assign(const float *coarse, int K, int d, const float *x, int64_t n, int32_t *cells,
                    void *stream);
size_t qadc_ivf_group_workspace_bytes(int64_t n, int K);
int qadc_ivf_group(const int32_t *cells, int64_t n, int K, int64_t *list_off, uint32_t *ids,
                   void *workspace, size_t workspace_bytes, void *stream);
int qadc_ivf_encode(const float *coarse, int K, const float *codebooks, int d, int m, const float *x,
                    int64_t n, const int32_t *cells, const uint32_t *ids, int64_t n_list,
                    uint8_t *codes, void *stream);

/*
 * Inverted multi-index as the coarse partition (Section 5, related work: Quick ADC needs no minimum
 * list size and so combines with the finer partition of a multi-index).  The coarse quantizer is
 * the product of two quantizers of K centroids over the two halves of the vector: cell (i, j) has
 * id i*K + j and centroid (halves[0][i], halves[1][j]).  An index over those K*K cells is a
 * qadc_ivf_index: build it with qadc_multi_index_assign -> qadc_ivf_group -> qadc_ivf_encode (coarse =
 * the output of qadc_multi_index_cells) and search it with qadc_ivf_search, probes_in = the output of
 * qadc_multi_index_probes.
 *   halves [2][K][d/2] f32, K <= 16384, d even
 *
 * At the usual size of a multi-index (K = 2^14, 2^28 cells for 10^9 vectors) most cells are empty:
 * neither K*K centroids nor K*K list boundaries are stored.  qadc_multi_index_group writes the lists
 * of the occupied cells only, qadc_multi_index_encode takes the residuals from the half-centroids,
 * the qadc_ivf_index carries halves and cell_ids in place of coarse, and qadc_multi_index_slots turns
 * the cells of qadc_multi_index_probes into list numbers (an empty cell becomes an unused slot).
 *
 * qadc_multi_index_cells:  coarse[i*K + j] = (halves[0][i], halves[1][j]);  coarse [K*K][d] f32 (output;
 *   K*K*d < 2^39)
 * qadc_multi_index_assign: cells[v] = K * (closest of halves[0] to the first half of x[v]) + (closest
 *   of halves[1] to its second half), float64 distances, ties to the lowest;  x [n][d];  cells [n] i32
 * qadc_multi_index_probes: probes[q] = the nprobe (<= 256) cells with the smallest d1[i] + d2[j],
 *   smallest first, equal sums by cell id; d1, d2 = float32 squared distances of the query's halves to
 *   the half-centroids (summed in increasing component).  Found from the min(nprobe, K) closest
 *   half-centroids of each half, never from the K*K sums.  Slots beyond K*K cells are -1.
 *   queries [nq][d] f32, nq <= 65535;  probes [nq][nprobe] i32 (output)
 *   workspace >= qadc_multi_index_workspace_bytes(K, nq, nprobe) (0: unsupported arguments),
 *   16-byte aligned; it need not be cleared.
 * qadc_multi_index_group: the list order of a database over the occupied cells: a stable sort of
 *   the vectors by cell id.  n_lists[0] = L = number of distinct cells in `cells`; cell_ids[0..L-1] =
 *   those cells, ascending; list_off[s] = number of vectors in cells below cell_ids[s], list_off[L] =
 *   number of vectors placed; ids[list_off[s] + r] = the r-th vector of cell cell_ids[s] in input
 *   order.  An entry of `cells` outside [0, K*K) is left out.
 *   cells [n] i32, n <= 2^32;  max_lists >= min(n, K*K): the capacity of cell_ids [max_lists] u32
 *   and list_off [max_lists + 1] i64 (outputs, device);  ids [n] u32 (output);  n_lists [1] i64
 *   (output, device);  workspace >= qadc_multi_index_group_workspace_bytes(n, K) (0: unsupported),
 *   16-byte aligned; it need not be cleared.
 * qadc_multi_index_encode: codes[p] = the code of x[ids[p]] - (halves[0][c / K], halves[1][c % K]),
 *   c = cells[ids[p]], float32 subtraction, encoded as qadc_ivf_encode does (ksub = 16, m even: a
 *   sub-vector lies in one half).  A row whose id or cell is out of range is written as zero bytes.
 *   x [n][d] f32;  cells [n] i32;  ids [n_list] u32;  codes [n_list][m/2] u8 (output)
 * qadc_multi_index_slots: slots[e] = s with cell_ids[s] == cells[e], or -1 when no list has that
 *   cell (or cells[e] < 0).  cell_ids [n_lists] u32 ascending;  cells, slots [count] i32 (slots is
 *   the output; the two may be the same array)
 */
int qadc_multi_index_cells(const float *halves, int K, int d, float *coarse, void *stream);
int qadc_multi_index_assign(const float *halves, int K, int d, const float *x, int64_t n, int32_t *cells,
                            void *stream);
size_t qadc_multi_index_workspace_bytes(int K, int nq, int nprobe);
int qadc_multi_index_probes(const float *halves, int K, int d, const float *queries, int nq, int nprobe,
                            int32_t *probes, void *workspace, size_t workspace_bytes, void *stream);
size_t qadc_multi_index_group_workspace_bytes(int64_t n, int K);
int qadc_multi_index_group(const int32_t *cells, int64_t n, int K, int64_t max_lists, uint32_t *cell_ids,
                           int64_t *list_off, uint32_t *ids, int64_t *n_lists, void *workspace,
                           size_t workspace_bytes, void *stream);
int qadc_multi_index_encode(const float *halves, int K, const float *codebooks, int d, int m, const float *x,
                            int64_t n, const int32_t *cells, const uint32_t *ids, int64_t n_list,
                            uint8_t *codes, void *stream);
int qadc_multi_index_slots(const uint32_t *cell_ids, int64_t n_lists, const int32_t *cells, int64_t count,
                           int32_t *slots, void *stream);

/*
 * Rotation of an optimized product quantizer, Section 2.1: opq(x) = pq(R x), R^T R = I.
 *     y[i][r] = sum_t rot[r][t] * x[i][t]
 * with products and sums in float64 in increasing t and one rounding to float32.  At query time
 * it precedes the Tables step (its cost belongs to that step, Section 4.3): rotate the queries,
 * then call qadc_build_luts / qadc_search / qadc_ivf_search with the rotated queries and the
 * codebooks trained on rotated data.  The same call rotates database vectors before
 * qadc_pq_encode.  The library does not check that rot is orthonormal.
 *   rot [d][d] f32;  x [n][d] f32;  y [n][d] f32 (output; must not overlap x)
 */
int qadc_rotate(const float *rot, int d, const float *x, int64_t n, float *y, void *stream);

/*
 * Per-kernel timing for benchmarks (the paper reports Index / Tables / Scan times
 * separately, Section 4.3).  While enabled, the library launches the kernels named
 * below with a start and a stop HIP event attached to each dispatch (the kernel's own
 * duration on its stream); qadc_profile_read waits for the recorded events and
 * returns the summed duration and the number of launches since profiling was enabled.
 * Process-wide state, not thread-safe; host pointers.
 */
#define QADC_PROF_SCAN   0  /* code-streaming kernel of qadc_scan_topk */
#define QADC_PROF_MERGE  1  /* cross-workgroup top-R kernel of qadc_scan_topk */
#define QADC_PROF_SEED   2  /* kernels that sample the codes for the bound of a scan (large inputs only) */
#define QADC_PROF_IVF_INDEX  3  /* Index step of qadc_ivf_search (coarse distances, cell choice) */
#define QADC_PROF_IVF_TABLES 4  /* Tables step of qadc_ivf_search (tables, qmax, quantization)   */
#define QADC_PROF_TABLES     5  /* qadc_build_luts kernel */
#define QADC_PROF_QUANTIZE   6  /* qadc_quantize_luts kernel */
#define QADC_PROF_PREPARE    7  /* tables + quantizer + sampling kernel of qadc_search */
#define QADC_PROF_ROTATE     8  /* qadc_rotate kernel */
#define QADC_PROF_IVF_SHARED 9  /* shared-list scan kernel of qadc_ivf_search (large batches) */
#define QADC_PROF_COUNT  10
int qadc_profile_enable(int on);
/* As qadc_profile_enable(1), but only the kernels of slot `which` carry events: their neighbours in
 * the stream are launched as in an untimed run. */
int qadc_profile_only(int which);
int qadc_profile_read(int which, double *total_ms, int64_t *launches);

/*
 * Database side, Section 2.1: trains the m codebooks of a product quantizer, each by
 * `iters` iterations of Lloyd's k-means on the matching sub-vectors of the learning set,
 * started from the sub-vectors of the ksub rows `init_rows`.  An iteration assigns each
 * sub-vector to its closest centroid (float64 distances from the differences, ties to the
 * lowest index) and replaces each centroid by the mean of its sub-vectors (float64 sum in
 * row order, stored as float32; a centroid that owns nothing keeps its value).
 *   train      [n][d] f32
 *   init_rows  [ksub] i64 distinct row numbers (device); a number outside [0, n) is clamped
 *   codebooks  [m][ksub][d/m] f32   (output)
 *   workspace  >= n * m bytes
 */
int qadc_pq_train(const float *train, int64_t n, int d, int m, int ksub, const int64_t *init_rows,
                  int iters, float *codebooks, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace a call needs (0 when it needs none, or on bad arguments). */
size_t qadc_workspace_bytes(int call, int64_t n, int m, int nq, int R);

/*
 * Clears a workspace (asynchronous memset on `stream`).  Required before the first call
 * that uses the workspace and before a call of another shape (see the conventions at the
 * top); a call leaves the workspace ready for the next call of its own shape.  Do not
 * record it into a HIP graph: clear the workspace before capture.
 */
int qadc_workspace_init(void *workspace, size_t bytes, void *stream);

/* Message of the last failing call on this thread ("" when none). */
const char *qadc_last_error(void);

/* Library version string. */
const char *qadc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* QADC_H */
