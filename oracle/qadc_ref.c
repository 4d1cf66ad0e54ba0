/*
 * Plain scalar C twin of the CPU oracle -- TEST INFRASTRUCTURE, not product.
 *
 * Same steps as oracle/qadc_oracle.py, written as straight loops so that the
 * large parity cases (10^7 codes and more) and the CPU-baseline timing finish
 * in seconds.  No intrinsics, no blocking, no reordering: one code at a time,
 * tables in increasing j.  It shares nothing with the HIP library.
 *
 * Paper: "Accelerated Nearest Neighbor Search with Quick ADC" (ICMR'17).
 *   Section 2.1  enc(x) = argmin_i ||x^j - C^j[i]||, codes of m*b bits
 *   Eq. (2)      adc(y,c) = sum_j D^j[c[j]]
 *   Alg. 1       scan with a binary heap of size R
 *   Alg. 2       mask 0x0f / lookup / saturating add / shift right 4
 *
 * Standard layout (Fig. 2a): code i is m/2 bytes, byte j = c[2j] | c[2j+1] << 4.
 * Top-R: the R smallest under the total order (distance, index), ascending;
 * missing entries: index 0xFFFFFFFF, distance `cap` (u8) or +inf (f32).
 * Parallelism: one query per thread (Section 3.1), nothing else.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ encode */

/* Section 2.1: one sub-quantizer index per sub-space, float64 distances, ties
 * to the lowest index.  ksub == 16: two indices per byte (standard layout);
 * ksub == 256: one byte per index.  x [n][d], codebooks [m][ksub][d/m]. */
void ref_pq_encode(const float *x, int64_t n, int d, int m, int ksub,
                   const float *codebooks, uint8_t *codes)
{
    const int dsub = d / m;
    const int row = (ksub == 16) ? m / 2 : m;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n; ++r) {
        uint8_t *out = codes + r * row;
        if (ksub == 16) memset(out, 0, (size_t)row);
        for (int j = 0; j < m; ++j) {
            const float *xs = x + r * d + j * dsub;
            int best = 0;
            double bestd = INFINITY;
            for (int i = 0; i < ksub; ++i) {
                const float *c = codebooks + ((size_t)j * ksub + i) * dsub;
                double acc = 0.0;
                for (int t = 0; t < dsub; ++t) {
                    double df = (double)xs[t] - (double)c[t];
                    acc += df * df;
                }
                if (acc < bestd) { bestd = acc; best = i; }
            }
            if (ksub == 16) out[j >> 1] |= (uint8_t)(best << ((j & 1) * 4));
            else out[j] = (uint8_t)best;
        }
    }
}

/* ------------------------------------------------------------- distances */

/* Alg. 2 quick_adc_block for one code: per byte, low nibble -> table 2j,
 * saturating add, shift right four, -> table 2j+1, saturating add. */
static inline unsigned qadc_one(const uint8_t *code, int m, const uint8_t *qlut, unsigned cap)
{
    unsigned acc = 0;
    for (int j = 0; j < m / 2; ++j) {
        unsigned comps = code[j];
        unsigned masked = comps & 0x0f;
        acc += qlut[(2 * j) * 16 + masked];
        if (acc > cap) acc = cap;
        comps >>= 4;
        masked = comps & 0x0f;
        acc += qlut[(2 * j + 1) * 16 + masked];
        if (acc > cap) acc = cap;
    }
    return acc;
}

/* The same chain for 6-bit components: component j is bits 6j .. 6j+5 of the code read as a
 * little-endian number; one 64-entry table per component. */
static inline unsigned sixbit_at(const uint8_t *code, int j)
{
    unsigned c = 0;
    for (int b = 0; b < 6; ++b) {
        const int bit = 6 * j + b;
        c |= ((code[bit >> 3] >> (bit & 7)) & 1u) << b;
    }
    return c;
}

static inline unsigned qadc_one_sixbit(const uint8_t *code, int m, const uint8_t *qlut, unsigned cap)
{
    unsigned acc = 0;
    for (int j = 0; j < m; ++j) {
        acc += qlut[j * 64 + sixbit_at(code, j)];
        if (acc > cap) acc = cap;
    }
    return acc;
}

/* The same chain for 8-bit components (one byte, one 256-entry table per component). */
static inline unsigned qadc_one_bytes(const uint8_t *code, int m, const uint8_t *qlut, unsigned cap)
{
    unsigned acc = 0;
    for (int j = 0; j < m; ++j) {
        acc += qlut[j * 256 + code[j]];
        if (acc > cap) acc = cap;
    }
    return acc;
}

/* Eq. (2) in float32, increasing j.  ksub 16 (nibbles) or 256 (bytes). */
static inline float adc_one(const uint8_t *code, int m, int ksub, const float *lut)
{
    float acc = 0.0f;
    if (ksub == 16) {
        for (int j = 0; j < m; ++j) {
            unsigned c = (code[j >> 1] >> ((j & 1) * 4)) & 0x0f;
            acc += lut[j * 16 + c];
        }
    } else {
        for (int j = 0; j < m; ++j) acc += lut[j * ksub + code[j]];
    }
    return acc;
}

void ref_scan_u8(const uint8_t *codes, int64_t n, int m, const uint8_t *qlut, int cap,
                 uint8_t *sums)
{
    for (int64_t i = 0; i < n; ++i)
        sums[i] = (uint8_t)qadc_one(codes + i * (m / 2), m, qlut, (unsigned)cap);
}

void ref_adc_f32(const uint8_t *codes, int64_t n, int m, int ksub, const float *lut, float *out)
{
    const int row = (ksub == 16) ? m / 2 : m;
    for (int64_t i = 0; i < n; ++i) out[i] = adc_one(codes + i * row, m, ksub, lut);
}

/* --------------------------------------------------- binary heap of size R */

/* Max-heap on (distance, index): the root is the worst neighbour kept.  A new
 * pair enters when the heap is not full or when it is smaller than the root. */
typedef struct { double d; int64_t i; } pair_t;

static inline int pair_less(pair_t a, pair_t b)
{
    return a.d < b.d || (a.d == b.d && a.i < b.i);
}

static void heap_push(pair_t *h, int *len, int R, pair_t p)
{
    if (*len < R) {
        int k = (*len)++;
        h[k] = p;
        while (k > 0) {
            int par = (k - 1) / 2;
            if (!pair_less(h[par], h[k])) break;
            pair_t t = h[par]; h[par] = h[k]; h[k] = t;
            k = par;
        }
        return;
    }
    if (!pair_less(p, h[0])) return;
    h[0] = p;
    int k = 0;
    for (;;) {
        int l = 2 * k + 1, r = l + 1, big = k;
        if (l < R && pair_less(h[big], h[l])) big = l;
        if (r < R && pair_less(h[big], h[r])) big = r;
        if (big == k) break;
        pair_t t = h[big]; h[big] = h[k]; h[k] = t;
        k = big;
    }
}

static int pair_cmp(const void *a, const void *b)
{
    pair_t x = *(const pair_t *)a, y = *(const pair_t *)b;
    return pair_less(x, y) ? -1 : pair_less(y, x) ? 1 : 0;
}

/* ----------------------------------------------------------- scan + top-R */

/* Alg. 2 quick_adc_scan for nq queries over the same n codes; qluts
 * [nq][m][16]; out_idx [nq][R] u32, out_dist [nq][R] u8. */
void ref_scan_topk_u8(const uint8_t *codes, int64_t n, int m, const uint8_t *qluts, int nq,
                      int cap, int R, uint32_t *out_idx, uint8_t *out_dist)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        pair_t *h = (pair_t *)malloc(sizeof(pair_t) * (size_t)R);
        int len = 0;
        const uint8_t *qlut = qluts + (size_t)q * m * 16;
        for (int64_t i = 0; i < n; ++i) {
            pair_t p = { (double)qadc_one(codes + i * (m / 2), m, qlut, (unsigned)cap), i };
            heap_push(h, &len, R, p);
        }
        qsort(h, (size_t)len, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < R; ++r) {
            out_idx[(size_t)q * R + r] = r < len ? (uint32_t)h[r].i : 0xFFFFFFFFu;
            out_dist[(size_t)q * R + r] = r < len ? (uint8_t)h[r].d : (uint8_t)cap;
        }
        free(h);
    }
}

/* Saturating scan of 8-bit codes [n][m] with quantized tables qluts [nq][m][256]. */
void ref_scan_topk_u8_bytes(const uint8_t *codes, int64_t n, int m, const uint8_t *qluts, int nq,
                            int cap, int R, uint32_t *out_idx, uint8_t *out_dist)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        pair_t *h = (pair_t *)malloc(sizeof(pair_t) * (size_t)R);
        int len = 0;
        const uint8_t *qlut = qluts + (size_t)q * m * 256;
        for (int64_t i = 0; i < n; ++i) {
            pair_t p = { (double)qadc_one_bytes(codes + i * m, m, qlut, (unsigned)cap), i };
            heap_push(h, &len, R, p);
        }
        qsort(h, (size_t)len, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < R; ++r) {
            out_idx[(size_t)q * R + r] = r < len ? (uint32_t)h[r].i : 0xFFFFFFFFu;
            out_dist[(size_t)q * R + r] = r < len ? (uint8_t)h[r].d : (uint8_t)cap;
        }
        free(h);
    }
}

/* Saturating scan of 6-bit codes [n][3m/4] with quantized tables qluts [nq][m][64]. */
void ref_scan_topk_u8_sixbit(const uint8_t *codes, int64_t n, int m, const uint8_t *qluts, int nq,
                             int cap, int R, uint32_t *out_idx, uint8_t *out_dist)
{
    const int nbytes = 3 * m / 4;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        pair_t *h = (pair_t *)malloc(sizeof(pair_t) * (size_t)R);
        int len = 0;
        const uint8_t *qlut = qluts + (size_t)q * m * 64;
        for (int64_t i = 0; i < n; ++i) {
            pair_t p = { (double)qadc_one_sixbit(codes + i * nbytes, m, qlut, (unsigned)cap), i };
            heap_push(h, &len, R, p);
        }
        qsort(h, (size_t)len, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < R; ++r) {
            out_idx[(size_t)q * R + r] = r < len ? (uint32_t)h[r].i : 0xFFFFFFFFu;
            out_dist[(size_t)q * R + r] = r < len ? (uint8_t)h[r].d : (uint8_t)cap;
        }
        free(h);
    }
}

/* Alg. 1 scan in float32 for nq queries; luts [nq][m][ksub]. */
void ref_scan_topk_f32(const uint8_t *codes, int64_t n, int m, int ksub, const float *luts,
                       int nq, int R, uint32_t *out_idx, float *out_dist)
{
    const int row = (ksub == 16) ? m / 2 : m;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        pair_t *h = (pair_t *)malloc(sizeof(pair_t) * (size_t)R);
        int len = 0;
        const float *lut = luts + (size_t)q * m * ksub;
        for (int64_t i = 0; i < n; ++i) {
            pair_t p = { (double)adc_one(codes + i * row, m, ksub, lut), i };
            heap_push(h, &len, R, p);
        }
        qsort(h, (size_t)len, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < R; ++r) {
            out_idx[(size_t)q * R + r] = r < len ? (uint32_t)h[r].i : 0xFFFFFFFFu;
            out_dist[(size_t)q * R + r] = r < len ? (float)h[r].d : INFINITY;
        }
        free(h);
    }
}
