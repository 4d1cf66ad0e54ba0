// Database side of product quantization on gfx950 (Section 2.1 of the paper):
// enc(x) = (i_0 .. i_{m-1}), i_j = argmin_i || x^j - C^j[i] ||^2, written in the
// standard code layout; for an inverted index (Section 2.2) the vector encoded at storage
// position p is the residual x[ids[p]] - coarse[cells[ids[p]]].  Not on the query path.

#include "qadc_common.h"

namespace qadc {

// Where the centroids of the cells come from: a table of K rows, or the two half-quantizers of a
// multi-index (cell c = i*Kh + j, centroid (halves[0][i], halves[1][j]); with m even a sub-vector
// lies inside one half).  `off` = first dimension of the sub-vector.
struct CellCentroids {
    const float *coarse;
    const float *halves;
    int K;   // cells: ids outside [0, K) are invalid
    int Kh;
};

__device__ inline const float *centroid_part(const CellCentroids &cc, int c, int off, int d)
{
    if (cc.coarse) return cc.coarse + (size_t)c * d + off;
    const int dh = d >> 1;
    const int i = c / cc.Kh, j = c - i * cc.Kh;
    return off < dh ? cc.halves + (size_t)i * dh + off : cc.halves + ((size_t)cc.Kh + j) * dh + (off - dh);
}

// One thread per output byte.  ksub == 16: the byte holds components 2jb (low
// nibble) and 2jb+1 (high nibble); ksub == 256: the byte is component jb.
// Distances in float64 from the float32 differences' exact values, summed in increasing t with
// separate multiply and add; ties go to the lowest index.  With `coarse`, row r of the output
// encodes the float32 residual of vector ids[r].
template <int KSUB>
__global__ __launch_bounds__(256) void pq_encode_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ x, int64_t n,
    uint8_t *__restrict__ codes, CellCentroids cc, const int32_t *__restrict__ cells,
    const uint32_t *__restrict__ ids, int64_t n_x)
{
#pragma clang fp contract(off)
    const int dsub = d / m;
    const int row = (KSUB == 16) ? m / 2 : m;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * row) return;
    const int64_t r = gid / row;
    const int jb = (int)(gid - r * row);
    const int64_t src = ids ? (int64_t)ids[r] : r;
    const bool resid = cc.coarse || cc.halves;
    int c = 0;
    if (resid) {  // an id or a cell out of range: a zero byte, no access
        if (src >= n_x) { codes[gid] = 0; return; }
        c = cells[src];
        if (c < 0 || c >= cc.K) { codes[gid] = 0; return; }
    }
    const int ncomp = (KSUB == 16) ? 2 : 1;
    unsigned out = 0;
    for (int h = 0; h < ncomp; ++h) {
        const int j = (KSUB == 16) ? 2 * jb + h : jb;
        const float *xs = x + src * d + (int64_t)j * dsub;
        const float *bs = resid ? centroid_part(cc, c, j * dsub, d) : nullptr;
        const float *cb = codebooks + (size_t)j * KSUB * dsub;
        double best = __builtin_inf();
        unsigned arg = 0;
        for (int i = 0; i < KSUB; ++i) {
            double acc = 0.0;
            for (int t = 0; t < dsub; ++t) {
                const float xv = bs ? xs[t] - bs[t] : xs[t];
                const double df = (double)xv - (double)cb[i * dsub + t];
                acc += df * df;
            }
            if (acc < best) { best = acc; arg = (unsigned)i; }
        }
        out |= arg << (4 * h);
    }
    codes[gid] = (uint8_t)out;
}

// ksub == 64 (6-bit components): one thread per group of four components = three output bytes;
// component j is bits 6j .. 6j+5 of the code read as a little-endian number.  Arithmetic as above.
__global__ __launch_bounds__(256) void pq_encode6_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ x, int64_t n,
    uint8_t *__restrict__ codes)
{
#pragma clang fp contract(off)
    const int dsub = d / m;
    const int groups = m / 4;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * groups) return;
    const int64_t r = gid / groups;
    const int gq = (int)(gid - r * groups);
    unsigned out = 0;
    for (int h = 0; h < 4; ++h) {
        const int j = 4 * gq + h;
        const float *xs = x + r * d + (int64_t)j * dsub;
        const float *cb = codebooks + (size_t)j * 64 * dsub;
        double best = __builtin_inf();
        unsigned arg = 0;
        for (int i = 0; i < 64; ++i) {
            double acc = 0.0;
            for (int t = 0; t < dsub; ++t) {
                const double df = (double)xs[t] - (double)cb[i * dsub + t];
                acc += df * df;
            }
            if (acc < best) { best = acc; arg = (unsigned)i; }
        }
        out |= arg << (6 * h);
    }
    uint8_t *o = codes + r * (int64_t)(3 * groups) + 3 * gq;
    o[0] = (uint8_t)out;
    o[1] = (uint8_t)(out >> 8);
    o[2] = (uint8_t)(out >> 16);
}

// ksub == 16 with the codebooks in LDS as [j][t][16] floats: one thread per output byte; for each
// component it reads x^j[t] once and advances the 16 distances together, each still summed in
// increasing t.  Same arithmetic and result as pq_encode_kernel<16>.
__global__ __launch_bounds__(256) void pq_encode16_lds_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ x, int64_t n,
    uint8_t *__restrict__ codes, CellCentroids cc, const int32_t *__restrict__ cells,
    const uint32_t *__restrict__ ids, int64_t n_x)
{
#pragma clang fp contract(off)
    extern __shared__ __attribute__((aligned(16))) float cbt[];   // [m][dsub][16]
    const int dsub = d / m;
    for (int e = threadIdx.x; e < d * 16; e += 256) {
        const int j = e / (16 * dsub), rem = e - j * 16 * dsub;   // codebooks[j][i][t]
        const int i = rem / dsub, t = rem - i * dsub;
        cbt[(j * dsub + t) * 16 + i] = codebooks[e];
    }
    __syncthreads();
    const int row = m / 2;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * row) return;
    const int64_t r = gid / row;
    const int jb = (int)(gid - r * row);
    const int64_t src = ids ? (int64_t)ids[r] : r;
    const bool resid = cc.coarse || cc.halves;
    int c = 0;
    if (resid) {
        if (src >= n_x) { codes[gid] = 0; return; }
        c = cells[src];
        if (c < 0 || c >= cc.K) { codes[gid] = 0; return; }
    }
    unsigned out = 0;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int j = 2 * jb + h;
        const float *xs = x + src * d + (int64_t)j * dsub;
        const float *bs = resid ? centroid_part(cc, c, j * dsub, d) : nullptr;
        double acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.0;
        for (int t = 0; t < dsub; ++t) {
            const float xv = bs ? xs[t] - bs[t] : xs[t];
            const float4 *c4 = reinterpret_cast<const float4 *>(cbt + (j * dsub + t) * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 c = c4[q];
                const float cv[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const double df = (double)xv - (double)cv[k];
                    acc[4 * q + k] += df * df;
                }
            }
        }
        double best = __builtin_inf();
        unsigned arg = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (acc[i] < best) { best = acc[i]; arg = (unsigned)i; }
        out |= arg << (4 * h);
    }
    codes[gid] = (uint8_t)out;
}

static int encode_launch(const char *name, const float *codebooks, int d, int m, int ksub, const float *x,
                         int64_t n, uint8_t *codes, CellCentroids cc, const int32_t *cells,
                         const uint32_t *ids, int64_t n_x, hipStream_t st)
{
    if (m < 1 || d < 1 || d % m != 0 || (ksub != 16 && ksub != 64 && ksub != 256) || (ksub == 16 && (m & 1)) ||
        (ksub == 64 && ((m & 3) || cc.coarse || cc.halves)) || n < 0)
        return fail(QADC_EINVAL, "%s: unsupported d=%d m=%d ksub=%d", name, d, m, ksub);
    if (n == 0) return QADC_OK;
    if (!codebooks || !x || !codes) return fail(QADC_EINVAL, "%s: null pointer", name);
    if (ksub == 64) {
        const int64_t blocks6 = ceil_div(n * (m / 4), 256);
        if (blocks6 > 0x7fffffffll) return fail(QADC_EINVAL, "%s: n too large for one call", name);
        hipLaunchKernelGGL(pq_encode6_kernel, dim3((unsigned)blocks6), dim3(256), 0, st, codebooks, d, m, x, n, codes);
        QADC_HIP_TRY(hipGetLastError());
        return QADC_OK;
    }
    const int64_t total = n * (ksub == 16 ? m / 2 : m);
    const int64_t blocks = ceil_div(total, 256);
    if (blocks > 0x7fffffffll) return fail(QADC_EINVAL, "%s: n too large for one call", name);
    if (ksub == 16 && (size_t)d * 64 <= 65536)
        hipLaunchKernelGGL(pq_encode16_lds_kernel, dim3((unsigned)blocks), dim3(256), (size_t)d * 64, st,
                           codebooks, d, m, x, n, codes, cc, cells, ids, n_x);
    else if (ksub == 16)
        hipLaunchKernelGGL(pq_encode_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, st, codebooks, d,
                           m, x, n, codes, cc, cells, ids, n_x);
    else
        hipLaunchKernelGGL(pq_encode_kernel<256>, dim3((unsigned)blocks), dim3(256), 0, st, codebooks,
                           d, m, x, n, codes, cc, cells, ids, n_x);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

int pq_encode(const float *codebooks, int d, int m, int ksub, const float *x, int64_t n,
              uint8_t *codes, hipStream_t st)
{
    return encode_launch("qadc_pq_encode", codebooks, d, m, ksub, x, n, codes, CellCentroids{nullptr, nullptr, 0, 0},
                         nullptr, nullptr, n, st);
}

// codes[p] = enc(x[ids[p]] - coarse[cells[ids[p]]]) for the n_list storage positions p
int ivf_encode(const float *coarse, int K, const float *codebooks, int d, int m, const float *x, int64_t n,
               const int32_t *cells, const uint32_t *ids, int64_t n_list, uint8_t *codes, hipStream_t st)
{
    if (K < 1 || n < 0) return fail(QADC_EINVAL, "qadc_ivf_encode: K=%d n=%lld", K, (long long)n);
    if (n_list > 0 && (!coarse || !cells || !ids)) return fail(QADC_EINVAL, "qadc_ivf_encode: null pointer");
    return encode_launch("qadc_ivf_encode", codebooks, d, m, 16, x, n_list, codes,
                         CellCentroids{coarse, nullptr, K, 0}, cells, ids, n, st);
}

// codes[p] = enc(x[ids[p]] - (halves[0][c / Kh], halves[1][c % Kh])), c = cells[ids[p]]
int multi_index_encode(const float *halves, int Kh, const float *codebooks, int d, int m, const float *x,
                       int64_t n, const int32_t *cells, const uint32_t *ids, int64_t n_list, uint8_t *codes,
                       hipStream_t st)
{
    if (Kh < 1 || Kh > 16384 || n < 0 || d < 2 || (d & 1))
        return fail(QADC_EINVAL, "qadc_multi_index_encode: K=%d d=%d n=%lld", Kh, d, (long long)n);
    if (n_list > 0 && (!halves || !cells || !ids)) return fail(QADC_EINVAL, "qadc_multi_index_encode: null pointer");
    return encode_launch("qadc_multi_index_encode", codebooks, d, m, 16, x, n_list, codes,
                         CellCentroids{nullptr, halves, Kh * Kh, Kh}, cells, ids, n, st);
}

}  // namespace qadc
