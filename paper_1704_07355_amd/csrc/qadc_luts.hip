// Tables step (Eq. (1) of the paper) and 8-bit quantization of the tables
// (Section 3.3) on gfx950.  Both are tiny next to the scan: one workgroup per
// query, everything staged in LDS.

#include "qadc_scan_common.h"

namespace qadc {

// ------------------------------------------------------------------ Eq. (1)

// luts[q][j][i] = sum_t (y[q][j*dsub+t] - base[q][j*dsub+t] - C[j][i][t])^2.
// Differences and the sum are taken in float64 and rounded once to float32, so
// a residual query (y - base) loses nothing to an intermediate rounding.
__global__ __launch_bounds__(256) void build_luts_kernel(
    const float *__restrict__ codebooks, int d, int m, int ksub, const float *__restrict__ queries,
    const float *__restrict__ base, float *__restrict__ luts)
{
    extern __shared__ double yq[];  // [d]
    const int q = blockIdx.x;
    const int dsub = d / m;
    for (int t = threadIdx.x; t < d; t += blockDim.x) {
        double y = (double)queries[(size_t)q * d + t];
        if (base) y -= (double)base[(size_t)q * d + t];
        yq[t] = y;
    }
    __syncthreads();
    const int entries = m * ksub;
    for (int e = threadIdx.x; e < entries; e += blockDim.x) {
        const int j = e / ksub;
        const float *c = codebooks + (size_t)e * dsub;
        const double *y = yq + j * dsub;
        double acc = 0.0;
        for (int t = 0; t < dsub; ++t) {
            const double df = y[t] - (double)c[t];
            acc += df * df;
        }
        luts[(size_t)q * entries + e] = (float)acc;
    }
}

int build_luts(const float *codebooks, int d, int m, int ksub, const float *queries,
               const float *base, int nq, float *luts, hipStream_t st)
{
    if (!codebooks || !queries || !luts) return fail(QADC_EINVAL, "qadc_build_luts: null pointer");
    if (m < 1 || d < m || d % m != 0 || (ksub != 16 && ksub != 64 && ksub != 256) || nq < 0 || d > 8192)
        return fail(QADC_EINVAL, "qadc_build_luts: unsupported d=%d m=%d ksub=%d nq=%d", d, m, ksub, nq);
    if (nq == 0) return QADC_OK;
    launch(QADC_PROF_TABLES, build_luts_kernel, dim3(nq), dim3(256), (size_t)d * sizeof(double), st,
           codebooks, d, m, ksub, queries, base, luts);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

// -------------------------------------------------------------- Section 3.3

constexpr int QUANT_NT = 1024;
constexpr int QUANT_MAX_M = 64;

// KSUB = 16: 4-bit components, two per code byte (the paper's case).  KSUB = 256: 8-bit components,
// one per code byte, the same quantizer applied to the 256-entry tables of Section 2.1's
// standard product quantizer.  KSUB = 64: 6-bit components (the paper's Conclusion), stored back to
// back, least significant bit first, four per three bytes.
template <int KSUB>
__global__ __launch_bounds__(QUANT_NT) void quantize_luts_kernel(
    const float *__restrict__ luts, int ngroup, int m, const uint8_t *__restrict__ init_codes,
    int n_init, const float *__restrict__ qmax_in, int R, int nbins, int qmin_mode,
    uint8_t *__restrict__ qluts, float *__restrict__ bias_out, float *__restrict__ delta_out,
    float *__restrict__ qmax_out)
{
    __shared__ float lut0[QUANT_MAX_M * 16];
    __shared__ unsigned cand[QADC_MAX_INIT];
    __shared__ unsigned bias_ord[QUANT_MAX_M];
    __shared__ float bias[QUANT_MAX_M];
    __shared__ float delta_s;
    __shared__ SelectScratch sc;

    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    constexpr int LOG = KSUB == 16 ? 4 : KSUB == 64 ? 6 : 8;
    const int entries = m * KSUB;
    const float *lq = luts + (size_t)q * ngroup * entries;

    if (KSUB == 16)
        for (int e = tid; e < entries; e += QUANT_NT) lut0[e] = lq[e];
    for (int j = tid; j < m; j += QUANT_NT) bias_ord[j] = 0xffffffffu;
    __syncthreads();

    // qmax: R-th smallest float ADC distance (Eq. (2), float32, increasing j) of the init codes
    float qmax;
    if (init_codes) {
        const int B = KSUB == 16 ? m / 2 : KSUB == 64 ? 3 * m / 4 : m;
        for (int i = tid; i < n_init; i += QUANT_NT) {
            const uint8_t *c = init_codes + (size_t)i * B;
            float acc = 0.0f;
            if (KSUB == 64) {
                for (int j = 0; j < m; ++j) {
                    const int bit = 6 * j, k = bit >> 3, sh = bit & 7;
                    unsigned v = c[k];
                    if (sh > 2) v |= (unsigned)c[k + 1] << 8;  // the field crosses into the next byte
                    acc = acc + lq[j * 64 + ((v >> sh) & 63u)];  // the first table set
                }
            } else
            for (int jb = 0; jb < B; ++jb) {
                const unsigned comps = c[jb];
                if (KSUB == 16) {
                    acc = acc + lut0[(2 * jb) * 16 + (comps & 15u)];
                    acc = acc + lut0[(2 * jb + 1) * 16 + (comps >> 4)];
                } else {
                    acc = acc + lq[jb * 256 + comps];  // the first table set; cached after the first touch
                }
            }
            cand[i] = f2ord(acc);
        }
        __syncthreads();
        const unsigned need = (unsigned)min(R, n_init);
        qmax = ord2f(block_radix_select<unsigned, 4>(cand, (unsigned)n_init, need, &sc));
    } else {
        qmax = qmax_in[q];
    }

    // bias_j = minimum of table j over every table set of the query.  A thread meets the same
    // table positions in every set (entries and the thread count divide one another): minimum in
    // a register first, one LDS atomic per position.
    if (entries >= QUANT_NT) {
        for (int pos = tid; pos < entries; pos += QUANT_NT) {
            unsigned mn = 0xffffffffu;
#pragma unroll 8
            for (int g = 0; g < ngroup; ++g) mn = min(mn, f2ord(lq[(size_t)g * entries + pos]));
            atomicMin(&bias_ord[pos >> LOG], mn);
        }
    } else {
        const int pos = tid % entries;
        unsigned mn = 0xffffffffu;
#pragma unroll 8
        for (int g = tid / entries; g < ngroup; g += QUANT_NT / entries)
            mn = min(mn, f2ord(lq[(size_t)g * entries + pos]));
        atomicMin(&bias_ord[pos >> LOG], mn);
    }
    __syncthreads();
    if (tid == 0) {
        float qmin;
        if (qmin_mode == QADC_QMIN_GLOBAL) {
            unsigned g = 0xffffffffu;
            for (int j = 0; j < m; ++j) g = min(g, bias_ord[j]);
            qmin = ord2f(g);
            for (int j = 0; j < m; ++j) bias[j] = qmin;
        } else {
            qmin = 0.0f;
            for (int j = 0; j < m; ++j) {
                bias[j] = ord2f(bias_ord[j]);
                qmin = qmin + bias[j];
            }
        }
        float delta = __fdiv_rn(qmax - qmin, (float)nbins);
        if (!(delta > 0.0f)) delta = 1.0f;
        delta_s = delta;
        if (delta_out) delta_out[q] = delta;
        if (qmax_out) qmax_out[q] = qmax;
    }
    __syncthreads();
    const float delta = delta_s;
    if (bias_out)
        for (int j = tid; j < m; j += QUANT_NT) bias_out[(size_t)q * m + j] = bias[j];

    const float top = (float)nbins;
    uint8_t *qq = qluts + (size_t)q * ngroup * entries;
#pragma unroll 4
    for (int e = tid; e < ngroup * entries; e += QUANT_NT) {
        const float off = fmaxf(0.0f, lq[e] - bias[(e % entries) >> LOG]);
        const float t = floorf(__fdiv_rn(off, delta));
        qq[e] = (t < top) ? (uint8_t)t : (uint8_t)nbins;
    }
}

int quantize_luts(int ksub, const float *luts, int nq, int ngroup, int m, const uint8_t *init_codes,
                  int64_t n_init, const float *qmax_in, int R, int nbins, int qmin_mode,
                  uint8_t *qluts, float *bias, float *delta, float *qmax_out, hipStream_t st)
{
    if (!luts || !qluts) return fail(QADC_EINVAL, "qadc_quantize_luts: null pointer");
    const int mm = ksub == 256 ? 2 * m : m;  // 8-bit components: m in {4, 8, 16, 32}
    if (!(mm == 8 || mm == 16 || mm == 32 || (mm == 64 && ksub != 64)) || nq < 0 || ngroup < 1)
        return fail(QADC_EINVAL, "qadc_quantize_luts: unsupported m=%d nq=%d ngroup=%d", m, nq, ngroup);
    if (nbins < 1 || nbins > 255 || R < 1)
        return fail(QADC_EINVAL, "qadc_quantize_luts: nbins=%d R=%d", nbins, R);
    if (qmin_mode != QADC_QMIN_PER_TABLE && qmin_mode != QADC_QMIN_GLOBAL)
        return fail(QADC_EINVAL, "qadc_quantize_luts: qmin_mode=%d", qmin_mode);
    if (init_codes) {
        if (n_init < 1 || n_init > QADC_MAX_INIT)
            return fail(QADC_EINVAL, "qadc_quantize_luts: n_init=%lld not in 1..%d", (long long)n_init,
                        QADC_MAX_INIT);
    } else if (!qmax_in) {
        return fail(QADC_EINVAL, "qadc_quantize_luts: neither init_codes nor qmax_in given");
    }
    if (nq == 0) return QADC_OK;
    if (ksub == 16)
        launch(QADC_PROF_QUANTIZE, quantize_luts_kernel<16>, dim3(nq), dim3(QUANT_NT), 0, st, luts, ngroup, m,
               init_codes, (int)n_init, qmax_in, R, nbins, qmin_mode, qluts, bias, delta, qmax_out);
    else if (ksub == 64)
        launch(QADC_PROF_QUANTIZE, quantize_luts_kernel<64>, dim3(nq), dim3(QUANT_NT), 0, st, luts, ngroup, m,
               init_codes, (int)n_init, qmax_in, R, nbins, qmin_mode, qluts, bias, delta, qmax_out);
    else
        launch(QADC_PROF_QUANTIZE, quantize_luts_kernel<256>, dim3(nq), dim3(QUANT_NT), 0, st, luts, ngroup, m,
               init_codes, (int)n_init, qmax_in, R, nbins, qmin_mode, qluts, bias, delta, qmax_out);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
