// Database side of product quantization on gfx950 (Section 2.1 of the paper):
// enc(x) = (i_0 .. i_{m-1}), i_j = argmin_i || x^j - C^j[i] ||^2, written in the
// standard code layout.  Used to build large synthetic databases in HBM; it is
// not on the query path.

#include "qadc_common.h"

namespace qadc {

// One thread per output byte.  ksub == 16: the byte holds components 2jb (low
// nibble) and 2jb+1 (high nibble); ksub == 256: the byte is component jb.
// Distances in float32 from the differences; ties go to the lowest index.
template <int KSUB>
__global__ __launch_bounds__(256) void pq_encode_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ x, int64_t n,
    uint8_t *__restrict__ codes)
{
    const int dsub = d / m;
    const int row = (KSUB == 16) ? m / 2 : m;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * row) return;
    const int64_t r = gid / row;
    const int jb = (int)(gid - r * row);
    const int ncomp = (KSUB == 16) ? 2 : 1;
    unsigned out = 0;
    for (int h = 0; h < ncomp; ++h) {
        const int j = (KSUB == 16) ? 2 * jb + h : jb;
        const float *xs = x + r * d + (int64_t)j * dsub;
        const float *cb = codebooks + (size_t)j * KSUB * dsub;
        float best = __builtin_inff();
        unsigned arg = 0;
        for (int i = 0; i < KSUB; ++i) {
            float acc = 0.0f;
            for (int t = 0; t < dsub; ++t) {
                const float df = xs[t] - cb[i * dsub + t];
                acc += df * df;
            }
            if (acc < best) { best = acc; arg = (unsigned)i; }
        }
        out |= arg << (4 * h);
    }
    codes[gid] = (uint8_t)out;
}

int pq_encode(const float *codebooks, int d, int m, int ksub, const float *x, int64_t n,
              uint8_t *codes, hipStream_t st)
{
    if (!codebooks || !x || !codes) return fail(QADC_EINVAL, "qadc_pq_encode: null pointer");
    if (m < 1 || d % m != 0 || (ksub != 16 && ksub != 256) || (ksub == 16 && (m & 1)) || n < 0)
        return fail(QADC_EINVAL, "qadc_pq_encode: unsupported d=%d m=%d ksub=%d", d, m, ksub);
    if (n == 0) return QADC_OK;
    const int64_t total = n * (ksub == 16 ? m / 2 : m);
    const int64_t blocks = ceil_div(total, 256);
    if (blocks > 0x7fffffffll) return fail(QADC_EINVAL, "qadc_pq_encode: n too large for one call");
    if (ksub == 16)
        hipLaunchKernelGGL(pq_encode_kernel<16>, dim3((unsigned)blocks), dim3(256), 0, st, codebooks, d,
                           m, x, n, codes);
    else
        hipLaunchKernelGGL(pq_encode_kernel<256>, dim3((unsigned)blocks), dim3(256), 0, st, codebooks,
                           d, m, x, n, codes);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
