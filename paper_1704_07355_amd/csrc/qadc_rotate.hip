// Rotation of an optimized product quantizer on gfx950 (Section 2.1 of the paper):
// opq(x) = pq(R x) with R orthonormal.  y[i][r] = sum_t R[r][t] * x[i][t], products and sums in
// float64 in increasing t, one rounding to float32 -- the arithmetic of the Tables step, so that
// a rotated query loses nothing before its tables are computed.  At query time this is part of
// the Tables step (Section 4.3 counts it there); the same kernel rotates the database vectors
// before they are encoded.
//
// Many vectors (database side, query batches): a small blocked matrix product on the vector ALU; a
// workgroup of 256 threads computes a tile of 64 vectors x 64 outputs, 16 components of t at a
// time through LDS, 4 x 4 outputs per thread.  A few vectors (queries one at a time): one
// wavefront per output, the lanes split t and their partial sums are added by a butterfly, so
// that a query's rotation is one round trip to memory instead of d / 16 of them.

#include "qadc_common.h"
#include "qadc_profile.h"
#include "qadc.h"

namespace qadc {

constexpr int ROT_TM = 64;  // vectors per workgroup
constexpr int ROT_TN = 64;  // outputs per workgroup
constexpr int ROT_TK = 16;  // components per step

__global__ __launch_bounds__(256) void rotate_kernel(const float *__restrict__ rot, int d,
                                                     const float *__restrict__ x, int64_t n,
                                                     float *__restrict__ y)
{
    __shared__ double xs[ROT_TK][ROT_TM + 1];
    __shared__ double rs[ROT_TK][ROT_TN + 1];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;  // outputs 4*tx.., vectors 4*ty..
    const int64_t i0 = (int64_t)blockIdx.y * ROT_TM;
    const int r0 = blockIdx.x * ROT_TN;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

    for (int t0 = 0; t0 < d; t0 += ROT_TK) {
        // 64 x 16 elements of x and of R, four of each per thread, zero beyond the edges
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + e * 256;
            const int row = idx >> 4, col = idx & 15;  // row: vector / output, col: component
            const int t = t0 + col;
            const int64_t i = i0 + row;
            const int r = r0 + row;
            xs[col][row] = (i < n && t < d) ? (double)x[i * d + t] : 0.0;
            rs[col][row] = (r < d && t < d) ? (double)rot[(size_t)r * d + t] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < ROT_TK; ++kk) {
            double xv[4], rv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) xv[a] = xs[kk][4 * ty + a];
#pragma unroll
            for (int b = 0; b < 4; ++b) rv[b] = rs[kk][4 * tx + b];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fma(xv[a], rv[b], acc[a][b]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int64_t i = i0 + 4 * ty + a;
        if (i >= n) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int r = r0 + 4 * tx + b;
            if (r < d) y[i * d + r] = (float)acc[a][b];
        }
    }
}

// y[i][r] for r = 4 * blockIdx.x + wave, i = blockIdx.y: lane l adds the components t = l, l + 64,
// ... in increasing t, then the 64 partial sums are added pairwise.
__global__ __launch_bounds__(256) void rotate_few_kernel(const float *__restrict__ rot, int d,
                                                         const float *__restrict__ x,
                                                         float *__restrict__ y)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t i = blockIdx.y;
    if (r >= d) return;  // whole wave
    const float *xr = x + i * d;
    const float *rr = rot + (size_t)r * d;
    double acc = 0.0;
    for (int t = lane; t < d; t += 64) acc = fma((double)rr[t], (double)xr[t], acc);
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
    if (lane == 0) y[i * d + r] = (float)acc;
}

constexpr int ROT_FEW = 32;  // up to this many vectors take the one-wavefront-per-output kernel

int rotate(const float *rot, int d, const float *x, int64_t n, float *y, hipStream_t st)
{
    if (d < 1 || n < 0) return fail(QADC_EINVAL, "qadc_rotate: d=%d n=%lld", d, (long long)n);
    if (n == 0) return QADC_OK;
    if (!rot || !x || !y) return fail(QADC_EINVAL, "qadc_rotate: null pointer");
    if (x == y) return fail(QADC_EINVAL, "qadc_rotate: x and y must not overlap");
    if (n <= ROT_FEW) {
        launch(QADC_PROF_ROTATE, rotate_few_kernel, dim3((unsigned)ceil_div(d, 4), (unsigned)n), dim3(256), 0, st,
               rot, d, x, y);
        QADC_HIP_TRY(hipGetLastError());
        return QADC_OK;
    }
    const int64_t gy = ceil_div(n, ROT_TM);
    if (gy > 65535) {  // the y dimension of a grid is 16 bits wide: rows in slabs
        const int64_t slab = 65535ll * ROT_TM;
        for (int64_t s = 0; s < n; s += slab) {
            const int rc = rotate(rot, d, x + s * d, std::min(slab, n - s), y + s * d, st);
            if (rc != QADC_OK) return rc;
        }
        return QADC_OK;
    }
    launch(QADC_PROF_ROTATE, rotate_kernel, dim3((unsigned)ceil_div(d, ROT_TN), (unsigned)gy), dim3(256), 0, st,
           rot, d, x, n, y);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
