// Product-quantizer training on gfx950 (Section 2.1 of the paper: one k-centroid codebook
// per sub-space, each a Lloyd k-means).  Database side, not on the query path: it exists so
// that large synthetic databases can be trained, encoded and searched without leaving HBM.
//
// One iteration = assign every learning vector's sub-vector to its closest centroid
// (float64 distances from the differences, ties to the lowest index), then replace each
// centroid by the mean of its sub-vectors (float64 sum in row order, stored as float32);
// a centroid that owns nothing keeps its value.  No atomics: the result is deterministic.

#include "qadc_common.h"

namespace qadc {

// A row number outside [0, n) is clamped to the nearest row: nothing outside `train` is read.
__global__ void train_init_kernel(const float *__restrict__ train, int64_t n, int d, int m, int ksub,
                                  const int64_t *__restrict__ init_rows, float *__restrict__ cb)
{
    const int dsub = d / m;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;  // (j, i, t)
    if (e >= m * ksub * dsub) return;
    const int t = e % dsub, i = (e / dsub) % ksub, j = e / (dsub * ksub);
    const int64_t row = min(max(init_rows[i], (int64_t)0), n - 1);
    cb[e] = train[row * d + j * dsub + t];
}

__global__ void train_assign_kernel(const float *__restrict__ train, int64_t n, int d, int m, int ksub,
                                    const float *__restrict__ cb, uint8_t *__restrict__ labels)
{
    const int dsub = d / m;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // (r, j)
    if (gid >= n * m) return;
    const int64_t r = gid / m;
    const int j = (int)(gid - r * m);
    const float *xs = train + r * d + j * dsub;
    const float *c = cb + (size_t)j * ksub * dsub;
    double best = __builtin_inf();
    int arg = 0;
    for (int i = 0; i < ksub; ++i) {
        double acc = 0.0;
        for (int t = 0; t < dsub; ++t) {
            const double df = (double)xs[t] - (double)c[i * dsub + t];
            acc += df * df;
        }
        if (acc < best) { best = acc; arg = i; }
    }
    labels[gid] = (uint8_t)arg;
}

__global__ void train_update_kernel(const float *__restrict__ train, int64_t n, int d, int m, int ksub,
                                    const uint8_t *__restrict__ labels, float *__restrict__ cb)
{
    const int dsub = d / m;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;  // (j, i, t)
    if (e >= m * ksub * dsub) return;
    const int t = e % dsub, i = (e / dsub) % ksub, j = e / (dsub * ksub);
    double sum = 0.0;
    int64_t cnt = 0;
    for (int64_t r = 0; r < n; ++r) {
        if (labels[r * m + j] == (uint8_t)i) {
            sum += (double)train[r * d + j * dsub + t];
            ++cnt;
        }
    }
    if (cnt) cb[e] = (float)(sum / (double)cnt);
}

int pq_train(const float *train, int64_t n, int d, int m, int ksub, const int64_t *init_rows, int iters,
             float *codebooks, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    if (!train || !init_rows || !codebooks) return fail(QADC_EINVAL, "qadc_pq_train: null pointer");
    if (m < 1 || d < m || d % m != 0 || (ksub != 16 && ksub != 64 && ksub != 256) || n < 1 || iters < 0)
        return fail(QADC_EINVAL, "qadc_pq_train: unsupported n=%lld d=%d m=%d ksub=%d iters=%d",
                    (long long)n, d, m, ksub, iters);
    if (!workspace || workspace_bytes < (size_t)n * m)
        return fail(QADC_ENOMEM, "qadc_pq_train: workspace %zu < %zu bytes", workspace_bytes, (size_t)n * m);
    uint8_t *labels = (uint8_t *)workspace;
    const int entries = m * ksub * (d / m);
    hipLaunchKernelGGL(train_init_kernel, dim3((unsigned)ceil_div(entries, 256)), dim3(256), 0, st, train,
                       n, d, m, ksub, init_rows, codebooks);
    for (int it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(train_assign_kernel, dim3((unsigned)ceil_div(n * m, 256)), dim3(256), 0, st,
                           train, n, d, m, ksub, codebooks, labels);
        hipLaunchKernelGGL(train_update_kernel, dim3((unsigned)ceil_div(entries, 64)), dim3(64), 0, st,
                           train, n, d, m, ksub, labels, codebooks);
    }
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
