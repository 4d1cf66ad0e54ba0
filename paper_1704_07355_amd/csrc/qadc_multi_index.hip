// Inverted multi-index as the coarse partition (the finer partition the paper's related-work
// section proposes to combine with Quick ADC, which needs no minimum list size).
//
// The coarse quantizer is the product of two quantizers of K centroids over the two halves of
// the vector: cell (i, j), id i*K + j, has the centroid (halves[0][i], halves[1][j]) and the
// distance of a query to it is d1[i] + d2[j].  After the Index step everything is the inverted
// index search over K*K cells (qadc_ivf_search with the probes given), so this file holds only
//
//   cells    the K*K centroids written out, the `coarse` of a qadc_ivf_index (small K only);
//   probes   the nprobe cells with the smallest d1[i] + d2[j] without forming the K*K sums;
//   slots    the list number of a cell in an index that keeps lists for its occupied cells only.
//
// probes: 2K half distances per query (float32, summed in increasing component with one fused
// multiply-add each, as the Index step of the inverted index), the T = min(nprobe, K) smallest
// of each half in order, then the pairs of ranks (a, b) with (a+1)(b+1) <= nprobe -- a cell
// outside that corner has at least nprobe cells in front of it, every pair of lower ranks -- whose
// sums are ranked exactly under (sum, cell id).  That corner holds about nprobe * ln(nprobe)
// pairs; the multi-sequence algorithm visits the same corner one cell at a time from a priority
// queue, which a workgroup replaces by ranking all of it at once.

#include "qadc_scan_common.h"
#include <algorithm>

namespace qadc {

void ivf_select_smallest(const float *dist, int rows, int K, int count, int32_t *out, hipStream_t st);

constexpr int MI_MAX_K = 16384;      // K*K cells <= 2^28: a cell id fits an int32
constexpr int MI_MAX_NPROBE = 256;   // as qadc_ivf_search
constexpr int MI_MAX_PAIRS = 2048;   // sum over a of floor(256 / a) = 1546

// coarse[(i*K + j)][t] = t < dh ? halves[0][i][t] : halves[1][j][t - dh]
__global__ __launch_bounds__(256) void mi_cells_kernel(const float *__restrict__ halves, int K, int dh,
                                                       float *__restrict__ coarse, int64_t total)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int d = 2 * dh;
    const int64_t cell = e / d;
    const int t = (int)(e % d);
    const int i = (int)(cell / K), j = (int)(cell % K);
    coarse[e] = t < dh ? halves[((size_t)i) * dh + t] : halves[((size_t)K + j) * dh + (t - dh)];
}

// hd[(q*2 + h)][i] = sum_t (y[q][h*dh + t] - halves[h][i][t])^2, float32, increasing t, one fused
// multiply-add per component.  Grid (ceil(K / 256), 2, nq); the query's half sits in LDS.
__global__ __launch_bounds__(256) void mi_half_dist_kernel(const float *__restrict__ halves, int K, int dh,
                                                           const float *__restrict__ queries, int nq,
                                                           float *__restrict__ hd)
{
    extern __shared__ float yh[];  // [dh]
    const int h = blockIdx.y, q = blockIdx.z;
    const float *y = queries + (size_t)q * (2 * dh) + (size_t)h * dh;
    for (int t = threadIdx.x; t < dh; t += 256) yh[t] = y[t];
    __syncthreads();
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= K) return;
    const float *c = halves + ((size_t)h * K + i) * dh;
    float acc = 0.0f;
    for (int t = 0; t < dh; ++t) {
        const float df = yh[t] - c[t];
        acc = __builtin_fmaf(df, df, acc);
    }
    hd[((size_t)q * 2 + h) * K + i] = acc;
}

// One workgroup per query.  top[(q*2 + h)][r] = the half-centroid of rank r of half h.  The
// candidate pairs are laid out by rank a of the first half: row a holds b = 0 .. nb(a)-1,
// nb(a) = min(T, nprobe / (a+1)).  Keys order(sum) << 32 | cell are unique, so a key's rank among
// the candidates is its place among the probes.
__global__ __launch_bounds__(256) void mi_combine_kernel(const float *__restrict__ hd,
                                                         const int32_t *__restrict__ top, int K, int T,
                                                         int nprobe, int32_t *__restrict__ probes)
{
    __shared__ uint64_t keys[MI_MAX_PAIRS];
    __shared__ float d1[MI_MAX_NPROBE], d2[MI_MAX_NPROBE];
    __shared__ int c1[MI_MAX_NPROBE], c2[MI_MAX_NPROBE];
    __shared__ int row_off[MI_MAX_NPROBE + 1];
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    for (int r = tid; r < T; r += 256) {
        const int a = top[((size_t)q * 2) * T + r], b = top[((size_t)q * 2 + 1) * T + r];
        c1[r] = a;
        c2[r] = b;
        d1[r] = hd[((size_t)q * 2) * K + a];
        d2[r] = hd[((size_t)q * 2 + 1) * K + b];
    }
    for (int a = tid; a < T; a += 256) row_off[a + 1] = min(T, nprobe / (a + 1));  // sizes first
    __syncthreads();
    if (tid == 0) {
        row_off[0] = 0;
        for (int a = 0; a < T; ++a) row_off[a + 1] += row_off[a];
    }
    __syncthreads();
    const int P = row_off[T];  // <= MI_MAX_PAIRS (checked on the host)
    for (int p = tid; p < P; p += 256) {
        int lo = 0, hi = T - 1;  // the row a with row_off[a] <= p < row_off[a + 1]
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (row_off[mid] <= p) lo = mid; else hi = mid - 1;
        }
        const int a = lo, b = p - row_off[lo];
        const float sum = d1[a] + d2[b];
        keys[p] = ((uint64_t)f2ord(sum) << 32) | (uint64_t)(unsigned)(c1[a] * K + c2[b]);
    }
    __syncthreads();
    const int need = min(nprobe, P);
    for (int p = tid; p < P; p += 256) {
        const uint64_t k = keys[p];
        int rank = 0;
        for (int o = 0; o < P; ++o) rank += (keys[o] < k) ? 1 : 0;
        if (rank < need) probes[(size_t)q * nprobe + rank] = (int32_t)(unsigned)k;
    }
    for (int r = need + tid; r < nprobe; r += 256) probes[(size_t)q * nprobe + r] = -1;  // fewer cells than probes
}

int multi_index_cells(const float *halves, int K, int d, float *coarse, hipStream_t st)
{
    if (K < 1 || K > MI_MAX_K || d < 2 || (d & 1))
        return fail(QADC_EINVAL, "qadc_multi_index_cells: K=%d d=%d", K, d);
    if (!halves || !coarse) return fail(QADC_EINVAL, "qadc_multi_index_cells: null pointer");
    const int64_t total = (int64_t)K * K * d;
    const int64_t grid = ceil_div(total, 256);
    if (grid > 0x7fffffffll) return fail(QADC_EINVAL, "qadc_multi_index_cells: K*K*d too large");
    hipLaunchKernelGGL(mi_cells_kernel, dim3((unsigned)grid), dim3(256), 0, st, halves, K, d / 2, coarse, total);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

static int mi_pairs(int T, int nprobe)
{
    int p = 0;
    for (int a = 0; a < T; ++a) p += std::min(T, nprobe / (a + 1));
    return p;
}

struct MiPlan {
    int T;
    size_t hd_off, top_off, total;
};

static bool mi_plan(int K, int nq, int nprobe, MiPlan *p)
{
    if (K < 1 || K > MI_MAX_K || nq < 1 || nq > 65535 || nprobe < 1 || nprobe > MI_MAX_NPROBE) return false;
    p->T = std::min(nprobe, K);
    if (mi_pairs(p->T, nprobe) > MI_MAX_PAIRS) return false;
    p->hd_off = 0;
    p->top_off = align_up((size_t)nq * 2 * K * sizeof(float), 256);
    p->total = p->top_off + align_up((size_t)nq * 2 * p->T * sizeof(int32_t), 256);
    return true;
}

size_t multi_index_workspace(int K, int nq, int nprobe)
{
    MiPlan p;
    return mi_plan(K, nq, nprobe, &p) ? p.total : 0;
}

int multi_index_probes(const float *halves, int K, int d, const float *queries, int nq, int nprobe,
                       int32_t *probes, void *workspace, size_t workspace_bytes, hipStream_t st)
{
    if (nq == 0) return QADC_OK;
    MiPlan p;
    if (d < 2 || (d & 1) || d / 2 > 8192 || !mi_plan(K, nq, nprobe, &p))
        return fail(QADC_EINVAL, "qadc_multi_index_probes: K=%d d=%d nq=%d nprobe=%d", K, d, nq, nprobe);
    if (!halves || !queries || !probes || !workspace)
        return fail(QADC_EINVAL, "qadc_multi_index_probes: null pointer");
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
        return fail(QADC_EINVAL, "qadc_multi_index_probes: workspace not 16-byte aligned");
    if (workspace_bytes < p.total)
        return fail(QADC_ENOMEM, "qadc_multi_index_probes: workspace of %zu bytes, %zu needed", workspace_bytes,
                    p.total);
    char *ws = static_cast<char *>(workspace);
    float *hd = reinterpret_cast<float *>(ws + p.hd_off);
    int32_t *top = reinterpret_cast<int32_t *>(ws + p.top_off);
    const int dh = d / 2;
    launch(QADC_PROF_IVF_INDEX, mi_half_dist_kernel, dim3((unsigned)ceil_div(K, 256), 2, (unsigned)nq), dim3(256),
           (size_t)dh * sizeof(float), st, halves, K, dh, queries, nq, hd);
    ivf_select_smallest(hd, 2 * nq, K, p.T, top, st);
    launch(QADC_PROF_IVF_INDEX, mi_combine_kernel, dim3((unsigned)nq), dim3(256), 0, st, (const float *)hd,
           (const int32_t *)top, K, p.T, nprobe, probes);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

// slots[e] = place of cells[e] in the ascending cell_ids, -1 when it is not there
__global__ __launch_bounds__(256) void mi_slots_kernel(const uint32_t *__restrict__ cell_ids, int64_t n_lists,
                                                       const int32_t *__restrict__ cells, int64_t count,
                                                       int32_t *__restrict__ slots)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    const int32_t c = cells[e];
    int32_t out = -1;
    if (c >= 0 && n_lists > 0) {
        int64_t lo = 0, hi = n_lists - 1;  // first place whose cell is >= c
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (cell_ids[mid] < (uint32_t)c) lo = mid + 1; else hi = mid;
        }
        if (cell_ids[lo] == (uint32_t)c) out = (int32_t)lo;
    }
    slots[e] = out;
}

int multi_index_slots(const uint32_t *cell_ids, int64_t n_lists, const int32_t *cells, int64_t count,
                      int32_t *slots, hipStream_t st)
{
    if (n_lists < 0 || n_lists > 0x7fffffffll || count < 0)
        return fail(QADC_EINVAL, "qadc_multi_index_slots: n_lists=%lld count=%lld", (long long)n_lists,
                    (long long)count);
    if (count == 0) return QADC_OK;
    if (!cells || !slots || (n_lists > 0 && !cell_ids)) return fail(QADC_EINVAL, "qadc_multi_index_slots: null pointer");
    const int64_t grid = ceil_div(count, 256);
    if (grid > 0x7fffffffll) return fail(QADC_EINVAL, "qadc_multi_index_slots: count too large for one call");
    launch(QADC_PROF_IVF_INDEX, mi_slots_kernel, dim3((unsigned)grid), dim3(256), 0, st, cell_ids, n_lists, cells,
           count, slots);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
