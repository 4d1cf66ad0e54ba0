// qadc_search_static: the exhaustive search of qadc_search for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops): the scratch of the scan lives in a
// file-scope device array instead of a caller's workspace.  Everything else -- kernels, plans,
// results -- is qadc_search's.

#include <mutex>

#include "qadc_scan_common.h"

namespace qadc {

int search_u8(const float *, int, int, const float *, int, const uint8_t *, int64_t, int, int, int, int,
              uint32_t *, uint8_t *, uint8_t *, void *, size_t, hipStream_t);
size_t search_workspace(int64_t, int, int, int);

constexpr size_t STATIC_SCRATCH_BYTES = 32ull << 20;
static_assert(STATIC_SCRATCH_BYTES == QADC_STATIC_SCRATCH_BYTES, "header and library disagree");

// One copy per GPU, at an address of its own on each: host code never uses this name as a pointer,
// only the address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

__global__ void static_scratch_clear_kernel(uint4 *p, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        p[i] = make_uint4(0, 0, 0, 0);
}

namespace {
constexpr int MAX_DEVICES = 64;
struct DeviceScratch {
    void *ptr = nullptr;   // device address of `scratch` on this GPU
    bool clean = false;    // control words known to be zero where the next call of the shape below keeps them
    // shape of the last call: a call of another shape lays the array out differently, and the table
    // data the last one left may lie where the new one keeps its control words
    int64_t n = -1;
    int m = 0, nb = 0, R = 0;
};
DeviceScratch g_dev[MAX_DEVICES];
std::mutex g_mu;
}  // namespace

int search_static(const float *codebooks, int d, int m, const float *queries, int nq,
                  const uint8_t *codes, int64_t n, int R, int init, int nbins, int qmin_mode,
                  uint32_t *out_idx, uint8_t *out_dist, uint8_t *qluts_out, hipStream_t st)
{
    knobs_refresh();
    if (nq < 0) return fail(QADC_EINVAL, "qadc_search_static: nq=%d", nq);
    if (nq == 0) return QADC_OK;
    // the largest number of queries per launch sequence whose scratch fits the array
    int nb = nq;
    size_t need = search_workspace(n, m, nb, R);
    if (need == 0)
        return fail(QADC_EINVAL, "qadc_search_static: unsupported n=%lld m=%d nq=%d R=%d", (long long)n, m, nq, R);
    while (need > STATIC_SCRATCH_BYTES && nb > 1) {
        nb = (nb + 1) / 2;
        need = search_workspace(n, m, nb, R);
        if (need == 0)
            return fail(QADC_EINVAL, "qadc_search_static: unsupported n=%lld m=%d nq=%d R=%d", (long long)n, m, nb, R);
    }
    if (need > STATIC_SCRATCH_BYTES)
        return fail(QADC_ENOMEM,
                    "qadc_search_static: one query over n=%lld m=%d R=%d needs %zu bytes of scratch, the static "
                    "array holds %zu: use qadc_search with a workspace",
                    (long long)n, m, R, need, (size_t)STATIC_SCRATCH_BYTES);

    int dev = 0;
    QADC_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(QADC_EINVAL, "qadc_search_static: device %d", dev);
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceScratch &ds = g_dev[dev];
    if (!ds.ptr) {
        void *p = nullptr;
        QADC_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255) != 0)
            return fail(QADC_EHIP, "qadc_search_static: bad address %p for the scratch array", p);
        ds.ptr = p;
    }
    if (ds.n != n || ds.m != m || ds.nb != nb || ds.R != R) ds.clean = false;
    ds.n = n; ds.m = m; ds.nb = nb; ds.R = R;
    if (!ds.clean) {
        // first call on this GPU, a call of a new shape, or a call failed part-way: a fill kernel, not
        // a memset node, so that a caller may capture the call into a graph
        hipLaunchKernelGGL(static_scratch_clear_kernel, dim3(2048), dim3(256), 0, st, (uint4 *)ds.ptr,
                           STATIC_SCRATCH_BYTES / 16);
        QADC_HIP_TRY(hipGetLastError());
        ds.clean = true;
    }
    for (int q0 = 0; q0 < nq; q0 += nb) {
        const int cnt = min(nb, nq - q0);
        const int rc = search_u8(codebooks, d, m, queries + (size_t)q0 * d, cnt, codes, n, R, init, nbins,
                                 qmin_mode, out_idx + (size_t)q0 * R, out_dist + (size_t)q0 * R,
                                 qluts_out ? qluts_out + (size_t)q0 * m * 16 : nullptr, ds.ptr,
                                 STATIC_SCRATCH_BYTES, st);
        if (rc != QADC_OK) {
            if (rc == QADC_EHIP) ds.clean = false;  // kernels may have run: clear before the next use
            return rc;
        }
    }
    return QADC_OK;
}

}  // namespace qadc

extern "C" {

int qadc_search_static(const float *codebooks, int d, int m, const float *queries, int nq,
                       const uint8_t *codes, int64_t n, int R, int init, int nbins, int qmin_mode,
                       uint32_t *out_idx, uint8_t *out_dist, uint8_t *qluts_out, void *stream)
{
    return qadc::search_static(codebooks, d, m, queries, nq, codes, n, R, init, nbins, qmin_mode, out_idx,
                               out_dist, qluts_out, (hipStream_t)stream);
}

size_t qadc_static_scratch_bytes(void) { return qadc::STATIC_SCRATCH_BYTES; }

}  // extern "C"
