// Alg. 1 of the paper on gfx950: the float ADC scan, adc(y, c) = sum_j D^j[c[j]] (Eq. (2)),
// added in float32 in increasing j, for 4-bit codes (16-entry tables) and for the usual
// 8-bit codes (256-entry tables), with exact top-R under the order (distance, index).
//
// This is the reference the quantized scan is compared against (recall, speed).  The float
// tables of the query sit in LDS (1 KiB for 16x4, 8 KiB for 8x8: the sizes of the paper's
// Table 1); codes are streamed as in the quantized scan.  A candidate key is
// order(distance) << 32 | index among the workgroup's codes; each workgroup keeps an LDS
// list that is cut back to its R smallest keys by an exact radix select whenever it fills,
// and reports at most R keys; the merge kernel orders the R smallest of all of them.

#include "qadc_scan_common.h"

namespace qadc {

constexpr int F32_NT = 512;

struct F32Shared {
    SelectScratch sel;
    unsigned ccnt;
    unsigned tcnt[3];
};

// KSUB = 16: ROW = m/2 bytes per code, two components per byte; KSUB = 256: ROW = m bytes.
template <int KSUB, int ROW>
__global__ __launch_bounds__(F32_NT) void scan_f32_kernel(
    const uint8_t *__restrict__ codes, int64_t n, const float *__restrict__ luts, int R,
    char *__restrict__ ws, size_t ws_stride, size_t counts_off, size_t lists_off)
{
    constexpr int NT = F32_NT;
    using C = ScanCfg<ROW, NT>;
    constexpr int M = (KSUB == 16) ? 2 * ROW : ROW;
    __shared__ float lut[M * KSUB];
    __shared__ uint64_t keys[C::CAP];
    __shared__ F32Shared sh;

    const int tid = threadIdx.x;
    const int q = blockIdx.y;
    const int g = blockIdx.x;
    const int64_t G = gridDim.x;
    if ((int64_t)g * C::TILE >= n) return;  // uniform

    const float *lq = luts + (size_t)q * M * KSUB;
    for (int e = tid; e < M * KSUB; e += NT) lut[e] = lq[e];
    if (tid == 0) sh.tcnt[0] = 0;
    __syncthreads();

    uint64_t lim = ~0ull;  // keys >= lim cannot be among the R best of this workgroup's codes
    unsigned have = 0;
    int rot = 0;
    unsigned rel = 0;
    for (int64_t t0 = (int64_t)g * C::TILE; t0 < n; t0 += G * C::TILE, rel += C::TILE) {
        unsigned *ctr = &sh.tcnt[rot];
        const int nxt = (rot == 2) ? 0 : rot + 1;
        if (tid == 0) sh.tcnt[nxt] = 0;
        uint4 w[2];
        int nc[2];
        tile_load<ROW, NT>(codes, t0, n, w, nc);

        uint64_t k[C::CPT];
        if constexpr (ROW <= 16) {
            constexpr int CPV = 16 / ROW;
#pragma unroll
            for (int v = 0; v < 2; ++v) {
#pragma unroll
                for (int c = 0; c < CPV; ++c) {
                    float acc = 0.0f;
#pragma unroll
                    for (int jb = 0; jb < ROW; ++jb) {
                        const unsigned b = byte_of(w[v], c * ROW + jb);
                        if constexpr (KSUB == 16) {
                            acc = acc + lut[(2 * jb) * 16 + (b & 15u)];
                            acc = acc + lut[(2 * jb + 1) * 16 + (b >> 4)];
                        } else {
                            acc = acc + lut[jb * 256 + b];
                        }
                    }
                    const unsigned li = rel + (unsigned)((v * NT + tid) * CPV + c);
                    k[v * CPV + c] = (c < nc[v]) ? (((uint64_t)f2ord(acc) << 32) | li) : ~0ull;
                }
            }
        } else {
            float acc = 0.0f;
#pragma unroll
            for (int jb = 0; jb < 32; ++jb) {
                const unsigned b = byte_of(w[jb >> 4], jb & 15);
                if constexpr (KSUB == 16) {
                    acc = acc + lut[(2 * jb) * 16 + (b & 15u)];
                    acc = acc + lut[(2 * jb + 1) * 16 + (b >> 4)];
                } else {
                    acc = acc + lut[jb * 256 + b];
                }
            }
            k[0] = nc[0] ? (((uint64_t)f2ord(acc) << 32) | (rel + (unsigned)tid)) : ~0ull;
        }

#pragma unroll
        for (int c = 0; c < C::CPT; ++c) {
            const bool pass = k[c] < lim;
            const unsigned slot = have + wave_append_slot(pass, ctr);
            if (pass) keys[slot] = k[c];
        }
        __syncthreads();
        have += *ctr;
        rot = nxt;
        if (have > (unsigned)SCAN_SLACK) {
            const uint64_t kth = compact_candidates<uint64_t, 8, NT, C::CAP>(keys, have, (unsigned)R,
                                                                              &sh.sel, &sh.ccnt);
            lim = min(lim, kth + 1ull);
            have = (unsigned)R;
        }
    }

    if (have > (unsigned)R) {
        compact_candidates<uint64_t, 8, NT, C::CAP>(keys, have, (unsigned)R, &sh.sel, &sh.ccnt);
        have = (unsigned)R;
    }
    if (have == 0) return;
    unsigned *counts = reinterpret_cast<unsigned *>(ws + (size_t)q * ws_stride + counts_off);
    uint64_t *dst = reinterpret_cast<uint64_t *>(ws + (size_t)q * ws_stride + lists_off) + (size_t)g * R;
    if (tid == 0) counts[g] = have;
    for (unsigned i = tid; i < have; i += NT) {
        const uint64_t key = keys[i];
        const uint64_t r = key & 0xffffffffull;
        const uint64_t idx = ((r / C::TILE) * (uint64_t)G + (uint64_t)g) * C::TILE + r % C::TILE;
        dst[i] = (key & 0xffffffff00000000ull) | idx;
    }
}

struct F32Plan {
    int ROW, KSUB, G, qbatch;
    ScanLayout l;
    size_t ws_bytes;
};

static bool make_f32_plan(int variant, int64_t n, int m, int nq, int R, F32Plan *p)
{
    if (variant == QADC_F32_4BIT) {
        if (!(m == 8 || m == 16 || m == 32 || m == 64)) return false;
        p->ROW = m / 2;
        p->KSUB = 16;
    } else if (variant == QADC_F32_8BIT) {
        if (!(m == 4 || m == 8 || m == 16 || m == 32)) return false;
        p->ROW = m;
        p->KSUB = 256;
    } else {
        return false;
    }
    if (n < 0 || n > 0xfffffffell || nq < 1 || R < 1 || R > QADC_MAX_R) return false;
    const int cpt = (p->ROW <= 16) ? SCAN_VEC * (16 / p->ROW) : 1;
    const int tile = F32_NT * cpt;
    const int64_t tiles = n > 0 ? ceil_div(n, tile) : 1;
    int64_t G = env_int("QADC_SCAN_F32_WGS", 512);
    if (G < 1) G = 1;
    if (G > tiles) G = tiles;
    const int64_t max_tiles_per_wg = 0xffffffffll / tile;
    if (ceil_div(tiles, G) > max_tiles_per_wg) G = ceil_div(tiles, max_tiles_per_wg);
    p->G = (int)G;
    p->l = scan_layout(p->G, R);
    p->qbatch = scan_query_batch(p->l.stride, nq);
    p->ws_bytes = p->l.stride * (size_t)p->qbatch;
    return true;
}

template <int KSUB>
static void dispatch_f32(const F32Plan &p, const uint8_t *codes, int64_t n, const float *luts, int nq,
                         int R, char *ws, hipStream_t st)
{
    dim3 grid(p.G, nq), block(F32_NT);
#define QADC_F32_CASE(ROW_)                                                                        \
    case ROW_:                                                                                     \
        launch(QADC_PROF_SCAN, (scan_f32_kernel<KSUB, ROW_>), grid, block, 0, st, codes, n, luts, R, ws, \
               p.l.stride, p.l.counts_off, p.l.lists_off);                                         \
        break;
    switch (p.ROW) {
        QADC_F32_CASE(4)
        QADC_F32_CASE(8)
        QADC_F32_CASE(16)
        QADC_F32_CASE(32)
    }
#undef QADC_F32_CASE
}

int scan_topk_f32(int variant, const uint8_t *codes, int64_t n, int m, const float *luts, int nq,
                  int R, uint32_t *out_idx, float *out_dist, void *workspace, size_t workspace_bytes,
                  hipStream_t st)
{
    F32Plan p;
    if (!make_f32_plan(variant, n, m, nq, R, &p))
        return fail(QADC_EINVAL, "qadc_scan_topk: unsupported variant=%d n=%lld m=%d nq=%d R=%d", variant,
                    (long long)n, m, nq, R);
    if (((uintptr_t)codes & 15) != 0) return fail(QADC_EINVAL, "qadc_scan_topk: codes must be 16-byte aligned");
    if (workspace_bytes < p.ws_bytes || !workspace)
        return fail(QADC_ENOMEM, "qadc_scan_topk: workspace %zu < %zu bytes", workspace_bytes, p.ws_bytes);
    if (((uintptr_t)workspace & 255) != 0)
        return fail(QADC_EINVAL, "qadc_scan_topk: workspace must be 256-byte aligned");
    char *ws = (char *)workspace;
    const int M = m;
    for (int q0 = 0; q0 < nq; q0 += p.qbatch) {
        const int nb = min(p.qbatch, nq - q0);
        const float *lq = luts + (size_t)q0 * M * p.KSUB;
        if (p.KSUB == 16) dispatch_f32<16>(p, codes, n, lq, nb, R, ws, st);
        else dispatch_f32<256>(p, codes, n, lq, nb, R, ws, st);
        launch(QADC_PROF_MERGE, (merge_topk_kernel<float, 8>), dim3(nb), dim3(MERGE_NT), 0, st, ws,
               p.l.stride, p.l.counts_off, p.l.lists_off, p.G, (unsigned)min((int64_t)R, n), R,
               __builtin_inff(), out_idx + (size_t)q0 * R, out_dist + (size_t)q0 * R, (size_t)0, (size_t)0, 0,
               0, (unsigned *)nullptr);
    }
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

size_t scan_topk_f32_workspace(int variant, int64_t n, int m, int nq, int R)
{
    F32Plan p;
    if (!make_f32_plan(variant, n, m, nq, R, &p)) return 0;
    return p.ws_bytes;
}

}  // namespace qadc
