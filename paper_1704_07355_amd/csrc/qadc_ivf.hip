// Non-exhaustive search (Sections 2.2 and 2.3 of the paper) with Quick ADC on gfx950:
//   Index   squared distances of the query to the K coarse centroids, the nprobe closest cells
//   Tables  one set of m float tables per probed cell, on the residual y - centroid (Eq. (1))
//   qmax    float ADC of the first `init` codes met walking the probed lists in probe order
//           (Section 3.3), then ONE 8-bit quantizer per query shared by all its cells, so
//           that quantized sums of different cells compare
//   Scan    every code of every probed list: pair-table lookups, clamped sum (Alg. 2),
//           key = sum << 32 | storage position; R smallest keys per query; ids[position]
// Inverted lists are skewed (a few lists hold millions of codes, most a few thousand), so a
// query's lists are cut into units of at most IVF_UNIT codes; a query gets workgroups in
// proportion to its number of units, each taking a contiguous range of them.

#include <algorithm>

#include "qadc_scan_common.h"

namespace qadc {

#ifndef QADC_IVF_EARLY_STAGES
// (a check at a quarter and at half of the bytes measured the same as the one check at half)
#define QADC_IVF_EARLY_STAGES(B) ((B) >= 4 ? 2 : 1)
#endif
constexpr int IVF_MAX_NPROBE = 256;
constexpr int IVF_NT = 256;      // threads of the scan workgroups
constexpr int IVF_UNIT_TILES = 8;
constexpr int IVF_WIDE_MAX_Q = 12;  // calls of up to this many queries scan with workgroups of 1024 threads

// A few queries: the tables of the probed cells stay float in memory, and every kernel that needs a
// cell's 8-bit tables applies the query's quantizer (Section 3.3) itself -- the arithmetic of
// quantize_luts_kernel, entry by entry -- which saves a pass over the tables between launches.
struct IvfQuantizer {
    const float *luts;   // [nq][nprobe][m][16]; null: the tables are quantized in memory
    const float *bias;   // [nq][m]
    const float *delta;  // [nq]
};

__device__ __forceinline__ unsigned quantize_entry(float D, float bias, float delta, unsigned nbins)
{
    const float off = fmaxf(0.0f, D - bias);
    const float t = floorf(__fdiv_rn(off, delta));
    return (t < (float)nbins) ? (unsigned)(uint8_t)t : nbins;
}

// entries 4 w .. 4 w + 3 of a cell's tables (inside one table: a table has 16 entries) as four bytes
__device__ __forceinline__ unsigned quantize_word(const float *cell_luts, int w, const float *bias, float delta,
                                                  unsigned nbins)
{
    const float4 v = *reinterpret_cast<const float4 *>(cell_luts + 4 * w);
    const float b = bias[w >> 2];
    return quantize_entry(v.x, b, delta, nbins) | (quantize_entry(v.y, b, delta, nbins) << 8) |
           (quantize_entry(v.z, b, delta, nbins) << 16) | (quantize_entry(v.w, b, delta, nbins) << 24);
}

// The control words of a query's scan -- the histograms of its control block and the counts of its
// report regions -- are cleared at the start of every call: calls of different shapes lay the
// workspace out differently, and what one call left as table data may lie where the next one keeps
// its counts.  Called by a whole workgroup for its query.
__device__ __forceinline__ void ivf_clear_control(char *base, size_t counts_off, int W, size_t countsA_off)
{
    unsigned *gh = reinterpret_cast<unsigned *>(base);  // ScanHeader::ghist comes first
    for (int i = threadIdx.x; i < GH_REP * 256; i += blockDim.x) gh[i] = 0;
    unsigned *counts = reinterpret_cast<unsigned *>(base + counts_off);
    for (int i = threadIdx.x; i < W; i += blockDim.x) counts[i] = 0;
    if (countsA_off && threadIdx.x == 0) *reinterpret_cast<unsigned *>(base + countsA_off) = 0;
}

// Where the kernels of the Index step clear a query's control words (calls of a few queries, which
// have no qmax kernel to do it); scan_ws null: not here.
struct IvfClear {
    char *scan_ws;
    size_t ws_stride, counts_off, countsA_off;
    int W;
};

// ------------------------------------------------------------------ Index

// dist[q][c] = sum_t (y[q][t] - coarse[c][t])^2, float32, summed in increasing t with one fused
// multiply-add per component -- the same operations in the same order for a pair whatever the
// batch, so that the cells a query gets do not depend on the queries sent with it.
// A workgroup computes 16*AQ queries x 128 cells, 16 components of both at a time through LDS,
// AQ x 8 distances per thread.  Thread (tx, ty) owns queries AQ*ty.. and the cells
// 32*k + 2*tx + e, so that a wavefront's 8-byte LDS reads of the cells are contiguous.  AQ = 8
// (128 queries per workgroup) for batches, AQ = 1 (16 queries) for a few queries, whose cost is
// then one pass over the centroids.
constexpr int IVF_CT = 128;  // cells per workgroup
constexpr int IVF_CK = 16;   // components per step

template <int AQ>
__global__ __launch_bounds__(256) void ivf_coarse_dist_kernel(
    const float *__restrict__ coarse, int K, int d, const float *__restrict__ queries, int nq,
    float *__restrict__ dist, unsigned *__restrict__ blockmin, int nblk)
{
    constexpr int QT = 16 * AQ;
    __shared__ __attribute__((aligned(16))) float ys[IVF_CK][QT + 4];
    __shared__ __attribute__((aligned(16))) float cs[IVF_CK][IVF_CT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int c0 = blockIdx.x * IVF_CT;
    const int q0 = blockIdx.y * QT;
    float acc[AQ][8];
#pragma unroll
    for (int a = 0; a < AQ; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[a][b] = 0.0f;
    // the 16 components of the next step are requested while the current ones are used
    float cn[8], yn[8];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int idx = tid + e * 256;
            const int row = idx >> 4, col = idx & 15;
            const int t = t0 + col;
            const int c = c0 + row;
            cn[e] = (c < K && t < d) ? coarse[(size_t)c * d + t] : 0.0f;
            yn[e] = 0.0f;
            if (row < QT) {
                const int q = q0 + row;
                if (q < nq && t < d) yn[e] = queries[(size_t)q * d + t];
            }
        }
    };
    fetch(0);
    for (int t0 = 0; t0 < d; t0 += IVF_CK) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int idx = tid + e * 256;
            const int row = idx >> 4, col = idx & 15;
            cs[col][row] = cn[e];
            if (row < QT) ys[col][row] = yn[e];
        }
        __syncthreads();
        if (t0 + IVF_CK < d) fetch(t0 + IVF_CK);  // uniform
#pragma unroll 4
        for (int kk = 0; kk < IVF_CK; ++kk) {
            float yv[AQ], cv[8];
            if constexpr (AQ % 4 == 0) {
#pragma unroll
                for (int a = 0; a < AQ; a += 4) {
                    const float4 v = *reinterpret_cast<const float4 *>(&ys[kk][AQ * ty + a]);
                    yv[a] = v.x; yv[a + 1] = v.y; yv[a + 2] = v.z; yv[a + 3] = v.w;
                }
            } else {
#pragma unroll
                for (int a = 0; a < AQ; ++a) yv[a] = ys[kk][AQ * ty + a];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float2 v = *reinterpret_cast<const float2 *>(&cs[kk][32 * k + 2 * tx]);
                cv[2 * k] = v.x; cv[2 * k + 1] = v.y;
            }
#pragma unroll
            for (int a = 0; a < AQ; ++a)
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const float df = yv[a] - cv[b];
                    acc[a][b] = fmaf(df, df, acc[a][b]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < AQ; ++a) {
        const int q = q0 + AQ * ty + a;
        unsigned mn = 0xffffffffu;  // smallest distance of this query over the workgroup's cells, as its image
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = c0 + 32 * k + 2 * tx;
            if (c < K) mn = min(mn, f2ord(acc[a][2 * k]));
            if (c + 1 < K) mn = min(mn, f2ord(acc[a][2 * k + 1]));
            if (q >= nq) continue;
            if (c + 1 < K && (K & 1) == 0) {  // K even: the pair is 8-byte aligned
                *reinterpret_cast<float2 *>(&dist[(size_t)q * K + c]) = make_float2(acc[a][2 * k], acc[a][2 * k + 1]);
            } else {
                if (c < K) dist[(size_t)q * K + c] = acc[a][2 * k];
                if (c + 1 < K) dist[(size_t)q * K + c + 1] = acc[a][2 * k + 1];
            }
        }
        if (blockmin) {  // uniform: the 16 lanes tx of a query are neighbours in the wavefront
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) mn = min(mn, (unsigned)__shfl_xor((int)mn, o));
            if (tx == 0 && q < nq) blockmin[(size_t)q * nblk + blockIdx.x] = mn;
        }
    }
}

// The same distances for up to a few dozen queries, whose cost is one pass over the centroids: the
// workgroup's 128 centroids are requested at once (IVF_FEW_DK components of each, 64 KiB in flight per
// workgroup) and staged in LDS as they lie in memory; thread t then walks the components of cell
// t % 128, four at a time, for the queries 8 (t / 128) .. + 7 of the workgroup's 16, whose components
// every lane of the wavefront reads from the same LDS address.  Also written: the smallest distance of every
// (query, workgroup) as its order-preserving image, from which the selection kernel finds its
// threshold without reading the row.
constexpr int IVF_FEW_DK = 128;  // components staged at a time
constexpr int IVF_FEW_Q = 16;    // queries per workgroup

// acc[a] += sum over the staged components of (y_a - c)^2 for the first NQ queries of a thread: c = the
// thread's centroid row, ys = its first query's row (rows ld floats apart), four components at a time.
// (A padded component is 0 - 0: the fused multiply-add leaves the sum as it is.)
template <int NQ>
__device__ __forceinline__ void few_walk(const float *c_row, const float *ys, int ld, int dk4, float (&acc)[8])
{
    float a[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) a[i] = acc[i];
#pragma unroll 2
    for (int kk = 0; kk < 4 * dk4; kk += 4) {
        const float4 c = *reinterpret_cast<const float4 *>(c_row + kk);
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const float4 y = *reinterpret_cast<const float4 *>(ys + i * ld + kk);
            float df = y.x - c.x;
            a[i] = fmaf(df, df, a[i]);
            df = y.y - c.y;
            a[i] = fmaf(df, df, a[i]);
            df = y.z - c.z;
            a[i] = fmaf(df, df, a[i]);
            df = y.w - c.w;
            a[i] = fmaf(df, df, a[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < NQ; ++i) acc[i] = a[i];
}

__global__ __launch_bounds__(256) void ivf_coarse_dist_few_kernel(
    const float *__restrict__ coarse, int K, int d, const float *__restrict__ queries, int nq,
    float *__restrict__ dist, unsigned *__restrict__ blockmin, int nblk, int vec4)
{
    constexpr int LD = IVF_FEW_DK + 4;  // rows 16-byte aligned, eight neighbouring cells on all the banks
    constexpr int QH = IVF_FEW_Q / 2;   // queries per thread
    __shared__ __attribute__((aligned(16))) float cs[IVF_CT][LD];
    __shared__ __attribute__((aligned(16))) float ys[IVF_FEW_Q][LD];
    __shared__ unsigned wmin[256 / WAVE][QH];
    const int tid = threadIdx.x;
    const int cell = tid & (IVF_CT - 1);
    const int c0 = blockIdx.x * IVF_CT;
    const int qh = QH * (tid / IVF_CT);                 // first query of this thread among the workgroup's
    const int q0 = blockIdx.y * IVF_FEW_Q + qh;         // (the same for a whole wavefront)
    const int nmine = min(QH, nq - q0);                            // its queries (may be <= 0)
    float acc[QH];
#pragma unroll
    for (int a = 0; a < QH; ++a) acc[a] = 0.0f;
    for (int t0 = 0; t0 < d; t0 += IVF_FEW_DK) {  // uniform
        const int dk = min(IVF_FEW_DK, d - t0);
        const int dk4 = (dk + 3) >> 2;  // groups of four components, the last one padded with zeros
        if (t0) __syncthreads();  // everybody is done with the previous components
        if (vec4) {  // d a multiple of four, rows 16-byte aligned
            constexpr int PER = IVF_CT * (IVF_FEW_DK / 4) / 256;  // 16 loads per thread, all in flight
            float4 v[PER];
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int idx = tid + e * 256;
                const int row = idx / dk4, col4 = idx - row * dk4;
                v[e] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (row < IVF_CT && c0 + row < K)
                    v[e] = *reinterpret_cast<const float4 *>(coarse + (size_t)(c0 + row) * d + t0 + 4 * col4);
            }
            for (int idx = tid; idx < IVF_FEW_Q * dk4; idx += 256) {
                const int row = idx / dk4, col4 = idx - row * dk4;
                float4 y = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                const int q = blockIdx.y * IVF_FEW_Q + row;
                if (q < nq) y = *reinterpret_cast<const float4 *>(queries + (size_t)q * d + t0 + 4 * col4);
                *reinterpret_cast<float4 *>(&ys[row][4 * col4]) = y;
            }
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int idx = tid + e * 256;
                const int row = idx / dk4, col4 = idx - row * dk4;
                if (row < IVF_CT) *reinterpret_cast<float4 *>(&cs[row][4 * col4]) = v[e];
            }
        } else {
            for (int idx = tid; idx < IVF_FEW_Q * 4 * dk4; idx += 256) {
                const int row = idx / (4 * dk4), col = idx - row * (4 * dk4);
                const int q = blockIdx.y * IVF_FEW_Q + row;
                ys[row][col] = (q < nq && col < dk) ? queries[(size_t)q * d + t0 + col] : 0.0f;
            }
            for (int idx = tid; idx < IVF_CT * 4 * dk4; idx += 256) {
                const int row = idx / (4 * dk4), col = idx - row * (4 * dk4);
                cs[row][col] = (c0 + row < K && col < dk) ? coarse[(size_t)(c0 + row) * d + t0 + col] : 0.0f;
            }
        }
        __syncthreads();
        if (nmine <= 0) continue;  // uniform in a wavefront: no query for it
        // the walk, compiled for every number of queries a thread can have (no test per query inside)
        switch (nmine) {
        case 1: few_walk<1>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        case 2: few_walk<2>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        case 3: few_walk<3>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        case 4: few_walk<4>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        case 5: few_walk<5>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        case 6: few_walk<6>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        case 7: few_walk<7>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        default: few_walk<8>(&cs[cell][0], &ys[qh][0], IVF_FEW_DK + 4, dk4, acc); break;
        }
    }
    const int c = c0 + cell;
    unsigned mn[QH];
#pragma unroll
    for (int a = 0; a < QH; ++a) {
        mn[a] = 0xffffffffu;
        if (a < nmine && c < K) {
            dist[(size_t)(q0 + a) * K + c] = acc[a];
            mn[a] = f2ord(acc[a]);
        }
    }
    if (!blockmin) return;  // uniform
    // smallest image per query: inside the wavefront, then across the two wavefronts of a query
#pragma unroll
    for (int a = 0; a < QH; ++a) {
        if (a < nmine) {  // uniform in a wavefront
#pragma unroll
            for (int o = 1; o < WAVE; o <<= 1) mn[a] = min(mn[a], (unsigned)__shfl_xor((int)mn[a], o));
        }
        if (lane_id() == 0) wmin[tid / WAVE][a] = mn[a];
    }
    __syncthreads();
    if (tid < IVF_FEW_Q) {
        const int h = tid / QH, a = tid % QH;  // wavefronts 2h and 2h + 1 hold query 8h + a
        const int q = blockIdx.y * IVF_FEW_Q + tid;
        if (q < nq) blockmin[(size_t)q * nblk + blockIdx.x] = min(wmin[2 * h][a], wmin[2 * h + 1][a]);
    }
}

// probes[q][0..nprobe) = the nprobe closest cells, closest first, ties to the lowest cell id.
// Keys are order(dist) << 32 | cell (unique).  Thread t looks at cells t, t + NT, ...  The
// need-th smallest of the threads' minima, T, bounds the need-th smallest key of the whole
// row from above (need threads each hold a key <= T), and only those need threads can hold
// keys <= T: at most need * ceil(K / NT) candidates, normally about `need` of them.  A second
// pass over the row gathers the candidates in LDS, where the exact selection runs.  A
// candidate list that does not fit takes the radix select over the whole row instead.
// With `blockmin` (the smallest distance of every run of IVF_CT cells, at least `need` runs): T = the
// need-th smallest of those minima, by the same argument, and only the runs whose minimum is <= T are
// read at all -- the row is not walked twice by one workgroup.
constexpr int IVF_SEL_NT = 1024;
constexpr int IVF_SEL_CAP = 4096;
constexpr int IVF_SEL_MAXBLK = 4096;  // runs of cells whose minima fit in LDS

__global__ __launch_bounds__(IVF_SEL_NT) void ivf_select_probes_kernel(
    const float *__restrict__ dist, int K, int nprobe, int32_t *__restrict__ probes,
    const unsigned *__restrict__ blockmin, int nblk, IvfClear clr)
{
    constexpr int NT = IVF_SEL_NT;
    if (clr.scan_ws) {  // uniform
        ivf_clear_control(clr.scan_ws + (size_t)blockIdx.x * clr.ws_stride, clr.counts_off, clr.W, clr.countsA_off);
    }
    __shared__ SelectScratch sc;
    __shared__ uint64_t cand[IVF_SEL_CAP];  // thread minima first, then the candidates
    __shared__ unsigned cnt;
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    const float *dq = dist + (size_t)q * K;
    const unsigned need = (unsigned)min(nprobe, K);

    if (blockmin) {  // uniform
        __shared__ unsigned bm[IVF_SEL_MAXBLK];
        __shared__ unsigned hits[IVF_SEL_MAXBLK];
        __shared__ unsigned nhit_s;
        for (int b = tid; b < nblk; b += NT) bm[b] = blockmin[(size_t)q * nblk + b];
        if (tid == 0) { cnt = 0; nhit_s = 0; }
        __syncthreads();
        // the three leading bytes of the need-th smallest minimum, everything below them set
        unsigned Tm = block_radix_select_each<unsigned, 3>(
            [&](auto f) {
                for (int b = tid; b < nblk; b += NT) f(bm[b] >> 8);
            },
            need, &sc);
        Tm = (Tm << 8) | 0xffu;
        for (int b = tid; b < nblk; b += NT)
            if (bm[b] <= Tm) hits[atomicAdd(&nhit_s, 1u)] = (unsigned)b;
        __syncthreads();
        const unsigned ncell = nhit_s * (unsigned)IVF_CT;
        for (unsigned i0 = tid; i0 < ncell; i0 += 4 * NT) {
            float v[4];
            int c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned i = i0 + u * NT;
                c[u] = i < ncell ? (int)(hits[i / IVF_CT] * IVF_CT + i % IVF_CT) : K;
                v[u] = c[u] < K ? dq[c[u]] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned o = f2ord(v[u]);
                if (c[u] < K && o <= Tm) {
                    const unsigned slot = atomicAdd(&cnt, 1u);
                    if (slot < (unsigned)IVF_SEL_CAP) cand[slot] = ((uint64_t)o << 32) | (uint64_t)(unsigned)c[u];
                }
            }
        }
    } else {
    // this thread's smallest key: smallest value, lowest cell among equals (cells grow with c)
    // (eight loads in flight per thread: the row is read at memory speed, not one latency per cell)
    uint64_t mine = ~0ull;
    for (int c0 = tid; c0 < K; c0 += 8 * NT) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * NT;
            v[u] = c < K ? dq[c] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * NT;
            if (c < K) mine = min(mine, ((uint64_t)f2ord(v[u]) << 32) | (uint64_t)(unsigned)c);
        }
    }
    const int nmin = min(K, NT);  // threads that hold at least one key
    if (tid < nmin) cand[tid] = mine;
    if (tid == 0) cnt = 0;
    __syncthreads();
    // Any T at or above the need-th smallest minimum will do: the three leading bytes of the
    // distance decide it (three histogram passes instead of eight), everything below is set.
    uint64_t T = block_radix_select_each<uint64_t, 3>(
        [&](auto f) {
            for (int i = tid; i < nmin; i += NT) f(cand[i] >> 40);
        },
        need, &sc);
    T = (T << 40) | 0xffffffffffull;
    __syncthreads();  // everybody has T; the minima may be overwritten
    // second pass over the row, by every thread as the first (only a thread whose minimum is <= T
    // finds anything, but a few threads walking their cells alone would pay a latency per cell)
    for (int c0 = tid; c0 < K; c0 += 8 * NT) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * NT;
            v[u] = c < K ? dq[c] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * NT;
            const uint64_t k = ((uint64_t)f2ord(v[u]) << 32) | (uint64_t)(unsigned)c;
            if (c < K && k <= T) {
                const unsigned slot = atomicAdd(&cnt, 1u);
                if (slot < (unsigned)IVF_SEL_CAP) cand[slot] = k;
            }
        }
    }
    }
    __syncthreads();
    const unsigned ncand = cnt;
    const bool in_lds = ncand <= (unsigned)IVF_SEL_CAP;
    __syncthreads();

    auto each_row = [&](auto f) {
        for (int c = tid; c < K; c += NT) f(((uint64_t)f2ord(dq[c]) << 32) | (uint64_t)(unsigned)c);
    };
    if (ncand <= (unsigned)NT) {
        // a thread per candidate: its rank among all of them is its place among the probes
        if ((unsigned)tid < ncand) {
            const uint64_t k = cand[tid];
            unsigned rank = 0;
            for (unsigned j = 0; j < ncand; ++j) rank += (cand[j] < k) ? 1u : 0u;
            if (rank < need) probes[(size_t)q * nprobe + rank] = (int32_t)(unsigned)k;
        }
        for (unsigned i = need + tid; i < (unsigned)nprobe; i += NT) probes[(size_t)q * nprobe + i] = -1;
        return;  // uniform
    }
    uint64_t kth;
    if (in_lds) kth = block_radix_select<uint64_t, 8>(cand, ncand, need, &sc);
    else kth = block_radix_select_each<uint64_t, 8>(each_row, need, &sc);
    // the winners (exactly `need`: keys are unique), ordered by rank
    __shared__ uint64_t sel[IVF_MAX_NPROBE];
    if (tid == 0) cnt = 0;
    __syncthreads();
    if (in_lds) {
        for (unsigned i = tid; i < ncand; i += NT)
            if (cand[i] <= kth) sel[atomicAdd(&cnt, 1u)] = cand[i];
    } else {
        each_row([&](uint64_t k) {
            if (k <= kth) sel[atomicAdd(&cnt, 1u)] = k;
        });
    }
    __syncthreads();
    for (unsigned i = tid; i < (unsigned)nprobe; i += NT) {
        if (i >= need) {
            probes[(size_t)q * nprobe + i] = -1;
        } else {
            const uint64_t k = sel[i];
            unsigned rank = 0;
            for (unsigned j = 0; j < need; ++j) rank += (sel[j] < k) ? 1u : 0u;
            probes[(size_t)q * nprobe + rank] = (int32_t)(unsigned)k;
        }
    }
}

// rows of `dist` [rows][K] -> out[rows][count]: the count smallest of each row, smallest first
// (for the multi-index's half distances)
void ivf_select_smallest(const float *dist, int rows, int K, int count, int32_t *out, hipStream_t st)
{
    launch(QADC_PROF_IVF_INDEX, ivf_select_probes_kernel, dim3((unsigned)rows), dim3(IVF_SEL_NT), 0, st, dist, K,
           count, out, (const unsigned *)nullptr, 0, IvfClear{nullptr, 0, 0, 0, 0});
}

// ----------------------------------------------------------------- Tables

// luts[q][p][j][i] = || (y_q - coarse[probes[q][p]])^j - C^j[i] ||^2, float64 inside, one
// rounding to float32 (same arithmetic as the exhaustive tables kernel).  Unused probe slots
// (cell id < 0) get +inf tables: nothing of them is ever scanned.
__global__ __launch_bounds__(256) void ivf_build_luts_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ queries,
    const float *__restrict__ coarse, const float *__restrict__ halves, const uint32_t *__restrict__ cell_ids,
    int Kh, const int32_t *__restrict__ probes, int nprobe, float *__restrict__ luts)
{
    extern __shared__ double yr[];  // [d]
    const int p = blockIdx.x, q = blockIdx.y;
    const int cell = probes[(size_t)q * nprobe + p];
    const int dsub = d / m;
    const int entries = m * 16;
    float *out = luts + ((size_t)q * nprobe + p) * entries;
    if (cell < 0) {
        for (int e = threadIdx.x; e < entries; e += blockDim.x) out[e] = __builtin_inff();
        return;
    }
    if (coarse) {
        for (int t = threadIdx.x; t < d; t += blockDim.x)
            yr[t] = (double)queries[(size_t)q * d + t] - (double)coarse[(size_t)cell * d + t];
    } else {  // list `cell` of a multi-index: the centroid is a pair of half-centroids
        const int dh = d >> 1;
        const unsigned id = cell_ids[cell];
        const float *h0 = halves + (size_t)(id / (unsigned)Kh) * dh;
        const float *h1 = halves + ((size_t)Kh + id % (unsigned)Kh) * dh;
        for (int t = threadIdx.x; t < d; t += blockDim.x)
            yr[t] = (double)queries[(size_t)q * d + t] - (double)(t < dh ? h0[t] : h1[t - dh]);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < entries; e += blockDim.x) {
        const int j = e >> 4;
        const float *c = codebooks + (size_t)e * dsub;
        const double *y = yr + j * dsub;
        double acc = 0.0;
        for (int t = 0; t < dsub; ++t) {
            const double df = y[t] - (double)c[t];
            acc += df * df;
        }
        out[e] = (float)acc;
    }
}

// The same tables for batches: one workgroup per query, one thread per table entry (m * 16 threads);
// the thread keeps its centroid's sub-vector in registers and walks the query's probed cells, reading
// the cell's coarse centroid (or half-centroids) where its sub-vector lies.  Same arithmetic, value by
// value, as ivf_build_luts_kernel; a workgroup per (query, cell) spends most of its time starting up.
template <int DSUB>
__global__ __launch_bounds__(1024) void ivf_build_luts_batch_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ queries,
    const float *__restrict__ coarse, const float *__restrict__ halves, const uint32_t *__restrict__ cell_ids,
    int Kh, const int32_t *__restrict__ probes, int nprobe, float *__restrict__ luts)
{
    const int q = blockIdx.x;
    const int e = threadIdx.x;  // entry: table j = e / 16, centroid e % 16
    constexpr int dsub = DSUB;  // d / m
    const int entries = m * 16;
    if (e >= entries) return;
    const int j = e >> 4;
    const int t0 = j * dsub;
    double c[DSUB], y[DSUB];
#pragma unroll
    for (int t = 0; t < dsub; ++t) {
        c[t] = (double)codebooks[(size_t)e * dsub + t];
        y[t] = (double)queries[(size_t)q * d + t0 + t];
    }
    const int dh = d >> 1;
    for (int p = 0; p < nprobe; ++p) {
        const int cell = probes[(size_t)q * nprobe + p];
        float *out = luts + ((size_t)q * nprobe + p) * entries;
        if (cell < 0) {
            out[e] = __builtin_inff();
            continue;
        }
        const float *cen;  // the centroid's components t0 .. t0 + dsub - 1 (inside one half)
        if (coarse) {
            cen = coarse + (size_t)cell * d + t0;
        } else {
            const unsigned id = cell_ids[cell];
            cen = t0 < dh ? halves + (size_t)(id / (unsigned)Kh) * dh + t0
                          : halves + ((size_t)Kh + id % (unsigned)Kh) * dh + (t0 - dh);
        }
        double acc = 0.0;
#pragma unroll
        for (int t = 0; t < dsub; ++t) {
            const double df = (y[t] - (double)cen[t]) - c[t];
            acc += df * df;
        }
        out[e] = (float)acc;
    }
}

// ------------------------------------------------------------------- qmax

// qmax[q] = min(R, n_walk)-th smallest float ADC distance (Eq. (2), float32, increasing j)
// of the first n_walk = min(init, codes in the probed lists) codes met walking the lists in
// probe order, each code with the tables of its own cell; 0 when the lists are empty.
__global__ __launch_bounds__(1024) void ivf_qmax_kernel(
    const int64_t *__restrict__ list_off, const uint8_t *__restrict__ codes, int m,
    const int32_t *__restrict__ probes, int nprobe, const float *__restrict__ luts, int init, int R,
    float *__restrict__ qmax, long long unit, unsigned *__restrict__ qunits, int64_t n_total,
    char *__restrict__ ws, size_t ws_stride, size_t counts_off, int W, size_t countsA_off)
{
    ivf_clear_control(ws + (size_t)blockIdx.x * ws_stride, counts_off, W, countsA_off);
    __shared__ unsigned cand[QADC_MAX_INIT];
    __shared__ unsigned units_s;
    __shared__ long long start[IVF_MAX_NPROBE + 1];  // codes before probe p in the walk
    __shared__ long long lo[IVF_MAX_NPROBE];
    __shared__ SelectScratch sc;
    const int q = blockIdx.x;
    const int tid = threadIdx.x;
    const int B = m / 2;
    // list lengths one thread per probe, exclusive prefix sum
    __shared__ unsigned long long wsum[1024 / WAVE];
    unsigned long long len = 0;
    if (tid == 0) units_s = 0;
    __syncthreads();
    if (tid < nprobe) {
        const int cell = probes[(size_t)q * nprobe + tid];
        long long l = 0, h = 0;
        if (cell >= 0) { l = list_off[cell]; h = list_off[cell + 1]; }
        if (l < 0 || h > n_total || h < l) l = h = 0;  // offsets that are not a list: nothing is read
        lo[tid] = l;
        len = (unsigned long long)(h - l);
        // units the scan kernel cuts this list into (the same expression as there)
        if (h > l) atomicAdd(&units_s, (unsigned)((h - l / 16 * 16 + unit - 1) / unit));
    }
    {
        const int l = lane_id();
        unsigned long long inc = len;
#pragma unroll
        for (int dd = 1; dd < WAVE; dd <<= 1) {
            const unsigned long long up = __shfl_up(inc, dd);
            if (l >= dd) inc += up;
        }
        if (l == WAVE - 1) wsum[tid / WAVE] = inc;
        __syncthreads();
        unsigned long long before = 0;
        for (int wv = 0; wv < tid / WAVE; ++wv) before += wsum[wv];
        if (tid < nprobe) start[tid] = (long long)(before + inc - len);
        if (tid == nprobe - 1) start[nprobe] = (long long)(before + inc);
    }
    __syncthreads();
    if (tid == 0) qunits[q] = units_s;
    const long long total = start[nprobe];
    const int n_walk = (int)min((long long)init, total);
    if (n_walk == 0) {  // uniform
        if (tid == 0) qmax[q] = 0.0f;
        return;
    }
    for (int i = tid; i < n_walk; i += blockDim.x) {
        int p = 0;
        while (start[p + 1] <= i) ++p;  // lists are few; the walk is short
        // the code as 32-bit words (B is a multiple of 4), then its table entries four bytes at a
        // time: the eight loads of a word are in flight together, the sum keeps the order of j
        const unsigned *cw = reinterpret_cast<const unsigned *>(codes + (size_t)(lo[p] + (i - start[p])) * B);
        const float *lut = luts + ((size_t)q * nprobe + p) * m * 16;
        float acc = 0.0f;
        for (int k = 0; k < B / 4; ++k) {
            const unsigned w = cw[k];
            float e[8];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const unsigned comps = (w >> (8 * b)) & 0xffu;
                const int jb = 4 * k + b;
                e[2 * b] = lut[(2 * jb) * 16 + (comps & 15u)];
                e[2 * b + 1] = lut[(2 * jb + 1) * 16 + (comps >> 4)];
            }
#pragma unroll
            for (int b = 0; b < 8; ++b) acc = acc + e[b];
        }
        cand[i] = f2ord(acc);
    }
    __syncthreads();
    const unsigned need = (unsigned)min(R, n_walk);
    const unsigned kth = block_radix_select<unsigned, 4>(cand, (unsigned)n_walk, need, &sc);
    if (tid == 0) qmax[q] = ord2f(kth);
}

// Calls of a few queries: Tables and the sums of the qmax walk in one launch.  Workgroup (p, q)
// builds the float tables of the query's p-th cell (the arithmetic of ivf_build_luts_kernel), leaves
// the minimum of each table, and computes the float ADC sums of the init codes that the walk of
// ivf_qmax_kernel takes from its list, with the tables still in LDS ...
constexpr int IVF_FRONT_NT = 256;

__global__ __launch_bounds__(IVF_FRONT_NT) void ivf_front_kernel(
    const float *__restrict__ codebooks, int d, int m, const float *__restrict__ queries,
    const float *__restrict__ coarse, const float *__restrict__ halves, const uint32_t *__restrict__ cell_ids,
    int Kh, const int32_t *__restrict__ probes, int nprobe, float *__restrict__ luts,
    const int64_t *__restrict__ list_off, const uint8_t *__restrict__ codes, int64_t n_total, int init,
    long long unit, unsigned *__restrict__ qunits, unsigned *__restrict__ cand,
    unsigned *__restrict__ mins, unsigned *__restrict__ nwalk_out)
{
    constexpr int NT = IVF_FRONT_NT;
    extern __shared__ double yr[];  // [d]
    __shared__ float lut_s[64 * 16];
    __shared__ unsigned long long wsum[NT / WAVE];
    __shared__ long long start_s[2], lo_s, total_s;
    __shared__ unsigned units_s;
    const int p = blockIdx.x, q = blockIdx.y;
    const int tid = threadIdx.x;
    const int dsub = d / m;
    const int entries = m * 16;
    const int B = m / 2;

    // geometry of the walk: list lengths one thread per probe, exclusive prefix sum
    static_assert(IVF_MAX_NPROBE <= NT, "one thread per probe");
    unsigned long long len = 0;
    long long my_lo = 0;
    if (tid == 0) units_s = 0;
    __syncthreads();
    if (tid < nprobe) {
        const int c = probes[(size_t)q * nprobe + tid];
        long long l = 0, h = 0;
        if (c >= 0) { l = list_off[c]; h = list_off[c + 1]; }
        if (l < 0 || h > n_total || h < l) l = h = 0;  // offsets that are not a list: nothing is read
        my_lo = l;
        len = (unsigned long long)(h - l);
        // units the scan kernel cuts this list into (the same expression as there)
        if (h > l) atomicAdd(&units_s, (unsigned)((h - l / 16 * 16 + unit - 1) / unit));
    }
    // this cell's residual while those loads travel
    const int cell = probes[(size_t)q * nprobe + p];
    if (cell >= 0) {
        if (coarse) {
            for (int t = tid; t < d; t += NT)
                yr[t] = (double)queries[(size_t)q * d + t] - (double)coarse[(size_t)cell * d + t];
        } else {  // list `cell` of a multi-index: the centroid is a pair of half-centroids
            const int dh = d >> 1;
            const unsigned id = cell_ids[cell];
            const float *h0 = halves + (size_t)(id / (unsigned)Kh) * dh;
            const float *h1 = halves + ((size_t)Kh + id % (unsigned)Kh) * dh;
            for (int t = tid; t < d; t += NT)
                yr[t] = (double)queries[(size_t)q * d + t] - (double)(t < dh ? h0[t] : h1[t - dh]);
        }
    }
    {
        const int l = lane_id();
        unsigned long long inc = len;
#pragma unroll
        for (int dd = 1; dd < WAVE; dd <<= 1) {
            const unsigned long long up = __shfl_up(inc, dd);
            if (l >= dd) inc += up;
        }
        if (l == WAVE - 1) wsum[tid / WAVE] = inc;
        __syncthreads();  // (also: the residual is complete)
        unsigned long long before = 0;
        for (int wv = 0; wv < tid / WAVE; ++wv) before += wsum[wv];
        if (tid == p) {
            start_s[0] = (long long)(before + inc - len);
            start_s[1] = (long long)(before + inc);
            lo_s = my_lo;
        }
        if (tid == nprobe - 1) total_s = (long long)(before + inc);
    }
    // Tables, Eq. (1) on the residual: float64 differences and sums, one rounding
    float *out = luts + ((size_t)q * nprobe + p) * entries;
    for (int e = tid; e < entries; e += NT) {
        float v = __builtin_inff();  // an unused probe slot: nothing of it is ever scanned
        if (cell >= 0) {
            const int j = e >> 4;
            const float *c = codebooks + (size_t)e * dsub;
            const double *y = yr + j * dsub;
            double acc = 0.0;
            for (int t = 0; t < dsub; ++t) {
                const double df = y[t] - (double)c[t];
                acc += df * df;
            }
            v = (float)acc;
        }
        out[e] = v;
        lut_s[e] = v;
    }
    __syncthreads();
    if (p == 0 && tid == 0) qunits[q] = units_s;
    // minimum of each table, as its order-preserving image
    if (tid < m) {
        unsigned mn = 0xffffffffu;
        for (int i = 0; i < 16; ++i) mn = min(mn, f2ord(lut_s[tid * 16 + i]));
        mins[((size_t)q * nprobe + p) * m + tid] = mn;
    }
    // the walk's codes that lie in this list: float32 sums in increasing j (as ivf_qmax_kernel)
    const long long total = total_s;
    const int n_walk = (int)min((long long)init, total);
    {
        const long long s0 = start_s[0], s1 = min(start_s[1], (long long)n_walk);
        for (long long i = s0 + tid; i < s1; i += NT) {
            const unsigned *cw = reinterpret_cast<const unsigned *>(codes + (size_t)(lo_s + (i - s0)) * B);
            float acc = 0.0f;
            for (int k = 0; k < B / 4; ++k) {
                const unsigned w = cw[k];
                float e[8];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const unsigned comps = (w >> (8 * b)) & 0xffu;
                    const int jb = 4 * k + b;
                    e[2 * b] = lut_s[(2 * jb) * 16 + (comps & 15u)];
                    e[2 * b + 1] = lut_s[(2 * jb + 1) * 16 + (comps >> 4)];
                }
#pragma unroll
                for (int b = 0; b < 8; ++b) acc = acc + e[b];
            }
            cand[(size_t)q * QADC_MAX_INIT + i] = f2ord(acc);
        }
    }
    if (p == 0 && tid == 0) nwalk_out[q] = (unsigned)n_walk;
}

// ... then one workgroup per query selects qmax among the sums, joins the minima of the tables into
// the biases and derives delta: the arithmetic of quantize_luts_kernel.  (A launch of its own: the
// kernel boundary makes the sums visible; a count of finished workgroups with memory fences, tried
// first, made every workgroup of the launch before write the L2 back.)
constexpr int IVF_FINISH_NT = 1024;

__global__ __launch_bounds__(IVF_FINISH_NT) void ivf_finish_kernel(
    const unsigned *__restrict__ cand, const unsigned *__restrict__ mins, const unsigned *__restrict__ nwalk,
    int nprobe, int m, int R, int nbins, int qmin_mode, float *__restrict__ qmax_out,
    float *__restrict__ qbias, float *__restrict__ qdelta)
{
    constexpr int NT = IVF_FINISH_NT;
    __shared__ unsigned cand_s[QADC_MAX_INIT];
    __shared__ float bias_s[64];
    __shared__ unsigned bias_ord[64];
    __shared__ SelectScratch sc;
    const int q = blockIdx.x;
    const int tid = threadIdx.x;
    const int n_walk = (int)nwalk[q];
    for (int i = tid; i < n_walk; i += NT) cand_s[i] = cand[(size_t)q * QADC_MAX_INIT + i];
    for (int e = tid; e < m; e += NT) bias_ord[e] = 0xffffffffu;
    __syncthreads();
    for (int e = tid; e < nprobe * m; e += NT)  // (m divides NT: a thread meets the same table every round)
        atomicMin(&bias_ord[e % m], mins[(size_t)q * nprobe * m + e]);
    __syncthreads();
    if (tid < m) bias_s[tid] = ord2f(bias_ord[tid]);
    __syncthreads();
    float qmax = 0.0f;  // (no code in the probed lists)
    if (n_walk > 0)     // uniform
        qmax = ord2f(block_radix_select<unsigned, 4>(cand_s, (unsigned)n_walk, (unsigned)min(R, n_walk), &sc));
    if (tid == 0) {
        float qmin;
        if (qmin_mode == QADC_QMIN_GLOBAL) {
            qmin = bias_s[0];
            for (int j = 1; j < m; ++j) qmin = fminf(qmin, bias_s[j]);
            for (int j = 0; j < m; ++j) bias_s[j] = qmin;
        } else {
            qmin = 0.0f;
            for (int j = 0; j < m; ++j) qmin = qmin + bias_s[j];
        }
        float delta = __fdiv_rn(qmax - qmin, (float)nbins);
        if (!(delta > 0.0f)) delta = 1.0f;
        qdelta[q] = delta;
        qmax_out[q] = qmax;
    }
    __syncthreads();
    if (tid < m) qbias[(size_t)q * m + tid] = bias_s[tid];
}

// ------------------------------------------------------------------- Seed
//
// A bound for the scan: the quantized sums (Alg. 2) of a sample of the query's codes -- the
// first `per_list` codes of every probed list -- are histogrammed by one workgroup per query;
// the bin where the running count reaches R bounds the query's R-th smallest sum from above.
// It is left in the first word of the query's control block as bound + 1 (0: no bound).
// The sample uses the 16-entry tables directly (two lookups per code byte): building pair
// tables for every cell would cost more than the sample itself.
constexpr int IVF_SEED_NT = 1024;
constexpr int IVF_SEED_PROBES = 16;  // closest cells whose lists are sampled
constexpr int IVF_SEED_PCH = 32;  // probed cells whose tables are in LDS at a time

template <int B>
__global__ __launch_bounds__(IVF_SEED_NT) void ivf_seed_kernel(
    const int64_t *__restrict__ list_off, const uint8_t *__restrict__ codes,
    const int32_t *__restrict__ probes, int nprobe, const uint8_t *__restrict__ qluts, int cap_i,
    int R, int per_list, char *__restrict__ ws, size_t ws_stride, int64_t n_total, int long_shift, int nseed,
    IvfQuantizer fq)
{
    constexpr int NT = IVF_SEED_NT;
    constexpr int TAB = 2 * B * 16;  // bytes of one cell's quantized tables
    __shared__ __attribute__((aligned(16))) uint8_t tab[IVF_SEED_PCH * TAB];
    __shared__ long long lo[IVF_MAX_NPROBE];
    __shared__ int len[IVF_MAX_NPROBE];
    __shared__ int more[IVF_MAX_NPROBE];  // codes sampled beyond per_list (long lists, long_shift > 0)
    __shared__ unsigned hist[256];
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    // a few queries: the probed lists of a query are split over gridDim.y workgroups, which add
    // their histograms into the query's control block
    const int parts = gridDim.y;
    // (nseed <= nprobe: only the lists of the nseed closest cells are sampled)
    const int per_part = (nseed + parts - 1) / parts;
    const int p_begin = blockIdx.y * per_part, p_end = min(nseed, p_begin + per_part);
    const unsigned cap = (unsigned)cap_i;
    if (tid < nprobe) {
        const int cell = probes[(size_t)q * nprobe + tid];
        long long l = 0, h = 0;
        if (cell >= 0) { l = list_off[cell]; h = list_off[cell + 1]; }
        if (l < 0 || h > n_total || h < l) l = h = 0;  // offsets that are not a list: nothing is read
        lo[tid] = l;
        len[tid] = (int)min((long long)per_list, h - l);
        // with long_shift the sample of a list is at least its 2^-long_shift part: the bound then
        // reflects the lists in proportion to their lengths
        more[tid] = long_shift > 0 ? (int)max(0ll, min((h - l) >> long_shift, 1ll << 30) - per_list) : 0;
    }
    for (int e = tid; e < 256; e += NT) hist[e] = 0;
    for (int p0 = p_begin; p0 < p_end; p0 += IVF_SEED_PCH) {  // uniform
        const int np = min(IVF_SEED_PCH, p_end - p0);
        __syncthreads();  // geometry and histogram ready; nobody still reads the previous tables
        if (fq.luts) {  // uniform
            const float *src = fq.luts + ((size_t)q * nprobe + p0) * TAB;
            const float delta = fq.delta[q];
            for (int e = tid; e < np * (TAB / 4); e += NT)
                reinterpret_cast<unsigned *>(tab)[e] =
                    quantize_word(src + (size_t)(e / (TAB / 4)) * TAB, e % (TAB / 4),
                                  fq.bias + (size_t)q * (2 * B), delta, cap);
        } else {
            const unsigned *src = reinterpret_cast<const unsigned *>(qluts + ((size_t)q * nprobe + p0) * TAB);
            for (int e = tid; e < np * (TAB / 4); e += NT) reinterpret_cast<unsigned *>(tab)[e] = src[e];
        }
        __syncthreads();
        for (int i = tid; i < np * per_list; i += NT) {
            const int pp = i / per_list, c = i - pp * per_list;
            if (c >= len[p0 + pp]) continue;
            const unsigned *cw = reinterpret_cast<const unsigned *>(codes + (size_t)(lo[p0 + pp] + c) * B);
            const uint8_t *t = tab + pp * TAB;
            unsigned sum = 0;
#pragma unroll
            for (int k = 0; k < B / 4; ++k) {
                const unsigned x = cw[k];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const unsigned v = (x >> (8 * b)) & 0xffu;
                    const int jb = 4 * k + b;
                    sum += (unsigned)t[(2 * jb) * 16 + (v & 15u)] + (unsigned)t[(2 * jb + 1) * 16 + (v >> 4)];
                }
            }
            if (sum < cap) atomicAdd(&hist[sum], 1u);  // saturated sums carry no information
        }
        for (int pp = 0; pp < np; ++pp) {  // uniform
            const int extra = more[p0 + pp];
            const uint8_t *t = tab + pp * TAB;
            for (int c = per_list + tid; c < per_list + extra; c += NT) {
                const unsigned *cw = reinterpret_cast<const unsigned *>(codes + (size_t)(lo[p0 + pp] + c) * B);
                unsigned sum = 0;
#pragma unroll
                for (int k = 0; k < B / 4; ++k) {
                    const unsigned x = cw[k];
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const unsigned v = (x >> (8 * b)) & 0xffu;
                        const int jb = 4 * k + b;
                        sum += (unsigned)t[(2 * jb) * 16 + (v & 15u)] + (unsigned)t[(2 * jb + 1) * 16 + (v >> 4)];
                    }
                }
                if (sum < cap) atomicAdd(&hist[sum], 1u);
            }
        }
    }
    __syncthreads();
    ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
    if (parts > 1) {
        // ghist[1][bin]: the query's histogram over all parts; every workgroup of the scan kernel derives
        // the bound from it (the launch boundary orders the two; no count of finished parts, no fences)
        if (tid < 256 && hist[tid])
            __hip_atomic_fetch_add(&hdr->ghist[1][tid], hist[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;  // uniform
    }
    if (tid < WAVE) {
        unsigned h[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) h[b] = hist[4 * tid + b];
        const unsigned t = wave_threshold_bin<4>(h, (unsigned)R);
        if (tid == 0) hdr->ghist[0][0] = (t < 256u) ? t + 1u : 0u;
    }
}

// ------------------------------------------------------------------- Scan

constexpr int IVF_MAP_NT = 1024;
constexpr int IVF_MAP_MAXQ = 4096;   // queries per batch, at most
constexpr unsigned IVF_NO_WG = 0xffffffffu;

// Workgroups of the scan: query q gets W_q = clamp(ceil(units_q / units_per_wg), 1, Wmax) of them
// (work in proportion to the lists it probes); the queries with the most work come first in the
// grid, so that the longest-running workgroups start first.  wgmap[b] = q << 12 | g for workgroup
// b of the grid, IVF_NO_WG beyond the last one.  One workgroup; nb <= IVF_MAP_MAXQ, Wmax <= 4096.
// With `flags`, a query whose flag is not 1 is scanned over its other set of cells (see ivf_scan_kernel)
// and its units are qunits_alt's.
__global__ __launch_bounds__(IVF_MAP_NT) void ivf_wgmap_kernel(const unsigned *__restrict__ qunits, int nb,
                                                              int units_per_wg, int Wmax,
                                                              unsigned *__restrict__ wgmap,
                                                              const unsigned *__restrict__ qunits_alt,
                                                              const unsigned *__restrict__ flags)
{
    __shared__ unsigned un[IVF_MAP_MAXQ];      // units of query q
    __shared__ unsigned byrank[IVF_MAP_MAXQ];  // query at rank r
    __shared__ unsigned start[IVF_MAP_MAXQ + 1];  // first workgroup of rank r
    __shared__ unsigned wsum[IVF_MAP_NT / WAVE];
    __shared__ unsigned carry;
    const int tid = threadIdx.x;
    auto wgs_of = [&](unsigned u) {
        return (unsigned)min((long long)Wmax, max(1ll, ((long long)u + units_per_wg - 1) / units_per_wg));
    };
    for (int q = tid; q < nb; q += IVF_MAP_NT) un[q] = (flags && flags[q] != 1u) ? qunits_alt[q] : qunits[q];
    if (tid == 0) carry = 0;
    __syncthreads();
    // rank by (units descending, query ascending): a total order, so ranks are distinct.  (With
    // `flags` the long lists have been scanned elsewhere and what is left is short and even: the
    // queries keep their order, which saves the nb x nb comparisons.)
    for (int q = tid; q < nb; q += IVF_MAP_NT) {
        if (flags) {
            byrank[q] = (unsigned)q;
            continue;
        }
        const unsigned u = un[q];
        unsigned r = 0;
        for (int o = 0; o < nb; ++o) {
            const unsigned v = un[o];
            r += (v > u || (v == u && o < q)) ? 1u : 0u;
        }
        byrank[r] = (unsigned)q;
    }
    __syncthreads();
    // exclusive running sum of the workgroup counts in rank order
    for (int r0 = 0; r0 < nb; r0 += IVF_MAP_NT) {
        const int r = r0 + tid;
        const unsigned w = r < nb ? wgs_of(un[byrank[r]]) : 0u;
        unsigned inc = w;
        const int l = lane_id();
#pragma unroll
        for (int dd = 1; dd < WAVE; dd <<= 1) {
            const unsigned up = __shfl_up(inc, dd);
            if (l >= dd) inc += up;
        }
        if (l == WAVE - 1) wsum[tid / WAVE] = inc;
        __syncthreads();
        unsigned before = carry;
        for (int wv = 0; wv < tid / WAVE; ++wv) before += wsum[wv];
        if (r < nb) start[r] = before + inc - w;
        __syncthreads();
        if (tid == IVF_MAP_NT - 1) carry = before + inc;
        __syncthreads();
    }
    if (tid == 0) start[nb] = carry;
    __syncthreads();
    const unsigned total = start[nb];
    const unsigned slots = (unsigned)nb * (unsigned)Wmax;
    for (unsigned b = tid; b < slots; b += IVF_MAP_NT) {
        unsigned v = IVF_NO_WG;
        if (b < total) {
            int lo_r = 0, hi_r = nb;  // last rank whose first workgroup is <= b
            while (hi_r - lo_r > 1) {
                const int mid = (lo_r + hi_r) >> 1;
                if (start[mid] <= b) lo_r = mid; else hi_r = mid;
            }
            v = (byrank[lo_r] << 12) | (b - start[lo_r]);
        }
        wgmap[b] = v;
    }
}


struct IvfShared {
    SelectScratch sel;
    unsigned ccnt;
    unsigned tcnt[3];
    unsigned tau;
    unsigned fcnt;                         // append counter of the barrier-free pass
    unsigned long long wsum[1024 / WAVE];  // unit counts of the wavefronts (prefix sum)
    long long ustart[IVF_MAX_NPROBE + 1];  // units before probe p
    long long a0[IVF_MAX_NPROBE];          // list start rounded down to 16 codes
    long long lo[IVF_MAX_NPROBE];
    long long hi[IVF_MAX_NPROBE];
};

// NT threads per workgroup: IVF_NT for batches; 1024 for a few queries, whose lists must be read
// by few workgroups at once (a workgroup has one tile in flight and the next one requested).
template <int B, int NT>
__global__ __launch_bounds__(NT) void ivf_scan_kernel(
    const int64_t *__restrict__ list_off, const uint8_t *__restrict__ codes, int64_t n_total,
    const int32_t *__restrict__ probes, int nprobe, const uint8_t *__restrict__ qluts, int cap_i,
    int R, int units_per_wg, int Wmax, const unsigned *__restrict__ wgmap, char *__restrict__ ws,
    size_t ws_stride, size_t counts_off, size_t lists_off, const int32_t *__restrict__ probes_alt,
    const unsigned *__restrict__ flags, IvfQuantizer fq, int hist_bound)
{
    using C = ScanCfg<B, NT>;
    constexpr long long UNIT = (long long)IVF_UNIT_TILES * IVF_NT * C::CPT;  // the same codes whatever NT
    static_assert(UNIT % C::TILE == 0, "whole tiles per unit");
    // without a map (a few queries): Wmax workgroup slots per query, in query order
    const unsigned me = wgmap ? wgmap[blockIdx.x]
                              : ((blockIdx.x / (unsigned)Wmax) << 12) | (blockIdx.x % (unsigned)Wmax);  // uniform
    if (me == IVF_NO_WG) return;
    __shared__ __attribute__((aligned(16))) uint8_t ptab[B * 256];
    __shared__ __attribute__((aligned(16))) uint8_t qlut_s[2 * B * 16];
    __shared__ uint64_t keys[C::CAP];
    __shared__ IvfShared sh;

    const int tid = threadIdx.x;
    const int q = (int)(me >> 12);
    const int g = (int)(me & 4095u);
    const unsigned cap = (unsigned)cap_i;
    // bound + 1 left by the seed kernel (uniform load), 0 when there is none; hist_bound: the seed
    // kernel's workgroups left the query's histogram instead, and the bound is derived below
    const ScanHeader *hdr_in = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride);
    unsigned tau1 = hist_bound ? 0u : hdr_in->ghist[0][0];
    unsigned hb[4] = {0, 0, 0, 0};
    if (hist_bound && tid < WAVE) {
        const uint4 v = *reinterpret_cast<const uint4 *>(&hdr_in->ghist[1][4 * tid]);
        hb[0] = v.x; hb[1] = v.y; hb[2] = v.z; hb[3] = v.w;
    }

    // Geometry of the probed lists, one thread per probe, then an exclusive prefix sum of the
    // unit counts.
    static_assert(IVF_MAX_NPROBE <= NT, "one thread per probe");
    unsigned long long my_units = 0;
    // (with flags: a query whose flag is not 1 leaves some of its cells to the shared-list scan and
    // takes the others, probes_alt, here; the tables stay indexed by the slot)
    const int32_t *pr = (flags && flags[q] != 1u) ? probes_alt : probes;  // uniform
    if (tid < nprobe) {
        const int cell = pr[(size_t)q * nprobe + tid];
        long long l = 0, h = 0;
        if (cell >= 0) { l = list_off[cell]; h = list_off[cell + 1]; }
        if (l < 0 || h > n_total || h < l) l = h = 0;  // offsets that are not a list: nothing is read
        const long long a = l / 16 * 16;
        sh.lo[tid] = l;
        sh.hi[tid] = h;
        sh.a0[tid] = a;
        my_units = (h > l) ? (unsigned long long)((h - a + UNIT - 1) / UNIT) : 0ull;
    }
    {
        const int l = lane_id();
        unsigned long long inc = my_units;
#pragma unroll
        for (int dd = 1; dd < WAVE; dd <<= 1) {
            const unsigned long long up = __shfl_up(inc, dd);
            if (l >= dd) inc += up;
        }
        if (l == WAVE - 1) sh.wsum[tid / WAVE] = inc;
        __syncthreads();
        unsigned long long before = 0;
        for (int wv = 0; wv < tid / WAVE; ++wv) before += sh.wsum[wv];
        if (tid < nprobe) sh.ustart[tid] = (long long)(before + inc - my_units);
        if (tid == nprobe - 1) sh.ustart[nprobe] = (long long)(before + inc);
        if (tid == 0) { sh.tcnt[0] = 0; sh.fcnt = 0; }
    }
    if (hist_bound && tid < WAVE) {  // the bin where the running count of the sample reaches R
        const unsigned t = wave_threshold_bin<4>(hb, (unsigned)R);
        if (tid == 0) sh.tau = (t < 256u) ? t + 1u : 0u;
    }
    for (int e = tid; e < 256; e += NT) sh.sel.hist[e] = 0;
    __syncthreads();
    if (hist_bound) tau1 = sh.tau;  // uniform
    const long long units = sh.ustart[nprobe];
    // Workgroups of this query: in proportion to its work (a query whose cell is one of the few
    // huge lists gets up to Wmax of them, a query of short lists a handful) -- the count the
    // map kernel derived from the same number of units.
    const int W = (int)min((long long)Wmax, max(1ll, (units + units_per_wg - 1) / units_per_wg));
    if (g >= W) return;  // uniform; with a map it cannot happen

    uint64_t lim = ~0ull;  // keys >= lim cannot be among the R best of this workgroup's codes
    unsigned have = 0;
    int rot = 0;
    int cur_p = -1;
    bool first_tile = true;
    const long long ub = units * g / W, ue = units * (g + 1) / W;

    // probe of unit u (binary search, same result in every thread)
    auto probe_of = [&](long long u) {
        int lo_p = 0, hi_p = nprobe;
        while (hi_p - lo_p > 1) {
            const int mid = (lo_p + hi_p) >> 1;
            if (sh.ustart[mid] <= u) lo_p = mid; else hi_p = mid;
        }
        return lo_p;
    };
    // pair tables of probe p (called by the whole workgroup)
    auto load_tables = [&](int p) {
        __syncthreads();  // nobody still reads the previous pair tables
        if (fq.luts) {  // uniform
            const float *lt = fq.luts + ((size_t)q * nprobe + p) * (2 * B) * 16;
            const float delta = fq.delta[q];
            for (int e = tid; e < 2 * B * 4; e += NT)
                reinterpret_cast<unsigned *>(qlut_s)[e] =
                    quantize_word(lt, e, fq.bias + (size_t)q * (2 * B), delta, cap);
        } else {
            const uint8_t *qlut = qluts + ((size_t)q * nprobe + p) * (2 * B) * 16;
            for (int e = tid; e < 2 * B * 4; e += NT)
                reinterpret_cast<unsigned *>(qlut_s)[e] = reinterpret_cast<const unsigned *>(qlut)[e];
        }
        __syncthreads();
        for (int e = tid; e < B * 256; e += NT) {
            const int jb = e >> 8, v = e & 255;
            const unsigned s = (unsigned)qlut_s[(2 * jb) * 16 + (v & 15)] +
                               (unsigned)qlut_s[(2 * jb + 1) * 16 + (v >> 4)];
            ptab[e] = (uint8_t)min(s, cap);
        }
        __syncthreads();
    };

    // With a bound: no barrier inside a unit.  The bound is below the saturation value, so a
    // sum that passes needs no clamp; the append code only runs in waves with a hit.  After
    // each unit the list is looked at: the nearest cells hold most of a query's candidates, so
    // the workgroups that scan them cut their list back to its R smallest keys (which tightens
    // their own bound) whenever it grows.  Should the list overflow inside a unit, everything
    // is redone by the careful pass below.
    bool careful = true;
    if (tau1 != 0u) {
        careful = false;
        lim = (uint64_t)tau1 << 32;  // keys with sum <= bound
        for (long long u = ub; u < ue; ++u) {  // uniform
            const int p = probe_of(u);
            const long long lo = sh.lo[p], hi = sh.hi[p];
            const long long u0 = sh.a0[p] + (u - sh.ustart[p]) * UNIT;
            const long long u1 = min(hi, u0 + UNIT);
            // The next tile of the unit is requested before the current one is used; on a change of
            // list the new tables are requested first and the unit's first tile right behind them
            // (loads return in the order they were issued), so the tile travels while the pair
            // tables are rebuilt.
            uint4 w[2], wn[2];
            int nc[2], ncn[2];
            const bool new_list = p != cur_p;  // uniform
            unsigned qword = 0;
            float4 fword = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (new_list && tid < 2 * B * 4) {
                if (fq.luts)  // uniform
                    fword = reinterpret_cast<const float4 *>(fq.luts + ((size_t)q * nprobe + p) * (2 * B) * 16)[tid];
                else
                    qword = reinterpret_cast<const unsigned *>(qluts + ((size_t)q * nprobe + p) * (2 * B) * 16)[tid];
            }
            asm volatile("" ::: "memory");
            tile_load<B, NT>(codes, u0, n_total, wn, ncn);
            asm volatile("" ::: "memory");
            if (new_list) {
                __syncthreads();  // nobody still reads the previous pair tables
                if (fq.luts && tid < 2 * B * 4) {  // the query's quantizer applied to the four entries
                    const float b = fq.bias[(size_t)q * (2 * B) + (tid >> 2)];
                    const float delta = fq.delta[q];
                    qword = quantize_entry(fword.x, b, delta, cap) | (quantize_entry(fword.y, b, delta, cap) << 8) |
                            (quantize_entry(fword.z, b, delta, cap) << 16) | (quantize_entry(fword.w, b, delta, cap) << 24);
                }
                if (tid < 2 * B * 4) reinterpret_cast<unsigned *>(qlut_s)[tid] = qword;
                __syncthreads();
                for (int e = tid; e < B * 256; e += NT) {
                    const int jb = e >> 8, v = e & 255;
                    const unsigned sum = (unsigned)qlut_s[(2 * jb) * 16 + (v & 15)] +
                                         (unsigned)qlut_s[(2 * jb + 1) * 16 + (v >> 4)];
                    ptab[e] = (uint8_t)min(sum, cap);
                }
                __syncthreads();
                cur_p = p;
            }
            for (long long t0 = u0; t0 < u1; t0 += C::TILE) {
                w[0] = wn[0]; w[1] = wn[1];
                nc[0] = ncn[0]; nc[1] = ncn[1];
                if (t0 + C::TILE < u1) tile_load<B, NT>(codes, t0 + C::TILE, n_total, wn, ncn);  // uniform
                // Sums only; positions, validity and keys are worked out in the wavefronts that hold a
                // sum small enough to pass (a slot without a code may hold one too: it is dropped there).
                // Entries are not negative, so a code whose first half of the bytes already sums to more
                // than a passing sum may cannot pass: only the lanes that hold a code still in the race
                // look up the other half (a wavefront without one skips it; with few lanes left they no
                // longer collide on the LDS banks), the others keep their partial sum.
                // a key below lim has a sum of at most (lim - 1) >> 32
                const unsigned limsum = (unsigned)((lim - 1ull) >> 32);
                unsigned sm[C::CPT];
                if constexpr (B <= 16) {
                    constexpr int CPV = 16 / B;
                    // stages of bytes, a check after each but the last
                    constexpr int NS = QADC_IVF_EARLY_STAGES(B);
                    constexpr int cut[4] = {0, NS == 3 ? B / 4 : (NS == 2 ? B / 2 : B), NS == 3 ? B / 2 : B, B};
#pragma unroll
                    for (int c = 0; c < 2 * CPV; ++c) sm[c] = 0;
                    bool go = true;
#pragma unroll
                    for (int st = 0; st < NS; ++st) {
                        if (go) {
                            unsigned part = 0xffffffffu;
#pragma unroll
                            for (int v = 0; v < 2; ++v) {
#pragma unroll
                                for (int c = 0; c < CPV; ++c) {
                                    unsigned s = sm[v * CPV + c];
#pragma unroll
                                    for (int jb = cut[st]; jb < cut[st + 1]; ++jb)
                                        s += ptab[jb * 256 + byte_of(w[v], c * B + jb)];
                                    sm[v * CPV + c] = s;
                                    part = min(part, s);
                                }
                            }
                            go = part <= limsum;
                        }
                    }
                } else {
                    unsigned s = 0;
#pragma unroll
                    for (int jb = 0; jb < 16; ++jb) s += ptab[jb * 256 + byte_of(w[0], jb)];
                    if (s <= limsum) {
#pragma unroll
                        for (int jb = 16; jb < 32; ++jb) s += ptab[jb * 256 + byte_of(w[1], jb & 15)];
                    }
                    sm[0] = s;
                }
                unsigned best = sm[0];
#pragma unroll
                for (int c = 1; c < C::CPT; ++c) best = min(best, sm[c]);
                if (__ballot(best <= limsum) != 0ull) {
#pragma unroll
                    for (int c = 0; c < C::CPT; ++c) {
                        long long pos;
                        bool valid;
                        if constexpr (B <= 16) {
                            constexpr int CPV = 16 / B;
                            const int v = c / CPV, cc = c % CPV;
                            pos = t0 + (long long)((v * NT + tid) * CPV + cc);
                            valid = (cc < nc[v]) && pos >= lo && pos < u1;
                        } else {
                            pos = t0 + tid;
                            valid = nc[0] && pos >= lo && pos < u1;
                        }
                        const uint64_t key = ((uint64_t)sm[c] << 32) | (uint64_t)pos;
                        const bool pass = valid && key < lim;
                        const unsigned slot = wave_append_slot(pass, &sh.fcnt);
                        if (pass && slot < (unsigned)C::CAP) keys[slot] = key;
                    }
                }
            }
            __syncthreads();
            have = sh.fcnt;
            __syncthreads();  // everybody has read the count before the next unit bumps it
            if (have > (unsigned)C::CAP) { careful = true; break; }  // uniform: keys were dropped
            // cut the list back once it holds more than R keys and has grown past half its slack
            // (a list of at most R keys is the workgroup's result so far: nothing to drop)
            if (have > max((unsigned)R, (unsigned)SCAN_SLACK / 2)) {
                const uint64_t kth = compact_candidates<uint64_t, 5, NT, C::CAP>(
                    keys, have, (unsigned)R, &sh.sel, &sh.ccnt);
                lim = min(lim, kth + 1ull);
                have = (unsigned)R;
                if (tid == 0) sh.fcnt = (unsigned)R;
                __syncthreads();
            }
        }
        if (careful) { have = 0; cur_p = -1; lim = ~0ull; }
    }

    // Careful pass.  Workgroup g takes a contiguous range of the query's units: consecutive
    // units mostly belong to the same list, so the pair tables are rebuilt only when the list
    // changes.
    for (long long u = ub; careful && u < ue; ++u) {  // uniform
        const int p = probe_of(u);
        if (p != cur_p) { load_tables(p); cur_p = p; }
        const long long lo = sh.lo[p], hi = sh.hi[p];
        const long long u0 = sh.a0[p] + (u - sh.ustart[p]) * UNIT;
        const long long u1 = min(hi, u0 + UNIT);
        for (long long t0 = u0; t0 < u1; t0 += C::TILE) {
            unsigned *ctr = &sh.tcnt[rot];
            const int nxt = (rot == 2) ? 0 : rot + 1;
            if (tid == 0) sh.tcnt[nxt] = 0;
            uint4 w[2];
            int nc[2];
            tile_load<B, NT>(codes, t0, n_total, w, nc);  // may reach into the neighbouring lists
            uint64_t k[C::CPT];
            if constexpr (B <= 16) {
                constexpr int CPV = 16 / B;
#pragma unroll
                for (int v = 0; v < 2; ++v) {
#pragma unroll
                    for (int c = 0; c < CPV; ++c) {
                        unsigned s = 0;
#pragma unroll
                        for (int jb = 0; jb < B; ++jb) s += ptab[jb * 256 + byte_of(w[v], c * B + jb)];
                        s = min(s, cap);
                        const long long pos = t0 + (long long)((v * NT + tid) * CPV + c);
                        const bool valid = (c < nc[v]) && pos >= lo && pos < u1;
                        k[v * CPV + c] = valid ? (((uint64_t)s << 32) | (uint64_t)pos) : ~0ull;
                    }
                }
            } else {
                unsigned s = 0;
#pragma unroll
                for (int jb = 0; jb < 32; ++jb) s += ptab[jb * 256 + byte_of(w[jb >> 4], jb & 15)];
                s = min(s, cap);
                const long long pos = t0 + tid;
                const bool valid = nc[0] && pos >= lo && pos < u1;
                k[0] = valid ? (((uint64_t)s << 32) | (uint64_t)pos) : ~0ull;
            }

            if (first_tile) {
                // bound the workgroup's share by its own first tile: the bin of the R-th
                // smallest unsaturated sum (keys above it cannot be among the R best)
#pragma unroll
                for (int c = 0; c < C::CPT; ++c)
                    if (k[c] != ~0ull && (unsigned)(k[c] >> 32) < cap)
                        atomicAdd(&sh.sel.hist[(unsigned)(k[c] >> 32)], 1u);
                __syncthreads();
                if (tid < WAVE) {
                    const int l = tid;
                    unsigned h0 = sh.sel.hist[4 * l], h1 = sh.sel.hist[4 * l + 1];
                    unsigned h2 = sh.sel.hist[4 * l + 2], h3 = sh.sel.hist[4 * l + 3];
                    const unsigned tot = h0 + h1 + h2 + h3;
                    unsigned inc = tot;
#pragma unroll
                    for (int dd = 1; dd < WAVE; dd <<= 1) {
                        const unsigned up = __shfl_up(inc, dd);
                        if (l >= dd) inc += up;
                    }
                    const unsigned long long mm = __ballot(inc >= (unsigned)R);
                    unsigned t = cap;
                    if (mm) {
                        const int fl = __ffsll((long long)mm) - 1;
                        unsigned run = inc - tot, bin = 4u * l + 3u;
                        const unsigned hh[4] = {h0, h1, h2, h3};
                        bool found = false;
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            run += hh[b];
                            if (!found && run >= (unsigned)R) { bin = 4u * l + b; found = true; }
                        }
                        t = __shfl(bin, fl);
                    }
                    if (tid == 0) sh.tau = min(t, cap);
                }
                __syncthreads();
                lim = ((uint64_t)sh.tau + 1ull) << 32;
                first_tile = false;
            }

            uint64_t best = k[0];
#pragma unroll
            for (int c = 1; c < C::CPT; ++c) best = min(best, k[c]);
            if (__ballot(best < lim) != 0ull) {  // the append code only runs in waves with a hit
#pragma unroll
                for (int c = 0; c < C::CPT; ++c) {
                    const bool pass = k[c] < lim;
                    const unsigned slot = have + wave_append_slot(pass, ctr);
                    if (pass) keys[slot] = k[c];
                }
            }
            __syncthreads();
            have += *ctr;
            rot = nxt;
            if (have > (unsigned)SCAN_SLACK) {
                const uint64_t kth = compact_candidates<uint64_t, 5, NT, C::CAP>(
                    keys, have, (unsigned)R, &sh.sel, &sh.ccnt);
                lim = min(lim, kth + 1ull);
                have = (unsigned)R;
            }
        }
    }

    if (have > (unsigned)R) {
        compact_candidates<uint64_t, 5, NT, C::CAP>(keys, have, (unsigned)R, &sh.sel, &sh.ccnt);
        have = (unsigned)R;
    }
    if (have == 0) return;
    unsigned *counts = reinterpret_cast<unsigned *>(ws + (size_t)q * ws_stride + counts_off);
    uint64_t *dst = reinterpret_cast<uint64_t *>(ws + (size_t)q * ws_stride + lists_off) + (size_t)g * R;
    if (tid == 0) counts[g] = have;
    for (unsigned i = tid; i < have; i += NT) dst[i] = keys[i];
}

// out_ids[q][r] = ids[position] for the positions the merge kernel wrote (in place).  Anything
// that is not a storage position becomes the padding value.
// Cells given by the caller: a cell outside [0, K) and a cell that an earlier slot of the same
// query already names become unused slots (-1) -- a list is scanned once, so that keys stay
// unique, and nothing outside list_off is read.
__global__ void ivf_take_probes_kernel(const int32_t *__restrict__ in, int nprobe, int K, int64_t total,
                                       int32_t *__restrict__ probes, IvfClear clr, int nq)
{
    if (clr.scan_ws && (int)blockIdx.x < nq) {  // uniform: workgroup b also clears the control words of query b
        ivf_clear_control(clr.scan_ws + (size_t)blockIdx.x * clr.ws_stride, clr.counts_off, clr.W, clr.countsA_off);
    }
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int64_t row = i / nprobe * nprobe;
    int cell = in[i];
    if (cell < 0 || cell >= K) cell = -1;
    for (int64_t o = row; cell >= 0 && o < i; ++o)
        if (in[o] == cell) cell = -1;
    probes[i] = cell;
}

// ------------------------------------------------------------------- host

int quantize_luts(int, const float *, int, int, int, const uint8_t *, int64_t, const float *, int, int,
                  int, uint8_t *, float *, float *, float *, hipStream_t);

struct IvfPlan {
    int qb, W;
    int qd;  // queries per pass of the Index step (its distances take K floats per query)
    int seed_per_list;  // codes sampled per probed list for the bound of the scan (0: no seed kernel)
    ScanLayout l;
    size_t off_dist, off_bmin, off_front, off_probes, off_luts, off_qluts, off_qmax, off_units, off_map, off_scan, bytes;
    // shared-list scan of large batches (ivf_shared_scan): a second report region per query, the
    // pairs sorted by cell and their offsets
    bool shared;
    int shared_wgs;
    size_t stride, countsA_off, listsA_off;
    size_t off_paircnt, off_pairoff, off_item0, off_item1, off_pairs, off_taus, off_flags, off_plight, off_ulight;
    int shared_min_pairs;
};

constexpr int IVF_SHARED_PITCH = MERGE_CAP;   // keys of a query's region: what the merge kernel holds in LDS
constexpr int IVF_SHARED_MIN_Q = 384;         // smallest batch whose popular lists are scanned once for all (even at 360 on 65536 Zipf lists)
constexpr int IVF_SHARED_MAX_R = 128;         // the region must hold a few dozen times R keys
constexpr int IVF_SHARED_MAX_K = 1 << 18;     // one workgroup sums the per-cell counts

constexpr int IVF_SHARED_MIN_PAIRS = 4;       // pairs of a cell from which its list is scanned once for all of them

int ivf_shared_scan(int, const int64_t *, const uint8_t *, int64_t, int, const int32_t *, int, int, const uint8_t *,
                    int, char *, size_t, size_t, size_t, int, unsigned *, unsigned *, unsigned *, unsigned *,
                    unsigned *, unsigned *, unsigned *, int32_t *, unsigned *, long long, int, int, hipStream_t);

static bool make_ivf_plan(const qadc_ivf_index *ix, int nq, int nprobe, int R, IvfPlan *p)
{
    if (!ix || nq < 1 || nprobe < 1 || nprobe > IVF_MAX_NPROBE || R < 1 || R > QADC_MAX_R) return false;
    if (!(ix->m == 8 || ix->m == 16 || ix->m == 32 || ix->m == 64)) return false;
    if (ix->d < ix->m || ix->d % ix->m || ix->K < 1 || ix->n < 0 || ix->n > 0xfffffffell) return false;
    // Most workgroups a query can get: 128 for up to 128 queries, fewer for larger calls, about
    // 16384 workgroup slots per launch (measured at N = 1e9: 4096 queries 161 K queries/s with 24 to
    // 32 against 156 K with 128; 1024 queries best with 24, 512 with 32 to 48, 256 with 64, 128 with
    // 96 to 128); the regions of a query shrink with it, so a launch holds more queries.
    // (13 to 63 queries: 256, measured 0.286 against 0.320 ms at 16 queries, 0.402 against 0.458 at 32)
    int w_def = 16384 / nq;
    if (w_def < 24) w_def = 24;
    // (up to 4 queries: 192, one query 0.0744 against 0.0780 ms)
    if (w_def > 128) w_def = (nq > IVF_WIDE_MAX_Q && nq < 64) ? 256 : nq <= 4 ? 192 : 128;
    p->W = knob_or(knobs().ivf_wgs, w_def);
    if (p->W < 1) p->W = 1;
    if (p->W > 4096) p->W = 4096;
    // about 1/16 of an average list, between 64 and 1024 codes
    int64_t spl = ix->n / ix->K / 16;
    if (spl < 64) spl = 64;
    if (spl > 1024) spl = 1024;
    p->seed_per_list = knob_or(knobs().ivf_seed, 1) ? (int)spl : 0;
    p->l = scan_layout(p->W, R);
    // large batches over a moderate number of cells: every list is scanned once for all the queries
    // that probe it (QADC_IVF_SHARED=1 / 0 forces / forbids it)
    const int shared_knob = knobs().ivf_shared;
    p->shared = R <= IVF_SHARED_MAX_R && ix->K <= IVF_SHARED_MAX_K && p->seed_per_list > 0 && ix->m <= 64 &&
                (shared_knob >= 0 ? shared_knob != 0 : nq >= IVF_SHARED_MIN_Q);
    p->shared_wgs = std::max(1, std::min(65535, knob_or(knobs().ivf_shared_wgs, 32768)));
    p->shared_min_pairs = std::max(1, knob_or(knobs().ivf_shared_min_pairs, IVF_SHARED_MIN_PAIRS));
    p->stride = p->l.stride;
    p->countsA_off = p->listsA_off = 0;
    if (p->shared) {
        p->countsA_off = p->l.stride;
        p->listsA_off = p->countsA_off + 256;
        p->stride = p->listsA_off + align_up((size_t)IVF_SHARED_PITCH * sizeof(uint64_t), 256);
    }
    const size_t kdist = ix->coarse ? (size_t)ix->K : 0;  // the Index step's distances
    const size_t per_q = align_up((size_t)nprobe * 4, 256) + align_up((size_t)nprobe * ix->m * 16 * 4, 256) +
                         align_up((size_t)nprobe * ix->m * 16, 256) + 256 + 4 + (size_t)p->W * 4 + p->stride +
                         (p->shared ? (size_t)nprobe * 8 + 12 : 0);
    // Queries per launch sequence.  The shared-list scan gains with every query that joins the batch
    // (more pairs per list), so it takes up to IVF_MAP_MAXQ queries in up to 1.5 GiB; the per-query
    // scan is indifferent and stays within 512 MiB.  The Index step's distances (K floats per query)
    // are computed for at most 256 MiB of queries at a time inside a sequence.
    const size_t budget = p->shared ? (1536ull << 20) : (512ull << 20);
    const size_t dist_budget = p->shared ? (256ull << 20) : 0;
    int64_t qb = (int64_t)(budget / (per_q + (p->shared ? 0 : align_up(kdist * 4, 256))));
    if (qb < 1) qb = 1;
    if (qb > nq) qb = nq;
    if (qb > IVF_MAP_MAXQ) qb = IVF_MAP_MAXQ;
    p->qb = (int)qb;
    int64_t qd = qb;  // queries per pass of the Index step
    if (dist_budget && kdist) qd = std::max<int64_t>(1, std::min<int64_t>(qb, (int64_t)(dist_budget / (kdist * 4))));
    p->qd = (int)qd;
    size_t o = 0;
    p->off_dist = o;   o += align_up((size_t)qd * kdist * 4, 256);
    p->off_bmin = o;   o += align_up((size_t)qd * ceil_div((int64_t)kdist, (int64_t)IVF_CT) * 4, 256);  // minima of the runs of cells
    // calls of up to 32 queries (ivf_front_kernel): biases [32][64], deltas, lengths of the walks, the sums of the init
    // codes [32][QADC_MAX_INIT], the minima of the tables [32][nprobe][m]
    p->off_front = o;
    o += 32 * 64 * 4 + 256 + 256 + (size_t)32 * QADC_MAX_INIT * 4 + align_up((size_t)32 * nprobe * ix->m * 4, 256);
    p->off_probes = o; o += align_up((size_t)qb * nprobe * 4, 256);
    p->off_luts = o;   o += align_up((size_t)qb * nprobe * ix->m * 16 * 4, 256);
    p->off_qluts = o;  o += align_up((size_t)qb * nprobe * ix->m * 16, 256);
    p->off_qmax = o;   o += align_up((size_t)qb * 4, 256);
    p->off_units = o;  o += align_up((size_t)qb * 4, 256);
    p->off_map = o;    o += align_up((size_t)qb * p->W * 4, 256);
    p->off_scan = o;   o += p->stride * (size_t)qb;
    p->off_paircnt = p->off_pairoff = p->off_item0 = p->off_item1 = p->off_pairs = p->off_taus = p->off_flags = 0;
    p->off_plight = p->off_ulight = 0;
    if (p->shared) {
        const size_t kk = align_up(((size_t)ix->K + 1) * 4, 256);
        p->off_paircnt = o; o += kk + 4096;  // (+ the totals of the 1024-cell blocks of the running sums)
        p->off_pairoff = o; o += kk;
        p->off_item0 = o;   o += kk;
        p->off_item1 = o;   o += kk;
        p->off_pairs = o;   o += align_up((size_t)qb * nprobe * 4, 256);
        p->off_taus = o;    o += align_up((size_t)qb * 4, 256);
        p->off_flags = o;   o += align_up((size_t)qb * 4, 256);
        p->off_plight = o;  o += align_up((size_t)qb * nprobe * 4, 256);
        p->off_ulight = o;  o += align_up((size_t)qb * 4, 256);
    }
    p->bytes = o;
    return true;
}

size_t ivf_workspace_bytes(const qadc_ivf_index *ix, int nq, int nprobe, int R)
{
    IvfPlan p;
    if (!make_ivf_plan(ix, nq, nprobe, R, &p)) return 0;
    return p.bytes;
}

int ivf_search(const qadc_ivf_index *ix, const float *queries, int nq, int nprobe, int R, int init,
               int nbins, int qmin_mode, const int32_t *probes_in, uint32_t *out_ids,
               uint8_t *out_dist, int32_t *dbg_probes, uint8_t *dbg_qluts, void *workspace,
               size_t workspace_bytes, hipStream_t st)
{
    IvfPlan p;
    if (nq == 0) return QADC_OK;  // nothing asked for, whatever the pointers
    if (!ix || !queries || !out_ids || !out_dist)
        return fail(QADC_EINVAL, "qadc_ivf_search: null pointer");
    if (!make_ivf_plan(ix, nq, nprobe, R, &p))
        return fail(QADC_EINVAL, "qadc_ivf_search: unsupported nq=%d nprobe=%d R=%d d=%d m=%d K=%d", nq,
                    nprobe, R, ix->d, ix->m, ix->K);
    if (!ix->list_off || !ix->codes || !ix->ids || !ix->codebooks)
        return fail(QADC_EINVAL, "qadc_ivf_search: index has a null pointer");
    if (!ix->coarse) {
        if (!ix->halves || !ix->cell_ids || ix->Kh < 1 || ix->Kh > 16384 || (ix->d & 1))
            return fail(QADC_EINVAL, "qadc_ivf_search: index has neither coarse centroids nor half-centroids with "
                                     "cell ids (Kh=%d d=%d)", ix->Kh, ix->d);
        if (!probes_in)
            return fail(QADC_EINVAL, "qadc_ivf_search: an index without coarse centroids is searched with probes_in "
                                     "(list numbers from qadc_multi_index_slots)");
    }
    if (init < 1 || init > QADC_MAX_INIT || nbins < 1 || nbins > 255)
        return fail(QADC_EINVAL, "qadc_ivf_search: init=%d nbins=%d", init, nbins);
    if (((uintptr_t)ix->codes & 15) != 0)
        return fail(QADC_EINVAL, "qadc_ivf_search: codes must be 16-byte aligned");
    if (!workspace || workspace_bytes < p.bytes)
        return fail(QADC_ENOMEM, "qadc_ivf_search: workspace %zu < %zu bytes", workspace_bytes, p.bytes);
    if (((uintptr_t)workspace & 255) != 0)
        return fail(QADC_EINVAL, "qadc_ivf_search: workspace must be 256-byte aligned");
    const int d = ix->d, m = ix->m, K = ix->K;
    char *ws = (char *)workspace;
    float *dist = (float *)(ws + p.off_dist);
    int32_t *probes = (int32_t *)(ws + p.off_probes);
    float *luts = (float *)(ws + p.off_luts);
    uint8_t *qluts = (uint8_t *)(ws + p.off_qluts);
    float *qmax = (float *)(ws + p.off_qmax);
    unsigned *qunits = (unsigned *)(ws + p.off_units);
    unsigned *wgmap = (unsigned *)(ws + p.off_map);
    char *scan_ws = ws + p.off_scan;
    const int cpt = (m / 2 <= 16) ? SCAN_VEC * (16 / (m / 2)) : 1;
    const long long unit = (long long)IVF_UNIT_TILES * IVF_NT * cpt;  // codes per unit of the scan kernel

    for (int q0 = 0; q0 < nq; q0 += p.qb) {
        const int nb = min(p.qb, nq - q0);
        const float *yq = queries + (size_t)q0 * d;
        // A few queries: Tables and the sums of the qmax walk in one launch, the quantizer's parameters in a
        // second (ivf_front_kernel, ivf_finish_kernel); the tables stay float and are quantized by the kernels that read them; the Index step's kernels
        // clear the control words.
        const bool front = nb <= 32 && !p.shared;
        float *qbias = (float *)(ws + p.off_front);
        float *qdelta = qbias + 32 * 64;
        unsigned *nwalk = (unsigned *)(qdelta + 64);
        unsigned *cand = nwalk + 64;
        unsigned *tmins = cand + (size_t)32 * QADC_MAX_INIT;
        IvfClear clr = {nullptr, 0, 0, 0, 0};
        if (front) clr = IvfClear{scan_ws, p.stride, p.l.counts_off, p.countsA_off, p.W};
        // Index
        if (probes_in) {
            const int64_t np_total = (int64_t)nb * nprobe;
            launch(QADC_PROF_IVF_INDEX, ivf_take_probes_kernel,
                   dim3((unsigned)std::max<int64_t>(ceil_div(np_total, 256), front ? nb : 0)), dim3(256), 0, st,
                   probes_in + (size_t)q0 * nprobe, nprobe, K, np_total, probes, clr, nb);
        } else {
            for (int i0 = 0; i0 < nb; i0 += p.qd) {
                const int ni = min(p.qd, nb - i0);
                const float *yi = yq + (size_t)i0 * d;
                // the minima of the runs of IVF_CT cells go with the distances, and the selection reads
                // only the runs that matter (when there are enough runs)
                unsigned *bmin = nullptr;
                const int nblk = (int)ceil_div(K, IVF_CT);
                if (nblk >= 2 * nprobe && nblk <= IVF_SEL_MAXBLK) bmin = (unsigned *)(ws + p.off_bmin);
                if (nb > 32) {
                    dim3 grid((unsigned)nblk, (unsigned)ceil_div(ni, 128));
                    launch(QADC_PROF_IVF_INDEX, ivf_coarse_dist_kernel<8>, grid, dim3(256), 0, st, ix->coarse, K, d,
                           yi, ni, dist, bmin, nblk);
                } else {
                    const int vec4 = (d % 4 == 0 && ((uintptr_t)ix->coarse & 15) == 0 && ((uintptr_t)yi & 15) == 0) ? 1 : 0;
                    dim3 grid((unsigned)nblk, (unsigned)ceil_div(ni, IVF_FEW_Q));
                    launch(QADC_PROF_IVF_INDEX, ivf_coarse_dist_few_kernel, grid, dim3(256), 0, st, ix->coarse, K, d,
                           yi, ni, dist, bmin, nblk, vec4);
                }
                launch(QADC_PROF_IVF_INDEX, ivf_select_probes_kernel, dim3(ni), dim3(IVF_SEL_NT), 0, st, dist, K,
                       nprobe, probes + (size_t)i0 * nprobe, (const unsigned *)bmin, (int)ceil_div(K, IVF_CT), clr);
            }
        }
        IvfQuantizer fq = {nullptr, nullptr, nullptr};
        int rc = QADC_OK;
        if (front) {
            launch(QADC_PROF_IVF_TABLES, ivf_front_kernel, dim3(nprobe, nb), dim3(IVF_FRONT_NT),
                   (size_t)d * sizeof(double), st, ix->codebooks, d, m, yq, ix->coarse, ix->halves, ix->cell_ids,
                   ix->Kh, probes, nprobe, luts, ix->list_off, ix->codes, ix->n, init, unit, qunits, cand, tmins,
                   nwalk);
            launch(QADC_PROF_IVF_TABLES, ivf_finish_kernel, dim3(nb), dim3(IVF_FINISH_NT), 0, st,
                   (const unsigned *)cand, (const unsigned *)tmins, (const unsigned *)nwalk, nprobe, m, R, nbins,
                   qmin_mode, qmax, qbias, qdelta);
            fq = IvfQuantizer{luts, qbias, qdelta};
            if (dbg_qluts)  // the 8-bit tables are wanted in memory after all
                rc = quantize_luts(16, luts, nb, nprobe, m, nullptr, 0, qmax, R, nbins, qmin_mode, qluts, nullptr,
                                   nullptr, nullptr, st);
        } else {
            // Tables
            bool batch_tables = nb >= 64;
            if (batch_tables) {
#define QADC_LUTS_CASE(D_)                                                                                       \
    case D_:                                                                                                    \
        launch(QADC_PROF_IVF_TABLES, ivf_build_luts_batch_kernel<D_>, dim3(nb), dim3(m * 16), 0, st, ix->codebooks, d, \
               m, yq, ix->coarse, ix->halves, ix->cell_ids, ix->Kh, probes, nprobe, luts);                      \
        break;
                switch (d / m) {
                    QADC_LUTS_CASE(2)
                    QADC_LUTS_CASE(4)
                    QADC_LUTS_CASE(6)
                    QADC_LUTS_CASE(8)
                    QADC_LUTS_CASE(16)
                default:
                    batch_tables = false;
                }
#undef QADC_LUTS_CASE
            }
            if (!batch_tables)
                launch(QADC_PROF_IVF_TABLES, ivf_build_luts_kernel, dim3(nprobe, nb), dim3(256),
                       (size_t)d * sizeof(double), st, ix->codebooks, d, m, yq, ix->coarse, ix->halves, ix->cell_ids,
                       ix->Kh, probes, nprobe, luts);
            // (a few queries: a thread per init code, so that the walk is one round of loads)
            launch(QADC_PROF_IVF_TABLES, ivf_qmax_kernel, dim3(nb), dim3(nb <= 32 ? 1024 : 256), 0, st, ix->list_off, ix->codes,
                   m, probes, nprobe, luts, init, R, qmax, unit, qunits, ix->n, scan_ws, p.stride, p.l.counts_off,
                   p.W, p.countsA_off);
            rc = quantize_luts(16, luts, nb, nprobe, m, nullptr, 0, qmax, R, nbins, qmin_mode, qluts, nullptr,
                               nullptr, nullptr, st);
        }
        if (rc != QADC_OK) return rc;
        // Scan: up to p.W workgroups per query, one per `upw` units of its lists (batches that fill
        // the GPU by their number alone), one per unit otherwise
        dim3 grid((unsigned)p.W * (unsigned)nb);
        const int upw = nb >= 64 ? max(1, knob_or(knobs().ivf_units, 16)) : 1;
        // a few queries: their lists are sampled by several workgroups each
        const int seed_parts_env = knob_or(knobs().ivf_seed_parts, 0);
        // (measured at N = 1e9: one query best with 16, 16 and 32 queries with 8, 64 with 4; the shared-list
        // scan reads the bound itself and needs it in one piece)
        const int parts_def = p.shared || nb >= 256 ? 1 : nb >= 64 ? 4 : nb >= 16 ? 8 : 16;
        const int seed_parts = p.shared ? 1 : min(seed_parts_env > 0 ? seed_parts_env : parts_def, nprobe);
        // the bound is sampled from the lists of the closest cells only: they hold most of a query's best
        // codes, and the sample is most of the seed kernel's cost
        const int nseed = std::min(nprobe, std::max(1, knob_or(knobs().ivf_seed_probes, IVF_SEED_PROBES)));
        unsigned *flags = p.shared ? (unsigned *)(ws + p.off_flags) : nullptr;
#define QADC_IVF_SEED_CASE(B_)                                                                          \
    case B_:                                                                                           \
        launch(QADC_PROF_SEED, ivf_seed_kernel<B_>, dim3(nb, seed_parts), dim3(IVF_SEED_NT), 0, st,    \
               ix->list_off, ix->codes, probes, nprobe, qluts, nbins, R, p.seed_per_list, scan_ws,     \
               p.stride, ix->n, p.shared ? 8 : 0, nseed, fq);                                          \
        break;
        if (p.seed_per_list > 0) {
            switch (m / 2) {
                QADC_IVF_SEED_CASE(4)
                QADC_IVF_SEED_CASE(8)
                QADC_IVF_SEED_CASE(16)
                QADC_IVF_SEED_CASE(32)
            }
        }
#undef QADC_IVF_SEED_CASE
        int32_t *probes_light = p.shared ? (int32_t *)(ws + p.off_plight) : nullptr;
        unsigned *qunits_light = p.shared ? (unsigned *)(ws + p.off_ulight) : nullptr;
        if (p.shared) {
            // the lists wanted by many queries once for all of them; then the per-query kernel takes the
            // remaining cells of every query (all cells of a query left flagged 1)
            rc = ivf_shared_scan(m / 2, ix->list_off, ix->codes, ix->n, K, probes, nb, nprobe, qluts, R, scan_ws,
                                 p.stride, p.countsA_off, p.listsA_off, IVF_SHARED_PITCH,
                                 (unsigned *)(ws + p.off_paircnt), (unsigned *)(ws + p.off_pairoff),
                                 (unsigned *)(ws + p.off_item0), (unsigned *)(ws + p.off_item1),
                                 (unsigned *)(ws + p.off_pairs), (unsigned *)(ws + p.off_taus), flags, probes_light,
                                 qunits_light, unit, p.shared_min_pairs, p.shared_wgs, st);
            if (rc != QADC_OK) return rc;
        }
        // (a few queries need no map: every query gets its p.W workgroup slots in turn)
        const bool mapped = nb >= 64 || p.shared;
        // a few queries: workgroups of 1024 threads (measured at N = 1e9: 1 query 0.121 against 0.136 ms,
        // 4 queries 0.163 against 0.181, 8 queries 0.208 against 0.220, 12 the same, 16 slower)
        const bool wide_wgs = !mapped && nb <= knob_or(knobs().ivf_wide_q, IVF_WIDE_MAX_Q);
        if (mapped)
            launch(QADC_PROF_SEED, ivf_wgmap_kernel, dim3(1), dim3(IVF_MAP_NT), 0, st, qunits, nb, upw, p.W, wgmap,
                   (const unsigned *)qunits_light, (const unsigned *)flags);
        const int hist_bound = (p.seed_per_list > 0 && seed_parts > 1) ? 1 : 0;
#define QADC_IVF_CASE(B_)                                                                              \
    case B_:                                                                                          \
        if (wide_wgs)                                                                                  \
            launch(QADC_PROF_SCAN, ivf_scan_kernel<B_, 1024>, grid, dim3(1024), 0, st, ix->list_off, ix->codes, \
                   ix->n, probes, nprobe, qluts, nbins, R, upw, p.W, mapped ? wgmap : (unsigned *)nullptr, scan_ws, \
                   p.stride, p.l.counts_off, p.l.lists_off, (const int32_t *)probes_light,              \
                   (const unsigned *)flags, fq, hist_bound);                                           \
        else                                                                                           \
            launch(QADC_PROF_SCAN, ivf_scan_kernel<B_, IVF_NT>, grid, dim3(IVF_NT), 0, st, ix->list_off, ix->codes, \
                   ix->n, probes, nprobe, qluts, nbins, R, upw, p.W, mapped ? wgmap : (unsigned *)nullptr, scan_ws, \
                   p.stride, p.l.counts_off, p.l.lists_off, (const int32_t *)probes_light,              \
                   (const unsigned *)flags, fq, hist_bound);                                           \
        break;
        switch (m / 2) {
            QADC_IVF_CASE(4)
            QADC_IVF_CASE(8)
            QADC_IVF_CASE(16)
            QADC_IVF_CASE(32)
        }
#undef QADC_IVF_CASE
        uint32_t *oi = out_ids + (size_t)q0 * R;
        rc = launch_merge<uint8_t, 5>(nb, st, scan_ws, p.stride, p.l.counts_off, p.l.lists_off, p.W,
                                      (unsigned)R, R, (uint8_t)nbins, oi, out_dist + (size_t)q0 * R, p.countsA_off,
                                      p.listsA_off, p.shared ? 1 : 0, p.shared ? IVF_SHARED_PITCH : 0, flags,
                                      (const uint32_t *)ix->ids, (int64_t)ix->n);  // positions -> vector ids
        if (rc != QADC_OK) return rc;
        if (dbg_probes)
            QADC_HIP_TRY(hipMemcpyAsync(dbg_probes + (size_t)q0 * nprobe, probes,
                                        (size_t)nb * nprobe * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        if (dbg_qluts)
            QADC_HIP_TRY(hipMemcpyAsync(dbg_qluts + (size_t)q0 * nprobe * m * 16, qluts,
                                        (size_t)nb * nprobe * m * 16, hipMemcpyDeviceToDevice, st));
    }
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
