// Shared-list form of the inverted-index scan (Section 2.3 of the paper with the tables of
// Section 3.3) for large batches on gfx950.
//
// A batch of a few thousand queries probes the same inverted lists over and over: with 4096
// queries x 64 cells over 65536 Zipf-sized lists, half of all (query, code) pairs fall on the dozen
// longest lists, each wanted by tens of queries, while most lists are wanted by one to four.
// Scanning query by query reads a popular list once per query and is bound by memory.  Here the
// (query, cell) pairs of the batch are counted per cell; the cells probed by at least `min_pairs`
// pairs are scanned ONCE for all their pairs, 32 pairs at a time, on the matrix units: the sum of a
// code for a pair is a one-hot row times the pair's tables (see scan_u8_mfma_kernel for the operand
// layout), so 32 codes x 32 pairs cost m/4 sparse matrix instructions and a code byte fetched from
// memory is used up to 32 times.  Every pair has its own tables (the residual of its query against
// its cell); the bound a sum must meet is its query's.  The other cells stay with the per-query
// kernel (ivf_scan_kernel), which is given the query's remaining cells; the merge kernel joins the
// two reports.
//
// Selection.  A query's first bound comes from the seed kernel (whose sample takes 1/256 of a long
// list, so that the bound reflects the lists in proportion to their lengths); sums at or below the
// bound are appended to the query's region of the workspace with one atomic per (pair, chunk).  To
// keep that region small the scan runs in two parts: first the leading 1/16 of every shared list,
// after which the R-th smallest sum found so far replaces the query's bound and the keys beyond it
// are dropped, then the rest.  A query whose region still overflows, or that has no bound at all,
// is flagged (1) and redone over all its cells by the per-query kernel.  Results do not depend on
// the route: every code whose sum is at or below a valid bound is reported, and the merge orders by
// (sum, storage position).

#include "qadc_scan_common.h"
#include "qadc_onehot.h"

namespace qadc {

constexpr unsigned IVFS_NONE = 0xffffffffu;
constexpr int IVFS_CHUNK = 4096;   // codes of a list per work item, at most (relative positions fit 24 bits)
constexpr int IVFS_LC = 64;        // keys a wavefront holds per pair before it writes them out

// codes of the leading part of a list of n codes: 1/16, whole 32-code steps, at least one
__host__ __device__ inline long long ivfs_lead(long long n)
{
    long long s = ((n + 15) / 16 + 31) / 32 * 32;
    return s < n ? s : n;
}

__global__ __launch_bounds__(256) void ivfs_zero_kernel(unsigned *__restrict__ p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

// One thread per (query, probe slot): counts the pairs of every cell; the thread of a query's
// first slot copies the query's bound and sets its flag (IVFS_NONE and 1 when the seed kernel found none).
__global__ __launch_bounds__(256) void ivfs_count_kernel(const int32_t *__restrict__ probes, int nprobe,
                                                         int64_t npairs, int K, const char *__restrict__ ws,
                                                         size_t ws_stride, unsigned *__restrict__ pair_cnt,
                                                         unsigned *__restrict__ taus, unsigned *__restrict__ flags)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= npairs) return;
    const int cell = probes[i];
    if (cell >= 0 && cell < K) atomicAdd(&pair_cnt[cell], 1u);
    if (i % nprobe == 0) {
        const int64_t q = i / nprobe;
        const unsigned tau1 = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride)->ghist[0][0];
        taus[q] = tau1 ? tau1 - 1u : IVFS_NONE;
        flags[q] = tau1 ? 2u : 1u;  // 2: shared lists here, the others by the per-query kernel; 1: all by that one
    }
}

// Exclusive running sums over the cells of (pairs, work items of the leading parts, work items of the
// rest).  A cell with P >= min_pairs pairs and n codes is ceil(P / qw) sets of pairs times
// ceil(len / IVFS_CHUNK) chunks of either part; a cell with fewer pairs is no work here.  Two launches:
// every workgroup sums its 1024 cells and leaves its totals in blk[3][nblk]; then every workgroup adds
// the totals of the workgroups before it (one workgroup walking all the cells took 64 rounds of
// barriers and LDS chains for 65536 cells).
constexpr int IVFS_OFF_NT = 1024;

__global__ __launch_bounds__(IVFS_OFF_NT) void ivfs_offsets_kernel(const unsigned *__restrict__ pair_cnt,
                                                                   const int64_t *__restrict__ list_off, int K,
                                                                   int64_t n_total, int qw, int min_pairs,
                                                                   unsigned *__restrict__ pair_off,
                                                                   unsigned *__restrict__ item_off0,
                                                                   unsigned *__restrict__ item_off1,
                                                                   unsigned *__restrict__ blk)
{
    __shared__ unsigned wsum[3][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nblk = gridDim.x;
    const int c = blockIdx.x * IVFS_OFF_NT + tid;
    unsigned v[3] = {0, 0, 0};
    if (c < K) {
        const unsigned P = pair_cnt[c];
        long long l = list_off[c], h = list_off[c + 1];
        if (l < 0 || h > n_total || h < l) l = h = 0;  // offsets that are not a list: no work
        const long long n = h - l, s = ivfs_lead(n);
        const unsigned sets = P >= (unsigned)min_pairs ? (P + (unsigned)qw - 1u) / (unsigned)qw : 0u;
        v[0] = P;
        v[1] = sets * (unsigned)((s + IVFS_CHUNK - 1) / IVFS_CHUNK);
        v[2] = sets * (unsigned)((n - s + IVFS_CHUNK - 1) / IVFS_CHUNK);
    }
    unsigned inc[3] = {v[0], v[1], v[2]};
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const unsigned o = __shfl_up(inc[k], s);
            if (lane >= s) inc[k] += o;
        }
    }
    if (lane == 63) {
#pragma unroll
        for (int k = 0; k < 3; ++k) wsum[k][wave] = inc[k];
    }
    __syncthreads();
    unsigned before[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        before[k] = 0;
        for (int w = 0; w < wave; ++w) before[k] += wsum[k][w];
    }
    if (c < K) {
        pair_off[c] = before[0] + inc[0] - v[0];
        item_off0[c] = before[1] + inc[1] - v[1];
        item_off1[c] = before[2] + inc[2] - v[2];
    }
    if (tid == IVFS_OFF_NT - 1) {
#pragma unroll
        for (int k = 0; k < 3; ++k) blk[k * nblk + blockIdx.x] = before[k] + inc[k];
    }
}

__global__ __launch_bounds__(IVFS_OFF_NT) void ivfs_offsets_add_kernel(int K, const unsigned *__restrict__ blk,
                                                                       unsigned *__restrict__ pair_off,
                                                                       unsigned *__restrict__ item_off0,
                                                                       unsigned *__restrict__ item_off1)
{
    __shared__ unsigned base_s[3], all_s[3];
    const int tid = threadIdx.x;
    const int nblk = gridDim.x;
    if (tid < 3) { base_s[tid] = 0; all_s[tid] = 0; }
    __syncthreads();
    for (int b = tid; b < nblk; b += IVFS_OFF_NT) {  // at most 256 workgroups: one round
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const unsigned t = blk[k * nblk + b];
            if (t) {
                if (b < (int)blockIdx.x) atomicAdd(&base_s[k], t);
                atomicAdd(&all_s[k], t);
            }
        }
    }
    __syncthreads();
    const int c = blockIdx.x * IVFS_OFF_NT + tid;
    if (c < K) {
        pair_off[c] += base_s[0];
        item_off0[c] += base_s[1];
        item_off1[c] += base_s[2];
    }
    if (blockIdx.x == 0 && tid == 0) {
        pair_off[K] = all_s[0];
        item_off0[K] = all_s[1];
        item_off1[K] = all_s[2];
    }
}

// One thread per pair: its place among the pairs of its cell (in no particular order: each pair's
// finds go to its own query).  Takes the counts back down to zero.
__global__ __launch_bounds__(256) void ivfs_place_kernel(const int32_t *__restrict__ probes, int64_t npairs, int K,
                                                         const unsigned *__restrict__ pair_off,
                                                         unsigned *__restrict__ pair_cnt,
                                                         unsigned *__restrict__ pairs)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= npairs) return;
    const int cell = probes[i];
    if (cell < 0 || cell >= K) return;
    const unsigned old = atomicSub(&pair_cnt[cell], 1u);
    pairs[pair_off[cell] + old - 1u] = (unsigned)i;
}

// One wavefront per workgroup; the work items (cell, set of 32 pairs, chunk of one part of the
// cell's list) are dealt to the workgroups in turn.  The arithmetic of an item is that of
// scan_u8_mfma_kernel with one group of 32 "queries" = pairs.
template <int B>
__global__ __launch_bounds__(64) void ivfs_scan_kernel(
    int part, const int64_t *__restrict__ list_off, const uint8_t *__restrict__ codes, int64_t n_total, int K,
    const unsigned *__restrict__ pair_off, const unsigned *__restrict__ item_off,
    const unsigned *__restrict__ pairs, int nprobe, const uint8_t *__restrict__ qluts,
    const unsigned *__restrict__ taus, char *__restrict__ ws, size_t ws_stride, size_t countsA_off,
    size_t listsA_off, int pitchA, unsigned *__restrict__ flags)
{
    constexpr int WPC = B / 4;   // 32-bit words per code
    constexpr int QW = 32;       // pairs per wavefront
    constexpr int LC = IVFS_LC;
    constexpr int SUB = 2;       // 32-code steps per load
    constexpr int SHIFT = 128 * 2 * B;  // the matrix units multiply signed bytes: entries go in minus 128
    constexpr int NP = B / 2;    // pairs of code bytes = instructions per 32-code step
    __shared__ unsigned keys[QW][LC];
    __shared__ unsigned cnt[QW];
    __shared__ v2i_t nibval[16];
    __shared__ v2i_t nibpos[16];

    const int l = threadIdx.x;
    const int row = l & 31, half = l >> 5;
    if (l < QW) cnt[l] = 0;
    if (l < 16) onehot_nibble_entry(l, nibval, nibpos);
    __syncthreads();
    const unsigned total = item_off[K];

    for (unsigned item = blockIdx.x; item < total; item += gridDim.x) {  // uniform
        // the cell of the item: the last one whose first item is not beyond it
        int clo = 0, chi = K;
        while (chi - clo > 1) {
            const int mid = (clo + chi) >> 1;
            if (item_off[mid] <= item) clo = mid; else chi = mid;
        }
        const int cell = clo;
        const unsigned p0 = pair_off[cell], P = pair_off[cell + 1] - p0;
        long long ll = list_off[cell], lh = list_off[cell + 1];
        if (P == 0 || ll < 0 || lh > n_total || lh <= ll) continue;  // cannot happen with consistent offsets
        const unsigned sets = (P + QW - 1) / QW;
        const unsigned local = item - item_off[cell];
        const unsigned set = local % sets, ch = local / sets;
        const long long lead = ivfs_lead(lh - ll);
        const long long r0 = part == 0 ? ll : ll + lead, r1 = part == 0 ? ll + lead : lh;
        const int64_t c0 = r0 + (long long)ch * IVFS_CHUNK;
        const int64_t c1 = min((long long)r1, (long long)c0 + IVFS_CHUNK);
        if (c0 >= c1) continue;

        // this lane's pair: its tables (code byte jb: the 16 entries of table 2jb + half) and bound
        const unsigned k = set * QW + (unsigned)row;
        const bool live = k < P;
        const unsigned pr = pairs[p0 + min(k, P - 1u)];
        const unsigned q = pr / (unsigned)nprobe;
        int thr = -1 - SHIFT;  // nothing passes
        if (live) {
            const unsigned t = taus[q];
            if (t != IVFS_NONE) thr = (int)t - SHIFT;
        }
        v8i_t tb[NP];
#pragma unroll
        for (int jp = 0; jp < NP; ++jp) {
            const v4i_t *src = reinterpret_cast<const v4i_t *>(qluts + ((size_t)pr * (2 * B) + 4 * jp + 2 * half) * 16);
            const v4i_t e0 = src[0], e1 = src[1];
            const int flip = live ? (int)0x80808080u : 0, keep = live ? -1 : 0;
            tb[jp] = v8i_t{(e0[0] ^ flip) & keep, (e0[1] ^ flip) & keep, (e0[2] ^ flip) & keep, (e0[3] ^ flip) & keep,
                           (e1[0] ^ flip) & keep, (e1[1] ^ flip) & keep, (e1[2] ^ flip) & keep, (e1[3] ^ flip) & keep};
        }

        // Writes the pairs' keys to their queries' regions and empties the lists.  Lane k < 32 reports
        // for pair k of the set, which is its own (half 0).
        auto flush = [&]() {
            __syncthreads();
            if (l < QW) {
                const unsigned c = min(cnt[l], (unsigned)LC);
                if (c) {
                    char *base = ws + (size_t)q * ws_stride;
                    unsigned *counts = reinterpret_cast<unsigned *>(base + countsA_off);
                    uint64_t *dst = reinterpret_cast<uint64_t *>(base + listsA_off);
                    const unsigned slot = atomicAdd(&counts[0], c);
                    if (slot + c <= (unsigned)pitchA) {
                        for (unsigned i = 0; i < c; ++i) {
                            const unsigned key = keys[l][i];
                            dst[slot + i] = ((uint64_t)(key >> 24) << 32) | (uint64_t)(c0 + (key & 0xffffffu));
                        }
                    } else {
                        flags[q] = 1u;  // the region is full: this query is redone on its own
                    }
                    cnt[l] = 0;
                }
            }
            __syncthreads();
        };

        unsigned cw[SUB][WPC], cn[SUB][WPC];
        auto fetch = [&](int64_t t0, unsigned (&dst)[SUB][WPC]) {
#pragma unroll
            for (int s = 0; s < SUB; ++s) {
                const int64_t i = min(t0 + 32 * s + row, c1 - 1);
                const unsigned *src = reinterpret_cast<const unsigned *>(codes + i * B);
#pragma unroll
                for (int w = 0; w < WPC; ++w) dst[s][w] = src[w];
            }
        };
        struct Operand {
            v2i_t v0, v1;
            int p0, p1;
        };
        auto operand = [&](const unsigned (&w)[WPC], int jp) {
            const unsigned x = onehot_nibble_offsets(w[jp >> 1], half);
            const unsigned o0 = __builtin_amdgcn_ubfe(x, 16 * (jp & 1), 8), o1 = __builtin_amdgcn_ubfe(x, 16 * (jp & 1) + 8, 8);
            const char *tv = reinterpret_cast<const char *>(nibval), *tp = reinterpret_cast<const char *>(nibpos);
            return Operand{*reinterpret_cast<const v2i_t *>(tv + o0), *reinterpret_cast<const v2i_t *>(tv + o1),
                           *reinterpret_cast<const int *>(tp + o0), *reinterpret_cast<const int *>(tp + o1)};
        };
        // Result v of a lane: code (v / 4) * 8 + half * 4 + v % 4 of the step, pair `row`.
        auto test = [&](const v16i_t &sum, unsigned rel) {
            int lo = sum[0];
#pragma unroll
            for (int v = 1; v < 15; v += 2) lo = min(min(lo, sum[v]), sum[v + 1]);
            lo = min(lo, sum[15]);
            if (__ballot(lo <= thr) == 0ull) return;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int qm = min(min(sum[4 * u], sum[4 * u + 1]), min(sum[4 * u + 2], sum[4 * u + 3]));
                if (__ballot(qm <= thr) == 0ull) continue;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const unsigned li = rel + (unsigned)(u * 8 + half * 4 + w);
                    if (c0 + (int64_t)li < c1 && sum[4 * u + w] <= thr) {
                        const unsigned slot = atomicAdd(&cnt[row], 1u);
                        if (slot < (unsigned)LC) keys[row][slot] = ((unsigned)(sum[4 * u + w] + SHIFT) << 24) | li;
                    }
                }
            }
            // a step adds at most 32 keys to a pair's list: written out once a list is half full, it never
            // runs over
            __syncthreads();
            const bool full = l < QW && cnt[l] > (unsigned)(LC - 32);
            if (__ballot(full) != 0ull) flush();
        };

        fetch(c0, cn);
        Operand a0 = operand(cn[0], 0), a1 = operand(cn[0], NP > 1 ? 1 : 0);
        for (int64_t t0 = c0; t0 < c1; t0 += 32 * SUB) {  // uniform
#pragma unroll
            for (int s = 0; s < SUB; ++s)
#pragma unroll
                for (int w = 0; w < WPC; ++w) cw[s][w] = cn[s][w];
            if (t0 + 32 * SUB < c1) fetch(t0 + 32 * SUB, cn);
#pragma unroll
            for (int s = 0; s < SUB; ++s) {
                if (t0 + 32 * s >= c1) break;  // uniform
                v16i_t acc = mfma_zero_acc();
#pragma unroll
                for (int jp = 0; jp < NP; ++jp) {
                    const Operand a = a0;
                    a0 = a1;
                    if (jp + 2 < NP) a1 = operand(cw[s], jp + 2);
                    else if (s + 1 < SUB) a1 = operand(cw[s + 1], (jp + 2 - NP) % NP);
                    else a1 = operand(cn[0], (jp + 2 - NP) % NP);
                    asm volatile("" ::: "memory");
                    const v4i_t av = v4i_t{a.v0[0], a.v0[1], a.v1[0], a.v1[1]};
                    int ap0 = a.p0, ap1 = a.p1;
                    asm volatile("" : "+v"(ap0), "+v"(ap1));
                    const int ap = ap0 | (ap1 << 16);
                    acc = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, tb[jp], acc, ap, 0, 0);
                }
                test(acc, (unsigned)(t0 - c0) + 32u * s);
            }
        }
        flush();
    }
}

// One workgroup per query, between the two parts of the scan: the R-th smallest sum among the
// keys reported so far replaces the query's bound when it is tighter, and only the keys within the
// new bound stay in the region (the others cannot be among the R best).
constexpr int IVFS_REFINE_NT = 256;
__global__ __launch_bounds__(IVFS_REFINE_NT) void ivfs_refine_kernel(char *__restrict__ ws, size_t ws_stride,
                                                                     size_t countsA_off, size_t listsA_off,
                                                                     int pitchA, int R, unsigned *__restrict__ taus,
                                                                     const unsigned *__restrict__ flags)
{
    constexpr int NT = IVFS_REFINE_NT;
    __shared__ uint64_t lkeys[MERGE_CAP];
    __shared__ unsigned hist[256];
    __shared__ unsigned tnew, kept;
    const int q = blockIdx.x, tid = threadIdx.x;
    if (flags[q] == 1u || pitchA > MERGE_CAP) return;  // uniform
    char *base = ws + (size_t)q * ws_stride;
    unsigned *counts = reinterpret_cast<unsigned *>(base + countsA_off);
    const unsigned c = counts[0];
    if (c < (unsigned)R || c > (unsigned)pitchA) return;  // uniform
    uint64_t *keys = reinterpret_cast<uint64_t *>(base + listsA_off);
    for (int i = tid; i < 256; i += NT) hist[i] = 0;
    if (tid == 0) { tnew = 256u; kept = 0; }
    __syncthreads();
    for (unsigned i = tid; i < c; i += NT) {
        const uint64_t k = keys[i];
        lkeys[i] = k;
        atomicAdd(&hist[(unsigned)(k >> 32) & 255u], 1u);
    }
    __syncthreads();
    if (tid < WAVE) {
        unsigned h[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) h[b] = hist[4 * tid + b];
        const unsigned t = wave_threshold_bin<4>(h, (unsigned)R);
        if (tid == 0) tnew = t;
    }
    __syncthreads();
    const unsigned t = tnew;
    if (t >= 256u || t >= taus[q]) return;  // uniform: no tighter bound
    for (unsigned i = tid; i < c; i += NT) {
        const uint64_t k = lkeys[i];
        if (((unsigned)(k >> 32) & 255u) <= t) keys[atomicAdd(&kept, 1u)] = k;
    }
    __syncthreads();
    if (tid == 0) {
        taus[q] = t;
        counts[0] = kept;
    }
}

// One wavefront per query, after the shared lists are scanned: the cells that are left to the
// per-query kernel (-1 in the slots of the shared cells), their units of work as ivf_qmax_kernel
// counts them, and the query's tightened bound back into its control block for that kernel.
__global__ __launch_bounds__(256) void ivfs_light_kernel(const int32_t *__restrict__ probes, int nprobe, int nb, int K,
                                                         const unsigned *__restrict__ pair_off, int min_pairs,
                                                         const int64_t *__restrict__ list_off, int64_t n_total,
                                                         long long unit, const unsigned *__restrict__ flags,
                                                         const unsigned *__restrict__ taus, char *__restrict__ ws,
                                                         size_t ws_stride, int32_t *__restrict__ probes_light,
                                                         unsigned *__restrict__ qunits_light)
{
    const int q = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nb) return;  // whole wavefront
    const int lane = threadIdx.x & 63;
    unsigned units = 0;
    for (int p = lane; p < nprobe; p += 64) {
        int cell = probes[(size_t)q * nprobe + p];
        if (cell >= 0 && cell < K && pair_off[cell + 1] - pair_off[cell] >= (unsigned)min_pairs) cell = -1;
        probes_light[(size_t)q * nprobe + p] = cell;
        if (cell >= 0 && cell < K) {
            const long long l = list_off[cell], h = list_off[cell + 1];
            if (l >= 0 && h <= n_total && h > l) units += (unsigned)((h - l / 16 * 16 + unit - 1) / unit);
        }
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) units += __shfl_xor(units, s);
    if (lane == 0) {
        qunits_light[q] = units;
        if (flags[q] == 2u && taus[q] != IVFS_NONE)
            reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride)->ghist[0][0] = taus[q] + 1u;
    }
}

// The shared part of the scan of one batch (after the seed kernel): pairs by cell, the two parts
// with the bounds refined in between, then what is left for the per-query kernel.  Every array is
// device memory of the sizes named in IvfPlan.
int ivf_shared_scan(int B, const int64_t *list_off, const uint8_t *codes, int64_t n_total, int K,
                    const int32_t *probes, int nb, int nprobe, const uint8_t *qluts, int R, char *scan_ws,
                    size_t ws_stride, size_t countsA_off, size_t listsA_off, int pitchA, unsigned *pair_cnt,
                    unsigned *pair_off, unsigned *item_off0, unsigned *item_off1, unsigned *pairs, unsigned *taus,
                    unsigned *flags, int32_t *probes_light, unsigned *qunits_light, long long unit, int min_pairs,
                    int wgs, hipStream_t st)
{
    const int64_t npairs = (int64_t)nb * nprobe;
    const unsigned pgrid = (unsigned)ceil_div(npairs, 256);
    launch(QADC_PROF_SEED, ivfs_zero_kernel, dim3((unsigned)ceil_div(K, 256)), dim3(256), 0, st, pair_cnt, (int64_t)K);
    launch(QADC_PROF_SEED, ivfs_count_kernel, dim3(pgrid), dim3(256), 0, st, probes, nprobe, npairs, K,
           (const char *)scan_ws, ws_stride, pair_cnt, taus, flags);
    const unsigned ogrid = (unsigned)ceil_div(K, IVFS_OFF_NT);
    unsigned *blk = pair_cnt + (size_t)K + 1;  // (the region of pair_cnt has room for 3 x 256 totals behind it)
    launch(QADC_PROF_SEED, ivfs_offsets_kernel, dim3(ogrid), dim3(IVFS_OFF_NT), 0, st, (const unsigned *)pair_cnt,
           list_off, K, n_total, 32, min_pairs, pair_off, item_off0, item_off1, blk);
    launch(QADC_PROF_SEED, ivfs_offsets_add_kernel, dim3(ogrid), dim3(IVFS_OFF_NT), 0, st, K, (const unsigned *)blk,
           pair_off, item_off0, item_off1);
    launch(QADC_PROF_SEED, ivfs_place_kernel, dim3(pgrid), dim3(256), 0, st, probes, npairs, K,
           (const unsigned *)pair_off, pair_cnt, pairs);
#define QADC_IVFS_CASE(B_)                                                                                      \
    case B_:                                                                                                   \
        launch(QADC_PROF_IVF_SHARED, ivfs_scan_kernel<B_>, dim3((unsigned)wgs), dim3(64), 0, st, 0, list_off, codes,  \
               n_total, K, (const unsigned *)pair_off, (const unsigned *)item_off0, (const unsigned *)pairs,   \
               nprobe, qluts, (const unsigned *)taus, scan_ws, ws_stride, countsA_off, listsA_off, pitchA,     \
               flags);                                                                                         \
        launch(QADC_PROF_SEED, ivfs_refine_kernel, dim3((unsigned)nb), dim3(IVFS_REFINE_NT), 0, st, scan_ws,    \
               ws_stride, countsA_off, listsA_off, pitchA, R, taus, (const unsigned *)flags);                  \
        launch(QADC_PROF_IVF_SHARED, ivfs_scan_kernel<B_>, dim3((unsigned)wgs), dim3(64), 0, st, 1, list_off, codes,  \
               n_total, K, (const unsigned *)pair_off, (const unsigned *)item_off1, (const unsigned *)pairs,   \
               nprobe, qluts, (const unsigned *)taus, scan_ws, ws_stride, countsA_off, listsA_off, pitchA,     \
               flags);                                                                                         \
        break;
    switch (B) {
        QADC_IVFS_CASE(4)
        QADC_IVFS_CASE(8)
        QADC_IVFS_CASE(16)
        QADC_IVFS_CASE(32)
    default:
        return fail(QADC_EINVAL, "qadc_ivf_search: %d code bytes", B);
    }
#undef QADC_IVFS_CASE
    launch(QADC_PROF_SEED, ivfs_light_kernel, dim3((unsigned)ceil_div(nb, 4)), dim3(256), 0, st, probes, nprobe, nb, K,
           (const unsigned *)pair_off, min_pairs, list_off, n_total, unit, (const unsigned *)flags,
           (const unsigned *)taus, scan_ws, ws_stride, probes_light, qunits_light);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
