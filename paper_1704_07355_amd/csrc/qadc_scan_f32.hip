// Alg. 1 of the paper on gfx950: the float ADC scan, adc(y, c) = sum_j D^j[c[j]] (Eq. (2)),
// added in float32 in increasing j, for 4-bit codes (16-entry tables) and for the usual
// 8-bit codes (256-entry tables), with exact top-R under the order (distance, index).
//
// This is the reference the quantized scan is compared against (recall, speed).  The float
// tables of the query sit in LDS (1 KiB for 16x4, 8 KiB for 8x8: the sizes of the paper's
// Table 1); codes are streamed as in the quantized scan.  A candidate key is
// order(distance) << 32 | index among the workgroup's codes.  Large databases get a bound as
// the quantized scan does, on a monotone 8-bit image of the distance (range kernel + seed
// kernel), and a barrier-free pass; otherwise, or on overflow, each workgroup keeps an LDS
// list that is cut back to its R smallest keys by an exact radix select whenever it fills.
// A workgroup reports at most R keys; the merge kernel orders the R smallest of all of them.

#include <mutex>

#include <algorithm>

#include "qadc_scan_common.h"

namespace qadc {

constexpr int F32_NT = 512;
constexpr int F32_RANGE_CODES = 1024;  // codes looked at to place the bins of the bound

struct F32Shared {
    SelectScratch sel;
    unsigned ccnt;
    unsigned tcnt[3];
    unsigned tau;
    unsigned fcnt;
};

// Bins for the grid-wide bound: a monotone map of the float distance onto 0..255, uniform
// between `lo` (the smallest sum the tables allow) and the R-th smallest distance of the
// first codes -- the range Section 3.3 of the paper gives the quantized tables.  Monotone,
// so "bin <= tau" never drops a code that beats one it keeps; the exact order is decided on
// the float keys afterwards.
struct F32Range {
    float lo, scale;
};

__device__ __forceinline__ unsigned f32_bin(float d, F32Range r)
{
    const float t = fmaxf(0.0f, d - r.lo) * r.scale;
    return (unsigned)fminf(t, 255.0f);
}

// Float tables of one query -> LDS.
template <int KSUB, int ROW, int NT>
__device__ __forceinline__ void load_float_tables(const float *__restrict__ lq, float *lut)
{
    constexpr int M = (KSUB == 16) ? 2 * ROW : ROW;
    for (int e = threadIdx.x; e < M * KSUB; e += NT) lut[e] = lq[e];
}

// Eq. (2) for the codes of one thread's tile slot: float32 sums in increasing j.
template <int KSUB, int ROW, int NT>
__device__ __forceinline__ void tile_dists(const uint4 (&w)[2], const float *lut,
                                           float (&d)[ScanCfg<ROW, NT>::CPT])
{
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
                d[v * CPV + c] = acc;
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
        d[0] = acc;
    }
}

template <int ROW, int NT>
__device__ __forceinline__ bool slot_valid(const int (&nc)[2], int slot)
{
    if constexpr (ROW <= 16) return (slot % (16 / ROW)) < nc[slot / (16 / ROW)];
    else return nc[0] != 0;
}

template <int ROW, int NT>
__device__ __forceinline__ unsigned slot_index(int slot)
{
    if constexpr (ROW <= 16) {
        constexpr int CPV = 16 / ROW;
        return (unsigned)(((slot / CPV) * NT + threadIdx.x) * CPV + slot % CPV);
    } else {
        return threadIdx.x;
    }
}

// Range kernel: one workgroup per query; lo = sum_j min_i D^j[i] (float32, increasing j),
// hi = the min(R, n0)-th smallest distance of the first n0 codes; scale = 255 / (hi - lo).
template <int KSUB, int ROW>
__global__ __launch_bounds__(F32_NT) void f32_range_kernel(
    const uint8_t *__restrict__ codes, int n0, const float *__restrict__ luts, int R,
    F32Range *__restrict__ ranges)
{
    constexpr int NT = F32_NT;
    constexpr int M = (KSUB == 16) ? 2 * ROW : ROW;
    __shared__ float lut[M * KSUB];
    __shared__ unsigned cand[F32_RANGE_CODES];
    __shared__ float tmin[M];
    __shared__ SelectScratch sc;
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    load_float_tables<KSUB, ROW, NT>(luts + (size_t)q * M * KSUB, lut);
    __syncthreads();
    if (tid < M) {
        float b = lut[tid * KSUB];
        for (int i = 1; i < KSUB; ++i) b = fminf(b, lut[tid * KSUB + i]);
        tmin[tid] = b;
    }
    for (int i = tid; i < n0; i += NT) {
        const uint8_t *c = codes + (size_t)i * ROW;
        float acc = 0.0f;
        for (int jb = 0; jb < ROW; ++jb) {
            const unsigned b = c[jb];
            if constexpr (KSUB == 16) {
                acc = acc + lut[(2 * jb) * 16 + (b & 15u)];
                acc = acc + lut[(2 * jb + 1) * 16 + (b >> 4)];
            } else {
                acc = acc + lut[jb * 256 + b];
            }
        }
        cand[i] = f2ord(acc);
    }
    __syncthreads();
    const unsigned kth = block_radix_select<unsigned, 4>(cand, (unsigned)n0, (unsigned)min(R, n0), &sc);
    if (tid == 0) {
        float lo = 0.0f;
        for (int j = 0; j < M; ++j) lo = lo + tmin[j];
        const float hi = ord2f(kth);
        F32Range r;
        r.lo = lo;
        r.scale = (hi > lo) ? 255.0f / (hi - lo) : 0.0f;
        ranges[q] = r;
    }
}

// Seed kernel of the float scan: a sample of tiles is binned and the lowest bins of each
// workgroup are added to the query's grid-wide histogram, exactly as in the quantized scan.
template <int KSUB, int ROW>
__global__ __launch_bounds__(F32_NT) void seed_f32_kernel(
    const uint8_t *__restrict__ codes, int64_t n, const float *__restrict__ luts,
    const F32Range *__restrict__ ranges, int R, unsigned flush_need, int64_t seed_stride,
    char *__restrict__ ws, size_t ws_stride)
{
    constexpr int NT = F32_NT;
    using C = ScanCfg<ROW, NT>;
    constexpr int M = (KSUB == 16) ? 2 * ROW : ROW;
    __shared__ float lut[M * KSUB];
    __shared__ unsigned hist[256];
    const int tid = threadIdx.x;
    const int q = blockIdx.y;
    const int g = blockIdx.x;
    const int64_t c0 = (int64_t)g * seed_stride;
    const int64_t c1 = min(n, c0 + C::TILE);
    if (c0 >= c1) return;
    uint4 w[2];
    int nc[2];
    tile_load<ROW, NT>(codes, c0, c1, w, nc);
    load_float_tables<KSUB, ROW, NT>(luts + (size_t)q * M * KSUB, lut);
    for (int e = tid; e < 256; e += NT) hist[e] = 0;
    const F32Range r = ranges[q];
    __syncthreads();
    float d[C::CPT];
    tile_dists<KSUB, ROW, NT>(w, lut, d);
#pragma unroll
    for (int c = 0; c < C::CPT; ++c) {
        const unsigned bin = f32_bin(d[c], r);
        if (slot_valid<ROW, NT>(nc, c) && bin < 255u) atomicAdd(&hist[bin], 1u);
    }
    __syncthreads();
    if (tid < WAVE) {
        unsigned h[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) h[b] = hist[4 * tid + b];
        const unsigned f = min(wave_threshold_bin<4>(h, (unsigned)R), wave_threshold_bin<4>(h, flush_need));
        ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
        unsigned *ghist = hdr->ghist[g % GH_REP];
        for (unsigned b0 = 0; b0 <= f && b0 < 256u; b0 += WAVE) {  // uniform
            const unsigned bin = b0 + tid;
            const unsigned c = hist[bin];
            if (bin <= f && bin < 255u && c)
                __hip_atomic_fetch_add(&ghist[bin], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Scan kernel.  KSUB = 16: ROW = m/2 bytes per code, two components per byte; KSUB = 256:
// ROW = m bytes.  Workgroup g takes tiles g, g+G, ...  With a grid-wide bound the pass is
// barrier-free (keys whose bin is at or below the bound are appended to the LDS list); on
// overflow, or without a bound, the careful pass runs: one barrier per tile, the list cut
// back to its R smallest keys by an exact radix select whenever it fills.
template <int KSUB, int ROW>
__global__ __launch_bounds__(F32_NT) void scan_f32_kernel(
    const uint8_t *__restrict__ codes, int64_t n, const float *__restrict__ luts,
    const F32Range *__restrict__ ranges, int has_seed, int R, char *__restrict__ ws,
    size_t ws_stride, size_t counts_off, size_t lists_off, const unsigned *__restrict__ redo_flags)
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
    if (redo_flags && redo_flags[q] == 0) return;  // uniform: only the queries the tiled scan gave up on
    const ScanHeader *hdr = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride);

    if (tid < WAVE) {
        unsigned t = 256, carry = 0;
        for (unsigned b0 = 0; b0 < 256 && has_seed; b0 += 128) {  // uniform
            const unsigned bin = b0 + 2u * tid;
            unsigned h[2] = {0, 0};
#pragma unroll
            for (int r = 0; r < GH_REP; ++r) {
                const uint2 v = *reinterpret_cast<const uint2 *>(&hdr->ghist[r][bin]);
                h[0] += v.x;
                h[1] += v.y;
            }
            unsigned tot;
            const unsigned hit = wave_threshold_bin<2>(h, (unsigned)R - carry, &tot);
            if (hit < 128u) { t = b0 + hit; break; }
            carry += tot;
        }
        if (tid == 0) { sh.tau = t; sh.fcnt = 0; sh.tcnt[0] = 0; }
    }
    load_float_tables<KSUB, ROW, NT>(luts + (size_t)q * M * KSUB, lut);
    __syncthreads();

    const bool seeded = sh.tau < 255u;  // uniform (bin 255 is never counted)
    unsigned have = 0;
    bool careful = !seeded;
    if (seeded) {
        const unsigned tau = sh.tau;
        const F32Range r = ranges[q];
        unsigned rel = 0;
        for (int64_t t0 = (int64_t)g * C::TILE; t0 < n; t0 += G * C::TILE, rel += C::TILE) {
            uint4 w[2];
            int nc[2];
            tile_load<ROW, NT>(codes, t0, n, w, nc);
            float d[C::CPT];
            tile_dists<KSUB, ROW, NT>(w, lut, d);
            bool pass[C::CPT], any = false;
#pragma unroll
            for (int c = 0; c < C::CPT; ++c) {
                pass[c] = slot_valid<ROW, NT>(nc, c) && f32_bin(d[c], r) <= tau;
                any = any || pass[c];
            }
            if (__ballot(any) != 0ull) {  // the append code only runs in waves with a hit
#pragma unroll
                for (int c = 0; c < C::CPT; ++c) {
                    const unsigned slot = wave_append_slot(pass[c], &sh.fcnt);
                    if (pass[c] && slot < (unsigned)C::CAP)
                        keys[slot] = ((uint64_t)f2ord(d[c]) << 32) | (rel + slot_index<ROW, NT>(c));
                }
            }
        }
        __syncthreads();
        have = sh.fcnt;
        careful = have > (unsigned)C::CAP;  // keys were dropped: start over, carefully
    }

    if (careful) {
        uint64_t lim = ~0ull;  // keys >= lim cannot be among the R best of this workgroup's codes
        have = 0;
        int rot = 0;
        unsigned rel = 0;
        for (int64_t t0 = (int64_t)g * C::TILE; t0 < n; t0 += G * C::TILE, rel += C::TILE) {
            unsigned *ctr = &sh.tcnt[rot];
            const int nxt = (rot == 2) ? 0 : rot + 1;
            if (tid == 0) sh.tcnt[nxt] = 0;
            uint4 w[2];
            int nc[2];
            tile_load<ROW, NT>(codes, t0, n, w, nc);
            float d[C::CPT];
            tile_dists<KSUB, ROW, NT>(w, lut, d);
#pragma unroll
            for (int c = 0; c < C::CPT; ++c) {
                const uint64_t key = slot_valid<ROW, NT>(nc, c)
                                         ? (((uint64_t)f2ord(d[c]) << 32) | (rel + slot_index<ROW, NT>(c)))
                                         : ~0ull;
                const bool pass = key < lim;
                const unsigned slot = have + wave_append_slot(pass, ctr);
                if (pass) keys[slot] = key;
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

// ------------------------------------------------------------------ query batches
//
// Query-tiled form of the float scan for 8-bit codes (KSUB = 256): a workgroup scans a chunk of
// the database for eight queries at once.  The eight queries' tables are interleaved in LDS:
// entry (j, v) is 32 bytes = eight float32 entries D_q^j[v], so one code byte costs two 16-byte
// LDS reads and eight adds, and a code fetched from memory serves eight queries.  Each sum is
// float32 in increasing j, exactly as in scan_f32_kernel.  Bounds: each query's bin bound from
// its sampled histogram (read by one wavefront per query at the start); sums whose bin is at or
// below it go to small per-query LDS lists; a list that overflows marks its query for
// scan_f32_kernel, which redoes that query alone, and the merge kernel takes whichever report
// is valid.  Workgroup ids map to (query group, chunk) so that the groups of a chunk follow
// each other in each XCD's share of the ids.
constexpr int F32T_Q = 8;
constexpr int F32T_LCAP = 64;
constexpr int F32T_MAX_CHUNKS = 1024;
constexpr int F32T_MIN_Q = 8;

template <int KSUB, int ROW>
__global__ __launch_bounds__(F32_NT) void scan_f32_tiled_kernel(
    const uint8_t *__restrict__ codes, int64_t n, int64_t chunk, int nq, const float *__restrict__ luts,
    const F32Range *__restrict__ ranges, int R, char *__restrict__ ws, size_t ws_stride, size_t countsA_off,
    size_t listsA_off, unsigned *__restrict__ flags)
{
    constexpr int NT = F32_NT;
    static_assert(NT / WAVE == F32T_Q, "one wavefront per query reads its bound");
    using C = ScanCfg<ROW, NT>;
    // table entry (component, value) = eight floats, one per query of the group: [ROW * 256][2]
    // float4 for 8-bit components, [2 * ROW * 16][2] for 4-bit ones
    constexpr int ENTRIES = KSUB == 256 ? ROW * 256 : 2 * ROW * 16;
    extern __shared__ float4 ftab[];
    __shared__ uint64_t keys[F32T_Q][F32T_LCAP];
    __shared__ unsigned cnt[F32T_Q];
    __shared__ unsigned tau_s[F32T_Q];

    const int tid = threadIdx.x;
    const int ngroups = (nq + F32T_Q - 1) / F32T_Q;
    const unsigned id = blockIdx.x, slot_id = id >> 3;
    const int grp = (int)(slot_id % (unsigned)ngroups);
    const int gc = (int)((slot_id / (unsigned)ngroups) * 8u + (id & 7u));
    const int q0 = grp * F32T_Q;
    const int64_t c0 = (int64_t)gc * chunk;
    const int64_t c1 = min(n, c0 + chunk);
    if (c0 >= c1) return;  // uniform

    uint4 w[2];
    int nc[2];
    tile_load<ROW, NT>(codes, c0, c1, w, nc);

    {   // wavefront k: the bound of query q0 + k from its histogram (255: nothing is known)
        const int k = tid / WAVE, l = tid % WAVE;
        unsigned t = 256;
        if (q0 + k < nq) {  // whole wavefronts
            const ScanHeader *hdr = reinterpret_cast<const ScanHeader *>(ws + (size_t)(q0 + k) * ws_stride);
            unsigned carry = 0;
            for (unsigned b0 = 0; b0 < 256; b0 += 128) {  // uniform
                const unsigned bin = b0 + 2u * l;
                unsigned h[2] = {0, 0};
#pragma unroll
                for (int r = 0; r < GH_REP; ++r) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(&hdr->ghist[r][bin]);
                    h[0] += v.x;
                    h[1] += v.y;
                }
                unsigned tot;
                const unsigned hit = wave_threshold_bin<2>(h, (unsigned)R - carry, &tot);
                if (hit < 128u) { t = b0 + hit; break; }
                carry += tot;
            }
        }
        if (l == 0) { tau_s[k] = t; cnt[k] = 0; }
    }
    for (int e = tid; e < ENTRIES; e += NT) {
        float v[F32T_Q];
#pragma unroll
        for (int k = 0; k < F32T_Q; ++k) {
            const int q = q0 + k;
            v[k] = (q < nq) ? luts[(size_t)q * ENTRIES + e] : __builtin_inff();
        }
        ftab[2 * e] = make_float4(v[0], v[1], v[2], v[3]);
        ftab[2 * e + 1] = make_float4(v[4], v[5], v[6], v[7]);
    }
    __syncthreads();
    // a query without a usable bound (bin 255 is never counted) lets everything through: its list
    // overflows and it is redone alone
    unsigned tau[F32T_Q];
    F32Range rg[F32T_Q];
#pragma unroll
    for (int k = 0; k < F32T_Q; ++k) {
        tau[k] = tau_s[k];
        rg[k] = (q0 + k < nq) ? ranges[q0 + k] : F32Range{0.0f, 0.0f};
    }

    unsigned rel = 0;
    for (int64_t t0 = c0; t0 < c1; t0 += C::TILE, rel += C::TILE) {
        if (rel) tile_load<ROW, NT>(codes, t0, c1, w, nc);
        constexpr int CPV = 16 / ROW;
#pragma unroll
        for (int v = 0; v < 2; ++v) {
#pragma unroll
            for (int c = 0; c < CPV; ++c) {
                float acc[F32T_Q];
#pragma unroll
                for (int k = 0; k < F32T_Q; ++k) acc[k] = 0.0f;
                auto add = [&](unsigned e) {  // float32 additions in increasing component order
                    const float4 lo4 = ftab[2 * e], hi4 = ftab[2 * e + 1];
                    acc[0] = acc[0] + lo4.x; acc[1] = acc[1] + lo4.y; acc[2] = acc[2] + lo4.z; acc[3] = acc[3] + lo4.w;
                    acc[4] = acc[4] + hi4.x; acc[5] = acc[5] + hi4.y; acc[6] = acc[6] + hi4.z; acc[7] = acc[7] + hi4.w;
                };
#pragma unroll
                for (int jb = 0; jb < ROW; ++jb) {
                    const unsigned b = byte_of(w[v], c * ROW + jb);
                    if constexpr (KSUB == 256) {
                        add((unsigned)jb * 256u + b);
                    } else {  // two 4-bit components per byte: the low nibble is the even one
                        add((unsigned)(2 * jb) * 16u + (b & 15u));
                        add((unsigned)(2 * jb + 1) * 16u + (b >> 4));
                    }
                }
                const bool valid = c < nc[v];
                const unsigned li = rel + (unsigned)((v * NT + tid) * CPV + c);
                bool pass[F32T_Q], any = false;
#pragma unroll
                for (int k = 0; k < F32T_Q; ++k) {
                    pass[k] = valid && (q0 + k < nq) && (tau[k] >= 255u || f32_bin(acc[k], rg[k]) <= tau[k]);
                    any = any || pass[k];
                }
                if (__ballot(any) != 0ull) {  // the append code only runs in waves with a hit
#pragma unroll
                    for (int k = 0; k < F32T_Q; ++k) {
                        const unsigned slot = wave_append_slot(pass[k], &cnt[k]);
                        if (pass[k] && slot < (unsigned)F32T_LCAP)
                            keys[k][slot] = ((uint64_t)f2ord(acc[k]) << 32) | li;
                    }
                }
            }
        }
    }
    __syncthreads();

#pragma unroll 1
    for (int k = 0; k < F32T_Q; ++k) {
        const int q = q0 + k;
        if (q >= nq) break;
        const unsigned c = cnt[k];
        if (c == 0) continue;
        if (c > (unsigned)F32T_LCAP) {  // keys were dropped: this query is redone on its own
            if (tid == 0) flags[q] = 1u;
            continue;
        }
        char *base = ws + (size_t)q * ws_stride;
        unsigned *counts = reinterpret_cast<unsigned *>(base + countsA_off);
        uint64_t *dst = reinterpret_cast<uint64_t *>(base + listsA_off) + (size_t)gc * F32T_LCAP;
        if (tid == 0) counts[gc] = c;
        for (unsigned i = tid; i < c; i += NT) {
            const uint64_t key = keys[k][i];
            dst[i] = (key & 0xffffffff00000000ull) | (uint64_t)(c0 + (int64_t)(key & 0xffffffffull));
        }
    }
}

struct F32Plan {
    int ROW, KSUB, G, qbatch;
    int seed_wgs;
    int64_t seed_stride;
    unsigned flush_need;
    ScanLayout l;
    size_t stride;        // bytes of workspace per query
    bool tiled;           // batches go through the query-tiled kernel
    int GC;               // database chunks of the tiled kernel
    int64_t chunk;
    size_t countsA_off, listsA_off, flags_off, tiled_lds;
    size_t ranges_off, ws_bytes;
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
    int64_t G = knob_or(knobs().scan_f32_wgs, 1024);
    if (G < 1) G = 1;
    if (G > tiles) G = tiles;
    const int64_t max_tiles_per_wg = 0xffffffffll / tile;
    if (ceil_div(tiles, G) > max_tiles_per_wg) G = ceil_div(tiles, max_tiles_per_wg);
    p->G = (int)G;
    // sample for the grid-wide bound, as in the quantized scan
    p->seed_wgs = 0;
    p->seed_stride = 0;
    p->flush_need = 16;
    if (tiles >= knob_or(knobs().seed_min_tiles, 64) * 2) {
        int64_t S = tiles / 40;
        if (S < 256) S = 256;
        if (S > 1024) S = 1024;
        if (S > tiles / 4) S = tiles / 4;
        p->seed_wgs = (int)S;
        p->seed_stride = (n / S) / 16 * 16;
        int64_t fl = ceil_div(4ll * R, S);
        if (fl < 16) fl = 16;
        if (fl > R) fl = R;
        p->flush_need = (unsigned)fl;
    }
    // batches: query-tiled kernel over chunks (8-bit codes: a table entry per byte; 4-bit codes: two
    // per byte), the single-query kernel only redoes queries whose lists overflowed
    p->tiled = false;
    p->GC = 0;
    p->chunk = 0;
    p->tiled_lds = (size_t)(p->KSUB == 256 ? p->ROW * 256 : 2 * p->ROW * 16) * 2 * sizeof(float4);
    if (p->ROW <= 16 && p->seed_wgs > 0 && nq >= F32T_MIN_Q && knob_or(knobs().tiled, 1) != 0) {
        const int64_t groups = ceil_div(nq, F32T_Q);
        const int64_t want = std::max<int64_t>(1, std::min<int64_t>(F32T_MAX_CHUNKS, ceil_div(1024, groups)));
        int64_t chunk = ceil_div(ceil_div(n, F32T_MAX_CHUNKS), tile) * tile;
        int64_t by_fill = ceil_div(ceil_div(n, want), tile) * tile;
        if (by_fill > 64ll * tile) by_fill = 64ll * tile;
        if (by_fill < 8ll * tile) by_fill = 8ll * tile;
        if (chunk < by_fill) chunk = by_fill;
        if (chunk <= 0xffffffffll) {
            p->tiled = true;
            p->chunk = chunk;
            p->GC = (int)ceil_div(n, chunk);
            if (p->G > 256) p->G = 256;
        }
    }
    p->l = scan_layout(p->G, R);
    p->stride = p->l.stride;
    p->countsA_off = p->listsA_off = p->flags_off = 0;
    if (p->tiled) {
        p->countsA_off = p->stride;
        p->listsA_off = p->countsA_off + align_up((size_t)p->GC * sizeof(unsigned), 256);
        p->stride = p->listsA_off + align_up((size_t)p->GC * F32T_LCAP * sizeof(uint64_t), 256);
    }
    p->qbatch = scan_query_batch(p->stride, nq);
    p->ranges_off = p->stride * (size_t)p->qbatch;
    p->ws_bytes = p->ranges_off + align_up((size_t)p->qbatch * sizeof(F32Range), 256);
    if (p->tiled) {
        p->flags_off = p->ws_bytes;
        p->ws_bytes = p->flags_off + align_up((size_t)p->qbatch * sizeof(unsigned), 256);
    }
    return true;
}

template <int KSUB, int ROW>
static int launch_f32_tiled(const F32Plan &p, const uint8_t *codes, int64_t n, const float *luts, int nq, int R,
                            const F32Range *ranges, char *ws, unsigned *flags, hipStream_t st)
{
    if constexpr (ROW <= 16) {
        static std::once_flag attr_once;  // the kernel may use more dynamic LDS than the default limit
        hipError_t attr_rc = hipSuccess;
        std::call_once(attr_once, [&] {
            attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_f32_tiled_kernel<KSUB, ROW>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.tiled_lds);  // fixed by KSUB, ROW
        });
        QADC_HIP_TRY(attr_rc);
        const unsigned gc8 = (unsigned)ceil_div(p.GC, 8) * 8u;  // chunk slots, eight at a time
        dim3 grid((unsigned)ceil_div(nq, F32T_Q) * gc8);
        launch(QADC_PROF_SCAN, (scan_f32_tiled_kernel<KSUB, ROW>), grid, dim3(F32_NT), p.tiled_lds, st, codes, n, p.chunk,
               nq, luts, ranges, R, ws, p.stride, p.countsA_off, p.listsA_off, flags);
    }
    return QADC_OK;
}

// Seed (large databases), query-tiled scan (batches), single-query scan: of
// everything, or of the queries the tiled scan flagged.  `flags`: null without a tiled scan.
template <int KSUB>
static int dispatch_f32(const F32Plan &p, const uint8_t *codes, int64_t n, const float *luts, int nq,
                        int R, char *ws, unsigned *flags, hipStream_t st)
{
    dim3 grid(p.G, nq), block(F32_NT);
    F32Range *ranges = reinterpret_cast<F32Range *>(ws + p.ranges_off);
    const int n0 = (int)min((int64_t)F32_RANGE_CODES, n);
#define QADC_F32_CASE(ROW_)                                                                          \
    case ROW_:                                                                                       \
        if (p.seed_wgs > 0) {                                                                        \
            launch(QADC_PROF_SEED, (f32_range_kernel<KSUB, ROW_>), dim3(nq), block, 0, st, codes, n0, luts, R, \
                   ranges);                                                                          \
            launch(QADC_PROF_SEED, (seed_f32_kernel<KSUB, ROW_>), dim3(p.seed_wgs, nq), block, 0, st, codes, n, \
                   luts, (const F32Range *)ranges, R, p.flush_need, p.seed_stride, ws, p.stride);     \
        }                                                                                            \
        if (flags) {                                                                                 \
            const int rc = launch_f32_tiled<KSUB, ROW_>(p, codes, n, luts, nq, R, ranges, ws, flags, st);  \
            if (rc != QADC_OK) return rc;                                                            \
        }                                                                                            \
        launch(QADC_PROF_SCAN, (scan_f32_kernel<KSUB, ROW_>), grid, block, 0, st, codes, n, luts,     \
               (const F32Range *)ranges, p.seed_wgs > 0 ? 1 : 0, R, ws, p.stride, p.l.counts_off,     \
               p.l.lists_off, (const unsigned *)flags);                                              \
        break;
    switch (p.ROW) {
        QADC_F32_CASE(4)
        QADC_F32_CASE(8)
        QADC_F32_CASE(16)
        QADC_F32_CASE(32)
    }
#undef QADC_F32_CASE
    return QADC_OK;
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
        unsigned *flags = (p.tiled && nb >= F32T_MIN_Q) ? reinterpret_cast<unsigned *>(ws + p.flags_off) : nullptr;
        int rc = (p.KSUB == 16) ? dispatch_f32<16>(p, codes, n, lq, nb, R, ws, flags, st)
                                : dispatch_f32<256>(p, codes, n, lq, nb, R, ws, flags, st);
        if (rc != QADC_OK) return rc;
        rc = launch_merge<float, 8>(nb, st, ws, p.stride, p.l.counts_off, p.l.lists_off, p.G,
                                    (unsigned)min((int64_t)R, n), R, __builtin_inff(),
                                    out_idx + (size_t)q0 * R, out_dist + (size_t)q0 * R, p.countsA_off,
                                    p.listsA_off, flags ? p.GC : 0, (int)F32T_LCAP, flags, (const uint32_t *)nullptr,
                                    (int64_t)0);
        if (rc != QADC_OK) return rc;
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
