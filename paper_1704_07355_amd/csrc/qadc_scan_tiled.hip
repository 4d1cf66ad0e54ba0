// Query-tiled form of the Quick ADC scan (Alg. 2 of the paper) for batches of queries on
// gfx950: a workgroup scans a chunk of the database for a group of TQ = 8 queries at once,
// so that a code fetched from memory serves eight lookups-and-sums; the workgroups of the
// other query groups of the batch walk the same chunk at the same time and meet in L2.
//
// The eight queries' pair tables are interleaved in LDS: entry (jb, v) is 16 bytes = eight
// 16-bit pair sums min(cap, q[2jb][v & 15] + q[2jb+1][v >> 4]), one per query.  One code byte
// = one 16-byte LDS read + four 32-bit adds (the 16-bit lanes cannot carry into each other:
// 32 bytes x 255 < 65536), i.e. 8 lookup-adds per LDS access.  The clamp at `cap` is applied
// when a sum is kept.
//
// Selection: each query's grid-wide bound (from the seed kernel's histogram) is known
// before the scan starts; sums at or below it are appended to small per-query LDS lists.  A
// list that overflows marks its query for the single-query kernel, which redoes that query
// alone with its exact machinery; the merge kernel takes whichever result is valid.

#include "qadc_scan_common.h"
#include "qadc_scan_tiled.h"

namespace qadc {

// Two 16-bit lanes per register: saturating a - b, and min.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_sub_sat_u16(unsigned a, unsigned b)
{
    const u16x2 r = __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    return __builtin_bit_cast(unsigned, r);
}
__device__ __forceinline__ unsigned pk_min_u16(unsigned a, unsigned b)
{
    const u16x2 r = __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    return __builtin_bit_cast(unsigned, r);
}

// tau[q] = bin where the running count of query q's histogram reaches R, or 256.
__global__ __launch_bounds__(256) void scan_tau_kernel(const char *__restrict__ ws, size_t ws_stride,
                                                       int nq, int R, unsigned *__restrict__ taus)
{
    const int q = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;  // whole wave
    const int l = lane_id();
    const ScanHeader *hdr = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride);
    unsigned t = 256, carry = 0;
    for (unsigned b0 = 0; b0 < 256; b0 += 128) {
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
    if (l == 0) taus[q] = t;
}

template <int B>
__global__ __launch_bounds__(tiled_nt(B)) void scan_u8_tiled_kernel(
    const uint8_t *__restrict__ codes, int64_t n, int64_t chunk, int nq, int cap_i,
    const unsigned *__restrict__ taus, const char *__restrict__ ws, size_t ws_stride,
    size_t countsA_off, size_t listsA_off, unsigned *__restrict__ flags)
{
    constexpr int NT = tiled_nt(B);
    using C = ScanCfg<B, NT>;
    extern __shared__ uint4 tab[];  // [B * 256] entries of eight 16-bit pair sums
    __shared__ unsigned keys[TILED_Q][TILED_LCAP];
    __shared__ unsigned cnt[TILED_Q];

    const int tid = threadIdx.x;
    const int q0 = blockIdx.x * TILED_Q;
    const int gc = blockIdx.y;
    const unsigned cap = (unsigned)cap_i;
    const int64_t c0 = (int64_t)gc * chunk;
    const int64_t c1 = min(n, c0 + chunk);
    if (c0 >= c1) return;

    uint4 w[2];
    int nc[2];
    tile_load<B, NT>(codes, c0, c1, w, nc);

    // interleave the eight queries' pair tables
    for (int e = tid; e < B * 256; e += NT) {
        unsigned v[TILED_Q];
#pragma unroll
        for (int k = 0; k < TILED_Q; ++k) {
            const int q = q0 + k;
            v[k] = 1;  // no query in this slot: sums stay above its bound of "nothing passes"
            if (q < nq) v[k] = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride)->ptab[e];
        }
        tab[e] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
    }
    if (tid < TILED_Q) cnt[tid] = 0;
    // a sum passes when it is <= thr (signed compare; -1: no query in this slot)
    int thr[TILED_Q];
#pragma unroll
    for (int k = 0; k < TILED_Q; ++k) {
        const int q = q0 + k;
        thr[k] = -1;
        if (q < nq) {
            const unsigned t = taus[q];
            thr[k] = (t >= cap) ? 0xffff : (int)t;
        }
    }
    // thr + 1 of two queries per register (saturating at 0xffff, which no sum reaches; 0 where
    // there is no query): lane k of (acc -sat- thr1) is zero exactly when query k's sum passes.
    unsigned thr1[TILED_Q / 2];
#pragma unroll
    for (int i = 0; i < TILED_Q / 2; ++i)
        thr1[i] = (unsigned)min(thr[2 * i] + 1, 0xffff) | ((unsigned)min(thr[2 * i + 1] + 1, 0xffff) << 16);
    __syncthreads();

    unsigned rel = 0;
    for (int64_t t0 = c0; t0 < c1; t0 += C::TILE, rel += C::TILE) {
        if (rel) tile_load<B, NT>(codes, t0, c1, w, nc);
        constexpr int CPV = (B <= 16) ? 16 / B : 1;
        constexpr int NV = (B <= 16) ? 2 : 1;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
#pragma unroll
            for (int c = 0; c < CPV; ++c) {
                unsigned a0 = 0, a1 = 0, a2 = 0, a3 = 0;
                if constexpr (B <= 16) {
#pragma unroll
                    for (int jb = 0; jb < B; ++jb) {
                        const uint4 e = tab[jb * 256 + byte_of(w[v], c * B + jb)];
                        a0 += e.x; a1 += e.y; a2 += e.z; a3 += e.w;
                    }
                } else {
#pragma unroll
                    for (int jb = 0; jb < 32; ++jb) {
                        const uint4 e = tab[jb * 256 + byte_of(w[jb >> 4], jb & 15)];
                        a0 += e.x; a1 += e.y; a2 += e.z; a3 += e.w;
                    }
                }
                const bool valid = (B <= 16) ? (c < nc[v]) : (nc[0] != 0);
                const unsigned li = rel + (unsigned)((B <= 16) ? (v * NT + tid) * CPV + c : tid);
                // does any of the eight sums pass?  (rare: the append code is skipped otherwise)
                const unsigned z = pk_min_u16(pk_min_u16(pk_sub_sat_u16(a0, thr1[0]), pk_sub_sat_u16(a1, thr1[1])),
                                              pk_min_u16(pk_sub_sat_u16(a2, thr1[2]), pk_sub_sat_u16(a3, thr1[3])));
                const bool any = valid && min(z & 0xffffu, z >> 16) == 0u;
                if (__ballot(any) != 0ull) {
                    const unsigned acc[4] = {a0, a1, a2, a3};
#pragma unroll
                    for (int k = 0; k < TILED_Q; ++k) {
                        const unsigned s = (k & 1) ? (acc[k >> 1] >> 16) : (acc[k >> 1] & 0xffffu);
                        const bool pass = valid && (int)s <= thr[k];
                        const unsigned slot = wave_append_slot(pass, &cnt[k]);
                        if (pass && slot < (unsigned)TILED_LCAP) keys[k][slot] = (min(s, cap) << 24) | li;
                    }
                }
            }
        }
    }
    __syncthreads();

#pragma unroll 1
    for (int k = 0; k < TILED_Q; ++k) {
        const int q = q0 + k;
        if (q >= nq) break;
        const unsigned c = cnt[k];
        if (c == 0) continue;
        if (c > (unsigned)TILED_LCAP) {  // keys were dropped: this query is redone on its own
            if (tid == 0) flags[q] = 1u;
            continue;
        }
        char *base = const_cast<char *>(ws) + (size_t)q * ws_stride;
        unsigned *counts = reinterpret_cast<unsigned *>(base + countsA_off);
        uint64_t *dst = reinterpret_cast<uint64_t *>(base + listsA_off) + (size_t)gc * TILED_LCAP;
        if (tid == 0) counts[gc] = c;
        for (unsigned i = tid; i < c; i += NT) {
            const unsigned key = keys[k][i];
            dst[i] = ((uint64_t)(key >> 24) << 32) | (uint64_t)(c0 + (key & 0xffffffu));
        }
    }
}

bool make_tiled_plan(int64_t n, int m, int nq, TiledPlan *t)
{
    t->B = m / 2;
    const int cpt = (t->B <= 16) ? SCAN_VEC * (16 / t->B) : 1;
    const int tile = tiled_nt(t->B) * cpt;
    // chunks: at most TILED_MAX_CHUNKS per query, at least 64 tiles long, a multiple of the tile,
    // below 2^24 codes (index bits of a key)
    int64_t chunk = ceil_div(ceil_div(n, TILED_MAX_CHUNKS), tile) * tile;
    if (chunk < 64ll * tile) chunk = 64ll * tile;
    const int64_t max_chunk = ((1ll << 24) - 1) / tile * tile;
    if (chunk > max_chunk) return false;
    t->chunk = chunk;
    t->GC = (int)ceil_div(n, chunk);
    t->lds_bytes = (size_t)t->B * 256 * sizeof(uint4);
    return t->GC >= 1 && t->GC <= 65535 && nq >= 1;
}

template <int B>
static int launch_tiled(const TiledPlan &t, const uint8_t *codes, int64_t n, int nq, int cap,
                        const unsigned *taus, char *ws, size_t ws_stride, size_t countsA_off,
                        size_t listsA_off, unsigned *flags, hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        QADC_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_u8_tiled_kernel<B>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)t.lds_bytes));
        attr_set = true;
    }
    dim3 grid((unsigned)ceil_div(nq, TILED_Q), (unsigned)t.GC);
    launch(QADC_PROF_SCAN, scan_u8_tiled_kernel<B>, grid, dim3(tiled_nt(B)), t.lds_bytes, st, codes, n, t.chunk,
           nq, cap, taus, (const char *)ws, ws_stride, countsA_off, listsA_off, flags);
    return QADC_OK;
}

int run_tiled_scan(const TiledPlan &t, const uint8_t *codes, int64_t n, int nq, int cap, int R,
                   unsigned *taus, char *ws, size_t ws_stride, size_t countsA_off, size_t listsA_off,
                   unsigned *flags, hipStream_t st)
{
    launch(QADC_PROF_SEED, scan_tau_kernel, dim3((unsigned)ceil_div(nq, 4)), dim3(256), 0, st,
           (const char *)ws, ws_stride, nq, R, taus);
    switch (t.B) {
    case 4: return launch_tiled<4>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    case 8: return launch_tiled<8>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    case 16: return launch_tiled<16>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    default: return launch_tiled<32>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    }
}

}  // namespace qadc
