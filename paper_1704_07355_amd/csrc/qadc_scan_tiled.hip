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
// Groups of sixteen queries whose bounds are all small take a denser form of the same idea
// (scan_u8_tiled16_kernel: byte lanes, sixteen queries per LDS read).
//
// Selection: each query's grid-wide bound (from the seed kernel's histogram) is known
// before the scan starts; sums at or below it are appended to small per-query LDS lists.  A
// list that overflows marks its query for the single-query kernel, which redoes that query
// alone with its exact machinery; the merge kernel takes whichever result is valid.

#include <mutex>

#include "qadc_scan_common.h"
#include <algorithm>

#include "qadc_scan_tiled.h"
#include "qadc_onehot.h"

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

// Workgroup id -> (query group, database chunk).  Workgroups are handed to the 8 XCDs in turn,
// each XCD with an L2 of its own: XCD x = id % 8 takes the chunks congruent to x, and all query
// groups of a chunk follow each other in its share of the ids, so that the chunk is fetched
// from HBM once and every XCD gets the same mix of groups, whichever of them are active.
__device__ __forceinline__ void tiled_group_and_chunk(int ngroups, int &grp, int &chunk)
{
    const unsigned id = blockIdx.x;
    const unsigned slot = id >> 3;
    grp = (int)(slot % (unsigned)ngroups);
    chunk = (int)((slot / (unsigned)ngroups) * 8u + (id & 7u));
}

constexpr int TILED16_GP = 2;                       // code bytes summed in byte lanes
constexpr unsigned TILED16_CL = 255 / TILED16_GP;   // entries are clamped to this

// Which kernel scans a group of 16 queries is decided by the largest bound in the group (see the
// byte-lane kernel below).
__device__ __forceinline__ unsigned tiled_group_bound(const unsigned *__restrict__ taus, int q0, int nq)
{
    unsigned t = 0;
    for (int k = 0; k < 16; ++k)
        if (q0 + k < nq) t = max(t, taus[q0 + k]);
    return t;
}
// true: byte lanes (scan_u8_tiled16_kernel);  false: 16-bit lanes (scan_u8_tiled_kernel)
__device__ __forceinline__ bool tiled_group_in_bytes(unsigned bound, unsigned cl)
{
    return bound < cl;
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
    int grp, gc;
    tiled_group_and_chunk((nq + TILED_Q - 1) / TILED_Q, grp, gc);
    const int q0 = grp * TILED_Q;
    const unsigned cap = (unsigned)cap_i;
    const int64_t c0 = (int64_t)gc * chunk;
    const int64_t c1 = min(n, c0 + chunk);
    if (c0 >= c1) return;
    // uniform: groups of 16 queries whose bounds are small are scanned by the byte-lane kernels
    if (tiled_group_in_bytes(tiled_group_bound(taus, q0 / 16 * 16, nq), TILED16_CL)) return;

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

// Byte-lane form for sixteen queries.  When every bound of a group of 16 queries is below
// CL = 255 / GP, a sum can only pass if each of its table entries is at most the bound, so the
// entries may be clamped to CL without changing which sums pass or their values.  Clamped
// entries of GP consecutive code bytes then add up inside the four byte lanes of a register
// without a carry (GP * CL <= 255): a 16-byte LDS entry serves 16 queries, and the widening
// to 16-bit lanes is paid once per GP code bytes.  GP = 2 is used (bounds <= 126; GP = 4 needs
// bounds <= 62 and measures no faster: the kernel is bound by LDS bank conflicts of the
// 16-byte reads, not by the adds).  Groups with a larger bound are left to the 16-bit kernel
// above.  Both kernels are launched over the whole batch; a workgroup whose group belongs to
// the other kernel exits at once.
template <int B, int GP>
__global__ __launch_bounds__(tiled_nt(B)) void scan_u8_tiled16_kernel(
    const uint8_t *__restrict__ codes, int64_t n, int64_t chunk, int nq,
    const unsigned *__restrict__ taus, const char *__restrict__ ws, size_t ws_stride,
    size_t countsA_off, size_t listsA_off, unsigned *__restrict__ flags)
{
    constexpr int NT = tiled_nt(B);
    constexpr int TQ = 16;
    constexpr unsigned CL = 255 / GP;
    using C = ScanCfg<B, NT>;
    extern __shared__ uint4 tab[];  // [B * 256] entries of sixteen clamped pair sums
    __shared__ unsigned keys[TQ][TILED_LCAP];
    __shared__ unsigned cnt[TQ];

    const int tid = threadIdx.x;
    int grp, gc;
    tiled_group_and_chunk((nq + TQ - 1) / TQ, grp, gc);
    const int q0 = grp * TQ;
    const int64_t c0 = (int64_t)gc * chunk;
    const int64_t c1 = min(n, c0 + chunk);
    if (c0 >= c1) return;
    static_assert(CL == TILED16_CL, "the two kernels must agree on who scans a group");
    if (!tiled_group_in_bytes(tiled_group_bound(taus, q0, nq), CL)) return;  // uniform

    uint4 w[2];
    int nc[2];
    tile_load<B, NT>(codes, c0, c1, w, nc);

    // interleave the sixteen queries' clamped pair tables; a missing query gets CL everywhere
    for (int e = tid; e < B * 256; e += NT) {
        unsigned d[4] = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < TQ; ++k) {
            const int q = q0 + k;
            unsigned v = CL;
            if (q < nq) v = min(CL, (unsigned)reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride)->ptab[e]);
            d[k >> 2] |= v << (8 * (k & 3));
        }
        tab[e] = make_uint4(d[0], d[1], d[2], d[3]);
    }
    if (tid < TQ) cnt[tid] = 0;
    // Query k of the group lives in byte (k & 3) of entry dword (k >> 2), and after widening in
    // 16-bit lane ((k >> 1) & 1) of accumulator 2 * (k >> 2) + (k & 1).  bound + 1 per lane
    // (0 where there is no query): lane of (acc -sat- thr1) is zero exactly when the sum passes.
    unsigned thr[TQ];
    unsigned thr1[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) thr1[i] = 0;
#pragma unroll
    for (int k = 0; k < TQ; ++k) {
        const int q = q0 + k;
        thr[k] = 0xffffffffu;  // no query
        if (q < nq) {
            thr[k] = taus[q];
            thr1[2 * (k >> 2) + (k & 1)] |= (thr[k] + 1u) << (16 * ((k >> 1) & 1));
        }
    }
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
                unsigned a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int j0 = 0; j0 < B; j0 += GP) {
                    uint4 e = make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int j = 0; j < GP; ++j) {
                        const int jb = j0 + j;
                        unsigned byte;
                        if constexpr (B <= 16) byte = byte_of(w[v], c * B + jb);
                        else byte = byte_of(w[jb >> 4], jb & 15);
                        const uint4 f = tab[jb * 256 + byte];
                        e.x += f.x; e.y += f.y; e.z += f.z; e.w += f.w;  // byte lanes: GP * CL <= 255
                    }
                    const unsigned ed[4] = {e.x, e.y, e.z, e.w};
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        a[2 * d] += __builtin_amdgcn_perm(0u, ed[d], 0x0c020c00u);      // bytes 0, 2
                        a[2 * d + 1] += __builtin_amdgcn_perm(0u, ed[d], 0x0c030c01u);  // bytes 1, 3
                    }
                }
                const bool valid = (B <= 16) ? (c < nc[v]) : (nc[0] != 0);
                const unsigned li = rel + (unsigned)((B <= 16) ? (v * NT + tid) * CPV + c : tid);
                unsigned z = pk_sub_sat_u16(a[0], thr1[0]);
#pragma unroll
                for (int i = 1; i < 8; ++i) z = pk_min_u16(z, pk_sub_sat_u16(a[i], thr1[i]));
                const bool any = valid && min(z & 0xffffu, z >> 16) == 0u;
                if (__ballot(any) != 0ull) {
#pragma unroll
                    for (int k = 0; k < TQ; ++k) {
                        const unsigned acc = a[2 * (k >> 2) + (k & 1)];
                        const unsigned sum = ((k >> 1) & 1) ? (acc >> 16) : (acc & 0xffffu);
                        const bool pass = valid && thr[k] != 0xffffffffu && sum <= thr[k];
                        const unsigned slot = wave_append_slot(pass, &cnt[k]);
                        if (pass && slot < (unsigned)TILED_LCAP) keys[k][slot] = (sum << 24) | li;
                    }
                }
            }
        }
    }
    __syncthreads();

#pragma unroll 1
    for (int k = 0; k < TQ; ++k) {
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

// smallest batches for the matrix-core kernel (from 16 queries with 8 code bytes or more, from 32
// with 4: measured against the vector-ALU kernels over 10 M codes) and for its forms with 64 and 128
// queries per wavefront
static int mfma_min_q(int B)
{
    return std::max(1, knob_or(knobs().mfma_min_q, B >= 8 ? TILED_MFMA_MIN_Q : 2 * TILED_MFMA_MIN_Q));
}
static int mfma_min_q2() { return std::max(1, knob_or(knobs().mfma_min_q2, TILED_MFMA_MIN_Q2)); }
// 128 queries per wavefront (codes of up to 8 bytes): when the last set of 128 is more than half full
static bool mfma_four(int B, int nq)
{
    const int min_q4 = std::max(1, knob_or(knobs().mfma_min_q4, TILED_MFMA_MIN_Q4));
    return B <= 8 && nq >= min_q4 && ((nq & 127) == 0 || (nq & 127) > 64);
}

bool make_tiled_plan(int64_t n, int m, int nq, bool codes4, TiledPlan *t)
{
    t->B = m / 2;
    const int cpt = (t->B <= 16) ? SCAN_VEC * (16 / t->B) : 1;
    const int tile = tiled_nt(t->B) * cpt;
    // 4-bit codes and a batch that fills a good part of a wavefront's 32 or 64 queries: the
    // matrix-core kernel scans it
    t->mfma = codes4 && nq >= mfma_min_q(t->B) && knob_or(knobs().tiled_mfma, 1) != 0;
    // chunks: at most TILED_MAX_CHUNKS per query, a multiple of the tile, below 2^24 codes (index
    // bits of a key); as long as possible (a workgroup builds its tables once per chunk) while
    // groups x chunks still make about four workgroups per compute unit: 64 tiles with many query
    // groups, down to 8 tiles for a batch of one or two groups over a short database.  The
    // matrix-core kernel runs one wavefront per (32 or 64 queries, chunk): it wants about 4096 of
    // them (two to four per SIMD, twice over), each at least two tiles long, so a batch of one or
    // two such sets is cut into up to TILED_MFMA_MAX_CHUNKS chunks.
    const int64_t groups = ceil_div(nq, 16);
    int64_t want = std::max<int64_t>(1, std::min<int64_t>(TILED_MAX_CHUNKS, ceil_div(1024, groups)));
    int64_t lo = 8, hi = 64, max_chunks = TILED_MAX_CHUNKS;
    if (t->mfma) {
        const int qw = mfma_four(t->B, nq) ? 128 : (t->B <= 16 && nq >= mfma_min_q2()) ? 64 : 32;
        // more chunks for small batches, as long as the lists of the whole batch (516 bytes per
        // query and chunk) stay within half of the 256 MiB that one launch's workspace may take:
        // beyond that the batch would be split into two launches
        max_chunks = std::min<int64_t>(TILED_MFMA_MAX_CHUNKS,
                                       std::max<int64_t>(TILED_MAX_CHUNKS, (128ll << 20) / (516ll * nq)));
        // never fewer than 512 chunks, however many sets of queries there are: a query's few
        // thousand candidates must stay well below the 64 (or 32) keys a wavefront can report per
        // query and chunk, or queries overflow and are redone one by one
        want = std::max<int64_t>(512, ceil_div(std::max(64, knob_or(knobs().mfma_waves, 4096)), ceil_div(nq, qw)));
        want = std::min<int64_t>(max_chunks, want);
        lo = 2;
        hi = 1ll << 40;
    }
    int64_t chunk = ceil_div(ceil_div(n, max_chunks), tile) * tile;
    int64_t by_fill = ceil_div(ceil_div(n, want), tile) * tile;
    if (by_fill > hi * tile) by_fill = hi * tile;
    if (by_fill < lo * tile) by_fill = lo * tile;
    if (chunk < by_fill) chunk = by_fill;
    const int64_t max_chunk = ((1ll << 24) - 1) / tile * tile;
    if (chunk > max_chunk) return false;
    t->chunk = chunk;
    t->GC = (int)ceil_div(n, chunk);
    t->lds_bytes = (size_t)t->B * 256 * sizeof(uint4);
    return t->GC >= 1 && t->GC <= 65535 && nq >= 1;
}

// ------------------------------------------------------------------ matrix-core form
//
// The lookups of a batch as a matrix product on the MFMA units: with onehot(c) the 16-vector that
// is 1 at position c, the sum of a code for a query is  sum_j onehot(c_j) . q^j  -- a row of 0/1
// bytes times a column of table entries, exact in int32.  A one-hot row is a structured-sparse row
// (one non-zero in 16, so at most two in every four), which is what the sparse matrix instruction
// takes: one v_smfmac_i32_32x32x64_i8 multiplies 32 codes by 32 queries over 64 values of k = four
// tables = two code bytes, and occupies the matrix pipe as long as the dense 32x32x32 instruction
// (32 cycles).  Operands, as found by probing the instruction with single non-zeros:
//   B (dense, 32 bytes per lane): lane (query = lane mod 32, half = lane / 32) holds k = 32 half ..
//     32 half + 31, i.e. the 16 entries of tables 4jp + 2 half and 4jp + 2 half + 1 of its query as
//     they lie in memory;
//   A (compressed, 16 bytes per lane + a register of 2-bit positions): lane (code = lane mod 32,
//     half) holds 16 stored values in pairs, pair g of the first eight for k = 16 half + 4g .. + 3,
//     pair g of the last eight for k = 32 + 16 half + 4g .. + 3; each stored value carries the
//     position (0..3) of its k inside the four.  So lanes 0..31 take the LOW nibbles of code bytes
//     2jp and 2jp + 1 (tables 4jp and 4jp + 2), lanes 32..63 the HIGH nibbles (tables 4jp + 1 and
//     4jp + 3): a nibble c puts a 1 into the first value of pair c / 4 with position c mod 4.
//   The 8 value bytes and the 16 position bits of a nibble come from a 16-entry table in LDS.
// So two code bytes cost one instruction for 32 codes x 32 queries, and the tables stay in
// registers for the whole scan.  A workgroup is ONE wavefront: it scans a chunk for 32 G queries
// (G groups of 32, G independent accumulator chains).  Lane l of the 32 x 32 result holds 16 sums
// of query (l mod 32): each is compared with that query's bound, and the rare pass is appended to
// the query's list in LDS.  Outputs as the other query-tiled kernels: lists per (query, chunk), a
// flag on overflow.  (The matrix units multiply signed bytes; the entries go in shifted by 128.)
constexpr int MFMA_SUB = 2;    // 32-code steps per load

// G: groups of 32 queries per wavefront.  2 for large batches of up to 32 code bytes (the table
// operands of 64 queries fill 128 registers when B = 16); 1 for B = 32 and for batches that would
// leave most of a 64-query wavefront empty.
template <int B, int G>
__global__ __launch_bounds__(64) void scan_u8_mfma_kernel(
    const uint8_t *__restrict__ codes, int64_t n, int64_t chunk, int nq, int cap_i,
    const uint8_t *__restrict__ qluts, const unsigned *__restrict__ taus, char *__restrict__ ws,
    size_t ws_stride, size_t countsA_off, size_t listsA_off, unsigned *__restrict__ flags)
{
    constexpr int WPC = B / 4;   // 32-bit words per code
    constexpr int QW = 32 * G;   // queries per wavefront
    constexpr int LC = (G > 2) ? TILED_LCAP / 2 : TILED_LCAP;  // keys kept per query (LDS: 16 KiB of lists)
    __shared__ unsigned keys[QW][LC];
    __shared__ unsigned cnt[QW];
    // of nibble c, at offset 8 c of either table: the 8 value bytes (byte 2 (c / 4) is 1) and the
    // position bits.  (Two tables, so that the two reads of a nibble stay an 8-byte and a 4-byte read
    // that land in the operand's registers, instead of one 12-byte read that has to be moved there.)
    __shared__ v2i_t nibval[16];
    __shared__ v2i_t nibpos[16];

    const int l = threadIdx.x;
    const int row = l & 31, half = l >> 5;
    int set, gc;
    tiled_group_and_chunk((nq + QW - 1) / QW, set, gc);
    const int q0 = set * QW;
    const unsigned cap = (unsigned)cap_i;
    const int64_t c0 = (int64_t)gc * chunk;
    const int64_t c1 = min(n, c0 + chunk);
    if (c0 >= c1) return;  // uniform

    // this lane's table entries: for code byte jb, the 16 entries of table 2jb + half of query
    // q0 + 32g + row (zeros for a query that does not exist: it never passes)
    // The matrix unit multiplies SIGNED bytes: an entry e goes in as e - 128 (= e xor 0x80), every
    // sum then comes out as sum - 128 * (2B tables) and the bounds are shifted by the same amount.
    constexpr int SHIFT = 128 * 2 * B;
    constexpr int NP = B / 2;  // pairs of code bytes = instructions per 32-code step and group
    v8i_t tb[G][NP];
    int thr[G];  // a shifted sum passes when it is <= thr
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int q = q0 + 32 * g + row;
        thr[g] = -1 - SHIFT;  // no query in this slot: nothing passes
        if (q < nq) {
            const unsigned t = taus[q];
            thr[g] = ((t >= cap) ? 0x7fffffff : (int)t) - SHIFT;
        }
#pragma unroll
        for (int jp = 0; jp < NP; ++jp) {  // (loads without a branch around them: all in flight at once)
            const v4i_t *src = reinterpret_cast<const v4i_t *>(qluts + ((size_t)min(q, nq - 1) * (2 * B) + 4 * jp + 2 * half) * 16);
            const v4i_t e0 = src[0], e1 = src[1];
            const int flip = (q < nq) ? (int)0x80808080u : 0, keep = (q < nq) ? -1 : 0;
            tb[g][jp] = v8i_t{(e0[0] ^ flip) & keep, (e0[1] ^ flip) & keep, (e0[2] ^ flip) & keep, (e0[3] ^ flip) & keep,
                              (e1[0] ^ flip) & keep, (e1[1] ^ flip) & keep, (e1[2] ^ flip) & keep, (e1[3] ^ flip) & keep};
        }
    }
    for (int i = l; i < QW; i += 64) cnt[i] = 0;
    if (l < 16) onehot_nibble_entry(l, nibval, nibpos);
    __syncthreads();

    // codes: lane (row, half) reads code `row` of each 32-code step (both halves read the same code).
    // Past the end of the chunk the last code is read again: loads without a branch around them, and
    // sums of positions beyond the chunk are never kept.
    unsigned cw[MFMA_SUB][WPC], cn[MFMA_SUB][WPC];
    auto fetch = [&](int64_t t0, unsigned (&dst)[MFMA_SUB][WPC]) {
#pragma unroll
        for (int s = 0; s < MFMA_SUB; ++s) {
            const int64_t i = min(t0 + 32 * s + row, c1 - 1);
            const unsigned *src = reinterpret_cast<const unsigned *>(codes + i * B);
#pragma unroll
            for (int k = 0; k < WPC; ++k) dst[s][k] = src[k];
        }
    };
    fetch(c0, cn);
    // the sparse operand of code bytes 2jp and 2jp + 1 of a code whose words are w[]: this lane's
    // nibble of either byte; its value bytes (8) and position bits come from the nibble table in LDS
    // at offset 8 * nibble (an 8-byte and a 4-byte read each, straight into their registers)
    struct Operand {  // as read; put together only where it is used, so that nothing waits for the reads early
        v2i_t v0, v1;
        int p0, p1;
    };
    auto operand = [&](const unsigned (&w)[WPC], int jp) {
        // every byte of x: 8 * (this lane's nibble of the code byte), the offset of the nibble's entries
        const unsigned x = onehot_nibble_offsets(w[jp >> 1], half);
        const unsigned o0 = __builtin_amdgcn_ubfe(x, 16 * (jp & 1), 8), o1 = __builtin_amdgcn_ubfe(x, 16 * (jp & 1) + 8, 8);
        const char *tv = reinterpret_cast<const char *>(nibval), *tp = reinterpret_cast<const char *>(nibpos);
        return Operand{*reinterpret_cast<const v2i_t *>(tv + o0), *reinterpret_cast<const v2i_t *>(tv + o1),
                       *reinterpret_cast<const int *>(tp + o0), *reinterpret_cast<const int *>(tp + o1)};
    };
    // Tests the G x 16 sums a lane holds after a step whose first code is `rel` (relative to c0).
    // Result v of a lane: code (v / 4) * 8 + half * 4 + v % 4 of the step, query row (+32g).
    auto test = [&](const v16i_t (&sum)[G], unsigned rel) {
        // the smallest of a group's 16 sums against its bound (three-input minima: 8 operations)
        int lo[G];
        bool any = false;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            lo[g] = sum[g][0];
#pragma unroll
            for (int v = 1; v < 15; v += 2) lo[g] = min(min(lo[g], sum[g][v]), sum[g][v + 1]);
            lo[g] = min(lo[g], sum[g][15]);
            any = any | (lo[g] <= thr[g]);
        }
        if (__ballot(any) != 0ull) {  // some sum of the step passes: which group, which four results, which one
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (__ballot(lo[g] <= thr[g]) == 0ull) continue;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int qm = min(min(sum[g][4 * u], sum[g][4 * u + 1]), min(sum[g][4 * u + 2], sum[g][4 * u + 3]));
                    if (__ballot(qm <= thr[g]) == 0ull) continue;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const unsigned li = rel + (unsigned)(u * 8 + half * 4 + w);
                        if (c0 + (int64_t)li < c1 && sum[g][4 * u + w] <= thr[g]) {
                            const unsigned slot = atomicAdd(&cnt[32 * g + row], 1u);
                            if (slot < (unsigned)LC)
                                keys[32 * g + row][slot] = (min((unsigned)(sum[g][4 * u + w] + SHIFT), cap) << 24) | li;
                        }
                    }
                }
            }
        }
    };
    // the operands are read two products ahead, across the steps as well
    Operand a0 = operand(cn[0], 0), a1 = operand(cn[0], NP > 1 ? 1 : 0);
    for (int64_t t0 = c0; t0 < c1; t0 += 32 * MFMA_SUB) {  // uniform
#pragma unroll
        for (int s = 0; s < MFMA_SUB; ++s)
#pragma unroll
            for (int k = 0; k < WPC; ++k) cw[s][k] = cn[s][k];
        if (t0 + 32 * MFMA_SUB < c1) fetch(t0 + 32 * MFMA_SUB, cn);  // the next codes travel meanwhile
#pragma unroll
        for (int s = 0; s < MFMA_SUB; ++s) {
            if (t0 + 32 * s >= c1) break;  // uniform
            v16i_t acc[G];  // (the sparse instruction has no zero addend: cleared by hand)
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = mfma_zero_acc();
#pragma unroll
            for (int jp = 0; jp < NP; ++jp) {
                const Operand a = a0;
                a0 = a1;
                // (past the last step of the last load these are operands nobody uses)
                if (jp + 2 < NP) a1 = operand(cw[s], jp + 2);
                else if (s + 1 < MFMA_SUB) a1 = operand(cw[s + 1], (jp + 2 - NP) % NP);
                else a1 = operand(cn[0], (jp + 2 - NP) % NP);
                asm volatile("" ::: "memory");  // the reads above are issued before the products below, not sunk to their use
                const v4i_t av = v4i_t{a.v0[0], a.v0[1], a.v1[0], a.v1[1]};
                int p0 = a.p0, p1 = a.p1;
                asm volatile("" : "+v"(p0), "+v"(p1));  // the position halves are joined here, not right behind their reads
                const int ap = p0 | (p1 << 16);
#pragma unroll
                for (int g = 0; g < G; ++g)
                    acc[g] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(av, tb[g][jp], acc[g], ap, 0, 0);
            }
            test(acc, (unsigned)(t0 - c0) + 32u * s);
        }
    }
    __syncthreads();

    // a lane reports for query q0 + k, k = lane, lane + 64
    for (int k = l; k < QW; k += 64) {
        const int q = q0 + k;
        if (q >= nq) break;
        const unsigned c = cnt[k];
        if (c > (unsigned)LC) {
            flags[q] = 1u;  // keys were dropped: this query is redone on its own
        } else if (c) {
            char *base = ws + (size_t)q * ws_stride;
            unsigned *counts = reinterpret_cast<unsigned *>(base + countsA_off);
            uint64_t *dst = reinterpret_cast<uint64_t *>(base + listsA_off) + (size_t)gc * TILED_LCAP;
            counts[gc] = c;
            for (unsigned i = 0; i < c; ++i) {
                const unsigned key = keys[k][i];
                dst[i] = ((uint64_t)(key >> 24) << 32) | (uint64_t)(c0 + (key & 0xffffffu));
            }
        }
    }
}

template <int B, int G>
static int launch_tiled_mfma(const TiledPlan &t, const uint8_t *codes, int64_t n, int nq, int cap,
                             const uint8_t *qluts, const unsigned *taus, char *ws, size_t ws_stride,
                             size_t countsA_off, size_t listsA_off, unsigned *flags, hipStream_t st)
{
    const unsigned gc8 = (unsigned)ceil_div(t.GC, 8) * 8u;
    dim3 grid((unsigned)ceil_div(nq, 32 * G) * gc8);
    launch(QADC_PROF_SCAN, (scan_u8_mfma_kernel<B, G>), grid, dim3(64), 0, st, codes, n, t.chunk, nq, cap, qluts, taus,
           ws, ws_stride, countsA_off, listsA_off, flags);
    return QADC_OK;
}

template <int B>
static int launch_tiled(const TiledPlan &t, const uint8_t *codes, int64_t n, int nq, int cap,
                        const unsigned *taus, char *ws, size_t ws_stride, size_t countsA_off,
                        size_t listsA_off, unsigned *flags, hipStream_t st)
{
    static std::once_flag attr_once;  // the kernels use more dynamic LDS than the default limit (size fixed by B)
    hipError_t attr_rc = hipSuccess;
    std::call_once(attr_once, [&] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_u8_tiled_kernel<B>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)t.lds_bytes);
        if (attr_rc == hipSuccess)
            attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_u8_tiled16_kernel<B, TILED16_GP>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)t.lds_bytes);
    });
    QADC_HIP_TRY(attr_rc);
    // every group of 16 queries is scanned by exactly one of the two kernels
    const unsigned gc8 = (unsigned)ceil_div(t.GC, 8) * 8u;  // chunk slots, eight at a time
    dim3 grid16((unsigned)ceil_div(nq, 16) * gc8);
    launch(QADC_PROF_SCAN, (scan_u8_tiled16_kernel<B, TILED16_GP>), grid16, dim3(tiled_nt(B)), t.lds_bytes, st, codes, n,
           t.chunk, nq, taus, (const char *)ws, ws_stride, countsA_off, listsA_off, flags);
    dim3 grid((unsigned)ceil_div(nq, TILED_Q) * gc8);
    launch(QADC_PROF_SCAN, scan_u8_tiled_kernel<B>, grid, dim3(tiled_nt(B)), t.lds_bytes, st, codes, n, t.chunk,
           nq, cap, taus, (const char *)ws, ws_stride, countsA_off, listsA_off, flags);
    return QADC_OK;
}

// ------------------------------------------------------------------ seed for batches
//
// The bound of a scan comes from a sample of the database (see seed_u8_kernel).  For a batch the
// sample is the same codes for every query, so it is scanned in the query-tiled way too: a
// workgroup walks a few sample tiles for eight queries at once (16-bit lanes, as
// scan_u8_tiled_kernel) and counts every sum in the query's histogram in LDS; at the end one
// wavefront per query adds the lowest bins (the workgroup's best `flush_need` codes, never
// beyond its own R-th) to the query's grid-wide histogram.  The pair tables of the batch are
// written to the control blocks beforehand by ptab_build_kernel.

// hdr->ptab of every query: ptab[jb][v] = min(cap, q[2jb][v & 15] + q[2jb+1][v >> 4]); `wide`:
// 8-bit components, min(cap, q[jb][v]).  Four entries per thread.
template <int B>
__global__ __launch_bounds__(256) void ptab_build_kernel(const uint8_t *__restrict__ qluts, int cap_i,
                                                         int wide, char *__restrict__ ws, size_t ws_stride)
{
    const int q = blockIdx.x;
    const unsigned cap = (unsigned)cap_i;
    const uint8_t *ql = qluts + (size_t)q * (wide ? B * 256 : 2 * B * 16);
    ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
    for (int e4 = threadIdx.x; e4 < B * 64; e4 += 256) {
        unsigned packed = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = 4 * e4 + k;
            const int jb = e >> 8, v = e & 255;
            const unsigned sum = wide ? (unsigned)ql[e]
                                      : (unsigned)ql[(2 * jb) * 16 + (v & 15)] + (unsigned)ql[(2 * jb + 1) * 16 + (v >> 4)];
            packed |= min(sum, cap) << (8 * k);
        }
        reinterpret_cast<unsigned *>(hdr->ptab)[e4] = packed;
    }
}

template <int B>
__global__ __launch_bounds__(tiled_nt(B)) void seed_u8_tiled_kernel(
    const uint8_t *__restrict__ codes, int64_t n, int nq, int cap_i, int R, unsigned flush_need,
    int64_t stride, int tiles_per_wg, int n_tiles, char *__restrict__ ws, size_t ws_stride)
{
    constexpr int NT = tiled_nt(B);
    using C = ScanCfg<B, NT>;
    extern __shared__ uint4 tab[];  // [B * 256] entries of eight 16-bit pair sums
    __shared__ unsigned hist[TILED_Q][256];

    const int tid = threadIdx.x;
    const int ngroups = (nq + TILED_Q - 1) / TILED_Q;
    const int grp = (int)(blockIdx.x % (unsigned)ngroups);
    const int part = (int)(blockIdx.x / (unsigned)ngroups);
    const int q0 = grp * TILED_Q;
    const unsigned cap = (unsigned)cap_i;
    const int t_begin = part * tiles_per_wg;
    const int t_end = min(n_tiles, t_begin + tiles_per_wg);
    if (t_begin >= t_end) return;  // uniform

    uint4 w[2];
    int nc[2];
    {
        const int64_t c0 = (int64_t)t_begin * stride;
        tile_load<B, NT>(codes, c0, min(n, c0 + C::TILE), w, nc);
    }
    for (int e = tid; e < B * 256; e += NT) {
        unsigned v[TILED_Q];
#pragma unroll
        for (int k = 0; k < TILED_Q; ++k) {
            const int q = q0 + k;
            v[k] = 0;
            if (q < nq) v[k] = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride)->ptab[e];
        }
        tab[e] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
    }
    for (int e = tid; e < TILED_Q * 256; e += NT) (&hist[0][0])[e] = 0;
    __syncthreads();

    for (int t = t_begin; t < t_end; ++t) {  // uniform
        // the next sample tile is requested before this one is used
        uint4 wn[2] = {w[0], w[1]};
        int ncn[2] = {nc[0], nc[1]};
        if (t + 1 < t_end) {
            const int64_t c1 = (int64_t)(t + 1) * stride;
            tile_load<B, NT>(codes, c1, min(n, c1 + C::TILE), wn, ncn);
        }
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
                const unsigned acc[4] = {a0, a1, a2, a3};
#pragma unroll
                for (int k = 0; k < TILED_Q; ++k) {
                    const unsigned sum = (k & 1) ? (acc[k >> 1] >> 16) : (acc[k >> 1] & 0xffffu);
                    // saturated sums carry no information; a slot without a query counts nothing
                    if (valid && q0 + k < nq && sum < cap) atomicAdd(&hist[k][sum], 1u);
                }
            }
        }
        w[0] = wn[0]; w[1] = wn[1];
        nc[0] = ncn[0]; nc[1] = ncn[1];
    }
    __syncthreads();

    // wavefront k reports for query q0 + k
    const int k = tid / WAVE;
    const int l = tid % WAVE;
    if (k < TILED_Q && q0 + k < nq) {  // whole wavefronts
        unsigned h[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) h[b] = hist[k][4 * l + b];
        const unsigned f = min(wave_threshold_bin<4>(h, (unsigned)R), wave_threshold_bin<4>(h, flush_need));
        ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)(q0 + k) * ws_stride);
        unsigned *ghist = hdr->ghist[part % GH_REP];
        for (unsigned b0 = 0; b0 <= f && b0 < 256u; b0 += WAVE) {  // uniform over the wavefront
            const unsigned bin = b0 + l;
            const unsigned c = hist[k][bin];
            if (bin <= f && bin < cap && c)
                __hip_atomic_fetch_add(&ghist[bin], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <int B>
static int launch_tiled_seed(const TiledPlan &t, const uint8_t *codes, int64_t n, const uint8_t *qluts, int nq,
                             int cap, int R, int wide, int64_t sample_codes, char *ws, size_t ws_stride,
                             hipStream_t st)
{
    static std::once_flag attr_once;
    hipError_t attr_rc = hipSuccess;
    std::call_once(attr_once, [&] {
        attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(&seed_u8_tiled_kernel<B>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)t.lds_bytes);
    });
    QADC_HIP_TRY(attr_rc);
    constexpr int cpt = (B <= 16) ? SCAN_VEC * (16 / B) : 1;
    const int64_t tile = (int64_t)tiled_nt(B) * cpt;
    int64_t n_tiles = std::max<int64_t>(1, sample_codes / tile);
    if (n_tiles > n / tile) n_tiles = std::max<int64_t>(1, n / tile);
    const int64_t stride = std::max<int64_t>(tile, (n / n_tiles) / 16 * 16);
    const int64_t groups = ceil_div(nq, TILED_Q);
    // tiles per workgroup: long enough for the table build to pay, short enough to fill the GPU
    int64_t tpw = n_tiles * groups / 1024;
    if (tpw < 4) tpw = 4;
    if (tpw > 32) tpw = 32;
    const int64_t parts = ceil_div(n_tiles, tpw);
    int64_t flush = ceil_div(4ll * R, parts);
    if (flush < 16) flush = 16;
    if (flush > R) flush = R;
    launch(QADC_PROF_SEED, ptab_build_kernel<B>, dim3((unsigned)nq), dim3(256), 0, st, qluts, cap, wide, ws,
           ws_stride);
    launch(QADC_PROF_SEED, seed_u8_tiled_kernel<B>, dim3((unsigned)(groups * parts)), dim3(tiled_nt(B)), t.lds_bytes,
           st, codes, n, nq, cap, R, (unsigned)flush, stride, (int)tpw, (int)n_tiles, ws, ws_stride);
    return QADC_OK;
}

int run_tiled_seed(const TiledPlan &t, const uint8_t *codes, int64_t n, const uint8_t *qluts, int nq, int cap,
                   int R, int wide, int64_t sample_codes, char *ws, size_t ws_stride, hipStream_t st)
{
    switch (t.B) {
    case 4: return launch_tiled_seed<4>(t, codes, n, qluts, nq, cap, R, wide, sample_codes, ws, ws_stride, st);
    case 8: return launch_tiled_seed<8>(t, codes, n, qluts, nq, cap, R, wide, sample_codes, ws, ws_stride, st);
    case 16: return launch_tiled_seed<16>(t, codes, n, qluts, nq, cap, R, wide, sample_codes, ws, ws_stride, st);
    default: return launch_tiled_seed<32>(t, codes, n, qluts, nq, cap, R, wide, sample_codes, ws, ws_stride, st);
    }
}

int run_tiled_scan(const TiledPlan &t, const uint8_t *codes, int64_t n, int nq, int cap, int R,
                   unsigned *taus, char *ws, size_t ws_stride, size_t countsA_off, size_t listsA_off,
                   unsigned *flags, const uint8_t *qluts16, hipStream_t st)
{
    launch(QADC_PROF_SEED, scan_tau_kernel, dim3((unsigned)ceil_div(nq, 4)), dim3(256), 0, st,
           (const char *)ws, ws_stride, nq, R, taus);
    // (a last, short sub-batch of a large batch goes to the other kernels, over the same chunks)
    // (its table operands are 16-byte loads: tables at any other alignment go the other way too)
    if (t.mfma && qluts16 && reinterpret_cast<uintptr_t>(qluts16) % 16 == 0 && nq >= mfma_min_q(t.B)) {
#define QADC_MFMA_ARGS t, codes, n, nq, cap, qluts16, taus, ws, ws_stride, countsA_off, listsA_off, flags, st
        const bool two = t.B <= 16 && nq >= mfma_min_q2();  // 64 queries per wavefront
        const bool four = mfma_four(t.B, nq);               // 128
        switch (t.B) {
        case 4: return four ? launch_tiled_mfma<4, 4>(QADC_MFMA_ARGS) : two ? launch_tiled_mfma<4, 2>(QADC_MFMA_ARGS) : launch_tiled_mfma<4, 1>(QADC_MFMA_ARGS);
        case 8: return four ? launch_tiled_mfma<8, 4>(QADC_MFMA_ARGS) : two ? launch_tiled_mfma<8, 2>(QADC_MFMA_ARGS) : launch_tiled_mfma<8, 1>(QADC_MFMA_ARGS);
        case 16: return two ? launch_tiled_mfma<16, 2>(QADC_MFMA_ARGS) : launch_tiled_mfma<16, 1>(QADC_MFMA_ARGS);
        default: return launch_tiled_mfma<32, 1>(QADC_MFMA_ARGS);
        }
#undef QADC_MFMA_ARGS
    }
    switch (t.B) {
    case 4: return launch_tiled<4>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    case 8: return launch_tiled<8>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    case 16: return launch_tiled<16>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    default: return launch_tiled<32>(t, codes, n, nq, cap, taus, ws, ws_stride, countsA_off, listsA_off, flags, st);
    }
}

}  // namespace qadc
