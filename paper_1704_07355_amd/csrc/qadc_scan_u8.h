// Device helpers shared by the kernels that scan 4-bit codes with 8-bit tables (Alg. 2 of the
// paper): pair tables in LDS, sums of a tile of codes, candidate keys.
#pragma once

#include "qadc_scan_common.h"

namespace qadc {

struct ScanShared {
    SelectScratch sel;
    unsigned ccnt;     // append counter of a compaction
    unsigned tcnt[3];  // append counters of the tiles, used in rotation
    unsigned tau;      // threshold bin published by wave 0
    unsigned fcnt;     // append counter of the barrier-free pass (may run past the list's end)
};

#ifndef QADC_EARLY_STAGES
// (a check at a quarter and at half of the bytes measured the same as the one check at half)
#define QADC_EARLY_STAGES(B) ((B) >= 4 ? 2 : 1)
#endif

// One pair-table entry, known to the compiler as a byte value.
__device__ __forceinline__ unsigned pair_entry(const uint8_t *ptab, int jb, unsigned v)
{
    const unsigned e = ptab[jb * 256 + v];
    __builtin_assume(e < 256u);
    return e;
}

// Component j of code c of a thread's 48 bytes of 6-bit codes (compile-time position).
template <int BYTES>
__device__ __forceinline__ unsigned sixbit_field(const uint4 (&w)[3], int c, int j)
{
    const int bit = c * BYTES * 8 + 6 * j;
    const int word = bit >> 5, sh = bit & 31;
    auto dword = [&](int i) {
        const uint4 &v = w[i >> 2];
        return (i & 3) == 0 ? v.x : (i & 3) == 1 ? v.y : (i & 3) == 2 ? v.z : v.w;
    };
    const unsigned lo = dword(word);
    if (sh <= 26) return (lo >> sh) & 63u;
    return __funnelshift_r(lo, dword(word + 1), sh) & 63u;  // the field crosses into the next word
}

// Sum of the table entries of code c of a thread's 6-bit codes over the components [first, last).
template <int B, int NT>
__device__ __forceinline__ unsigned sixbit_sum(const uint4 (&w)[3], const uint8_t *ptab, int c, int first, int last)
{
    using C = ScanCfg<B, NT>;
    unsigned s = 0;
#pragma unroll
    for (int j = first; j < last; ++j) s += ptab[j * 64 + sixbit_field<C::BYTES>(w, c, j)];
    return s;
}

// Lookups, sum, clamp, key = sum << 24 | index among the workgroup's codes (NO_KEY where no
// code; FULL: every slot of the tile holds a code).
template <int B, int NT, bool FULL = false>
__device__ __forceinline__ void tile_keys(const uint4 (&w)[ScanCfg<B, NT>::NVEC], const int (&nc)[2], unsigned rel0,
                                          const uint8_t *ptab, unsigned cap,
                                          unsigned (&k)[ScanCfg<B, NT>::CPT])
{
    const int tid = threadIdx.x;
    if constexpr (ScanCfg<B, NT>::SIX) {
        using C = ScanCfg<B, NT>;
#pragma unroll
        for (int c = 0; c < C::CPT; ++c) {
            unsigned s = sixbit_sum<B, NT>(w, ptab, c, 0, C::M6);
            s = min(s, cap);
            const unsigned key = (s << 24) | (rel0 + SixbitLayout<C::BYTES>::slot(tid, c));
            k[c] = (FULL || ((nc[0] >> c) & 1)) ? key : NO_KEY;
        }
    } else if constexpr (B <= 16) {
        constexpr int CPV = 16 / B;
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const unsigned li0 = rel0 + (unsigned)((v * NT + tid) * CPV);
#pragma unroll
            for (int c = 0; c < CPV; ++c) {
                unsigned s = 0;
#pragma unroll
                for (int jb = 0; jb < B; ++jb) s += pair_entry(ptab, jb, byte_of(w[v], c * B + jb));
                s = min(s, cap);
                const unsigned key = (s << 24) | (li0 + c);
                k[v * CPV + c] = (FULL || c < nc[v]) ? key : NO_KEY;
            }
        }
    } else {
        unsigned s = 0;
#pragma unroll
        for (int jb = 0; jb < 16; ++jb) s += pair_entry(ptab, jb, byte_of(w[0], jb));
#pragma unroll
        for (int jb = 0; jb < 16; ++jb) s += pair_entry(ptab, 16 + jb, byte_of(w[1], jb));
        s = min(s, cap);
        k[0] = (FULL || nc[0]) ? ((s << 24) | (rel0 + (unsigned)tid)) : NO_KEY;
    }
}

// Unclamped sums of a whole tile (every slot holds a code), for the pass that only keeps sums at or
// below `bound`, itself smaller than the saturation value.  Entries are not negative, so a code
// whose first B/2 bytes already sum to more than the bound cannot pass: the lookups of the other
// bytes are done only by the lanes that hold a code still in the race (a wavefront without one skips
// them; with few lanes left they no longer collide on the LDS banks), and the others report their
// partial sum, which is above the bound as the full one would be.
template <int B, int NT>
__device__ __forceinline__ void tile_sums(const uint4 (&w)[ScanCfg<B, NT>::NVEC], const uint8_t *ptab, unsigned bound,
                                          unsigned (&sm)[ScanCfg<B, NT>::CPT])
{
    if constexpr (ScanCfg<B, NT>::SIX) {
        // two stages of m / 2 components, a check between them
        using C = ScanCfg<B, NT>;
        constexpr int NL = C::M6;
        unsigned best = 0xffffffffu;
#pragma unroll
        for (int c = 0; c < C::CPT; ++c) {
            sm[c] = sixbit_sum<B, NT>(w, ptab, c, 0, NL / 2);
            best = min(best, sm[c]);
        }
        if (best <= bound) {
#pragma unroll
            for (int c = 0; c < C::CPT; ++c) sm[c] += sixbit_sum<B, NT>(w, ptab, c, NL / 2, NL);
        }
    } else if constexpr (B <= 16) {
        constexpr int CPV = 16 / B;
        // the bytes are summed in stages, with a check after each stage but the last
        constexpr int NS = QADC_EARLY_STAGES(B);
        constexpr int cut[4] = {0, NS == 3 ? B / 4 : (NS == 2 ? B / 2 : B), NS == 3 ? B / 2 : B, B};
#pragma unroll
        for (int c = 0; c < 2 * CPV; ++c) sm[c] = 0;
        bool go = true;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            if (go) {
                unsigned best = 0xffffffffu;
#pragma unroll
                for (int v = 0; v < 2; ++v) {
#pragma unroll
                    for (int c = 0; c < CPV; ++c) {
                        unsigned s = sm[v * CPV + c];
#pragma unroll
                        for (int jb = cut[st]; jb < cut[st + 1]; ++jb) s += pair_entry(ptab, jb, byte_of(w[v], c * B + jb));
                        sm[v * CPV + c] = s;
                        best = min(best, s);
                    }
                }
                go = best <= bound;
            }
        }
    } else {
        unsigned s = 0;
#pragma unroll
        for (int jb = 0; jb < 16; ++jb) s += pair_entry(ptab, jb, byte_of(w[0], jb));
        if (s <= bound) {
#pragma unroll
            for (int jb = 0; jb < 16; ++jb) s += pair_entry(ptab, 16 + jb, byte_of(w[1], jb));
        }
        sm[0] = s;
    }
}

// Index of slot c of this thread inside a tile (the layout tile_load and tile_keys use).
template <int B, int NT>
__device__ __forceinline__ unsigned tile_slot_index(int c)
{
    if constexpr (ScanCfg<B, NT>::SIX) {
        return SixbitLayout<ScanCfg<B, NT>::BYTES>::slot((int)threadIdx.x, c);
    } else if constexpr (B <= 16) {
        constexpr int CPV = 16 / B;
        return (unsigned)(((c / CPV) * NT + (int)threadIdx.x) * CPV + c % CPV);
    } else {
        return threadIdx.x;
    }
}

// Pair tables of one query in LDS: ptab[jb][v] = min(cap, q[2jb][v & 15] + q[2jb+1][v >> 4]).
// `wide`: 8-bit components, the byte-indexed table is the caller's table of component jb itself.
template <int B, int NT>
__device__ __forceinline__ void build_pair_tables(const uint8_t *__restrict__ qlut, unsigned cap,
                                                  uint8_t *ptab, bool wide = false)
{
    if constexpr (ScanCfg<B, NT>::SIX) {  // 6-bit components: the caller's m tables of 64 entries
        for (int e = threadIdx.x; e < ScanCfg<B, NT>::TAB_BYTES; e += NT) ptab[e] = (uint8_t)min((unsigned)qlut[e], cap);
        return;
    } else {
    if (wide) {
        for (int e = threadIdx.x; e < B * 256; e += NT) ptab[e] = (uint8_t)min((unsigned)qlut[e], cap);
        return;
    }
    for (int e = threadIdx.x; e < B * 256; e += NT) {
        const int jb = e >> 8, v = e & 255;
        const unsigned s = (unsigned)qlut[(2 * jb) * 16 + (v & 15)] +
                           (unsigned)qlut[(2 * jb + 1) * 16 + (v >> 4)];
        ptab[e] = (uint8_t)min(s, cap);
    }
    }
}

// Ascending bitonic sort of 4 * 64 values held four per lane by one wavefront: element
// e = 4 * lane + r.  Exchanges at distance < 4 stay inside a lane, the others go through
// __shfl_xor.  Called by a whole wavefront.
__device__ __forceinline__ void wave_bitonic_sort4(unsigned (&v)[4])
{
    const unsigned lane = (unsigned)lane_id();
#pragma unroll
    for (unsigned k = 2; k <= 256; k <<= 1) {
#pragma unroll
        for (unsigned j = k >> 1; j > 0; j >>= 1) {
            if (j >= 4) {
#pragma unroll
                for (unsigned r = 0; r < 4; ++r) {
                    const unsigned e = 4 * lane + r;
                    const unsigned other = __shfl_xor(v[r], (int)(j >> 2));
                    const bool up = (e & k) == 0, lower = (e & j) == 0;
                    v[r] = (lower == up) ? min(v[r], other) : max(v[r], other);
                }
            } else {
#pragma unroll
                for (unsigned r = 0; r < 4; ++r) {
                    if ((r & j) == 0) {
                        const unsigned e = 4 * lane + r;
                        const bool up = (e & k) == 0;
                        const unsigned a = v[r], b = v[r ^ j];
                        v[r] = up ? min(a, b) : max(a, b);
                        v[r ^ j] = up ? max(a, b) : min(a, b);
                    }
                }
            }
        }
    }
}

}  // namespace qadc
