// Pieces shared by the scan kernels of the Quick ADC library (gfx950): workspace layout,
// tile loads, candidate-list compaction, the cross-workgroup merge kernel.
#pragma once

#include <stdlib.h>

#include "qadc_select.h"
#include "qadc_profile.h"

namespace qadc {

constexpr int SCAN_VEC = 2;               // 16-byte loads per thread and tile
constexpr int SCAN_SLACK = QADC_MAX_R;    // candidate slots beyond one tile
constexpr int GH_REP = 2;                 // replicas of the grid-wide histogram
constexpr unsigned NO_KEY = 0xffffffffu;

// Per-query control block in the workspace, followed by counts[G] (keys reported by each
// workgroup) and lists[G][R] (the keys).  Block and counts must be all zero when the scan
// kernel starts; the merge kernel leaves every word the call wrote zeroed again.
struct alignas(256) ScanHeader {
    unsigned ghist[GH_REP][256];  // sums of the best codes of every seed tile
    uint8_t ptab[32 * 256];       // the query's pair tables, left by the seed kernel for the scan
};

// Geometry of a scan.  B = bytes per code for 4-bit components (two per byte; also for 8-bit
// components, one per byte); B = SIXBIT + m for codes of m 6-bit components (3m/4 bytes, stored
// back to back, least significant bit first), whose thread takes 48 contiguous bytes per tile.
constexpr int SIXBIT = 1000;
template <int B, int NT>
struct ScanCfg {
    static constexpr bool SIX = B >= SIXBIT;
    static constexpr int M6 = SIX ? B - SIXBIT : 0;               // 6-bit components per code
    static constexpr int BYTES = SIX ? 3 * M6 / 4 : B;            // bytes per code
    static constexpr int NVEC = SIX ? 3 : SCAN_VEC;               // 16-byte loads per thread and tile
    static constexpr int CPV = (!SIX && B <= 16) ? 16 / B : 1;    // codes per 16-byte load (4-bit)
    static constexpr int CPT = SIX ? 48 / BYTES : ((B <= 16) ? SCAN_VEC * CPV : 1);  // codes per thread and tile
    static constexpr int TILE = NT * CPT;
    static constexpr int CAP = TILE + SCAN_SLACK;
    static constexpr int TAB_BYTES = SIX ? M6 * 64 : B * 256;     // lookup tables of a query in LDS
};

__device__ __forceinline__ unsigned byte_of(const uint4 &v, int k)
{
    const unsigned w = (k < 4) ? v.x : (k < 8) ? v.y : (k < 12) ? v.z : v.w;
    return (w >> (8 * (k & 3))) & 0xffu;
}

// Keys with sum <= tau are exactly the keys below this limit.
__device__ __forceinline__ unsigned limit_of_bin(unsigned tau)
{
    return tau >= 255u ? NO_KEY : ((tau + 1u) << 24);
}

// Called by one whole wave; h[b] is the count of bin NB*lane+b.  Returns, in every lane,
// the smallest bin whose inclusive running count reaches `need`, or 64*NB when none does.
template <int NB>
__device__ __forceinline__ unsigned wave_threshold_bin(const unsigned (&h)[NB], unsigned need,
                                                       unsigned *total = nullptr)
{
    const int l = lane_id();
    unsigned tot = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b) tot += h[b];
    unsigned inc = tot;
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        const unsigned up = __shfl_up(inc, d);
        if (l >= d) inc += up;
    }
    if (total) *total = __shfl(inc, WAVE - 1);
    const unsigned long long m = __ballot(inc >= need);
    if (m == 0) return (unsigned)(WAVE * NB);
    const int first = __ffsll((long long)m) - 1;
    unsigned run = inc - tot, bin = (unsigned)(NB * l + NB - 1);
    bool found = false;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        run += h[b];
        if (!found && run >= need) { bin = (unsigned)(NB * l + b); found = true; }
    }
    return __shfl(bin, first);
}

// Cuts keys[0..cnt) back to its `keep` smallest keys and returns the largest key kept.  A list
// of at most `keep` keys is left as it is (the value returned then bounds nothing).  K = key
// type, NBYTES = key bytes that can be non-zero.  Called by every thread of the workgroup with
// the same cnt and keep; `ccnt` is an LDS counter of the workgroup.  The caller's list then
// holds min(cnt, keep) keys.
template <typename K, int NBYTES, int NT, int CAP>
__device__ K compact_candidates(K *keys, unsigned cnt, unsigned keep, SelectScratch *sel,
                                unsigned *ccnt)
{
    if (cnt <= keep) return ~(K)0 - 1;  // uniform
    const K kth = block_radix_select<K, NBYTES>(keys, cnt, keep, sel);
    constexpr int PER = (CAP + NT - 1) / NT;
    K mine[PER];
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        unsigned i = threadIdx.x + t * NT;
        mine[t] = (i < cnt) ? keys[i] : ~(K)0;
    }
    if (threadIdx.x == 0) *ccnt = 0;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        unsigned i = threadIdx.x + t * NT;
        bool ok = (i < cnt) && (mine[t] <= kth);
        unsigned slot = wave_append_slot(ok, ccnt);
        if (ok) keys[slot] = mine[t];
    }
    __syncthreads();
    return kth;
}

// 16-byte streaming load: the codes are read once per query, so they are fetched with the
// non-temporal hint and do not displace the tables and candidate lists from the caches.
typedef unsigned v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 stream_load16(const uint8_t *p)
{
    const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 12-byte streaming load (the address is a multiple of four).
typedef unsigned v3u __attribute__((ext_vector_type(3)));
typedef v3u v3u_a4 __attribute__((aligned(4)));
__device__ __forceinline__ v3u stream_load12(const uint8_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const v3u_a4 *>(p));
}

// How a wavefront shares out its 64 * 48 bytes of 6-bit codes: in groups of whole codes of 12 or
// 24 bytes, group g of lane l being group 64 g + l of the wavefront's bytes, so that one load
// instruction reads consecutive groups.  The thread keeps its groups one after the other: code c of
// the thread starts at byte c * BYTES of its 48 bytes and is code
// (64 (c / CPG) + l) * CPG + c % CPG of the wavefront.
template <int BYTES>
struct SixbitLayout {
    static constexpr int UPG = BYTES > 12 ? BYTES / 12 : 1;   // 12-byte loads per group
    static constexpr int CPG = BYTES > 12 ? 1 : 12 / BYTES;   // codes per group
    static constexpr int GROUPS = 4 / UPG;                    // groups per thread and tile
    static_assert(BYTES == 6 || BYTES == 12 || BYTES == 24, "6-bit codes of 8, 16 or 32 components");
    // index of code c of thread `tid` inside the tile
    static __device__ __forceinline__ unsigned slot(int tid, int c)
    {
        constexpr int CPT = 48 / BYTES;
        return (unsigned)((tid & ~(WAVE - 1)) * CPT + ((c / CPG) * WAVE + (tid & (WAVE - 1))) * CPG + c % CPG);
    }
};

// The two 16-byte loads of one thread for the tile starting at code t0 (6-bit components: its
// four groups, as three vectors).  FULL: the whole
// tile lies inside the database (t0 + TILE <= c1), no bounds to check.
template <int B, int NT, bool FULL = false>
__device__ __forceinline__ void tile_load(const uint8_t *__restrict__ codes, int64_t t0, int64_t c1,
                                          uint4 (&w)[ScanCfg<B, NT>::NVEC], int (&nc)[2])
{
    const int tid = threadIdx.x;
    if constexpr (ScanCfg<B, NT>::SIX) {
        // 6-bit components: four groups of 12 or 24 bytes per thread (sixbit_layout); nc[0] = bit c
        // set when code c of the thread lies inside the database
        using C = ScanCfg<B, NT>;
        using L = SixbitLayout<C::BYTES>;
        const int64_t wave0 = t0 + (int64_t)(tid & ~(WAVE - 1)) * C::CPT;  // first code of the wavefront
        const int lane = tid & (WAVE - 1);
        unsigned d[12];
        nc[0] = 0;
        nc[1] = 0;
#pragma unroll
        for (int g = 0; g < L::GROUPS; ++g) {
            const int64_t first = wave0 + (int64_t)(g * WAVE + lane) * L::CPG;  // first code of the group
            const uint8_t *p = codes + first * C::BYTES;
            if (FULL || first + L::CPG <= c1) {
#pragma unroll
                for (int u = 0; u < L::UPG; ++u) {
                    const v3u v = stream_load12(p + 12 * u);
                    d[(g * L::UPG + u) * 3] = v.x;
                    d[(g * L::UPG + u) * 3 + 1] = v.y;
                    d[(g * L::UPG + u) * 3 + 2] = v.z;
                }
                nc[0] |= ((1 << L::CPG) - 1) << (g * L::CPG);
            } else {  // ragged end of the database: byte loads, no read past the end
                const int have = first < c1 ? (int)(c1 - first) : 0;
                unsigned tmp[3 * L::UPG];
#pragma unroll
                for (int k = 0; k < 3 * L::UPG; ++k) tmp[k] = 0;
                for (int k = 0; k < have * C::BYTES; ++k) tmp[k >> 2] |= (unsigned)p[k] << (8 * (k & 3));
#pragma unroll
                for (int k = 0; k < 3 * L::UPG; ++k) d[g * L::UPG * 3 + k] = tmp[k];
                nc[0] |= ((1 << have) - 1) << (g * L::CPG);
            }
        }
#pragma unroll
        for (int v = 0; v < 3; ++v) w[v] = make_uint4(d[4 * v], d[4 * v + 1], d[4 * v + 2], d[4 * v + 3]);
    } else if constexpr (FULL) {
        if constexpr (B <= 16) {
            constexpr int CPV = 16 / B;
#pragma unroll
            for (int v = 0; v < 2; ++v) {
                w[v] = stream_load16(codes + (t0 + ((int64_t)v * NT + tid) * CPV) * B);
                nc[v] = CPV;
            }
        } else {
            w[0] = stream_load16(codes + (t0 + tid) * B);
            w[1] = stream_load16(codes + (t0 + tid) * B + 16);
            nc[0] = 1;
            nc[1] = 0;
        }
    } else if constexpr (B <= 16) {
        constexpr int CPV = 16 / B;
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            const int64_t base = t0 + ((int64_t)v * NT + tid) * CPV;
            w[v] = make_uint4(0, 0, 0, 0);
            nc[v] = 0;
            if (base + CPV <= c1) {
                w[v] = stream_load16(codes + base * B);
                nc[v] = CPV;
            } else if (base < c1) {  // ragged end of the database: byte loads, no read past the end
                nc[v] = (int)(c1 - base);
                unsigned tmp[4] = {0, 0, 0, 0};
                for (int k = 0; k < nc[v] * B; ++k)
                    tmp[k >> 2] |= (unsigned)codes[base * B + k] << (8 * (k & 3));
                w[v] = make_uint4(tmp[0], tmp[1], tmp[2], tmp[3]);
            }
        }
    } else {
        const int64_t i = t0 + tid;
        w[0] = w[1] = make_uint4(0, 0, 0, 0);
        nc[0] = nc[1] = 0;
        if (i < c1) {
            w[0] = stream_load16(codes + i * B);
            w[1] = stream_load16(codes + i * B + 16);
            nc[0] = 1;
        }
    }
}

// One pair-table entry, known to the compiler as a byte value.
// Order-preserving map float -> unsigned (any sign), and back.
__device__ __forceinline__ unsigned f2ord(float f)
{
    const unsigned b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float ord2f(unsigned o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}


// ---------------------------------------------------------------- merge

constexpr int MERGE_NT = 1024;
constexpr int MERGE_CAP = 6144;   // keys staged in LDS
constexpr int MERGE_WG_PER_THREAD = 8;
constexpr int MERGE_FLAT_G = 256;        // regions and ...
constexpr int MERGE_FLAT_SLOTS = 32768;  // ... key slots up to which every slot is visited

// R best of the keys reported by the G workgroups of each query (64-bit keys
// dist << 32 | index, at most R per workgroup), ordered; then everything the call wrote
// in the workspace is cleared.  KBYTES = significant key bytes (5 for u8 distances).
// DistT = uint8_t: the distance is the key's bits 32..39; float: bits 32..63 (ordered image).
//
// Usual case (a few hundred to a few thousand keys in all): the keys are gathered in LDS; one
// histogram pass over the eight most significant bits in which they differ at all finds the
// bin of the R-th key; the keys up to that bin are ranked against each other by counting,
// which selects and orders in one step.  Massive ties fall back to the full radix select.
// Two report regions may exist per query: region B (G workgroups, up to R keys each) written
// by the single-query kernels, and region A (GA workgroups, up to pitchA keys each) written
// by the query-tiled kernel.  flags[q]: 0 = region A holds the result of query q; 1 = region A is
// incomplete and region B holds the result; 2 = the result is spread over both regions (the lists
// of an inverted index scanned partly by one kernel, partly by the other).  Without flags only
// region B exists.
template <typename DistT, int KBYTES>
__global__ __launch_bounds__(MERGE_NT) void merge_topk_kernel(
    char *__restrict__ ws, size_t ws_stride, size_t counts_off, size_t lists_off, int G,
    unsigned need, int R, DistT pad_dist, uint32_t *__restrict__ out_idx,
    DistT *__restrict__ out_dist, size_t countsA_off, size_t listsA_off, int GA, int pitchA,
    unsigned *__restrict__ flags, const uint32_t *__restrict__ ids, int64_t n_ids)
{
    // need = min(R, number of codes scanned): at least that many keys were reported.
    // ids: the keys' low words are storage positions and out_idx gets ids[position] (inverted index).
    __shared__ uint64_t lkeys[MERGE_CAP];
    __shared__ uint64_t cand[MERGE_NT];
    __shared__ SelectScratch sc;
    __shared__ unsigned lcnt, ccnt;
    __shared__ unsigned long long all_or, all_and;
    __shared__ unsigned fcnt[MERGE_FLAT_G];

    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
    unsigned *counts = reinterpret_cast<unsigned *>(ws + (size_t)q * ws_stride + counts_off);
    uint64_t *lists = reinterpret_cast<uint64_t *>(ws + (size_t)q * ws_stride + lists_off);
    int pitch = R;
    const unsigned flag = flags ? flags[q] : 1u;  // uniform
    const bool redone = flags && flag == 1u;
    const bool both = flag == 2u;
    unsigned *countsA = reinterpret_cast<unsigned *>(ws + (size_t)q * ws_stride + countsA_off);
    uint64_t *listsA = reinterpret_cast<uint64_t *>(ws + (size_t)q * ws_stride + listsA_off);
    if (flag == 0u) {                             // the tiled kernel's report is the result
        counts = reinterpret_cast<unsigned *>(ws + (size_t)q * ws_stride + countsA_off);
        lists = reinterpret_cast<uint64_t *>(ws + (size_t)q * ws_stride + listsA_off);
        G = GA;
        pitch = pitchA;
    }
    // Few, well-filled regions (inverted-index scans, short databases): every slot of every
    // region is visited, a slot per thread at a time, so that the loads are spread over the whole
    // workgroup instead of one thread walking each region.
    const bool flat = G <= MERGE_FLAT_G && (size_t)G * pitch <= (size_t)MERGE_FLAT_SLOTS;  // uniform
    // every reported key, spread over the threads by workgroup (after the gather below)
    auto each_key = [&](auto f) {
        if (flat) {
            for (unsigned sidx = tid; sidx < (unsigned)G * pitch; sidx += MERGE_NT) {
                const unsigned g = sidx / (unsigned)pitch, i = sidx - g * (unsigned)pitch;
                if (i < fcnt[g]) f(lists[sidx]);
            }
        }
        for (int g = tid; g < G && !flat; g += MERGE_NT) {
            const unsigned c = min(counts[g], (unsigned)pitch);
            const uint64_t *l = lists + (size_t)g * pitch;
            for (unsigned i = 0; i < c; i += 8) {  // eight loads in flight before the first use
                uint64_t k[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) k[u] = (i + u < c) ? l[i + u] : 0;
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (i + u < c) f(k[u]);
            }
        }
        if (both) {
            for (int g = 0; g < GA; ++g) {
                const unsigned c = min(countsA[g], (unsigned)pitchA);
                for (unsigned i = tid; i < c; i += MERGE_NT) f(listsA[(size_t)g * pitchA + i]);
            }
        }
    };

    auto index_of = [&](uint32_t pos) -> uint32_t {
        if (!ids) return pos;
        return ((int64_t)pos < n_ids) ? ids[pos] : 0xffffffffu;
    };

    // Gather, region by region.
    if (tid == 0) { lcnt = 0; ccnt = 0; all_or = 0ull; all_and = ~0ull; }
    for (int i = tid; i < 256; i += MERGE_NT) sc.hist[i] = 0;
    __syncthreads();
    // Histogram bits.  Integer distances: the distance byte itself, counted while gathering.
    // Float distances: the eight most significant bits in which the keys differ at all (the
    // bits above them agree), found from the OR and the AND of all keys, counted afterwards.
    constexpr bool ADAPT = sizeof(DistT) != 1;
    unsigned long long my_or = 0ull, my_and = ~0ull;
    auto take = [&](uint64_t k) {
        const unsigned slot = atomicAdd(&lcnt, 1u);
        if (slot < (unsigned)MERGE_CAP) lkeys[slot] = k;
        if constexpr (ADAPT) {
            my_or |= k;
            my_and &= k;
        } else {
            atomicAdd(&sc.hist[(unsigned)(k >> 32) & 255u], 1u);
        }
    };
    unsigned mycnt[MERGE_WG_PER_THREAD];
    if (flat) {
        for (int g = tid; g < G; g += MERGE_NT) fcnt[g] = min(counts[g], (unsigned)pitch);
        __syncthreads();
        for (unsigned sidx = tid; sidx < (unsigned)G * pitch; sidx += MERGE_NT) {
            const unsigned g = sidx / (unsigned)pitch, i = sidx - g * (unsigned)pitch;
            if (i < fcnt[g]) take(lists[sidx]);
        }
    } else {
#pragma unroll
        for (int t = 0; t < MERGE_WG_PER_THREAD; ++t) {
            const int g = tid + t * MERGE_NT;
            mycnt[t] = 0;
            if (g < G) {
                // count and first key fetched together: most regions hold zero or one key
                const unsigned c = min(counts[g], (unsigned)pitch);
                const uint64_t *l = lists + (size_t)g * pitch;
                const uint64_t k0 = l[0];
                mycnt[t] = c;
                if (c) take(k0);
                for (unsigned i = 1; i < c; i += 4) {  // four loads in flight
                    uint64_t k[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) k[u] = (i + u < c) ? l[i + u] : 0;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i + u < c) take(k[u]);
                }
            }
        }
        for (int g = tid + MERGE_WG_PER_THREAD * MERGE_NT; g < G; g += MERGE_NT) {  // very wide grids
            const unsigned c = min(counts[g], (unsigned)pitch);
            for (unsigned i = 0; i < c; ++i) take(lists[(size_t)g * pitch + i]);
        }
    }
    if (both) {  // region A on top of region B (few regions, spread over the whole workgroup)
        for (int g = 0; g < GA; ++g) {
            const unsigned c = min(countsA[g], (unsigned)pitchA);
            for (unsigned i = tid; i < c; i += MERGE_NT) take(listsA[(size_t)g * pitchA + i]);
        }
    }
    if constexpr (ADAPT) {
        if (my_or != 0ull || my_and != ~0ull) {
            atomicOr(&all_or, my_or);
            atomicAnd(&all_and, my_and);
        }
    }
    __syncthreads();
    unsigned total = lcnt;
    need = min(need, total);
    bool in_lds = total <= (unsigned)MERGE_CAP;
    if constexpr (!ADAPT) {
        // More keys than LDS holds (loose bounds, many regions): the histogram counted all of them, so
        // the bin of the need-th key is known, and only the keys up to that bin are gathered again.
        if (!in_lds && need > 0) {  // uniform
            select_bin(&sc, need);
            __syncthreads();
            const unsigned bin = sc.bin;
            const unsigned upto = need - sc.need + sc.hist[bin];  // keys in the bins up to `bin`
            __syncthreads();
            if (upto <= (unsigned)MERGE_CAP) {
                if (tid == 0) lcnt = 0;
                __syncthreads();
                each_key([&](uint64_t k) {
                    if (((unsigned)(k >> 32) & 255u) <= bin) lkeys[atomicAdd(&lcnt, 1u)] = k;
                });
                __syncthreads();
                total = upto;
                in_lds = true;
            }
        }
    }
    int TOP = 32;
    if constexpr (ADAPT) {
        const unsigned long long diff = all_or ^ all_and;
        const int top = diff ? 63 - __clzll((long long)diff) : 7;
        TOP = top > 7 ? top - 7 : 0;
        if (in_lds)
            for (unsigned i = tid; i < total; i += MERGE_NT)
                atomicAdd(&sc.hist[(unsigned)(lkeys[i] >> TOP) & 255u], 1u);
        __syncthreads();
    }

    bool done = false;
    if (need > 0 && in_lds) {
        // bin of the need-th key by its most significant byte, and the keys up to that bin
        select_bin(&sc, need);
        __syncthreads();
        const unsigned bin = sc.bin;
        for (unsigned i = tid; i < total; i += MERGE_NT) {
            const uint64_t k = lkeys[i];
            if (((unsigned)(k >> TOP) & 255u) <= bin) {
                const unsigned slot = atomicAdd(&ccnt, 1u);
                if (slot < (unsigned)MERGE_NT) cand[slot] = k;
            }
        }
        __syncthreads();
        const unsigned nc = ccnt;
        if (nc <= (unsigned)MERGE_NT) {  // uniform: rank the candidates against each other
            if ((unsigned)tid < nc) {
                const uint64_t k = cand[tid];
                unsigned rank = 0;
                for (unsigned j = 0; j < nc; ++j) rank += (cand[j] < k) ? 1u : 0u;
                if (rank < need) {
                    DistT d;
                    if constexpr (sizeof(DistT) == 1) d = (DistT)((k >> 32) & 0xff);
                    else d = ord2f((unsigned)(k >> 32));
                    out_idx[(size_t)q * R + rank] = index_of((uint32_t)k);
                    out_dist[(size_t)q * R + rank] = d;
                }
            }
            done = true;
        }
        __syncthreads();
    }

    if (need > 0 && !done) {
        // full radix select, then order the winners by rank
        uint64_t kth;
        if (in_lds) kth = block_radix_select<uint64_t, KBYTES>(lkeys, total, need, &sc);
        else kth = block_radix_select_each<uint64_t, KBYTES>(each_key, need, &sc);
        __syncthreads();
        uint64_t mine[MERGE_CAP / MERGE_NT];
        if (in_lds) {
#pragma unroll
            for (int t = 0; t < MERGE_CAP / MERGE_NT; ++t) {
                const unsigned i = tid + t * MERGE_NT;
                mine[t] = (i < total) ? lkeys[i] : ~0ull;
            }
        }
        if (tid == 0) lcnt = 0;
        __syncthreads();
        if (in_lds) {
#pragma unroll
            for (int t = 0; t < MERGE_CAP / MERGE_NT; ++t) {
                const unsigned i = tid + t * MERGE_NT;
                const bool ok = (i < total) && mine[t] <= kth;
                const unsigned slot = wave_append_slot(ok, &lcnt);
                if (ok) lkeys[slot] = mine[t];
            }
        } else {
            each_key([&](uint64_t k) {
                if (k <= kth) lkeys[atomicAdd(&lcnt, 1u)] = k;  // exactly `need` keys: they are unique
            });
        }
        __syncthreads();
        for (unsigned i = tid; i < need; i += MERGE_NT) {
            const uint64_t k = lkeys[i];
            unsigned rank = 0;
            for (unsigned j = 0; j < need; ++j) rank += (lkeys[j] < k) ? 1u : 0u;
            DistT d;
            if constexpr (sizeof(DistT) == 1) d = (DistT)((k >> 32) & 0xff);
            else d = ord2f((unsigned)(k >> 32));
            out_idx[(size_t)q * R + rank] = index_of((uint32_t)k);
            out_dist[(size_t)q * R + rank] = d;
        }
    }
    for (unsigned i = need + tid; i < (unsigned)R; i += MERGE_NT) {
        out_idx[(size_t)q * R + i] = 0xffffffffu;
        out_dist[(size_t)q * R + i] = pad_dist;
    }

    // Leave every word this call wrote in the workspace zero again, so that the next call
    // finds clean control blocks wherever its own layout puts them.
    if (flat) {
        for (unsigned sidx = tid; sidx < (unsigned)G * pitch; sidx += MERGE_NT) {
            const unsigned g = sidx / (unsigned)pitch, i = sidx - g * (unsigned)pitch;
            if (i < fcnt[g]) lists[sidx] = 0;
        }
        for (int g = tid; g < G; g += MERGE_NT)
            if (fcnt[g]) counts[g] = 0;
    } else {
#pragma unroll
        for (int t = 0; t < MERGE_WG_PER_THREAD; ++t) {
            const int g = tid + t * MERGE_NT;
            if (g < G && mycnt[t]) {
                for (unsigned i = 0; i < mycnt[t]; ++i) lists[(size_t)g * pitch + i] = 0;
                counts[g] = 0;
            }
        }
        for (int g = tid + MERGE_WG_PER_THREAD * MERGE_NT; g < G; g += MERGE_NT) {
            const unsigned c = min(counts[g], (unsigned)pitch);
            for (unsigned i = 0; i < c; ++i) lists[(size_t)g * pitch + i] = 0;
            if (c) counts[g] = 0;
        }
    }
    if (redone || both) {  // the abandoned report of the tiled kernel, or the second half of the result
        __syncthreads();  // (both: every thread is done reading region A)
        for (int g = 0; g < GA; ++g) {
            const unsigned c = min(countsA[g], (unsigned)pitchA);
            for (unsigned i = tid; i < c; i += MERGE_NT) listsA[(size_t)g * pitchA + i] = 0;
        }
        __syncthreads();
        for (int g = tid; g < GA; g += MERGE_NT) countsA[g] = 0;
        if (tid == 0) flags[q] = 0;
    }
    unsigned *z = reinterpret_cast<unsigned *>(hdr);
    for (int i = tid; i < (int)(sizeof(ScanHeader) / 4); i += MERGE_NT) z[i] = 0;
}

// One merge workgroup per query.
template <typename DistT, int KBYTES, typename... Args>
inline int launch_merge(int nq, hipStream_t st, Args... args)
{
    launch(QADC_PROF_MERGE, (merge_topk_kernel<DistT, KBYTES>), dim3(nq), dim3(MERGE_NT), 0, st,
           args...);
    return QADC_OK;
}

// Workspace layout of one scan call: per query a ScanHeader, counts[G], lists[G][R].
struct ScanLayout {
    size_t counts_off, lists_off, stride;
};

inline ScanLayout scan_layout(int G, int R)
{
    ScanLayout l;
    l.counts_off = sizeof(ScanHeader);
    l.lists_off = l.counts_off + align_up((size_t)G * sizeof(unsigned), 256);
    l.stride = l.lists_off + align_up((size_t)G * R * sizeof(uint64_t), 256);
    return l;
}

// Queries per launch so that the workspace stays within 256 MiB.
inline int scan_query_batch(size_t stride, int nq)
{
    int64_t qb = (int64_t)((256ull << 20) / stride);
    if (qb < 1) qb = 1;
    if (qb > nq) qb = nq;
    if (qb > 65535) qb = 65535;
    return (int)qb;
}

// Tuning knobs: the QADC_* environment variables.  They change launch shapes and which of the
// equivalent kernels runs, never a result.  An entry point reads them ONCE, when it is called
// (knobs_refresh), into the calling thread's copy; everything below it uses that copy.  -1: not set.
struct Knobs {
    int scan_nt, scan_wgs, seed_min_tiles, seed_wgs, tiled, tiled_seed, scan_f32_wgs;
    int tiled_mfma, mfma_min_q, mfma_min_q2, mfma_min_q4, mfma_waves;
    int ivf_wgs, ivf_seed, ivf_units, ivf_seed_parts, ivf_shared, ivf_shared_wgs, ivf_shared_min_pairs, ivf_seed_probes,
        ivf_wide_q;
};
const Knobs &knobs();
void knobs_refresh();
inline int knob_or(int value, int dflt) { return value >= 0 ? value : dflt; }

}  // namespace qadc
