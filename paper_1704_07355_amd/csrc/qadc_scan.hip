// Scan step + top-R of Quick ADC on gfx950 (Alg. 2 of the paper; Alg. 1 for the
// float variants lives in qadc_scan_f32.hip).
//
// Data flow of one query:
//   codes (HBM, standard layout, streamed once, 16 B per lane per load)
//     -> per code: one LDS lookup per code BYTE in a 256-entry "pair table"
//        ptab[jb][v] = min(cap, q[2jb][v & 15] + q[2jb+1][v >> 4]), summed and
//        clamped once at `cap`.  Entries are non-negative, so this equals the
//        chain of saturating adds of Alg. 2 (mask 0x0f, lookup, add, shift).
//     -> key = sum << 24 | (index inside the workgroup's chunk); keys below the
//        workgroup's running threshold are appended to an LDS candidate list
//        (one atomic per wavefront), which is cut back to its R smallest keys
//        by an exact radix select whenever it fills up.
//     -> every workgroup writes its R best as 64-bit keys sum << 32 | index;
//        a second kernel selects and orders the R best of all of them.
// The total order (sum, index) is carried by the integer keys, so the result
// does not depend on how the grid is cut or on the order waves run in.

#include "qadc_select.h"
#include "qadc_profile.h"

namespace qadc {

constexpr int SCAN_VEC = 2;               // 16-byte loads per thread and tile
constexpr int SCAN_SLACK = QADC_MAX_R;    // candidate slots beyond one tile
constexpr uint64_t PAD_KEY = ~0ull;

template <int B, int NT>
struct ScanCfg {
    static constexpr int CPV = (B <= 16) ? 16 / B : 1;            // codes per thread-load
    static constexpr int CPT = (B <= 16) ? SCAN_VEC * CPV : 1;    // codes per thread and tile
    static constexpr int TILE = NT * CPT;
    static constexpr int CAP = TILE + SCAN_SLACK;
};

struct ScanShared {
    SelectScratch sel;
    unsigned ccnt;     // append counter of a compaction
    unsigned tcnt[3];  // append counters of the tiles, used in rotation
};

__device__ __forceinline__ unsigned byte_of(const uint4 &v, int k)
{
    const unsigned w = (k < 4) ? v.x : (k < 8) ? v.y : (k < 12) ? v.z : v.w;
    return (w >> (8 * (k & 3))) & 0xffu;
}

// Cuts keys[0..cnt) back to its `keep` smallest keys (cnt > keep) and returns
// the largest key kept.  Called by every thread of the workgroup.
template <int NT, int CAP>
__device__ unsigned compact_candidates(unsigned *keys, unsigned cnt, unsigned keep, ScanShared *sh)
{
    const unsigned kth = block_radix_select<unsigned, 4>(keys, cnt, keep, &sh->sel);
    constexpr int PER = (CAP + NT - 1) / NT;
    unsigned mine[PER];
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        unsigned i = threadIdx.x + t * NT;
        mine[t] = (i < cnt) ? keys[i] : 0xffffffffu;
    }
    if (threadIdx.x == 0) sh->ccnt = 0;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < PER; ++t) {
        unsigned i = threadIdx.x + t * NT;
        bool ok = (i < cnt) && (mine[t] <= kth);
        unsigned slot = wave_append_slot(ok, &sh->ccnt);
        if (ok) keys[slot] = mine[t];
    }
    __syncthreads();
    return kth;
}

template <int B, int NT>
__global__ __launch_bounds__(NT) void scan_u8_kernel(
    const uint8_t *__restrict__ codes, int64_t n, const uint8_t *__restrict__ qluts, int cap,
    int R, int64_t chunk, uint64_t *__restrict__ part)
{
    using C = ScanCfg<B, NT>;
    __shared__ __attribute__((aligned(16))) uint8_t ptab[B * 256];
    __shared__ unsigned keys[C::CAP];
    __shared__ ScanShared sh;

    const int tid = threadIdx.x;
    const int q = blockIdx.y;
    const int g = blockIdx.x;
    const int G = gridDim.x;
    const uint8_t *qlut = qluts + (size_t)q * (2 * B) * 16;

    for (int e = tid; e < B * 256; e += NT) {
        const int jb = e >> 8, v = e & 255;
        unsigned s = (unsigned)qlut[(2 * jb) * 16 + (v & 15)] + (unsigned)qlut[(2 * jb + 1) * 16 + (v >> 4)];
        ptab[e] = (uint8_t)min(s, (unsigned)cap);
    }
    if (tid == 0) sh.tcnt[0] = 0;
    __syncthreads();

    const int64_t c0 = (int64_t)g * chunk;
    const int64_t c1 = min(n, c0 + chunk);
    unsigned thr = 0xffffffffu;  // keys >= thr cannot be among the R best of this chunk
    unsigned have = 0;           // candidates in keys[] before the current tile (uniform)
    int rot = 0;

    // One barrier per tile: the tile's appends go through counter tcnt[rot]; after the
    // barrier everybody adds its final value to `have`.  The counter of the next tile
    // is cleared one tile ahead, when no wave can still be reading or bumping it.
    for (int64_t t0 = c0; t0 < c1; t0 += C::TILE) {
        unsigned *ctr = &sh.tcnt[rot];
        const int nxt = (rot == 2) ? 0 : rot + 1;
        if (tid == 0) sh.tcnt[nxt] = 0;
        if constexpr (B <= 16) {
#pragma unroll
            for (int v = 0; v < SCAN_VEC; ++v) {
                const int64_t base = t0 + ((int64_t)v * NT + tid) * C::CPV;
                uint4 w = make_uint4(0, 0, 0, 0);
                int nc = 0;
                if (base + C::CPV <= c1) {
                    w = *reinterpret_cast<const uint4 *>(codes + base * B);
                    nc = C::CPV;
                } else if (base < c1) {
                    nc = (int)(c1 - base);
                    unsigned tmp[4] = {0, 0, 0, 0};
                    for (int k = 0; k < nc * B; ++k)
                        tmp[k >> 2] |= (unsigned)codes[base * B + k] << (8 * (k & 3));
                    w = make_uint4(tmp[0], tmp[1], tmp[2], tmp[3]);
                }
#pragma unroll
                for (int c = 0; c < C::CPV; ++c) {
                    unsigned s = 0;
#pragma unroll
                    for (int jb = 0; jb < B; ++jb) s += ptab[jb * 256 + byte_of(w, c * B + jb)];
                    s = min(s, (unsigned)cap);
                    const unsigned key = (s << 24) | (unsigned)(base + c - c0);
                    const bool pass = (c < nc) && (key < thr);
                    const unsigned slot = have + wave_append_slot(pass, ctr);
                    if (pass) keys[slot] = key;
                }
            }
        } else {  // B == 32: one code per thread and tile, two 16-byte loads
            const int64_t i = t0 + tid;
            bool pass = false;
            unsigned key = 0;
            if (i < c1) {
                const uint4 w0 = *reinterpret_cast<const uint4 *>(codes + i * B);
                const uint4 w1 = *reinterpret_cast<const uint4 *>(codes + i * B + 16);
                unsigned s = 0;
#pragma unroll
                for (int jb = 0; jb < 16; ++jb) s += ptab[jb * 256 + byte_of(w0, jb)];
#pragma unroll
                for (int jb = 0; jb < 16; ++jb) s += ptab[(16 + jb) * 256 + byte_of(w1, jb)];
                s = min(s, (unsigned)cap);
                key = (s << 24) | (unsigned)(i - c0);
                pass = key < thr;
            }
            const unsigned slot = have + wave_append_slot(pass, ctr);
            if (pass) keys[slot] = key;
        }
        __syncthreads();
        have += *ctr;
        rot = nxt;
        if (have > (unsigned)SCAN_SLACK) {  // the next tile might not fit: keep the R best
            thr = compact_candidates<NT, C::CAP>(keys, have, (unsigned)R, &sh);
            have = (unsigned)R;
        }
    }

    unsigned cnt = have;
    if (cnt > (unsigned)R) {
        compact_candidates<NT, C::CAP>(keys, cnt, (unsigned)R, &sh);
        cnt = (unsigned)R;
    }
    uint64_t *dst = part + ((size_t)q * G + g) * R;
    for (int i = tid; i < R; i += NT) {
        uint64_t k = PAD_KEY;
        if ((unsigned)i < cnt) {
            const unsigned key = keys[i];
            k = ((uint64_t)(key >> 24) << 32) | (uint64_t)(c0 + (key & 0xffffffu));
        }
        dst[i] = k;
    }
}

// ---------------------------------------------------------------- merge

constexpr int MERGE_NT = 1024;
constexpr int MERGE_CAP = 4096;

// R best of `total` 64-bit keys (dist << 32 | index; PAD_KEY = absent), ordered.
// DistT = uint8_t: the distance is the key's bits 32..39; float: bits 32..63.
template <typename DistT, int KBYTES>
__global__ __launch_bounds__(MERGE_NT) void merge_topk_kernel(
    const uint64_t *__restrict__ part, unsigned total, unsigned need, int R, DistT pad_dist,
    uint32_t *__restrict__ out_idx, DistT *__restrict__ out_dist)
{
    // need = min(R, number of codes scanned): at least that many real keys are in `part`.
    __shared__ uint64_t lkeys[MERGE_CAP];
    __shared__ SelectScratch sc;
    __shared__ unsigned lcnt;

    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    const uint64_t *src = part + (size_t)q * total;
    constexpr uint64_t KMASK = (KBYTES == 8) ? ~0ull : ((1ull << (8 * (KBYTES & 7))) - 1);
    if (need == 0) {
        for (unsigned i = tid; i < (unsigned)R; i += MERGE_NT) {
            out_idx[(size_t)q * R + i] = 0xffffffffu;
            out_dist[(size_t)q * R + i] = pad_dist;
        }
        return;
    }

    // first pass over the most significant byte: the bin of the R-th key
    for (int i = tid; i < 256; i += MERGE_NT) sc.hist[i] = 0;
    if (tid == 0) lcnt = 0;
    __syncthreads();
    constexpr int TOP = (KBYTES - 1) * 8;
    for (unsigned i = tid; i < total; i += MERGE_NT)
        atomicAdd(&sc.hist[(unsigned)((src[i] & KMASK) >> TOP) & 255u], 1u);
    __syncthreads();
    select_bin(&sc, need);
    __syncthreads();
    const unsigned bin = sc.bin;
    const unsigned upto = (need - sc.need) + sc.hist[bin];  // keys whose top byte <= bin
    __syncthreads();

    uint64_t kth;
    const bool in_lds = upto <= (unsigned)MERGE_CAP;
    if (in_lds) {
        for (unsigned i0 = 0; i0 < total; i0 += MERGE_NT) {
            const unsigned i = i0 + tid;
            uint64_t k = (i < total) ? (src[i] & KMASK) : ~0ull;
            const bool ok = (i < total) && ((unsigned)(k >> TOP) & 255u) <= bin;
            const unsigned slot = wave_append_slot(ok, &lcnt);
            if (ok) lkeys[slot] = k;
        }
        __syncthreads();
        kth = block_radix_select<uint64_t, KBYTES>(lkeys, upto, need, &sc);
    } else {
        kth = block_radix_select<uint64_t, KBYTES>(src, total, need, &sc) & KMASK;
        // PAD_KEY masked to KBYTES still compares above every real key
    }
    __syncthreads();

    // gather the `need` keys <= kth into lkeys[0..need) (reusing the list), then order by rank
    uint64_t mine[MERGE_CAP / MERGE_NT];
    if (in_lds) {
#pragma unroll
        for (int t = 0; t < MERGE_CAP / MERGE_NT; ++t) {
            const unsigned i = tid + t * MERGE_NT;
            mine[t] = (i < upto) ? lkeys[i] : ~0ull;
        }
    }
    if (tid == 0) lcnt = 0;
    __syncthreads();
    if (in_lds) {
#pragma unroll
        for (int t = 0; t < MERGE_CAP / MERGE_NT; ++t) {
            const unsigned i = tid + t * MERGE_NT;
            const bool ok = (i < upto) && mine[t] <= kth;
            const unsigned slot = wave_append_slot(ok, &lcnt);
            if (ok) lkeys[slot] = mine[t];
        }
    } else {
        for (unsigned i0 = 0; i0 < total; i0 += MERGE_NT) {
            const unsigned i = i0 + tid;
            const uint64_t k = (i < total) ? (src[i] & KMASK) : ~0ull;
            const bool ok = (i < total) && k <= kth;
            const unsigned slot = wave_append_slot(ok, &lcnt);
            if (ok) lkeys[slot] = k;
        }
    }
    __syncthreads();

    for (unsigned i = tid; i < (unsigned)R; i += MERGE_NT) {
        if (i >= need) {
            out_idx[(size_t)q * R + i] = 0xffffffffu;
            out_dist[(size_t)q * R + i] = pad_dist;
        } else {
            const uint64_t k = lkeys[i];
            unsigned rank = 0;
            for (unsigned j = 0; j < need; ++j) rank += (lkeys[j] < k) ? 1u : 0u;
            const uint32_t idx = (uint32_t)k;
            DistT d;
            if constexpr (sizeof(DistT) == 1) d = (DistT)((k >> 32) & 0xff);
            else d = __uint_as_float((unsigned)(k >> 32));
            if (idx == 0xffffffffu) d = pad_dist;  // a padding key was selected (fewer than R codes)
            out_idx[(size_t)q * R + rank] = idx;
            out_dist[(size_t)q * R + rank] = d;
        }
    }
}

// ---------------------------------------------------------------- host

struct ScanPlan {
    int B, NT, tile, G, qbatch;
    int64_t chunk;
    size_t ws_bytes;
};

static int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return (s && *s) ? atoi(s) : dflt;
}

static bool make_scan_plan(int variant, int64_t n, int m, int nq, int R, ScanPlan *p)
{
    if (variant != QADC_U8_4BIT) return false;
    if (!(m == 8 || m == 16 || m == 32 || m == 64)) return false;
    if (n < 0 || n > 0xfffffffell || nq < 1 || R < 1 || R > QADC_MAX_R) return false;
    p->B = m / 2;
    p->NT = env_int("QADC_SCAN_NT", 512) == 1024 ? 1024 : 512;
    const int cpt = (p->B <= 16) ? SCAN_VEC * (16 / p->B) : 1;
    p->tile = p->NT * cpt;
    const int64_t tiles = n > 0 ? ceil_div(n, p->tile) : 1;
    int64_t G = env_int("QADC_SCAN_WGS", p->NT == 1024 ? 256 : 512);
    if (G < 1) G = 1;
    if (G > tiles) G = tiles;
    const int64_t max_chunk = ((1ll << 24) - 1) / p->tile * p->tile;
    int64_t chunk = ceil_div(tiles, G) * p->tile;
    if (chunk > max_chunk) chunk = max_chunk;
    p->chunk = chunk;
    p->G = (int)(n > 0 ? ceil_div(n, chunk) : 1);
    const size_t per_query = (size_t)p->G * R * sizeof(uint64_t);
    int64_t qb = (int64_t)((256ull << 20) / per_query);
    if (qb < 1) qb = 1;
    if (qb > nq) qb = nq;
    if (qb > 65535) qb = 65535;
    p->qbatch = (int)qb;
    p->ws_bytes = align_up(per_query * (size_t)qb, 256);
    return true;
}

template <int B, int NT>
static void launch_scan_u8(const ScanPlan &p, const uint8_t *codes, int64_t n, const uint8_t *qluts,
                           int nq, int cap, int R, uint64_t *part, hipStream_t st)
{
    dim3 grid(p.G, nq);
    hipLaunchKernelGGL((scan_u8_kernel<B, NT>), grid, dim3(NT), 0, st, codes, n, qluts, cap, R,
                       p.chunk, part);
}

template <int NT>
static void dispatch_scan_u8(const ScanPlan &p, const uint8_t *codes, int64_t n,
                             const uint8_t *qluts, int nq, int cap, int R, uint64_t *part,
                             hipStream_t st)
{
    switch (p.B) {
    case 4: launch_scan_u8<4, NT>(p, codes, n, qluts, nq, cap, R, part, st); break;
    case 8: launch_scan_u8<8, NT>(p, codes, n, qluts, nq, cap, R, part, st); break;
    case 16: launch_scan_u8<16, NT>(p, codes, n, qluts, nq, cap, R, part, st); break;
    default: launch_scan_u8<32, NT>(p, codes, n, qluts, nq, cap, R, part, st); break;
    }
}

int scan_topk_u8(const uint8_t *codes, int64_t n, int m, const uint8_t *qluts, int nq, int R,
                 int nbins, uint32_t *out_idx, uint8_t *out_dist, void *workspace,
                 size_t workspace_bytes, hipStream_t st)
{
    ScanPlan p;
    if (!make_scan_plan(QADC_U8_4BIT, n, m, nq, R, &p))
        return fail(QADC_EINVAL, "qadc_scan_topk: unsupported n=%lld m=%d nq=%d R=%d",
                    (long long)n, m, nq, R);
    if (nbins < 1 || nbins > 255) return fail(QADC_EINVAL, "qadc_scan_topk: nbins=%d not in 1..255", nbins);
    if (((uintptr_t)codes & 15) != 0) return fail(QADC_EINVAL, "qadc_scan_topk: codes must be 16-byte aligned");
    if (workspace_bytes < p.ws_bytes || !workspace)
        return fail(QADC_ENOMEM, "qadc_scan_topk: workspace %zu < %zu bytes", workspace_bytes, p.ws_bytes);
    uint64_t *part = (uint64_t *)workspace;
    for (int q0 = 0; q0 < nq; q0 += p.qbatch) {
        const int nb = min(p.qbatch, nq - q0);
        const uint8_t *ql = qluts + (size_t)q0 * m * 16;
        prof_begin(QADC_PROF_SCAN, st);
        if (p.NT == 1024) dispatch_scan_u8<1024>(p, codes, n, ql, nb, nbins, R, part, st);
        else dispatch_scan_u8<512>(p, codes, n, ql, nb, nbins, R, part, st);
        prof_end(QADC_PROF_SCAN, st);
        prof_begin(QADC_PROF_MERGE, st);
        hipLaunchKernelGGL((merge_topk_kernel<uint8_t, 5>), dim3(nb), dim3(MERGE_NT), 0, st, part,
                           (unsigned)(p.G * R), (unsigned)min((int64_t)R, n), R, (uint8_t)nbins, out_idx + (size_t)q0 * R,
                           out_dist + (size_t)q0 * R);
        prof_end(QADC_PROF_MERGE, st);
    }
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

size_t scan_topk_u8_workspace(int64_t n, int m, int nq, int R)
{
    ScanPlan p;
    if (!make_scan_plan(QADC_U8_4BIT, n, m, nq, R, &p)) return 0;
    return p.ws_bytes;
}

}  // namespace qadc
