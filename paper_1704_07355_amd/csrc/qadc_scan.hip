// Scan step + top-R of Quick ADC on gfx950 (Alg. 2 of the paper), one query per launch row.
//
// Data flow of one query:
//   codes (HBM, standard layout, streamed once, 16 B per lane per load; workgroup g of G takes
//   tiles g, g+G, ...)
//     -> per code: one LDS lookup per code BYTE in a 256-entry "pair table"
//        ptab[jb][v] = min(cap, q[2jb][v & 15] + q[2jb+1][v >> 4]), summed and clamped once at
//        `cap`.  Entries are non-negative, so this equals the chain of saturating adds of
//        Alg. 2 (mask 0x0f, lookup, add, shift).
//     -> key = sum << 24 | (index among the workgroup's own codes).
//   Selection never stores more than a few hundred keys per workgroup:
//     * a seed step (seed_u8_kernel, or the fused prepare_u8_kernel of qadc_search) scans a
//       sample of tiles spread over the database and adds the lowest bins of each sample
//       tile's sum histogram to a per-query histogram in the workspace; the bin where its
//       running count reaches R bounds the R-th smallest sum of the WHOLE database;
//     * the scan kernel reads that bound once and keeps only keys at or below it in an LDS
//       list (one LDS atomic per wavefront with a hit, no barrier in the streaming loop);
//     * without a bound (small databases), or should the list overflow (adversarial order,
//       massive ties), the workgroup runs a careful pass: one barrier per tile, a bound from
//       its own first tile, the list cut back to its R smallest keys by an exact radix select
//       whenever it fills -- so the result never depends on a bound being good, only the
//       speed does.
//   merge_topk_kernel (one workgroup per query) orders the R smallest of the reported keys
//   (sum << 32 | index) and clears whatever the call wrote in the workspace.
// The total order (sum, index) is carried by the integer keys, so the result does not depend
// on how the grid is cut or on the order waves run in.

#include "qadc_scan_common.h"
#include <algorithm>

#include "qadc_scan_u8.h"
#include "qadc_scan_tiled.h"

namespace qadc {

// Seed kernel: a sample of the database (`tiles_per_wg` tiles per workgroup, all tiles spread
// evenly) is scanned and histogrammed by sum.  Each workgroup adds the counts of its lowest
// bins (its best `flush_need` codes, never beyond its own R-th) to the query's grid-wide
// histogram.  The bin where that histogram's running count reaches R bounds the R-th
// smallest sum of the whole database from above: the scan kernel only keeps keys at or
// below it.
template <int B>
__global__ __launch_bounds__(1024) void seed_u8_kernel(
    const uint8_t *__restrict__ codes, int64_t n, const uint8_t *__restrict__ qluts, int cap_i,
    int R, unsigned flush_need, int64_t seed_stride, int tiles_per_wg, char *__restrict__ ws,
    size_t ws_stride, int wide)
{
    constexpr int NT = 1024;
    using C = ScanCfg<B, NT>;
    __shared__ __attribute__((aligned(16))) uint8_t ptab[C::TAB_BYTES];
    __shared__ unsigned hist[256];

    const int tid = threadIdx.x;
    const int q = blockIdx.y;
    const int g = blockIdx.x;
    const unsigned cap = (unsigned)cap_i;
    int64_t c0 = (int64_t)g * tiles_per_wg * seed_stride;
    if (c0 >= n) return;

    uint4 w[C::NVEC];
    int nc[2];
    tile_load<B, NT>(codes, c0, min(n, c0 + C::TILE), w, nc);
    build_pair_tables<B, NT>(qluts + (size_t)q * (C::SIX || wide ? C::TAB_BYTES : 2 * B * 16), cap, ptab, wide != 0);
    for (int e = tid; e < 256; e += NT) hist[e] = 0;
    __syncthreads();

    if (g == 0) {  // the scan kernel takes the pair tables from here instead of rebuilding them
        ScanHeader *hdr0 = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
        for (int e = tid; e < C::TAB_BYTES / 4; e += NT)
            reinterpret_cast<unsigned *>(hdr0->ptab)[e] = reinterpret_cast<const unsigned *>(ptab)[e];
    }
    for (int t = 0; t < tiles_per_wg && c0 < n; ++t, c0 += seed_stride) {  // uniform
        // the next sample tile is requested before this one is used
        uint4 wn[C::NVEC];
#pragma unroll
        for (int v = 0; v < C::NVEC; ++v) wn[v] = w[v];
        int ncn[2] = {nc[0], nc[1]};
        const int64_t c1 = c0 + seed_stride;
        if (t + 1 < tiles_per_wg && c1 < n) tile_load<B, NT>(codes, c1, min(n, c1 + C::TILE), wn, ncn);
        unsigned k[C::CPT];
        tile_keys<B, NT>(w, nc, 0u, ptab, cap, k);
#pragma unroll
        for (int c = 0; c < C::CPT; ++c)
            if ((k[c] >> 24) < cap) atomicAdd(&hist[k[c] >> 24], 1u);  // NO_KEY has sum 255 >= cap
#pragma unroll
        for (int v = 0; v < C::NVEC; ++v) w[v] = wn[v];
        nc[0] = ncn[0]; nc[1] = ncn[1];
    }
    __syncthreads();
    if (tid < WAVE) {
        unsigned h[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) h[b] = hist[4 * tid + b];
        const unsigned f = min(wave_threshold_bin<4>(h, (unsigned)R),
                               wave_threshold_bin<4>(h, flush_need));
        ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
        unsigned *ghist = hdr->ghist[g % GH_REP];
        // lane l reports bins l, l+64, ...: the low bins of a workgroup travel as ONE request
        for (unsigned b0 = 0; b0 <= f && b0 < 256u; b0 += WAVE) {  // uniform
            const unsigned bin = b0 + tid;
            const unsigned c = hist[bin];
            if (bin <= f && bin < cap && c)
                __hip_atomic_fetch_add(&ghist[bin], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Prepare kernel of qadc_search: Tables (Eq. (1)), the init scan and the quantizer of
// Section 3.3, the pair tables and the seed sample of the scan, all in one launch.  Every
// workgroup recomputes the query's (tiny) tables for itself -- 16 x d subtractions and
// multiplies and `init` float ADC sums -- so that nothing has to travel between workgroups
// before the sample can be scanned; workgroup 0 writes the tables out.  The arithmetic is
// the one of build_luts_kernel and quantize_luts_kernel, operation for operation.
constexpr int PREP_MAX_D = 2048;
constexpr int PREP_INIT_PER_LANE = 4;  // init codes per lane of the wavefront that selects qmax

template <int B>
__global__ __launch_bounds__(1024) void prepare_u8_kernel(
    const float *__restrict__ codebooks, int d, const float *__restrict__ queries,
    const uint8_t *__restrict__ codes, int64_t n, int n_init, int R, int nbins, int qmin_mode,
    unsigned flush_need, int64_t seed_stride, float *__restrict__ luts_out,
    uint8_t *__restrict__ qluts_out, float *__restrict__ bias_out, float *__restrict__ delta_out,
    float *__restrict__ qmax_out, char *__restrict__ ws, size_t ws_stride)
{
    constexpr int NT = 1024;
    constexpr int M = 2 * B;
    using C = ScanCfg<B, NT>;
    __shared__ double yq[PREP_MAX_D];
    __shared__ float lut[M * 16];
    __shared__ __attribute__((aligned(16))) unsigned cand[QADC_MAX_INIT];
    __shared__ __attribute__((aligned(16))) uint8_t ptab[B * 256];
    __shared__ __attribute__((aligned(16))) uint8_t qlut_s[M * 16];
    __shared__ float bias[M];
    __shared__ SelectScratch sc;
    __shared__ unsigned qmax_ord;
    __shared__ float delta_s;

    const int tid = threadIdx.x;
    const int q = blockIdx.y;
    const int g = blockIdx.x;
    const unsigned cap = (unsigned)nbins;
    const int dsub = d / M;
    const int64_t c0 = (int64_t)g * seed_stride;
    const int64_t c1 = min(n, c0 + C::TILE);

    // Every global load the set-up needs is issued here, before the first wait.  Loads come
    // back in the order they were issued, so the small ones the tables wait for go first: the
    // query, this thread's centroid (one table entry per thread) and init code; the sample
    // tile (32 KiB per workgroup) follows and is in flight during the whole set-up.
    static_assert(PREP_MAX_D <= 2 * NT, "two query components per thread");
    float yv[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) yv[t] = (tid + t * NT < d) ? queries[(size_t)q * d + tid + t * NT] : 0.0f;
    constexpr int DREG = 16;  // sub-space dimensions held in registers
    float cv[DREG];
    const bool cv_regs = dsub <= DREG;  // uniform
    if (cv_regs && tid < M * 16) {
        const float *c = codebooks + (size_t)tid * dsub;
#pragma unroll
        for (int t = 0; t < DREG; ++t) cv[t] = (t < dsub) ? c[t] : 0.0f;
    }
    // init codes: wavefront 0 takes up to 4 per lane (the usual init of a few hundred codes)
    constexpr int IPL = PREP_INIT_PER_LANE;
    const bool small_init = n_init <= WAVE * IPL;  // uniform
    unsigned cw[IPL][B / 4];
    if (small_init && tid < WAVE) {
#pragma unroll
        for (int r = 0; r < IPL; ++r) {
            const int i = tid * IPL + r;
            if (i < n_init) {
                const unsigned *c = reinterpret_cast<const unsigned *>(codes + (size_t)i * B);
#pragma unroll
                for (int k = 0; k < B / 4; ++k) cw[r][k] = c[k];
            }
        }
    }
    asm volatile("" ::: "memory");
    uint4 w[2];
    int nc[2] = {0, 0};
    if (c0 < c1) tile_load<B, NT>(codes, c0, c1, w, nc);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int t = 0; t < 2; ++t)
        if (tid + t * NT < d) yq[tid + t * NT] = (double)yv[t];
    __syncthreads();

    // Tables, Eq. (1): float64 differences and sums, one rounding
    if (tid < M * 16) {
        const int j = tid >> 4;
        const double *y = yq + j * dsub;
        double acc = 0.0;
        if (cv_regs) {
#pragma unroll
            for (int t = 0; t < DREG; ++t) {
                if (t < dsub) {
                    const double df = y[t] - (double)cv[t];
                    acc += df * df;
                }
            }
        } else {
            const float *c = codebooks + (size_t)tid * dsub;
            for (int t = 0; t < dsub; ++t) {
                const double df = y[t] - (double)c[t];
                acc += df * df;
            }
        }
        lut[tid] = (float)acc;
    }
    for (int e = tid; e < 256; e += NT) sc.hist[e] = 0;  // rank counters / histogram, used below
    __syncthreads();

    // qmax: the min(R, n_init)-th smallest float ADC distance (float32, increasing j) of the init codes
    const unsigned need = (unsigned)min(R, n_init);
    if (small_init) {
        // uniform.  Wavefront 0 alone: four distances per lane, a bitonic sort of the 256 values
        // across the wavefront (no workgroup barrier), the need-th smallest read off.
        if (tid < WAVE) {
            unsigned v[IPL];
#pragma unroll
            for (int r = 0; r < IPL; ++r) {
                v[r] = 0xffffffffu;  // slots beyond the init codes sort last
                if (tid * IPL + r < n_init) {
                    float acc = 0.0f;
#pragma unroll
                    for (int jb = 0; jb < B; ++jb) {
                        const unsigned comps = (cw[r][jb >> 2] >> (8 * (jb & 3))) & 0xffu;
                        acc = acc + lut[(2 * jb) * 16 + (comps & 15u)];
                        acc = acc + lut[(2 * jb + 1) * 16 + (comps >> 4)];
                    }
                    v[r] = f2ord(acc);
                }
            }
            wave_bitonic_sort4(v);
            const unsigned want = need - 1u;  // element index: lane want / 4, slot want % 4
            const unsigned pick = (want & 3u) == 0u ? v[0] : (want & 3u) == 1u ? v[1] : (want & 3u) == 2u ? v[2] : v[3];
            const unsigned kth = __shfl(pick, (int)(want >> 2));
            if (tid == 0) qmax_ord = kth;
        }
    } else {
        for (int i = tid; i < n_init; i += NT) {
            const uint8_t *c = codes + (size_t)i * B;
            float acc = 0.0f;
            for (int jb = 0; jb < B; ++jb) {
                const unsigned comps = c[jb];
                acc = acc + lut[(2 * jb) * 16 + (comps & 15u)];
                acc = acc + lut[(2 * jb + 1) * 16 + (comps >> 4)];
            }
            cand[i] = f2ord(acc);
        }
        __syncthreads();
        const unsigned kth = block_radix_select<unsigned, 4>(cand, (unsigned)n_init, need, &sc);
        if (tid == 0) qmax_ord = kth;
        __syncthreads();
        for (int e = tid; e < 256; e += NT) sc.hist[e] = 0;
    }

    // quantizer of Section 3.3 (the per-table minima do not wait for qmax: the last wavefront
    // computes them while the first one sorts)
    if (tid >= NT - M) {
        const int j = tid - (NT - M);
        float b = lut[j * 16];
        for (int i = 1; i < 16; ++i) b = fminf(b, lut[j * 16 + i]);
        bias[j] = b;
    }
    __syncthreads();
    if (tid == 0) {
        const float qmax = ord2f(qmax_ord);
        float qmin;
        if (qmin_mode == QADC_QMIN_GLOBAL) {
            qmin = bias[0];
            for (int j = 1; j < M; ++j) qmin = fminf(qmin, bias[j]);
            for (int j = 0; j < M; ++j) bias[j] = qmin;
        } else {
            qmin = 0.0f;
            for (int j = 0; j < M; ++j) qmin = qmin + bias[j];
        }
        float delta = __fdiv_rn(qmax - qmin, (float)nbins);
        if (!(delta > 0.0f)) delta = 1.0f;
        delta_s = delta;
        if (g == 0) {
            if (delta_out) delta_out[q] = delta;
            if (qmax_out) qmax_out[q] = qmax;
        }
    }
    __syncthreads();
    if (tid < M * 16) {
        const float off = fmaxf(0.0f, lut[tid] - bias[tid >> 4]);
        const float t = floorf(__fdiv_rn(off, delta_s));
        const uint8_t qv = (t < (float)nbins) ? (uint8_t)t : (uint8_t)nbins;
        qlut_s[tid] = qv;
        if (g == 0) {
            if (qluts_out) qluts_out[(size_t)q * M * 16 + tid] = qv;
            if (luts_out) luts_out[(size_t)q * M * 16 + tid] = lut[tid];
            if (bias_out && (tid & 15) == 0) bias_out[(size_t)q * M + (tid >> 4)] = bias[tid >> 4];
        }
    }
    __syncthreads();

    // pair tables, handed to the scan kernel by workgroup 0
    for (int e = tid; e < B * 256; e += NT) {
        const int jb = e >> 8, v = e & 255;
        const unsigned s = (unsigned)qlut_s[(2 * jb) * 16 + (v & 15)] +
                           (unsigned)qlut_s[(2 * jb + 1) * 16 + (v >> 4)];
        ptab[e] = (uint8_t)min(s, cap);
    }
    __syncthreads();
    ScanHeader *hdr = reinterpret_cast<ScanHeader *>(ws + (size_t)q * ws_stride);
    if (g == 0)
        for (int e = tid; e < B * 64; e += NT)
            reinterpret_cast<unsigned *>(hdr->ptab)[e] = reinterpret_cast<const unsigned *>(ptab)[e];
    if (c0 >= c1) return;  // uniform: no sample tile for this workgroup

    // seed sample, as in seed_u8_kernel
    unsigned k[C::CPT];
    tile_keys<B, NT>(w, nc, 0u, ptab, cap, k);
#pragma unroll
    for (int c = 0; c < C::CPT; ++c)
        if ((k[c] >> 24) < cap) atomicAdd(&sc.hist[k[c] >> 24], 1u);
    __syncthreads();
    if (tid < WAVE) {
        unsigned h[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) h[b] = sc.hist[4 * tid + b];
        const unsigned f = min(wave_threshold_bin<4>(h, (unsigned)R),
                               wave_threshold_bin<4>(h, flush_need));
        unsigned *ghist = hdr->ghist[g % GH_REP];
        for (unsigned b0 = 0; b0 <= f && b0 < 256u; b0 += WAVE) {  // uniform
            const unsigned bin = b0 + tid;
            const unsigned c = sc.hist[bin];
            if (bin <= f && bin < cap && c)
                __hip_atomic_fetch_add(&ghist[bin], c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Scan kernel.  The database is cut into tiles of TILE codes; workgroup g of G takes tiles
// g, g+G, g+2G, ... so that at any moment the grid reads one contiguous window of HBM.
// A candidate key is sum << 24 | (it * TILE + offset in tile), `it` counting the workgroup's
// own tiles: inside a workgroup that order is the order of the global indices.
//
// With a grid-wide bound from the seed kernel the pass is barrier-free: keys at or below
// the bound (a handful per workgroup) are appended to the LDS list with one atomic per
// wavefront.  If the list ever overflows, or when there is no bound (small databases),
// the workgroup runs the careful pass instead: one barrier per tile, the first tile
// histogrammed for a bound of its own, the list cut back to its R smallest keys by an exact
// radix select whenever it fills up -- so the result never depends on the bound being
// good, only the speed does.
template <int B, int NT>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(B >= SIXBIT ? 4 : 8))) void scan_u8_kernel(
    const uint8_t *__restrict__ codes, int64_t n, const uint8_t *__restrict__ qluts, int cap_i,
    int R, int mode, char *__restrict__ ws, size_t ws_stride, size_t counts_off,
    size_t lists_off, const unsigned *__restrict__ redo_flags)
{
    using C = ScanCfg<B, NT>;
    const int has_seed = mode & 1;   // the seed kernel ran: bound and pair tables are in the control block
    const bool wide = (mode & 2) != 0;  // 8-bit components: qluts holds one 256-entry table per byte
    __shared__ __attribute__((aligned(16))) uint8_t ptab[C::TAB_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t qlut_s[C::SIX ? 16 : 2 * B * 16];
    __shared__ unsigned keys[C::CAP];
    __shared__ ScanShared sh;

    const int tid = threadIdx.x;
    const int q = blockIdx.y;
    const int g = blockIdx.x;
    const int64_t G = gridDim.x;
    const unsigned cap = (unsigned)cap_i;
    const ScanHeader *hdr = reinterpret_cast<const ScanHeader *>(ws + (size_t)q * ws_stride);
    if ((int64_t)g * C::TILE >= n) return;  // uniform: no tile for this workgroup
    if (redo_flags && redo_flags[q] == 0) return;  // uniform: only the queries the tiled scan gave up on

    // Loads are returned in the order they were issued: the small ones the set-up waits for
    // (the seed kernel's pair tables and the low half of its histogram) go first, the first
    // tile of codes after them, so that set-up runs while the tile is in flight.
    constexpr int PIECES = C::TAB_BYTES / 16;      // 16-byte pieces of the tables
    constexpr int PPT = (PIECES + NT - 1) / NT;    // ... per thread
    uint4 pt[PPT];
    uint2 gh[GH_REP];
    if (has_seed) {
#pragma unroll
        for (int t = 0; t < PPT; ++t)
            if (tid + t * NT < PIECES) pt[t] = reinterpret_cast<const uint4 *>(hdr->ptab)[tid + t * NT];
        if (tid < WAVE) {
#pragma unroll
            for (int r = 0; r < GH_REP; ++r) gh[r] = *reinterpret_cast<const uint2 *>(&hdr->ghist[r][2 * tid]);
        }
        asm volatile("" ::: "memory");
    }
    uint4 w[C::NVEC];
    int nc[2];
    tile_load<B, NT>(codes, (int64_t)g * C::TILE, n, w, nc);
    asm volatile("" ::: "memory");

    // The grid-wide bound left by the seed kernel: the bin where the running count of the
    // summed replicas reaches R, or 256.  Pair tables: those of the seed kernel, or built here.
    if (tid < WAVE) {
        unsigned t = 256, carry = 0;
        for (unsigned b0 = 0; b0 < 256 && has_seed; b0 += 128) {  // uniform
            unsigned h[2] = {0, 0};
            if (b0 == 0) {
#pragma unroll
                for (int r = 0; r < GH_REP; ++r) { h[0] += gh[r].x; h[1] += gh[r].y; }
            } else {
#pragma unroll
                for (int r = 0; r < GH_REP; ++r) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(&hdr->ghist[r][b0 + 2u * tid]);
                    h[0] += v.x;
                    h[1] += v.y;
                }
            }
            unsigned tot;
            const unsigned hit = wave_threshold_bin<2>(h, (unsigned)R - carry, &tot);
            if (hit < 128u) { t = b0 + hit; break; }
            carry += tot;  // still below R
        }
        if (tid == 0) { sh.tau = t; sh.fcnt = 0; sh.tcnt[0] = 0; }
    }
    for (int e = tid; e < 256; e += NT) sh.sel.hist[e] = 0;
    if (has_seed) {
#pragma unroll
        for (int t = 0; t < PPT; ++t)
            if (tid + t * NT < PIECES) reinterpret_cast<uint4 *>(ptab)[tid + t * NT] = pt[t];
    } else if (C::SIX || wide) {
        build_pair_tables<B, NT>(qluts + (size_t)q * C::TAB_BYTES, cap, ptab, true);
    } else if constexpr (!C::SIX) {
        const uint8_t *qlut = qluts + (size_t)q * (2 * B) * 16;
        for (int e = tid; e < 2 * B * 4; e += NT)
            reinterpret_cast<unsigned *>(qlut_s)[e] = reinterpret_cast<const unsigned *>(qlut)[e];
        __syncthreads();
        for (int e = tid; e < B * 256; e += NT) {
            const int jb = e >> 8, v = e & 255;
            const unsigned s = (unsigned)qlut_s[(2 * jb) * 16 + (v & 15)] +
                               (unsigned)qlut_s[(2 * jb + 1) * 16 + (v >> 4)];
            ptab[e] = (uint8_t)min(s, cap);
        }
    }
    __syncthreads();

    const bool seeded = sh.tau < 256u;  // uniform
    unsigned lim = seeded ? limit_of_bin(sh.tau) : NO_KEY;  // keys >= lim cannot be among the R best
    unsigned have = 0;  // candidates in keys[] (uniform)
    bool careful = !seeded;

    if (seeded) {
        // Barrier-free pass.  The bound is below the saturation value (the seed histogram only
        // counts unsaturated sums), so a sum that passes needs no clamp; whole tiles are tested
        // with one comparison per thread and the append code runs only in waves with a hit.
        const unsigned tau = sh.tau;
        unsigned rel = 0;
        for (int64_t t0 = (int64_t)g * C::TILE; t0 < n; t0 += G * C::TILE, rel += C::TILE) {
            if (t0 + C::TILE <= n) {  // uniform: a whole tile, no bounds to check
                if (rel) tile_load<B, NT, true>(codes, t0, n, w, nc);
                unsigned sm[C::CPT];
                tile_sums<B, NT>(w, ptab, tau, sm);
                unsigned best = sm[0];
#pragma unroll
                for (int c = 1; c < C::CPT; ++c) best = min(best, sm[c]);
                if (__ballot(best <= tau) != 0ull) {
#pragma unroll
                    for (int c = 0; c < C::CPT; ++c) {
                        const bool pass = sm[c] <= tau;
                        const unsigned slot = wave_append_slot(pass, &sh.fcnt);
                        if (pass && slot < (unsigned)C::CAP)
                            keys[slot] = (sm[c] << 24) | (rel + tile_slot_index<B, NT>(c));
                    }
                }
            } else {
                if (rel) tile_load<B, NT>(codes, t0, n, w, nc);
                unsigned k[C::CPT];
                tile_keys<B, NT>(w, nc, rel, ptab, cap, k);
#pragma unroll
                for (int c = 0; c < C::CPT; ++c) {
                    const bool pass = k[c] < lim;
                    const unsigned slot = wave_append_slot(pass, &sh.fcnt);
                    if (pass && slot < (unsigned)C::CAP) keys[slot] = k[c];
                }
            }
        }
        __syncthreads();
        have = sh.fcnt;
        careful = have > (unsigned)C::CAP;  // keys were dropped: start over, carefully
        if (careful) tile_load<B, NT>(codes, (int64_t)g * C::TILE, n, w, nc);
    }

    if (careful) {
        // One barrier per tile: the tile's appends go through counter tcnt[rot]; after the
        // barrier everybody adds its final value to `have`.  The counter of the next tile
        // is cleared one tile ahead, when no wave can still be reading or bumping it.
        have = 0;
        int rot = 0;
        unsigned rel = 0;
        for (int64_t t0 = (int64_t)g * C::TILE; t0 < n; t0 += G * C::TILE, rel += C::TILE) {
            unsigned *ctr = &sh.tcnt[rot];
            const int nxt = (rot == 2) ? 0 : rot + 1;
            if (tid == 0) sh.tcnt[nxt] = 0;
            if (rel) tile_load<B, NT>(codes, t0, n, w, nc);
            unsigned k[C::CPT];
            tile_keys<B, NT>(w, nc, rel, ptab, cap, k);

            if (rel == 0 && !seeded) {
                // No grid-wide bound: bound the workgroup's share by its own first tile.
                // Histogram of the tile's unsaturated sums -> the bin of its R-th smallest.
#pragma unroll
                for (int c = 0; c < C::CPT; ++c)
                    if ((k[c] >> 24) < cap) atomicAdd(&sh.sel.hist[k[c] >> 24], 1u);
                __syncthreads();
                if (tid < WAVE) {
                    unsigned h[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) h[b] = sh.sel.hist[4 * tid + b];
                    const unsigned t = wave_threshold_bin<4>(h, (unsigned)R);
                    if (tid == 0) sh.tau = min(t, cap);
                }
                __syncthreads();
                lim = limit_of_bin(sh.tau);
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
            if (have > (unsigned)SCAN_SLACK) {  // the next tile might not fit: keep the R best
                const unsigned kth = compact_candidates<unsigned, 4, NT, C::CAP>(keys, have, (unsigned)R, &sh.sel, &sh.ccnt);
                lim = min(lim, kth + 1u);  // keys are unique: later ones must be below the R-th kept
                have = (unsigned)R;
            }
        }
    }

    if (have > (unsigned)R) {
        compact_candidates<unsigned, 4, NT, C::CAP>(keys, have, (unsigned)R, &sh.sel, &sh.ccnt);
        have = (unsigned)R;
    }
    if (have == 0) return;  // counts[g] stays zero
    unsigned *counts = reinterpret_cast<unsigned *>(ws + (size_t)q * ws_stride + counts_off);
    uint64_t *dst = reinterpret_cast<uint64_t *>(ws + (size_t)q * ws_stride + lists_off) + (size_t)g * R;
    if (tid == 0) counts[g] = have;
    for (unsigned i = tid; i < have; i += NT) {
        const unsigned key = keys[i];
        const uint64_t rel = key & 0xffffffu;
        const uint64_t idx = ((rel / C::TILE) * (uint64_t)G + (uint64_t)g) * C::TILE + rel % C::TILE;
        dst[i] = ((uint64_t)(key >> 24) << 32) | idx;
    }
}

// ---------------------------------------------------------------- host

struct ScanPlan {
    int B, NT, G, qbatch;
    bool wide;            // 8-bit components (QADC_U8_8BIT): a code byte is one component
    bool tiled;           // batches go through the query-tiled kernel
    TiledPlan t;
    size_t countsA_off, listsA_off, taus_off, flags_off;
    int64_t chunk;
    int seed_wgs;         // 0: no seed kernel
    int64_t seed_stride;  // codes between the sampled tiles
    unsigned flush_need;
    size_t counts_off, lists_off, stride, ws_bytes;
};

static bool make_scan_plan(int variant, int64_t n, int m, int nq, int R, ScanPlan *p)
{
    if (variant != QADC_U8_4BIT && variant != QADC_U8_8BIT && variant != QADC_U8_6BIT) return false;
    p->wide = variant == QADC_U8_8BIT;
    const bool six = variant == QADC_U8_6BIT;  // 6-bit components: B = SIXBIT + m, a thread takes 48 bytes per tile
    if (p->wide) m *= 2;  // bytes per code = m / 2 below
    if (!(m == 8 || m == 16 || m == 32 || (m == 64 && !six))) return false;
    if (n < 0 || n > 0xfffffffell || nq < 1 || R < 1 || R > QADC_MAX_R) return false;
    p->B = six ? SIXBIT + m : m / 2;
    const int nt = knob_or(knobs().scan_nt, 256);
    p->NT = (nt == 1024 || nt == 512) ? nt : 256;
    const int cpt = six ? 64 / m : (p->B <= 16) ? SCAN_VEC * (16 / p->B) : 1;
    const int tile = p->NT * cpt;
    const int64_t tiles = n > 0 ? ceil_div(n, tile) : 1;
    // every workgroup takes tiles g, g+G, ...; its tiles must number below 2^24 / tile, the
    // range of the index bits of a candidate key
    int64_t G = knob_or(knobs().scan_wgs, 2048);
    if (G < 1) G = 1;
    if (G > tiles) G = tiles;
    const int64_t max_tiles_per_wg = ((1ll << 24) - 1) / tile;
    if (ceil_div(tiles, G) > max_tiles_per_wg) G = ceil_div(tiles, max_tiles_per_wg);
    p->G = (int)G;
    p->chunk = 0;
    // Seed kernel: worth its launch once the database is many tiles long.  It samples up to
    // SEED_WGS tiles of 1024-thread workgroups, spread evenly; each reports a few times its
    // share of R codes to the grid-wide histogram.
    const int seed_tile = 1024 * cpt;
    const int64_t seed_tiles = n / seed_tile;
    p->seed_wgs = 0;
    p->seed_stride = 0;
    p->flush_need = 16;
    if (seed_tiles >= knob_or(knobs().seed_min_tiles, 64)) {
        int64_t S = knob_or(knobs().seed_wgs, 0);
        if (S <= 0) {  // about 1/40 of the database, between 256 and 1024 tiles
            S = seed_tiles / 40;
            if (S < 256) S = 256;
            if (S > 1024) S = 1024;
        }
        if (S > seed_tiles / 4) S = seed_tiles / 4;
        if (S < 1) S = 1;
        p->seed_wgs = (int)S;
        p->seed_stride = (n / S) / 16 * 16;
        int64_t fl = ceil_div(4ll * R, S);
        if (fl < 16) fl = 16;
        if (fl > R) fl = R;
        p->flush_need = (unsigned)fl;
    }
    p->tiled = !six && p->seed_wgs > 0 && nq >= TILED_MIN_Q && knob_or(knobs().tiled, 1) != 0 &&
               make_tiled_plan(n, m, nq, !p->wide, &p->t);
    if (p->tiled && p->G > 256) p->G = 256;  // the single-query kernel only redoes rare queries
    const ScanLayout l = scan_layout(p->G, R);
    p->counts_off = l.counts_off;
    p->lists_off = l.lists_off;
    p->stride = l.stride;
    p->countsA_off = p->listsA_off = p->taus_off = p->flags_off = 0;
    if (p->tiled) {
        p->countsA_off = p->stride;
        p->listsA_off = p->countsA_off + align_up((size_t)p->t.GC * sizeof(unsigned), 256);
        p->stride = p->listsA_off + align_up((size_t)p->t.GC * TILED_LCAP * sizeof(uint64_t), 256);
    }
    p->qbatch = scan_query_batch(p->stride, nq);
    // a call cut into several launches: whole sets of queries per launch (the batched kernels take
    // 16 to 128 queries per workgroup; a launch that ends in a nearly empty set wastes its share)
    if (p->tiled && p->qbatch < nq && p->qbatch >= 128) p->qbatch = p->qbatch / 128 * 128;
    p->ws_bytes = p->stride * (size_t)p->qbatch;
    if (p->tiled) {
        p->taus_off = p->ws_bytes;
        p->flags_off = p->taus_off + align_up((size_t)p->qbatch * sizeof(unsigned), 256);
        p->ws_bytes = p->flags_off + align_up((size_t)p->qbatch * sizeof(unsigned), 256);
    }
    return true;
}

template <int B, int NT>
static void launch_scan_u8(const ScanPlan &p, const uint8_t *codes, int64_t n, const uint8_t *qluts,
                           int nq, int cap, int R, char *ws, const unsigned *redo_flags, hipStream_t st)
{
    dim3 grid(p.G, nq);
    launch(QADC_PROF_SCAN, (scan_u8_kernel<B, NT>), grid, dim3(NT), 0, st, codes, n, qluts, cap, R,
                       (p.seed_wgs > 0 ? 1 : 0) | (p.wide ? 2 : 0), ws, p.stride, p.counts_off, p.lists_off,
                       redo_flags);
}

static int dispatch_seed_u8(const ScanPlan &p, const uint8_t *codes, int64_t n,
                            const uint8_t *qluts, int nq, int cap, int R, char *ws, hipStream_t st)
{
    // batches that the query-tiled kernels scan are sampled in the query-tiled way too
    if (p.tiled && nq >= TILED_MIN_Q && knob_or(knobs().tiled_seed, 1) != 0) {
        const int cpt = (p.B <= 16) ? SCAN_VEC * (16 / p.B) : 1;
        // (at most 512 sample tiles unless QADC_SEED_WGS says otherwise: N = 1e8, m = 32, 256 queries: 1024
        // tiles 0.42 ms of sampling, 512 tiles 0.22 ms and 0.07 ms more in the scan, 256 tiles 0.12 and 0.21)
        const int tiles = knobs().seed_wgs > 0 ? p.seed_wgs : std::min(p.seed_wgs, 512);
        return run_tiled_seed(p.t, codes, n, qluts, nq, cap, R, p.wide ? 1 : 0, (int64_t)tiles * 1024 * cpt,
                              ws, p.stride, st);
    }
    // batches: several tiles per workgroup, so that building the pair tables pays
    const int tpw = (nq >= TILED_MIN_Q) ? 8 : 1;
    dim3 grid((unsigned)ceil_div(p.seed_wgs, tpw), nq);
    const unsigned flush = (unsigned)min((int64_t)R, (int64_t)p.flush_need * tpw);
    switch (p.B) {
    case 4:
        launch(QADC_PROF_SEED, seed_u8_kernel<4>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, p.wide ? 1 : 0);
        break;
    case 8:
        launch(QADC_PROF_SEED, seed_u8_kernel<8>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, p.wide ? 1 : 0);
        break;
    case 16:
        launch(QADC_PROF_SEED, seed_u8_kernel<16>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, p.wide ? 1 : 0);
        break;
    case 32:
        launch(QADC_PROF_SEED, seed_u8_kernel<32>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, p.wide ? 1 : 0);
        break;
    case SIXBIT + 8:
        launch(QADC_PROF_SEED, seed_u8_kernel<SIXBIT + 8>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, 0);
        break;
    case SIXBIT + 16:
        launch(QADC_PROF_SEED, seed_u8_kernel<SIXBIT + 16>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, 0);
        break;
    default:
        launch(QADC_PROF_SEED, seed_u8_kernel<SIXBIT + 32>, grid, dim3(1024), 0, st, codes, n, qluts, cap, R,
                           flush, p.seed_stride, tpw, ws, p.stride, 0);
        break;
    }
    return QADC_OK;
}

template <int NT>
static void dispatch_scan_u8(const ScanPlan &p, const uint8_t *codes, int64_t n,
                             const uint8_t *qluts, int nq, int cap, int R, char *ws,
                             const unsigned *redo_flags, hipStream_t st)
{
    switch (p.B) {
    case 4: launch_scan_u8<4, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    case 8: launch_scan_u8<8, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    case 16: launch_scan_u8<16, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    case 32: launch_scan_u8<32, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    case SIXBIT + 8: launch_scan_u8<SIXBIT + 8, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    case SIXBIT + 16: launch_scan_u8<SIXBIT + 16, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    default: launch_scan_u8<SIXBIT + 32, NT>(p, codes, n, qluts, nq, cap, R, ws, redo_flags, st); break;
    }
}

// Scan + merge of one batch whose control blocks are ready (seed/prepare kernel done or not needed).
static int scan_and_merge_u8(const ScanPlan &p, const uint8_t *codes, int64_t n, const uint8_t *qluts,
                             int nb, int nbins, int R, char *ws, uint32_t *out_idx, uint8_t *out_dist,
                             hipStream_t st)
{
    unsigned *flags = nullptr;
    if (p.tiled && nb >= TILED_MIN_Q) {
        unsigned *taus = reinterpret_cast<unsigned *>(ws + p.taus_off);
        flags = reinterpret_cast<unsigned *>(ws + p.flags_off);
        const int rc = run_tiled_scan(p.t, codes, n, nb, nbins, R, taus, ws, p.stride, p.countsA_off,
                                      p.listsA_off, flags, p.wide ? nullptr : qluts, st);
        if (rc != QADC_OK) return rc;
    }
    if (p.NT == 1024) dispatch_scan_u8<1024>(p, codes, n, qluts, nb, nbins, R, ws, flags, st);
    else if (p.NT == 512) dispatch_scan_u8<512>(p, codes, n, qluts, nb, nbins, R, ws, flags, st);
    else dispatch_scan_u8<256>(p, codes, n, qluts, nb, nbins, R, ws, flags, st);
    return launch_merge<uint8_t, 5>(nb, st, ws, p.stride, p.counts_off, p.lists_off, p.G,
                                    (unsigned)min((int64_t)R, n), R, (uint8_t)nbins, out_idx, out_dist,
                                    p.countsA_off, p.listsA_off, flags ? p.t.GC : 0, (int)TILED_LCAP, flags,
                                    (const uint32_t *)nullptr, (int64_t)0);
}

int scan_topk_u8(int variant, const uint8_t *codes, int64_t n, int m, const uint8_t *qluts, int nq, int R,
                 int nbins, uint32_t *out_idx, uint8_t *out_dist, void *workspace,
                 size_t workspace_bytes, hipStream_t st)
{
    ScanPlan p;
    if (!make_scan_plan(variant, n, m, nq, R, &p))
        return fail(QADC_EINVAL, "qadc_scan_topk: unsupported n=%lld m=%d nq=%d R=%d",
                    (long long)n, m, nq, R);
    if (nbins < 1 || nbins > 255) return fail(QADC_EINVAL, "qadc_scan_topk: nbins=%d not in 1..255", nbins);
    if (((uintptr_t)codes & 15) != 0) return fail(QADC_EINVAL, "qadc_scan_topk: codes must be 16-byte aligned");
    if (((uintptr_t)qluts & 3) != 0) return fail(QADC_EINVAL, "qadc_scan_topk: luts must be 4-byte aligned");
    if (workspace_bytes < p.ws_bytes || !workspace)
        return fail(QADC_ENOMEM, "qadc_scan_topk: workspace %zu < %zu bytes", workspace_bytes, p.ws_bytes);
    if (((uintptr_t)workspace & 255) != 0)
        return fail(QADC_EINVAL, "qadc_scan_topk: workspace must be 256-byte aligned");
    char *ws = (char *)workspace;
    for (int q0 = 0; q0 < nq; q0 += p.qbatch) {
        const int nb = min(p.qbatch, nq - q0);
        const uint8_t *ql = qluts + (size_t)q0 * m * (p.wide ? 256 : variant == QADC_U8_6BIT ? 64 : 16);
        if (p.seed_wgs > 0) {
            const int rs = dispatch_seed_u8(p, codes, n, ql, nb, nbins, R, ws, st);
            if (rs != QADC_OK) return rs;
        }
        const int rc = scan_and_merge_u8(p, codes, n, ql, nb, nbins, R, ws, out_idx + (size_t)q0 * R,
                                         out_dist + (size_t)q0 * R, st);
        if (rc != QADC_OK) return rc;
    }
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

int build_luts(const float *, int, int, int, const float *, const float *, int, float *, hipStream_t);
int quantize_luts(int, const float *, int, int, int, const uint8_t *, int64_t, const float *, int, int,
                  int, uint8_t *, float *, float *, float *, hipStream_t);

// Workspace of qadc_search: the scan workspace, then float tables and quantized tables of a batch.
static size_t search_extra_bytes(int m, int qbatch)
{
    return align_up((size_t)qbatch * m * 16 * sizeof(float), 256) + align_up((size_t)qbatch * m * 16, 256);
}

size_t search_workspace(int64_t n, int m, int nq, int R)
{
    ScanPlan p;
    if (!make_scan_plan(QADC_U8_4BIT, n, m, nq, R, &p)) return 0;
    return p.ws_bytes + search_extra_bytes(m, p.qbatch);
}

int search_u8(const float *codebooks, int d, int m, const float *queries, int nq, const uint8_t *codes,
              int64_t n, int R, int init, int nbins, int qmin_mode, uint32_t *out_idx,
              uint8_t *out_dist, uint8_t *qluts_out, void *workspace, size_t workspace_bytes,
              hipStream_t st)
{
    ScanPlan p;
    if (!codebooks || !queries || !out_idx || !out_dist || (!codes && n > 0))
        return fail(QADC_EINVAL, "qadc_search: null pointer");
    if (nq == 0) return QADC_OK;
    if (!make_scan_plan(QADC_U8_4BIT, n, m, nq, R, &p) || d < m || d % m != 0 || d > PREP_MAX_D)
        return fail(QADC_EINVAL, "qadc_search: unsupported n=%lld d=%d m=%d nq=%d R=%d", (long long)n, d, m,
                    nq, R);
    if (nbins < 1 || nbins > 255 || init < 1 || init > QADC_MAX_INIT || n < 1)
        return fail(QADC_EINVAL, "qadc_search: nbins=%d init=%d n=%lld", nbins, init, (long long)n);
    if (qmin_mode != QADC_QMIN_PER_TABLE && qmin_mode != QADC_QMIN_GLOBAL)
        return fail(QADC_EINVAL, "qadc_search: qmin_mode=%d", qmin_mode);
    if (((uintptr_t)codes & 15) != 0) return fail(QADC_EINVAL, "qadc_search: codes must be 16-byte aligned");
    const size_t need = p.ws_bytes + search_extra_bytes(m, p.qbatch);
    if (!workspace || workspace_bytes < need)
        return fail(QADC_ENOMEM, "qadc_search: workspace %zu < %zu bytes", workspace_bytes, need);
    if (((uintptr_t)workspace & 255) != 0)
        return fail(QADC_EINVAL, "qadc_search: workspace must be 256-byte aligned");
    char *ws = (char *)workspace;
    float *luts = (float *)(ws + p.ws_bytes);
    uint8_t *qluts = (uint8_t *)(ws + p.ws_bytes + align_up((size_t)p.qbatch * m * 16 * sizeof(float), 256));
    const int n_init = (int)min((int64_t)init, n);
    for (int q0 = 0; q0 < nq; q0 += p.qbatch) {
        const int nb = min(p.qbatch, nq - q0);
        const float *yq = queries + (size_t)q0 * d;
        uint8_t *ql_out = qluts_out ? qluts_out + (size_t)q0 * m * 16 : nullptr;
        if (p.seed_wgs > 0 && nb < TILED_MIN_Q) {
            // few queries: one launch; every sampling workgroup recomputes the tables it needs
            dim3 grid(p.seed_wgs, nb);
#define QADC_PREP_CASE(B_)                                                                            \
    case B_:                                                                                         \
        launch(QADC_PROF_PREPARE, prepare_u8_kernel<B_>, grid, dim3(1024), 0, st, codebooks, d, yq, codes, \
               n, n_init, R, nbins, qmin_mode, p.flush_need, p.seed_stride, (float *)nullptr, ql_out, \
               (float *)nullptr, (float *)nullptr, (float *)nullptr, ws, p.stride);                  \
        break;
            switch (p.B) {
                QADC_PREP_CASE(4)
                QADC_PREP_CASE(8)
                QADC_PREP_CASE(16)
                QADC_PREP_CASE(32)
            }
#undef QADC_PREP_CASE
        } else {
            // a batch, or a small database: tables and quantizer once per query by their own
            // kernels, then the sampling kernel (large databases) or a self-seeding scan
            int rc = build_luts(codebooks, d, m, 16, yq, nullptr, nb, luts, st);
            if (rc != QADC_OK) return rc;
            rc = quantize_luts(16, luts, nb, 1, m, codes, n_init, nullptr, R, nbins, qmin_mode, qluts, nullptr,
                               nullptr, nullptr, st);
            if (rc != QADC_OK) return rc;
            if (ql_out)
                QADC_HIP_TRY(hipMemcpyAsync(ql_out, qluts, (size_t)nb * m * 16, hipMemcpyDeviceToDevice, st));
            if (p.seed_wgs > 0) {
                rc = dispatch_seed_u8(p, codes, n, qluts, nb, nbins, R, ws, st);
                if (rc != QADC_OK) return rc;
            }
        }
        const int rc = scan_and_merge_u8(p, codes, n, qluts, nb, nbins, R, ws, out_idx + (size_t)q0 * R,
                                         out_dist + (size_t)q0 * R, st);
        if (rc != QADC_OK) return rc;
    }
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

size_t scan_topk_u8_workspace(int variant, int64_t n, int m, int nq, int R)
{
    ScanPlan p;
    if (!make_scan_plan(variant, n, m, nq, R, &p)) return 0;
    return p.ws_bytes;
}

int workspace_init(void *workspace, size_t bytes, hipStream_t st)
{
    if (!workspace && bytes) return fail(QADC_EINVAL, "qadc_workspace_init: null workspace");
    if (bytes) QADC_HIP_TRY(hipMemsetAsync(workspace, 0, bytes, st));
    return QADC_OK;
}

}  // namespace qadc
