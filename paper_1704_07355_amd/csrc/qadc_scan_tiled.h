// Interface of the query-tiled scan (qadc_scan_tiled.hip) towards the scan driver.
#pragma once

#include "qadc_common.h"

namespace qadc {

constexpr int TILED_Q = 8;             // queries per workgroup
// threads per workgroup: with m = 64 (B = 32) one workgroup's tables fill 128 KiB of the LDS,
// so that workgroup is made twice as large to keep enough wavefronts on the CU
constexpr int tiled_nt(int B) { return B >= 32 ? 1024 : 512; }
constexpr int TILED_LCAP = 64;         // keys a workgroup can report per query
constexpr int TILED_MAX_CHUNKS = 1024; // database chunks per query
constexpr int TILED_MFMA_MAX_CHUNKS = 4096;  // the same for small batches on the matrix-core kernel
constexpr int TILED_MIN_Q = 8;         // smallest batch worth tiling
constexpr int TILED_MFMA_MIN_Q = 16;   // smallest batch for the matrix-core kernel (32 queries per wavefront; twice that below 8 code bytes)
constexpr int TILED_MFMA_MIN_Q2 = 64;  // smallest batch for its 64-queries-per-wavefront form
constexpr int TILED_MFMA_MIN_Q4 = 128; // ... for 128 queries per wavefront (codes of up to 8 bytes)

struct TiledPlan {
    int B, GC;
    int64_t chunk;
    size_t lds_bytes;
    bool mfma;  // (sub-)batches of TILED_MFMA_MIN_Q queries or more go to the matrix-core kernel
};

// codes4: 4-bit codes with the queries' 16-entry tables at hand (what the matrix-core kernel reads)
bool make_tiled_plan(int64_t n, int m, int nq, bool codes4, TiledPlan *t);

// tau kernel + tiled scan kernel for `nq` queries whose control blocks (histogram, pair
// tables) were filled by the seed/prepare kernel.  qluts16: the queries' 16-entry quantized
// tables [nq][m][16] when the codes are 4-bit (null for 8-bit components).  Region A of query q: counts at
// ws + q*ws_stride + countsA_off ([GC] u32), lists at + listsA_off ([GC][TILED_LCAP] u64).
int run_tiled_scan(const TiledPlan &t, const uint8_t *codes, int64_t n, int nq, int cap, int R,
                   unsigned *taus, char *ws, size_t ws_stride, size_t countsA_off, size_t listsA_off,
                   unsigned *flags, const uint8_t *qluts16, hipStream_t st);

// Pair tables of the batch + the sampled histograms behind the bounds, in the query-tiled way:
// what seed_u8_kernel does per query.  `sample_codes`: codes of the sample per query.
int run_tiled_seed(const TiledPlan &t, const uint8_t *codes, int64_t n, const uint8_t *qluts, int nq, int cap,
                   int R, int wide, int64_t sample_codes, char *ws, size_t ws_stride, hipStream_t st);

}  // namespace qadc
