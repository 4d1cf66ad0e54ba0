// Shared host/device helpers of the Quick ADC HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "qadc.h"

namespace qadc {

// Thread-local message of the last failing call.
char *err_buf();
int fail(int code, const char *fmt, ...);

#define QADC_HIP_TRY(expr)                                                              \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess)                                                           \
            return qadc::fail(QADC_EHIP, "%s: %s", #expr, hipGetErrorString(e_));       \
    } while (0)

constexpr int WAVE = 64;

__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

// Number of set bits of `m` below this lane.
__device__ __forceinline__ unsigned rank_in_mask(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32),
                                     __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// Wave-aggregated append to an LDS list: lanes with `pred` get distinct slots
// counter .. counter+k-1 with one atomic per wave.  Returns the slot (valid when pred).
__device__ __forceinline__ unsigned wave_append_slot(bool pred, unsigned *counter)
{
    unsigned long long m = __ballot(pred);
    unsigned base = 0;
    if (m == 0) return 0;
    int leader = __ffsll((long long)m) - 1;
    if (lane_id() == leader) base = atomicAdd(counter, (unsigned)__popcll(m));
    base = __shfl(base, leader);
    return base + rank_in_mask(m);
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

}  // namespace qadc
