// Optional per-kernel timing: while enabled, kernels are launched with a start and a stop
// event attached to the dispatch itself, so the measured time is the kernel's own duration.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

namespace qadc {
bool prof_open(int which, hipEvent_t *start, hipEvent_t *stop);
int profile_enable(int on);
int profile_only(int which);
int profile_read(int which, double *total_ms, int64_t *launches);

// Launches `kernel`; `which` names the profiling slot its duration is added to (-1: none).
template <typename F, typename... Args>
inline void launch(int which, F kernel, dim3 grid, dim3 block, size_t shmem, hipStream_t st, Args... args)
{
    hipEvent_t a = nullptr, b = nullptr;
    if (which >= 0 && prof_open(which, &a, &b))
        hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)shmem, st, a, b, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, shmem, st, args...);
}
}  // namespace qadc
