#pragma once
#include <hip/hip_runtime.h>

namespace qadc {
bool prof_on();
void prof_begin(int which, hipStream_t st);
void prof_end(int which, hipStream_t st);
int profile_enable(int on);
int profile_read(int which, double *total_ms, int64_t *launches);
}  // namespace qadc
