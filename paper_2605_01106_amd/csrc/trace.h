// Development aid: with HH_KERNEL_TRACE defined, TR(i) makes thread 0 of every workgroup record
// the 100 MHz wall clock in slot i of a per-workgroup record (up to 4096 workgroups, 16 slots).
// Without it TR(i) is empty.
#pragma once
#include <hip/hip_runtime.h>

namespace hh {
#ifdef HH_KERNEL_TRACE
__device__ long long g_kernel_trace[4096 * 16];
#define TR(i) do { if (threadIdx.x == 0) g_kernel_trace[((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 + (i)] = wall_clock64(); } while (0)
#else
#define TR(i)
#endif

}  // namespace hh
