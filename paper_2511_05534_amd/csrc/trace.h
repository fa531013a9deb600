// Phase stamps for kernel tuning.  Build with -DFLOWMM_TRACE to make thread 0 of every workgroup
// write the 100 MHz wall clock at the TRACE(k) points of a kernel into a buffer (16 slots per
// workgroup) that the translation unit's own setter installs (no stamps while it has installed none).
// Without the macro TRACE is empty.
#pragma once
#include <hip/hip_runtime.h>

#ifdef FLOWMM_TRACE
namespace flowmm {
namespace {
__device__ unsigned long long *g_trace;
}
}  // namespace flowmm
#define TRACE(k)                                                                                          \
  do {                                                                                                    \
    if (threadIdx.x == 0 && g_trace != nullptr)                                                           \
      g_trace[(((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 + (k)] = wall_clock64(); \
  } while (0)
#else
#define TRACE(k)
#endif
