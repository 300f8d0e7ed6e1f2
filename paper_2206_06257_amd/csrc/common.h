// Shared host/device helpers of libdat (GPU library only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/dat.h"

namespace dat {

// Records the text of a failed HIP call for dat_last_error() and maps it to DAT_ERR_HIP.
dat_status hip_fail(hipError_t e, const char* what, const char* file, int line);

#define DAT_HIP(call)                                                              \
  do {                                                                             \
    hipError_t e_ = (call);                                                        \
    if (e_ != hipSuccess) return ::dat::hip_fail(e_, #call, __FILE__, __LINE__);   \
  } while (0)

#define DAT_LAUNCH_CHECK() DAT_HIP(hipGetLastError())

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

typedef uint16_t bf16_t;   // raw bf16 bit pattern

// fp32 -> bf16, round to nearest even; NaN stays NaN.
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

}  // namespace dat
