// Shared host/device helpers of libdat (GPU library only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/dat.h"

namespace dat {

// Records the text of a failed HIP call for dat_last_error() and maps it to DAT_ERR_HIP.
dat_status hip_fail(hipError_t e, const char* what, const char* file, int line);

// Records a message of the library's own for dat_last_error() and returns `status`.
dat_status fail_with(dat_status status, const char* text);

#define DAT_HIP(call)                                                              \
  do {                                                                             \
    hipError_t e_ = (call);                                                        \
    if (e_ != hipSuccess) return ::dat::hip_fail(e_, #call, __FILE__, __LINE__);   \
  } while (0)

#define DAT_LAUNCH_CHECK() DAT_HIP(hipGetLastError())

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

typedef uint16_t bf16_t;   // raw bf16 bit pattern

// fp32 -> bf16, round to nearest even; NaN stays (quiet) NaN.  Compiles to v_cvt_pk_bf16_f32, whose
// results equal the integer formulation (u + 0x7fff + lsb) >> 16 for every non-NaN input.
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values in one instruction: `lo` in bits 0..15, `hi` in bits 16..31
__device__ __forceinline__ uint32_t f2bf_pack(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Input gradient of a train-mode batch normalisation for one element, from the per-channel constants
//   a = gamma*rstd,  p = -a*rstd*(sum dy*xhat)/rows,  q = -a*(sum dy)/rows,  mu = batch mean:
//   dx = gamma*rstd*(dy - mean(dy) - xhat*mean(dy*xhat)) = a*dy + p*(x - mu) + q.
// Five single-rounded fp32 operations in this order wherever it is evaluated (the stand-alone pass and
// the convolution that applies it while loading its operand), so both give the same bits.
__device__ __forceinline__ float bn_input_grad(float dy, float x, float a, float p, float q, float mu) {
  const float t = __fmul_rn(p, __fsub_rn(x, mu));
  return __fadd_rn(__fadd_rn(__fmul_rn(a, dy), t), q);
}
// Layout of the constants: channel c at tab[(c/8)*32 + which*8 + c%8], which = 0..3 for a, p, q, mu.
constexpr int kBnTabFloatsPerChannel = 4;

}  // namespace dat
