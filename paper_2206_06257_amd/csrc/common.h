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
// Per-tensor abs-max of the parameter gradients (the quantizer's scale), taken where the gradients are written.
// |v| is compared through its bit pattern (non-negative floats order like unsigned integers, NaN patterns above
// Inf), so the result is exact and independent of the order of the updates.  Every tensor has kAbsmaxWays slots,
// 128 bytes apart (one cache line each); a workgroup raises slot (workgroup index mod kAbsmaxWays), so the
// hundreds of thousands of short workgroups of a large tensor do not queue on one address, and
// absmax_fold_kernel takes the maximum over the ways afterwards.  A writer reads its slot when it starts
// (absmax_peek, off the critical path) and issues the atomic only when it can raise the value: a stale read
// can only cause a superfluous atomic, never a missing one, because stored values only grow.
constexpr int kAbsmaxWays = 16, kAbsmaxStride = 32;   // uint32 units
__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }
__device__ __forceinline__ uint32_t* absmax_way(uint32_t* tensor_slots, unsigned workgroup) {
  return tensor_slots + (workgroup % kAbsmaxWays) * kAbsmaxStride;
}
__device__ __forceinline__ uint32_t absmax_peek(const uint32_t* slot) { return __builtin_nontemporal_load(slot); }
__device__ __forceinline__ void absmax_raise(uint32_t* slot, uint32_t seen, uint32_t m) {
  if (m > seen) atomicMax(slot, m);
}
__device__ __forceinline__ void absmax_publish(uint32_t* slot, uint32_t m) { absmax_raise(slot, absmax_peek(slot), m); }
// The slot groups (kAbsmaxWays slots each) of the two tensors a finishing kernel writes (for a batch normalisation:
// beta gradient, gamma gradient), or null.
struct ParamAbsmax { uint32_t* first; uint32_t* second; };

// Layout of the constants: channel c at tab[(c/8)*32 + which*8 + c%8], which = 0..3 for a, p, q, mu.
constexpr int kBnTabFloatsPerChannel = 4;

}  // namespace dat
