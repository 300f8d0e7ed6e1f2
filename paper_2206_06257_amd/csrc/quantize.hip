// Randomized b-bit gradient quantizer of DAT (Alg. A1 step 7; appendix "Additional details on
// gradient quantization", Eqs. (rand_q), (xi)) and its inverse, as three HBM-streaming kernels
// over the flat gradient vector: a segmented abs-max (one scale per parameter tensor), the
// stochastic-rounding encoder, and the decoder.  One launch covers all tensors: each thread
// finds the tensor of its first element by binary search in the offset table and then only
// walks forward, so tensors of any length (down to one element) cost no extra launches.
//
// Exactness: every fp32 operation below is a single correctly rounded operation (explicit
// __f*_rn intrinsics, file built with -ffp-contract=off) so codes are reproducible bit for bit
// from the definition in include/dat.h.
#include "common.h"
#include "philox.h"

namespace dat {
namespace {

constexpr int kThreads = 256;
constexpr int kIter = 8;          // groups per thread
constexpr uint32_t kStreamQuant = 0;

__device__ __forceinline__ int find_tensor(const int64_t* off, int T, int64_t i) {
  // largest t with off[t] <= i  (off[0] = 0, off[T] = d > i); empty tensors are skipped
  int lo = 0, hi = T;
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (off[mid] <= i) lo = mid; else hi = mid;
  }
  return lo;
}

// The offset table in LDS (T <= kTabMax): the binary search and every tensor boundary a thread crosses then
// cost LDS reads instead of dependent global loads.  Returns the table to use (generic pointer).
constexpr int kTabMax = 1024;
__device__ __forceinline__ const int64_t* stage_offsets(const int64_t* __restrict__ off, int T, int64_t* s_off) {
  if (T > kTabMax) return off;
  for (int i = threadIdx.x; i <= T; i += blockDim.x) s_off[i] = off[i];
  __syncthreads();
  return s_off;
}

__global__ void fill_u32_kernel(uint32_t* p, int n, uint32_t v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// ---- segmented abs-max -------------------------------------------------------------------
// |g| is compared through its bit pattern (non-negative floats order like unsigned integers,
// NaN patterns sort above Inf, so a NaN or Inf anywhere surfaces in the scale).
__global__ __launch_bounds__(kThreads) void absmax_kernel(const float* __restrict__ g,
                                                          const int64_t* off, int T,
                                                          int64_t d, uint32_t* __restrict__ scale_bits) {
  // A workgroup owns 16 K consecutive elements, hence a run of consecutive tensors starting at
  // `tfirst`.  Per-tensor maxima are first combined in LDS (slot = tensor - tfirst) and only the
  // touched slots go to global memory: one global atomic per workgroup and tensor.  Thousands of
  // atomics on one L2 address would otherwise dominate the kernel.
  constexpr int kIterA = 2 * kIter;                // groups per thread
  constexpr int kSlots = 128;
  __shared__ uint32_t s_max[kSlots];
  __shared__ int s_tfirst;
  __shared__ int64_t s_off[kTabMax + 1];
  off = stage_offsets(off, T, s_off);
  const int64_t ngroups = (d + 3) >> 2;
  const int64_t grp0 = (int64_t)blockIdx.x * (kThreads * kIterA);
  if (threadIdx.x == 0) s_tfirst = find_tensor(off, T, min(grp0 << 2, d - 1));
  if (threadIdx.x < kSlots) s_max[threadIdx.x] = 0u;
  __syncthreads();
  const int tfirst = s_tfirst;
  int t = tfirst;
  int64_t next = off[t + 1];
  uint32_t m = 0;
  auto flush = [&]() {
    if (m) {
      const int slot = t - tfirst;
      if (slot < kSlots) atomicMax(&s_max[slot], m); else atomicMax(scale_bits + t, m);
    }
    m = 0;
  };
  int64_t grp = grp0 + threadIdx.x;
  for (int it = 0; it < kIterA; it += 4) {
    // four groups per trip (16 elements, 4 KiB apart) so that four loads are in flight; the fast
    // path needs all of them inside the current tensor
    const int64_t ifirst = grp << 2, ilast = ((grp + 3 * kThreads) << 2) + 3;
    if (ifirst < next && ilast < d && ilast < next) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(g + ((grp + u * kThreads) << 2));
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t a = __float_as_uint(v[u].x) & 0x7fffffffu, b = __float_as_uint(v[u].y) & 0x7fffffffu;
        const uint32_t c = __float_as_uint(v[u].z) & 0x7fffffffu, e = __float_as_uint(v[u].w) & 0x7fffffffu;
        m = max(max(m, max(a, b)), max(c, e));
      }
      grp += 4 * kThreads;
      continue;
    }
    for (int u = 0; u < 4; ++u, grp += kThreads) {
      if (grp >= ngroups) break;
      const int64_t i0 = grp << 2;
      while (i0 >= next) { flush(); ++t; next = off[t + 1]; }
      if (i0 + 3 < d && i0 + 3 < next) {           // whole group inside the tensor
        const float4 v = *reinterpret_cast<const float4*>(g + i0);
        const uint32_t a = __float_as_uint(v.x) & 0x7fffffffu, b = __float_as_uint(v.y) & 0x7fffffffu;
        const uint32_t c = __float_as_uint(v.z) & 0x7fffffffu, e = __float_as_uint(v.w) & 0x7fffffffu;
        m = max(max(m, max(a, b)), max(c, e));
      } else {
        for (int j = 0; j < 4; ++j) {
          const int64_t i = i0 + j;
          if (i >= d) break;
          while (i >= next) { flush(); ++t; next = off[t + 1]; }
          m = max(m, __float_as_uint(g[i]) & 0x7fffffffu);
        }
      }
    }
  }
  flush();
  __syncthreads();
  if (threadIdx.x < kSlots && s_max[threadIdx.x]) atomicMax(scale_bits + tfirst + threadIdx.x, s_max[threadIdx.x]);
}

// ---- encoder / decoder ------------------------------------------------------------------
template <int BITS> struct Fmt {
  static constexpr int kEpt = BITS >= 8 ? 4 : 32 / BITS;   // elements per thread-group
  static constexpr int kWords = kEpt * BITS / 32;          // 32-bit words per group
  static constexpr int kS = (1 << (BITS - 1)) - 1;
};

struct TensorCursor {
  int t; int64_t next; float mul; bool ok;
};

template <int BITS>
__device__ __forceinline__ void enc_enter(TensorCursor& c, const float* __restrict__ scales) {
  const float sc = scales[c.t];
  c.ok = sc > 0.0f && sc < __builtin_inff();
  c.mul = c.ok ? __fdiv_rn((float)Fmt<BITS>::kS, sc) : 0.0f;
}

template <int BITS>
__device__ __forceinline__ int encode_one(float g, float u, const TensorCursor& c) {
  if (!c.ok) return 0;
  const float r = __fmul_rn(fabsf(g), c.mul);
  const float l = floorf(r);
  const float p = __fsub_rn(r, l);
  float mag = __fadd_rn(l, u < p ? 1.0f : 0.0f);
  mag = fminf(mag, (float)Fmt<BITS>::kS);
  const int code = (int)mag;
  return g < 0.0f ? -code : code;
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float* __restrict__ g,
                                                            const int64_t* off, int T,
                                                            int64_t d, uint64_t seed,
                                                            const float* __restrict__ scales,
                                                            uint8_t* __restrict__ q) {
  constexpr int EPT = Fmt<BITS>::kEpt, WORDS = Fmt<BITS>::kWords;
  __shared__ int64_t s_off[kTabMax + 1];
  off = stage_offsets(off, T, s_off);
  const int64_t ngroups = (d + EPT - 1) / EPT;
  int64_t grp = (int64_t)blockIdx.x * (kThreads * kIter) + threadIdx.x;
  if (grp >= ngroups) return;
  // with four elements per group (8 and 16 bit) the eight groups of a thread are fetched before the first one is
  // encoded: eight loads in flight instead of one
  constexpr bool PRE = EPT == 4;
  float4 pre[PRE ? kIter : 1];
  if (PRE) {
#pragma unroll
    for (int it = 0; it < kIter; ++it) {
      const int64_t gi = grp + (int64_t)it * kThreads;
      pre[it] = (gi * EPT + EPT <= d) ? *reinterpret_cast<const float4*>(g + gi * EPT) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  TensorCursor c;
  c.t = find_tensor(off, T, grp * EPT);
  c.next = off[c.t + 1];
  enc_enter<BITS>(c, scales);
  if (PRE) {
    // all eight groups of this thread inside the current tensor and inside the vector (the common case: tensors are
    // much longer than the 8 K elements a workgroup covers): one scale, no boundary tests, whole words stored
    const int64_t ilast = (grp + (int64_t)(kIter - 1) * kThreads) * EPT + (EPT - 1);
    if (ilast < c.next && ilast < d) {
      uint32_t* dst = reinterpret_cast<uint32_t*>(q);
#pragma unroll
      for (int it = 0; it < kIter; ++it) {
        const int64_t gi = grp + (int64_t)it * kThreads;
        const PhiloxWords w = philox_block((uint64_t)gi, seed, kStreamQuant);      // EPT == 4: element index / 4 = group index
        const float v[4] = {pre[it].x, pre[it].y, pre[it].z, pre[it].w};
        const float u[4] = {u24(w.w0), u24(w.w1), u24(w.w2), u24(w.w3)};
        uint32_t word[WORDS];
#pragma unroll
        for (int wd = 0; wd < WORDS; ++wd) word[wd] = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t field = (uint32_t)encode_one<BITS>(v[j], u[j], c) & ((1u << BITS) - 1u);
          word[(j * BITS) / 32] |= field << ((j * BITS) % 32);
        }
#pragma unroll
        for (int wd = 0; wd < WORDS; ++wd) dst[gi * WORDS + wd] = word[wd];
      }
      return;
    }
  }
#pragma unroll
  for (int it = 0; it < kIter; ++it, grp += kThreads) {
    if (grp >= ngroups) break;
    const int64_t i0 = grp * EPT;
    float v[EPT]; float u[EPT];
    const bool full = i0 + EPT <= d;
    if (full) {
      if (PRE) {
        v[0] = pre[it].x; v[1] = pre[it].y; v[2] = pre[it].z; v[3] = pre[it].w;
      } else {
#pragma unroll
        for (int j = 0; j < EPT; j += 4) {
          const float4 f = *reinterpret_cast<const float4*>(g + i0 + j);
          v[j] = f.x; v[j + 1] = f.y; v[j + 2] = f.z; v[j + 3] = f.w;
        }
      }
    } else {
      for (int j = 0; j < EPT; ++j) v[j] = (i0 + j < d) ? g[i0 + j] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < EPT; j += 4) {
      const PhiloxWords w = philox_block((uint64_t)((i0 + j) >> 2), seed, kStreamQuant);
      u[j] = u24(w.w0); u[j + 1] = u24(w.w1); u[j + 2] = u24(w.w2); u[j + 3] = u24(w.w3);
    }
    uint32_t word[WORDS];
#pragma unroll
    for (int wd = 0; wd < WORDS; ++wd) word[wd] = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      const int64_t i = i0 + j;
      int code = 0;
      if (i < d) {
        while (i >= c.next) { ++c.t; c.next = off[c.t + 1]; enc_enter<BITS>(c, scales); }
        code = encode_one<BITS>(v[j], u[j], c);
      }
      const uint32_t field = (uint32_t)code & (BITS == 32 ? 0xffffffffu : ((1u << BITS) - 1u));
      word[(j * BITS) / 32] |= field << ((j * BITS) % 32);
    }
    if (full) {
      uint32_t* dst = reinterpret_cast<uint32_t*>(q) + grp * WORDS;
#pragma unroll
      for (int wd = 0; wd < WORDS; ++wd) dst[wd] = word[wd];
    } else {   // ragged tail: never write past ceil(d*BITS/8) bytes
      const int64_t byte0 = grp * WORDS * 4, nbytes = (d * BITS + 7) / 8;
      for (int b = 0; b < WORDS * 4 && byte0 + b < nbytes; ++b)
        q[byte0 + b] = (uint8_t)(word[b >> 2] >> ((b & 3) * 8));
    }
  }
}

template <int BITS>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t* __restrict__ q,
                                                              const int64_t* off, int T,
                                                              int64_t d, const float* __restrict__ scales,
                                                              float* __restrict__ out) {
  constexpr int EPT = Fmt<BITS>::kEpt, WORDS = Fmt<BITS>::kWords;
  __shared__ int64_t s_off[kTabMax + 1];
  off = stage_offsets(off, T, s_off);
  const int64_t ngroups = (d + EPT - 1) / EPT;
  int64_t grp = (int64_t)blockIdx.x * (kThreads * kIter) + threadIdx.x;
  if (grp >= ngroups) return;
  int t = find_tensor(off, T, grp * EPT);
  int64_t next = off[t + 1];
  float step = __fdiv_rn(scales[t], (float)Fmt<BITS>::kS);
  for (int it = 0; it < kIter; ++it, grp += kThreads) {
    if (grp >= ngroups) break;
    const int64_t i0 = grp * EPT;
    const bool full = i0 + EPT <= d;
    uint32_t word[WORDS];
    if (full) {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(q) + grp * WORDS;
#pragma unroll
      for (int wd = 0; wd < WORDS; ++wd) word[wd] = src[wd];
    } else {
      const int64_t byte0 = grp * WORDS * 4, nbytes = (d * BITS + 7) / 8;
#pragma unroll
      for (int wd = 0; wd < WORDS; ++wd) word[wd] = 0;
      for (int b = 0; b < WORDS * 4 && byte0 + b < nbytes; ++b)
        word[b >> 2] |= (uint32_t)q[byte0 + b] << ((b & 3) * 8);
    }
    float r[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
      const int64_t i = i0 + j;
      if (i < d) {
        while (i >= next) { ++t; next = off[t + 1]; step = __fdiv_rn(scales[t], (float)Fmt<BITS>::kS); }
      }
      const uint32_t field = word[(j * BITS) / 32] >> ((j * BITS) % 32);
      const int code = ((int)(field << (32 - BITS))) >> (32 - BITS);   // sign-extend
      r[j] = __fmul_rn((float)code, step);
    }
    if (full) {
#pragma unroll
      for (int j = 0; j < EPT; j += 4)
        *reinterpret_cast<float4*>(out + i0 + j) = make_float4(r[j], r[j + 1], r[j + 2], r[j + 3]);
    } else {
      for (int j = 0; j < EPT && i0 + j < d; ++j) out[i0 + j] = r[j];
    }
  }
}

__global__ void philox_uniform_kernel(uint64_t start, int64_t n, uint64_t seed, uint32_t stream_id,
                                      float* __restrict__ out) {
  int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n) return;
  const uint64_t i = start + (uint64_t)k;
  const PhiloxWords w = philox_block(i >> 2, seed, stream_id);
  const uint32_t sel = (uint32_t)(i & 3);
  out[k] = u24(sel == 0 ? w.w0 : sel == 1 ? w.w1 : sel == 2 ? w.w2 : w.w3);
}

inline unsigned blocks_for(int64_t ngroups) {
  return (unsigned)((ngroups + (int64_t)kThreads * kIter - 1) / ((int64_t)kThreads * kIter));
}

bool bits_ok(int bits) { return bits == 2 || bits == 4 || bits == 8 || bits == 16; }

}  // namespace
}  // namespace dat

using namespace dat;

extern "C" size_t dat_quantized_bytes(int64_t d, int bits) {
  if (d < 0 || !bits_ok(bits)) return 0;
  return (size_t)((d * bits + 7) / 8);
}

extern "C" dat_status dat_quantize(const float* grads, const int64_t* offsets_dev, int num_tensors,
                                   int64_t d, int bits, uint64_t seed, uint8_t* q, float* scales,
                                   void* stream) {
  if (!grads || !offsets_dev || !q || !scales || num_tensors < 1 || d < 0 || !bits_ok(bits)) return DAT_ERR_ARG;
  if (!aligned(grads, 16) || !aligned(q, 4) || !aligned(scales, 4)) return DAT_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((num_tensors + 255) / 256), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(scales), num_tensors, 0u);
  DAT_LAUNCH_CHECK();
  if (d == 0) return DAT_OK;
  hipLaunchKernelGGL(absmax_kernel, dim3((blocks_for((d + 3) / 4) + 1) / 2), dim3(kThreads), 0, st, grads,
                     offsets_dev, num_tensors, d, reinterpret_cast<uint32_t*>(scales));
  DAT_LAUNCH_CHECK();
#define DAT_Q_LAUNCH(B)                                                                          \
  hipLaunchKernelGGL(quantize_kernel<B>, dim3(blocks_for((d + Fmt<B>::kEpt - 1) / Fmt<B>::kEpt)), \
                     dim3(kThreads), 0, st, grads, offsets_dev, num_tensors, d, seed, scales, q)
  switch (bits) {
    case 2: DAT_Q_LAUNCH(2); break;
    case 4: DAT_Q_LAUNCH(4); break;
    case 8: DAT_Q_LAUNCH(8); break;
    default: DAT_Q_LAUNCH(16); break;
  }
#undef DAT_Q_LAUNCH
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

extern "C" dat_status dat_quantize_scaled(const float* grads, const int64_t* offsets_dev, int num_tensors, int64_t d, int bits,
                                          uint64_t seed, const float* scales, uint8_t* q, void* stream) {
  if (!grads || !offsets_dev || !q || !scales || num_tensors < 1 || d < 0 || !bits_ok(bits)) return DAT_ERR_ARG;
  if (!aligned(grads, 16) || !aligned(q, 4) || !aligned(scales, 4)) return DAT_ERR_ARG;
  if (d == 0) return DAT_OK;
  hipStream_t st = (hipStream_t)stream;
#define DAT_Q_LAUNCH(B)                                                                          \
  hipLaunchKernelGGL(quantize_kernel<B>, dim3(blocks_for((d + Fmt<B>::kEpt - 1) / Fmt<B>::kEpt)), \
                     dim3(kThreads), 0, st, grads, offsets_dev, num_tensors, d, seed, scales, q)
  switch (bits) {
    case 2: DAT_Q_LAUNCH(2); break;
    case 4: DAT_Q_LAUNCH(4); break;
    case 8: DAT_Q_LAUNCH(8); break;
    default: DAT_Q_LAUNCH(16); break;
  }
#undef DAT_Q_LAUNCH
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

extern "C" dat_status dat_dequantize(const uint8_t* q, const float* scales, const int64_t* offsets_dev,
                                     int num_tensors, int64_t d, int bits, float* grads_out,
                                     void* stream) {
  if (!q || !scales || !offsets_dev || !grads_out || num_tensors < 1 || d < 0 || !bits_ok(bits)) return DAT_ERR_ARG;
  if (!aligned(grads_out, 16) || !aligned(q, 4)) return DAT_ERR_ARG;
  if (d == 0) return DAT_OK;
  hipStream_t st = (hipStream_t)stream;
#define DAT_DQ_LAUNCH(B)                                                                           \
  hipLaunchKernelGGL(dequantize_kernel<B>, dim3(blocks_for((d + Fmt<B>::kEpt - 1) / Fmt<B>::kEpt)), \
                     dim3(kThreads), 0, st, q, offsets_dev, num_tensors, d, scales, grads_out)
  switch (bits) {
    case 2: DAT_DQ_LAUNCH(2); break;
    case 4: DAT_DQ_LAUNCH(4); break;
    case 8: DAT_DQ_LAUNCH(8); break;
    default: DAT_DQ_LAUNCH(16); break;
  }
#undef DAT_DQ_LAUNCH
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

extern "C" dat_status dat_philox_uniform(uint64_t start, int64_t n, uint64_t seed, uint32_t stream_id,
                                         float* out, void* stream) {
  if (!out || n < 0) return DAT_ERR_ARG;
  if (n == 0) return DAT_OK;
  hipLaunchKernelGGL(philox_uniform_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     (hipStream_t)stream, start, n, seed, stream_id, out);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}
