// After the worker block: the server's aggregation of quantized gradients, Eq. (grad_agg), and the
// outer-minimisation oracle A(.) as the layer-wise adaptive learning rate of Eq. (3) with the LAMB
// direction of Alg. A2.  All kernels stream the flat parameter vector once (HBM-bound) and walk the
// tensor table like the quantizer does; per-tensor squared norms are accumulated in fp64, first in
// LDS slots per workgroup, then with one global atomic per workgroup and tensor.
#include "kernels.h"

namespace dat {
namespace {

constexpr int kT = 256;
constexpr int kIter = 8;
constexpr int kSlots = 128;

__device__ __forceinline__ int find_tensor(const int64_t* __restrict__ off, int T, int64_t i) {
  int lo = 0, hi = T;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= i) lo = mid; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ void atomic_add_f64(double* p, double v) { atomicAdd(p, v); }

// m, v, u updated in place; norms[0][t] += sum theta^2, norms[1][t] += sum u^2.
__global__ __launch_bounds__(kT) void lamb_direction_kernel(const float* __restrict__ theta, const float* __restrict__ g,
                                                            float* __restrict__ m, float* __restrict__ v,
                                                            float* __restrict__ u, const int64_t* __restrict__ off,
                                                            int T, int64_t d, LambParams hp, double* __restrict__ norms) {
  __shared__ double s_n[2][kSlots];
  __shared__ int s_tfirst;
  const int64_t i_begin = (int64_t)blockIdx.x * (kT * kIter);
  if (threadIdx.x == 0) s_tfirst = find_tensor(off, T, min(i_begin, d - 1));
  if (threadIdx.x < kSlots) { s_n[0][threadIdx.x] = 0.0; s_n[1][threadIdx.x] = 0.0; }
  __syncthreads();
  const int tfirst = s_tfirst;
  int t = tfirst;
  int64_t next = off[t + 1];
  double a_th = 0.0, a_u = 0.0;
  auto flush = [&]() {
    if (a_th != 0.0 || a_u != 0.0) {
      const int slot = t - tfirst;
      if (slot < kSlots) { atomic_add_f64(&s_n[0][slot], a_th); atomic_add_f64(&s_n[1][slot], a_u); }
      else { atomic_add_f64(norms + t, a_th); atomic_add_f64(norms + T + t, a_u); }
    }
    a_th = 0.0; a_u = 0.0;
  };
  for (int it = 0; it < kIter; ++it) {
    const int64_t i = i_begin + (int64_t)it * kT + threadIdx.x;
    if (i >= d) break;
    while (i >= next) { flush(); ++t; next = off[t + 1]; }
    const float th = theta[i], gi = g[i];
    float ui;
    if (hp.use_adam) {
      const float mi = hp.b1 * m[i] + (1.0f - hp.b1) * gi;
      const float vi = hp.b2 * v[i] + (1.0f - hp.b2) * gi * gi;
      m[i] = mi; v[i] = vi;
      ui = (mi * hp.inv_bc1) / (sqrtf(vi * hp.inv_bc2) + hp.zeta);
    } else {
      ui = gi;
    }
    ui += hp.wd * th;
    u[i] = ui;
    a_th += (double)th * (double)th;
    a_u += (double)ui * (double)ui;
  }
  flush();
  __syncthreads();
  if (threadIdx.x < kSlots && tfirst + (int)threadIdx.x < T) {
    if (s_n[0][threadIdx.x] != 0.0) atomic_add_f64(norms + tfirst + threadIdx.x, s_n[0][threadIdx.x]);
    if (s_n[1][threadIdx.x] != 0.0) atomic_add_f64(norms + T + tfirst + threadIdx.x, s_n[1][threadIdx.x]);
  }
}

// theta_i <- theta_i - eta * tau(||theta_i||) / ||u_i|| * u_i
__global__ __launch_bounds__(kT) void lalr_apply_kernel(float* __restrict__ theta, const float* __restrict__ u,
                                                        const int64_t* __restrict__ off, int T, int64_t d,
                                                        LambParams hp, const double* __restrict__ norms) {
  const int64_t i_begin = (int64_t)blockIdx.x * (kT * kIter);
  int64_t i = i_begin + threadIdx.x;
  if (i >= d) return;
  int t = find_tensor(off, T, i);
  int64_t next = off[t + 1];
  auto rate_of = [&](int tt) -> float {
    const double nth = sqrt(norms[tt]), nu = sqrt(norms[T + tt]);
    if (!(nu > 0.0)) return 0.0f;
    const double tau = fmin(fmax(nth, (double)hp.c_l), (double)hp.c_u);
    return (float)((double)hp.eta * tau / nu);
  };
  float rate = rate_of(t);
  for (int it = 0; it < kIter; ++it, i += kT) {
    if (i >= d) break;
    while (i >= next) { ++t; next = off[t + 1]; rate = rate_of(t); }
    theta[i] = theta[i] - rate * u[i];
  }
}

__global__ void zero_f64_kernel(double* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.0;
}

// ---- aggregation of M quantized gradients ------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(kT) void aggregate_kernel(AggregateArgs a) {
  constexpr int EPW = 32 / BITS;                      // codes per 32-bit word
  constexpr int S = (1 << (BITS - 1)) - 1;
  const int64_t nwords = (a.d * BITS + 31) / 32;
  int64_t wi = (int64_t)blockIdx.x * (kT * kIter) + threadIdx.x;
  if (wi >= nwords) return;
  int t = find_tensor(a.offsets, a.T, wi * EPW);
  int64_t next = a.offsets[t + 1];
  const int64_t nbytes = (a.d * BITS + 7) / 8;
  for (int it = 0; it < kIter; ++it, wi += kT) {
    if (wi >= nwords) break;
    const int64_t i0 = wi * EPW;
    float acc[EPW];
    int tt[EPW];
#pragma unroll
    for (int j = 0; j < EPW; ++j) {
      acc[j] = 0.0f;
      const int64_t i = i0 + j;
      if (i < a.d) { while (i >= next) { ++t; next = a.offsets[t + 1]; } }
      tt[j] = t;
    }
    const bool full = (wi + 1) * 4 <= nbytes;
    for (int w = 0; w < a.M; ++w) {
      uint32_t word = 0;
      if (full) word = reinterpret_cast<const uint32_t*>(a.q[w])[wi];
      else for (int b = 0; b < 4 && wi * 4 + b < nbytes; ++b) word |= (uint32_t)a.q[w][wi * 4 + b] << (8 * b);
#pragma unroll
      for (int j = 0; j < EPW; ++j) {
        const int code = ((int)(word << (32 - BITS * (j + 1)))) >> (32 - BITS);
        const float step = __fdiv_rn(a.scales[w][tt[j]], (float)S);
        acc[j] = __fadd_rn(acc[j], __fmul_rn((float)code, step));
      }
    }
#pragma unroll
    for (int j = 0; j < EPW; ++j)
      if (i0 + j < a.d) a.out[i0 + j] = __fdiv_rn(acc[j], (float)a.M);
  }
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + (int64_t)kT * kIter - 1) / ((int64_t)kT * kIter)); }

}  // namespace

dat_status launch_lamb(float* theta, const float* g, float* m, float* v, float* u, const int64_t* off, int T, int64_t d,
                       const LambParams& hp, double* norms, hipStream_t st) {
  hipLaunchKernelGGL(zero_f64_kernel, dim3((2 * T + 255) / 256), dim3(256), 0, st, norms, 2 * T);
  DAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(lamb_direction_kernel, dim3(blocks_for(d)), dim3(kT), 0, st, theta, g, m, v, u, off, T, d, hp, norms);
  DAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(lalr_apply_kernel, dim3(blocks_for(d)), dim3(kT), 0, st, theta, u, off, T, d, hp, norms);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace dat

using namespace dat;

extern "C" dat_status dat_aggregate(const uint8_t* const* q, const float* const* scales, int M, const int64_t* offsets_dev,
                                    int num_tensors, int64_t d, int bits, float* out, void* stream) {
  if (!q || !scales || !offsets_dev || !out || M < 1 || M > DAT_MAX_WORKERS || num_tensors < 1 || d < 0) return DAT_ERR_ARG;
  if (bits != 2 && bits != 4 && bits != 8 && bits != 16) return DAT_ERR_ARG;
  AggregateArgs a;
  for (int i = 0; i < M; ++i) {
    if (!q[i] || !scales[i] || !aligned(q[i], 4)) return DAT_ERR_ARG;
    a.q[i] = q[i]; a.scales[i] = scales[i];
  }
  a.M = M; a.offsets = offsets_dev; a.T = num_tensors; a.d = d; a.out = out;
  if (d == 0) return DAT_OK;
  const int64_t nwords = (d * bits + 31) / 32;
  hipStream_t st = (hipStream_t)stream;
  switch (bits) {
    case 2: hipLaunchKernelGGL(aggregate_kernel<2>, dim3(blocks_for(nwords)), dim3(kT), 0, st, a); break;
    case 4: hipLaunchKernelGGL(aggregate_kernel<4>, dim3(blocks_for(nwords)), dim3(kT), 0, st, a); break;
    case 8: hipLaunchKernelGGL(aggregate_kernel<8>, dim3(blocks_for(nwords)), dim3(kT), 0, st, a); break;
    default: hipLaunchKernelGGL(aggregate_kernel<16>, dim3(blocks_for(nwords)), dim3(kT), 0, st, a); break;
  }
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}
