// fp32 convolutions by direct summation (one thread per output element, fp64 accumulate): the
// DAT_F32 path.  Small networks only (the tiny CNN of the fp32 configuration, and reduced-size
// runs of the ResNets that cross-check the bf16 MFMA path); not a tuned kernel.
#include "kernels.h"

namespace dat {
namespace {
constexpr int kT = 256;

__global__ __launch_bounds__(kT) void direct_fwd_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                        const float* __restrict__ res, float* __restrict__ y, ConvGeom g) {
  const int64_t o = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (o >= (int64_t)g.B * g.Ho * g.Wo * g.Cout) return;
  const int co = (int)(o % g.Cout);
  int64_t p = o / g.Cout;
  const int wo = (int)(p % g.Wo); p /= g.Wo;
  const int ho = (int)(p % g.Ho);
  const int n = (int)(p / g.Ho);
  double acc = 0.0;
  for (int r = 0; r < g.k; ++r) {
    const int hi = ho * g.stride + r - g.pad;
    if (hi < 0 || hi >= g.H) continue;
    for (int s = 0; s < g.k; ++s) {
      const int wi = wo * g.stride + s - g.pad;
      if (wi < 0 || wi >= g.W) continue;
      const float* xp = x + (((int64_t)n * g.H + hi) * g.W + wi) * g.Cin;
      const float* wp = w + (((int64_t)co * g.k + r) * g.k + s) * g.Cin;
      for (int ci = 0; ci < g.Cin; ++ci) acc += (double)xp[ci] * (double)wp[ci];
    }
  }
  if (res) acc += (double)res[o];
  y[o] = (float)acc;
}

__global__ __launch_bounds__(kT) void direct_bwd_data_kernel(const float* __restrict__ dy, const float* __restrict__ w,
                                                             float* __restrict__ dx, ConvGeom g, int accumulate) {
  const int64_t o = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (o >= (int64_t)g.B * g.H * g.W * g.Cin) return;
  const int ci = (int)(o % g.Cin);
  int64_t p = o / g.Cin;
  const int wi = (int)(p % g.W); p /= g.W;
  const int hi = (int)(p % g.H);
  const int n = (int)(p / g.H);
  double acc = 0.0;
  for (int r = 0; r < g.k; ++r) {
    const int th = hi + g.pad - r;
    if (th < 0 || th % g.stride != 0) continue;
    const int ho = th / g.stride;
    if (ho >= g.Ho) continue;
    for (int s = 0; s < g.k; ++s) {
      const int tw = wi + g.pad - s;
      if (tw < 0 || tw % g.stride != 0) continue;
      const int wo = tw / g.stride;
      if (wo >= g.Wo) continue;
      const float* dp = dy + (((int64_t)n * g.Ho + ho) * g.Wo + wo) * g.Cout;
      const float* wp = w + ((int64_t)r * g.k + s) * g.Cin + ci;
      const int64_t wstride = (int64_t)g.k * g.k * g.Cin;
      for (int co = 0; co < g.Cout; ++co) acc += (double)dp[co] * (double)wp[co * wstride];
    }
  }
  if (accumulate) acc += (double)dx[o];
  dx[o] = (float)acc;
}

// one wavefront per weight element: lanes stride over the B*Ho*Wo output pixels
__global__ __launch_bounds__(kT) void direct_bwd_weight_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                               float* __restrict__ dw, ConvGeom g, float scale) {
  const int64_t wave = ((int64_t)blockIdx.x * kT + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (wave >= (int64_t)g.Cout * g.k * g.k * g.Cin) return;
  const int ci = (int)(wave % g.Cin);
  int64_t p = wave / g.Cin;
  const int s = (int)(p % g.k); p /= g.k;
  const int r = (int)(p % g.k);
  const int co = (int)(p / g.k);
  double acc = 0.0;
  const int64_t npix = (int64_t)g.B * g.Ho * g.Wo;
  for (int64_t q = lane; q < npix; q += 64) {
    const int wo = (int)(q % g.Wo);
    const int ho = (int)((q / g.Wo) % g.Ho);
    const int n = (int)(q / ((int64_t)g.Wo * g.Ho));
    const int hi = ho * g.stride + r - g.pad, wi = wo * g.stride + s - g.pad;
    if (hi < 0 || hi >= g.H || wi < 0 || wi >= g.W) continue;
    acc += (double)dy[q * g.Cout + co] * (double)x[(((int64_t)n * g.H + hi) * g.W + wi) * g.Cin + ci];
  }
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) acc += __shfl_xor(acc, sft);
  if (lane == 0) dw[wave] = (float)(acc * (double)scale);
}

inline unsigned nblk(int64_t n) { return (unsigned)((n + kT - 1) / kT); }
}  // namespace

dat_status conv_direct_forward(const float* x, const float* w, const float* res, float* y, const ConvGeom& g, hipStream_t st) {
  hipLaunchKernelGGL(direct_fwd_kernel, dim3(nblk((int64_t)g.B * g.Ho * g.Wo * g.Cout)), dim3(kT), 0, st, x, w, res, y, g);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status conv_direct_backward_data(const float* dy, const float* w, float* dx, const ConvGeom& g, bool accumulate, hipStream_t st) {
  hipLaunchKernelGGL(direct_bwd_data_kernel, dim3(nblk((int64_t)g.B * g.H * g.W * g.Cin)), dim3(kT), 0, st, dy, w, dx, g, (int)accumulate);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status conv_direct_backward_weight(const float* x, const float* dy, float* dw, const ConvGeom& g, float scale, hipStream_t st) {
  hipLaunchKernelGGL(direct_bwd_weight_kernel, dim3(nblk((int64_t)g.Cout * g.k * g.k * g.Cin * 64)), dim3(kT), 0, st, x, dy, dw, g, scale);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace dat
