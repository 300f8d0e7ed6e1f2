// Elementwise part of the inner maximisation (Alg. A1 step 5; unified PGD/FGSM update of Sec.
// "Methodologies"): start point z_0, the projected sign step
//     z <- clip(z + alpha*sign(G), -eps, eps);  z <- min(max(z, -x), 1-x)
// and the network input (x + z, clipped to [0,1], normalised, stored in the model's dtype),
// fused into one HBM pass.  A thread owns 4 pixels = 12 fp32 values = three 16-byte vectors
// of each stream, so every access is a full-width coalesced vector access.
// All fp32 operations are single correctly rounded operations (-ffp-contract=off).
#include "kernels.h"
#include "philox.h"

namespace dat {
namespace {

constexpr uint32_t kStreamInit = 1;
constexpr int kThreads = 256;

__device__ __forceinline__ float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ float box_clip(float d, float x) {
  return clampf(d, -x, __fsub_rn(1.0f, x));
}

__device__ __forceinline__ float sign_step(float d, float g, float eps, float alpha) {
  const float s = g > 0.0f ? alpha : (g < 0.0f ? -alpha : 0.0f);
  return clampf(__fadd_rn(d, s), -eps, eps);
}

struct InArgs { void* ptr; int bf16; int normalize; float m0, m1, m2, s0, s1, s2; int bh, bw; };

__device__ __forceinline__ float net_value(float x, float d, bool has_delta, const InArgs& a, int c) {
  float v = has_delta ? clampf(__fadd_rn(x, d), 0.0f, 1.0f) : x;
  if (a.normalize) {
    const float m = c == 0 ? a.m0 : (c == 1 ? a.m1 : a.m2);
    const float s = c == 0 ? a.s0 : (c == 1 ? a.s1 : a.s2);
    v = __fmul_rn(__fsub_rn(v, m), s);
  }
  return v;
}

// MODE 0: init, 1: update, 2: input only.  One thread = up to 4 pixels starting at pixel 4*q.
template <int MODE>
__global__ __launch_bounds__(kThreads) void attack_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ G,
                                                          const float* __restrict__ given,
                                                          float* __restrict__ delta, int64_t npix,
                                                          float eps, float alpha, int init_mode,
                                                          uint64_t seed, InArgs in) {
  const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t p0 = q * 4;
  if (p0 >= npix) return;
  const int64_t e0 = p0 * 3;
  const int np = (int)min((int64_t)4, npix - p0);
  const bool full = np == 4;
  float xv[12], dv[12], gv[12];
  if (full) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const float4 f = reinterpret_cast<const float4*>(x + e0)[j];
      xv[4 * j] = f.x; xv[4 * j + 1] = f.y; xv[4 * j + 2] = f.z; xv[4 * j + 3] = f.w;
    }
  } else {
    for (int j = 0; j < 12; ++j) xv[j] = j < np * 3 ? x[e0 + j] : 0.0f;
  }
  const bool has_delta = MODE != 2 || delta != nullptr;
  if (MODE == 0) {
    if (init_mode == DAT_INIT_UNIFORM) {
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const PhiloxWords w = philox_block((uint64_t)(e0 >> 2) + j, seed, kStreamInit);
        const uint32_t ww[4] = {w.w0, w.w1, w.w2, w.w3};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float t = __fsub_rn(__fmul_rn(2.0f, u24(ww[k])), 1.0f);   // exact: (2u-1) on a 2^-23 grid
          dv[4 * j + k] = __fmul_rn(t, eps);
        }
      }
    } else if (init_mode == DAT_INIT_GIVEN) {
      for (int j = 0; j < 12; ++j) dv[j] = j < np * 3 ? clampf(given[e0 + j], -eps, eps) : 0.0f;
    } else {
#pragma unroll
      for (int j = 0; j < 12; ++j) dv[j] = 0.0f;
    }
#pragma unroll
    for (int j = 0; j < 12; ++j) dv[j] = box_clip(dv[j], xv[j]);
  } else if (MODE == 1) {
    if (full) {
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const float4 f = reinterpret_cast<const float4*>(delta + e0)[j];
        dv[4 * j] = f.x; dv[4 * j + 1] = f.y; dv[4 * j + 2] = f.z; dv[4 * j + 3] = f.w;
        const float4 h = reinterpret_cast<const float4*>(G + e0)[j];
        gv[4 * j] = h.x; gv[4 * j + 1] = h.y; gv[4 * j + 2] = h.z; gv[4 * j + 3] = h.w;
      }
    } else {
      for (int j = 0; j < 12; ++j) { dv[j] = j < np * 3 ? delta[e0 + j] : 0.0f; gv[j] = j < np * 3 ? G[e0 + j] : 0.0f; }
    }
#pragma unroll
    for (int j = 0; j < 12; ++j) dv[j] = box_clip(sign_step(dv[j], gv[j], eps, alpha), xv[j]);
  } else {
    if (delta) for (int j = 0; j < 12; ++j) dv[j] = j < np * 3 ? delta[e0 + j] : 0.0f;
    else for (int j = 0; j < 12; ++j) dv[j] = 0.0f;
  }
  if (MODE != 2) {
    if (full) {
#pragma unroll
      for (int j = 0; j < 3; ++j)
        reinterpret_cast<float4*>(delta + e0)[j] = make_float4(dv[4 * j], dv[4 * j + 1], dv[4 * j + 2], dv[4 * j + 3]);
    } else {
      for (int j = 0; j < np * 3; ++j) delta[e0 + j] = dv[j];
    }
  }
  if (in.ptr) {
    float nv[12];
#pragma unroll
    for (int j = 0; j < 12; ++j) nv[j] = net_value(xv[j], dv[j], has_delta, in, j % 3);
    if (in.bf16) {
      uint4* dst = reinterpret_cast<uint4*>(in.ptr);          // 8 bf16 = 16 bytes per pixel
      for (int p = 0; p < np; ++p) {
        uint4 o;
        o.x = f2bf_pack(nv[3 * p], nv[3 * p + 1]);
        o.y = (uint32_t)f2bf(nv[3 * p + 2]);
        o.z = 0u; o.w = 0u;
        int64_t slot = p0 + p;
        if (in.bw) {   // 2x2 pixel blocks: pixel (n,h,w) -> block (n, h/2, w/2), position (h%2)*2 + w%2
          const uint32_t pix = (uint32_t)slot, w = pix % (uint32_t)in.bw, hn = pix / (uint32_t)in.bw;
          const uint32_t h = hn % (uint32_t)in.bh, n = hn / (uint32_t)in.bh;
          slot = ((int64_t)(n * (uint32_t)(in.bh >> 1) + (h >> 1)) * (uint32_t)(in.bw >> 1) + (w >> 1)) * 4 + (h & 1u) * 2 + (w & 1u);
        }
        dst[slot] = o;
      }
    } else {
      float* dst = reinterpret_cast<float*>(in.ptr) + e0;
      if (full) {
#pragma unroll
        for (int j = 0; j < 3; ++j)
          reinterpret_cast<float4*>(dst)[j] = make_float4(nv[4 * j], nv[4 * j + 1], nv[4 * j + 2], nv[4 * j + 3]);
      } else {
        for (int j = 0; j < np * 3; ++j) dst[j] = nv[j];
      }
    }
  }
}

InArgs pack(const NetInputDesc& d) {
  InArgs a;
  a.ptr = d.ptr; a.bf16 = d.bf16; a.normalize = d.normalize;
  a.m0 = d.mean[0]; a.m1 = d.mean[1]; a.m2 = d.mean[2];
  a.s0 = d.inv_std[0]; a.s1 = d.inv_std[1]; a.s2 = d.inv_std[2];
  a.bh = d.bf16 ? d.block_h : 0; a.bw = d.bf16 ? d.block_w : 0;
  return a;
}

unsigned grid_for(int64_t npix) { return (unsigned)(((npix + 3) / 4 + kThreads - 1) / kThreads); }

const NetInputDesc kNoInput = {nullptr, 0, 0, {0, 0, 0}, {1, 1, 1}, 0, 0};

}  // namespace

dat_status launch_attack_init(const float* x, int64_t npix, float eps, dat_init init, float* delta,
                              const NetInputDesc& in, hipStream_t st) {
  if (npix == 0) return DAT_OK;
  hipLaunchKernelGGL(attack_kernel<0>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, (const float*)nullptr,
                     init.delta0, delta, npix, eps, 0.0f, (int)init.mode, init.seed, pack(in));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_attack_update(const float* x, const float* G, float* delta, int64_t npix, float eps,
                                float alpha, const NetInputDesc& in, hipStream_t st) {
  if (npix == 0) return DAT_OK;
  hipLaunchKernelGGL(attack_kernel<1>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, G, (const float*)nullptr,
                     delta, npix, eps, alpha, 0, (uint64_t)0, pack(in));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_make_input(const float* x, const float* delta, int64_t npix, const NetInputDesc& in,
                             hipStream_t st) {
  if (npix == 0) return DAT_OK;
  hipLaunchKernelGGL(attack_kernel<2>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, (const float*)nullptr,
                     (const float*)nullptr, const_cast<float*>(delta), npix, 0.0f, 0.0f, 0, (uint64_t)0, pack(in));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace dat

using namespace dat;

static bool init_ok(const dat_init& init) {
  if (init.mode != DAT_INIT_ZERO && init.mode != DAT_INIT_UNIFORM && init.mode != DAT_INIT_GIVEN) return false;
  if (init.mode == DAT_INIT_GIVEN && (!init.delta0 || !aligned(init.delta0, 4))) return false;
  return true;
}

extern "C" dat_status dat_pgd_init(const float* x, int64_t N, float eps, dat_init init, float* delta,
                                   void* stream) {
  if (!x || !delta || N < 0 || N % 3 != 0 || !(eps >= 0.0f) || !init_ok(init)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(delta, 16)) return DAT_ERR_ARG;
  return launch_attack_init(x, N / 3, eps, init, delta, kNoInput, (hipStream_t)stream);
}

extern "C" dat_status dat_pgd_update(const float* x, const float* G, float* delta, int64_t N, float eps,
                                     float alpha, void* stream) {
  if (!x || !G || !delta || N < 0 || N % 3 != 0 || !(eps >= 0.0f) || !(alpha >= 0.0f)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(G, 16) || !aligned(delta, 16)) return DAT_ERR_ARG;
  return launch_attack_update(x, G, delta, N / 3, eps, alpha, kNoInput, (hipStream_t)stream);
}
