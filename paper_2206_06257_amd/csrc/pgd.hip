// Elementwise part of the inner maximisation (Alg. A1 step 5; unified PGD/FGSM update of Sec.
// "Methodologies"): start point z_0, the projected sign step
//     z <- clip(z + alpha*sign(G), -eps, eps);  z <- min(max(z, -x), 1-x)
// and the network input (x + z, clipped to [0,1], normalised, stored in the model's dtype),
// fused into one HBM pass whose wavefronts read and write whole kilobytes of consecutive memory.
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

// MODE 0: init, 1: update, 2: input only, 3: update with the gradient read from the bf16 network-input gradient
// (`gnet`, laid out like the network input: one 16-byte vector of 8 channels per pixel, or -- behind a 7x7/2 stem --
// 2x2 pixel blocks of 4 channels, 8 bytes per pixel) instead of an fp32 copy -- only its sign
// enters the step, and the positive normalisation scale does not change it.  A workgroup owns 1024 consecutive pixels = 768 float4 of each
// fp32 stream; thread t touches float4 number j*256 + t (j = 0..2) of that chunk, so every load and
// store of a wavefront covers 1 KB of consecutive memory.  The update itself is elementwise.  The bf16
// network input is stored per pixel (one 16-byte vector of 8 channels), so the rounded values are
// regrouped through LDS: thread t then writes pixels 4t .. 4t+3 of the chunk.
constexpr int kPixPerBlock = 4 * kThreads;        // 1024

__device__ __forceinline__ void load4(const float* __restrict__ p, int64_t e, int64_t n, float v[4]) {
  if (e + 4 <= n) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 f = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p + e));   // streamed once
    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = e + k < n ? p[e + k] : 0.0f;
  }
}

__device__ __forceinline__ void store4(float* __restrict__ p, int64_t e, int64_t n, const float v[4]) {
  if (e + 4 <= n) {
    *reinterpret_cast<float4*>(p + e) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) if (e + k < n) p[e + k] = v[k];
  }
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void attack_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ G,
                                                          const float* __restrict__ given,
                                                          float* __restrict__ delta, int64_t npix,
                                                          float eps, float alpha, int init_mode,
                                                          uint64_t seed, InArgs in, const void* __restrict__ gnet) {
  __shared__ __attribute__((aligned(16))) uint16_t stage[kPixPerBlock * 3];
  __shared__ __attribute__((aligned(16))) uint16_t gstage[MODE == 3 ? kPixPerBlock * 3 : 8];
  const int tid = threadIdx.x;
  const int64_t n = npix * 3;
  const int64_t ebase = (int64_t)blockIdx.x * (kPixPerBlock * 3);
  const bool has_delta = MODE != 2 || delta != nullptr;
  const bool to_lds = in.ptr && in.bf16;
  // where this thread's pixels 4t .. 4t+3 live in the per-pixel tensors (network input and its gradient)
  const int64_t p0 = (int64_t)blockIdx.x * kPixPerBlock + 4 * tid;
  int64_t slot[4];
  if (in.bw && (in.bw & 3) == 0) {
    // 2x2 pixel blocks, image width a multiple of 4: the thread's four pixels share a row (p0 is a multiple of 4), so
    // one decomposition of p0 serves all of them (the divisions by the run-time width and height are ~35 VALU
    // operations each)
    const uint32_t pix = (uint32_t)p0, w0 = pix % (uint32_t)in.bw, hn = pix / (uint32_t)in.bw;
    const uint32_t h = hn % (uint32_t)in.bh, nimg = hn / (uint32_t)in.bh;
    const int64_t rowbase = (int64_t)(nimg * (uint32_t)(in.bh >> 1) + (h >> 1)) * (uint32_t)(in.bw >> 1);
#pragma unroll
    for (int p = 0; p < 4; ++p) slot[p] = (rowbase + ((w0 + p) >> 1)) * 4 + (h & 1u) * 2 + ((w0 + p) & 1u);
  } else {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      slot[p] = p0 + p;
      if (in.bw) {   // 2x2 pixel blocks: pixel (n,h,w) -> block (n, h/2, w/2), position (h%2)*2 + w%2
        const uint32_t pix = (uint32_t)slot[p], ww = pix % (uint32_t)in.bw, hn = pix / (uint32_t)in.bw;
        const uint32_t h = hn % (uint32_t)in.bh, nimg = hn / (uint32_t)in.bh;
        slot[p] = ((int64_t)(nimg * (uint32_t)(in.bh >> 1) + (h >> 1)) * (uint32_t)(in.bw >> 1) + (ww >> 1)) * 4 + (h & 1u) * 2 + (ww & 1u);
      }
    }
  }
  // every global load of the update is issued before the first barrier (the pixels and the perturbation below, the
  // gradient here): one memory round trip per workgroup instead of two
  float xs[3][4], ds[3][4];
  if (MODE == 1 || MODE == 3) {
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int64_t e = ebase + 4 * (int64_t)(j * kThreads + tid);
      if (e < n) { load4(x, e, n, xs[j]); load4(delta, e, n, ds[j]); }
    }
  }
  if (MODE == 3) {
    // the three gradient channels of each pixel, regrouped through LDS into the element order of the fp32 streams
    // the first three channels of a pixel are its first 8 bytes; pixels are 16 bytes apart, 8 in the blocked layout
    const unsigned char* gsrc = reinterpret_cast<const unsigned char*>(gnet);
    const int pix_bytes = in.bw ? 8 : 16;
    uint32_t gw[4][2];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      gw[p][0] = 0u; gw[p][1] = 0u;
      if (p0 + p < npix) { const uint2 v = *reinterpret_cast<const uint2*>(gsrc + slot[p] * pix_bytes); gw[p][0] = v.x; gw[p][1] = v.y; }
    }
    // halfwords 3p .. 3p+2 of the thread's 12: (c0 c1) (c2 c0') (c1' c2') ...
    uint32_t o[6];
    o[0] = gw[0][0];
    o[1] = (gw[0][1] & 0xffffu) | (gw[1][0] << 16);
    o[2] = (gw[1][0] >> 16) | (gw[1][1] << 16);
    o[3] = gw[2][0];
    o[4] = (gw[2][1] & 0xffffu) | (gw[3][0] << 16);
    o[5] = (gw[3][0] >> 16) | (gw[3][1] << 16);
    uint2* d2 = reinterpret_cast<uint2*>(&gstage[12 * tid]);
    d2[0] = make_uint2(o[0], o[1]); d2[1] = make_uint2(o[2], o[3]); d2[2] = make_uint2(o[4], o[5]);
    __syncthreads();
  }
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int f = j * kThreads + tid;               // float4 number inside the chunk
    const int64_t e = ebase + 4 * (int64_t)f;
    float xv[4], dv[4];
    if (e < n) {
      if (MODE == 1 || MODE == 3) {
#pragma unroll
        for (int k = 0; k < 4; ++k) { xv[k] = xs[j][k]; dv[k] = ds[j][k]; }
      } else {
        load4(x, e, n, xv);
      }
      if (MODE == 0) {
        if (init_mode == DAT_INIT_UNIFORM) {
          const PhiloxWords w = philox_block((uint64_t)(e >> 2), seed, kStreamInit);
          const uint32_t ww[4] = {w.w0, w.w1, w.w2, w.w3};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float t = __fsub_rn(__fmul_rn(2.0f, u24(ww[k])), 1.0f);   // exact: (2u-1) on a 2^-23 grid
            dv[k] = __fmul_rn(t, eps);
          }
        } else if (init_mode == DAT_INIT_GIVEN) {
          load4(given, e, n, dv);
#pragma unroll
          for (int k = 0; k < 4; ++k) dv[k] = clampf(dv[k], -eps, eps);
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k) dv[k] = 0.0f;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) dv[k] = box_clip(dv[k], xv[k]);
      } else if (MODE == 1) {
        float gv[4];
        load4(G, e, n, gv);
#pragma unroll
        for (int k = 0; k < 4; ++k) dv[k] = box_clip(sign_step(dv[k], gv[k], eps, alpha), xv[k]);
      } else if (MODE == 3) {
        const uint2 gp = *reinterpret_cast<const uint2*>(&gstage[4 * f]);
        const float gv[4] = {__uint_as_float(gp.x << 16), __uint_as_float(gp.x & 0xffff0000u), __uint_as_float(gp.y << 16), __uint_as_float(gp.y & 0xffff0000u)};
#pragma unroll
        for (int k = 0; k < 4; ++k) dv[k] = box_clip(sign_step(dv[k], gv[k], eps, alpha), xv[k]);
      } else {
        if (delta) load4(delta, e, n, dv);
        else {
#pragma unroll
          for (int k = 0; k < 4; ++k) dv[k] = 0.0f;
        }
      }
      if (MODE != 2) store4(delta, e, n, dv);
      if (in.ptr) {
        float nv[4];
        const int c0 = (4 * f) % 3;                 // the chunk starts on a pixel boundary
#pragma unroll
        for (int k = 0; k < 4; ++k) { int c = c0 + k; c = c >= 3 ? c - 3 : c; c = c >= 3 ? c - 3 : c; nv[k] = net_value(xv[k], dv[k], has_delta, in, c); }
        if (to_lds) {
          uint2 pk;
          pk.x = f2bf_pack(nv[0], nv[1]); pk.y = f2bf_pack(nv[2], nv[3]);
          *reinterpret_cast<uint2*>(&stage[4 * f]) = pk;
        } else {
          store4(reinterpret_cast<float*>(in.ptr), e, n, nv);
        }
      }
    }
  }
  if (!to_lds) return;
  __syncthreads();
  if (p0 >= npix) return;
  const int np = (int)min((int64_t)4, npix - p0);
  uint32_t w[6];                                     // 12 bf16 = pixels 4t .. 4t+3
  {
    const uint2* src = reinterpret_cast<const uint2*>(&stage[12 * tid]);
    const uint2 a = src[0], b = src[1], c = src[2];
    w[0] = a.x; w[1] = a.y; w[2] = b.x; w[3] = b.y; w[4] = c.x; w[5] = c.y;
  }
  // halfwords 3p, 3p+1, 3p+2 of the 12 -> (c0 c1) (c2 0) of pixel p
  uint2 o[4];
  o[0] = make_uint2(w[0], w[1] & 0xffffu);
  o[1] = make_uint2((w[1] >> 16) | (w[2] << 16), w[2] >> 16);
  o[2] = make_uint2(w[3], w[4] & 0xffffu);
  o[3] = make_uint2((w[4] >> 16) | (w[5] << 16), w[5] >> 16);
  if (in.bw) {
    // 2x2 pixel blocks of 4 channels: 8 bytes per pixel; two pixels of one row and one block are 16 contiguous bytes
    uint2* dst = reinterpret_cast<uint2*>(in.ptr);
    if ((in.bw & 3) == 0 && np == 4) {
      *reinterpret_cast<uint4*>(dst + slot[0]) = make_uint4(o[0].x, o[0].y, o[1].x, o[1].y);
      *reinterpret_cast<uint4*>(dst + slot[2]) = make_uint4(o[2].x, o[2].y, o[3].x, o[3].y);
    } else {
#pragma unroll
      for (int p = 0; p < 4; ++p) if (p < np) dst[slot[p]] = o[p];
    }
  } else {
    uint4* dst = reinterpret_cast<uint4*>(in.ptr);      // 8 bf16 = 16 bytes per pixel
#pragma unroll
    for (int p = 0; p < 4; ++p) if (p < np) dst[slot[p]] = make_uint4(o[p].x, o[p].y, 0u, 0u);
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

unsigned grid_for(int64_t npix) { return (unsigned)((npix + kPixPerBlock - 1) / kPixPerBlock); }

// the 2x2-block layout decomposes the pixel index in 32 bits
bool pixels_ok(int64_t npix, const NetInputDesc& in) { return !(in.bf16 && in.block_w) || npix < (1ll << 32); }

const NetInputDesc kNoInput = {nullptr, 0, 0, {0, 0, 0}, {1, 1, 1}, 0, 0};

}  // namespace

dat_status launch_attack_init(const float* x, int64_t npix, float eps, dat_init init, float* delta,
                              const NetInputDesc& in, hipStream_t st) {
  if (npix == 0) return DAT_OK;
  if (!pixels_ok(npix, in)) return DAT_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(attack_kernel<0>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, (const float*)nullptr,
                     init.delta0, delta, npix, eps, 0.0f, (int)init.mode, init.seed, pack(in), (const void*)nullptr);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_attack_update(const float* x, const float* G, float* delta, int64_t npix, float eps,
                                float alpha, const NetInputDesc& in, hipStream_t st) {
  if (npix == 0) return DAT_OK;
  if (!pixels_ok(npix, in)) return DAT_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(attack_kernel<1>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, G, (const float*)nullptr,
                     delta, npix, eps, alpha, 0, (uint64_t)0, pack(in), (const void*)nullptr);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_attack_update_netgrad(const float* x, const void* gnet, float* delta, int64_t npix, float eps,
                                        float alpha, const NetInputDesc& in, hipStream_t st) {
  if (npix == 0) return DAT_OK;
  if (!in.ptr || !in.bf16 || !gnet) return DAT_ERR_ARG;
  if (!pixels_ok(npix, in)) return DAT_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(attack_kernel<3>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, (const float*)nullptr, (const float*)nullptr,
                     delta, npix, eps, alpha, 0, (uint64_t)0, pack(in), gnet);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_make_input(const float* x, const float* delta, int64_t npix, const NetInputDesc& in,
                             hipStream_t st) {
  if (npix == 0) return DAT_OK;
  if (!pixels_ok(npix, in)) return DAT_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(attack_kernel<2>, dim3(grid_for(npix)), dim3(kThreads), 0, st, x, (const float*)nullptr,
                     (const float*)nullptr, const_cast<float*>(delta), npix, 0.0f, 0.0f, 0, (uint64_t)0, pack(in), (const void*)nullptr);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace dat

using namespace dat;

static bool init_ok(const dat_init& init) {
  if (init.mode != DAT_INIT_ZERO && init.mode != DAT_INIT_UNIFORM && init.mode != DAT_INIT_GIVEN) return false;
  if (init.mode == DAT_INIT_GIVEN && (!init.delta0 || !aligned(init.delta0, 16))) return false;   // read as 16-byte vectors
  return true;
}

extern "C" dat_status dat_pgd_init(const float* x, int64_t N, float eps, dat_init init, float* delta,
                                   void* stream) {
  if (!x || !delta || N < 0 || N % 3 != 0 || !(eps >= 0.0f) || !init_ok(init)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(delta, 16)) return DAT_ERR_ARG;
  return launch_attack_init(x, N / 3, eps, init, delta, kNoInput, (hipStream_t)stream);
}

extern "C" dat_status dat_make_xadv(const float* x, const float* delta, int64_t N, float* x_adv, void* stream) {
  if (!x || !delta || !x_adv || N < 0 || N % 3 != 0) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(delta, 16) || !aligned(x_adv, 16)) return DAT_ERR_ARG;
  const NetInputDesc out = {x_adv, 0, 0, {0, 0, 0}, {1, 1, 1}, 0, 0};   // fp32 pixels, no normalisation
  return launch_make_input(x, delta, N / 3, out, (hipStream_t)stream);
}

extern "C" dat_status dat_pgd_update(const float* x, const float* G, float* delta, int64_t N, float eps,
                                     float alpha, void* stream) {
  if (!x || !G || !delta || N < 0 || N % 3 != 0 || !(eps >= 0.0f) || !(alpha >= 0.0f)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(G, 16) || !aligned(delta, 16)) return DAT_ERR_ARG;
  return launch_attack_update(x, G, delta, N / 3, eps, alpha, kNoInput, (hipStream_t)stream);
}
