// Non-convolution layers of the networks and their backward passes: train-mode batch
// normalisation fused with residual add and ReLU, bias+ReLU, 3x3/2 max-pool, global average
// pool, the linear classifier, and the softmax cross-entropy gradient.  All are HBM-streaming
// kernels over NHWC tensors: a thread owns 8 consecutive channels of one pixel (one 16-byte
// vector in bf16, two in fp32) so that a wavefront touches contiguous memory.
//
// Per-channel reductions (batch statistics, BN/bias gradients) are two-stage and
// deterministic: slabs of rows are reduced in registers + LDS in a fixed order into a
// [slab][channel] table, which one thread per channel then sums in fp64.
#include "kernels.h"

namespace dat {
namespace {

constexpr int kT = 256;
constexpr int kMaxSlabs = 1024;      // slabs of a per-channel reduction
constexpr int kMaxApplySlabs = 8192;  // slabs of an elementwise pass

template <typename T> struct V8;
template <> struct V8<float> {
  struct Raw { float4 a, b; };
  static __device__ __forceinline__ Raw load_raw_nt(const float* p) { return Raw{reinterpret_cast<const float4*>(p)[0], reinterpret_cast<const float4*>(p)[1]}; }
  static __device__ __forceinline__ void unpack(const Raw& r, float v[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
  }
  static __device__ __forceinline__ void load_nt(const float* p, float v[8]) { load(p, v); }
  static __device__ __forceinline__ void load(const float* p, float v[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float v[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
  }
};
template <> struct V8<bf16_t> {
  // the 16 bytes as loaded (streaming read), unpacked only where they are used: four registers in flight, not eight
  typedef uint32_t Raw __attribute__((ext_vector_type(4)));
  static __device__ __forceinline__ Raw load_raw_nt(const bf16_t* p) { return __builtin_nontemporal_load(reinterpret_cast<const Raw*>(p)); }
  static __device__ __forceinline__ void unpack(const Raw& a, float v[8]) {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(w[j] << 16); v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u); }
  }
  // streaming read: the line is not needed again soon (leaves the caches to the tensors that are)
  static __device__ __forceinline__ void load_nt(const bf16_t* p, float v[8]) {
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    const u4 a = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(w[j] << 16); v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u); }
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float v[8]) {
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[2 * j] = __uint_as_float(w[j] << 16); v[2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u); }
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float v[8]) {
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = f2bf_pack(v[2 * j], v[2 * j + 1]);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

__device__ __forceinline__ void load8f(const float* p, float v[8]) { V8<float>::load(p, v); }

struct SlabPlan { int tpr, rpp, nslabs; int64_t rows_per_slab; };

// Row slabs for the streaming kernels: a workgroup owns `rows_per_slab` consecutive rows; thread
// (rr, cv) = (tid / tpr, tid % tpr) walks rows rr, rr+rpp, ... of the slab for channel vector cv,
// so per-channel parameters stay in registers.  Enough slabs to fill 256 CUs several times over.
SlabPlan plan_slabs(int64_t rows, int C, int max_slabs) {
  SlabPlan p;
  p.tpr = C / 8;
  p.rpp = kT / p.tpr;
  if (p.rpp < 1) p.rpp = 1;
  int64_t want = (rows + (int64_t)p.rpp * 8 - 1) / ((int64_t)p.rpp * 8);
  p.nslabs = (int)(want < 1 ? 1 : (want > max_slabs ? max_slabs : want));
  p.rows_per_slab = (rows + p.nslabs - 1) / p.nslabs;
  p.rows_per_slab = (p.rows_per_slab + p.rpp - 1) / p.rpp * p.rpp;
  p.nslabs = (int)((rows + p.rows_per_slab - 1) / p.rows_per_slab);
  return p;
}

// ---- backward of BN + ReLU feeding a 3x3/2 max-pool, on 2x2 pixel blocks ------------------------
// A thread owns the pixels (2i+a, 2j+b), a, b in {0,1}, of 8 channels.  POOL: d(out) of those pixels is
// not read from memory but gathered from the pool's output gradient -- the four pixels lie in the windows
// (i+dh, j+dw), dh, dw in {0,1}, at window position (a+1-2dh, b+1-2dw) when both are >= 0, and receive the
// gradient of every window whose recorded arg-max position that is, summed in fp32 in the order
// (dh, dw) = (0,0), (0,1), (1,0), (1,1) and rounded once to the storage type: the value the pool's own
// backward pass would have stored.  Four window loads serve four pixels.
struct PoolArgs {
  const uint8_t* arg;     // [B][Ho][Wo][C] window position of the maximum
  const void* dpooled;    // [B][Ho][Wo][C]
  int B, H, W, Ho, Wo;
};

template <typename T, bool POOL>
__device__ __forceinline__ void block_dout(const PoolArgs& pa, const T* __restrict__ dout, int n, int i, int j, int C, int c0, float g[2][2][8]) {
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) g[a][b][e] = 0.f;
  if (POOL) {
#pragma unroll
    for (int dh = 0; dh < 2; ++dh)
#pragma unroll
      for (int dw = 0; dw < 2; ++dw) {
        const int ho = i + dh, wo = j + dw;
        if (ho >= pa.Ho || wo >= pa.Wo) continue;
        const int64_t o = (((int64_t)n * pa.Ho + ho) * pa.Wo + wo) * C + c0;
        const uint2 pk = *reinterpret_cast<const uint2*>(pa.arg + o);
        float d[8]; V8<T>::load(reinterpret_cast<const T*>(pa.dpooled) + o, d);
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const int r = a + 1 - 2 * dh, c = b + 1 - 2 * dw;
            if (r < 0 || c < 0) continue;
            const uint32_t me = 3 * r + c;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const uint32_t pe = ((e < 4 ? pk.x : pk.y) >> (8 * (e & 3))) & 0xffu;
              if (pe == me) g[a][b][e] += d[e];
            }
          }
      }
    if (sizeof(T) == 2) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int e = 0; e < 8; ++e) g[a][b][e] = bf2f(f2bf(g[a][b][e]));
    }
  } else {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int h = 2 * i + a, w = 2 * j + b;
        if (h < pa.H && w < pa.W) V8<T>::load(dout + (((int64_t)n * pa.H + h) * pa.W + w) * C + c0, g[a][b]);
      }
  }
}

// (sum dy, sum dy*xhat) per channel, dy = d(out) .* mask, one slab of [2][C] per workgroup: a workgroup walks
// `blocks_per_slab` consecutive 2x2 blocks, kT / (C/8) at a time; the threads of one channel vector are folded
// through LDS in a fixed order.
template <typename T, bool POOL>
__global__ __launch_bounds__(kT) void block_reduce_kernel(const T* __restrict__ x, const uint8_t* __restrict__ mask, const T* __restrict__ dout,
                                                          const float* __restrict__ mean, const float* __restrict__ rstd, int C, int tpr,
                                                          int64_t nblocks, int64_t blocks_per_slab, float* __restrict__ partial, PoolArgs pa) {
  __shared__ float red[2][kT][8];
  const int tid = threadIdx.x, rr = tid / tpr, cv = tid % tpr, rpp = kT / tpr;
  const int c0 = cv * 8;
  const int Hb = (pa.H + 1) / 2, Wb = (pa.W + 1) / 2;
  float a1[8], a2[8], mu[8], rs[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { a1[e] = 0.f; a2[e] = 0.f; }
  load8f(mean + c0, mu); load8f(rstd + c0, rs);
  const int64_t b0 = (int64_t)blockIdx.x * blocks_per_slab, b1 = min(nblocks, b0 + blocks_per_slab);
  if (rr < rpp) {
    for (int64_t blk = b0 + rr; blk < b1; blk += rpp) {
      // (block counts stay below 2^31, checked on the host: 32-bit divisions, a quarter of the 64-bit ones' cost)
      const uint32_t t = (uint32_t)blk / (uint32_t)Wb;
      const int j = (int)((uint32_t)blk - t * (uint32_t)Wb), n = (int)(t / (uint32_t)Hb), i = (int)(t - (uint32_t)n * (uint32_t)Hb);
      float g[2][2][8];
      block_dout<T, POOL>(pa, dout, n, i, j, C, c0, g);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int h = 2 * i + a, w = 2 * j + b;
          if (h >= pa.H || w >= pa.W) continue;
          const int64_t o = (((int64_t)n * pa.H + h) * pa.W + w) * C + c0;
          float xv[8]; V8<T>::load(x + o, xv);
          const uint32_t mk = mask[o >> 3];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float ge = ((mk >> e) & 1u) ? g[a][b][e] : 0.f;
            a1[e] += ge; a2[e] += ge * ((xv[e] - mu[e]) * rs[e]);
          }
        }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { red[0][tid][e] = a1[e]; red[1][tid][e] = a2[e]; }
  __syncthreads();
  if (rr == 0) {
    for (int q = 1; q < rpp; ++q) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { a1[e] += red[0][q * tpr + cv][e]; a2[e] += red[1][q * tpr + cv][e]; }
    }
    float* p = partial + (int64_t)blockIdx.x * 2 * C;
    V8<float>::store(p + c0, a1);
    V8<float>::store(p + C + c0, a2);
  }
}

// dx = bn_input_grad(d(out) .* mask, x, constants) for the four pixels of a block.
template <typename T, bool POOL>
__global__ __launch_bounds__(kT) void block_apply_kernel(const T* __restrict__ x, const uint8_t* __restrict__ mask, const T* __restrict__ dout,
                                                         T* __restrict__ dx, int dx_acc, int C, int tpr, int64_t nblocks,
                                                         const float* __restrict__ tab, PoolArgs pa) {
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= nblocks * tpr) return;
  // (vector counts stay below 2^31, checked on the host: 32-bit divisions)
  const uint32_t blk = (uint32_t)v / (uint32_t)tpr;
  const int cv = (int)((uint32_t)v - blk * (uint32_t)tpr);
  const int c0 = cv * 8;
  const int Hb = (pa.H + 1) / 2, Wb = (pa.W + 1) / 2;
  const uint32_t t = blk / (uint32_t)Wb;
  const int j = (int)(blk - t * (uint32_t)Wb), n = (int)(t / (uint32_t)Hb), i = (int)(t - (uint32_t)n * (uint32_t)Hb);
  float ka[8], kp[8], kq[8], mu[8];
  load8f(tab + cv * 32, ka); load8f(tab + cv * 32 + 8, kp); load8f(tab + cv * 32 + 16, kq); load8f(tab + cv * 32 + 24, mu);
  float g[2][2][8];
  block_dout<T, POOL>(pa, dout, n, i, j, C, c0, g);
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int h = 2 * i + a, w = 2 * j + b;
      if (h >= pa.H || w >= pa.W) continue;
      const int64_t o = (((int64_t)n * pa.H + h) * pa.W + w) * C + c0;
      float xv[8], q[8]; V8<T>::load(x + o, xv);
      const uint32_t mk = mask[o >> 3];
#pragma unroll
      for (int e = 0; e < 8; ++e) q[e] = bn_input_grad(((mk >> e) & 1u) ? g[a][b][e] : 0.f, xv[e], ka[e], kp[e], kq[e], mu[e]);
      if (dx_acc) {
        float od[8]; V8<T>::load(dx + o, od);
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] += od[e];
      }
      V8<T>::store(dx + o, q);
    }
}

// ---- per-channel two-value reduction -------------------------------------------------------
// MODE 0: (sum x, sum x^2)            -- batch statistics
// MODE 1: (sum dy, sum dy*xhat)       -- BN backward, dy = dout masked by out > 0 when relu
// MODE 2: (sum dy, 0)                 -- bias backward
//
// dual_reduce_kernel: MODE 1 for two normalisations that share dy (the last one of a residual branch and the
// one on its projection shortcut, whose sum passes one ReLU): (sum dy, sum dy*xhat) and (sum dy, sum dy*xhat2)
// from one read of dy and the mask.
template <typename T>
__global__ __launch_bounds__(kT) void dual_reduce_kernel(const T* __restrict__ x, const T* __restrict__ x2,
                                                         const uint8_t* __restrict__ mask, const T* __restrict__ dout,
                                                         const float* __restrict__ mean, const float* __restrict__ rstd,
                                                         const float* __restrict__ mean2, const float* __restrict__ rstd2,
                                                         int64_t rows, int C, int tpr, int rpp, int64_t rows_per_slab,
                                                         float* __restrict__ partial, float* __restrict__ partial2) {
  __shared__ float red[3][kT][8];
  const int tid = threadIdx.x, rr = tid / tpr, cv = tid % tpr;
  const bool active = rr < rpp;
  const int c0 = cv * 8;
  float a1[8], a2[8], a3[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { a1[j] = 0.f; a2[j] = 0.f; a3[j] = 0.f; }
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_slab;
  const int64_t r1 = min(rows, r0 + rows_per_slab);
  if (active) {
    float mu[8], rs[8], mu2[8], rs2[8];
    load8f(mean + c0, mu); load8f(rstd + c0, rs); load8f(mean2 + c0, mu2); load8f(rstd2 + c0, rs2);
    constexpr int U = 2;
    for (int64_t rb = r0 + rr; rb < r1; rb += (int64_t)rpp * U) {
      float xv[U][8], yv[U][8], gv[U][8];
      uint32_t mk[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t r = rb + (int64_t)u * rpp;
        const int64_t o = r * C + c0;
        mk[u] = 0xffu;
        if (r < r1) {
          V8<T>::load(x + o, xv[u]); V8<T>::load(x2 + o, yv[u]); V8<T>::load(dout + o, gv[u]);
          if (mask) mk[u] = mask[o >> 3];
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t r = rb + (int64_t)u * rpp;
        if (r < r1) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float g = ((mk[u] >> j) & 1u) ? gv[u][j] : 0.f;
            a1[j] += g; a2[j] += g * ((xv[u][j] - mu[j]) * rs[j]); a3[j] += g * ((yv[u][j] - mu2[j]) * rs2[j]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) { red[0][tid][j] = a1[j]; red[1][tid][j] = a2[j]; red[2][tid][j] = a3[j]; }
  __syncthreads();
  if (rr == 0) {
    for (int q = 1; q < rpp; ++q) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { a1[j] += red[0][q * tpr + cv][j]; a2[j] += red[1][q * tpr + cv][j]; a3[j] += red[2][q * tpr + cv][j]; }
    }
    float* p = partial + (int64_t)blockIdx.x * 2 * C;
    V8<float>::store(p + c0, a1);
    V8<float>::store(p + C + c0, a2);
    float* p2 = partial2 + (int64_t)blockIdx.x * 2 * C;
    V8<float>::store(p2 + c0, a1);
    V8<float>::store(p2 + C + c0, a3);
  }
}

template <typename T, int MODE>
__global__ __launch_bounds__(kT) void colreduce_kernel(const T* __restrict__ x, const T* __restrict__ out,
                                                       const uint8_t* __restrict__ mask,
                                                       const T* __restrict__ dout, const float* __restrict__ mean,
                                                       const float* __restrict__ rstd, int relu, int64_t rows, int C,
                                                       int tpr, int rpp, int64_t rows_per_slab,
                                                       float* __restrict__ partial) {
  __shared__ float red[2][kT][8];
  const int tid = threadIdx.x, rr = tid / tpr, cv = tid % tpr;
  const bool active = rr < rpp;
  const int c0 = cv * 8;
  float a1[8], a2[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { a1[j] = 0.f; a2[j] = 0.f; }
  float mu[8], rs[8];
  if (MODE == 1 && active) { load8f(mean + c0, mu); load8f(rstd + c0, rs); }
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_slab;
  const int64_t r1 = min(rows, r0 + rows_per_slab);
  if (active) {
    constexpr int U = 4;
    for (int64_t rb = r0 + rr; rb < r1; rb += (int64_t)rpp * U) {
      float xv[U][8], gv[U][8], ov[U][8];
      uint32_t mk[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t r = rb + (int64_t)u * rpp;
        const int64_t o = r * C + c0;
        mk[u] = 0xffu;
        if (r < r1) {
          if (MODE == 0 || MODE == 1) V8<T>::load(x + o, xv[u]);
          if (MODE != 0) {
            V8<T>::load(dout + o, gv[u]);
            if (relu) { if (mask) mk[u] = mask[o >> 3]; else V8<T>::load(out + o, ov[u]); }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t r = rb + (int64_t)u * rpp;
        if (r < r1) {
          if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { a1[j] += xv[u][j]; a2[j] += xv[u][j] * xv[u][j]; }
          } else {
            if (relu) {
              if (mask) {
#pragma unroll
                for (int j = 0; j < 8; ++j) if (!((mk[u] >> j) & 1u)) gv[u][j] = 0.f;
              } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) if (!(ov[u][j] > 0.f)) gv[u][j] = 0.f;
              }
            }
            if (MODE == 1) {
#pragma unroll
              for (int j = 0; j < 8; ++j) { a1[j] += gv[u][j]; a2[j] += gv[u][j] * ((xv[u][j] - mu[j]) * rs[j]); }
            } else {
#pragma unroll
              for (int j = 0; j < 8; ++j) a1[j] += gv[u][j];
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) { red[0][tid][j] = a1[j]; red[1][tid][j] = a2[j]; }
  __syncthreads();
  if (rr == 0) {
    for (int q = 1; q < rpp; ++q) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { a1[j] += red[0][q * tpr + cv][j]; a2[j] += red[1][q * tpr + cv][j]; }
    }
    float* p = partial + (int64_t)blockIdx.x * 2 * C;
    V8<float>::store(p + c0, a1);
    V8<float>::store(p + C + c0, a2);
  }
}

// MODE 0: mean / rstd.  MODE 1,2: sums[0..C) = s1, sums[C..2C) = s2 and optional scaled copies.
// A workgroup owns 8 channels; 32 thread groups each sum every 32nd slab in fp64 (four loads in
// flight), then the 32 group results are added in a fixed order.
template <int MODE>
__global__ __launch_bounds__(kT) void colfinal_kernel(const float* __restrict__ partial, int nslabs, int C, int64_t rows,
                                                      float* __restrict__ o1, float* __restrict__ o2, float* __restrict__ e1,
                                                      float* __restrict__ e2, float scale,
                                                      const float* __restrict__ gamma = nullptr, const float* __restrict__ mean = nullptr,
                                                      const float* __restrict__ rstd = nullptr, float* __restrict__ tab = nullptr,
                                                      int stride = 0, int off2 = 0, ParamAbsmax am = ParamAbsmax{nullptr, nullptr}) {
  if (stride == 0) { stride = 2 * C; off2 = C; }     // slab = [2][C]: the two sums are rows 0 and 1
  __shared__ double sh[2][32][8];
  const int cl = threadIdx.x & 7, grp = threadIdx.x >> 3;
  const int c = blockIdx.x * 8 + cl;
  // abs-max slots of the two gradient tensors: read now, in flight with the slab loads (see absmax_peek)
  uint32_t* const slot1 = (MODE != 0 && am.first && e1) ? absmax_way(am.first, blockIdx.x) : nullptr;
  uint32_t* const slot2 = (MODE != 0 && am.second && e2) ? absmax_way(am.second, blockIdx.x) : nullptr;
  const uint32_t seen1 = (slot1 && grp == 0) ? absmax_peek(slot1) : 0u, seen2 = (slot2 && grp == 0) ? absmax_peek(slot2) : 0u;
  double s1 = 0.0, s2 = 0.0;
  if (c < C) {
    // eight slabs per round trip; slabs past the end contribute +0 (exact), so the order of the adds is fixed
    for (int s = grp; s < nslabs; s += 256) {
      float a[8], b[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int su = s + 32 * u;
        const int sc = su < nslabs ? su : nslabs - 1;     // unconditional in-range loads, selected afterwards
        a[u] = partial[(int64_t)sc * stride + c];
        b[u] = partial[(int64_t)sc * stride + off2 + c];
        if (su >= nslabs) { a[u] = 0.f; b[u] = 0.f; }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) { s1 += (double)a[u]; s2 += (double)b[u]; }
    }
  }
  sh[0][grp][cl] = s1; sh[1][grp][cl] = s2;
  __syncthreads();
  if (grp != 0 || c >= C) return;
  s1 = 0.0; s2 = 0.0;
  for (int g = 0; g < 32; ++g) { s1 += sh[0][g][cl]; s2 += sh[1][g][cl]; }
  if (MODE == 0) {
    const double m = s1 / (double)rows;
    double var = s2 / (double)rows - m * m;
    if (var < 0.0) var = 0.0;
    o1[c] = (float)m;
    o2[c] = (float)(1.0 / sqrt(var + 1e-5));
  } else {
    o1[c] = (float)s1;
    if (o2) o2[c] = (float)s2;
    if (e1) e1[c] = (float)(s1 * (double)scale);
    if (e2) e2[c] = (float)(s2 * (double)scale);
    // (threads 0..7 of the workgroup are here, some perhaps not: one atomic each, at most C per tensor)
    if (slot1) absmax_raise(slot1, seen1, abs_bits((float)(s1 * (double)scale)));
    if (slot2) absmax_raise(slot2, seen2, abs_bits((float)(s2 * (double)scale)));
    if (tab) {   // constants of bn_input_grad for this channel
      const double a = (double)gamma[c] * (double)rstd[c];
      float* t = tab + (c >> 3) * 32 + (c & 7);
      t[0] = (float)a;
      t[8] = (float)(-a * (double)rstd[c] * s2 / (double)rows);
      t[16] = (float)(-a * s1 / (double)rows);
      t[24] = mean[c];
    }
  }
}

// Sums groups of 32 consecutive slabs (fixed order): [S][W] -> [ceil(S/32)][W], W = 2*C columns.
__global__ __launch_bounds__(kT) void slab_fold_kernel(const float* __restrict__ in, int S, int W, float* __restrict__ out) {
  const int col = blockIdx.y * kT + threadIdx.x;
  if (col >= W) return;
  const int s0 = blockIdx.x * 32;
  // all 32 loads are issued before the first add (one memory round trip instead of 32); rows past the
  // end contribute +0, which leaves the running sum unchanged
  float v[32];
#pragma unroll
  for (int u = 0; u < 32; ++u) {
    const int su = s0 + u;
    v[u] = in[(int64_t)(su < S ? su : S - 1) * W + col];
    if (su >= S) v[u] = 0.f;
  }
  float t = 0.f;
#pragma unroll
  for (int u = 0; u < 32; ++u) t += v[u];
  out[(int64_t)blockIdx.x * W + col] = t;
}

// RES: 0 no residual, 1 a stored residual, 2 the residual is the INPUT of a second normalisation without activation
// (the one on a projection shortcut), normalised here and rounded to the storage type -- exactly what a pass of its
// own would have stored.  (Compile-time, so that the common cases do not carry the second set of per-channel constants
// in registers: occupancy is what keeps this pass at the streaming rate.)
template <typename T, int RES>
__global__ __launch_bounds__(kT) void bnact_fwd_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                       T* __restrict__ out, uint8_t* __restrict__ mask, int64_t rows, int C, int tpr, int rpp,
                                                       int64_t rows_per_slab,
                                                       const float* __restrict__ mean, const float* __restrict__ rstd,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       int relu, const float* __restrict__ rmean, const float* __restrict__ rrstd,
                                                       const float* __restrict__ rgamma, const float* __restrict__ rbeta) {
  const int tid = threadIdx.x, rr = tid / tpr, cv = tid % tpr;
  if (rr >= rpp) return;
  const int c0 = cv * 8;
  float mu[8], rs[8], ga[8], be[8];
  load8f(mean + c0, mu); load8f(rstd + c0, rs); load8f(gamma + c0, ga); load8f(beta + c0, be);
  float rmu[RES == 2 ? 8 : 1], rrs[RES == 2 ? 8 : 1], rga[RES == 2 ? 8 : 1], rbe[RES == 2 ? 8 : 1];
  if (RES == 2) { load8f(rmean + c0, rmu); load8f(rrstd + c0, rrs); load8f(rgamma + c0, rga); load8f(rbeta + c0, rbe); }
  // slabs are walked from the end of the tensor: the rows the producing kernel wrote (or the
  // preceding reduction read) last are still in the 256 MB memory-side cache
  const int64_t r0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * rows_per_slab;
  const int64_t r1 = min(rows, r0 + rows_per_slab);
  // rows in flight per thread: with a residual stream one (83 registers, five waves per SIMD: 5.8 TB/s on the largest
  // tensors, against 4.6 TB/s with four rows in flight at two waves per SIMD), without one four
  constexpr int U = RES ? 1 : 4;
  for (int64_t rb = r0 + rr; rb < r1; rb += (int64_t)rpp * U) {
    typename V8<T>::Raw xr[U], rv[RES ? U : 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = rb + (int64_t)u * rpp;
      if (r < r1) { xr[u] = V8<T>::load_raw_nt(x + r * C + c0); if (RES) rv[u] = V8<T>::load_raw_nt(res + r * C + c0); }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = rb + (int64_t)u * rpp;
      if (r < r1) {
        float xv[8], rj[8], o[8];
        V8<T>::unpack(xr[u], xv);
        if (RES) V8<T>::unpack(rv[u], rj);
        uint32_t bits = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          o[j] = ga[j] * ((xv[j] - mu[j]) * rs[j]) + be[j];
          if (RES == 2) {
            rj[j] = rga[j] * ((rj[j] - rmu[j]) * rrs[j]) + rbe[j];
            if (sizeof(T) == 2) rj[j] = bf2f(f2bf(rj[j]));
          }
          if (RES) o[j] += rj[j];
          if (relu) o[j] = o[j] > 0.f ? o[j] : 0.f;
          bits |= (o[j] > 0.f ? 1u : 0u) << j;
        }
        V8<T>::store(out + r * C + c0, o);
        // one bit per element: out > 0 (what the backward pass needs of `out`); a positive fp32
        // value never rounds to zero in the storage type, so this equals the sign of the stored value
        if (mask) mask[(r * C + c0) >> 3] = (uint8_t)bits;
      }
    }
  }
}

// Normalisation + ReLU followed by a 3x3/2 max-pool (padding 1) in one pass: the activated tensor is not
// stored, only what later passes need of it -- the pooled maxima, the arg-max positions, and the one-bit
// ReLU mask of every pixel.  A thread owns one pooled pixel x 8 channels and the mask bytes of the pixels
// (2ho..2ho+1, 2wo..2wo+1), i.e. window positions (1..2, 1..2).  Values are rounded to the storage type
// before they are compared, so ties fall as they would between stored values.
template <typename T>
__global__ __launch_bounds__(kT) void bnact_pool_fwd_kernel(const T* __restrict__ x, T* __restrict__ pooled, uint8_t* __restrict__ arg,
                                                            uint8_t* __restrict__ mask, int B, int H, int W, int C, int Ho, int Wo,
                                                            const float* __restrict__ mean, const float* __restrict__ rstd,
                                                            const float* __restrict__ gamma, const float* __restrict__ beta) {
  const int tpr = C / 8;
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= (int64_t)B * Ho * Wo * tpr) return;
  // (vector counts stay below 2^31, checked on the host: 32-bit divisions)
  const uint32_t p = (uint32_t)v / (uint32_t)tpr, q = p / (uint32_t)Wo;
  const int cv = (int)((uint32_t)v - p * (uint32_t)tpr), wo = (int)(p - q * (uint32_t)Wo);
  const int n = (int)(q / (uint32_t)Ho), ho = (int)(q - (uint32_t)n * (uint32_t)Ho);
  const int c0 = cv * 8;
  float mu[8], rs[8], ga[8], be[8];
  load8f(mean + c0, mu); load8f(rstd + c0, rs); load8f(gamma + c0, ga); load8f(beta + c0, be);
  float best[8]; uint32_t pos[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { best[j] = -__builtin_inff(); pos[j] = 0; }
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const int hi = ho * 2 + r - 1;
    if (hi < 0 || hi >= H) continue;
#pragma unroll
    for (int s_ = 0; s_ < 3; ++s_) {
      const int wi = wo * 2 + s_ - 1;
      if (wi < 0 || wi >= W) continue;
      const int64_t o = (((int64_t)n * H + hi) * W + wi) * C + c0;
      float xv[8]; V8<T>::load(x + o, xv);
      uint32_t bits = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float a = ga[j] * ((xv[j] - mu[j]) * rs[j]) + be[j];
        a = a > 0.f ? a : 0.f;
        bits |= (a > 0.f ? 1u : 0u) << j;
        if (sizeof(T) == 2) a = bf2f(f2bf(a));
        if (a > best[j]) { best[j] = a; pos[j] = 3 * r + s_; }
      }
      if (r >= 1 && s_ >= 1) mask[o >> 3] = (uint8_t)bits;
    }
  }
  V8<T>::store(pooled + v * 8, best);
  uint2 pk;
  pk.x = pos[0] | (pos[1] << 8) | (pos[2] << 16) | (pos[3] << 24);
  pk.y = pos[4] | (pos[5] << 8) | (pos[6] << 16) | (pos[7] << 24);
  *reinterpret_cast<uint2*>(arg + v * 8) = pk;
}

// GATE: how d(out) is gated by the activation: 0 not at all, 1 by the one-bit mask, 2 by the stored output (> 0).
// DXACC: add to the stored dx.  DRES: 0 no residual gradient, 1 written, 2 added to the stored one.
// (Compile-time, so that every case carries only the streams it reads in registers: occupancy is what keeps this
// pass at the streaming rate.)
template <typename T, int GATE, bool DXACC, int DRES>
__global__ __launch_bounds__(kT) void bnact_bwd_apply_kernel(const T* __restrict__ x, const T* __restrict__ out,
                                                             const uint8_t* __restrict__ mask,
                                                             const T* __restrict__ dout, T* __restrict__ dx,
                                                             T* __restrict__ dres,
                                                             int64_t rows, int C, int tpr, int rpp, int64_t rows_per_slab,
                                                             const float* __restrict__ tab) {
  const int tid = threadIdx.x, rr = tid / tpr, cv = tid % tpr;
  if (rr >= rpp) return;
  const int c0 = cv * 8;
  float ka[8], kp[8], kq[8], mu[8];
  load8f(tab + cv * 32, ka); load8f(tab + cv * 32 + 8, kp); load8f(tab + cv * 32 + 16, kq); load8f(tab + cv * 32 + 24, mu);
  // slabs are walked from the end of the tensor: the rows the producing kernel wrote (or the
  // preceding reduction read) last are still in the 256 MB memory-side cache
  const int64_t r0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * rows_per_slab;
  const int64_t r1 = min(rows, r0 + rows_per_slab);
  constexpr int U = 2;
  typedef typename V8<T>::Raw Raw;
  for (int64_t rb = r0 + rr; rb < r1; rb += (int64_t)rpp * U) {
    Raw gr[U], xr[U], ovr[GATE == 2 ? U : 1], odr[DXACC ? U : 1], orr[DRES == 2 ? U : 1];
    uint32_t mk[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = rb + (int64_t)u * rpp;
      mk[u] = 0xffu;
      if (r < r1) {
        const int64_t o = r * C + c0;
        gr[u] = V8<T>::load_raw_nt(dout + o); xr[u] = V8<T>::load_raw_nt(x + o);
        if (GATE == 1) mk[u] = mask[o >> 3];
        if (GATE == 2) ovr[u] = V8<T>::load_raw_nt(out + o);
        if (DXACC) odr[u] = V8<T>::load_raw_nt(dx + o);
        if (DRES == 2) orr[u] = V8<T>::load_raw_nt(dres + o);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = rb + (int64_t)u * rpp;
      if (r < r1) {
        const int64_t o = r * C + c0;
        float g[8], xv[8], q[8];
        V8<T>::unpack(gr[u], g); V8<T>::unpack(xr[u], xv);
        if (GATE == 1) {
#pragma unroll
          for (int j = 0; j < 8; ++j) if (!((mk[u] >> j) & 1u)) g[j] = 0.f;
        }
        if (GATE == 2) {
          float ov[8];
          V8<T>::unpack(ovr[u], ov);
#pragma unroll
          for (int j = 0; j < 8; ++j) if (!(ov[j] > 0.f)) g[j] = 0.f;
        }
        if (DRES) {
          if (DRES == 2) {
            float od[8];
            V8<T>::unpack(orr[u], od);
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = od[j] + g[j];
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) q[j] = g[j];
          }
          V8<T>::store(dres + o, q);
        }
        float od[8];
        if (DXACC) V8<T>::unpack(odr[u], od);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          q[j] = bn_input_grad(g[j], xv[j], ka[j], kp[j], kq[j], mu[j]);
          if (DXACC) q[j] += od[j];
        }
        V8<T>::store(dx + o, q);
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kT) void biasact_fwd_kernel(const T* __restrict__ x, T* __restrict__ out, int64_t nvec,
                                                         int tpr, const float* __restrict__ bias, int relu) {
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= nvec) return;
  float xv[8], b[8];
  V8<T>::load(x + v * 8, xv); load8f(bias + (int)(v % tpr) * 8, b);
#pragma unroll
  for (int j = 0; j < 8; ++j) { xv[j] += b[j]; if (relu && !(xv[j] > 0.f)) xv[j] = 0.f; }
  V8<T>::store(out + v * 8, xv);
}

template <typename T>
__global__ __launch_bounds__(kT) void biasact_bwd_kernel(const T* __restrict__ out, const T* __restrict__ dout,
                                                         T* __restrict__ dx, int acc, int64_t nvec, int relu) {
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= nvec) return;
  float g[8];
  V8<T>::load(dout + v * 8, g);
  if (relu) {
    float ov[8]; V8<T>::load(out + v * 8, ov);
#pragma unroll
    for (int j = 0; j < 8; ++j) if (!(ov[j] > 0.f)) g[j] = 0.f;
  }
  if (acc) {
    float old[8]; V8<T>::load(dx + v * 8, old);
#pragma unroll
    for (int j = 0; j < 8; ++j) g[j] += old[j];
  }
  V8<T>::store(dx + v * 8, g);
}

// 3x3 window, stride 2, padding 1.  The forward pass also records, per output element, which of
// the nine window positions (3*r+s) holds the FIRST maximum in row-major order.
template <typename T>
__global__ __launch_bounds__(kT) void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ out,
                                                         uint8_t* __restrict__ arg, int B, int H, int W, int C, int Ho, int Wo) {
  const int tpr = C / 8;
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= (int64_t)B * Ho * Wo * tpr) return;
  // (vector counts stay below 2^31, checked on the host: 32-bit divisions)
  const uint32_t p = (uint32_t)v / (uint32_t)tpr, q = p / (uint32_t)Wo;
  const int cv = (int)((uint32_t)v - p * (uint32_t)tpr), wo = (int)(p - q * (uint32_t)Wo);
  const int n = (int)(q / (uint32_t)Ho), ho = (int)(q - (uint32_t)n * (uint32_t)Ho);
  float best[8]; uint32_t pos[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { best[j] = -__builtin_inff(); pos[j] = 0; }
  for (int r = 0; r < 3; ++r) {
    const int hi = ho * 2 + r - 1;
    if (hi < 0 || hi >= H) continue;
    for (int s = 0; s < 3; ++s) {
      const int wi = wo * 2 + s - 1;
      if (wi < 0 || wi >= W) continue;
      float xv[8]; V8<T>::load(x + (((int64_t)n * H + hi) * W + wi) * C + cv * 8, xv);
#pragma unroll
      for (int j = 0; j < 8; ++j) if (xv[j] > best[j]) { best[j] = xv[j]; pos[j] = 3 * r + s; }
    }
  }
  V8<T>::store(out + v * 8, best);
  uint2 pk;
  pk.x = pos[0] | (pos[1] << 8) | (pos[2] << 16) | (pos[3] << 24);
  pk.y = pos[4] | (pos[5] << 8) | (pos[6] << 16) | (pos[7] << 24);
  *reinterpret_cast<uint2*>(arg + v * 8) = pk;
}

// Gather form: an input pixel receives the gradient of every window (at most four) whose recorded
// arg-max position it is; contributions are summed in fp32 and stored once.  A thread owns a 2x2 block
// of input pixels (rows 2i, 2i+1, columns 2j, 2j+1) of 8 channels: those four pixels lie in the windows
// (i..i+1) x (j..j+1) only, so four window loads serve four pixels.
template <typename T>
__global__ __launch_bounds__(kT) void maxpool_bwd_kernel(const uint8_t* __restrict__ arg, const T* __restrict__ dout,
                                                         T* __restrict__ dx, int acc, int B, int H, int W, int C,
                                                         int Ho, int Wo) {
  const int tpr = C / 8;
  const int Hb = (H + 1) / 2, Wb = (W + 1) / 2;
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= (int64_t)B * Hb * Wb * tpr) return;
  // (vector counts stay below 2^31, checked on the host: 32-bit divisions)
  const uint32_t p = (uint32_t)v / (uint32_t)tpr, q = p / (uint32_t)Wb;
  const int cv = (int)((uint32_t)v - p * (uint32_t)tpr), j = (int)(p - q * (uint32_t)Wb);
  const int n = (int)(q / (uint32_t)Hb), i = (int)(q - (uint32_t)n * (uint32_t)Hb);
  float sum[2][2][8];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 8; ++e) sum[a][b][e] = 0.f;
#pragma unroll
  for (int dh = 0; dh < 2; ++dh)
#pragma unroll
    for (int dw = 0; dw < 2; ++dw) {
      const int ho = i + dh, wo = j + dw;
      if (ho >= Ho || wo >= Wo) continue;
      const int64_t o = (((int64_t)n * Ho + ho) * Wo + wo) * C + cv * 8;
      const uint2 pk = *reinterpret_cast<const uint2*>(arg + o);
      float g[8]; V8<T>::load(dout + o, g);
      // window (ho, wo) covers rows 2ho-1 .. 2ho+1: position r of pixel row 2i+a is 2i+a - (2ho-1) = a + 1 - 2dh
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int r = a + 1 - 2 * dh, c = b + 1 - 2 * dw;
          if (r < 0 || c < 0) continue;                    // (r, c <= 2 always)
          const uint32_t me = 3 * r + c;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t pe = ((e < 4 ? pk.x : pk.y) >> (8 * (e & 3))) & 0xffu;
            if (pe == me) sum[a][b][e] += g[e];
          }
        }
    }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int h = 2 * i + a, w = 2 * j + b;
      if (h >= H || w >= W) continue;
      const int64_t o = (((int64_t)n * H + h) * W + w) * C + cv * 8;
      if (acc) {
        float old[8]; V8<T>::load(dx + o, old);
#pragma unroll
        for (int e = 0; e < 8; ++e) sum[a][b][e] += old[e];
      }
      V8<T>::store(dx + o, sum[a][b]);
    }
}

template <typename T>
__global__ __launch_bounds__(kT) void gap_fwd_kernel(const T* __restrict__ x, float* __restrict__ pooled, int B, int HW, int C) {
  const int tpr = C / 8;
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= (int64_t)B * tpr) return;
  const int cv = (int)(v % tpr), n = (int)(v / tpr);
  float s[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) s[j] = 0.f;
  // eight pixels per round trip, added in pixel order (pixels past the end are not loaded and add +0)
  const T* base = x + (int64_t)n * HW * C + cv * 8;
  for (int i0 = 0; i0 < HW; i0 += 8) {
    float xv[8][8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (i0 + u < HW) V8<T>::load(base + (int64_t)(i0 + u) * C, xv[u]);
      else {
#pragma unroll
        for (int j = 0; j < 8; ++j) xv[u][j] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) s[j] += xv[u][j];
  }
  const float inv = 1.0f / (float)HW;
#pragma unroll
  for (int j = 0; j < 8; ++j) s[j] *= inv;
  V8<float>::store(pooled + (int64_t)n * C + cv * 8, s);
}

template <typename T>
__global__ __launch_bounds__(kT) void gap_bwd_kernel(const float* __restrict__ dpooled, T* __restrict__ dx, int acc, int B,
                                                     int HW, int C) {
  const int tpr = C / 8;
  const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (v >= (int64_t)B * HW * tpr) return;
  // (vector counts stay below 2^31, checked on the host: 32-bit divisions)
  const uint32_t pix = (uint32_t)v / (uint32_t)tpr;
  const int cv = (int)((uint32_t)v - pix * (uint32_t)tpr), n = (int)(pix / (uint32_t)HW);
  float g[8]; load8f(dpooled + (int64_t)n * C + cv * 8, g);
  const float inv = 1.0f / (float)HW;
#pragma unroll
  for (int j = 0; j < 8; ++j) g[j] *= inv;
  if (acc) {
    float old[8]; V8<T>::load(dx + v * 8, old);
#pragma unroll
    for (int j = 0; j < 8; ++j) g[j] += old[j];
  }
  V8<T>::store(dx + v * 8, g);
}

// ---- linear classifier (fp32) --------------------------------------------------------------
// One small tiled SGEMM serves the three products of the layer:
//   C[m][n] = scale * sum_k A(m,k) * B(k,n) (+ bias[n]),  A(m,k) = A[m*sAm + k*sAk],  B(k,n) = B[k*sBk + n*sBn].
// 64x64 output tile per workgroup, 32-deep k tiles staged in LDS (padded rows), each thread a 4x4 block of
// outputs (rows ty + 16 r, columns tx + 16 c: conflict-free LDS reads, 8 per 16 multiply-adds).
// The matrices are a few MB; the point is only not to be latency-bound: the contraction
// can be split over gridDim.z (k range [z*kchunk, (z+1)*kchunk)); then raw partial sums go to
// ws[z][M][N] and splitk_reduce_kernel adds them in a fixed order.
__global__ __launch_bounds__(kT) void sgemm_kernel(const float* __restrict__ A, const float* __restrict__ Bm,
                                                   const float* __restrict__ bias, float* __restrict__ Cm, int M, int N,
                                                   int K, int64_t sAm, int64_t sAk, int64_t sBk, int64_t sBn, float scale,
                                                   int kchunk, float* __restrict__ ws, uint32_t* __restrict__ absmax) {
  __shared__ float As[64][33], Bs[64][33];           // As[m][k], Bs[n][k]
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
  const int kbeg = blockIdx.z * kchunk;
  K = min(K, kbeg + kchunk);
  for (int k0 = kbeg; k0 < K; k0 += 32) {
    float av[8], bv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int idx = tid + 256 * j;
      // walk the unit-stride dimension with consecutive threads
      const int am = sAk == 1 ? idx >> 5 : idx & 63, ak = sAk == 1 ? idx & 31 : idx >> 6;
      av[j] = (m0 + am < M && k0 + ak < K) ? A[(int64_t)(m0 + am) * sAm + (int64_t)(k0 + ak) * sAk] : 0.f;
      const int bn = sBk == 1 ? idx >> 5 : idx & 63, bk = sBk == 1 ? idx & 31 : idx >> 6;
      bv[j] = (n0 + bn < N && k0 + bk < K) ? Bm[(int64_t)(k0 + bk) * sBk + (int64_t)(n0 + bn) * sBn] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int idx = tid + 256 * j;
      As[sAk == 1 ? idx >> 5 : idx & 63][sAk == 1 ? idx & 31 : idx >> 6] = av[j];
      Bs[sBk == 1 ? idx >> 5 : idx & 63][sBk == 1 ? idx & 31 : idx >> 6] = bv[j];
    }
    __syncthreads();
#pragma unroll 8
    for (int k = 0; k < 32; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) { a[r] = As[ty + 16 * r][k]; b[r] = Bs[tx + 16 * r][k]; }
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] += a[r] * b[c];
    }
    __syncthreads();
  }
  uint32_t amax = 0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int m = m0 + ty + 16 * r;
    if (m >= M) continue;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int n = n0 + tx + 16 * c;
      if (n >= N) continue;
      if (ws) ws[((int64_t)blockIdx.z * M + m) * N + n] = acc[r][c];
      else {
        const float v = acc[r][c] * scale + (bias ? bias[n] : 0.f);
        Cm[(int64_t)m * N + n] = v;
        amax = max(amax, abs_bits(v));
      }
    }
  }
  if (absmax && !ws) {   // (uniform condition: every lane of the wavefront is here)
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, d));
    if ((tid & 63) == 0) absmax_publish(absmax_way(absmax, blockIdx.x + blockIdx.y), amax);
  }
}

__global__ void splitk_reduce_kernel(const float* __restrict__ ws, int splits, int64_t MN, int N, float scale,
                                     const float* __restrict__ bias, float* __restrict__ Cm, uint32_t* __restrict__ absmax) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t amax = 0;
  if (i < MN) {
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += ws[(int64_t)z * MN + i];
    const float v = s * scale + (bias ? bias[i % N] : 0.f);
    Cm[i] = v;
    amax = abs_bits(v);
  }
  if (absmax) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, d));
    if ((threadIdx.x & 63) == 0) absmax_publish(absmax_way(absmax, blockIdx.x), amax);
  }
}

__global__ void fc_bias_grad_kernel(const float* __restrict__ dz, float* __restrict__ db, int B, int O, float scale, uint32_t* __restrict__ absmax) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t amax = 0;
  if (o < O) {
    float s = 0.f;
    for (int n = 0; n < B; ++n) s += dz[(int64_t)n * O + o];
    const float v = s * scale;
    db[o] = v;
    amax = abs_bits(v);
  }
  if (absmax) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, d));
    if ((threadIdx.x & 63) == 0) absmax_publish(absmax_way(absmax, blockIdx.x), amax);
  }
}

// ---- softmax cross-entropy: one wavefront per sample ------------------------------------------
__global__ __launch_bounds__(64) void ce_kernel(const float* __restrict__ z, const int32_t* __restrict__ y,
                                                float* __restrict__ dz, float* __restrict__ loss_n, int B, int O, float gscale) {
  const int n = blockIdx.x, lane = threadIdx.x;
  const float* zn = z + (int64_t)n * O;
  float mx = -__builtin_inff();
  for (int c = lane; c < O; c += 64) mx = fmaxf(mx, zn[c]);
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s));
  float se = 0.f;
  for (int c = lane; c < O; c += 64) se += expf(zn[c] - mx);
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) se += __shfl_xor(se, s);
  const float lse = mx + logf(se);
  // a label outside [0, O) (caller-owned device memory the host cannot validate): no one-hot term, NaN loss, no access
  const int yn = y[n];
  const bool label_ok = (unsigned)yn < (unsigned)O;
  for (int c = lane; c < O; c += 64) dz[(int64_t)n * O + c] = (expf(zn[c] - lse) - (c == yn ? 1.f : 0.f)) * gscale;
  if (lane == 0) loss_n[n] = label_ok ? lse - zn[yn] : __builtin_nanf("");
}

// TRADES regulariser phi_n = KL(p_n || q_n), p = softmax(z_clean), q = softmax(z_adv); one wavefront per sample.
//   branch 0 (the x+delta pass): dz = (q - p) * gscale,                                   loss_n = phi_n
//   branch 1 (the clean pass):   dz = (lambda*(p - onehot) + p*(log p - log q - phi_n)) * gscale, loss_n = CE(z_clean, y)
// The two passes differ by an eps-sized perturbation, so everything is written in terms of the small
// differences d_k = z_clean_k - z_adv_k instead of differences of two log-softmax values:
//   r = sum_k q_k expm1(d_k);  log p_k - log q_k = t_k = d_k - log1p(r);  p_k = q_k exp(t_k);  q_k - p_k = -q_k expm1(t_k).
__global__ __launch_bounds__(64) void kl_kernel(const float* __restrict__ zc, const float* __restrict__ za,
                                                const int32_t* __restrict__ y, int branch, float lambda,
                                                float* __restrict__ dz, float* __restrict__ loss_n, int B, int O, float gscale) {
  const int n = blockIdx.x, lane = threadIdx.x;
  const float* c = zc + (int64_t)n * O;
  const float* a = za + (int64_t)n * O;
  float ma = -__builtin_inff();
  for (int k = lane; k < O; k += 64) ma = fmaxf(ma, a[k]);
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) ma = fmaxf(ma, __shfl_xor(ma, s));
  float sa = 0.f, sr = 0.f;
  for (int k = lane; k < O; k += 64) { const float e = expf(a[k] - ma); sa += e; sr += e * expm1f(c[k] - a[k]); }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) { sa += __shfl_xor(sa, s); sr += __shfl_xor(sr, s); }
  const float la = ma + logf(sa);            // log-sum-exp of the perturbed logits
  const float dl = log1pf(sr / sa);          // lse(clean) - lse(perturbed)
  float kl = 0.f;
  for (int k = lane; k < O; k += 64) { const float t = (c[k] - a[k]) - dl; kl += expf(a[k] - la + t) * t; }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) kl += __shfl_xor(kl, s);
  if (branch == 0) {
    for (int k = lane; k < O; k += 64) {
      const float t = (c[k] - a[k]) - dl;
      dz[(int64_t)n * O + k] = -expf(a[k] - la) * expm1f(t) * gscale;
    }
    if (lane == 0) loss_n[n] = kl;
  } else {
    const int yn = y[n];
    const bool label_ok = (unsigned)yn < (unsigned)O;      // as in ce_kernel
    for (int k = lane; k < O; k += 64) {
      const float t = (c[k] - a[k]) - dl, p = expf(a[k] - la + t);
      dz[(int64_t)n * O + k] = (lambda * (p - (k == yn ? 1.f : 0.f)) + p * (t - kl)) * gscale;
    }
    if (lane == 0) loss_n[n] = label_ok ? (la + dl) - c[yn] : __builtin_nanf("");
  }
}

// one wavefront: lane l adds elements l, l + 64, ... in fp64, then the lanes are combined in a fixed butterfly order
__global__ __launch_bounds__(64) void mean_kernel(const float* __restrict__ v, int n, float* __restrict__ out) {
  if (blockIdx.x != 0) return;
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 64) s += (double)v[i];
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d);
  if (threadIdx.x == 0) out[0] = (float)(s / n);
}

__global__ void round_bf16_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = bf2f(f2bf(src[i]));
}

// bh, bw > 0: g0 is stored as 2x2 pixel blocks of a bh x bw image ([bh/2][bw/2][4*Cpad] per sample)
template <typename T>
__global__ void input_grad_kernel(const T* __restrict__ g0, int Cpad, int64_t rows, float s0, float s1, float s2,
                                  float* __restrict__ gx, int bh, int bw) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * 3) return;
  int64_t r = i / 3; const int c = (int)(i % 3);
  if (bw) {
    const uint32_t pix = (uint32_t)r, w = pix % (uint32_t)bw, hn = pix / (uint32_t)bw;
    const uint32_t h = hn % (uint32_t)bh, n = hn / (uint32_t)bh;
    r = ((int64_t)(n * (uint32_t)(bh >> 1) + (h >> 1)) * (uint32_t)(bw >> 1) + (w >> 1)) * 4 + (h & 1u) * 2 + (w & 1u);
  }
  float v;
  if (sizeof(T) == 2) v = bf2f(((const bf16_t*)g0)[r * Cpad + c]); else v = ((const float*)g0)[r * Cpad + c];
  gx[i] = __fmul_rn(v, c == 0 ? s0 : (c == 1 ? s1 : s2));
}

__global__ void sgd_kernel(float* __restrict__ theta, const float* __restrict__ g, float lr, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) theta[i] = __fsub_rn(theta[i], __fmul_rn(lr, g[i]));
}

// scales[t] = max over the kAbsmaxWays slots of tensor t (bit patterns of non-negative floats)
__global__ void absmax_fold_kernel(const uint32_t* __restrict__ ways, int T, uint32_t* __restrict__ scales) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  uint32_t m = 0;
#pragma unroll
  for (int w = 0; w < kAbsmaxWays; ++w) m = max(m, ways[((int64_t)t * kAbsmaxWays + w) * kAbsmaxStride]);
  scales[t] = m;
}

__global__ void zero_kernel(uint32_t* __restrict__ p, int64_t nwords) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nwords) p[i] = 0u;
}

inline unsigned nblk(int64_t n) { return (unsigned)((n + kT - 1) / kT); }

template <typename T, int MODE>
dat_status colreduce(const void* x, const void* out, const uint8_t* mask, const void* dout, const float* mean, const float* rstd, int relu,
                     int64_t rows, int C, float* partial, hipStream_t st, SlabPlan& p) {
  p = plan_slabs(rows, C, kMaxSlabs);
  hipLaunchKernelGGL((colreduce_kernel<T, MODE>), dim3(p.nslabs), dim3(kT), 0, st, (const T*)x, (const T*)out, mask,
                     (const T*)dout, mean, rstd, relu, rows, C, p.tpr, p.rpp, p.rows_per_slab, partial);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace

size_t bn_partial_floats(int64_t rows, int C) { (void)rows; return (size_t)kMaxSlabs * 4 * C; }   // two sets of slabs (dual reduction)

size_t fold_floats(int nslabs, int C) { return nslabs > 512 ? (size_t)((nslabs + 31) / 32) * 3 * C : 0; }   // up to three sums per channel

dat_status bn_finalize_slabs(float* partial, int nslabs, int C, int64_t rows, int mode, float* o1, float* o2, float* dbeta,
                             float* dgamma, float scale, hipStream_t st, const float* gamma, const float* mean, const float* rstd,
                             float* tab, int nsum, int col2, bool fold, ParamAbsmax am) {
  const float* src = partial;
  const int W = nsum * C;
  if (nslabs > 512) {   // two-level: keep the final per-channel loop short
    float* folded = partial + (size_t)nslabs * W;
    const int S2 = (nslabs + 31) / 32;
    if (fold) {
      hipLaunchKernelGGL(slab_fold_kernel, dim3(S2, (W + kT - 1) / kT), dim3(kT), 0, st, partial, nslabs, W, folded);
      DAT_LAUNCH_CHECK();
    }
    src = folded; nslabs = S2;
  }
  if (mode == 1)
    hipLaunchKernelGGL(colfinal_kernel<0>, dim3((C + 7) / 8), dim3(kT), 0, st, src, nslabs, C, rows, o1, o2, (float*)nullptr, (float*)nullptr, 1.0f,
                       (const float*)nullptr, (const float*)nullptr, (const float*)nullptr, (float*)nullptr, W, col2 * C);
  else
    hipLaunchKernelGGL(colfinal_kernel<1>, dim3((C + 7) / 8), dim3(kT), 0, st, src, nslabs, C, rows, o1, o2, dbeta, dgamma, scale, gamma, mean, rstd, tab,
                       W, col2 * C, am);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

#define DAT_BY_DTYPE(dtype, CALL_F32, CALL_BF16) do { if ((dtype) == 0) { CALL_F32; } else { CALL_BF16; } } while (0)

dat_status bn_stats(const void* x, int dtype, int64_t rows, int C, float* partial, float* mean, float* rstd, hipStream_t st) {
  if (C % 8 != 0 || C > 8 * kT) return DAT_ERR_UNSUPPORTED;
  SlabPlan p; dat_status s;
  DAT_BY_DTYPE(dtype, s = (colreduce<float, 0>(x, nullptr, nullptr, nullptr, nullptr, nullptr, 0, rows, C, partial, st, p)),
               s = (colreduce<bf16_t, 0>(x, nullptr, nullptr, nullptr, nullptr, nullptr, 0, rows, C, partial, st, p)));
  if (s != DAT_OK) return s;
  hipLaunchKernelGGL(colfinal_kernel<0>, dim3((C + 7) / 8), dim3(kT), 0, st, partial, p.nslabs, C, rows, mean, rstd,
                     (float*)nullptr, (float*)nullptr, 1.0f);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status bnact_forward(const void* x, const void* res, void* out, uint8_t* mask, int dtype, int64_t rows, int C, const float* mean,
                         const float* rstd, const float* gamma, const float* beta, int relu, hipStream_t st, const BnParams* res_bn) {
  if (C % 8 != 0 || C > 8 * kT) return DAT_ERR_UNSUPPORTED;
  if (res_bn && !res) return DAT_ERR_ARG;
  const SlabPlan p = plan_slabs(rows, C, kMaxApplySlabs);
  const float* rm = res_bn ? res_bn->mean : nullptr; const float* rr = res_bn ? res_bn->rstd : nullptr;
  const float* rg = res_bn ? res_bn->gamma : nullptr; const float* rb = res_bn ? res_bn->beta : nullptr;
#define DAT_BNACT_FWD(T, RES) hipLaunchKernelGGL((bnact_fwd_kernel<T, RES>), dim3(p.nslabs), dim3(kT), 0, st, (const T*)x, (const T*)res, (T*)out, mask, rows, C, p.tpr, p.rpp, p.rows_per_slab, mean, rstd, gamma, beta, relu, rm, rr, rg, rb)
  const int rk = res_bn ? 2 : res ? 1 : 0;
  DAT_BY_DTYPE(dtype,
    { if (rk == 2) DAT_BNACT_FWD(float, 2); else if (rk == 1) DAT_BNACT_FWD(float, 1); else DAT_BNACT_FWD(float, 0); },
    { if (rk == 2) DAT_BNACT_FWD(bf16_t, 2); else if (rk == 1) DAT_BNACT_FWD(bf16_t, 1); else DAT_BNACT_FWD(bf16_t, 0); });
#undef DAT_BNACT_FWD
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status bnact_pool_forward(const void* x, void* pooled, uint8_t* arg, uint8_t* mask, int dtype, int B, int H, int W, int C, int Ho, int Wo,
                              const float* mean, const float* rstd, const float* gamma, const float* beta, hipStream_t st) {
  if (C % 8 != 0 || !mask || !arg) return DAT_ERR_ARG;
  const int64_t nvec = (int64_t)B * Ho * Wo * (C / 8);
  if (nvec >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;   // 32-bit vector indices in the kernel
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(bnact_pool_fwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, (const float*)x, (float*)pooled, arg, mask, B, H, W, C, Ho, Wo, mean, rstd, gamma, beta),
    hipLaunchKernelGGL(bnact_pool_fwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, (const bf16_t*)x, (bf16_t*)pooled, arg, mask, B, H, W, C, Ho, Wo, mean, rstd, gamma, beta));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status bn_backward_reduce(const void* x, const void* out, const uint8_t* mask, const void* dout, int dtype, int64_t rows, int C,
                              const float* mean, const float* rstd, const float* gamma, int relu, float* partial, float* sums,
                              float* tab, float* dgamma, float* dbeta, float scale, hipStream_t st, const BnSecond* second, ParamAbsmax am) {
  if (C % 8 != 0 || C > 8 * kT) return DAT_ERR_UNSUPPORTED;
  SlabPlan p;
  if (second) {
    if (!relu || !mask) return DAT_ERR_ARG;
    p = plan_slabs(rows, C, kMaxSlabs);
    float* partial2 = partial + (size_t)kMaxSlabs * 2 * C;
    DAT_BY_DTYPE(dtype,
      hipLaunchKernelGGL(dual_reduce_kernel<float>, dim3(p.nslabs), dim3(kT), 0, st, (const float*)x, (const float*)second->x, mask, (const float*)dout, mean, rstd, second->mean, second->rstd, rows, C, p.tpr, p.rpp, p.rows_per_slab, partial, partial2),
      hipLaunchKernelGGL(dual_reduce_kernel<bf16_t>, dim3(p.nslabs), dim3(kT), 0, st, (const bf16_t*)x, (const bf16_t*)second->x, mask, (const bf16_t*)dout, mean, rstd, second->mean, second->rstd, rows, C, p.tpr, p.rpp, p.rows_per_slab, partial, partial2));
    DAT_LAUNCH_CHECK();
    hipLaunchKernelGGL(colfinal_kernel<1>, dim3((C + 7) / 8), dim3(kT), 0, st, (const float*)partial2, p.nslabs, C, rows, second->sums, second->sums + C,
                       second->dbeta, second->dgamma, scale, second->gamma, second->mean, second->rstd, second->tab, 0, 0, second->am);
    DAT_LAUNCH_CHECK();
  } else {
    dat_status s;
    DAT_BY_DTYPE(dtype, s = (colreduce<float, 1>(x, out, mask, dout, mean, rstd, relu, rows, C, partial, st, p)),
                 s = (colreduce<bf16_t, 1>(x, out, mask, dout, mean, rstd, relu, rows, C, partial, st, p)));
    if (s != DAT_OK) return s;
  }
  hipLaunchKernelGGL(colfinal_kernel<1>, dim3((C + 7) / 8), dim3(kT), 0, st, (const float*)partial, p.nslabs, C, rows, sums, sums + C,
                     dbeta, dgamma, scale, gamma, mean, rstd, tab, 0, 0, am);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status bn_backward_apply(const void* x, const void* out, const uint8_t* mask, const void* dout, void* dx, bool dx_accumulate, void* dres,
                             bool dres_accumulate, int dtype, int64_t rows, int C, const float* tab, int relu, hipStream_t st) {
  if (C % 8 != 0 || C > 8 * kT) return DAT_ERR_UNSUPPORTED;
  const SlabPlan q = plan_slabs(rows, C, kMaxApplySlabs);
  const int gate = !relu ? 0 : mask ? 1 : 2, dr = !dres ? 0 : dres_accumulate ? 2 : 1;
#define DAT_BWD_APPLY(T, G, A, R) hipLaunchKernelGGL((bnact_bwd_apply_kernel<T, G, A, R>), dim3(q.nslabs), dim3(kT), 0, st, (const T*)x, (const T*)out, mask, (const T*)dout, (T*)dx, (T*)dres, rows, C, q.tpr, q.rpp, q.rows_per_slab, tab)
#define DAT_BWD_APPLY_R(T, G, A) do { if (dr == 0) DAT_BWD_APPLY(T, G, A, 0); else if (dr == 1) DAT_BWD_APPLY(T, G, A, 1); else DAT_BWD_APPLY(T, G, A, 2); } while (0)
#define DAT_BWD_APPLY_A(T, G) do { if (dx_accumulate) DAT_BWD_APPLY_R(T, G, true); else DAT_BWD_APPLY_R(T, G, false); } while (0)
#define DAT_BWD_APPLY_G(T) do { if (gate == 0) DAT_BWD_APPLY_A(T, 0); else if (gate == 1) DAT_BWD_APPLY_A(T, 1); else DAT_BWD_APPLY_A(T, 2); } while (0)
  DAT_BY_DTYPE(dtype, DAT_BWD_APPLY_G(float), DAT_BWD_APPLY_G(bf16_t));
#undef DAT_BWD_APPLY_G
#undef DAT_BWD_APPLY_A
#undef DAT_BWD_APPLY_R
#undef DAT_BWD_APPLY
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

// The two halves for a BN + ReLU whose output feeds a 3x3/2 max-pool, on 2x2 pixel blocks.  pool->gather: d(out) is
// gathered from the pool's output gradient (`dout` is not read); otherwise it is read from `dout`.  Both settings
// sum in the same order.
dat_status bn_pool_backward(const void* x, const uint8_t* mask, const void* dout, void* dx, bool dx_accumulate, bool skip_apply, int dtype, int C,
                            const float* mean, const float* rstd, const float* gamma, float* partial, float* sums, float* tab,
                            float* dgamma, float* dbeta, float scale, const PoolGrad& pg, hipStream_t st, ParamAbsmax am) {
  if (C % 8 != 0 || C > 8 * kT || !mask) return DAT_ERR_UNSUPPORTED;
  PoolArgs pa{pg.arg, pg.dpooled, pg.B, pg.H, pg.W, pg.Ho, pg.Wo};
  const int tpr = C / 8, rpp = kT / tpr;
  const int64_t nblocks = (int64_t)pg.B * ((pg.H + 1) / 2) * ((pg.W + 1) / 2);
  if (nblocks * tpr >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;   // 32-bit block / vector indices in the kernels
  const int64_t rows = (int64_t)pg.B * pg.H * pg.W;
  int64_t want = (nblocks + (int64_t)rpp * 8 - 1) / ((int64_t)rpp * 8);
  int nslabs = (int)(want < 1 ? 1 : (want > kMaxSlabs ? kMaxSlabs : want));
  int64_t bps = (nblocks + nslabs - 1) / nslabs;
  bps = (bps + rpp - 1) / rpp * rpp;
  nslabs = (int)((nblocks + bps - 1) / bps);
#define DAT_BLOCK_REDUCE(T, POOL)                                                                                              \
  hipLaunchKernelGGL((block_reduce_kernel<T, POOL>), dim3(nslabs), dim3(kT), 0, st, (const T*)x, mask, (const T*)dout, mean, rstd, C, tpr, \
                     nblocks, bps, partial, pa)
#define DAT_BLOCK_APPLY(T, POOL)                                                                                               \
  hipLaunchKernelGGL((block_apply_kernel<T, POOL>), dim3(nblk(nblocks * tpr)), dim3(kT), 0, st, (const T*)x, mask, (const T*)dout, (T*)dx,  \
                     (int)dx_accumulate, C, tpr, nblocks, (const float*)tab, pa)
  if (pg.gather) DAT_BY_DTYPE(dtype, DAT_BLOCK_REDUCE(float, true), DAT_BLOCK_REDUCE(bf16_t, true));
  else DAT_BY_DTYPE(dtype, DAT_BLOCK_REDUCE(float, false), DAT_BLOCK_REDUCE(bf16_t, false));
  DAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(colfinal_kernel<1>, dim3((C + 7) / 8), dim3(kT), 0, st, (const float*)partial, nslabs, C, rows, sums, sums + C,
                     dbeta, dgamma, scale, gamma, mean, rstd, tab, 0, 0, am);
  DAT_LAUNCH_CHECK();
  if (skip_apply) return DAT_OK;
  if (pg.gather) DAT_BY_DTYPE(dtype, DAT_BLOCK_APPLY(float, true), DAT_BLOCK_APPLY(bf16_t, true));
  else DAT_BY_DTYPE(dtype, DAT_BLOCK_APPLY(float, false), DAT_BLOCK_APPLY(bf16_t, false));
  DAT_LAUNCH_CHECK();
#undef DAT_BLOCK_REDUCE
#undef DAT_BLOCK_APPLY
  return DAT_OK;
}

dat_status biasact_forward(const void* x, void* out, int dtype, int64_t rows, int C, const float* bias, int relu, hipStream_t st) {
  const int64_t nvec = rows * (C / 8);
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(biasact_fwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, (const float*)x, (float*)out, nvec, C / 8, bias, relu),
    hipLaunchKernelGGL(biasact_fwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, (const bf16_t*)x, (bf16_t*)out, nvec, C / 8, bias, relu));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status biasact_backward(const void* out, const void* dout, void* dx, bool dx_accumulate, int dtype, int64_t rows, int C,
                            int relu, float* partial, float* dbias, float scale, hipStream_t st) {
  if (C % 8 != 0 || C > 8 * kT) return DAT_ERR_UNSUPPORTED;
  if (dbias) {
    SlabPlan p; dat_status s;
    DAT_BY_DTYPE(dtype, s = (colreduce<float, 2>(nullptr, out, nullptr, dout, nullptr, nullptr, relu, rows, C, partial, st, p)),
                 s = (colreduce<bf16_t, 2>(nullptr, out, nullptr, dout, nullptr, nullptr, relu, rows, C, partial, st, p)));
    if (s != DAT_OK) return s;
    hipLaunchKernelGGL(colfinal_kernel<2>, dim3((C + 7) / 8), dim3(kT), 0, st, partial, p.nslabs, C, rows, dbias,
                       (float*)nullptr, dbias, (float*)nullptr, scale);
    DAT_LAUNCH_CHECK();
  }
  const int64_t nvec = rows * (C / 8);
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(biasact_bwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, (const float*)out, (const float*)dout, (float*)dx, (int)dx_accumulate, nvec, relu),
    hipLaunchKernelGGL(biasact_bwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, (const bf16_t*)out, (const bf16_t*)dout, (bf16_t*)dx, (int)dx_accumulate, nvec, relu));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status maxpool_forward(const void* x, void* out, uint8_t* arg, int dtype, int B, int H, int W, int C, int Ho, int Wo, hipStream_t st) {
  const int64_t nvec = (int64_t)B * Ho * Wo * (C / 8);
  if (nvec >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;   // 32-bit vector indices in the kernel
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(maxpool_fwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, (const float*)x, (float*)out, arg, B, H, W, C, Ho, Wo),
    hipLaunchKernelGGL(maxpool_fwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, (const bf16_t*)x, (bf16_t*)out, arg, B, H, W, C, Ho, Wo));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status maxpool_backward(const uint8_t* arg, const void* dout, void* dx, bool accumulate, int dtype, int B, int H, int W, int C,
                            int Ho, int Wo, hipStream_t st) {
  const int64_t nvec = (int64_t)B * ((H + 1) / 2) * ((W + 1) / 2) * (C / 8);
  if (nvec >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;   // 32-bit vector indices in the kernel
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(maxpool_bwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, arg, (const float*)dout, (float*)dx, (int)accumulate, B, H, W, C, Ho, Wo),
    hipLaunchKernelGGL(maxpool_bwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, arg, (const bf16_t*)dout, (bf16_t*)dx, (int)accumulate, B, H, W, C, Ho, Wo));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status gap_forward(const void* x, float* pooled, int dtype, int B, int HW, int C, hipStream_t st) {
  const int64_t nvec = (int64_t)B * (C / 8);
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(gap_fwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, (const float*)x, pooled, B, HW, C),
    hipLaunchKernelGGL(gap_fwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, (const bf16_t*)x, pooled, B, HW, C));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status gap_backward(const float* dpooled, void* dx, bool accumulate, int dtype, int B, int HW, int C, hipStream_t st) {
  const int64_t nvec = (int64_t)B * HW * (C / 8);
  if (nvec >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;   // 32-bit vector indices in the kernel
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(gap_bwd_kernel<float>, dim3(nblk(nvec)), dim3(kT), 0, st, dpooled, (float*)dx, (int)accumulate, B, HW, C),
    hipLaunchKernelGGL(gap_bwd_kernel<bf16_t>, dim3(nblk(nvec)), dim3(kT), 0, st, dpooled, (bf16_t*)dx, (int)accumulate, B, HW, C));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

// ws (optional): room for fc_workspace_floats(B, I, O) floats; then long contractions are split so that the launch
// has a few hundred workgroups.
static dat_status sgemm(const float* A, const float* Bm, const float* bias, float* Cm, int M, int N, int K, int64_t sAm,
                        int64_t sAk, int64_t sBk, int64_t sBn, float scale, float* ws, hipStream_t st, uint32_t* absmax = nullptr) {
  const int tiles = ((N + 63) / 64) * ((M + 63) / 64);
  int splits = 1;
  if (ws && K >= 256) {
    splits = (1024 + tiles - 1) / tiles;
    if (splits > 8) splits = 8;
    if (splits > K / 64) splits = K / 64;
    if (splits < 1) splits = 1;
  }
  const int kchunk = ((K + splits - 1) / splits + 31) / 32 * 32;
  splits = (K + kchunk - 1) / kchunk;
  if (splits == 1) ws = nullptr;
  hipLaunchKernelGGL(sgemm_kernel, dim3((N + 63) / 64, (M + 63) / 64, splits), dim3(kT), 0, st, A, Bm, bias, Cm, M, N, K, sAm, sAk, sBk,
                     sBn, scale, kchunk, ws, absmax);
  DAT_LAUNCH_CHECK();
  if (ws) {
    const int64_t MN = (int64_t)M * N;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(nblk(MN)), dim3(kT), 0, st, (const float*)ws, splits, MN, N, scale, bias, Cm, absmax);
    DAT_LAUNCH_CHECK();
  }
  return DAT_OK;
}

size_t fc_workspace_floats(int B, int I, int O) { return (size_t)8 * B * (size_t)(I > O ? I : O); }

dat_status fc_forward(const float* f, const float* W, const float* b, float* logits, int B, int I, int O, float* ws, hipStream_t st) {
  // logits[n][o] = sum_i f[n][i] * W[o][i] + b[o]
  return sgemm(f, W, b, logits, B, O, I, I, 1, 1, I, 1.0f, ws, st);
}

dat_status fc_backward(const float* f, const float* W, const float* dz, float* df, float* dW, float* db, int B, int I, int O,
                       float scale, float* ws, hipStream_t st, ParamAbsmax am) {
  // df[n][i] = sum_o dz[n][o] * W[o][i]
  dat_status s = sgemm(dz, W, nullptr, df, B, I, O, O, 1, I, 1, 1.0f, ws, st);
  if (s != DAT_OK) return s;
  if (dW) {
    // dW[o][i] = scale * sum_n dz[n][o] * f[n][i];  db[o] = scale * sum_n dz[n][o]
    s = sgemm(dz, f, nullptr, dW, O, I, B, 1, O, I, 1, scale, nullptr, st, am.first);
    if (s != DAT_OK) return s;
    hipLaunchKernelGGL(fc_bias_grad_kernel, dim3((O + 255) / 256), dim3(256), 0, st, dz, db, B, O, scale, am.second);
    DAT_LAUNCH_CHECK();
  }
  return DAT_OK;
}

dat_status ce_forward_backward(const float* logits, const int32_t* y, float* dz, float* loss_n, float* loss_mean, int B, int O,
                               float gscale, hipStream_t st) {
  hipLaunchKernelGGL(ce_kernel, dim3(B), dim3(64), 0, st, logits, y, dz, loss_n, B, O, gscale);
  DAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(64), 0, st, loss_n, B, loss_mean);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status kl_forward_backward(const float* z_clean, const float* z_adv, const int32_t* y, int branch, float lambda, float* dz,
                               float* loss_n, float* loss_mean, int B, int O, float gscale, hipStream_t st) {
  hipLaunchKernelGGL(kl_kernel, dim3(B), dim3(64), 0, st, z_clean, z_adv, y, branch, lambda, dz, loss_n, B, O, gscale);
  DAT_LAUNCH_CHECK();
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(64), 0, st, loss_n, B, loss_mean);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_round_bf16_values(const float* src, float* dst, int64_t n, hipStream_t st) {
  if (n == 0) return DAT_OK;
  hipLaunchKernelGGL(round_bf16_kernel, dim3(nblk(n)), dim3(kT), 0, st, src, dst, n);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_input_grad(const void* g0, int dtype, int Cpad, int64_t rows, float s0, float s1, float s2, float* gx,
                             int block_h, int block_w, hipStream_t st) {
  if (rows >= (1ll << 32)) return DAT_ERR_UNSUPPORTED;
  DAT_BY_DTYPE(dtype,
    hipLaunchKernelGGL(input_grad_kernel<float>, dim3(nblk(rows * 3)), dim3(kT), 0, st, (const float*)g0, Cpad, rows, s0, s1, s2, gx, block_h, block_w),
    hipLaunchKernelGGL(input_grad_kernel<bf16_t>, dim3(nblk(rows * 3)), dim3(kT), 0, st, (const bf16_t*)g0, Cpad, rows, s0, s1, s2, gx, block_h, block_w));
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_sgd(float* theta, const float* g, float lr, int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(sgd_kernel, dim3(nblk(n)), dim3(kT), 0, st, theta, g, lr, n);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_absmax_fold(const uint32_t* ways, int T, uint32_t* scales, hipStream_t st) {
  hipLaunchKernelGGL(absmax_fold_kernel, dim3((T + 255) / 256), dim3(256), 0, st, ways, T, scales);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  const int64_t nwords = (int64_t)((bytes + 3) / 4);
  if (nwords == 0) return DAT_OK;
  hipLaunchKernelGGL(zero_kernel, dim3(nblk(nwords)), dim3(kT), 0, st, (uint32_t*)p, nwords);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace dat
