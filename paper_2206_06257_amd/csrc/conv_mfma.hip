// bf16 convolutions as implicit GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16,
// fp32 accumulate): forward, backward-data and backward-weight of the conv layers that make
// up dat_attack / dat_step.  Written for 64-wide wavefronts: a 256-thread workgroup is four
// waves (2x2, or 1x4 for 32-channel tiles), each wave owning a block of 32x32 MFMA accumulators.
//
// Forward / backward-data:
//   D[c][p] = sum_k Wt[c][k] * X[p][k],  k = (r, s, ci) flattened, ci fastest.
//   Wt rows are output channels ([Cout][k*k*Cin], K-contiguous); X[p][k] is the im2col view of
//   the NHWC input, gathered on the fly: 8 consecutive k are 8 consecutive channels of one tap,
//   i.e. one 16-byte vector.  Both operands sit in LDS as [row][BK k] tiles (BK = 32 or 64) with
//   an XOR swizzle of the 16-byte slots so that the 16-byte fragment reads of the 32 lanes
//   sharing a k-slot hit distinct banks.  Two kernels fill those tiles:
//   * `igemm_dma_kernel` (contraction channels a multiple of BK): global memory -> LDS directly
//     (global_load_lds_dwordx4), one LDS stage, four or more workgroups resident per CU;
//   * `igemm_ring_kernel` (long contractions into a multiple of 256 channels that fill the chip with one
//     round of tiles): 8 waves, 256-channel tiles, a ring of LDS stages filled by the same direct loads;
//   * `igemm_kernel` (any channel count, and the long 1x1 contractions into <= 64 channels):
//     global -> registers -> LDS, double buffered, loads running PF k-tiles ahead.
//   Backward-data is the same contraction over the output gradient: stride 1 with the flipped,
//   transposed filter ([Cin][k][k][Cout]); stride 2 as four launches, one per parity class of the
//   input pixels, each a dense stride-1 convolution with that class's sub-filter.
//   The shared epilogue adds an optional residual (or the previously stored gradient) in fp32,
//   rounds once to bf16, transposes through LDS, writes 16-byte channel vectors and can emit the
//   per-channel (sum, sum of squares) of what it stored: the batch statistics of the BN that follows.
//   Workgroups are numbered so that the channel tiles of one pixel tile land on the same XCD
//   (ids congruent mod 8 share an L2), which keeps the gathered activations L2-resident; layers
//   with a filter window also give every XCD one contiguous range of pixel tiles, so that the
//   rows neighbouring tiles share are re-read from that L2.
//
// Backward-weight (`wgrad_kernel`): dW[co][(r,s,ci)] = sum_p dY[p][co] * X[p][(r,s,ci)], a
// contraction over pixels, which are the strided dimension of both operands.  The tiles land in
// LDS as they are in memory ([pixel][channel], direct-to-LDS loads) and the MFMA fragments are
// read with the LDS transpose reads of gfx950 (ds_read_b64_tr_b16), which hand every lane four
// consecutive pixels of its channel.  The pixel range is split over gridDim.z; partial tiles go to a workspace
// and a second kernel sums them in a fixed order (deterministic).
#include <atomic>
#include <mutex>
#include <cstdlib>
#include "kernels.h"

namespace dat {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 256;


typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte vector (stays in registers)
union Frag { u32x4 u; bf16x8 v; };

// 16-byte slot permutation of a [row][NS slots] LDS tile (NS = 4: 64-byte rows, NS = 8: 128-byte
// rows).  Chosen so that the lanes of a fragment read (consecutive rows, same logical slot) touch
// distinct 16-byte bank groups both within any 8 consecutive rows x 128 bytes and within any 16
// consecutive rows x 256 bytes (LDS bank sweeps of 32 and of 64 banks).  Uses row bits 0..3 only.
template <int NS> __device__ __forceinline__ int swz(int row, int slot);
template <> __device__ __forceinline__ int swz<4>(int row, int slot) {
  const int f = (((row >> 2) & 1) << 1) | (((row >> 1) ^ (row >> 3)) & 1);
  return row * 64 + ((slot ^ f) << 4);
}
template <> __device__ __forceinline__ int swz<8>(int row, int slot) {
  const int f = (row & 7) ^ ((row >> 3) & 1);
  return row * 128 + ((slot ^ f) << 4);
}

// Out-of-range and padding vectors are read from this zero page instead of being masked.
__device__ __attribute__((aligned(16))) uint32_t g_zero_page[4] = {0u, 0u, 0u, 0u};

struct IgemmArgs {
  const bf16_t* in;     // [B][Hin][Win][Cin]
  const bf16_t* wt;     // [Cout][KH*KW*Cin]
  const bf16_t* res;    // optional [M][Cout] added before rounding
  const uint8_t* res_mask;   // optional: bit j of byte e/8 gates element e of `res` (a ReLU mask: res*mask is added)
  int res_even_only;         // `res` holds values only at pixels with even row and even column (ostep 1); the rest counts as zero
  bf16_t* out;          // [M][Cout], M = B*Hout*Wout
  int B, Hin, Win, Cin, Hout, Wout, Cout;   // Hout x Wout = grid of output pixels this launch computes
  int KH, KW, ostride, pad_h, pad_w;
  // Elements between neighbouring input pixels of a row (0: Cin, the ordinary case).  With 0 < xstride < Cin the
  // "Cin channels" of pixel w are the stored values of the pixels w .. w + Cin/xstride - 1, i.e. a filter row of
  // Cin/xstride taps read as one contiguous vector (igemm_dma_kernel with Cin equal to its k-tile only); a 16-byte
  // vector then lies in pixel w + offset/xstride and is zero when that pixel is outside the row.
  int xstride;
  // output pixel (n, a, b) is stored at row (n*outH + a*ostep + oh0)*outW + b*ostep + ow0 of `out`
  int outH, outW, ostep, oh0, ow0;
  int M, Ktot, nct, npt;
  // pixel tile -> XCD: interleaved (tile t on XCD t mod 8) or one contiguous range of tiles per XCD (neighbouring
  // tiles, which share filter-window rows, then share an L2)
  int xcd_contiguous;
  // Optional per-channel sums (sum v, sum v^2) of the stored (bf16-rounded) outputs -- the batch
  // statistics of the normalisation that follows -- one [2][Cout] slab per pixel tile at
  // stat_partial + (stat_slab0 + pixel_tile) * 2 * Cout.
  int stat_mode, stat_slab0;
  float* stat_partial;
  // stat_mode 2: the stored tensor is the output gradient of a batch normalisation with input stat_x (same
  // layout as `out`), ReLU mask stat_mask (or nullptr) and batch statistics stat_mean / stat_rstd; the slabs then
  // hold (sum v*m, sum v*m*xhat), the two sums of that normalisation's backward pass.
  const bf16_t* stat_x; const uint8_t* stat_mask; const float* stat_mean; const float* stat_rstd;
  // stat_mode 3 (128-channel tiles only): a second normalisation (input stat_x2, statistics stat_mean2 / stat_rstd2)
  // shares that output gradient; slabs are [3][Cout]: (sum v*m, sum v*m*xhat, sum v*m*xhat2).
  const bf16_t* stat_x2; const float* stat_mean2; const float* stat_rstd2;
  // Optional operand transform (1x1 stride-1 layers, igemm_kernel only): `in` is the output gradient of a batch
  // normalisation, and the operand actually contracted is that normalisation's input gradient,
  // bn_input_grad(in .* mask, xf_x, constants of the channel), rounded to bf16 -- formed while the tile moves from
  // registers to LDS instead of being written to memory by a pass of its own.
  const bf16_t* xf_x;        // [M][Cin] the normalisation's input
  const uint8_t* xf_mask;    // one bit per element of `in` (ReLU mask), or nullptr
  const float* xf_tab;       // 4*Cin floats, layout of bn_input_grad's constants
};

__device__ __forceinline__ int64_t out_row(const IgemmArgs& a, int m) {
  if (a.ostep == 1 && a.outH == a.Hout && a.outW == a.Wout) return m;
  const int HW = a.Hout * a.Wout;
  const int n = m / HW, rem = m - n * HW;
  const int ya = rem / a.Wout, xb = rem - ya * a.Wout;
  return ((int64_t)n * a.outH + ya * a.ostep + a.oh0) * a.outW + xb * a.ostep + a.ow0;
}

// ---- epilogue shared by the convolution kernels: (+res) -> bf16 -> LDS transpose -> 16-byte stores ----
// `lds` must hold TP rows of STG_STRIDE = 2*TC + 16 bytes (and [kThreads/(TC/8)][2][TC] floats for the
// statistics); every wave must be done with whatever else lived there (the caller ends on a barrier).
template <int TC, int TP, int WGC, int NT = kThreads>
__device__ __forceinline__ void igemm_epilogue(const IgemmArgs& a, f32x16 (&acc)[TC / WGC / 32][TP / (NT / 64 / WGC) / 32],
                                               unsigned char* lds, int c0, int m0, int pt) {
  constexpr int WGP = NT / 64 / WGC;
  constexpr int WC = TC / WGC, WP = TP / WGP;
  constexpr int NI = WC / 32, NJ = WP / 32;
  constexpr int STG_STRIDE = TC * 2 + 16;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wc = wave % WGC, wp = wave / WGC;
  // ---- epilogue: (+res) -> bf16 -> LDS transpose -> 16-byte stores -------------------------
  // accumulator element e of lane l in tile (i,j): channel = 8*(e/4) + 4*(l/32) + e%4, pixel = l%32.
  // All four waves stage their block at once (one barrier), then every thread streams 16-byte
  // channel vectors of whole pixel rows to global memory.
  // A residual (or the previously stored gradient) is first brought into the staging buffer with
  // the same coalesced 16-byte accesses the stores use; each lane then adds its accumulators to
  // the values at its own staging slots in fp32 and rounds once, in place.
  constexpr int CV = TC / 8;                       // channel vectors per pixel row
  constexpr int RPP = NT / CV;                     // pixel rows per store sweep
  constexpr int NU = (TP + RPP - 1) / RPP;         // sweeps
  // tile widths that are no power of two (160 channels: 20 vectors per row, 12 rows per sweep): the last
  // threads have no vector and the last sweep is short
  constexpr bool EXACT = NT % CV == 0 && TP % RPP == 0;
  const int cv = tid % CV, pr0 = tid / CV;
  auto row_ok = [&](int u) { return EXACT || (pr0 < RPP && pr0 + u * RPP < TP); };
  const int ch = c0 + cv * 8;
  if (a.res) {
    uint4 rv[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int m = m0 + pr0 + u * RPP;
      rv[u] = make_uint4(0u, 0u, 0u, 0u);
      bool take = row_ok(u) && m < a.M && ch < a.Cout;
      if (a.res_even_only && take) { const int q = m / a.Wout; take = !(((m - q * a.Wout) | (q % a.Hout)) & 1); }
      if (take) {
        const int64_t e = out_row(a, m) * a.Cout + ch;
        rv[u] = *reinterpret_cast<const uint4*>(a.res + e);
        if (a.res_mask) {
          const uint32_t k = a.res_mask[e >> 3];
          rv[u].x &= ((k & 1u) ? 0xffffu : 0u) | ((k & 2u) ? 0xffff0000u : 0u);
          rv[u].y &= ((k & 4u) ? 0xffffu : 0u) | ((k & 8u) ? 0xffff0000u : 0u);
          rv[u].z &= ((k & 16u) ? 0xffffu : 0u) | ((k & 32u) ? 0xffff0000u : 0u);
          rv[u].w &= ((k & 64u) ? 0xffffu : 0u) | ((k & 128u) ? 0xffff0000u : 0u);
        }
      }
    }
    // (the main loop ended with a barrier: every wave is done with the operand tiles)
#pragma unroll
    for (int u = 0; u < NU; ++u)
      if (row_ok(u)) *reinterpret_cast<uint4*>(lds + (pr0 + u * RPP) * STG_STRIDE + cv * 16) = rv[u];
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int prow = wp * WP + j * 32 + (lane & 31);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int chl = wc * WC + i * 32 + 8 * g + 4 * (lane >> 5);
        float v[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        uint2* slot = reinterpret_cast<uint2*>(lds + prow * STG_STRIDE + chl * 2);
        if (a.res) {
          const uint2 r = *slot;
          v[0] += __uint_as_float(r.x << 16); v[1] += __uint_as_float(r.x & 0xffff0000u);
          v[2] += __uint_as_float(r.y << 16); v[3] += __uint_as_float(r.y & 0xffff0000u);
        }
        uint2 pk;
        pk.x = f2bf_pack(v[0], v[1]);
        pk.y = f2bf_pack(v[2], v[3]);
        *slot = pk;
      }
    }
  __syncthreads();
  float s1[8], s2[8], s3[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { s1[j] = 0.f; s2[j] = 0.f; s3[j] = 0.f; }
  if (a.stat_mode == 3) {
    // as mode 2 below, for two normalisations sharing d(out)
    float mu[8], rs[8], mu2[8], rs2[8];
    if (ch < a.Cout) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { mu[j] = a.stat_mean[ch + j]; rs[j] = a.stat_rstd[ch + j]; mu2[j] = a.stat_mean2[ch + j]; rs2[j] = a.stat_rstd2[ch + j]; }
    }
    constexpr int H = (NU + 1) / 2;              // rows in two batches: half the operand registers
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      uint4 xv[H], yv[H]; uint32_t mk[H];
#pragma unroll
      for (int u = 0; u < H; ++u) {
        const int m = m0 + pr0 + (b * H + u) * RPP;
        xv[u] = make_uint4(0u, 0u, 0u, 0u); yv[u] = xv[u]; mk[u] = 0u;
        if (b * H + u < NU && row_ok(b * H + u) && m < a.M && ch < a.Cout) {
          const int64_t e = out_row(a, m) * a.Cout + ch;
          xv[u] = *reinterpret_cast<const uint4*>(a.stat_x + e);
          yv[u] = *reinterpret_cast<const uint4*>(a.stat_x2 + e);
          mk[u] = a.stat_mask ? (uint32_t)a.stat_mask[e >> 3] : 0xffu;
        }
      }
#pragma unroll
      for (int u = 0; u < H; ++u) {
        const int prow = pr0 + (b * H + u) * RPP, m = m0 + prow;
        if (b * H + u < NU && row_ok(b * H + u) && m < a.M && ch < a.Cout) {
          const uint4 pk = *reinterpret_cast<const uint4*>(lds + prow * STG_STRIDE + cv * 16);
          *reinterpret_cast<uint4*>(a.out + out_row(a, m) * a.Cout + ch) = pk;
          const uint32_t w[4] = {pk.x, pk.y, pk.z, pk.w}, xw[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w}, yw[4] = {yv[u].x, yv[u].y, yv[u].z, yv[u].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float v0 = ((mk[u] >> (2 * j)) & 1u) ? __uint_as_float(w[j] << 16) : 0.f;
            const float v1 = ((mk[u] >> (2 * j + 1)) & 1u) ? __uint_as_float(w[j] & 0xffff0000u) : 0.f;
            s1[2 * j] += v0; s1[2 * j + 1] += v1;
            s2[2 * j] = __builtin_fmaf(v0, (__uint_as_float(xw[j] << 16) - mu[2 * j]) * rs[2 * j], s2[2 * j]);
            s2[2 * j + 1] = __builtin_fmaf(v1, (__uint_as_float(xw[j] & 0xffff0000u) - mu[2 * j + 1]) * rs[2 * j + 1], s2[2 * j + 1]);
            s3[2 * j] = __builtin_fmaf(v0, (__uint_as_float(yw[j] << 16) - mu2[2 * j]) * rs2[2 * j], s3[2 * j]);
            s3[2 * j + 1] = __builtin_fmaf(v1, (__uint_as_float(yw[j] & 0xffff0000u) - mu2[2 * j + 1]) * rs2[2 * j + 1], s3[2 * j + 1]);
          }
        }
      }
    }
  } else if (a.stat_mode == 2) {
    // BN backward sums of the tile just computed: the normalisation's input and mask are fetched for all of this
    // thread's rows before the first one is used
    float mu[8], rs[8];
    if (ch < a.Cout) {
      const float4 m0v = *reinterpret_cast<const float4*>(a.stat_mean + ch), m1v = *reinterpret_cast<const float4*>(a.stat_mean + ch + 4);
      const float4 r0v = *reinterpret_cast<const float4*>(a.stat_rstd + ch), r1v = *reinterpret_cast<const float4*>(a.stat_rstd + ch + 4);
      mu[0] = m0v.x; mu[1] = m0v.y; mu[2] = m0v.z; mu[3] = m0v.w; mu[4] = m1v.x; mu[5] = m1v.y; mu[6] = m1v.z; mu[7] = m1v.w;
      rs[0] = r0v.x; rs[1] = r0v.y; rs[2] = r0v.z; rs[3] = r0v.w; rs[4] = r1v.x; rs[5] = r1v.y; rs[6] = r1v.z; rs[7] = r1v.w;
    }
    uint4 xv[NU]; uint32_t mk[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int m = m0 + pr0 + u * RPP;
      xv[u] = make_uint4(0u, 0u, 0u, 0u); mk[u] = 0u;
      if (row_ok(u) && m < a.M && ch < a.Cout) {
        const int64_t e = out_row(a, m) * a.Cout + ch;
        xv[u] = *reinterpret_cast<const uint4*>(a.stat_x + e);
        mk[u] = a.stat_mask ? (uint32_t)a.stat_mask[e >> 3] : 0xffu;
      }
    }
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int prow = pr0 + u * RPP, m = m0 + prow;
      if (row_ok(u) && m < a.M && ch < a.Cout) {
        const uint4 pk = *reinterpret_cast<const uint4*>(lds + prow * STG_STRIDE + cv * 16);
        *reinterpret_cast<uint4*>(a.out + out_row(a, m) * a.Cout + ch) = pk;
        const uint32_t w[4] = {pk.x, pk.y, pk.z, pk.w}, xw[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float v0 = ((mk[u] >> (2 * j)) & 1u) ? __uint_as_float(w[j] << 16) : 0.f;
          const float v1 = ((mk[u] >> (2 * j + 1)) & 1u) ? __uint_as_float(w[j] & 0xffff0000u) : 0.f;
          const float x0 = __uint_as_float(xw[j] << 16), x1 = __uint_as_float(xw[j] & 0xffff0000u);
          s1[2 * j] += v0; s2[2 * j] = __builtin_fmaf(v0, (x0 - mu[2 * j]) * rs[2 * j], s2[2 * j]);
          s1[2 * j + 1] += v1; s2[2 * j + 1] = __builtin_fmaf(v1, (x1 - mu[2 * j + 1]) * rs[2 * j + 1], s2[2 * j + 1]);
        }
      }
    }
  } else {
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const int prow = pr0 + u * RPP, m = m0 + prow;
    if (row_ok(u) && m < a.M && ch < a.Cout) {
      const uint4 pk = *reinterpret_cast<const uint4*>(lds + prow * STG_STRIDE + cv * 16);
      *reinterpret_cast<uint4*>(a.out + out_row(a, m) * a.Cout + ch) = pk;
      if (a.stat_mode) {
        const uint32_t w[4] = {pk.x, pk.y, pk.z, pk.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float v0 = __uint_as_float(w[j] << 16), v1 = __uint_as_float(w[j] & 0xffff0000u);
          s1[2 * j] += v0; s2[2 * j] = __builtin_fmaf(v0, v0, s2[2 * j]); s1[2 * j + 1] += v1; s2[2 * j + 1] = __builtin_fmaf(v1, v1, s2[2 * j + 1]);
        }
      }
    }
  }
  }
  if (a.stat_mode) {
    // fold the RPP row groups in a fixed order through LDS, one slab per pixel tile
    __syncthreads();
    const int ns = a.stat_mode == 3 ? 3 : 2;        // sums per channel
    float* red = reinterpret_cast<float*>(lds);     // [RPP][ns][TC]
    if (EXACT || pr0 < RPP) {
      // 16-byte stores: as single floats the lanes of a wave (8 floats apart, rows a multiple of 64 floats apart) would
      // land eight to a bank
      auto put = [&](int which, const float (&v)[8]) {
        float4* dst = reinterpret_cast<float4*>(red + (pr0 * ns + which) * TC + cv * 8);
        dst[0] = make_float4(v[0], v[1], v[2], v[3]);
        dst[1] = make_float4(v[4], v[5], v[6], v[7]);
      };
      put(0, s1); put(1, s2);
      if (ns == 3) put(2, s3);
    }
    __syncthreads();
    for (int q = tid; q < ns * TC; q += NT) {
      const int which = q / TC, c = q % TC;
      float t = 0.f;
      for (int g = 0; g < RPP; ++g) t += red[(g * ns + which) * TC + c];
      if (c0 + c < a.Cout) a.stat_partial[((int64_t)(a.stat_slab0 + pt) * ns + which) * a.Cout + c0 + c] = t;
    }
  }
}

template <int TC, int TP, int WGC, int PF, bool FAST, int BKT, int OCC, bool XF = false>
__global__ __launch_bounds__(kThreads, OCC) void igemm_kernel(IgemmArgs a) {
  static_assert(!XF || FAST, "the operand transform needs whole k-tiles of one tap");
  constexpr int WGP = 4 / WGC;                     // waves along channels x waves along pixels
  constexpr int WC = TC / WGC, WP = TP / WGP;      // wave tile
  constexpr int NI = WC / 32, NJ = WP / 32;        // MFMA tiles per wave
  constexpr int NS = BKT / 8;                      // 16-byte slots per tile row
  constexpr int RB = BKT * 2;                      // bytes per tile row
  constexpr int RPG = kThreads / NS;               // tile rows covered by one load per thread
  constexpr int KS = BKT / 16;                     // MFMA k-steps per tile
  constexpr int VW = (TC * NS + kThreads - 1) / kThreads, VX = TP * NS / kThreads;   // 16-byte vectors per thread per tile
  constexpr int TILE_BYTES = (TC + TP) * RB;
  constexpr int STG_STRIDE = TC * 2 + 16;
  constexpr int LDS_BYTES = (2 * TILE_BYTES > TP * STG_STRIDE) ? 2 * TILE_BYTES : TP * STG_STRIDE;
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];

  // XCD-aware tile numbering: workgroup ids congruent mod 8 run on the same XCD (one L2 each), so
  // all channel tiles of a pixel tile get ids 8 apart and share the gathered activations in one L2.
  // Pixel tiles are dealt to the XCDs round robin, or (layers with a filter window) in one contiguous
  // range per XCD.
  const int bid = blockIdx.x;
  const int q = bid >> 3;
  const int ct = q % a.nct;
  const int pt = a.xcd_contiguous ? (bid & 7) * ((a.npt + 7) >> 3) + (q / a.nct) : (q / a.nct) * 8 + (bid & 7);
  if (pt >= a.npt) return;
  const int c0 = ct * TC, m0 = pt * TP;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wc = wave % WGC, wp = wave / WGC;
  const int kvec = tid % NS, lrow = tid / NS;      // this thread's slot in the global->LDS copy

  // im2col row state for the activation vectors this thread fetches (32-bit element offsets)
  int hb[VX], wb[VX], nb[VX]; bool mv[VX];
  const int HW = a.Hout * a.Wout;
#pragma unroll
  for (int i = 0; i < VX; ++i) {
    const int m = m0 + lrow + RPG * i;
    mv[i] = m < a.M;
    const int mm = mv[i] ? m : 0;
    const int n = mm / HW, rem = mm - n * HW;
    const int ho = rem / a.Wout, wo = rem - ho * a.Wout;
    hb[i] = ho * a.ostride - a.pad_h; wb[i] = wo * a.ostride - a.pad_w;
    nb[i] = n * a.Hin * a.Win;
  }
  const int ntiles = (a.Ktot + BKT - 1) / BKT;
  const u32x4* zero_page = reinterpret_cast<const u32x4*>(g_zero_page);

  // Weight rows of this thread: offset of (row, k = kvec*8) and row validity; advances by BK per tile.
  int woff[VW]; bool wrow[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) {
    const int c = c0 + lrow + RPG * i;
    wrow[i] = (lrow + RPG * i < TC) & (c < a.Cout);
    woff[i] = (wrow[i] ? c : 0) * a.Ktot + kvec * 8;
  }
  // Activation state.  FAST (Cin % 32 == 0): a k-tile never straddles a filter tap, so the tap
  // (r,s), the bounds test and the pixel offset change only every Cin/32 tiles (a uniform branch);
  // in between the offset just advances by 32 channels.  Otherwise every vector decodes its own tap.
  int xoff[VX]; bool xok[VX];
  int kc0 = 0, kr = 0, ks = 0;                      // FAST: channel offset of the tile, current tap
  int kc, gr, gs;                                   // generic: this thread's channel / tap
  {
    const int k = kvec * 8;
    const int tap = k / a.Cin;
    kc = k - tap * a.Cin; gr = tap / a.KW; gs = tap - gr * a.KW;
  }
  auto retap = [&](int r, int s_, int cofs) {
#pragma unroll
    for (int i = 0; i < VX; ++i) {
      const int hi = hb[i] + r, wi = wb[i] + s_;
      xok[i] = mv[i] & (hi >= 0) & (wi >= 0) & (hi < a.Hin) & (wi < a.Win);
      xoff[i] = (nb[i] + hi * a.Win + wi) * a.Cin + cofs;
    }
  };

  // Global loads run PF tiles ahead of the MFMAs: tile t+1 sits in LDS (other buffer) while tiles
  // t+2 .. t+1+PF are in flight into PF register sets.  Every step issues the same number of
  // unconditional loads (invalid vectors read the zero page), so nothing waits on a load early.
  struct RegSet { u32x4 w[VW]; u32x4 x[VX]; u32x4 y[XF ? VX : 1]; uint32_t mk[XF ? VX : 1]; int kch; };
  RegSet rs[PF];
  extern __shared__ __attribute__((aligned(16))) float xf_tab_lds[];   // XF: the constants of all Cin channels
  int kf = 0;                                      // next tile to fetch
  auto fetch = [&](RegSet& r) {
    const bool tile_ok = kf < ntiles;
#pragma unroll
    for (int i = 0; i < VW; ++i) {
      const bool ok = tile_ok & wrow[i] & (FAST || kf * BKT + kvec * 8 < a.Ktot);
      const u32x4* p = ok ? reinterpret_cast<const u32x4*>(a.wt + woff[i]) : zero_page;
      r.w[i] = *p;
      woff[i] += BKT;
    }
    if (FAST) {
      if (kc0 == 0) retap(kr, ks, kvec * 8);       // uniform: first tile of a tap
      if (XF) r.kch = tile_ok ? kc0 : 0;
#pragma unroll
      for (int i = 0; i < VX; ++i) {
        const bool ok = tile_ok & xok[i];
        const u32x4* p = ok ? reinterpret_cast<const u32x4*>(a.in + xoff[i]) : zero_page;
        r.x[i] = *p;
        if (XF) {
          const u32x4* py = ok ? reinterpret_cast<const u32x4*>(a.xf_x + xoff[i]) : zero_page;
          r.y[i] = *py;
          const uint8_t* pm = (ok && a.xf_mask) ? a.xf_mask + (xoff[i] >> 3) : reinterpret_cast<const uint8_t*>(g_zero_page);
          r.mk[i] = a.xf_mask ? (uint32_t)*pm : (ok ? 0xffu : 0u);
        }
        xoff[i] += BKT;
      }
      kc0 += BKT;
      if (kc0 == a.Cin) { kc0 = 0; if (++ks == a.KW) { ks = 0; ++kr; } }
    } else {
      retap(gr, gs, kc);
      const bool kvalid = tile_ok & (kf * BKT + kvec * 8 < a.Ktot);
#pragma unroll
      for (int i = 0; i < VX; ++i) {
        const u32x4* p = (kvalid & xok[i]) ? reinterpret_cast<const u32x4*>(a.in + xoff[i]) : zero_page;
        r.x[i] = *p;
      }
      kc += BKT;
      while (kc >= a.Cin) { kc -= a.Cin; if (++gs == a.KW) { gs = 0; ++gr; } }
    }
    ++kf;
  };
  const int st_w = swz<NS>(lrow, kvec), st_x = TC * RB + swz<NS>(lrow, kvec);   // rows lrow + RPG*i share the swizzle (RPG % 16 == 0)
  auto stash = [&](int buf, const RegSet& r) {
    unsigned char* base = lds + buf * TILE_BYTES;
#pragma unroll
    for (int i = 0; i < VW; ++i)
      if (lrow + RPG * i < TC) *reinterpret_cast<u32x4*>(base + st_w + i * (RPG * RB)) = r.w[i];
    if (XF) {
      // the 8 channels of this thread's vectors: kch + kvec*8 .. +7
      const float* tb = xf_tab_lds + ((r.kch >> 3) + kvec) * 32;
      float ka[8], kp[8], kq[8], mu[8];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const float4 va = reinterpret_cast<const float4*>(tb)[h], vp = reinterpret_cast<const float4*>(tb + 8)[h];
        const float4 vq = reinterpret_cast<const float4*>(tb + 16)[h], vm = reinterpret_cast<const float4*>(tb + 24)[h];
        ka[4 * h] = va.x; ka[4 * h + 1] = va.y; ka[4 * h + 2] = va.z; ka[4 * h + 3] = va.w;
        kp[4 * h] = vp.x; kp[4 * h + 1] = vp.y; kp[4 * h + 2] = vp.z; kp[4 * h + 3] = vp.w;
        kq[4 * h] = vq.x; kq[4 * h + 1] = vq.y; kq[4 * h + 2] = vq.z; kq[4 * h + 3] = vq.w;
        mu[4 * h] = vm.x; mu[4 * h + 1] = vm.y; mu[4 * h + 2] = vm.z; mu[4 * h + 3] = vm.w;
      }
#pragma unroll
      for (int i = 0; i < VX; ++i) {
        u32x4 o;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const uint32_t gw = r.x[i][d], yw = r.y[i][d];
          const float g0 = ((r.mk[i] >> (2 * d)) & 1u) ? __uint_as_float(gw << 16) : 0.f;
          const float g1 = ((r.mk[i] >> (2 * d + 1)) & 1u) ? __uint_as_float(gw & 0xffff0000u) : 0.f;
          const float v0 = bn_input_grad(g0, __uint_as_float(yw << 16), ka[2 * d], kp[2 * d], kq[2 * d], mu[2 * d]);
          const float v1 = bn_input_grad(g1, __uint_as_float(yw & 0xffff0000u), ka[2 * d + 1], kp[2 * d + 1], kq[2 * d + 1], mu[2 * d + 1]);
          o[d] = f2bf_pack(v0, v1);
        }
        *reinterpret_cast<u32x4*>(base + st_x + i * (RPG * RB)) = o;
      }
    } else {
#pragma unroll
      for (int i = 0; i < VX; ++i) *reinterpret_cast<u32x4*>(base + st_x + i * (RPG * RB)) = r.x[i];
    }
  };
  // fragment read offsets (bytes inside a tile) per MFMA k-step
  int fa_off[KS][NI], fb_off[KS][NJ];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    const int slot = kk * 2 + (lane >> 5);
#pragma unroll
    for (int i = 0; i < NI; ++i) fa_off[kk][i] = swz<NS>(wc * WC + i * 32 + (lane & 31), slot);
#pragma unroll
    for (int j = 0; j < NJ; ++j) fb_off[kk][j] = TC * RB + swz<NS>(wp * WP + j * 32 + (lane & 31), slot);
  }

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  {
    // tiles 0 .. PF are all requested before the first one is waited for
    RegSet first;
    fetch(first);
#pragma unroll
    for (int p = 0; p < PF; ++p) fetch(rs[p]);
    if (XF) {
      for (int i = tid; i < a.Cin; i += kThreads)
        reinterpret_cast<float4*>(xf_tab_lds)[i] = reinterpret_cast<const float4*>(a.xf_tab)[i];
      __syncthreads();
    }
    stash(0, first);
  }
  __syncthreads();
  auto step = [&](int t, RegSet& r) {
    const unsigned char* base = lds + (t & 1) * TILE_BYTES;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      Frag fa[NI], fb[NJ];
#pragma unroll
      for (int i = 0; i < NI; ++i) fa[i].u = *reinterpret_cast<const u32x4*>(base + fa_off[kk][i]);
#pragma unroll
      for (int j = 0; j < NJ; ++j) fb[j].u = *reinterpret_cast<const u32x4*>(base + fb_off[kk][j]);
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
    }
    stash((t + 1) & 1, r);     // this register set holds tile t+1 (all zero past the end)
    fetch(r);                  // ... and now receives tile t+1+PF
    __syncthreads();
  };
  // main loop: whole groups of PF steps, no conditionals, so that the number of loads in flight
  // is the same on every path; then at most PF-1 guarded tail steps
  int kt = 0;
  for (; kt + PF <= ntiles; kt += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) step(kt + u, rs[u]);
  }
#pragma unroll
  for (int u = 0; u < PF - 1; ++u)
    if (kt + u < ntiles) step(kt + u, rs[u]);

  igemm_epilogue<TC, TP, WGC>(a, acc, lds, c0, m0, pt);
}

// ---- direct-to-LDS variant (contraction channels a multiple of 64) ---------------------------------
// Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4: every lane names
// its own 16-byte source, the 64 vectors of a wave land contiguously at a wave-uniform LDS address):
// no staging registers and no ds_write, so four workgroups stay resident per CU with 64-wide k-tiles,
// whose 128-byte rows use whole cache lines (the vector L1 moves ~0.45 lines per clock whether a wave
// uses all of a line or half of it).  One LDS stage per workgroup: load tile t, wait, compute, and
// only then overwrite it; the load latency is covered by the other resident workgroups.
// The XOR swizzle of the 16-byte slots is applied on the source side: the lane that fills physical
// slot p of a row fetches logical k-slot p ^ f(row).
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* gbl_void_ptr;

// ANYC: the contraction channels are no multiple of the k-tile (160 channels, 64-wide tiles), so a tile straddles
// filter taps: every lane follows the tap and channel of its own 16-byte vector (a vector never straddles: Cin % 8
// == 0), and the last tile is padded from the zero page.
template <int TC, int TP, int WGC, int OCC, int BKT, bool ANYC = false>
__global__ __launch_bounds__(kThreads, OCC) void igemm_dma_kernel(IgemmArgs a) {
  constexpr int KS = BKT / 16, NS = BKT / 8;              // MFMA k-steps per tile; 16-byte slots per tile row
  constexpr int WGP = 4 / WGC;
  constexpr int WC = TC / WGC, WP = TP / WGP;
  constexpr int NI = WC / 32, NJ = WP / 32;
  constexpr int RB = BKT * 2, RPG = kThreads / NS;        // bytes per tile row; tile rows covered by one load per thread
  constexpr int VW = (TC + RPG - 1) / RPG, VX = TP / RPG;
  constexpr int TILE_BYTES = (VW * RPG + TP) * RB;       // weight rows rounded up to whole load sweeps
  constexpr int XBASE = VW * RPG * RB;
  constexpr int STG_STRIDE = TC * 2 + 16;
  constexpr int RED_BYTES = (kThreads / (TC / 8)) * (TC >= 128 ? 3 : 2) * TC * 4;
  constexpr int E_BYTES = TP * STG_STRIDE > RED_BYTES ? TP * STG_STRIDE : RED_BYTES;
  constexpr int LDS_BYTES = TILE_BYTES > E_BYTES ? TILE_BYTES : E_BYTES;
  static_assert(TP % RPG == 0 && (BKT == 32 || BKT == 64), "tile rows must be whole load sweeps");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

  const int bid = blockIdx.x;
  const int q = bid >> 3;
  const int ct = q % a.nct;
  const int pt = a.xcd_contiguous ? (bid & 7) * ((a.npt + 7) >> 3) + (q / a.nct) : (q / a.nct) * 8 + (bid & 7);
  if (pt >= a.npt) return;
  const int c0 = ct * TC, m0 = pt * TP;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wc = wave % WGC, wp = wave / WGC;
  const int lrow = tid / NS;
  // logical k-slot behind physical slot tid % NS of row lrow: the XOR of swz<NS> is its own inverse
  const int kvec = (swz<NS>(lrow, tid % NS) - lrow * RB) >> 4;

  int hb[VX], wb[VX], nb[VX]; bool mv[VX];
  const int HW = a.Hout * a.Wout;
#pragma unroll
  for (int i = 0; i < VX; ++i) {
    const int m = m0 + lrow + RPG * i;
    mv[i] = m < a.M;
    const int mm = mv[i] ? m : 0;
    const int n = mm / HW, rem = mm - n * HW;
    const int ho = rem / a.Wout, wo = rem - ho * a.Wout;
    hb[i] = ho * a.ostride - a.pad_h; wb[i] = wo * a.ostride - a.pad_w;
    nb[i] = n * a.Hin * a.Win;
  }
  const int ntiles = ANYC ? (a.Ktot + BKT - 1) / BKT : a.Ktot / BKT;
  const unsigned char* zero_page = reinterpret_cast<const unsigned char*>(g_zero_page);
  const int ps = a.xstride ? a.xstride : a.Cin;         // elements between neighbouring input pixels
  const int xcol = (kvec * 8) / ps;                     // pixel this thread's vector lies in, relative to the tap (0 unless xstride is set)
  int woff[VW]; bool wrow[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) {
    const int c = c0 + lrow + RPG * i;
    wrow[i] = (lrow + RPG * i < TC) & (c < a.Cout);
    woff[i] = (wrow[i] ? c : 0) * a.Ktot + kvec * 8;
  }
  int xoff[VX]; bool xok[VX];
  int kc0 = 0, kr = 0, ks = 0;
  int kc, gr, gs, kw = kvec * 8;                          // ANYC: channel and tap of this lane's vector, its k index
  {
    const int tap = kw / a.Cin;
    kc = kw - tap * a.Cin; gr = tap / a.KW; gs = tap - gr * a.KW;
  }
  unsigned char* const wave_base = lds + wave * 1024;     // a wave's 64 vectors = 1 KB of consecutive tile rows
  // all loads of the next k-tile (a tile never straddles a filter tap: the tap, the bounds test and the
  // pixel offset change only every Cin/64 tiles, a uniform branch)
  auto fetch = [&]() {
#pragma unroll
    for (int i = 0; i < VW; ++i) {
      const unsigned char* p = (wrow[i] & (!ANYC || kw < a.Ktot)) ? reinterpret_cast<const unsigned char*>(a.wt + woff[i]) : zero_page;
      __builtin_amdgcn_global_load_lds((gbl_void_ptr)p, (lds_void_ptr)(wave_base + i * (RPG * RB)), 16, 0, 0);
      woff[i] += BKT;
    }
    if (ANYC) {
#pragma unroll
      for (int i = 0; i < VX; ++i) {
        const int hi = hb[i] + gr, wi = wb[i] + gs;
        const bool ok = mv[i] & (gr < a.KH) & (hi >= 0) & (wi >= 0) & (hi < a.Hin) & (wi < a.Win);
        const unsigned char* p = ok ? reinterpret_cast<const unsigned char*>(a.in + (nb[i] + hi * a.Win + wi) * a.Cin + kc) : zero_page;
        __builtin_amdgcn_global_load_lds((gbl_void_ptr)p, (lds_void_ptr)(wave_base + XBASE + i * (RPG * RB)), 16, 0, 0);
      }
      kw += BKT; kc += BKT;
      while (kc >= a.Cin) { kc -= a.Cin; if (++gs == a.KW) { gs = 0; ++gr; } }
      return;
    }
    if (kc0 == 0) {
#pragma unroll
      for (int i = 0; i < VX; ++i) {
        const int hi = hb[i] + kr, wi = wb[i] + ks;
        xok[i] = mv[i] & (hi >= 0) & (wi + xcol >= 0) & (hi < a.Hin) & (wi + xcol < a.Win);
        xoff[i] = (nb[i] + hi * a.Win + wi) * ps + kvec * 8;
      }
    }
#pragma unroll
    for (int i = 0; i < VX; ++i) {
      const unsigned char* p = xok[i] ? reinterpret_cast<const unsigned char*>(a.in + xoff[i]) : zero_page;
      __builtin_amdgcn_global_load_lds((gbl_void_ptr)p, (lds_void_ptr)(wave_base + XBASE + i * (RPG * RB)), 16, 0, 0);
      xoff[i] += BKT;
    }
    kc0 += BKT;
    if (kc0 == a.Cin) { kc0 = 0; if (++ks == a.KW) { ks = 0; ++kr; } }
  };
  // fragment byte offsets for k-step 0; k-step kk is the slot pair 2*kk further on, i.e. offset ^ (kk * 32)
  int fa_off[NI], fb_off[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) fa_off[i] = swz<NS>(wc * WC + i * 32 + (lane & 31), lane >> 5);
#pragma unroll
  for (int j = 0; j < NJ; ++j) fb_off[j] = XBASE + swz<NS>(wp * WP + j * 32 + (lane & 31), lane >> 5);

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  for (int t = 0; t < ntiles; ++t) {
    fetch();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's vectors have landed ...
    __builtin_amdgcn_s_barrier();                         // ... and so have everyone else's
    Frag fa[2][NI], fb[2][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i) fa[0][i].u = *reinterpret_cast<const u32x4*>(lds + fa_off[i]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) fb[0][j].u = *reinterpret_cast<const u32x4*>(lds + fb_off[j]);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      if (kk + 1 < KS) {                                   // fragments of the next k-step under this one's MFMAs
#pragma unroll
        for (int i = 0; i < NI; ++i) fa[(kk + 1) & 1][i].u = *reinterpret_cast<const u32x4*>(lds + (fa_off[i] ^ ((kk + 1) * 32)));
#pragma unroll
        for (int j = 0; j < NJ; ++j) fb[(kk + 1) & 1][j].u = *reinterpret_cast<const u32x4*>(lds + (fb_off[j] ^ ((kk + 1) * 32)));
      }
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i].v, fb[kk & 1][j].v, acc[i][j], 0, 0, 0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();                         // everyone is done reading before the stage is overwritten
  }
  igemm_epilogue<TC, TP, WGC>(a, acc, lds, c0, m0, pt);
}

template <int TC, int TP, int WGC, int OCC, int BKT = 64, bool ANYC = false>
dat_status launch_igemm_dma(IgemmArgs a, hipStream_t st) {
  if ((int64_t)a.B * a.Hin * a.Win * a.Cin >= (1ll << 31) || (int64_t)a.Cout * a.Ktot >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;
  if (ANYC ? (a.Cin % 8 != 0 || a.Ktot != a.KH * a.KW * a.Cin || a.Ktot < BKT || a.xstride != 0)
           : (a.Cin % BKT != 0 || a.Ktot < BKT || a.Ktot % BKT != 0)) return DAT_ERR_UNSUPPORTED;
  if (a.xstride && (a.Cin != BKT || a.xstride % 8 != 0 || a.Cin % a.xstride != 0)) return DAT_ERR_UNSUPPORTED;   // one tap per k-tile
  a.nct = (a.Cout + TC - 1) / TC;
  a.npt = (a.M + TP - 1) / TP;
  if (a.npt == 0) return DAT_OK;
  a.xcd_contiguous = a.KH * a.KW > 1;   // filter windows: neighbouring tiles re-read each other's rows
  const int npt8 = (a.npt + 7) / 8 * 8;
  hipLaunchKernelGGL((igemm_dma_kernel<TC, TP, WGC, OCC, BKT, ANYC>), dim3((unsigned)(npt8 * a.nct)), dim3(kThreads), 0, st, a);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

// ---- ring variant for long contractions that fill the chip with ONE round of large tiles -----------------------
// 8 waves, 256-channel tiles, S LDS stages of 64-wide k-tiles filled by the same direct-to-LDS loads.  While tile t
// is multiplied, the loads of tile t+S-1 are issued during its first k-step (spread over the MFMA groups so that the
// address queue never holds a burst from all waves), and `s_waitcnt vmcnt((S-2)*loads)` at the end of the tile
// waits for tile t+1 only.  Half the operand bytes per FLOP of the 128x128 kernel; it pays when the layer is one
// round of at most one workgroup per CU (pick_ring), where the single-stage kernel cannot hide the load latency
// behind other workgroups.
template <int TC, int TP, int WGC, int S>
__global__ __launch_bounds__(512) void igemm_ring_kernel(IgemmArgs a) {
  constexpr int NT = 512, BKT = 64, KS = BKT / 16;
  constexpr int WGP = NT / 64 / WGC;
  constexpr int WC = TC / WGC, WP = TP / WGP;
  constexpr int NI = WC / 32, NJ = WP / 32;
  constexpr int RB = 128, RPG = NT / 8;                   // bytes per tile row; tile rows covered by one load per thread
  constexpr int VW = TC / RPG, VX = TP / RPG;
  constexpr int NL = VW + VX;                             // loads per thread per tile
  constexpr int TILE_BYTES = (TC + TP) * RB;
  constexpr int E_BYTES = TP * (TC * 2 + 16);
  constexpr int LDS_BYTES = (S * TILE_BYTES > E_BYTES) ? S * TILE_BYTES : E_BYTES;
  static_assert(TC % RPG == 0 && TP % RPG == 0, "tile rows must be whole load sweeps");
  static_assert(S >= 2 && (S - 2) * NL <= 63, "vmcnt range");
  static_assert(NI >= 2 && VW % (NI / 2) == 0 && VX % (NI - NI / 2) == 0, "loads spread evenly over the MFMA groups of a k-step");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

  const int bid = blockIdx.x;
  const int q = bid >> 3;
  const int ct = q % a.nct;
  const int pt = (q / a.nct) * 8 + (bid & 7);
  if (pt >= a.npt) return;
  const int c0 = ct * TC, m0 = pt * TP;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wc = wave % WGC, wp = wave / WGC;
  const int lrow = tid >> 3;
  const int kvec = (swz<8>(lrow, tid & 7) - lrow * RB) >> 4;   // logical k-slot behind physical slot tid & 7 of row lrow

  int hb[VX], wb[VX], nb[VX]; bool mv[VX];
  const int HW = a.Hout * a.Wout;
#pragma unroll
  for (int i = 0; i < VX; ++i) {
    const int m = m0 + lrow + RPG * i;
    mv[i] = m < a.M;
    const int mm = mv[i] ? m : 0;
    const int n = mm / HW, rem = mm - n * HW;
    const int ho = rem / a.Wout, wo = rem - ho * a.Wout;
    hb[i] = ho * a.ostride - a.pad_h; wb[i] = wo * a.ostride - a.pad_w;
    nb[i] = n * a.Hin * a.Win;
  }
  const int ntiles = a.Ktot / BKT;
  const unsigned char* zero_page = reinterpret_cast<const unsigned char*>(g_zero_page);
  int woff[VW]; bool wrow[VW];
#pragma unroll
  for (int i = 0; i < VW; ++i) {
    const int c = c0 + lrow + RPG * i;
    wrow[i] = c < a.Cout;
    woff[i] = (wrow[i] ? c : 0) * a.Ktot + kvec * 8;
  }
  int xoff[VX]; bool xok[VX];
  int kc0 = 0, kr = 0, ks = 0, kf = 0;
  bool tile_ok = true;
  unsigned char* sb = lds;
  // the loads of tile kf into ring stage `stage`, one at a time (tiles past the end fetch the zero page so that
  // every tile issues the same number of loads and the vmcnt arithmetic stays exact)
  auto fetch_begin = [&](int stage) { tile_ok = kf < ntiles; sb = lds + stage * TILE_BYTES + wave * 1024; };
  auto fetch_w = [&](int i) {
    const unsigned char* p = (tile_ok & wrow[i]) ? reinterpret_cast<const unsigned char*>(a.wt + woff[i]) : zero_page;
    __builtin_amdgcn_global_load_lds((gbl_void_ptr)p, (lds_void_ptr)(sb + i * (RPG * RB)), 16, 0, 0);
    woff[i] += BKT;
  };
  auto fetch_tap = [&]() {
    if (kc0 != 0) return;
#pragma unroll
    for (int i = 0; i < VX; ++i) {
      const int hi = hb[i] + kr, wi = wb[i] + ks;
      xok[i] = mv[i] & (hi >= 0) & (wi >= 0) & (hi < a.Hin) & (wi < a.Win);
      xoff[i] = (nb[i] + hi * a.Win + wi) * a.Cin + kvec * 8;
    }
  };
  auto fetch_x = [&](int i) {
    const unsigned char* p = (tile_ok & xok[i]) ? reinterpret_cast<const unsigned char*>(a.in + xoff[i]) : zero_page;
    __builtin_amdgcn_global_load_lds((gbl_void_ptr)p, (lds_void_ptr)(sb + TC * RB + i * (RPG * RB)), 16, 0, 0);
    xoff[i] += BKT;
  };
  auto fetch_end = [&]() {
    kc0 += BKT;
    if (kc0 == a.Cin) { kc0 = 0; if (++ks == a.KW) { ks = 0; ++kr; } }
    ++kf;
  };
  int fa_off[NI], fb_off[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) fa_off[i] = swz<8>(wc * WC + i * 32 + (lane & 31), lane >> 5);
#pragma unroll
  for (int j = 0; j < NJ; ++j) fb_off[j] = TC * RB + swz<8>(wp * WP + j * 32 + (lane & 31), lane >> 5);

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

#pragma unroll
  for (int p = 0; p < S - 1; ++p) {
    fetch_begin(p);
#pragma unroll
    for (int i = 0; i < VW; ++i) fetch_w(i);
    fetch_tap();
#pragma unroll
    for (int i = 0; i < VX; ++i) fetch_x(i);
    fetch_end();
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * NL) : "memory");
  __builtin_amdgcn_s_barrier();
  int stage = 0, fstage = S - 1;
  for (int t = 0; t < ntiles; ++t) {
    const unsigned char* cur = lds + stage * TILE_BYTES;
    Frag fa[2][NI], fb[2][NJ];
#pragma unroll
    for (int i = 0; i < NI; ++i) fa[0][i].u = *reinterpret_cast<const u32x4*>(cur + fa_off[i]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) fb[0][j].u = *reinterpret_cast<const u32x4*>(cur + fb_off[j]);
    fetch_begin(fstage);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk & 1][i].v, fb[kk & 1][j].v, acc[i][j], 0, 0, 0);
        if (i == 0 && kk + 1 < KS) {                       // fragments of the next k-step under this one's MFMAs
#pragma unroll
          for (int ii = 0; ii < NI; ++ii) fa[(kk + 1) & 1][ii].u = *reinterpret_cast<const u32x4*>(cur + (fa_off[ii] ^ ((kk + 1) * 32)));
#pragma unroll
          for (int j = 0; j < NJ; ++j) fb[(kk + 1) & 1][j].u = *reinterpret_cast<const u32x4*>(cur + (fb_off[j] ^ ((kk + 1) * 32)));
        }
        if (kk == 0) {   // the next ring tile: weights behind the first half of this k-step's MFMA groups, pixels behind the second
          constexpr int H = NI / 2;
          if (i < H) {
#pragma unroll
            for (int u = 0; u < VW / H; ++u) fetch_w(i * (VW / H) + u);
            if (i == H - 1) fetch_tap();
          } else {
#pragma unroll
            for (int u = 0; u < VX / (NI - H); ++u) fetch_x((i - H) * (VX / (NI - H)) + u);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    fetch_end();
    // this wave's part of tile t+1 has landed once at most (S-2) tiles of loads are outstanding; the barrier then
    // covers every wave's part, and everyone is done reading `stage`
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((S - 2) * NL) : "memory");
    __builtin_amdgcn_s_barrier();
    stage = stage + 1 == S ? 0 : stage + 1;
    fstage = fstage + 1 == S ? 0 : fstage + 1;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the zero-page loads of the tail land in LDS too
  __builtin_amdgcn_s_barrier();
  igemm_epilogue<TC, TP, WGC, NT>(a, acc, lds, c0, m0, pt);
}

template <int TC, int TP, int WGC, int S>
dat_status launch_igemm_ring(IgemmArgs a, hipStream_t st) {
  if ((int64_t)a.B * a.Hin * a.Win * a.Cin >= (1ll << 31) || (int64_t)a.Cout * a.Ktot >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;
  if (a.Cin % 64 != 0 || a.Ktot < 64 || a.xf_tab) return DAT_ERR_UNSUPPORTED;
  a.nct = (a.Cout + TC - 1) / TC;
  a.npt = (a.M + TP - 1) / TP;
  if (a.npt == 0) return DAT_OK;
  const int npt8 = (a.npt + 7) / 8 * 8;
  hipLaunchKernelGGL((igemm_ring_kernel<TC, TP, WGC, S>), dim3((unsigned)(npt8 * a.nct)), dim3(512), 0, st, a);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

__global__ void widen_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = bf2f(src[i]);
}

// OCC: waves per SIMD the register allocation is held to (1 = no constraint)
// 1x1 stride-1 layers whose operand is transformed on the way into LDS (see IgemmArgs::xf_x)
template <int TC, int TP, int WGC, int PF, int BKT, int OCC>
dat_status launch_igemm_xf(IgemmArgs a, hipStream_t st) {
  if ((int64_t)a.B * a.Hin * a.Win * a.Cin >= (1ll << 31) || (int64_t)a.Cout * a.Ktot >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;
  if (a.KH != 1 || a.KW != 1 || a.ostride != 1 || a.Cin % BKT != 0 || a.Ktot != a.Cin) return DAT_ERR_UNSUPPORTED;
  const size_t tab_bytes = (size_t)a.Cin * kBnTabFloatsPerChannel * sizeof(float);
  if (tab_bytes > 32768) return DAT_ERR_UNSUPPORTED;
  a.nct = (a.Cout + TC - 1) / TC;
  a.npt = (a.M + TP - 1) / TP;
  if (a.npt == 0) return DAT_OK;
  a.xcd_contiguous = 0;
  const int npt8 = (a.npt + 7) / 8 * 8;
  hipLaunchKernelGGL((igemm_kernel<TC, TP, WGC, PF, true, BKT, OCC, true>), dim3((unsigned)(npt8 * a.nct)), dim3(kThreads), tab_bytes, st, a);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

template <int TC, int TP, int WGC, int PF, int BKT, int OCC = 1>
dat_status launch_igemm(IgemmArgs a, hipStream_t st) {
  // 32-bit element offsets inside the kernel
  if ((int64_t)a.B * a.Hin * a.Win * a.Cin >= (1ll << 31) || (int64_t)a.Cout * a.Ktot >= (1ll << 31)) return DAT_ERR_UNSUPPORTED;
  a.nct = (a.Cout + TC - 1) / TC;
  a.npt = (a.M + TP - 1) / TP;
  if (a.npt == 0) return DAT_OK;
  a.xcd_contiguous = a.KH * a.KW > 1;   // filter windows: neighbouring tiles re-read each other's rows
  const int npt8 = (a.npt + 7) / 8 * 8;
  if (a.Cin % BKT == 0 && a.Ktot > 0)
    hipLaunchKernelGGL((igemm_kernel<TC, TP, WGC, PF, true, BKT, OCC>), dim3((unsigned)(npt8 * a.nct)), dim3(kThreads), 0, st, a);
  else
    hipLaunchKernelGGL((igemm_kernel<TC, TP, WGC, PF, false, BKT, OCC>), dim3((unsigned)(npt8 * a.nct)), dim3(kThreads), 0, st, a);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

template <int TC, int TP, int WGC>
dat_status pick_depth(const IgemmArgs& a, hipStream_t st) {
  // short contractions (1x1 layers with few input channels) gain nothing from deep prefetch;
  // long ones use 64-wide k-tiles (half the barriers per MFMA) when a tile cannot straddle a tap
  if (a.Ktot <= 128) return launch_igemm<TC, TP, WGC, 1, 32>(a, st);
  if (a.Cin % 64 == 0) return launch_igemm<TC, TP, WGC, 2, 64>(a, st);
  return launch_igemm<TC, TP, WGC, 3, 32>(a, st);
}

// 128-channel tiles, measured over the ResNet-50 layer shapes: four resident workgroups per CU beat
// two workgroups with deep register prefetch on every layer; when the contraction channels are a
// multiple of 64 the direct-to-LDS kernel (whole cache lines, no staging registers) is another
// ~10 % faster than the register-staged one with 32-wide k-tiles.
dat_status pick_depth_wide(const IgemmArgs& a, hipStream_t st) {
  if (a.Cin % 64 == 0 && a.Ktot >= 64) return launch_igemm_dma<128, 128, 2, 4>(a, st);
  return launch_igemm<128, 128, 2, 1, 32, 4>(a, st);
}

std::atomic<int64_t> g_launches{0};

int compute_units() {
  static std::atomic<int> cached{0};
  int n = cached.load(std::memory_order_relaxed);
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached.store(n, std::memory_order_relaxed);
  }
  return n;
}

// Which ring configuration, if any, runs this launch: 0 none, 1 = 256 channels x 256 pixels, 2 = 256 x 128.
// Long contractions into a multiple of 256 channels whose tiles make one round of 60-100 % of the CUs (measured at
// B = 256: 14x14 3x3 256->256 82 -> 66 us and 1024->256 42 -> 35 us with 256x256 tiles; 7x7 3x3 512->512 87 -> 75 us
// and 2048->512 44 -> 37 us with 256x128; slower than the 128x128 kernel wherever several rounds are needed or the
// contraction is short).
std::atomic<bool> g_ring_enabled{true};
std::atomic<bool> g_tile160{true};
std::atomic<bool> g_narrow_underfilled{true};

int pick_ring(const IgemmArgs& a) {
  if (a.xf_tab || a.ostep != 1 || a.stat_slab0 != 0 || a.Cin % 64 != 0 || a.Ktot < 1024 || a.Cout % 256 != 0) return 0;
  if (!g_ring_enabled.load(std::memory_order_relaxed)) return 0;   // dat_set_kernel_option: every layer through the 128x128 kernels
  const int64_t cus = compute_units(), nct = a.Cout / 256;
  const int64_t t256 = ((int64_t)a.M + 255) / 256 * nct, t128 = ((int64_t)a.M + 127) / 128 * nct;
  if (t256 <= cus && 5 * t256 >= 3 * cus) return 1;
  if (t128 <= cus && 5 * t128 >= 3 * cus) return 2;
  return 0;
}

// pixel rows per tile (= per slab of epilogue statistics) of the configuration run_igemm selects
int pixel_tile(const IgemmArgs& a) { return pick_ring(a) == 1 ? 256 : 128; }

dat_status run_igemm(const IgemmArgs& a, hipStream_t st) {
  g_launches.fetch_add(1, std::memory_order_relaxed);
  if (a.Cin % 8 != 0 || a.Cout % 8 != 0) return DAT_ERR_UNSUPPORTED;
  if (a.stat_mode == 3 && (a.Cout <= 64 || a.xf_tab)) return DAT_ERR_UNSUPPORTED;   // three sums: 128-channel tiles only
  if (a.xstride) {   // overlapping input pixels: the direct-to-LDS kernel with one tap per 64-wide k-tile
    if (a.Cout > 64 || a.xf_tab) return DAT_ERR_UNSUPPORTED;
    return a.Cout <= 32 ? launch_igemm_dma<32, 128, 1, 6>(a, st) : launch_igemm_dma<64, 128, 2, 5>(a, st);
  }
  switch (pick_ring(a)) {
    case 1: return launch_igemm_ring<256, 256, 2, 2>(a, st);
    case 2: return launch_igemm_ring<256, 128, 4, 3>(a, st);
    default: break;
  }
  if (a.xf_tab) {
    // 64-channel results (contraction 256, four k-tiles): one register set in flight and three workgroups per CU
    // beat two sets at two workgroups (15.6 -> 14.8 ms per step over these launches); for the 128-channel results the
    // same change gained nothing
    if (a.Cout <= 64) return launch_igemm_xf<64, 128, 2, 1, 64, 3>(a, st);
    return launch_igemm_xf<128, 128, 2, 2, 32, 2>(a, st);
  }
  // widths that are a multiple of 160 but not of 128 (the wide ResNets' 160 and 320 channels): 160-channel tiles, each
  // wave all channels of 32 pixels -- no empty MFMA rows in a last tile, and the gathered activations are fetched
  // once per 160 instead of once per 128 output channels
  if (a.Cout % 160 == 0 && a.Cout % 128 != 0 && g_tile160.load(std::memory_order_relaxed)) {
    if (a.Cin % 64 == 0 && a.Ktot >= 64) return launch_igemm_dma<160, 128, 1, 3>(a, st);
    if (a.Cin % 32 == 0 && a.Ktot >= 512 && !a.xstride) return launch_igemm_dma<160, 128, 1, 3, 64, true>(a, st);   // 160 -> 160
    return launch_igemm<160, 128, 1, 1, 32, 3>(a, st);
  }
  // narrow channel tiles: the direct-to-LDS kernel wherever its k-tile divides the contraction channels,
  // except 1x1 layers with a long contraction into <= 64 channels (HBM-bound reads: deep register
  // prefetch with two workgroups per CU streams them at the copy rate)
  if (a.Cout <= 32) {
    if (a.Cin % 64 == 0 && a.Ktot >= 64) return launch_igemm_dma<32, 128, 1, 6>(a, st);
    return pick_depth<32, 128, 1>(a, st);
  }
  if (a.Cout <= 64) {
    if (a.Cin % 64 == 0 && a.Ktot >= 64 && (a.KH * a.KW > 1 || a.Ktot < 256)) return launch_igemm_dma<64, 128, 2, 5>(a, st);
    if (a.Cin % 64 != 0 && a.Cin % 32 == 0 && a.Ktot >= 32) return launch_igemm_dma<64, 128, 2, 5, 32>(a, st);
    return pick_depth<64, 128, 2>(a, st);
  }
  // Long contractions whose 128x128 tiles would leave at most one and a half workgroups per CU (4x4 and 7x7 maps at
  // small batch): the single-stage kernel hides its load latency only behind other resident workgroups, so 32-channel
  // tiles -- four times the workgroups -- finish sooner although each fetches the activation tile again.  (Two and
  // a half workgroups per CU are enough: the 640-channel layers of the wide ResNets lose 12 % this way.)
  if (a.stat_mode != 3 && a.Cin % 64 == 0 && a.Ktot >= 1024 && g_narrow_underfilled.load(std::memory_order_relaxed)) {
    const int64_t wgs128 = (int64_t)((a.M + 127) / 128) * ((a.Cout + 127) / 128);
    if (2 * wgs128 <= 3 * (int64_t)compute_units()) return launch_igemm_dma<32, 128, 1, 6>(a, st);
  }
  return pick_depth_wide(a, st);
}

// ---- weight layouts ---------------------------------------------------------------------------
// master fp32 [Cout][k][k][cin_real] -> w [Cout][k][k][Cin] bf16 (zero padded channels) and the
// backward-data operand wT.
//   stride 1: wT [Cin][k][k][Cout], wT[ci][r'][s'][co] = w[co][k-1-r'][k-1-s'][ci].
//   stride 2: the input pixels split into four parity classes (h%2, w%2); class (ph,pw) only sees
//     the taps r = rf + 2i, s = sf + 2j with rf = (ph+pad)%2, sf = (pw+pad)%2, and is a dense
//     stride-1 convolution of dY with that nr x ns sub-filter.  wT holds the four flipped
//     sub-filters back to back: class q = 2*ph+pw at offset Cin*Cout*(taps of earlier classes),
//     laid out [Cin][nr][ns][Cout].
struct ParityClass { int rf, nr, pad; };
__host__ __device__ inline ParityClass parity_class(int p, int k, int pad) {
  ParityClass c;
  c.rf = (p + pad) & 1;
  c.nr = (k - c.rf + 1) / 2;
  if (c.rf >= k) c.nr = 0;
  const int off = (p + pad - c.rf) / 2;
  c.pad = c.nr - 1 - off;
  return c;
}

__global__ void weight_transform_kernel(const float* __restrict__ master, bf16_t* __restrict__ w, bf16_t* __restrict__ wT,
                                        int Cout, int k, int cin_real, int Cin, int stride, int pad) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)Cout * k * k * Cin) return;
  const int ci = (int)(i % Cin);
  int64_t p = i / Cin;
  const int s = (int)(p % k); p /= k;
  const int r = (int)(p % k);
  const int co = (int)(p / k);
  const bf16_t v = ci < cin_real ? f2bf(master[(((int64_t)co * k + r) * k + s) * cin_real + ci]) : (bf16_t)0;
  w[i] = v;
  if (stride == 1) {
    wT[(((int64_t)ci * k + (k - 1 - r)) * k + (k - 1 - s)) * Cout + co] = v;
  } else {
    // the class whose first tap has the parity of r (resp. s)
    const int ph = (r + pad) & 1, pw = (s + pad) & 1;      // (ph+pad)%2 == r%2  <=>  ph == (r+pad)%2
    int64_t base = 0;
    for (int q = 0; q < 2 * ph + pw; ++q)
      base += (int64_t)parity_class(q >> 1, k, pad).nr * parity_class(q & 1, k, pad).nr;
    const ParityClass ch = parity_class(ph, k, pad), cw = parity_class(pw, k, pad);
    const int ii = (r - ch.rf) / 2, jj = (s - cw.rf) / 2;
    wT[base * Cin * Cout + (((int64_t)ci * ch.nr + (ch.nr - 1 - ii)) * cw.nr + (cw.nr - 1 - jj)) * Cout + co] = v;
  }
}

// ---- 7x7 stride-2 pad-3 stem as a 4x4 stride-1 convolution over 2x2 pixel blocks -----------------
// With 3 input channels the stem wastes most of a 32-row MFMA tile in backward-data and needs a per-vector
// tap decode in forward.  Storing the network input as 2x2 pixel blocks of 4 channels (3 used; 8 bytes per
// pixel, 32 per block),
//   x2[n][i][j][(ph*2+pw)*4 + c] = x[n][2i+ph][2j+pw][c]      (H, W even),
// turns it into a dense layer with 16 input channels:
//   forward:       y[ho][wo][co]  = sum_{a,b<4} sum_v  x2[ho-2+a][wo-2+b][v] * Vf[co][a][b][v]
//                  Vf[co][a][b][(ph,pw,c)] = W[co][2a+ph-1][2b+pw-1][c]
//   backward-data: dx2[i][j][v]   = sum_{a,b<4} sum_co dy[i-1+a][j-1+b][co] * Vb[v][a][b][co]
//                  Vb[(ph,pw,c)][a][b][co] = W[co][5+ph-2a][5+pw-2b][c]
// (filter taps outside 0..6 and channel 3 are zero: 49 of the 64 window/parity pairs are used), one launch
// each, all four pixel parities of the input gradient at once.  The four blocks of a window row are
// contiguous in memory, so the forward pass reads them as ONE tap of 64 channels (IgemmArgs::xstride = 16):
// a 4 x 1 filter over 64-channel pixels that overlap their neighbours.
constexpr int kStemV = 16;     // values per 2x2 block: 4 positions x 4 channels
__global__ void stem_weight_transform_kernel(const float* __restrict__ master, bf16_t* __restrict__ vf, bf16_t* __restrict__ vb,
                                             int Cout, int cin_real) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Cout * 16 * kStemV) return;
  {   // vf[co][a][b][v]
    const int v = i & 15, b = (i >> 4) & 3, a = (i >> 6) & 3, co = i >> 8;
    const int ph = v >> 3, pw = (v >> 2) & 1, c = v & 3;
    const int r = 2 * a + ph - 1, s = 2 * b + pw - 1;
    const bool ok = c < cin_real && r >= 0 && r < 7 && s >= 0 && s < 7;
    vf[i] = ok ? f2bf(master[((co * 7 + r) * 7 + s) * cin_real + c]) : (bf16_t)0;
  }
  {   // vb[v][a][b][co]
    const int co = i % Cout; int t = i / Cout;
    const int b = t & 3, a = (t >> 2) & 3, v = t >> 4;
    const int ph = v >> 3, pw = (v >> 2) & 1, c = v & 3;
    const int r = 5 + ph - 2 * a, s = 5 + pw - 2 * b;
    const bool ok = c < cin_real && r >= 0 && r < 7 && s >= 0 && s < 7;
    vb[i] = ok ? f2bf(master[((co * 7 + r) * 7 + s) * cin_real + c]) : (bf16_t)0;
  }
}

// dW[co][r][s][c] = dVf[co][a][b][(ph,pw,c)] with r = 2a+ph-1, s = 2b+pw-1
__global__ void stem_wgrad_gather_kernel(const float* __restrict__ dv, float* __restrict__ dw, int Cout, int cin_real, uint32_t* __restrict__ absmax) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t m = 0;
  if (i < Cout * 49 * cin_real) {
    const int c = i % cin_real; int t = i / cin_real;
    const int s = t % 7; t /= 7;
    const int r = t % 7; const int co = t / 7;
    const int ph = (r + 1) & 1, a = (r + 1) >> 1, pw = (s + 1) & 1, b = (s + 1) >> 1;
    const float v = dv[((co * 4 + a) * 4 + b) * kStemV + (ph * 2 + pw) * 4 + c];
    dw[i] = v;
    m = abs_bits(v);
  }
  if (absmax) {   // (all 64 lanes of every wavefront reach this point)
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    if ((threadIdx.x & 63) == 0) absmax_publish(absmax_way(absmax, blockIdx.x), m);
  }
}

// ---- backward-weight ----------------------------------------------------------------------------
struct WgradArgs {
  const bf16_t* x;      // [B][H][W][Cin]
  const bf16_t* dy;     // [M][Cout], M = B*Ho*Wo
  float* ws;            // [splits][Cout][Ktot]
  int B, H, W, Cin, Ho, Wo, Cout, k, stride, pad;
  int M, Ktot, pix_per_split;
};

// ---- backward-weight through the LDS transpose reads of gfx950 -----------------------------------------------
// The contraction runs over pixels, but both operands are stored with channels contiguous.  Instead of transposing
// 8x8 blocks in registers, this kernel lands the tiles in LDS as they are in memory --
// dY [64 pixels][TC channels] and the shifted X [64 pixels][TJ columns], by the direct-to-LDS loads of the forward
// kernel -- and reads MFMA fragments with ds_read_b64_tr_b16: inside every group of 16 lanes, lane i receives
// element i%4 of the 8-byte chunks named by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 (checked on the device).  With
// source lane j pointing at pixel pb + j/4, channels cb + 4*(j%4) .. +3, lane i ends up with four consecutive pixels
// of channel cb + i: two such reads are the eight k values of a 32x32x16 operand.
// LDS rows are 32-byte-segment swizzled by pixel so that the 4 pixels x 2 segments a half-wave touches cover all
// banks; the swizzle is applied on the source side of the direct loads (16-byte chunks keep their pair).
typedef short v4s16 __attribute__((ext_vector_type(4)));
union FragTr { v4s16 h[2]; bf16x8 v; };

template <int ROWB> __device__ __forceinline__ int tr_seg_flip(int pixel) {
  return ROWB == 256 ? 2 * (pixel & 3) : 2 * ((pixel >> 1) & 1);     // 256-byte rows: 8 segments; 128-byte rows: 4
}

template <int TC, int TJ>
__global__ __launch_bounds__(kThreads, 4) void wgrad_kernel(WgradArgs a) {
  constexpr int BP = 64;                           // pixels per LDS tile
  constexpr int RA = TC * 2, RBJ = TJ * 2;         // bytes per pixel row of the two tiles
  constexpr int CA = RA / 16, CJ = RBJ / 16;       // 16-byte chunks per row
  constexpr int NA = TC / 32, NB = TJ / 32;        // direct loads per thread and tile (1 KB per wave instruction)
  constexpr int WC = TC / 2, WJ = TJ / 2;
  constexpr int NI = WC / 32, NJ = WJ / 32;
  static_assert((RA == 128 || RA == 256) && RBJ == 256, "row swizzles are written for 128- and 256-byte rows");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[BP * (RA + RBJ)];
  unsigned char* const abase = lds;
  unsigned char* const bbase = lds + BP * RA;

  const int c0 = blockIdx.x * TC, j0 = blockIdx.y * TJ;
  const int split = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wc = wave & 1, wj = wave >> 1;
  const int p_begin = split * a.pix_per_split;
  const int p_end = min(a.M, p_begin + a.pix_per_split);
  const int HW = a.Ho * a.Wo;
  const unsigned char* zero_page = reinterpret_cast<const unsigned char*>(g_zero_page);

  // ---- what each of this thread's direct loads fetches: wave instruction q = i*4 + wave fills 1 KB = 64/CA pixel rows
  int a_pr[NA]; bool a_ok[NA]; int64_t a_off[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int pr = (i * 4 + wave) * (64 / CA) + lane / CA, pc = lane % CA;
    const int lc = ((((pc >> 1) ^ tr_seg_flip<RA>(pr)) << 1) | (pc & 1));     // logical chunk behind physical chunk pc
    a_pr[i] = pr;
    a_ok[i] = c0 + lc * 8 < a.Cout;
    a_off[i] = (int64_t)(p_begin + pr) * a.Cout + c0 + lc * 8;
  }
  int b_pr[NB], b_r[NB], b_s[NB], b_ci[NB], b_n[NB], b_ho[NB], b_wo[NB]; bool b_ok[NB];
  const int step_q = BP / a.Wo, step_r = BP - step_q * a.Wo;     // 64 pixels further = step_q rows and step_r columns
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int pr = (i * 4 + wave) * (64 / CJ) + lane / CJ, pc = lane % CJ;
    const int lc = ((((pc >> 1) ^ tr_seg_flip<RBJ>(pr)) << 1) | (pc & 1));
    const int j = j0 + lc * 8;
    b_pr[i] = pr;
    b_ok[i] = j < a.Ktot;
    const int jj = b_ok[i] ? j : 0, tap = jj / a.Cin;
    b_ci[i] = jj - tap * a.Cin; b_r[i] = tap / a.k; b_s[i] = tap - b_r[i] * a.k;
    const int p = p_begin + pr;
    b_n[i] = p / HW; const int rem = p - b_n[i] * HW;
    b_ho[i] = rem / a.Wo; b_wo[i] = rem - b_ho[i] * a.Wo;
  }
  unsigned char* const wave_a = abase + wave * 1024;
  unsigned char* const wave_b = bbase + wave * 1024;
  auto fetch = [&](int p0) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      const bool ok = a_ok[i] && p0 + a_pr[i] < p_end;
      const unsigned char* src = ok ? reinterpret_cast<const unsigned char*>(a.dy + a_off[i]) : zero_page;
      __builtin_amdgcn_global_load_lds((gbl_void_ptr)src, (lds_void_ptr)(wave_a + i * 4096), 16, 0, 0);
      a_off[i] += (int64_t)BP * a.Cout;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int hi = b_ho[i] * a.stride + b_r[i] - a.pad, wi = b_wo[i] * a.stride + b_s[i] - a.pad;
      const bool ok = b_ok[i] && p0 + b_pr[i] < p_end && hi >= 0 && hi < a.H && wi >= 0 && wi < a.W;
      const unsigned char* src = ok ? reinterpret_cast<const unsigned char*>(a.x + (((int64_t)b_n[i] * a.H + hi) * a.W + wi) * a.Cin + b_ci[i]) : zero_page;
      __builtin_amdgcn_global_load_lds((gbl_void_ptr)src, (lds_void_ptr)(wave_b + i * 4096), 16, 0, 0);
      // the same lane's pixel in the next tile
      b_wo[i] += step_r; b_ho[i] += step_q;
      if (b_wo[i] >= a.Wo) { b_wo[i] -= a.Wo; ++b_ho[i]; }
      while (b_ho[i] >= a.Ho) { b_ho[i] -= a.Ho; ++b_n[i]; }
    }
  };
  // ---- fragment addresses: lane = 16 g + j names pixel 8 (g/2) + j/4 (+ 4 for the second read, + 16 per k-step) and
  // the 8-byte chunk of channels 16 (g%2) + 4 (j%4) of its 32-channel block
  const int g = lane >> 4, jl = lane & 15;
  const int fpix = 8 * (g >> 1) + (jl >> 2);
  int fa_off[NI], fb_off[NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int byte = (wc * WC + i * 32 + 16 * (g & 1) + 4 * (jl & 3)) * 2;
    fa_off[i] = fpix * RA + ((((byte >> 5) ^ tr_seg_flip<RA>(fpix)) << 5) | (byte & 31));
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int byte = (wj * WJ + j * 32 + 16 * (g & 1) + 4 * (jl & 3)) * 2;
    fb_off[j] = BP * RA + fpix * RBJ + ((((byte >> 5) ^ tr_seg_flip<RBJ>(fpix)) << 5) | (byte & 31));
  }

  f32x16 acc[NI][NJ];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  for (int p0 = p_begin; p0 < p_end; p0 += BP) {
    fetch(p0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int kk = 0; kk < BP / 16; ++kk) {
      FragTr fa[NI], fb[NJ];
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          fa[i].h[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s16*)(lds + fa_off[i] + (kk * 16 + 4 * h) * RA));
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          fb[j].h[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s16*)(lds + fb_off[j] + (kk * 16 + 4 * h) * RBJ));
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i].v, fb[j].v, acc[i][j], 0, 0, 0);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
  }
  // ---- partial tile -> workspace[split][co][j]   (lane: column j = l%32, rows co = 8g+4h+e)
  float* dst = a.ws + (int64_t)split * a.Cout * a.Ktot;
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int col = j0 + wj * WJ + j * 32 + (lane & 31);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int co = c0 + wc * WC + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        if (co < a.Cout && col < a.Ktot) dst[(int64_t)co * a.Ktot + col] = acc[i][j][e];
      }
    }
}

// Sums the `splits` partial tiles in a fixed order: a workgroup owns 32 consecutive elements (one cache line per
// split); thread group g = tid / 32 adds splits g, g+8, ... (eight loads in flight), then the eight group sums
// are added in order.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ ws, int splits, int64_t per_split, int Cin, int cin_real,
                                                           float scale, float* __restrict__ dw, uint32_t* __restrict__ absmax) {
  __shared__ float sh[8][32];
  const int lane = threadIdx.x & 31, grp = threadIdx.x >> 5;
  uint32_t* const slot = absmax ? absmax_way(absmax, blockIdx.x) : nullptr;
  const uint32_t seen = (slot && threadIdx.x == 0) ? absmax_peek(slot) : 0u;   // in flight with the loads below
  const int64_t i = (int64_t)blockIdx.x * 32 + lane;
  const int64_t ic = i < per_split ? i : per_split - 1;
  float s = 0.f;
  for (int k0 = grp; k0 < splits; k0 += 64) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int k = k0 + 8 * u;
      v[u] = ws[(int64_t)(k < splits ? k : splits - 1) * per_split + ic];
      if (k >= splits) v[u] = 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  sh[grp][lane] = s;
  __syncthreads();
  if (grp != 0) return;
  // (the 32 lanes of group 0 stay together to the end: their maximum is combined by lane exchanges)
  const int ci = (int)(ic % Cin);
  const bool live = i < per_split && ci < cin_real;
  s = 0.f;
#pragma unroll
  for (int g = 0; g < 8; ++g) s += sh[g][lane];
  const float v = s * scale;
  if (live) dw[(i / Cin) * cin_real + ci] = v;
  if (absmax) {
    uint32_t m = live ? abs_bits(v) : 0u;
#pragma unroll
    for (int d = 16; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d));
    if (lane == 0) absmax_raise(slot, seen, m);
  }
}

struct WgradPlan { int splits, pix_per_split, gx, gy; bool narrow; };

WgradPlan plan_wgrad(const ConvGeom& g) {
  WgradPlan p;
  const int M = g.B * g.Ho * g.Wo, Ktot = g.k * g.k * g.Cin;
  p.narrow = g.Cout <= 64;
  const int TC = p.narrow ? 64 : 128;
  p.gx = (g.Cout + TC - 1) / TC;
  p.gy = (Ktot + 127) / 128;
  const int tiles = p.gx * p.gy;
  int splits = (2048 + tiles - 1) / tiles;
  const int max_by_pixels = (M + 255) / 256;
  if (splits > max_by_pixels) splits = max_by_pixels;
  if (splits < 1) splits = 1;
  if (splits > 512) splits = 512;
  int pps = (M + splits - 1) / splits;
  pps = (pps + 63) / 64 * 64;
  p.pix_per_split = pps;
  p.splits = (M + pps - 1) / pps;
  return p;
}

}  // namespace

size_t conv_mfma_wgrad_workspace(const ConvGeom& g) {
  const WgradPlan p = plan_wgrad(g);
  return (size_t)p.splits * g.Cout * g.k * g.k * g.Cin * sizeof(float);
}

static void set_stats(IgemmArgs& a, const ConvStats* s, int slab0) {
  a.stat_mode = 0; a.stat_slab0 = slab0; a.stat_partial = nullptr;
  a.stat_x = nullptr; a.stat_mask = nullptr; a.stat_mean = nullptr; a.stat_rstd = nullptr;
  a.stat_x2 = nullptr; a.stat_mean2 = nullptr; a.stat_rstd2 = nullptr;
  if (!s || !s->mode) return;
  a.stat_mode = s->mode; a.stat_partial = s->partial;
  if (s->mode >= 2) { a.stat_x = s->bn_x; a.stat_mask = s->bn_mask; a.stat_mean = s->bn_mean; a.stat_rstd = s->bn_rstd; }
  if (s->mode == 3) { a.stat_x2 = s->bn_x2; a.stat_mean2 = s->bn_mean2; a.stat_rstd2 = s->bn_rstd2; }
}

int64_t conv_mfma_launch_count() { return g_launches.load(std::memory_order_relaxed); }

constexpr int kPixelTile = 128;   // TP of every configuration run_igemm selects

int conv_stat_slabs(int64_t rows, int stride) {
  // stride 2 backward-data runs four launches over the parity classes: at most 3 extra partial tiles
  return (int)((rows + kPixelTile - 1) / kPixelTile) + (stride == 2 ? 4 : 0);
}

dat_status conv_mfma_forward(const bf16_t* x, const bf16_t* w, const bf16_t* res, bf16_t* y, const ConvGeom& g, ConvStats* stats, hipStream_t st) {
  IgemmArgs a;
  a.xstride = 0;
  a.xf_x = nullptr; a.xf_mask = nullptr; a.xf_tab = nullptr;
  a.in = x; a.wt = w; a.res = res; a.res_mask = nullptr; a.res_even_only = 0; a.out = y;
  a.B = g.B; a.Hin = g.H; a.Win = g.W; a.Cin = g.Cin; a.Hout = g.Ho; a.Wout = g.Wo; a.Cout = g.Cout;
  a.KH = g.k; a.KW = g.k; a.ostride = g.stride; a.pad_h = a.pad_w = g.pad;
  a.outH = g.Ho; a.outW = g.Wo; a.ostep = 1; a.oh0 = a.ow0 = 0;
  a.M = g.B * g.Ho * g.Wo; a.Ktot = g.k * g.k * g.Cin; a.nct = a.npt = 0;
  set_stats(a, stats, 0);
  if (stats) stats->nslabs = (a.M + pixel_tile(a) - 1) / pixel_tile(a);
  return run_igemm(a, st);
}

bool conv_mfma_sparse_writer_ok(const ConvGeom& g) { return g.k == 1 && g.stride == 2 && g.pad == 0; }

bool conv_mfma_bn_operand_ok(const ConvGeom& g) {
  // The convolution's output channels are the contraction of its backward-data pass, its input channels the
  // rows of the result.  Every channel tile of the result transforms the operand again, so this pays only when
  // one tile covers all of them (measured: break-even at two tiles, a loss beyond) and the contraction is at
  // least two k-tiles long.
  return g.k == 1 && g.stride == 1 && g.pad == 0 && g.Cin % 8 == 0 && g.Cin > 32 && g.Cin <= 128 && g.Cout >= 2 * g.Cin &&
         g.Cout % (g.Cin <= 64 ? 64 : 32) == 0 && (size_t)g.Cout * kBnTabFloatsPerChannel * sizeof(float) <= 32768;
}

dat_status conv_mfma_backward_data(const bf16_t* dy, const bf16_t* wT, bf16_t* dx, const ConvGeom& g, bool accumulate, ConvStats* stats, hipStream_t st,
                                   const bf16_t* masked_res, const uint8_t* res_mask, const BnOperand* bn, int sparse) {
  if (accumulate && masked_res) return DAT_ERR_ARG;
  if (sparse == 1 && (!conv_mfma_sparse_writer_ok(g) || accumulate || masked_res || bn || (stats && stats->mode))) return DAT_ERR_ARG;
  if (sparse == 2 && !accumulate) return DAT_ERR_ARG;
  if (bn && !conv_mfma_bn_operand_ok(g)) return DAT_ERR_UNSUPPORTED;
  IgemmArgs a;
  a.xstride = 0;
  a.xf_x = nullptr; a.xf_mask = nullptr; a.xf_tab = nullptr;
  if (bn) { a.xf_x = bn->x; a.xf_mask = bn->mask; a.xf_tab = bn->tab; }
  a.in = dy; a.res = accumulate ? dx : masked_res; a.res_mask = masked_res ? res_mask : nullptr; a.out = dx;
  a.res_even_only = (sparse == 2 && g.stride == 1) ? 1 : 0;
  a.B = g.B; a.Hin = g.Ho; a.Win = g.Wo; a.Cin = g.Cout; a.Cout = g.Cin;
  a.ostride = 1; a.outH = g.H; a.outW = g.W; a.nct = a.npt = 0;
  if (g.stride == 1) {
    a.wt = wT; a.Hout = g.H; a.Wout = g.W; a.KH = a.KW = g.k; a.pad_h = a.pad_w = g.k - 1 - g.pad;
    a.ostep = 1; a.oh0 = a.ow0 = 0;
    a.M = g.B * g.H * g.W; a.Ktot = g.k * g.k * g.Cout;
    set_stats(a, stats, 0);
    if (stats) stats->nslabs = (a.M + pixel_tile(a) - 1) / pixel_tile(a);
    return run_igemm(a, st);
  }
  if (g.stride != 2) return DAT_ERR_UNSUPPORTED;
  int64_t base = 0;
  int slab0 = 0;
  for (int q = 0; q < 4; ++q) {
    const int ph = q >> 1, pw = q & 1;
    const ParityClass ch = parity_class(ph, g.k, g.pad), cw = parity_class(pw, g.k, g.pad);
    a.wt = wT + base * g.Cin * g.Cout;
    a.Hout = (g.H - ph + 1) / 2; a.Wout = (g.W - pw + 1) / 2;
    a.KH = ch.nr; a.KW = cw.nr; a.pad_h = ch.pad; a.pad_w = cw.pad;
    a.ostep = 2; a.oh0 = ph; a.ow0 = pw;
    a.M = g.B * a.Hout * a.Wout; a.Ktot = ch.nr * cw.nr * g.Cout;
    const bool taps = a.Ktot != 0;
    if (!taps) a.KH = a.KW = 1;         // class without taps: the launch only writes zeros (or keeps the stored gradient)
    if (sparse == 2) a.res = q == 0 ? dx : nullptr;   // the stored gradient exists at even rows and columns only
    set_stats(a, stats, slab0);
    if (sparse == 1 && !taps) continue;               // left unwritten: the accumulating pass that follows skips them
    if (a.M > 0) { dat_status s = run_igemm(a, st); if (s != DAT_OK) return s; }
    slab0 += (a.M + kPixelTile - 1) / kPixelTile;
    base += (int64_t)ch.nr * cw.nr;
  }
  if (stats) stats->nslabs = slab0;
  return DAT_OK;
}

// ---- stem on 2x2 pixel blocks ---------------------------------------------------------------------
bool conv_mfma_stem_blocked_ok(const ConvGeom& g, int cin_real) {
  return g.k == 7 && g.stride == 2 && g.pad == 3 && g.Cin == 8 && cin_real <= 4 && g.H % 2 == 0 && g.W % 2 == 0 && g.Cout % 8 == 0 && g.Cout <= 64;
}

ConvGeom conv_mfma_stem_blocked_geom(const ConvGeom& g) {
  ConvGeom q = g;
  q.H = g.H / 2; q.W = g.W / 2; q.Cin = kStemV; q.k = 4; q.stride = 1; q.pad = 2;   // Ho, Wo, Cout unchanged
  return q;
}

dat_status launch_stem_weight_transform(const float* master, bf16_t* vf, bf16_t* vb, int Cout, int cin_real, hipStream_t st) {
  const int n = Cout * 16 * kStemV;
  hipLaunchKernelGGL(stem_weight_transform_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, master, vf, vb, Cout, cin_real);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status conv_mfma_stem_forward(const bf16_t* x2, const bf16_t* vf, bf16_t* y, const ConvGeom& g, ConvStats* stats, hipStream_t st) {
  IgemmArgs a;
  a.xstride = 0;
  a.xf_x = nullptr; a.xf_mask = nullptr; a.xf_tab = nullptr;
  a.in = x2; a.wt = vf; a.res = nullptr; a.res_mask = nullptr; a.res_even_only = 0; a.out = y;
  // a window row of four blocks is one contiguous 64-value vector: 4 x 1 taps of 64 "channels", pixels kStemV apart
  a.B = g.B; a.Hin = g.H / 2; a.Win = g.W / 2; a.Cin = 4 * kStemV; a.xstride = kStemV; a.Hout = g.Ho; a.Wout = g.Wo; a.Cout = g.Cout;
  a.KH = 4; a.KW = 1; a.ostride = 1; a.pad_h = a.pad_w = 2;
  a.outH = g.Ho; a.outW = g.Wo; a.ostep = 1; a.oh0 = a.ow0 = 0;
  a.M = g.B * g.Ho * g.Wo; a.Ktot = 16 * kStemV; a.nct = a.npt = 0;
  set_stats(a, stats, 0);
  if (stats) stats->nslabs = (a.M + kPixelTile - 1) / kPixelTile;
  return run_igemm(a, st);
}

dat_status conv_mfma_stem_backward_data(const bf16_t* dy, const bf16_t* vb, bf16_t* dx2, const ConvGeom& g, bool accumulate, hipStream_t st) {
  IgemmArgs a;
  a.xstride = 0;
  a.xf_x = nullptr; a.xf_mask = nullptr; a.xf_tab = nullptr;
  a.in = dy; a.wt = vb; a.res = accumulate ? dx2 : nullptr; a.res_mask = nullptr; a.res_even_only = 0; a.out = dx2;
  a.B = g.B; a.Hin = g.Ho; a.Win = g.Wo; a.Cin = g.Cout; a.Hout = g.H / 2; a.Wout = g.W / 2; a.Cout = kStemV;
  a.KH = a.KW = 4; a.ostride = 1; a.pad_h = a.pad_w = 1;
  a.outH = a.Hout; a.outW = a.Wout; a.ostep = 1; a.oh0 = a.ow0 = 0;
  a.M = g.B * a.Hout * a.Wout; a.Ktot = 16 * g.Cout; a.nct = a.npt = 0;
  set_stats(a, nullptr, 0);
  return run_igemm(a, st);
}

dat_status conv_mfma_backward_weight(const bf16_t* x, const bf16_t* dy, float* dw, int cin_real, const ConvGeom& g, float scale,
                                     void* ws, hipStream_t st, uint32_t* absmax) {
  if (g.Cin % 8 != 0 || g.Cout % 8 != 0) return DAT_ERR_UNSUPPORTED;
  const WgradPlan p = plan_wgrad(g);
  WgradArgs a;
  a.x = x; a.dy = dy; a.ws = (float*)ws;
  a.B = g.B; a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.Ho = g.Ho; a.Wo = g.Wo; a.Cout = g.Cout;
  a.k = g.k; a.stride = g.stride; a.pad = g.pad;
  a.M = g.B * g.Ho * g.Wo; a.Ktot = g.k * g.k * g.Cin; a.pix_per_split = p.pix_per_split;
  const dim3 grid((unsigned)p.gx, (unsigned)p.gy, (unsigned)p.splits);
  if (p.narrow) hipLaunchKernelGGL((wgrad_kernel<64, 128>), grid, dim3(kThreads), 0, st, a);
  else hipLaunchKernelGGL((wgrad_kernel<128, 128>), grid, dim3(kThreads), 0, st, a);
  DAT_LAUNCH_CHECK();
  const int64_t per_split = (int64_t)g.Cout * a.Ktot;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((per_split + 31) / 32)), dim3(256), 0, st, (const float*)ws, p.splits,
                     per_split, g.Cin, cin_real, scale, dw, absmax);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

dat_status launch_weight_transform(const float* master, bf16_t* w, bf16_t* wT, int Cout, int k, int cin_real, int Cin, int stride,
                                   int pad, hipStream_t st) {
  const int64_t n = (int64_t)Cout * k * k * Cin;
  hipLaunchKernelGGL(weight_transform_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, master, w, wT, Cout, k, cin_real, Cin, stride, pad);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

// dw [Cout][7][7][cin_real] through the blocked layer's gradient dv [Cout][4][4][16] (scratch, fp32).
dat_status conv_mfma_stem_backward_weight(const bf16_t* x2, const bf16_t* dy, float* dw, float* dv, int cin_real, const ConvGeom& g,
                                          float scale, void* ws, hipStream_t st, uint32_t* absmax) {
  const ConvGeom q = conv_mfma_stem_blocked_geom(g);
  const dat_status s = conv_mfma_backward_weight(x2, dy, dv, kStemV, q, scale, ws, st);
  if (s != DAT_OK) return s;
  const int n = g.Cout * 49 * cin_real;
  hipLaunchKernelGGL(stem_wgrad_gather_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const float*)dv, dw, g.Cout, cin_real, absmax);
  DAT_LAUNCH_CHECK();
  return DAT_OK;
}

}  // namespace dat

// ---- C entry points for per-shape tests and timing -----------------------------------------------
using namespace dat;

extern "C" dat_status dat_set_kernel_option(dat_kernel_option opt, int value) {
  switch (opt) {
    case DAT_KOPT_RING_KERNEL: g_ring_enabled.store(value != 0, std::memory_order_relaxed); return DAT_OK;
    case DAT_KOPT_TILE_160: g_tile160.store(value != 0, std::memory_order_relaxed); return DAT_OK;
    case DAT_KOPT_NARROW_UNDERFILLED: g_narrow_underfilled.store(value != 0, std::memory_order_relaxed); return DAT_OK;
  }
  return DAT_ERR_ARG;
}

static bool geom_from(int B, int H, int W, int Cin, int Cout, int k, int stride, int pad, ConvGeom* g) {
  if (B < 1 || H < 1 || W < 1 || Cin < 8 || Cout < 8 || Cin % 8 || Cout % 8 || k < 1 || pad < 0 || pad >= k) return false;
  if (stride != 1 && stride != 2) return false;
  g->B = B; g->H = H; g->W = W; g->Cin = Cin; g->Cout = Cout; g->k = k; g->stride = stride; g->pad = pad;
  g->Ho = (H + 2 * pad - k) / stride + 1; g->Wo = (W + 2 * pad - k) / stride + 1;
  if (g->Ho < 1 || g->Wo < 1) return false;
  if ((int64_t)B * H * W * Cin >= (1ll << 31) || (int64_t)B * g->Ho * g->Wo * Cout >= (1ll << 31)) return false;
  return true;
}

extern "C" dat_status dat_conv_forward(const uint16_t* x, const uint16_t* w, uint16_t* y, int B, int H, int W, int Cin,
                                       int Cout, int k, int stride, int pad, void* stream) {
  ConvGeom g;
  if (!x || !w || !y || !geom_from(B, H, W, Cin, Cout, k, stride, pad, &g)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(w, 16) || !aligned(y, 16)) return DAT_ERR_ARG;
  return conv_mfma_forward(x, w, nullptr, y, g, nullptr, (hipStream_t)stream);
}

extern "C" dat_status dat_conv_backward_data(const uint16_t* dy, const uint16_t* w, uint16_t* dx, int B, int H, int W,
                                             int Cin, int Cout, int k, int stride, int pad, void* stream) {
  ConvGeom g;
  if (!dy || !w || !dx || !geom_from(B, H, W, Cin, Cout, k, stride, pad, &g)) return DAT_ERR_ARG;
  if (!aligned(dy, 16) || !aligned(w, 16) || !aligned(dx, 16)) return DAT_ERR_ARG;
  // build the flipped transpose of w on the fly (test/timing path; the model caches it)
  hipStream_t st = (hipStream_t)stream;
  const size_t n = (size_t)Cout * k * k * Cin;
  float* wf = nullptr; bf16_t* w2 = nullptr; bf16_t* wT = nullptr;
  if (hipMalloc((void**)&wf, n * 4) != hipSuccess || hipMalloc((void**)&w2, n * 2) != hipSuccess ||
      hipMalloc((void**)&wT, n * 2) != hipSuccess) {
    (void)hipGetLastError();
    if (wf) (void)hipFree(wf);
    if (w2) (void)hipFree(w2);
    return DAT_ERR_NOMEM;
  }
  dat_status s = DAT_OK;
  hipLaunchKernelGGL(widen_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, wf, (int64_t)n);
  if (hipGetLastError() != hipSuccess) s = DAT_ERR_HIP;
  if (s == DAT_OK) s = launch_weight_transform(wf, w2, wT, Cout, k, Cin, Cin, stride, pad, st);
  if (s == DAT_OK) s = conv_mfma_backward_data(dy, wT, dx, g, false, nullptr, st);
  (void)hipStreamSynchronize(st);
  (void)hipFree(wf); (void)hipFree(w2); (void)hipFree(wT);
  return s;
}

extern "C" dat_status dat_conv_backward_weight(const uint16_t* x, const uint16_t* dy, float* dw, int B, int H, int W,
                                               int Cin, int Cout, int k, int stride, int pad, void* stream) {
  ConvGeom g;
  if (!x || !dy || !dw || !geom_from(B, H, W, Cin, Cout, k, stride, pad, &g)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(dw, 16)) return DAT_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  void* ws = nullptr;
  if (hipMalloc(&ws, conv_mfma_wgrad_workspace(g)) != hipSuccess) { (void)hipGetLastError(); return DAT_ERR_NOMEM; }
  dat_status s = conv_mfma_backward_weight(x, dy, dw, Cin, g, 1.0f, ws, st);
  (void)hipStreamSynchronize(st);
  (void)hipFree(ws);
  return s;
}

// ---- backward-weight without any allocation ------------------------------------------------------
// The split partial tiles of wgrad_kernel go to a buffer that is part of the library's device image instead
// of a workspace allocated per call: for callers that may not allocate (stream capture, serving loops).
// Each GPU holds its own copy of the array at its own address; in host code the array's name is only a handle
// for hipGetSymbolAddress, so the address is looked up once per device and that pointer is what the kernels get.
#define DAT_STATIC_SCRATCH_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[DAT_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
dat_status static_scratch(void** out) {
  int dev = -1;
  DAT_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail_with(DAT_ERR_UNSUPPORTED, "device ordinal beyond the static scratch table");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    DAT_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail_with(DAT_ERR_HIP, "hipGetSymbolAddress returned a null address for the static scratch");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DAT_OK;
}
}  // namespace

extern "C" size_t dat_conv_backward_weight_static_limit(void) { return (size_t)DAT_STATIC_SCRATCH_BYTES; }

extern "C" dat_status dat_conv_backward_weight_static(const uint16_t* x, const uint16_t* dy, float* dw, int B, int H, int W,
                                                      int Cin, int Cout, int k, int stride, int pad, void* stream) {
  ConvGeom g;
  if (!x || !dy || !dw || !geom_from(B, H, W, Cin, Cout, k, stride, pad, &g)) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(dw, 16)) return DAT_ERR_ARG;
  if (conv_mfma_wgrad_workspace(g) > (size_t)DAT_STATIC_SCRATCH_BYTES)
    return fail_with(DAT_ERR_UNSUPPORTED, "dat_conv_backward_weight_static: the split partial sums of this shape exceed the 32 MiB static scratch "
                                          "(use dat_conv_backward_weight)");
  void* ws = nullptr;
  const dat_status s = static_scratch(&ws);
  if (s != DAT_OK) return s;
  // every partial tile the reduction reads is written by this call's first launch: nothing to clear
  return conv_mfma_backward_weight(x, dy, dw, Cin, g, 1.0f, ws, (hipStream_t)stream);
}
