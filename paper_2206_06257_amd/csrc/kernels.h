// Internal launch interfaces between the translation units of libdat.
#pragma once
#include "common.h"

namespace dat {

// ---- attack elementwise kernels (pgd.hip) --------------------------------------------------
struct NetInputDesc {
  void* ptr;          // network input tensor, or nullptr
  int bf16;           // 1: bf16 NHWC with channels padded to 8 (pad = 0); 0: fp32 NHWC, 3 channels
  int normalize;
  float mean[3], inv_std[3];
  int block_h, block_w;   // bf16 only: image height/width when the tensor is stored as 2x2 pixel blocks of 4 channels ([H/2][W/2][4*4]: 8 bytes per pixel), else 0
};
// z_0 (and optionally the network input at x + z_0) for `npix` pixels of 3 channels.
dat_status launch_attack_init(const float* x, int64_t npix, float eps, dat_init init, float* delta,
                              const NetInputDesc& in, hipStream_t st);
// One projected sign step in place (and optionally the network input at the new point).
dat_status launch_attack_update(const float* x, const float* G, float* delta, int64_t npix, float eps,
                                float alpha, const NetInputDesc& in, hipStream_t st);
// The same step with the gradient taken from the bf16 network-input gradient `gnet` (the layout `in` describes; only
// the sign of its first three channels per pixel is used), for bf16 models: no fp32 copy of the gradient is made.
dat_status launch_attack_update_netgrad(const float* x, const void* gnet, float* delta, int64_t npix, float eps,
                                        float alpha, const NetInputDesc& in, hipStream_t st);
// Network input from pixels alone (delta = nullptr) or from x + delta.
dat_status launch_make_input(const float* x, const float* delta, int64_t npix, const NetInputDesc& in,
                             hipStream_t st);

}  // namespace dat

namespace dat {

// ---- tensors ---------------------------------------------------------------------------------
// All activation tensors are NHWC with `rows` = B*H*W pixels of C contiguous channels, stored
// as fp32 (dtype 0) or bf16 (dtype 1).  C is a multiple of 8.
struct ConvGeom {
  int B, H, W, Cin;      // input  [B,H,W,Cin]
  int Ho, Wo, Cout;      // output [B,Ho,Wo,Cout]
  int k, stride, pad;
};

// ---- fp32 direct convolutions (conv_direct.hip): the DAT_F32 path ------------------------------
dat_status conv_direct_forward(const float* x, const float* w, const float* res, float* y, const ConvGeom& g, hipStream_t st);
dat_status conv_direct_backward_data(const float* dy, const float* w, float* dx, const ConvGeom& g, bool accumulate, hipStream_t st);
dat_status conv_direct_backward_weight(const float* x, const float* dy, float* dw, const ConvGeom& g, float scale, hipStream_t st);

// ---- bf16 implicit-GEMM convolutions on MFMA (conv_mfma.hip): the DAT_BF16 path ----------------
// w: [Cout][k][k][Cin] bf16.  wT: the backward-data operand built by launch_weight_transform
// (flipped transpose for stride 1, four parity-class sub-filters for stride 2).
// Optional fused batch statistics: with mode 1 the forward (or backward-data) epilogue also writes
// per-channel (sum v, sum v^2) of everything it stores, as `nslabs` slabs of [2][C] floats in
// `partial` (C = channels of the stored tensor); conv_stat_slabs gives an upper bound for sizing.
// Reduce them with bn_finalize_slabs.
// Mode 2 (backward-data): the stored tensor is d(out) of a batch normalisation with input bn_x (same layout),
// ReLU mask bn_mask (or nullptr) and batch statistics bn_mean / bn_rstd; the slabs then hold
// (sum dy, sum dy*xhat), dy = d(out) .* mask: the sums of that normalisation's backward pass.
struct ConvStats {
  int mode;
  float* partial;
  int nslabs;            // out
  const bf16_t* bn_x; const uint8_t* bn_mask; const float* bn_mean; const float* bn_rstd;   // mode 2, 3
  // mode 3 (results with more than 64 channels): a second normalisation with input bn_x2 shares d(out); slabs are
  // [3][C]: (sum dy, sum dy*xhat, sum dy*xhat2)
  const bf16_t* bn_x2; const float* bn_mean2; const float* bn_rstd2;
};
// Number of MFMA convolution kernels (igemm) launched by this process so far.
int64_t conv_mfma_launch_count();
int conv_stat_slabs(int64_t rows, int stride);
dat_status conv_mfma_forward(const bf16_t* x, const bf16_t* w, const bf16_t* res, bf16_t* y, const ConvGeom& g, ConvStats* stats, hipStream_t st);
// masked_res (optional, instead of `accumulate`): dx = conv^T(dy) + masked_res .* mask, mask one bit per element (bit j of
// byte e/8): the gradient a residual connection carries past a ReLU, taken from the ReLU's output gradient directly.
// bn (optional, layers for which conv_mfma_bn_operand_ok holds): `dy` is the output gradient of the batch normalisation
// that follows this convolution; the pass then contracts bn_input_grad(dy .* mask, x, constants) rounded to bf16, i.e.
// what bnact_backward would have written as dx, without that tensor ever being stored.
struct BnOperand {
  const bf16_t* x;       // the normalisation's input (= this convolution's forward output)
  const uint8_t* mask;   // ReLU mask of the normalisation's output, or nullptr
  const float* tab;      // constants written by bnact_backward
};
bool conv_mfma_bn_operand_ok(const ConvGeom& g);
// sparse: 1 (1x1 stride-2 layers without padding, conv_mfma_sparse_writer_ok, not accumulating): only the input pixels
// the layer reads (even row, even column) are written; the other three quarters of dx, which would be zero, are
// left as they are.  2 (accumulating): the stored dx is such a tensor -- it is read at even rows and columns only
// and counts as zero elsewhere.  A pair of such calls gives the bits of a pair of plain calls without the zeros ever
// being written or read back.
bool conv_mfma_sparse_writer_ok(const ConvGeom& g);
dat_status conv_mfma_backward_data(const bf16_t* dy, const bf16_t* wT, bf16_t* dx, const ConvGeom& g, bool accumulate, ConvStats* stats, hipStream_t st,
                                   const bf16_t* masked_res = nullptr, const uint8_t* res_mask = nullptr, const BnOperand* bn = nullptr,
                                   int sparse = 0);
// dw fp32 [Cout][k][k][Cin_real] (Cin_real <= g.Cin: padded input channels are dropped), scaled.
// `ws` is a workspace of conv_mfma_wgrad_workspace(g) bytes.
size_t conv_mfma_wgrad_workspace(const ConvGeom& g);
// absmax (optional): the tensor's group of kAbsmaxWays slots that receive max |dw| (see absmax_way).
dat_status conv_mfma_backward_weight(const bf16_t* x, const bf16_t* dy, float* dw, int cin_real, const ConvGeom& g, float scale, void* ws, hipStream_t st,
                                     uint32_t* absmax = nullptr);
// A 7x7 stride-2 pad-3 convolution of an input with at most 4 real channels (H, W even) can run as a 4x4
// stride-1 convolution over 2x2 pixel blocks when the input tensor is stored blocked with 4 channels per pixel,
// x2[n][i][j][(ph*2+pw)*4 + c] = x[n][2i+ph][2j+pw][c]; `g` is always the original geometry.
// vf [Cout][4][4][16] and vb [16][4][4][Cout] are the forward and backward-data operands; dx2 is blocked too.
bool conv_mfma_stem_blocked_ok(const ConvGeom& g, int cin_real);
ConvGeom conv_mfma_stem_blocked_geom(const ConvGeom& g);
dat_status launch_stem_weight_transform(const float* master, bf16_t* vf, bf16_t* vb, int Cout, int cin_real, hipStream_t st);
dat_status conv_mfma_stem_forward(const bf16_t* x2, const bf16_t* vf, bf16_t* y, const ConvGeom& g, ConvStats* stats, hipStream_t st);
dat_status conv_mfma_stem_backward_data(const bf16_t* dy, const bf16_t* vb, bf16_t* dx2, const ConvGeom& g, bool accumulate, hipStream_t st);
// dv: [Cout][4][4][16] fp32 scratch; ws: conv_mfma_wgrad_workspace(conv_mfma_stem_blocked_geom(g)) bytes.
dat_status conv_mfma_stem_backward_weight(const bf16_t* x2, const bf16_t* dy, float* dw, float* dv, int cin_real, const ConvGeom& g,
                                          float scale, void* ws, hipStream_t st, uint32_t* absmax = nullptr);
// master fp32 [Cout][k][k][cin_real] -> w bf16 [Cout][k][k][Cin] (zero padded) and wT.
dat_status launch_weight_transform(const float* master, bf16_t* w, bf16_t* wT, int Cout, int k, int cin_real, int Cin, int stride, int pad, hipStream_t st);

// ---- everything that is not a convolution (layers.hip) -----------------------------------------
// Batch statistics of x[rows][C]: mean[C], rstd[C] = 1/sqrt(var + 1e-5) (biased variance).
// `partial` holds bn_partial_floats(rows, C) floats.
size_t bn_partial_floats(int64_t rows, int C);
dat_status bn_stats(const void* x, int dtype, int64_t rows, int C, float* partial, float* mean, float* rstd, hipStream_t st);
// Reduces `nslabs` slabs of [2][C] partial sums (from a convolution epilogue) in a fixed order.
//   mode 1: mean[C], rstd[C] from (sum x, sum x^2) over `rows` rows  (o1 = mean, o2 = rstd)
//   mode 2: sums[0..C) = sum dy, sums[C..2C) = sum dy*xhat (o1 = sums, o2 = sums + C), and
//           dbeta = scale*sum dy, dgamma = scale*sum dy*xhat when the pointers are non-null.
// `partial` must have room for fold_floats(nslabs, C) more floats after the slabs.
size_t fold_floats(int nslabs, int C);
//           With gamma/mean/rstd/tab the constants of bn_input_grad are written too.
//           nsum / col2: the slabs hold nsum rows of C sums each; the pair reduced is (row 0, row col2).  With three rows
//           call it once per pair; `fold` = false skips the folding of many slabs (done by an earlier call).
dat_status bn_finalize_slabs(float* partial, int nslabs, int C, int64_t rows, int mode, float* o1, float* o2, float* dbeta,
                             float* dgamma, float scale, hipStream_t st, const float* gamma = nullptr, const float* mean = nullptr,
                             const float* rstd = nullptr, float* tab = nullptr, int nsum = 2, int col2 = 1, bool fold = true,
                             ParamAbsmax am = ParamAbsmax{nullptr, nullptr});   // am: abs-max slots of (dbeta, dgamma)
// out = act(gamma*((x-mean)*rstd) + beta [+ res])
// mask (optional, rows*C/8 bytes): bit j of byte e/8 = (out[e] > 0), what the backward pass needs of `out`.
// res_bn (optional): `res` is the INPUT of a second normalisation without activation (the one on a projection
// shortcut); the residual added is its output rounded to the storage type, which is then never stored.
struct BnParams { const float* mean; const float* rstd; const float* gamma; const float* beta; };
dat_status bnact_forward(const void* x, const void* res, void* out, uint8_t* mask, int dtype, int64_t rows, int C, const float* mean,
                         const float* rstd, const float* gamma, const float* beta, int relu, hipStream_t st, const BnParams* res_bn = nullptr);
// Backward, first half.  dy = dout masked by (out > 0) if relu.  sums[0..C) = sum dy (= dbeta), sums[C..2C) = sum dy*xhat
// (= dgamma); dgamma/dbeta (fp32, may be null) receive scale*sums; tab (4*C floats) receives the per-channel constants
// of bn_input_grad.  second (optional; needs relu and mask): a second normalisation that sees the same dy -- its
// sums, constants and parameter gradients come out of the same pass over dy.
struct BnSecond {
  const void* x; const float* mean; const float* rstd; const float* gamma;
  float* sums; float* tab; float* dgamma; float* dbeta;
  ParamAbsmax am;      // abs-max slots of (dbeta, dgamma), or nulls
};
dat_status bn_backward_reduce(const void* x, const void* out, const uint8_t* mask, const void* dout, int dtype, int64_t rows, int C,
                              const float* mean, const float* rstd, const float* gamma, int relu, float* partial, float* sums,
                              float* tab, float* dgamma, float* dbeta, float scale, hipStream_t st, const BnSecond* second = nullptr,
                              ParamAbsmax am = ParamAbsmax{nullptr, nullptr});
// Backward, second half: dx (+)= bn_input_grad(dy, x, tab) = gamma*rstd*(dy - dbeta/rows - xhat*dgamma/rows); dres (+)= dy.
dat_status bn_backward_apply(const void* x, const void* out, const uint8_t* mask, const void* dout, void* dx, bool dx_accumulate, void* dres,
                             bool dres_accumulate, int dtype, int64_t rows, int C, const float* tab, int relu, hipStream_t st);
// Both halves for a BN + ReLU (mask required) whose output feeds a 3x3/2 max-pool (padding 1) and nothing else, walked
// in 2x2 pixel blocks.  gather = 1: d(out) is not read from `dout` but gathered from the pool's output gradient through
// the recorded arg-max positions (the pool's backward pass evaluated in place and rounded to the storage type like the
// tensor it replaces); gather = 0: d(out) is read from `dout`.  Same summation order either way.
struct PoolGrad { const uint8_t* arg; const void* dpooled; int B, H, W, Ho, Wo; int gather; };
dat_status bn_pool_backward(const void* x, const uint8_t* mask, const void* dout, void* dx, bool dx_accumulate, bool skip_apply, int dtype, int C,
                            const float* mean, const float* rstd, const float* gamma, float* partial, float* sums, float* tab,
                            float* dgamma, float* dbeta, float scale, const PoolGrad& pg, hipStream_t st,
                            ParamAbsmax am = ParamAbsmax{nullptr, nullptr});
// relu(gamma*((x-mean)*rstd)+beta) followed by the 3x3/2 max-pool in one pass: writes the pooled tensor, the arg-max
// positions (as maxpool_forward) and the ReLU mask of every input pixel (as bnact_forward); the activated tensor is not stored.
dat_status bnact_pool_forward(const void* x, void* pooled, uint8_t* arg, uint8_t* mask, int dtype, int B, int H, int W, int C, int Ho, int Wo,
                              const float* mean, const float* rstd, const float* gamma, const float* beta, hipStream_t st);
dat_status biasact_forward(const void* x, void* out, int dtype, int64_t rows, int C, const float* bias, int relu, hipStream_t st);
dat_status biasact_backward(const void* out, const void* dout, void* dx, bool dx_accumulate, int dtype, int64_t rows, int C,
                            int relu, float* partial, float* dbias, float scale, hipStream_t st);
// arg: one byte per output element, the window position (3*r+s) of the first maximum.
dat_status maxpool_forward(const void* x, void* out, uint8_t* arg, int dtype, int B, int H, int W, int C, int Ho, int Wo, hipStream_t st);
dat_status maxpool_backward(const uint8_t* arg, const void* dout, void* dx, bool accumulate, int dtype, int B, int H, int W, int C,
                            int Ho, int Wo, hipStream_t st);
// pooled[B][C] fp32 = mean over the HW pixels;  backward: dx (+)= dpooled/HW.
dat_status gap_forward(const void* x, float* pooled, int dtype, int B, int HW, int C, hipStream_t st);
dat_status gap_backward(const float* dpooled, void* dx, bool accumulate, int dtype, int B, int HW, int C, hipStream_t st);
// logits[B][O] = f[B][I] . W[O][I]^T + b;  backward: df, and (if dW) dW = scale * dz^T f, db = scale * sum dz.
// ws: optional scratch of fc_workspace_floats(B, I, O) floats (long contractions are then split over more workgroups and
// summed in a fixed order).
size_t fc_workspace_floats(int B, int I, int O);
dat_status fc_forward(const float* f, const float* W, const float* b, float* logits, int B, int I, int O, float* ws, hipStream_t st);
dat_status fc_backward(const float* f, const float* W, const float* dz, float* df, float* dW, float* db, int B, int I, int O,
                       float scale, float* ws, hipStream_t st, ParamAbsmax am = ParamAbsmax{nullptr, nullptr});   // am: slots of (dW, db)
// Softmax cross-entropy: loss_n per sample, dz = (softmax - onehot) * gscale; loss_mean[0] = mean loss_n.
dat_status ce_forward_backward(const float* logits, const int32_t* y, float* dz, float* loss_n, float* loss_mean, int B, int O,
                               float gscale, hipStream_t st);
// TRADES regulariser KL(softmax z_clean || softmax z_adv): logit gradient of one branch (0: the perturbed pass,
// dz = (q-p)*gscale, loss_n = KL; 1: the clean pass, dz = (lambda*(p-onehot) + p*(log p - log q - KL))*gscale, loss_n = CE).
dat_status kl_forward_backward(const float* z_clean, const float* z_adv, const int32_t* y, int branch, float lambda, float* dz,
                               float* loss_n, float* loss_mean, int B, int O, float gscale, hipStream_t st);
// fp32 -> bf16 copy (linear weights) ; first-layer gradient [rows][Cpad] -> gx[rows][3] * inv_std.
dat_status launch_round_bf16_values(const float* src, float* dst, int64_t n, hipStream_t st);
// block_h, block_w > 0: g0 is stored as 2x2 pixel blocks of a block_h x block_w image (Cpad = 4 then).
dat_status launch_input_grad(const void* g0, int dtype, int Cpad, int64_t rows, float s0, float s1, float s2, float* gx,
                             int block_h, int block_w, hipStream_t st);
dat_status launch_sgd(float* theta, const float* g, float lr, int64_t n, hipStream_t st);
dat_status launch_fill_zero(void* p, size_t bytes, hipStream_t st);
// Per-tensor abs-max slots (kAbsmaxWays per tensor, see absmax_way) -> one value per tensor.
dat_status launch_absmax_fold(const uint32_t* ways, int T, uint32_t* scales, hipStream_t st);

}  // namespace dat

namespace dat {

// ---- optimizer and aggregation (optim.hip) -------------------------------------------------------
struct LambParams {
  int use_adam;
  float eta, b1, b2, zeta, wd, c_l, c_u;
  float inv_bc1, inv_bc2;      // 1/(1-b1^t), 1/(1-b2^t)
};
// One LALR/LAMB step on the flat fp32 vectors; `norms` is a scratch of 2*T doubles.
dat_status launch_lamb(float* theta, const float* g, float* m, float* v, float* u, const int64_t* off, int T, int64_t d,
                       const LambParams& hp, double* norms, hipStream_t st);

struct AggregateArgs {
  const uint8_t* q[DAT_MAX_WORKERS];
  const float* scales[DAT_MAX_WORKERS];
  int M, T;
  const int64_t* offsets;
  int64_t d;
  float* out;
};

}  // namespace dat
