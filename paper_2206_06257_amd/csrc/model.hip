// Host side of libdat: the static layer graph of each architecture, its device memory, and
// the three passes built from it -- forward, backward-to-input, backward-with-weight-gradients
// -- plus the C entry points dat_attack / dat_step / dat_input_grad that sequence them
// (Alg. A1, worker block, steps 5 and 6).  No arithmetic happens here: every step is a kernel
// launch on the caller's stream.
//
// Gradient storage rule: every activation tensor has one gradient buffer in the model's
// storage type.  Contributions arrive in reverse op order; the first one is stored, later
// ones are added to the stored value (read-modify-write in the consumer's kernel).
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <math.h>
#include <vector>
#include "kernels.h"

using namespace dat;

namespace {

enum OpKind { OP_CONV, OP_BIASACT, OP_BNACT, OP_MAXPOOL, OP_GAP, OP_FC };

struct Shape { int H, W, C; int64_t numel() const { return (int64_t)H * W * C; } };

struct Op {
  OpKind kind;
  int in = -1, out = -1, res = -1;
  int k = 0, stride = 1, pad = 0, relu = 0;
  int p0 = -1, p1 = -1;
  int cin_real = 0;             // conv: channels of the parameter tensor (input may be padded)
  bf16_t* w16 = nullptr;        // conv, bf16 model: [Cout][k][k][Cin_padded]
  bf16_t* w16T = nullptr;       //   and the flipped transpose used by backward-data
  float* mean = nullptr;        // BN batch statistics of the last forward
  uint8_t* argmax = nullptr;    // max-pool: window position of the maximum, per output element
  float* rstd = nullptr;
  uint8_t* mask = nullptr;      // BN with ReLU: one bit per output element (out > 0), read by the backward pass
  float* sums = nullptr;        // BN backward: [2][C] sums (sum dy, sum dy*xhat)
  float* bn_tab = nullptr;      //   and the per-channel constants of the input gradient (4*C floats)
  int dy_bn = -1;               // conv: BN op whose output gradient this conv's backward-data launch completes -- its epilogue can emit that BN's sums
  bool dy_bn_last_of_many = false;   //   ... as the last of several convolutions that read that output (accumulating launch)
  bool sparse_first = false;    // conv (1x1, stride 2): its backward-data pass runs first of two convolutions' and writes only the pixels it reads
  bool sums_ready = false;      // BN: sums and constants already produced by the convolution that wrote d(out)
  int pool = -1;                // BN + ReLU read only by a max-pool: that op (one fused forward pass; the backward pass gathers d(out))
  int pooled_by = -1;           // max-pool evaluated by the BN before it
  int res_bn = -1;              // BN with residual: the residual is the output of this BN op (projection shortcut), which
                                //   this op evaluates itself from that op's input -- forward and the shared backward sums
  int absorbed_by = -1;         // BN on a projection shortcut: the BN op that evaluates it (its output tensor is never stored)
  bool apply_fusable = false;   // BN: its input gradient has one consumer, a 1x1 convolution that can form it while loading
  bool apply_deferred = false;  //   ... and does so in the current backward sweep (the gradient tensor is not written)
  bool stats_from_conv = false; // BN forward: mean/rstd come from the producing convolution's epilogue
  int fwd_bn = -1;              // conv: BN op normalising this conv's output (statistics fused into the epilogue)
  bool blocked = false;         // conv: 7x7/2 stem run on the 2x2-pixel-block layout of the network input
  int res_grad_from = -1;       // conv: BN op whose residual gradient (d out .* ReLU mask) this conv's backward-data adds itself
  bool res_grad_deferred = false;   // BN with residual: that gradient is not written, the conv above picks it up
  float* dv = nullptr;          //   its weight gradient in the blocked layer's shape, [Cout][4][4][16]
};

struct PTensor { int64_t off, numel; int fan_in, kind; };

}  // namespace

struct dat_model {
  dat_arch arch; int dtype; int maxB; int H, W, classes;
  int normalize = 0; float mean[3] = {0, 0, 0}, inv_std[3] = {1, 1, 1};
  bool fuse_bn_apply = true;         // dat_model_set_option(DAT_OPT_FUSE_BN_INPUT_GRAD)
  bool fuse_bn_sums = true;          // dat_model_set_option(DAT_OPT_FUSE_BN_SUMS)
  bool fuse_pgd_grad = true;         // dat_model_set_option(DAT_OPT_FUSE_PGD_GRADIENT)
  bool sparse_shortcut_grad = true;  // dat_model_set_option(DAT_OPT_SPARSE_SHORTCUT_GRADIENT)
  bool overlap_wgrad = true;         // dat_model_set_option(DAT_OPT_OVERLAP_WEIGHT_GRADIENTS)
  // Weight gradients of the convolutions run on a stream of the model's own beside the caller's: nothing later in the
  // backward sweep reads them, and they are bound by the matrix units and the operand gather while the normalisation
  // passes between the backward-data launches are bound by HBM.  One event per convolution orders each launch after
  // its output gradient is complete; wg_join brings the side stream back before the sweep returns.
  hipStream_t wg_stream = nullptr;
  std::vector<hipEvent_t> wg_events;
  hipEvent_t wg_join = nullptr;
  int64_t bn_sums_max_bytes = (int64_t)1 << 62;   //   ... only for d(out) tensors up to this size
  bool fuse_pool = true;             // dat_model_set_option(DAT_OPT_FUSE_STEM_POOL): BN + ReLU + max-pool in one forward pass, pool gradient gathered by the BN backward pass
  bool absorb_shortcut_bn = true;    // dat_model_set_option(DAT_OPT_ABSORB_SHORTCUT_BN)
  bool grad_scales = true;           // dat_model_set_option(DAT_OPT_GRADIENT_SCALES)
  std::vector<Shape> tens;           // logical per-sample shapes (channels as stored)
  std::vector<char> is_f32;          // pooled features and logits stay fp32 in every model
  std::vector<Op> ops;
  std::vector<PTensor> ptab;
  int64_t d = 0;
  std::vector<void*> allocs;
  float* master = nullptr;           // fp32 parameters, the optimizer's copy
  float* compute = nullptr;          // parameters as the kernels read them (bf16 model: linear W rounded)
  int64_t* offsets_dev = nullptr;
  std::vector<void*> act, grad;
  std::vector<char> ghas;
  float* partial = nullptr; float* sums = nullptr;
  float* loss_n = nullptr; float* loss_steps = nullptr; int loss_cap = 0;
  float* gx = nullptr;
  void* wgrad_ws = nullptr; size_t wgrad_ws_bytes = 0;
  float* host_stage = nullptr;       // pinned staging for loss values
  float* fc_ws = nullptr;            // split-K scratch of the classifier GEMMs
  float* z_keep = nullptr;           // logits of the clean pass, kept while the perturbed pass runs (TRADES regulariser)
  float* z_keep2 = nullptr;          //   ... and of the perturbed pass, kept while the clean pass runs again
  uint32_t* gscale_ways = nullptr;   // per parameter tensor kAbsmaxWays slots raised by the kernels that write its gradient
  uint32_t* gscale = nullptr;        // per parameter tensor: bit pattern of max |gradient| written by the last dat_step (bf16 models)
  bool gscale_valid = false;         //   ... and whether that call produced all of them
  float* g_tmp = nullptr;            // second gradient vector of a two-pass objective (allocated on first use)
  // A second set of everything a forward pass leaves for its backward pass (activations, batch statistics, ReLU masks,
  // pool positions; allocated on first use): the KL objective keeps the clean pass there while the perturbed pass runs,
  // instead of running the clean pass a second time for its branch of the gradient (dat_model_set_option(
  // DAT_OPT_KEEP_BOTH_PASSES)).  swap_bank exchanges the two sets; gradients and scratch buffers are shared.
  struct PassBank { std::vector<void*> act; std::vector<float*> mean, rstd; std::vector<uint8_t*> mask, argmax; bool ready = false; } bank2;
  bool keep_both_passes = true;
  float* opt_m = nullptr; float* opt_v = nullptr; float* opt_u = nullptr; double* opt_norms = nullptr;   // LAMB state
  // optional per-launch timing (dat_profile_*): one event pair per launch group
  bool prof = false;
  struct ProfRec { int cls; hipEvent_t a, b; double work; int64_t nlaunch; };
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t take_event() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    return e;
  }

  int esize() const { return dtype == DAT_BF16 ? 2 : 4; }
  int add_tensor(Shape s, bool f32 = false) { tens.push_back(s); is_f32.push_back(f32 ? 1 : 0); return (int)tens.size() - 1; }
  int add_param(int64_t n, int fan_in, int kind) { ptab.push_back({d, n, fan_in, kind}); d += n; return (int)ptab.size() - 1; }

  int conv(int in, int cout, int k, int stride, int pad, int res = -1) {
    Shape s = tens[in];
    Op op; op.kind = OP_CONV; op.in = in; op.res = res; op.k = k; op.stride = stride; op.pad = pad;
    op.cin_real = (in == 0) ? 3 : s.C;
    op.out = add_tensor({(s.H + 2 * pad - k) / stride + 1, (s.W + 2 * pad - k) / stride + 1, cout});
    op.p0 = add_param((int64_t)cout * k * k * op.cin_real, op.cin_real * k * k, 0);
    ops.push_back(op); return op.out;
  }
  int biasact(int in, int relu) {
    Op op; op.kind = OP_BIASACT; op.in = in; op.relu = relu; op.out = add_tensor(tens[in]);
    op.p0 = add_param(tens[in].C, 0, 1);
    ops.push_back(op); return op.out;
  }
  // branch_final marks the last normalisation of a residual branch (tensor kind 6)
  int bnact(int in, int relu, int res = -1, bool branch_final = false) {
    Op op; op.kind = OP_BNACT; op.in = in; op.relu = relu; op.res = res; op.out = add_tensor(tens[in]);
    op.p0 = add_param(tens[in].C, 0, branch_final ? 6 : 2); op.p1 = add_param(tens[in].C, 0, 3);
    ops.push_back(op); return op.out;
  }
  int maxpool(int in) {
    Shape s = tens[in];
    Op op; op.kind = OP_MAXPOOL; op.in = in; op.k = 3; op.stride = 2; op.pad = 1;
    op.out = add_tensor({(s.H - 1) / 2 + 1, (s.W - 1) / 2 + 1, s.C});
    ops.push_back(op); return op.out;
  }
  int gap(int in) {
    Op op; op.kind = OP_GAP; op.in = in; op.out = add_tensor({1, 1, tens[in].C}, true);
    ops.push_back(op); return op.out;
  }
  int fc(int in, int nout) {
    Op op; op.kind = OP_FC; op.in = in; op.out = add_tensor({1, 1, nout}, true);
    op.p0 = add_param((int64_t)nout * tens[in].C, tens[in].C, 4); op.p1 = add_param(nout, 0, 5);
    ops.push_back(op); return op.out;
  }
};

namespace {

// ---- architectures (Sec. "Experiment setup" names them; shapes are the standard ones) --------
int basic_block(dat_model& m, int x, int cout, int stride) {
  const int cin = m.tens[x].C;
  int y = m.bnact(m.conv(x, cout, 3, stride, 1), 1);
  y = m.conv(y, cout, 3, 1, 1);
  int sc = x;
  if (stride != 1 || cin != cout) sc = m.bnact(m.conv(x, cout, 1, stride, 0), 0);
  return m.bnact(y, 1, sc, true);
}

int bottleneck(dat_model& m, int x, int width, int stride) {
  const int cin = m.tens[x].C, cout = 4 * width;
  int y = m.bnact(m.conv(x, width, 1, 1, 0), 1);
  y = m.bnact(m.conv(y, width, 3, stride, 1), 1);
  y = m.conv(y, cout, 1, 1, 0);
  int sc = x;
  if (stride != 1 || cin != cout) sc = m.bnact(m.conv(x, cout, 1, stride, 0), 0);
  return m.bnact(y, 1, sc, true);
}

int wide_block(dat_model& m, int x, int cout, int stride) {
  const int cin = m.tens[x].C;
  const int o = m.bnact(x, 1);
  const int y = m.bnact(m.conv(o, cout, 3, stride, 1), 1, -1, true);
  int sc = x;
  if (stride != 1 || cin != cout) sc = m.conv(o, cout, 1, stride, 0);
  return m.conv(y, cout, 3, 1, 1, sc);
}

bool build_graph(dat_model& m) {
  int t = 0;
  switch (m.arch) {
    case DAT_ARCH_TINYCNN:
      t = m.biasact(m.conv(t, 16, 3, 1, 1), 1);
      t = m.biasact(m.conv(t, 32, 3, 2, 1), 1);
      break;
    case DAT_ARCH_RESNET18_CIFAR: {
      t = m.bnact(m.conv(t, 64, 3, 1, 1), 1);
      const int widths[4] = {64, 128, 256, 512};
      for (int g = 0; g < 4; ++g)
        for (int b = 0; b < 2; ++b) t = basic_block(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
      break;
    }
    case DAT_ARCH_WRN34_10:
    case DAT_ARCH_WRN28_10: {
      const int per_group = m.arch == DAT_ARCH_WRN34_10 ? 5 : 4;   // (depth - 4) / 6
      t = m.conv(t, 16, 3, 1, 1);
      const int widths[3] = {160, 320, 640};
      for (int g = 0; g < 3; ++g)
        for (int b = 0; b < per_group; ++b) t = wide_block(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
      t = m.bnact(t, 1);
      break;
    }
    case DAT_ARCH_PREACT_RESNET18: {   // pre-activation basic block = wide block of widening factor 1
      t = m.conv(t, 64, 3, 1, 1);
      const int widths[4] = {64, 128, 256, 512};
      for (int g = 0; g < 4; ++g)
        for (int b = 0; b < 2; ++b) t = wide_block(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
      t = m.bnact(t, 1);
      break;
    }
    case DAT_ARCH_RESNET50: {
      t = m.maxpool(m.bnact(m.conv(t, 64, 7, 2, 3), 1));
      const int widths[4] = {64, 128, 256, 512}, depth[4] = {3, 4, 6, 3};
      for (int g = 0; g < 4; ++g)
        for (int b = 0; b < depth[g]; ++b) t = bottleneck(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
      break;
    }
    case DAT_ARCH_TESTNET:
      t = m.maxpool(m.bnact(m.conv(t, 8, 3, 1, 1), 1));
      t = basic_block(m, t, 8, 1);
      t = basic_block(m, t, 16, 2);
      t = bottleneck(m, t, 8, 2);
      t = wide_block(m, t, 16, 1);
      t = wide_block(m, t, 16, 1);
      t = m.bnact(t, 1);
      break;
    default:
      return false;
  }
  m.fc(m.gap(t), m.classes);
  return true;
}

// Fusion links between the ops of a bf16 model, recomputed from scratch (dat_model_create, and dat_model_set_option for
// the two switches that change them).  They select launches only: every tensor keeps its buffer either way.
void link_fusions(dat_model& m) {
  for (Op& op : m.ops) {
    op.dy_bn = -1; op.dy_bn_last_of_many = false; op.sparse_first = false; op.sums_ready = false; op.pool = -1; op.pooled_by = -1;
    op.res_bn = -1; op.absorbed_by = -1; op.apply_fusable = false; op.apply_deferred = false; op.stats_from_conv = false;
    op.fwd_bn = -1; op.res_grad_from = -1; op.res_grad_deferred = false;   // (op.blocked is fixed at creation: the weights are stored that way)
  }
  // which BN normalises a conv's output (its batch statistics come from the conv epilogue)
  if (m.dtype == DAT_BF16) {
    const int nt = (int)m.tens.size();
    std::vector<int> producer(nt, -1), first_consumer(nt, -1);
    for (int i = 0; i < (int)m.ops.size(); ++i) {
      producer[m.ops[i].out] = i;
      if (first_consumer[m.ops[i].in] < 0) first_consumer[m.ops[i].in] = i;
      if (m.ops[i].res >= 0 && first_consumer[m.ops[i].res] < 0) first_consumer[m.ops[i].res] = i;
    }
    for (int i = 0; i < (int)m.ops.size(); ++i) {
      Op& op = m.ops[i];
      if (op.kind == OP_BNACT && producer[op.in] >= 0 && m.ops[producer[op.in]].kind == OP_CONV &&
          m.ops[producer[op.in]].fwd_bn < 0) {
        m.ops[producer[op.in]].fwd_bn = i;
        op.stats_from_conv = true;
      }
    }
    // BN + ReLU whose only reader is a 3x3/2 max-pool (the ImageNet stem): one pass writes the pooled tensor, the
    // arg-max positions and the ReLU mask; the full-resolution activation and its gradient are never stored.
    for (int b = 0; b < (int)m.ops.size(); ++b) {
      Op& bn = m.ops[b];
      if (bn.kind != OP_BNACT || !bn.relu || bn.res >= 0) continue;
      int users = 0, pool = -1;
      for (int c = 0; c < (int)m.ops.size(); ++c) {
        users += (m.ops[c].in == bn.out) + (m.ops[c].res == bn.out);
        if (m.ops[c].in == bn.out && m.ops[c].kind == OP_MAXPOOL) pool = c;
      }
      if (users == 1 && pool > b) { bn.pool = pool; m.ops[pool].pooled_by = b; }
    }
    // Projection shortcuts: out = relu(bn(y) + bn_s(y_s)).  bn_s's output has no other reader, so the final BN
    // normalises y_s itself, and in the backward sweep d out .* mask is the output gradient of both normalisations:
    // one pass over it gives both pairs of sums.  Neither bn_s's output nor its gradient is ever stored.
    for (int b = 0; b < (int)m.ops.size() && m.absorb_shortcut_bn; ++b) {
      Op& bn = m.ops[b];
      if (bn.kind != OP_BNACT || bn.res < 0 || !bn.relu) continue;
      const int p = producer[bn.res];
      if (p < 0 || m.ops[p].kind != OP_BNACT || m.ops[p].relu || m.ops[p].res >= 0 || !m.ops[p].stats_from_conv || p > b) continue;
      int users = 0;
      for (const Op& o : m.ops) users += (o.in == bn.res) + (o.res == bn.res);
      if (users != 1) continue;
      bn.res_bn = p; m.ops[p].absorbed_by = b;
    }
    // Identity shortcuts: out = relu(bn(y) + r) sends d out .* mask to r, and the only other gradient of r comes
    // from the backward-data pass of the convolution that reads r (earlier in the graph, so later in the backward
    // sweep).  That pass can add d out .* mask in its epilogue: the residual gradient is never written on its own.
    for (int b = 0; b < (int)m.ops.size(); ++b) {
      Op& bn = m.ops[b];
      if (bn.kind != OP_BNACT || bn.res <= 0 || !bn.relu || bn.res_bn >= 0) continue;
      int users = 0, conv = -1;
      for (int c = 0; c < (int)m.ops.size(); ++c) {
        if (m.ops[c].in == bn.res) { ++users; if (m.ops[c].kind == OP_CONV && c < b) conv = c; }
        if (m.ops[c].res == bn.res) ++users;
      }
      if (users == 2 && conv >= 0 && m.ops[conv].res_grad_from < 0) { m.ops[conv].res_grad_from = b; bn.res_grad_deferred = true; }
    }
    // A BN whose input is read by nothing else and was produced by a 1x1 stride-1 convolution: in a sweep without
    // weight gradients that convolution's backward-data pass applies the BN input-gradient formula to d(out) while
    // loading it, so the BN's input gradient is never stored.
    for (int b = 0; b < (int)m.ops.size(); ++b) {
      Op& bn = m.ops[b];
      if (bn.kind != OP_BNACT || !bn.stats_from_conv) continue;
      const int c = producer[bn.in];
      int users = 0;
      for (const Op& o : m.ops) users += (o.in == bn.in) + (o.res == bn.in);
      const Op& cv = m.ops[c];
      if (users != 1 || cv.fwd_bn != b || cv.res >= 0 || cv.in == 0) continue;
      ConvGeom g;
      g.B = 1; g.H = m.tens[cv.in].H; g.W = m.tens[cv.in].W; g.Cin = m.tens[cv.in].C; g.Ho = m.tens[cv.out].H; g.Wo = m.tens[cv.out].W;
      g.Cout = m.tens[cv.out].C; g.k = cv.k; g.stride = cv.stride; g.pad = cv.pad;
      bn.apply_fusable = conv_mfma_bn_operand_ok(g);
    }
    // A BN whose output is read by one convolution only: d(out) is complete when that convolution's backward-data
    // pass has written it, so its epilogue can accumulate the BN's backward sums from the tile it is storing.
    for (int c = 0; c < (int)m.ops.size(); ++c) {
      Op& cv = m.ops[c];
      if (cv.kind != OP_CONV || cv.in <= 0 || producer[cv.in] < 0) continue;
      const Op& bn = m.ops[producer[cv.in]];
      if (bn.kind != OP_BNACT || bn.absorbed_by >= 0 || bn.pool >= 0) continue;
      if (bn.res_bn >= 0 && m.tens[cv.in].C < 128) continue;   // two BNs on one d(out): three sums, wide tiles only
      int users = 0, conv_users = 0, first_user = -1;
      for (int o = 0; o < (int)m.ops.size(); ++o) {
        const int u = (m.ops[o].in == cv.in) + (m.ops[o].res == cv.in);
        users += u;
        if (u && first_user < 0) first_user = o;
        if (m.ops[o].in == cv.in && m.ops[o].kind == OP_CONV) ++conv_users;
      }
      // one reader; or two when the other one is an identity shortcut whose gradient this convolution's epilogue adds
      // itself; or several convolutions, of which this is the first in the graph and so the last to add its part
      if (users == 1 || (users == 2 && cv.res_grad_from >= 0)) cv.dy_bn = producer[cv.in];
      else if (conv_users == users && first_user == c) { cv.dy_bn = producer[cv.in]; cv.dy_bn_last_of_many = true; }
    }
    // A strided 1x1 projection whose input is read by exactly one other convolution, earlier in the graph: in the
    // backward sweep the projection writes its input gradient first, at the quarter of the pixels it reads, and the
    // other convolution adds to it knowing that the rest is zero (three quarters of the tensor neither written nor read).
    for (int c = 0; c < (int)m.ops.size(); ++c) {
      Op& cv = m.ops[c];
      if (cv.kind != OP_CONV || cv.in <= 0 || cv.blocked) continue;
      ConvGeom g; g.k = cv.k; g.stride = cv.stride; g.pad = cv.pad;
      if (!conv_mfma_sparse_writer_ok(g) || m.tens[cv.in].H % 2 != 0 || m.tens[cv.in].W % 2 != 0) continue;
      int users = 0, conv_users = 0, first_user = -1;
      for (int o = 0; o < (int)m.ops.size(); ++o) {
        const int u = (m.ops[o].in == cv.in) + (m.ops[o].res == cv.in);
        users += u;
        if (u && first_user < 0) first_user = o;
        if (m.ops[o].in == cv.in && m.ops[o].kind == OP_CONV) ++conv_users;
      }
      if (users == 2 && conv_users == 2 && first_user != c && m.ops[first_user].res_grad_from < 0 && (m.ops[first_user].stride == 1 || m.ops[first_user].stride == 2))
        cv.sparse_first = true;
    }
  }
}

// the ImageNet stem runs on 2x2 pixel blocks of the network input (tensor 0 is stored blocked)
void decide_blocked_stem(dat_model& m) {
  if (m.dtype != DAT_BF16) return;
  Op& first = m.ops[0];
  if (first.kind == OP_CONV && first.in == 0 && first.res < 0) {
    ConvGeom g;
    g.B = 1; g.H = m.tens[0].H; g.W = m.tens[0].W; g.Cin = m.tens[0].C; g.Ho = m.tens[first.out].H; g.Wo = m.tens[first.out].W;
    g.Cout = m.tens[first.out].C; g.k = first.k; g.stride = first.stride; g.pad = first.pad;
    bool only_consumer = true;
    for (size_t i = 1; i < m.ops.size(); ++i) if (m.ops[i].in == 0 || m.ops[i].res == 0) only_consumer = false;
    first.blocked = only_consumer && conv_mfma_stem_blocked_ok(g, first.cin_real);
  }
}

template <typename T>
dat_status dev_alloc(dat_model& m, T** p, size_t bytes) {
  void* q = nullptr;
  if (bytes == 0) bytes = 16;
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); return DAT_ERR_NOMEM; }
  m.allocs.push_back(q);
  *p = (T*)q;
  return DAT_OK;
}

#define DAT_TRY(expr) do { dat_status s_ = (expr); if (s_ != DAT_OK) return s_; } while (0)

// Launch group `expr` of class `cls` doing `work` algorithmic FLOPs or bytes; timed when profiling.
// A group counts as one launch unless it ran MFMA convolution kernels, which are counted one by one
// (a stride-2 backward-data pass is four of them).
#define DAT_PROF(m, cls, work, st, expr)                                            \
  do {                                                                              \
    if ((m).prof) {                                                                 \
      dat_model::ProfRec r_{(cls), (m).take_event(), (m).take_event(), (double)(work), 1}; \
      if (r_.a && r_.b) {                                                           \
        const int64_t n0_ = conv_mfma_launch_count();                               \
        DAT_HIP(hipEventRecord(r_.a, (st)));                                        \
        DAT_TRY(expr);                                                              \
        DAT_HIP(hipEventRecord(r_.b, (st)));                                        \
        if (conv_mfma_launch_count() > n0_) r_.nlaunch = conv_mfma_launch_count() - n0_; \
        (m).recs.push_back(r_);                                                     \
      } else { DAT_TRY(expr); }                                                     \
    } else { DAT_TRY(expr); }                                                       \
  } while (0)

double conv_flops(const ConvGeom& g, int cin_real) {
  return 2.0 * g.B * g.Ho * g.Wo * (double)g.Cout * g.k * g.k * cin_real;
}

ConvGeom geom_of(const dat_model& m, const Op& op, int B) {
  const Shape si = m.tens[op.in], so = m.tens[op.out];
  ConvGeom g;
  g.B = B; g.H = si.H; g.W = si.W; g.Cin = si.C; g.Ho = so.H; g.Wo = so.W; g.Cout = so.C;
  g.k = op.k; g.stride = op.stride; g.pad = op.pad;
  return g;
}

dat_status allocate(dat_model& m) {
  const int es = m.esize();
  DAT_TRY(dev_alloc(m, &m.master, (size_t)m.d * 4));
  if (m.dtype == DAT_BF16) DAT_TRY(dev_alloc(m, &m.compute, (size_t)m.d * 4)); else m.compute = m.master;
  DAT_TRY(dev_alloc(m, &m.offsets_dev, (m.ptab.size() + 1) * 8));
  std::vector<int64_t> off(m.ptab.size() + 1);
  for (size_t i = 0; i < m.ptab.size(); ++i) off[i] = m.ptab[i].off;
  off[m.ptab.size()] = m.d;
  DAT_HIP(hipMemcpy(m.offsets_dev, off.data(), off.size() * 8, hipMemcpyHostToDevice));
  m.act.assign(m.tens.size(), nullptr); m.grad.assign(m.tens.size(), nullptr); m.ghas.assign(m.tens.size(), 0);
  int cmax = 8;
  for (size_t t = 0; t < m.tens.size(); ++t) {
    const size_t bytes = (size_t)m.maxB * m.tens[t].numel() * (m.is_f32[t] ? 4 : es);
    DAT_TRY(dev_alloc(m, &m.act[t], bytes));
    DAT_TRY(dev_alloc(m, &m.grad[t], bytes));
    cmax = m.tens[t].C > cmax ? m.tens[t].C : cmax;
  }
  // the padded channels of a bf16 input tensor are written by the input kernels on every call
  size_t ws = 0;
  for (Op& op : m.ops) {
    if (op.kind == OP_BNACT) {
      DAT_TRY(dev_alloc(m, &op.mean, (size_t)m.tens[op.in].C * 4));
      DAT_TRY(dev_alloc(m, &op.rstd, (size_t)m.tens[op.in].C * 4));
      DAT_TRY(dev_alloc(m, &op.sums, (size_t)m.tens[op.in].C * 8));
      DAT_TRY(dev_alloc(m, &op.bn_tab, (size_t)m.tens[op.in].C * 16));
      if (op.relu) DAT_TRY(dev_alloc(m, &op.mask, (size_t)m.maxB * m.tens[op.in].numel() / 8));
    }
    if (op.kind == OP_MAXPOOL) DAT_TRY(dev_alloc(m, &op.argmax, (size_t)m.maxB * m.tens[op.out].numel()));
    if (op.kind == OP_CONV && m.dtype == DAT_BF16) {
      const size_t n = op.blocked ? (size_t)m.tens[op.out].C * 16 * 16 : (size_t)m.tens[op.out].C * op.k * op.k * m.tens[op.in].C;   // blocked: [Cout][4][4][16]
      DAT_TRY(dev_alloc(m, &op.w16, n * 2));
      DAT_TRY(dev_alloc(m, &op.w16T, n * 2));
      if (op.blocked) DAT_TRY(dev_alloc(m, &op.dv, n * 4));
      const ConvGeom gmax = geom_of(m, op, m.maxB);
      const size_t need = conv_mfma_wgrad_workspace(op.blocked ? conv_mfma_stem_blocked_geom(gmax) : gmax);
      ws = need > ws ? need : ws;
    }
  }
  m.wgrad_ws_bytes = ws;
  if (ws) DAT_TRY(dev_alloc(m, &m.wgrad_ws, ws));
  size_t partial_floats = bn_partial_floats(0, cmax);
  for (const Op& op : m.ops) {
    if (op.kind != OP_CONV || m.dtype != DAT_BF16) continue;
    const Shape si = m.tens[op.in], so = m.tens[op.out];
    const int sf = conv_stat_slabs((int64_t)m.maxB * so.H * so.W, 1), sb = conv_stat_slabs((int64_t)m.maxB * si.H * si.W, op.stride);
    const size_t need_f = (size_t)sf * 2 * so.C + fold_floats(sf, so.C), need_b = (size_t)sb * 3 * si.C + fold_floats(sb, si.C);
    partial_floats = std::max(partial_floats, std::max(need_f, need_b));
  }
  DAT_TRY(dev_alloc(m, &m.partial, partial_floats * 4));
  if (m.dtype == DAT_BF16) {   // default priority: work on streams of different priorities must not be mixed
    DAT_HIP(hipStreamCreateWithFlags(&m.wg_stream, hipStreamNonBlocking));
    DAT_HIP(hipEventCreateWithFlags(&m.wg_join, hipEventDisableTiming));
    for (const Op& op : m.ops)
      if (op.kind == OP_CONV) { hipEvent_t e; DAT_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming)); m.wg_events.push_back(e); }
  }
  DAT_TRY(dev_alloc(m, &m.gscale, m.ptab.size() * 4));
  DAT_TRY(dev_alloc(m, &m.gscale_ways, m.ptab.size() * kAbsmaxWays * kAbsmaxStride * 4));
  DAT_TRY(dev_alloc(m, &m.sums, (size_t)2 * cmax * 4));
  DAT_TRY(dev_alloc(m, &m.loss_n, (size_t)m.maxB * 4));
  m.loss_cap = 1024;
  DAT_TRY(dev_alloc(m, &m.loss_steps, (size_t)m.loss_cap * 4));
  DAT_TRY(dev_alloc(m, &m.gx, (size_t)m.maxB * m.H * m.W * 3 * 4));
  DAT_TRY(dev_alloc(m, &m.z_keep, (size_t)m.maxB * m.classes * 4));
  { const Op& fc = m.ops.back(); DAT_TRY(dev_alloc(m, &m.fc_ws, fc_workspace_floats(m.maxB, m.tens[fc.in].C, m.tens[fc.out].C) * 4)); }
  DAT_TRY(dev_alloc(m, &m.z_keep2, (size_t)m.maxB * m.classes * 4));
  if (hipHostMalloc((void**)&m.host_stage, (size_t)m.loss_cap * 4, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    return DAT_ERR_NOMEM;
  }
  DAT_TRY(launch_fill_zero(m.master, (size_t)m.d * 4, nullptr));
  if (m.compute != m.master) DAT_TRY(launch_fill_zero(m.compute, (size_t)m.d * 4, nullptr));
  DAT_HIP(hipDeviceSynchronize());
  return DAT_OK;
}

// Rebuilds what the kernels read from the fp32 master copy.
dat_status refresh_compute(dat_model& m, hipStream_t st) {
  if (m.dtype != DAT_BF16) return DAT_OK;
  DAT_HIP(hipMemcpyAsync(m.compute, m.master, (size_t)m.d * 4, hipMemcpyDeviceToDevice, st));
  for (Op& op : m.ops) {
    if (op.kind == OP_CONV && op.blocked)
      DAT_TRY(launch_stem_weight_transform(m.master + m.ptab[op.p0].off, op.w16, op.w16T, m.tens[op.out].C, op.cin_real, st));
    else if (op.kind == OP_CONV)
      DAT_TRY(launch_weight_transform(m.master + m.ptab[op.p0].off, op.w16, op.w16T, m.tens[op.out].C, op.k, op.cin_real,
                                      m.tens[op.in].C, op.stride, op.pad, st));
    if (op.kind == OP_FC)
      DAT_TRY(launch_round_bf16_values(m.master + m.ptab[op.p0].off, m.compute + m.ptab[op.p0].off, m.ptab[op.p0].numel, st));
  }
  return DAT_OK;
}

NetInputDesc input_desc(const dat_model& m) {
  NetInputDesc d;
  d.ptr = m.act[0]; d.bf16 = m.dtype == DAT_BF16; d.normalize = m.normalize;
  for (int c = 0; c < 3; ++c) { d.mean[c] = m.mean[c]; d.inv_std[c] = m.inv_std[c]; }
  const bool blocked = m.ops[0].kind == OP_CONV && m.ops[0].blocked;
  d.block_h = blocked ? m.H : 0; d.block_w = blocked ? m.W : 0;
  return d;
}

dat_status bn_forward_pair(dat_model& m, Op& op, int64_t rows, int C, hipStream_t st) {
  if (!op.stats_from_conv) DAT_TRY(bn_stats(m.act[op.in], m.dtype, rows, C, m.partial, op.mean, op.rstd, st));
  if (op.pool >= 0 && m.fuse_pool) {
    const Op& pl = m.ops[op.pool];
    const Shape si = m.tens[op.in], so = m.tens[pl.out];
    return bnact_pool_forward(m.act[op.in], m.act[pl.out], pl.argmax, op.mask, m.dtype, (int)(rows / ((int64_t)si.H * si.W)), si.H, si.W, C,
                              so.H, so.W, op.mean, op.rstd, m.compute + m.ptab[op.p0].off, m.compute + m.ptab[op.p1].off, st);
  }
  if (op.res_bn >= 0) {   // the residual is normalised on the fly from the shortcut BN's input
    const Op& sb = m.ops[op.res_bn];
    const BnParams rp{sb.mean, sb.rstd, m.compute + m.ptab[sb.p0].off, m.compute + m.ptab[sb.p1].off};
    return bnact_forward(m.act[op.in], m.act[sb.in], m.act[op.out], op.mask, m.dtype, rows, C, op.mean, op.rstd,
                         m.compute + m.ptab[op.p0].off, m.compute + m.ptab[op.p1].off, op.relu, st, &rp);
  }
  return bnact_forward(m.act[op.in], op.res >= 0 ? m.act[op.res] : nullptr, m.act[op.out], op.mask, m.dtype, rows, C, op.mean,
                       op.rstd, m.compute + m.ptab[op.p0].off, m.compute + m.ptab[op.p1].off, op.relu, st);
}

dat_status forward(dat_model& m, int B, hipStream_t st) {
  const int dt = m.dtype;
  for (Op& op : m.ops) {
    const Shape si = m.tens[op.in], so = m.tens[op.out];
    const int64_t rows_in = (int64_t)B * si.H * si.W;
    switch (op.kind) {
      case OP_CONV: {
        const ConvGeom g = geom_of(m, op, B);
        const void* res = op.res >= 0 ? m.act[op.res] : nullptr;
        if (dt == DAT_BF16) {
          ConvStats cs{};
          cs.mode = op.fwd_bn >= 0 ? 1 : 0; cs.partial = m.partial;
          if (op.blocked) DAT_PROF(m, DAT_PROF_CONV_FWD, conv_flops(g, op.cin_real), st, conv_mfma_stem_forward((const bf16_t*)m.act[op.in], op.w16, (bf16_t*)m.act[op.out], g, &cs, st));
          else DAT_PROF(m, DAT_PROF_CONV_FWD, conv_flops(g, op.cin_real), st, conv_mfma_forward((const bf16_t*)m.act[op.in], op.w16, (const bf16_t*)res, (bf16_t*)m.act[op.out], g, &cs, st));
          if (cs.mode) {   // batch statistics of the normalisation that follows, from the epilogue's partial sums
            Op& bn = m.ops[op.fwd_bn];
            DAT_PROF(m, DAT_PROF_BN, 0.0, st, bn_finalize_slabs(m.partial, cs.nslabs, so.C, (int64_t)B * so.H * so.W, 1, bn.mean, bn.rstd, nullptr, nullptr, 1.0f, st));
          }
        }
        else DAT_PROF(m, DAT_PROF_CONV_FWD, conv_flops(g, op.cin_real), st, conv_direct_forward((const float*)m.act[op.in], m.compute + m.ptab[op.p0].off, (const float*)res, (float*)m.act[op.out], g, st));
        break;
      }
      case OP_BIASACT:
        DAT_TRY(biasact_forward(m.act[op.in], m.act[op.out], dt, rows_in, si.C, m.compute + m.ptab[op.p0].off, op.relu, st));
        break;
      case OP_BNACT:
        if (op.absorbed_by >= 0) break;   // statistics came from the convolution; the absorbing BN does the rest
        // algorithmic bytes: read x twice (statistics, apply), read res, write out
        DAT_PROF(m, DAT_PROF_BN, (double)rows_in * si.C * m.esize() * (3 - (int)op.stats_from_conv + (op.res >= 0)), st,
                 bn_forward_pair(m, op, rows_in, si.C, st));
        break;
      case OP_MAXPOOL:
        if (op.pooled_by >= 0 && m.fuse_pool) break;
        DAT_TRY(maxpool_forward(m.act[op.in], m.act[op.out], op.argmax, dt, B, si.H, si.W, si.C, so.H, so.W, st));
        break;
      case OP_GAP:
        DAT_TRY(gap_forward(m.act[op.in], (float*)m.act[op.out], dt, B, si.H * si.W, si.C, st));
        break;
      case OP_FC:
        DAT_TRY(fc_forward((const float*)m.act[op.in], m.compute + m.ptab[op.p0].off, m.compute + m.ptab[op.p1].off,
                           (float*)m.act[op.out], B, si.C, so.C, m.fc_ws, st));
        break;
    }
  }
  return DAT_OK;
}

// Loss and logit gradient; `loss_slot` indexes m.loss_steps.
dat_status loss_grad(dat_model& m, const int32_t* y, int B, float gscale, int loss_slot, hipStream_t st) {
  const int t = m.ops.back().out;
  DAT_TRY(ce_forward_backward((const float*)m.act[t], y, (float*)m.grad[t], m.loss_n, m.loss_steps + loss_slot, B, m.classes, gscale, st));
  std::fill(m.ghas.begin(), m.ghas.end(), 0);
  m.ghas[t] = 1;
  return DAT_OK;
}

// grads == nullptr: backward to the input only (attack); otherwise also parameter gradients.
dat_status backward(dat_model& m, int B, float* grads, bool need_input_grad, hipStream_t st) {
  const int dt = m.dtype;
  // (per-launch timing keeps everything on one stream: its event pairs bracket launches on `st`)
  const bool side = grads && dt == DAT_BF16 && m.overlap_wgrad && m.wg_stream && !m.prof;
  size_t wg_used = 0;
  // Every kernel that writes a parameter gradient also raises that tensor's abs-max slot (the quantizer's scale):
  // bf16 models whose ops all have such writers.  The slots start at zero.
  bool fused_scales = grads && dt == DAT_BF16 && m.grad_scales;
  for (const Op& o : m.ops) if (o.kind == OP_BIASACT) fused_scales = false;
  m.gscale_valid = false;
  if (fused_scales) DAT_TRY(launch_fill_zero(m.gscale_ways, m.ptab.size() * kAbsmaxWays * kAbsmaxStride * 4, st));
  auto slot = [&](int p) -> uint32_t* { return fused_scales && p >= 0 ? m.gscale_ways + (size_t)p * kAbsmaxWays * kAbsmaxStride : nullptr; };
  for (int i = (int)m.ops.size() - 1; i >= 0; --i) {
    Op& op = m.ops[i];
    const Shape si = m.tens[op.in], so = m.tens[op.out];
    const int64_t rows_in = (int64_t)B * si.H * si.W, rows_out = (int64_t)B * so.H * so.W;
    float* g0 = grads && op.p0 >= 0 ? grads + m.ptab[op.p0].off : nullptr;
    float* g1 = grads && op.p1 >= 0 ? grads + m.ptab[op.p1].off : nullptr;
    switch (op.kind) {
      case OP_CONV: {
        const ConvGeom g = geom_of(m, op, B);
        if (op.res >= 0) {   // out = conv + res: the residual receives d out unchanged
          DAT_TRY(biasact_backward(nullptr, m.grad[op.out], m.grad[op.res], m.ghas[op.res], dt, rows_out, so.C, 0, nullptr, nullptr, 1.0f, st));
          m.ghas[op.res] = 1;
        }
        if (g0) {
          hipStream_t wst = st;
          if (side && wg_used < m.wg_events.size()) {   // d(out) of this layer is complete at this point of `st`
            hipEvent_t e = m.wg_events[wg_used++];
            DAT_HIP(hipEventRecord(e, st));
            DAT_HIP(hipStreamWaitEvent(m.wg_stream, e, 0));
            wst = m.wg_stream;
          }
          if (dt == DAT_BF16 && op.blocked) DAT_PROF(m, DAT_PROF_CONV_WGRAD, conv_flops(g, op.cin_real), wst, conv_mfma_stem_backward_weight((const bf16_t*)m.act[op.in], (const bf16_t*)m.grad[op.out], g0, op.dv, op.cin_real, g, 1.0f, m.wgrad_ws, wst, slot(op.p0)));
          else if (dt == DAT_BF16) DAT_PROF(m, DAT_PROF_CONV_WGRAD, conv_flops(g, op.cin_real), wst, conv_mfma_backward_weight((const bf16_t*)m.act[op.in], (const bf16_t*)m.grad[op.out], g0, op.cin_real, g, 1.0f, m.wgrad_ws, wst, slot(op.p0)));
          else DAT_PROF(m, DAT_PROF_CONV_WGRAD, conv_flops(g, op.cin_real), st, conv_direct_backward_weight((const float*)m.act[op.in], (const float*)m.grad[op.out], g0, g, 1.0f, st));
        }
        if (op.in != 0 || need_input_grad) {
          // sums of the BN whose output gradient this pass completes (nothing else has written it, nothing else will)
          ConvStats bs{}; ConvStats* bsp = nullptr;
          bool sparse_written = false;
          if (dt == DAT_BF16 && !op.blocked && op.dy_bn >= 0 && m.fuse_bn_sums && (bool)m.ghas[op.in] == op.dy_bn_last_of_many &&
              (int64_t)si.H * si.W * si.C * B * 2 <= m.bn_sums_max_bytes) {
            const Op& bn = m.ops[op.dy_bn];
            bs.mode = 2; bs.partial = m.partial; bs.bn_x = (const bf16_t*)m.act[bn.in]; bs.bn_mask = bn.relu ? bn.mask : nullptr;
            bs.bn_mean = bn.mean; bs.bn_rstd = bn.rstd;
            if (bn.res_bn >= 0) {   // the BN on the projection shortcut sees the same d(out)
              const Op& sb = m.ops[bn.res_bn];
              bs.mode = 3; bs.bn_x2 = (const bf16_t*)m.act[sb.in]; bs.bn_mean2 = sb.mean; bs.bn_rstd2 = sb.rstd;
            }
            bsp = &bs;
          }
          if (dt == DAT_BF16 && op.blocked) DAT_PROF(m, DAT_PROF_CONV_BWD_DATA, conv_flops(g, op.cin_real), st, conv_mfma_stem_backward_data((const bf16_t*)m.grad[op.out], op.w16T, (bf16_t*)m.grad[op.in], g, m.ghas[op.in], st));
          else if (dt == DAT_BF16 && op.fwd_bn >= 0 && m.ops[op.fwd_bn].apply_deferred) {
            Op& bn = m.ops[op.fwd_bn];
            bn.apply_deferred = false;
            const Op& top = bn.absorbed_by >= 0 ? m.ops[bn.absorbed_by] : bn;   // whose d(out) and mask this BN differentiates
            const BnOperand bo{(const bf16_t*)m.act[bn.in], top.relu ? top.mask : nullptr, bn.bn_tab};
            const bool rg = op.res_grad_from >= 0;
            if (rg && m.ghas[op.in]) return DAT_ERR_UNSUPPORTED;
            DAT_PROF(m, DAT_PROF_CONV_BWD_DATA_BN, conv_flops(g, op.cin_real), st,
                     conv_mfma_backward_data((const bf16_t*)m.grad[top.out], op.w16T, (bf16_t*)m.grad[op.in], g, rg ? false : (bool)m.ghas[op.in], bsp, st,
                                             rg ? (const bf16_t*)m.grad[m.ops[op.res_grad_from].out] : nullptr,
                                             rg ? m.ops[op.res_grad_from].mask : nullptr, &bo, (!rg && m.ghas[op.in] == 2) ? 2 : 0));
          }
          else if (dt == DAT_BF16 && op.res_grad_from >= 0) {
            if (m.ghas[op.in]) return DAT_ERR_UNSUPPORTED;   // by construction nothing else has written this gradient yet
            const Op& bn = m.ops[op.res_grad_from];
            DAT_PROF(m, DAT_PROF_CONV_BWD_DATA, conv_flops(g, op.cin_real), st, conv_mfma_backward_data((const bf16_t*)m.grad[op.out], op.w16T, (bf16_t*)m.grad[op.in], g, false, bsp, st, (const bf16_t*)m.grad[bn.out], bn.mask));
          }
          else if (dt == DAT_BF16) {
            // (see Op::sparse_first: the first of the two passes writes a quarter of the pixels, the second knows)
            const bool first_sparse = op.sparse_first && !m.ghas[op.in] && !bsp && m.sparse_shortcut_grad;
            const int sparse = first_sparse ? 1 : m.ghas[op.in] == 2 ? 2 : 0;
            DAT_PROF(m, DAT_PROF_CONV_BWD_DATA, conv_flops(g, op.cin_real), st, conv_mfma_backward_data((const bf16_t*)m.grad[op.out], op.w16T, (bf16_t*)m.grad[op.in], g, m.ghas[op.in], bsp, st, nullptr, nullptr, nullptr, sparse));
            if (first_sparse) sparse_written = true;
          }
          else DAT_PROF(m, DAT_PROF_CONV_BWD_DATA, conv_flops(g, op.cin_real), st, conv_direct_backward_data((const float*)m.grad[op.out], m.compute + m.ptab[op.p0].off, (float*)m.grad[op.in], g, m.ghas[op.in], st));
          m.ghas[op.in] = sparse_written ? 2 : 1;
          if (bsp) {   // finish that BN's sums, parameter gradients and input-gradient constants now
            Op& bn = m.ops[op.dy_bn];
            float* bg0 = grads ? grads + m.ptab[bn.p0].off : nullptr;
            float* bg1 = grads ? grads + m.ptab[bn.p1].off : nullptr;
            const int nsum = bs.mode == 3 ? 3 : 2;
            DAT_PROF(m, DAT_PROF_BN, 0.0, st, bn_finalize_slabs(m.partial, bs.nslabs, si.C, rows_in, 2, bn.sums, bn.sums + si.C, bg1, bg0, 1.0f, st,
                                                                 m.compute + m.ptab[bn.p0].off, bn.mean, bn.rstd, bn.bn_tab, nsum, 1, true,
                                                                 ParamAbsmax{slot(bn.p1), slot(bn.p0)}));
            if (bs.mode == 3) {
              Op& sb = m.ops[bn.res_bn];
              float* sg0 = grads ? grads + m.ptab[sb.p0].off : nullptr;
              float* sg1 = grads ? grads + m.ptab[sb.p1].off : nullptr;
              DAT_PROF(m, DAT_PROF_BN, 0.0, st, bn_finalize_slabs(m.partial, bs.nslabs, si.C, rows_in, 2, sb.sums, sb.sums + si.C, sg1, sg0, 1.0f, st,
                                                                   m.compute + m.ptab[sb.p0].off, sb.mean, sb.rstd, sb.bn_tab, 3, 2, false,
                                                                   ParamAbsmax{slot(sb.p1), slot(sb.p0)}));
            }
            bn.sums_ready = true;
          }
        }
        break;
      }
      case OP_BIASACT:
        DAT_TRY(biasact_backward(m.act[op.out], m.grad[op.out], m.grad[op.in], m.ghas[op.in], dt, rows_in, si.C, op.relu, m.partial, g0, 1.0f, st));
        m.ghas[op.in] = 1;
        break;
      case OP_BNACT: {
        // d(out) and ReLU mask this normalisation differentiates: its own, or (shortcut BN evaluated by the final BN
        // of the branch) those of that BN, whose backward step also produced this op's sums and constants
        const bool absorbed = op.absorbed_by >= 0;
        const Op& top = absorbed ? m.ops[op.absorbed_by] : op;
        const bool deferred = op.res_grad_deferred && dt == DAT_BF16;
        const bool writes_dres = op.res >= 0 && !deferred && op.res_bn < 0;
        void* dres = writes_dres ? m.grad[op.res] : nullptr;
        const bool dres_acc = writes_dres && m.ghas[op.res];
        // no weight gradients wanted, nothing stored in d(in) yet, no residual gradient to write: leave the input
        // gradient to the convolution below
        op.apply_deferred = op.apply_fusable && m.fuse_bn_apply && !grads && dt == DAT_BF16 && !m.ghas[op.in] && !dres;
        if (op.pool >= 0) {   // BN + ReLU feeding a max-pool: both halves on 2x2 pixel blocks
          const Op& pl = m.ops[op.pool];
          PoolGrad pg{pl.argmax, m.grad[pl.out], B, si.H, si.W, m.tens[pl.out].H, m.tens[pl.out].W, m.fuse_pool ? 1 : 0};
          DAT_PROF(m, DAT_PROF_BN, (double)rows_in * si.C * m.esize() * 4, st,
                   bn_pool_backward(m.act[op.in], op.mask, m.grad[op.out], m.grad[op.in], m.ghas[op.in], false, dt, si.C, op.mean, op.rstd,
                                    m.compute + m.ptab[op.p0].off, m.partial, op.sums, op.bn_tab, g0, g1, 1.0f, pg, st,
                                    ParamAbsmax{slot(op.p1), slot(op.p0)}));
          m.ghas[op.in] = 1;
          break;
        }
        const bool have_sums = op.sums_ready;
        op.sums_ready = false;
        if (!absorbed && !have_sums) {
          BnSecond sec{}; const BnSecond* second = nullptr;
          if (op.res_bn >= 0) {
            Op& sb = m.ops[op.res_bn];
            sec.x = m.act[sb.in]; sec.mean = sb.mean; sec.rstd = sb.rstd; sec.gamma = m.compute + m.ptab[sb.p0].off;
            sec.sums = sb.sums; sec.tab = sb.bn_tab;
            sec.dgamma = grads ? grads + m.ptab[sb.p0].off : nullptr; sec.dbeta = grads ? grads + m.ptab[sb.p1].off : nullptr;
            sec.am = ParamAbsmax{slot(sb.p1), slot(sb.p0)};
            second = &sec;
          }
          // algorithmic bytes: read x, dout (and mask) once for the sums ...
          DAT_PROF(m, DAT_PROF_BN, (double)rows_in * si.C * m.esize() * (2 + (second ? 1 : 0)), st,
                   bn_backward_reduce(m.act[op.in], m.act[op.out], op.mask, m.grad[op.out], dt, rows_in, si.C, op.mean, op.rstd,
                                      m.compute + m.ptab[op.p0].off, op.relu, m.partial, op.sums, op.bn_tab, g0, g1, 1.0f, st, second,
                                      ParamAbsmax{slot(op.p1), slot(op.p0)}));
        }
        if (!op.apply_deferred) {
          // ... and once more, plus writing dx (and dres), for the input gradient
          DAT_PROF(m, DAT_PROF_BN, (double)rows_in * si.C * m.esize() * (3 + (dres ? 1 : 0)), st,
                   bn_backward_apply(m.act[op.in], m.act[top.out], top.mask, m.grad[top.out], m.grad[op.in], m.ghas[op.in], dres, dres_acc, dt,
                                     rows_in, si.C, op.bn_tab, top.relu, st));
          m.ghas[op.in] = 1;
        }
        if (writes_dres) m.ghas[op.res] = 1;
        break;
      }
      case OP_MAXPOOL:
        if (op.pooled_by >= 0 && m.fuse_pool) break;   // the BN above gathers its d(out) from d(pooled)
        DAT_TRY(maxpool_backward(op.argmax, m.grad[op.out], m.grad[op.in], m.ghas[op.in], dt, B, si.H, si.W, si.C, so.H, so.W, st));
        m.ghas[op.in] = 1;
        break;
      case OP_GAP:
        DAT_TRY(gap_backward((const float*)m.grad[op.out], m.grad[op.in], m.ghas[op.in], dt, B, si.H * si.W, si.C, st));
        m.ghas[op.in] = 1;
        break;
      case OP_FC:
        DAT_TRY(fc_backward((const float*)m.act[op.in], m.compute + m.ptab[op.p0].off, (const float*)m.grad[op.out],
                            (float*)m.grad[op.in], g0, g1, B, si.C, so.C, 1.0f, m.fc_ws, st, ParamAbsmax{slot(op.p0), slot(op.p1)}));
        m.ghas[op.in] = 1;
        break;
    }
  }
  if (wg_used) {   // whatever follows on `st` (the caller's reads of `grads`, the next sweep's writes) waits for the side stream
    DAT_HIP(hipEventRecord(m.wg_join, m.wg_stream));
    DAT_HIP(hipStreamWaitEvent(st, m.wg_join, 0));
  }
  if (fused_scales) DAT_TRY(launch_absmax_fold(m.gscale_ways, (int)m.ptab.size(), m.gscale, st));
  m.gscale_valid = fused_scales;
  return DAT_OK;
}

dat_status pixel_grad(dat_model& m, int B, float* gx, hipStream_t st) {
  const bool n = m.normalize;
  const bool blocked = m.ops[0].kind == OP_CONV && m.ops[0].blocked;
  return launch_input_grad(m.grad[0], m.dtype, blocked ? 4 : m.tens[0].C, (int64_t)B * m.H * m.W, n ? m.inv_std[0] : 1.0f,
                           n ? m.inv_std[1] : 1.0f, n ? m.inv_std[2] : 1.0f, gx, blocked ? m.H : 0, blocked ? m.W : 0, st);
}

// One projected sign step from the input gradient the backward pass has just left in m.grad[0].  bf16 models read
// that tensor directly (only the sign of the gradient enters the step, and the normalisation scale 1/std is
// positive); fp32 models, or DAT_OPT_FUSE_PGD_GRADIENT = 0, go through the fp32 pixel gradient.
dat_status pgd_step(dat_model& m, const float* x, float* delta, int B, float eps, float alpha, const NetInputDesc& in, hipStream_t st) {
  const int64_t npix = (int64_t)B * m.H * m.W;
  const bool scales_ok = !m.normalize || (m.inv_std[0] > 0.0f && m.inv_std[1] > 0.0f && m.inv_std[2] > 0.0f);
  if (m.dtype == DAT_BF16 && m.fuse_pgd_grad && scales_ok) {
    // algorithmic bytes per element: x, delta, G read (12), delta written (4), bf16 input written (2)
    DAT_PROF(m, DAT_PROF_PGD, (double)npix * 3 * 18, st, launch_attack_update_netgrad(x, m.grad[0], delta, npix, eps, alpha, in, st));
    return DAT_OK;
  }
  DAT_TRY(pixel_grad(m, B, m.gx, st));
  DAT_PROF(m, DAT_PROF_PGD, (double)npix * 3 * (m.dtype == DAT_BF16 ? 18 : 20), st,
           launch_attack_update(x, m.gx, delta, npix, eps, alpha, in, st));
  return DAT_OK;
}

dat_status fetch_losses(dat_model& m, int count, float* host_out, hipStream_t st) {
  DAT_HIP(hipMemcpyAsync(m.host_stage, m.loss_steps, (size_t)count * 4, hipMemcpyDeviceToHost, st));
  DAT_HIP(hipStreamSynchronize(st));
  memcpy(host_out, m.host_stage, (size_t)count * 4);
  // the one place a value is on the host anyway: a NaN or infinite loss is reported (device outputs are written)
  for (int i = 0; i < count; ++i)
    if (!std::isfinite(host_out[i])) return fail_with(DAT_ERR_NONFINITE, "a requested loss value is NaN or infinite");
  return DAT_OK;
}

bool batch_ok(const dat_model* m, int B) { return B >= 1 && B <= m->maxB; }

}  // namespace

// =============================================================================================
extern "C" dat_status dat_model_create(dat_arch arch, dat_dtype dtype, int max_batch, int H, int W, int num_classes,
                                       const float* mean, const float* stdv, dat_model** out) {
  if (!out || max_batch < 1 || H < 1 || W < 1 || num_classes < 1) return DAT_ERR_ARG;
  if (dtype != DAT_F32 && dtype != DAT_BF16) return DAT_ERR_ARG;
  if ((mean == nullptr) != (stdv == nullptr)) return DAT_ERR_ARG;
  dat_model* m = new (std::nothrow) dat_model();
  if (!m) return DAT_ERR_NOMEM;
  m->arch = arch; m->dtype = dtype; m->maxB = max_batch; m->H = H; m->W = W; m->classes = num_classes;
  if (mean) {
    m->normalize = 1;
    for (int c = 0; c < 3; ++c) {
      if (!(stdv[c] > 0.0f)) { delete m; return DAT_ERR_ARG; }
      m->mean[c] = mean[c]; m->inv_std[c] = 1.0f / stdv[c];
    }
  }
  m->add_tensor({H, W, dtype == DAT_BF16 ? 8 : 3});
  if (!build_graph(*m)) { delete m; return DAT_ERR_UNSUPPORTED; }
  decide_blocked_stem(*m);
  link_fusions(*m);
  for (const Shape& s : m->tens)
    if (s.H < 1 || s.W < 1) { delete m; return DAT_ERR_SHAPE; }
  dat_status s = allocate(*m);
  if (s != DAT_OK) { dat_model_destroy(m); return s; }
  *out = m;
  return DAT_OK;
}

extern "C" dat_status dat_model_destroy(dat_model* m) {
  if (!m) return DAT_ERR_ARG;
  (void)hipDeviceSynchronize();
  for (void* p : m->allocs) (void)hipFree(p);
  for (auto& r : m->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (hipEvent_t e : m->pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : m->wg_events) (void)hipEventDestroy(e);
  if (m->wg_join) (void)hipEventDestroy(m->wg_join);
  if (m->wg_stream) (void)hipStreamDestroy(m->wg_stream);
  if (m->host_stage) (void)hipHostFree(m->host_stage);
  delete m;
  return DAT_OK;
}

extern "C" dat_status dat_model_num_params(const dat_model* m, int64_t* d, int* num_tensors) {
  if (!m) return DAT_ERR_ARG;
  if (d) *d = m->d;
  if (num_tensors) *num_tensors = (int)m->ptab.size();
  return DAT_OK;
}

extern "C" dat_status dat_model_tensor_table(const dat_model* m, int64_t* offsets, int32_t* fan_in, int32_t* kind) {
  if (!m || !offsets) return DAT_ERR_ARG;
  for (size_t i = 0; i < m->ptab.size(); ++i) {
    offsets[i] = m->ptab[i].off;
    if (fan_in) fan_in[i] = m->ptab[i].fan_in;
    if (kind) kind[i] = m->ptab[i].kind;
  }
  offsets[m->ptab.size()] = m->d;
  return DAT_OK;
}

extern "C" const int64_t* dat_model_offsets_device(const dat_model* m) { return m ? m->offsets_dev : nullptr; }

extern "C" dat_status dat_model_set_params(dat_model* m, const float* host_flat) {
  if (!m || !host_flat) return DAT_ERR_ARG;
  DAT_HIP(hipMemcpy(m->master, host_flat, (size_t)m->d * 4, hipMemcpyHostToDevice));
  DAT_TRY(refresh_compute(*m, nullptr));
  DAT_HIP(hipDeviceSynchronize());
  return DAT_OK;
}

extern "C" dat_status dat_model_get_params(const dat_model* m, float* host_flat) {
  if (!m || !host_flat) return DAT_ERR_ARG;
  DAT_HIP(hipDeviceSynchronize());
  DAT_HIP(hipMemcpy(host_flat, m->master, (size_t)m->d * 4, hipMemcpyDeviceToHost));
  return DAT_OK;
}

extern "C" dat_status dat_attack(dat_model* m, const float* x, const int32_t* y, int B, float eps, float alpha, int K,
                                 dat_init init, float* delta, float* loss_per_step, void* stream) {
  if (!m || !x || !y || !delta || K < 0 || !(eps >= 0.0f) || !(alpha >= 0.0f)) return DAT_ERR_ARG;
  if (init.mode != DAT_INIT_ZERO && init.mode != DAT_INIT_UNIFORM && init.mode != DAT_INIT_GIVEN) return DAT_ERR_ARG;
  if (init.mode == DAT_INIT_GIVEN && (!init.delta0 || !aligned(init.delta0, 16))) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(delta, 16)) return DAT_ERR_ARG;
  if (!batch_ok(m, B)) return DAT_ERR_SHAPE;
  if (loss_per_step && K + 1 > m->loss_cap) return DAT_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  const int64_t npix = (int64_t)B * m->H * m->W;
  const NetInputDesc in = input_desc(*m);
  DAT_TRY(launch_attack_init(x, npix, eps, init, delta, in, st));
  for (int k = 0; k < K; ++k) {
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(loss_grad(*m, y, B, 1.0f, loss_per_step ? k : 0, st));
    DAT_TRY(backward(*m, B, nullptr, true, st));
    DAT_TRY(pgd_step(*m, x, delta, B, eps, alpha, in, st));
  }
  if (loss_per_step) {
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(loss_grad(*m, y, B, 1.0f, K, st));
    DAT_TRY(fetch_losses(*m, K + 1, loss_per_step, st));
  }
  return DAT_OK;
}

extern "C" dat_status dat_step(dat_model* m, const float* x_adv, const int32_t* y, int B, float* grads, float* loss,
                               void* stream) {
  if (!m || !x_adv || !y || !grads) return DAT_ERR_ARG;
  if (!aligned(x_adv, 16) || !aligned(grads, 16)) return DAT_ERR_ARG;
  if (!batch_ok(m, B)) return DAT_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  DAT_TRY(launch_make_input(x_adv, nullptr, (int64_t)B * m->H * m->W, input_desc(*m), st));
  DAT_TRY(forward(*m, B, st));
  DAT_TRY(loss_grad(*m, y, B, 1.0f / (float)B, 0, st));
  DAT_TRY(backward(*m, B, grads, false, st));
  if (loss) DAT_TRY(fetch_losses(*m, 1, loss, st));
  return DAT_OK;
}

namespace {

// Logit gradient of one branch of the TRADES regulariser, from the kept clean logits and the logits in place.
dat_status kl_grad(dat_model& m, const float* z_clean, const float* z_adv, const int32_t* y, int branch, float lambda, int B,
                   float gscale, int loss_slot, hipStream_t st) {
  const int t = m.ops.back().out;
  DAT_TRY(kl_forward_backward(z_clean, z_adv, y, branch, lambda, (float*)m.grad[t], m.loss_n, m.loss_steps + loss_slot, B,
                              m.classes, gscale, st));
  std::fill(m.ghas.begin(), m.ghas.end(), 0);
  m.ghas[t] = 1;
  return DAT_OK;
}

dat_status ensure_bank(dat_model& m) {
  dat_model::PassBank& b = m.bank2;
  if (b.ready) return DAT_OK;
  const int es = m.esize();
  b.act.assign(m.tens.size(), nullptr);
  b.mean.assign(m.ops.size(), nullptr); b.rstd.assign(m.ops.size(), nullptr);
  b.mask.assign(m.ops.size(), nullptr); b.argmax.assign(m.ops.size(), nullptr);
  for (size_t t = 0; t < m.tens.size(); ++t)
    DAT_TRY(dev_alloc(m, &b.act[t], (size_t)m.maxB * m.tens[t].numel() * (m.is_f32[t] ? 4 : es)));
  for (size_t i = 0; i < m.ops.size(); ++i) {
    const Op& op = m.ops[i];
    if (op.mean) DAT_TRY(dev_alloc(m, &b.mean[i], (size_t)m.tens[op.in].C * 4));
    if (op.rstd) DAT_TRY(dev_alloc(m, &b.rstd[i], (size_t)m.tens[op.in].C * 4));
    if (op.mask) DAT_TRY(dev_alloc(m, &b.mask[i], (size_t)m.maxB * m.tens[op.in].numel() / 8));
    if (op.argmax) DAT_TRY(dev_alloc(m, &b.argmax[i], (size_t)m.maxB * m.tens[op.out].numel()));
  }
  b.ready = true;
  return DAT_OK;
}

void swap_bank(dat_model& m) {
  dat_model::PassBank& b = m.bank2;
  for (size_t t = 0; t < m.tens.size(); ++t) std::swap(m.act[t], b.act[t]);
  for (size_t i = 0; i < m.ops.size(); ++i) {
    Op& op = m.ops[i];
    std::swap(op.mean, b.mean[i]); std::swap(op.rstd, b.rstd[i]); std::swap(op.mask, b.mask[i]); std::swap(op.argmax, b.argmax[i]);
  }
}

dat_status keep_logits(dat_model& m, float* dst, int B, hipStream_t st) {
  DAT_HIP(hipMemcpyAsync(dst, m.act[m.ops.back().out], (size_t)B * m.classes * 4, hipMemcpyDeviceToDevice, st));
  return DAT_OK;
}

}  // namespace

extern "C" dat_status dat_attack_kl(dat_model* m, const float* x, int B, float eps, float alpha, int K, dat_init init,
                                    float* delta, float* loss_per_step, void* stream) {
  if (!m || !x || !delta || K < 0 || !(eps >= 0.0f) || !(alpha >= 0.0f)) return DAT_ERR_ARG;
  if (init.mode != DAT_INIT_ZERO && init.mode != DAT_INIT_UNIFORM && init.mode != DAT_INIT_GIVEN) return DAT_ERR_ARG;
  if (init.mode == DAT_INIT_GIVEN && (!init.delta0 || !aligned(init.delta0, 16))) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(delta, 16)) return DAT_ERR_ARG;
  if (!batch_ok(m, B)) return DAT_ERR_SHAPE;
  if (loss_per_step && K + 1 > m->loss_cap) return DAT_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  const int64_t npix = (int64_t)B * m->H * m->W;
  const NetInputDesc in = input_desc(*m);
  const float* z_adv = (const float*)m->act[m->ops.back().out];
  // the clean pass: its logits stay fixed during the ascent
  DAT_TRY(launch_make_input(x, nullptr, npix, in, st));
  DAT_TRY(forward(*m, B, st));
  DAT_TRY(keep_logits(*m, m->z_keep, B, st));
  DAT_TRY(launch_attack_init(x, npix, eps, init, delta, in, st));
  for (int k = 0; k < K; ++k) {
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(kl_grad(*m, m->z_keep, z_adv, nullptr, 0, 0.0f, B, 1.0f, loss_per_step ? k : 0, st));
    DAT_TRY(backward(*m, B, nullptr, true, st));
    DAT_TRY(pgd_step(*m, x, delta, B, eps, alpha, in, st));
  }
  if (loss_per_step) {
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(kl_grad(*m, m->z_keep, z_adv, nullptr, 0, 0.0f, B, 1.0f, K, st));
    DAT_TRY(fetch_losses(*m, K + 1, loss_per_step, st));
  }
  return DAT_OK;
}

extern "C" dat_status dat_step_reg(dat_model* m, const float* x, const float* x_adv, const int32_t* y, int B, float lambda,
                                   dat_phi phi, float* grads, float* losses, void* stream) {
  if (!m || !x || !x_adv || !y || !grads || !(lambda >= 0.0f)) return DAT_ERR_ARG;
  if (phi != DAT_PHI_CE && phi != DAT_PHI_TRADES_KL) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(x_adv, 16) || !aligned(grads, 16)) return DAT_ERR_ARG;
  if (!batch_ok(m, B)) return DAT_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  const int64_t npix = (int64_t)B * m->H * m->W;
  const NetInputDesc in = input_desc(*m);
  const float inv = 1.0f / (float)B;
  const bool two_pass = phi == DAT_PHI_TRADES_KL || lambda != 0.0f;
  if (two_pass && !m->g_tmp) DAT_TRY(dev_alloc(*m, &m->g_tmp, (size_t)m->d * 4));
  float host[2] = {0.0f, 0.0f};
  if (phi == DAT_PHI_CE) {
    if (lambda != 0.0f) {   // lambda * clean loss, its own forward/backward
      DAT_TRY(launch_make_input(x, nullptr, npix, in, st));
      DAT_TRY(forward(*m, B, st));
      DAT_TRY(loss_grad(*m, y, B, lambda * inv, 0, st));
      DAT_TRY(backward(*m, B, m->g_tmp, false, st));
    }
    DAT_TRY(launch_make_input(x_adv, nullptr, npix, in, st));
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(loss_grad(*m, y, B, inv, 1, st));
    DAT_TRY(backward(*m, B, grads, false, st));
  } else if (m->keep_both_passes && ensure_bank(*m) == DAT_OK) {
    // the clean pass stays in one set of buffers while the perturbed pass runs in the other; each branch's backward
    // sweep then finds its own activations (a failed allocation of the second set falls through to the path below)
    const int tz = m->ops.back().out;
    DAT_TRY(launch_make_input(x, nullptr, npix, in, st));
    DAT_TRY(forward(*m, B, st));
    const float* z_clean = (const float*)m->act[tz];
    swap_bank(*m);
    dat_status s = launch_make_input(x_adv, nullptr, npix, input_desc(*m), st);   // (the network input is one of the exchanged buffers)
    if (s == DAT_OK) s = forward(*m, B, st);
    const float* z_adv = (const float*)m->act[tz];
    if (s == DAT_OK) s = kl_grad(*m, z_clean, z_adv, y, 0, lambda, B, inv, 1, st);
    if (s == DAT_OK) s = backward(*m, B, grads, false, st);
    swap_bank(*m);                        // the clean pass is the model's current one again, also after an error
    DAT_TRY(s);
    DAT_TRY(kl_grad(*m, z_clean, z_adv, y, 1, lambda, B, inv, 0, st));
    DAT_TRY(backward(*m, B, m->g_tmp, false, st));
  } else {
    const float* z_here = (const float*)m->act[m->ops.back().out];
    // clean logits, then the perturbed pass and its branch of the gradient
    DAT_TRY(launch_make_input(x, nullptr, npix, in, st));
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(keep_logits(*m, m->z_keep, B, st));
    DAT_TRY(launch_make_input(x_adv, nullptr, npix, in, st));
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(kl_grad(*m, m->z_keep, z_here, y, 0, lambda, B, inv, 1, st));
    DAT_TRY(keep_logits(*m, m->z_keep2, B, st));
    DAT_TRY(backward(*m, B, grads, false, st));
    // the clean pass again (its activations were overwritten), with the clean branch's logit gradient
    DAT_TRY(launch_make_input(x, nullptr, npix, in, st));
    DAT_TRY(forward(*m, B, st));
    DAT_TRY(kl_grad(*m, z_here, m->z_keep2, y, 1, lambda, B, inv, 0, st));
    DAT_TRY(backward(*m, B, m->g_tmp, false, st));
  }
  if (two_pass) { DAT_TRY(launch_sgd(grads, m->g_tmp, -1.0f, m->d, st)); m->gscale_valid = false; }   // grads <- grads + g_tmp
  if (losses) {
    DAT_TRY(fetch_losses(*m, 2, host, st));
    losses[0] = (phi == DAT_PHI_CE && lambda == 0.0f) ? 0.0f : host[0];
    losses[1] = host[1];
  }
  return DAT_OK;
}

extern "C" dat_status dat_input_grad(dat_model* m, const float* x, const int32_t* y, int B, float* gx, float* logits,
                                     float* loss, void* stream) {
  if (!m || !x || !y || !gx) return DAT_ERR_ARG;
  if (!aligned(x, 16) || !aligned(gx, 16)) return DAT_ERR_ARG;
  if (!batch_ok(m, B)) return DAT_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  DAT_TRY(launch_make_input(x, nullptr, (int64_t)B * m->H * m->W, input_desc(*m), st));
  DAT_TRY(forward(*m, B, st));
  if (logits)
    DAT_HIP(hipMemcpyAsync(logits, m->act[m->ops.back().out], (size_t)B * m->classes * 4, hipMemcpyDeviceToDevice, st));
  DAT_TRY(loss_grad(*m, y, B, 1.0f, 0, st));
  DAT_TRY(backward(*m, B, nullptr, true, st));
  DAT_TRY(pixel_grad(*m, B, gx, st));
  if (loss) DAT_TRY(fetch_losses(*m, 1, loss, st));
  return DAT_OK;
}

extern "C" dat_status dat_model_grad_scales(const dat_model* m, const float** scales_dev) {
  if (!m || !scales_dev) return DAT_ERR_ARG;
  if (!m->gscale_valid) return fail_with(DAT_ERR_UNSUPPORTED, "dat_model_grad_scales: the last call on this model did not produce per-tensor abs-max values "
                                                              "(fp32 model, a model with bias layers, a two-pass objective, or no dat_step yet)");
  *scales_dev = reinterpret_cast<const float*>(m->gscale);
  return DAT_OK;
}

extern "C" dat_status dat_sgd_update(dat_model* m, const float* grads, float lr, void* stream) {
  if (!m || !grads) return DAT_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  DAT_TRY(launch_sgd(m->master, grads, lr, m->d, st));
  DAT_TRY(refresh_compute(*m, st));
  return DAT_OK;
}

extern "C" dat_status dat_model_set_option(dat_model* m, dat_option opt, int value) {
  if (!m) return DAT_ERR_ARG;
  switch (opt) {
    case DAT_OPT_FUSE_BN_INPUT_GRAD: m->fuse_bn_apply = value != 0; return DAT_OK;
    case DAT_OPT_FUSE_PGD_GRADIENT: m->fuse_pgd_grad = value != 0; return DAT_OK;
    case DAT_OPT_FUSE_BN_SUMS: m->fuse_bn_sums = value != 0; return DAT_OK;
    case DAT_OPT_SPARSE_SHORTCUT_GRADIENT: m->sparse_shortcut_grad = value != 0; return DAT_OK;
    case DAT_OPT_OVERLAP_WEIGHT_GRADIENTS: m->overlap_wgrad = value != 0; return DAT_OK;
    case DAT_OPT_ABSORB_SHORTCUT_BN: m->absorb_shortcut_bn = value != 0; link_fusions(*m); return DAT_OK;
    case DAT_OPT_FUSE_STEM_POOL: m->fuse_pool = value != 0; return DAT_OK;
    case DAT_OPT_GRADIENT_SCALES: m->grad_scales = value != 0; return DAT_OK;
    case DAT_OPT_KEEP_BOTH_PASSES: m->keep_both_passes = value != 0; return DAT_OK;
  }
  return DAT_ERR_ARG;
}

extern "C" dat_status dat_profile_enable(dat_model* m, int on) {
  if (!m) return DAT_ERR_ARG;
  DAT_HIP(hipDeviceSynchronize());
  for (auto& r : m->recs) { m->pool.push_back(r.a); m->pool.push_back(r.b); }
  m->recs.clear();
  m->prof = on != 0;
  return DAT_OK;
}

extern "C" dat_status dat_profile_read(dat_model* m, int cls, double* ms_total, int64_t* launches, double* work) {
  if (!m || cls < 0 || cls >= DAT_PROF_NUM_CLASSES) return DAT_ERR_ARG;
  DAT_HIP(hipDeviceSynchronize());
  double ms = 0.0, w = 0.0; int64_t n = 0;
  for (auto& r : m->recs) {
    if (r.cls != cls) continue;
    float t = 0.f;
    DAT_HIP(hipEventElapsedTime(&t, r.a, r.b));
    ms += t; w += r.work; n += r.nlaunch;
  }
  if (ms_total) *ms_total = ms;
  if (launches) *launches = n;
  if (work) *work = w;
  return DAT_OK;
}

extern "C" dat_status dat_lamb_update(dat_model* m, const float* grads, int use_adam, float eta, float beta1, float beta2,
                                      float zeta, float weight_decay, float c_l, float c_u, int t, void* stream) {
  if (!m || !grads || t < 1 || !(eta >= 0.0f) || !(c_u >= c_l)) return DAT_ERR_ARG;
  if (use_adam && (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f))) return DAT_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (!m->opt_u) {
    DAT_TRY(dev_alloc(*m, &m->opt_m, (size_t)m->d * 4));
    DAT_TRY(dev_alloc(*m, &m->opt_v, (size_t)m->d * 4));
    DAT_TRY(dev_alloc(*m, &m->opt_u, (size_t)m->d * 4));
    DAT_TRY(dev_alloc(*m, &m->opt_norms, m->ptab.size() * 2 * sizeof(double)));
    DAT_TRY(launch_fill_zero(m->opt_m, (size_t)m->d * 4, st));
    DAT_TRY(launch_fill_zero(m->opt_v, (size_t)m->d * 4, st));
  }
  LambParams hp;
  hp.use_adam = use_adam ? 1 : 0; hp.eta = eta; hp.b1 = beta1; hp.b2 = beta2; hp.zeta = zeta; hp.wd = weight_decay;
  hp.c_l = c_l; hp.c_u = c_u;
  hp.inv_bc1 = use_adam ? (float)(1.0 / (1.0 - pow((double)beta1, t))) : 1.0f;
  hp.inv_bc2 = use_adam ? (float)(1.0 / (1.0 - pow((double)beta2, t))) : 1.0f;
  DAT_TRY(launch_lamb(m->master, grads, m->opt_m, m->opt_v, m->opt_u, m->offsets_dev, (int)m->ptab.size(), m->d, hp,
                      m->opt_norms, st));
  DAT_TRY(refresh_compute(*m, st));
  return DAT_OK;
}

// ---- introspection for parity tests ---------------------------------------------------------------
extern "C" dat_status dat_inspect_counts(const dat_model* m, int* num_ops, int* num_tensors) {
  if (!m) return DAT_ERR_ARG;
  if (num_ops) *num_ops = (int)m->ops.size();
  if (num_tensors) *num_tensors = (int)m->tens.size();
  return DAT_OK;
}

extern "C" dat_status dat_inspect_op(const dat_model* m, int op, int32_t* info) {
  if (!m || !info || op < 0 || op >= (int)m->ops.size()) return DAT_ERR_ARG;
  const Op& o = m->ops[op];
  const int32_t v[10] = {(int32_t)o.kind, o.in, o.out, o.res, o.k, o.stride, o.pad, o.relu, o.p0, o.p1};
  for (int i = 0; i < 10; ++i) info[i] = v[i];
  return DAT_OK;
}

namespace {
// Activation tensors that exist in the layer graph but are never written in plain NHWC form by this model.
bool act_stored(const dat_model& m, int t) {
  if (t == 0) return m.dtype != DAT_BF16;   // bf16 network input: channels padded to 8, 2x2 pixel blocks behind a 7x7/2 stem
  for (const Op& o : m.ops) {
    if (o.out != t || o.kind != OP_BNACT) continue;
    if (o.absorbed_by >= 0) return false;
    if (o.pool >= 0 && m.fuse_pool) return false;
  }
  return true;
}
}  // namespace

extern "C" dat_status dat_inspect_tensor(const dat_model* m, int t, int32_t* info) {
  if (!m || !info || t < 0 || t >= (int)m->tens.size()) return DAT_ERR_ARG;
  const Shape s = m->tens[t];
  info[0] = s.H; info[1] = s.W; info[2] = s.C;
  info[3] = m->is_f32[t] ? 4 : m->esize();
  info[4] = act_stored(*m, t) ? 1 : 0;
  info[5] = (act_stored(*m, t) && m->ghas[t] == 1) ? 1 : 0;
  return DAT_OK;
}

extern "C" dat_status dat_inspect_read(dat_model* m, int which, int t, int B, void* host_dst, size_t bytes) {
  if (!m || !host_dst || t < 0 || t >= (int)m->tens.size() || (which != 0 && which != 1)) return DAT_ERR_ARG;
  if (!batch_ok(m, B)) return DAT_ERR_SHAPE;
  const size_t want = (size_t)B * m->tens[t].numel() * (m->is_f32[t] ? 4 : m->esize());
  if (bytes != want) return DAT_ERR_ARG;
  DAT_HIP(hipDeviceSynchronize());
  DAT_HIP(hipMemcpy(host_dst, which ? m->grad[t] : m->act[t], bytes, hipMemcpyDeviceToHost));
  return DAT_OK;
}

extern "C" dat_status dat_inspect_bn(dat_model* m, int op, float* mean_host, float* rstd_host) {
  if (!m || !mean_host || !rstd_host || op < 0 || op >= (int)m->ops.size() || m->ops[op].kind != OP_BNACT) return DAT_ERR_ARG;
  const size_t bytes = (size_t)m->tens[m->ops[op].in].C * 4;
  DAT_HIP(hipDeviceSynchronize());
  DAT_HIP(hipMemcpy(mean_host, m->ops[op].mean, bytes, hipMemcpyDeviceToHost));
  DAT_HIP(hipMemcpy(rstd_host, m->ops[op].rstd, bytes, hipMemcpyDeviceToHost));
  return DAT_OK;
}
