// dat_oracle.cpp -- plain CPU reference for one worker's distributed-adversarial-training
// step.  THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: only the test-suite, the smoke check
// and the benchmark's cpu_baseline leg may call it.  It shares no code with the GPU library.
//
// What it computes, following the paper (Liu et al., "Distributed Adversarial Training to
// Robustify Deep Neural Networks at Scale", UAI 2022):
//   * the inner maximisation of Eq. (1) / Alg. A1 step 5 by K projected sign-gradient steps
//     z_k = Proj_[-eps,eps](z_{k-1} + alpha * sign(grad_delta phi)), the unified PGD / FGSM
//     form given in the "Other add-ons" paragraph of Sec. "Methodologies";
//   * the local gradient of Alg. A1 step 6, Eq. (stoch_grad_batch), with lambda = 0 and
//     phi = cross-entropy: the batch MEAN of grad_theta CE at the perturbed samples;
//   * the randomized quantizer Q of Alg. A1 step 7, Eqs. (rand_q) and (xi) of appendix
//     "Additional details on gradient quantization", and its inverse used by Eq. (grad_agg);
//   * (next row) the layer-wise adaptive update of Eq. (3) and LAMB, Alg. A2.
//
// Arithmetic.  Network forward / backward run in fp64.  In "bf16 storage" mode every tensor
// that the GPU library keeps in bf16 (conv / linear weights, every stored activation and
// activation gradient) is rounded to bf16 (round-to-nearest-even) at the point it is stored;
// nothing else changes.  The perturbation update and the quantizer are defined in fp32 with
// one rounding per operation (built with -ffp-contract=off), because their results are
// compared bit for bit.
//
// Layout (an interface shared with the library, not code): activations NHWC, convolution
// weights [Cout][kh][kw][Cin], linear weights [out][in]; parameters form one flat vector in
// op order (conv: W [, bias]; batch-norm: gamma, beta; linear: W, b).
//
// Parity pins (tests/test_oracle_*.py): central finite differences, adjoint identities,
// closed-form softmax-CE gradient, published parameter counts of the three ResNets,
// Philox4x32-10 known answers, quantizer mean/variance closed forms, attack invariants,
// brute-force inner maximum of a linear model, an autograd mirror of every architecture and of
// the general objective.  Parity unpinned: (1) trained-model accuracies, which need data that does
// not exist in this build; (2) the PLACEMENT of the bf16 rounding points in bf16-storage mode --
// which tensors are rounded, and that a gradient with several contributions is stored after the
// first and re-rounded after each later one.  That placement mirrors the GPU library's storage
// schedule on purpose (it is a definition both sides share, the paper fixes no precision); the
// arithmetic between the rounding points is the fp64 mode's, which the pins above cover.
//
// Besides the whole-network entry points there is a stepping interface (orc_begin, orc_forward_op,
// orc_loss_backward_begin, orc_backward_op, orc_get/set/compare_tensor): one op at a time, with
// any stored tensor replaceable from outside, for teacher-forced comparisons; the tests show that
// stepping reproduces the whole-network results bit for bit.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// ----------------------------------------------------------------------------------------
// bf16 rounding of an fp64 value: round to nearest, ties to even, on the 8-bit-significand
// grid with fp32's exponent range.  Going through fp32 first would round twice, so the tie
// test is done on the fp64 value itself.
// ----------------------------------------------------------------------------------------
double round_bf16(double v) {
  if (!(v == v) || std::isinf(v) || v == 0.0) return v;
  int e;
  double m = std::frexp(v, &e);            // v = m * 2^e, 0.5 <= |m| < 1
  // bf16 keeps 8 significant bits: quantum is 2^(e-8); below the normal range the quantum
  // is fixed at 2^-133 (bf16 subnormals share fp32's smallest exponent).
  int qe = e - 8;
  if (qe < -133) qe = -133;
  double q = std::ldexp(1.0, qe);
  double r = std::nearbyint(v / q) * q;    // default rounding mode: nearest-even
  (void)m;
  if (std::fabs(r) > 3.3895313892515355e38) r = (v > 0 ? INFINITY : -INFINITY);
  return r;
}

// ----------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
// SC'11): ten rounds of two 32x32->64 multiplies with a Weyl-sequence key schedule.
// ----------------------------------------------------------------------------------------
struct U4 { uint32_t v[4]; };

U4 philox4x32_10(U4 ctr, uint32_t k0, uint32_t k1) {
  const uint64_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
  const uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
  for (int round = 0; round < 10; ++round) {
    uint64_t pa = MUL_A * (uint64_t)ctr.v[0];
    uint64_t pb = MUL_B * (uint64_t)ctr.v[2];
    U4 nx;
    nx.v[0] = (uint32_t)(pb >> 32) ^ ctr.v[1] ^ k0;
    nx.v[1] = (uint32_t)pb;
    nx.v[2] = (uint32_t)(pa >> 32) ^ ctr.v[3] ^ k1;
    nx.v[3] = (uint32_t)pa;
    ctr = nx;
    k0 += WEYL_A;
    k1 += WEYL_B;
  }
  return ctr;
}

// Uniform in [0,1) on a 2^-24 grid for flat element index i of random stream `stream`:
// counter = (i/4 low, i/4 high, stream, 0), key = seed halves, word i mod 4 of the block.
float uniform_at(uint64_t i, uint64_t seed, uint32_t stream) {
  U4 c;
  uint64_t blk = i >> 2;
  c.v[0] = (uint32_t)blk; c.v[1] = (uint32_t)(blk >> 32); c.v[2] = stream; c.v[3] = 0;
  U4 r = philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
  return (float)(r.v[i & 3] >> 8) * 5.9604644775390625e-8f;   // * 2^-24, exact
}

enum { STREAM_QUANT = 0, STREAM_INIT = 1 };

// ----------------------------------------------------------------------------------------
// Network description
// ----------------------------------------------------------------------------------------
enum OpKind { OP_CONV, OP_BIASACT, OP_BNACT, OP_MAXPOOL, OP_GAP, OP_FC };

struct Shape { int H, W, C; int64_t numel() const { return (int64_t)H * W * C; } };

struct Op {
  OpKind kind;
  int in, out;
  int res = -1;            // optional second input added before the activation / after conv
  int k = 0, stride = 1, pad = 0;
  int relu = 0;
  int p0 = -1, p1 = -1;    // indices into the parameter-tensor table
};

// kind: 0 conv W, 1 bias, 2 BN gamma, 3 BN beta, 4 fc W, 5 fc b, 6 gamma of the last BN of a residual branch
struct PTensor { int64_t off, numel; int fan_in; int kind; };

struct Model {
  int arch = 0, emu = 0, classes = 0;
  // Optional model of summation-order freedom: every convolution sum is multiplied by
  // (1 + jitter*h), h a fixed hash of the output index in [-1,1), before it is stored.  Two
  // correct bf16-storage implementations differ by such a factor (fp32 accumulation error
  // ~1e-7) which bf16 re-rounding then amplifies; tests use this to measure that floor.
  double jitter = 0.0;
  Shape in_shape{};
  bool normalize = false;
  float mean[3] = {0, 0, 0}, inv_std[3] = {1, 1, 1};
  std::vector<Shape> tens;
  std::vector<Op> ops;
  std::vector<PTensor> ptab;
  std::vector<double> theta;    // as used by the network (bf16-rounded where stored bf16)
  std::vector<double> master;   // unrounded fp32 master copy (what the SGD step updates)
  int64_t d = 0;

  // per-call state
  int B = 0;
  std::vector<std::vector<double>> act, gact;
  std::vector<char> ghas;
  std::vector<std::vector<double>> bn_mean, bn_rstd;   // indexed by op
  std::vector<double> gtheta;

  int add_tensor(Shape s) { tens.push_back(s); return (int)tens.size() - 1; }
  int add_param(int64_t n, int fan_in, int kind) {
    ptab.push_back({d, n, fan_in, kind}); d += n; return (int)ptab.size() - 1;
  }
  double rb(double v) const { return emu ? round_bf16(v) : v; }

  int conv(int in, int cout, int k, int stride, int pad, int res = -1) {
    Shape s = tens[in];
    Shape o{(s.H + 2 * pad - k) / stride + 1, (s.W + 2 * pad - k) / stride + 1, cout};
    Op op; op.kind = OP_CONV; op.in = in; op.out = add_tensor(o); op.res = res;
    op.k = k; op.stride = stride; op.pad = pad;
    op.p0 = add_param((int64_t)cout * k * k * s.C, s.C * k * k, 0);
    ops.push_back(op); return op.out;
  }
  int biasact(int in, int relu) {
    Shape s = tens[in];
    Op op; op.kind = OP_BIASACT; op.in = in; op.out = add_tensor(s); op.relu = relu;
    op.p0 = add_param(s.C, 0, 1);
    ops.push_back(op); return op.out;
  }
  int bnact(int in, int relu, int res = -1, bool branch_final = false) {
    Shape s = tens[in];
    Op op; op.kind = OP_BNACT; op.in = in; op.out = add_tensor(s); op.relu = relu; op.res = res;
    op.p0 = add_param(s.C, 0, branch_final ? 6 : 2); op.p1 = add_param(s.C, 0, 3);
    ops.push_back(op); return op.out;
  }
  int maxpool(int in) {   // 3x3 window, stride 2, padding 1
    Shape s = tens[in];
    Shape o{(s.H + 2 - 3) / 2 + 1, (s.W + 2 - 3) / 2 + 1, s.C};
    Op op; op.kind = OP_MAXPOOL; op.in = in; op.out = add_tensor(o); op.k = 3; op.stride = 2; op.pad = 1;
    ops.push_back(op); return op.out;
  }
  int gap(int in) {
    Shape s = tens[in];
    Op op; op.kind = OP_GAP; op.in = in; op.out = add_tensor({1, 1, s.C});
    ops.push_back(op); return op.out;
  }
  int fc(int in, int nout) {
    Shape s = tens[in];
    Op op; op.kind = OP_FC; op.in = in; op.out = add_tensor({1, 1, nout});
    op.p0 = add_param((int64_t)nout * s.C, s.C, 4); op.p1 = add_param(nout, 0, 5);
    ops.push_back(op); return op.out;
  }
};

// Architectures.  The paper only names them (Sec. "Experiment setup"); the shapes are the
// standard ones of the cited architecture papers.
enum { ARCH_TINYCNN = 0, ARCH_RESNET18_CIFAR = 1, ARCH_WRN34_10 = 2, ARCH_RESNET50 = 3, ARCH_PREACT_RESNET18 = 4, ARCH_WRN28_10 = 5,
       ARCH_TESTNET = 100, ARCH_LINEAR = 101 };

void build_tinycnn(Model& m) {
  int t = 0;
  t = m.conv(t, 16, 3, 1, 1); t = m.biasact(t, 1);
  t = m.conv(t, 32, 3, 2, 1); t = m.biasact(t, 1);
  t = m.gap(t);
  m.fc(t, m.classes);
}

int basic_block(Model& m, int x, int cout, int stride) {
  int cin = m.tens[x].C;
  int y = m.conv(x, cout, 3, stride, 1); y = m.bnact(y, 1);
  y = m.conv(y, cout, 3, 1, 1);
  int sc = x;
  if (stride != 1 || cin != cout) { sc = m.conv(x, cout, 1, stride, 0); sc = m.bnact(sc, 0); }
  return m.bnact(y, 1, sc, true);
}

void build_resnet18_cifar(Model& m) {
  int t = m.conv(0, 64, 3, 1, 1); t = m.bnact(t, 1);
  const int widths[4] = {64, 128, 256, 512};
  for (int g = 0; g < 4; ++g)
    for (int b = 0; b < 2; ++b) t = basic_block(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
  t = m.gap(t);
  m.fc(t, m.classes);
}

int bottleneck(Model& m, int x, int width, int stride) {
  int cin = m.tens[x].C, cout = 4 * width;
  int y = m.conv(x, width, 1, 1, 0); y = m.bnact(y, 1);
  y = m.conv(y, width, 3, stride, 1); y = m.bnact(y, 1);
  y = m.conv(y, cout, 1, 1, 0);
  int sc = x;
  if (stride != 1 || cin != cout) { sc = m.conv(x, cout, 1, stride, 0); sc = m.bnact(sc, 0); }
  return m.bnact(y, 1, sc, true);
}

void build_resnet50(Model& m) {
  int t = m.conv(0, 64, 7, 2, 3); t = m.bnact(t, 1);
  t = m.maxpool(t);
  const int widths[4] = {64, 128, 256, 512}, depth[4] = {3, 4, 6, 3};
  for (int g = 0; g < 4; ++g)
    for (int b = 0; b < depth[g]; ++b) t = bottleneck(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
  t = m.gap(t);
  m.fc(t, m.classes);
}

// Pre-activation wide block: o = relu(bn(x)); branch = conv(relu(bn(conv(o)))); the shortcut
// is x itself, or a strided 1x1 conv of o when the shape changes.
int wide_block(Model& m, int x, int cout, int stride) {
  int cin = m.tens[x].C;
  int o = m.bnact(x, 1);
  int y = m.conv(o, cout, 3, stride, 1); y = m.bnact(y, 1, -1, true);
  int sc = x;
  if (stride != 1 || cin != cout) sc = m.conv(o, cout, 1, stride, 0);
  return m.conv(y, cout, 3, 1, 1, sc);
}

void build_wrn(Model& m, int depth, int widen) {
  int n = (depth - 4) / 6;
  int t = m.conv(0, 16, 3, 1, 1);
  const int widths[3] = {16 * widen, 32 * widen, 64 * widen};
  for (int g = 0; g < 3; ++g)
    for (int b = 0; b < n; ++b) t = wide_block(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
  t = m.bnact(t, 1);
  t = m.gap(t);
  m.fc(t, m.classes);
}

// Pre-activation ResNet-18 (Sec. "Experiment setup": the CIFAR model the paper calls ResNet-18;
// He et al., identity mappings): a 3x3 stem without normalisation, pre-activation basic blocks
// [2,2,2,2] of widths 64..512 (the shortcut convolution reads the activated input), a final
// BN + ReLU, pooling and the classifier.  The block is the wide block with widening factor 1.
void build_preact_resnet18(Model& m) {
  int t = m.conv(0, 64, 3, 1, 1);
  const int widths[4] = {64, 128, 256, 512};
  for (int g = 0; g < 4; ++g)
    for (int b = 0; b < 2; ++b) t = wide_block(m, t, widths[g], (b == 0 && g > 0) ? 2 : 1);
  t = m.bnact(t, 1);
  t = m.gap(t);
  m.fc(t, m.classes);
}

// A small net touching every op kind, for finite differences.
void build_testnet(Model& m) {
  int t = m.conv(0, 8, 3, 1, 1); t = m.bnact(t, 1);
  t = m.maxpool(t);
  t = basic_block(m, t, 8, 1);
  t = basic_block(m, t, 16, 2);
  t = bottleneck(m, t, 8, 2);
  t = wide_block(m, t, 16, 1);
  t = wide_block(m, t, 16, 1);
  t = m.bnact(t, 1);
  t = m.gap(t);
  m.fc(t, m.classes);
}

// Global average pool + linear layer: logits are affine in the pixels (brute-force attack pin).
void build_linear(Model& m) { int t = m.gap(0); m.fc(t, m.classes); }

// ----------------------------------------------------------------------------------------
// Layer arithmetic: definitions written out.
// ----------------------------------------------------------------------------------------

// out[n,ho,wo,co] = sum_{r,s,ci} in[n, ho*st+r-p, wo*st+s-p, ci] * W[co,r,s,ci]  (+ res)
void conv_forward(Model& m, const Op& op, int B) {
  const Shape si = m.tens[op.in], so = m.tens[op.out];
  const double* in = m.act[op.in].data();
  const double* W = m.theta.data() + m.ptab[op.p0].off;
  const double* res = op.res >= 0 ? m.act[op.res].data() : nullptr;
  double* out = m.act[op.out].data();
  const int k = op.k, st = op.stride, p = op.pad, Ci = si.C, Co = so.C;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int ho = 0; ho < so.H; ++ho)
      for (int wo = 0; wo < so.W; ++wo)
        for (int co = 0; co < Co; ++co) {
          double acc = 0.0;
          for (int r = 0; r < k; ++r) {
            int hi = ho * st + r - p;
            if (hi < 0 || hi >= si.H) continue;
            for (int s = 0; s < k; ++s) {
              int wi = wo * st + s - p;
              if (wi < 0 || wi >= si.W) continue;
              const double* xp = in + (((int64_t)n * si.H + hi) * si.W + wi) * Ci;
              const double* wp = W + (((int64_t)co * k + r) * k + s) * Ci;
              double part = 0.0;
#pragma omp simd reduction(+ : part)
              for (int ci = 0; ci < Ci; ++ci) part += xp[ci] * wp[ci];
              acc += part;
            }
          }
          int64_t o = (((int64_t)n * so.H + ho) * so.W + wo) * Co + co;
          if (res) acc += res[o];
          if (m.jitter != 0.0) {
            uint64_t hsh = (uint64_t)o * 0x9E3779B97F4A7C15ull;
            hsh ^= hsh >> 29; hsh *= 0xBF58476D1CE4E5B9ull; hsh ^= hsh >> 32;
            acc *= 1.0 + m.jitter * ((double)(hsh & 0xFFFFFF) / 8388608.0 - 1.0);
          }
          out[o] = m.rb(acc);
        }
}

// Adds `v` into the gradient slot of tensor t following the storage rule: the first
// contribution is stored (rounded), later ones are added to the stored value and re-rounded.
struct GradSink {
  Model& m; int t; bool first; bool stored_bf16;
  GradSink(Model& mm, int tt, bool bf16_tensor = true)
      : m(mm), t(tt), first(!mm.ghas[tt]), stored_bf16(bf16_tensor) { mm.ghas[tt] = 1; }
  inline void put(int64_t i, double v) {
    double* g = m.gact[t].data();
    double s = first ? v : g[i] + v;
    g[i] = stored_bf16 ? m.rb(s) : s;
  }
};

void conv_backward(Model& m, const Op& op, int B, bool want_wgrad) {
  const Shape si = m.tens[op.in], so = m.tens[op.out];
  const double* in = m.act[op.in].data();
  const double* W = m.theta.data() + m.ptab[op.p0].off;
  const double* dout = m.gact[op.out].data();
  const int k = op.k, st = op.stride, p = op.pad, Ci = si.C, Co = so.C;

  if (op.res >= 0) {   // out = conv + res  =>  d res = d out (stored values, copied)
    GradSink sink(m, op.res);
    int64_t tot = (int64_t)B * so.numel();
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < tot; ++i) sink.put(i, dout[i]);
  }

  if (want_wgrad) {
    // dW[co,r,s,ci] = sum_{n,ho,wo} dout[n,ho,wo,co] * in[n,ho*st+r-p,wo*st+s-p,ci]
    double* dW = m.gtheta.data() + m.ptab[op.p0].off;
#pragma omp parallel for schedule(dynamic, 1)
    for (int co = 0; co < Co; ++co) {
      double* dw = dW + (int64_t)co * k * k * Ci;
      std::fill(dw, dw + (int64_t)k * k * Ci, 0.0);
      for (int n = 0; n < B; ++n)
        for (int ho = 0; ho < so.H; ++ho)
          for (int wo = 0; wo < so.W; ++wo) {
            double g = dout[(((int64_t)n * so.H + ho) * so.W + wo) * Co + co];
            if (g == 0.0) continue;
            for (int r = 0; r < k; ++r) {
              int hi = ho * st + r - p;
              if (hi < 0 || hi >= si.H) continue;
              for (int s = 0; s < k; ++s) {
                int wi = wo * st + s - p;
                if (wi < 0 || wi >= si.W) continue;
                const double* xp = in + (((int64_t)n * si.H + hi) * si.W + wi) * Ci;
                double* dp = dw + ((int64_t)r * k + s) * Ci;
#pragma omp simd
                for (int ci = 0; ci < Ci; ++ci) dp[ci] += g * xp[ci];
              }
            }
          }
    }
  }

  // din[n,hi,wi,ci] = sum over (ho,wo,r,s,co) that touch it of dout * W  (adjoint, scatter form)
  std::vector<double> din((size_t)B * si.numel(), 0.0);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < B; ++n)
    for (int ho = 0; ho < so.H; ++ho)
      for (int wo = 0; wo < so.W; ++wo)
        for (int co = 0; co < Co; ++co) {
          double g = dout[(((int64_t)n * so.H + ho) * so.W + wo) * Co + co];
          if (g == 0.0) continue;
          for (int r = 0; r < k; ++r) {
            int hi = ho * st + r - p;
            if (hi < 0 || hi >= si.H) continue;
            for (int s = 0; s < k; ++s) {
              int wi = wo * st + s - p;
              if (wi < 0 || wi >= si.W) continue;
              double* dp = din.data() + (((int64_t)n * si.H + hi) * si.W + wi) * Ci;
              const double* wp = W + (((int64_t)co * k + r) * k + s) * Ci;
#pragma omp simd
              for (int ci = 0; ci < Ci; ++ci) dp[ci] += g * wp[ci];
            }
          }
        }
  GradSink sink(m, op.in);
  int64_t tot = (int64_t)B * si.numel();
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < tot; ++i) sink.put(i, din[i]);
}

void biasact_forward(Model& m, const Op& op, int B) {
  const Shape s = m.tens[op.in];
  const double* in = m.act[op.in].data();
  const double* b = m.theta.data() + m.ptab[op.p0].off;
  double* out = m.act[op.out].data();
  int64_t rows = (int64_t)B * s.H * s.W;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c) {
      double v = in[i * s.C + c] + b[c];
      if (op.relu && !(v > 0.0)) v = 0.0;
      out[i * s.C + c] = m.rb(v);
    }
}

void biasact_backward(Model& m, const Op& op, int B) {
  const Shape s = m.tens[op.in];
  const double* out = m.act[op.out].data();
  const double* dout = m.gact[op.out].data();
  double* db = m.gtheta.data() + m.ptab[op.p0].off;
  int64_t rows = (int64_t)B * s.H * s.W;
  std::vector<double> acc(s.C, 0.0);
  GradSink sink(m, op.in);
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c) {
      double g = dout[i * s.C + c];
      if (op.relu && !(out[i * s.C + c] > 0.0)) g = 0.0;   // ReLU'(0) = 0
      acc[c] += g;
      sink.put(i * s.C + c, g);
    }
  for (int c = 0; c < s.C; ++c) db[c] = acc[c];
}

// Train-mode batch normalisation: statistics over (n,h,w) of the stored input, biased
// variance, eps = 1e-5; out = act(gamma * xhat + beta [+ res]).
void bnact_forward(Model& m, int opi, int B) {
  const Op& op = m.ops[opi];
  const Shape s = m.tens[op.in];
  const double* in = m.act[op.in].data();
  const double* gamma = m.theta.data() + m.ptab[op.p0].off;
  const double* beta = m.theta.data() + m.ptab[op.p1].off;
  const double* res = op.res >= 0 ? m.act[op.res].data() : nullptr;
  double* out = m.act[op.out].data();
  int64_t rows = (int64_t)B * s.H * s.W;
  std::vector<double>& mu = m.bn_mean[opi]; std::vector<double>& rs = m.bn_rstd[opi];
  mu.assign(s.C, 0.0); rs.assign(s.C, 0.0);
  // (channels are walked eight at a time so that a cache line is read once; every channel's sums
  // still run over the rows in order, one add per row)
#pragma omp parallel for schedule(static)
  for (int c0 = 0; c0 < s.C; c0 += 8) {
    const int nc = std::min(8, s.C - c0);
    double sum[8] = {0, 0, 0, 0, 0, 0, 0, 0}, sq[8] = {0, 0, 0, 0, 0, 0, 0, 0}, mean[8];
    for (int64_t i = 0; i < rows; ++i)
      for (int j = 0; j < nc; ++j) sum[j] += in[i * s.C + c0 + j];
    for (int j = 0; j < nc; ++j) mean[j] = sum[j] / (double)rows;
    for (int64_t i = 0; i < rows; ++i)
      for (int j = 0; j < nc; ++j) { double dlt = in[i * s.C + c0 + j] - mean[j]; sq[j] += dlt * dlt; }
    for (int j = 0; j < nc; ++j) {
      mu[c0 + j] = mean[j];
      rs[c0 + j] = 1.0 / std::sqrt(sq[j] / (double)rows + 1e-5);
    }
  }
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c) {
      double v = gamma[c] * ((in[i * s.C + c] - mu[c]) * rs[c]) + beta[c];
      if (res) v += res[i * s.C + c];
      if (op.relu && !(v > 0.0)) v = 0.0;
      out[i * s.C + c] = m.rb(v);
    }
}

// With dy the gradient after the activation mask:  dbeta = sum dy, dgamma = sum dy*xhat,
// dx = gamma*rstd*(dy - dbeta/M - xhat*dgamma/M)  (differentiates through mean and variance).
void bnact_backward(Model& m, int opi, int B) {
  const Op& op = m.ops[opi];
  const Shape s = m.tens[op.in];
  const double* in = m.act[op.in].data();
  const double* out = m.act[op.out].data();
  const double* dout = m.gact[op.out].data();
  const double* gamma = m.theta.data() + m.ptab[op.p0].off;
  double* dgamma = m.gtheta.data() + m.ptab[op.p0].off;
  double* dbeta = m.gtheta.data() + m.ptab[op.p1].off;
  int64_t rows = (int64_t)B * s.H * s.W;
  const std::vector<double>& mu = m.bn_mean[opi]; const std::vector<double>& rs = m.bn_rstd[opi];
  std::vector<double> dy((size_t)rows * s.C);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows * s.C; ++i) {
    double g = dout[i];
    if (op.relu && !(out[i] > 0.0)) g = 0.0;
    dy[i] = g;
  }
  if (op.res >= 0) {
    GradSink sink(m, op.res);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows * s.C; ++i) sink.put(i, dy[i]);
  }
#pragma omp parallel for schedule(static)
  for (int c0 = 0; c0 < s.C; c0 += 8) {   // (eight channels per cache line; per channel the rows in order)
    const int nc = std::min(8, s.C - c0);
    double sb[8] = {0, 0, 0, 0, 0, 0, 0, 0}, sg[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int64_t i = 0; i < rows; ++i)
      for (int j = 0; j < nc; ++j) {
        const int c = c0 + j;
        double xh = (in[i * s.C + c] - mu[c]) * rs[c];
        sb[j] += dy[i * s.C + c]; sg[j] += dy[i * s.C + c] * xh;
      }
    for (int j = 0; j < nc; ++j) { dbeta[c0 + j] = sb[j]; dgamma[c0 + j] = sg[j]; }
  }
  GradSink sink(m, op.in);
  const double invM = 1.0 / (double)rows;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c) {
      double xh = (in[i * s.C + c] - mu[c]) * rs[c];
      double v = gamma[c] * rs[c] * (dy[i * s.C + c] - dbeta[c] * invM - xh * dgamma[c] * invM);
      sink.put(i * s.C + c, v);
    }
}

void maxpool_forward(Model& m, const Op& op, int B) {
  const Shape si = m.tens[op.in], so = m.tens[op.out];
  const double* in = m.act[op.in].data();
  double* out = m.act[op.out].data();
#pragma omp parallel for schedule(static)
  for (int n = 0; n < B; ++n)
    for (int ho = 0; ho < so.H; ++ho)
      for (int wo = 0; wo < so.W; ++wo)
        for (int c = 0; c < si.C; ++c) {
          double best = -INFINITY;
          for (int r = 0; r < 3; ++r) for (int s = 0; s < 3; ++s) {
            int hi = ho * 2 + r - 1, wi = wo * 2 + s - 1;
            if (hi < 0 || hi >= si.H || wi < 0 || wi >= si.W) continue;
            double v = in[(((int64_t)n * si.H + hi) * si.W + wi) * si.C + c];
            if (v > best) best = v;
          }
          out[(((int64_t)n * so.H + ho) * so.W + wo) * si.C + c] = best;
        }
}

// The gradient of each window goes to its first maximum in (r,s) row-major order; an input
// covered by several windows receives the sum, rounded once.
void maxpool_backward(Model& m, const Op& op, int B) {
  const Shape si = m.tens[op.in], so = m.tens[op.out];
  const double* in = m.act[op.in].data();
  const double* dout = m.gact[op.out].data();
  std::vector<double> din((size_t)B * si.numel(), 0.0);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < B; ++n)
    for (int ho = 0; ho < so.H; ++ho)
      for (int wo = 0; wo < so.W; ++wo)
        for (int c = 0; c < si.C; ++c) {
          double best = -INFINITY; int64_t arg = -1;
          for (int r = 0; r < 3; ++r) for (int s = 0; s < 3; ++s) {
            int hi = ho * 2 + r - 1, wi = wo * 2 + s - 1;
            if (hi < 0 || hi >= si.H || wi < 0 || wi >= si.W) continue;
            int64_t idx = (((int64_t)n * si.H + hi) * si.W + wi) * si.C + c;
            if (in[idx] > best) { best = in[idx]; arg = idx; }
          }
          din[arg] += dout[(((int64_t)n * so.H + ho) * so.W + wo) * si.C + c];
        }
  GradSink sink(m, op.in);
  int64_t tot = (int64_t)B * si.numel();
  for (int64_t i = 0; i < tot; ++i) sink.put(i, din[i]);
}

void gap_forward(Model& m, const Op& op, int B) {   // mean over (h,w); kept unrounded
  const Shape s = m.tens[op.in];
  const double* in = m.act[op.in].data();
  double* out = m.act[op.out].data();
  int hw = s.H * s.W;
  for (int n = 0; n < B; ++n)
    for (int c = 0; c < s.C; ++c) {
      double sum = 0.0;
      for (int i = 0; i < hw; ++i) sum += in[((int64_t)n * hw + i) * s.C + c];
      out[(int64_t)n * s.C + c] = sum / hw;
    }
}

void gap_backward(Model& m, const Op& op, int B) {
  const Shape s = m.tens[op.in];
  const double* dout = m.gact[op.out].data();
  int hw = s.H * s.W;
  GradSink sink(m, op.in);
  for (int n = 0; n < B; ++n)
    for (int i = 0; i < hw; ++i)
      for (int c = 0; c < s.C; ++c)
        sink.put(((int64_t)n * hw + i) * s.C + c, dout[(int64_t)n * s.C + c] / hw);
}

void fc_forward(Model& m, const Op& op, int B) {
  const int ni = m.tens[op.in].C, no = m.tens[op.out].C;
  const double* in = m.act[op.in].data();
  const double* W = m.theta.data() + m.ptab[op.p0].off;
  const double* b = m.theta.data() + m.ptab[op.p1].off;
  double* out = m.act[op.out].data();
#pragma omp parallel for schedule(static)
  for (int n = 0; n < B; ++n)
    for (int o = 0; o < no; ++o) {
      double acc = 0.0;
      for (int i = 0; i < ni; ++i) acc += in[(int64_t)n * ni + i] * W[(int64_t)o * ni + i];
      out[(int64_t)n * no + o] = acc + b[o];
    }
}

void fc_backward(Model& m, const Op& op, int B) {
  const int ni = m.tens[op.in].C, no = m.tens[op.out].C;
  const double* in = m.act[op.in].data();
  const double* dout = m.gact[op.out].data();
  const double* W = m.theta.data() + m.ptab[op.p0].off;
  double* dW = m.gtheta.data() + m.ptab[op.p0].off;
  double* db = m.gtheta.data() + m.ptab[op.p1].off;
  for (int o = 0; o < no; ++o) {
    double sb = 0.0;
    for (int n = 0; n < B; ++n) sb += dout[(int64_t)n * no + o];
    db[o] = sb;
    for (int i = 0; i < ni; ++i) {
      double acc = 0.0;
      for (int n = 0; n < B; ++n) acc += dout[(int64_t)n * no + o] * in[(int64_t)n * ni + i];
      dW[(int64_t)o * ni + i] = acc;
    }
  }
  GradSink sink(m, op.in, false);   // the pooled features are not a bf16-stored tensor
  for (int n = 0; n < B; ++n)
    for (int i = 0; i < ni; ++i) {
      double acc = 0.0;
      for (int o = 0; o < no; ++o) acc += dout[(int64_t)n * no + o] * W[(int64_t)o * ni + i];
      sink.put((int64_t)n * ni + i, acc);
    }
}

// ----------------------------------------------------------------------------------------
// Whole-network passes
// ----------------------------------------------------------------------------------------
void prepare(Model& m, int B) {
  if (m.B == B && !m.act.empty()) return;
  m.B = B;
  m.act.assign(m.tens.size(), {});
  m.gact.assign(m.tens.size(), {});
  for (size_t t = 0; t < m.tens.size(); ++t) {
    m.act[t].assign((size_t)B * m.tens[t].numel(), 0.0);
    m.gact[t].assign((size_t)B * m.tens[t].numel(), 0.0);
  }
  m.bn_mean.assign(m.ops.size(), {}); m.bn_rstd.assign(m.ops.size(), {});
  m.gtheta.assign((size_t)m.d, 0.0);
}

// x: pixels in [0,1], fp32 NHWC.  The network input is (x - mean_c) * (1/std_c), evaluated in
// fp32 with one rounding per operation, then stored (bf16 in storage-emulation mode).
void load_input(Model& m, const float* x, int B) {
  const Shape s = m.in_shape;
  double* a = m.act[0].data();
  int64_t rows = (int64_t)B * s.H * s.W;
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c) {
      float v = x[i * s.C + c];
      if (m.normalize) { float t = v - m.mean[c % 3]; v = t * m.inv_std[c % 3]; }
      a[i * s.C + c] = m.rb((double)v);
    }
}

void forward(Model& m, int B) {
  for (size_t i = 0; i < m.ops.size(); ++i) {
    const Op& op = m.ops[i];
    switch (op.kind) {
      case OP_CONV: conv_forward(m, op, B); break;
      case OP_BIASACT: biasact_forward(m, op, B); break;
      case OP_BNACT: bnact_forward(m, (int)i, B); break;
      case OP_MAXPOOL: maxpool_forward(m, op, B); break;
      case OP_GAP: gap_forward(m, op, B); break;
      case OP_FC: fc_forward(m, op, B); break;
    }
  }
}

// Softmax cross-entropy.  loss_n = logsumexp(z_n) - z_n[y_n];  d loss_n / d z = softmax - onehot.
// `scale` multiplies the logit gradient: 1 for the attack (sum of per-sample losses, so every
// sample sees its own loss gradient), 1/B for the outer step (batch mean).  Returns mean loss.
double ce_loss_and_grad(Model& m, const int32_t* y, int B, double scale) {
  int t = m.ops.back().out, nc = m.tens[t].C;
  const double* z = m.act[t].data();
  double* dz = m.gact[t].data();
  double total = 0.0;
  for (int n = 0; n < B; ++n) {
    const double* zn = z + (int64_t)n * nc;
    double mx = zn[0];
    for (int c = 1; c < nc; ++c) mx = std::max(mx, zn[c]);
    double se = 0.0;
    for (int c = 0; c < nc; ++c) se += std::exp(zn[c] - mx);
    double lse = mx + std::log(se);
    total += lse - zn[y[n]];
    for (int c = 0; c < nc; ++c)
      dz[(int64_t)n * nc + c] = (std::exp(zn[c] - lse) - (c == y[n] ? 1.0 : 0.0)) * scale;
  }
  std::fill(m.ghas.begin(), m.ghas.end(), 0);
  m.ghas[t] = 1;
  return total / B;
}

void backward(Model& m, int B, bool want_wgrad) {
  for (int i = (int)m.ops.size() - 1; i >= 0; --i) {
    const Op& op = m.ops[i];
    switch (op.kind) {
      case OP_CONV: conv_backward(m, op, B, want_wgrad); break;
      case OP_BIASACT: biasact_backward(m, op, B); break;
      case OP_BNACT: bnact_backward(m, i, B); break;
      case OP_MAXPOOL: maxpool_backward(m, op, B); break;
      case OP_GAP: gap_backward(m, op, B); break;
      case OP_FC: fc_backward(m, op, B); break;
    }
  }
}

// Gradient of the loss w.r.t. the pixels: chain rule through the affine normalisation.
void pixel_grad(const Model& m, int B, float* gx) {
  const Shape s = m.in_shape;
  const double* g0 = m.gact[0].data();
  int64_t rows = (int64_t)B * s.H * s.W;
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c)
      gx[i * s.C + c] = (float)(g0[i * s.C + c] * (m.normalize ? (double)m.inv_std[c % 3] : 1.0));
}

inline float clampf(float v, float lo, float hi) { return v < lo ? lo : (v > hi ? hi : v); }

// One projected sign-gradient step in fp32 (one rounding per operation):
//   delta <- Proj_[-eps,eps](delta + alpha * sign(G)), sign(0) = 0;
//   then delta is clipped to [-x, 1-x] so that x + delta stays a valid image.
void pgd_update(const float* x, const float* G, float* delta, int64_t N, float eps, float alpha) {
  for (int64_t i = 0; i < N; ++i) {
    float g = G[i];
    float step = g > 0.0f ? alpha : (g < 0.0f ? -alpha : 0.0f);
    float d = clampf(delta[i] + step, -eps, eps);
    float lo = -x[i], hi = 1.0f - x[i];
    d = clampf(d, lo, hi);
    delta[i] = d;
  }
}

void make_xadv(const float* x, const float* delta, float* xadv, int64_t N) {
  for (int64_t i = 0; i < N; ++i) xadv[i] = clampf(x[i] + delta[i], 0.0f, 1.0f);
}

}  // namespace

// ========================================================================================
// C interface (ctypes)
// ========================================================================================
extern "C" {

void* orc_model_create(int arch, int bf16_storage, int H, int W, int num_classes,
                       const float* mean, const float* stdv) {
  Model* m = new Model();
  m->arch = arch; m->emu = bf16_storage; m->classes = num_classes;
  m->in_shape = {H, W, 3};
  m->add_tensor(m->in_shape);
  if (mean && stdv) {
    m->normalize = true;
    for (int c = 0; c < 3; ++c) { m->mean[c] = mean[c]; m->inv_std[c] = 1.0f / stdv[c]; }
  }
  switch (arch) {
    case ARCH_TINYCNN: build_tinycnn(*m); break;
    case ARCH_RESNET18_CIFAR: build_resnet18_cifar(*m); break;
    case ARCH_WRN34_10: build_wrn(*m, 34, 10); break;
    case ARCH_RESNET50: build_resnet50(*m); break;
    case ARCH_PREACT_RESNET18: build_preact_resnet18(*m); break;
    case ARCH_WRN28_10: build_wrn(*m, 28, 10); break;
    case ARCH_TESTNET: build_testnet(*m); break;
    case ARCH_LINEAR: build_linear(*m); break;
    default: delete m; return nullptr;
  }
  m->theta.assign((size_t)m->d, 0.0);
  m->master.assign((size_t)m->d, 0.0);
  m->ghas.assign(m->tens.size(), 0);
  return m;
}

void orc_model_destroy(void* h) { delete (Model*)h; }
void orc_set_accum_jitter(void* h, double rel) { ((Model*)h)->jitter = rel; }
int64_t orc_num_params(void* h) { return ((Model*)h)->d; }
int orc_num_tensors(void* h) { return (int)((Model*)h)->ptab.size(); }
int orc_num_classes(void* h) { return ((Model*)h)->classes; }

// offsets[num_tensors+1], fan_in[num_tensors], kind[num_tensors]
void orc_tensor_table(void* h, int64_t* offsets, int32_t* fan_in, int32_t* kind) {
  Model* m = (Model*)h;
  for (size_t i = 0; i < m->ptab.size(); ++i) {
    offsets[i] = m->ptab[i].off;
    if (fan_in) fan_in[i] = m->ptab[i].fan_in;
    if (kind) kind[i] = m->ptab[i].kind;
  }
  offsets[m->ptab.size()] = m->d;
}

void orc_set_params(void* h, const float* flat) {
  Model* m = (Model*)h;
  for (const PTensor& p : m->ptab)
    for (int64_t i = p.off; i < p.off + p.numel; ++i) {
      m->master[i] = flat[i];
      bool stored_bf16 = (p.kind == 0 || p.kind == 4);
      m->theta[i] = stored_bf16 ? m->rb((double)flat[i]) : (double)flat[i];
    }
}

void orc_get_params(void* h, float* flat) {
  Model* m = (Model*)h;
  for (int64_t i = 0; i < m->d; ++i) flat[i] = (float)m->master[i];
}

// Forward + loss + backward at the given (already perturbed) pixels.
//   reduction: 0 = sum of per-sample losses (attack), 1 = batch mean (outer step).
//   Any of logits / gx / gtheta may be NULL.  Returns the mean loss.
double orc_loss_grad(void* h, const float* x, const int32_t* y, int B, int reduction,
                     float* logits, float* gx, float* gtheta) {
  Model* m = (Model*)h;
  prepare(*m, B);
  load_input(*m, x, B);
  forward(*m, B);
  int t = m->ops.back().out;
  if (logits) for (int64_t i = 0; i < (int64_t)B * m->classes; ++i) logits[i] = (float)m->act[t][i];
  double loss = ce_loss_and_grad(*m, y, B, reduction == 0 ? 1.0 : 1.0 / B);
  if (gx || gtheta) {
    backward(*m, B, gtheta != nullptr);
    if (gx) pixel_grad(*m, B, gx);
    if (gtheta) for (int64_t i = 0; i < m->d; ++i) gtheta[i] = (float)m->gtheta[i];
  }
  return loss;
}

// Same in fp64 end to end, for finite differences: parameters are read from `theta64`
// (not rounded), pixels from x64 are used as the network input as they are.
double orc_loss_f64(void* h, const double* theta64, const double* x64, const int32_t* y, int B,
                    int reduction, double* gx64, double* gtheta64) {
  Model* m = (Model*)h;
  int saved = m->emu; m->emu = 0;
  prepare(*m, B);
  std::vector<double> keep = m->theta;
  std::copy(theta64, theta64 + m->d, m->theta.begin());
  const Shape s = m->in_shape;
  int64_t rows = (int64_t)B * s.H * s.W;
  for (int64_t i = 0; i < rows; ++i)
    for (int c = 0; c < s.C; ++c) {
      double v = x64[i * s.C + c];
      if (m->normalize) v = (v - (double)m->mean[c]) * (double)m->inv_std[c];
      m->act[0][i * s.C + c] = v;
    }
  forward(*m, B);
  double loss = ce_loss_and_grad(*m, y, B, reduction == 0 ? 1.0 : 1.0 / B);
  if (reduction == 0) loss *= B;
  if (gx64 || gtheta64) {
    backward(*m, B, gtheta64 != nullptr);
    if (gx64)
      for (int64_t i = 0; i < rows; ++i)
        for (int c = 0; c < s.C; ++c)
          gx64[i * s.C + c] = m->gact[0][i * s.C + c] * (m->normalize ? (double)m->inv_std[c] : 1.0);
    if (gtheta64) std::copy(m->gtheta.begin(), m->gtheta.end(), gtheta64);
  }
  m->theta = keep; m->emu = saved;
  return loss;
}

}  // extern "C"

// ---- the general worker objective of Eq. (prob_DAT) ------------------------------------------------
//   F = (1/B) sum_n [ lambda * CE(z(x_n), y_n) + phi_n ],
//   phi = 0 (labeled data):  phi_n = CE(z(x_n + delta_n), y_n)
//   phi = 1 (TRADES regulariser, "DAT with unlabeled data"): phi_n = KL(p(x_n) || p(x_n + delta_n)),
//           p(.) = softmax of the logits; no label enters phi.
// Every network evaluation is its own train-mode forward pass (batch statistics of that pass).
// d phi_n / d z_adv = q - p;  d phi_n / d z_clean = p .* (log p - log q - phi_n)   (q = p(x+delta)).
namespace {

void softmax_rows(const std::vector<double>& z, int B, int nc, std::vector<double>& logp) {
  logp.resize(z.size());
  for (int n = 0; n < B; ++n) {
    const double* zn = z.data() + (int64_t)n * nc;
    double mx = zn[0];
    for (int c = 1; c < nc; ++c) mx = std::max(mx, zn[c]);
    double se = 0.0;
    for (int c = 0; c < nc; ++c) se += std::exp(zn[c] - mx);
    const double lse = mx + std::log(se);
    for (int c = 0; c < nc; ++c) logp[(int64_t)n * nc + c] = zn[c] - lse;
  }
}

void install_logit_grad(Model& m, const std::vector<double>& dz) {
  const int t = m.ops.back().out;
  std::copy(dz.begin(), dz.end(), m.gact[t].begin());
  std::fill(m.ghas.begin(), m.ghas.end(), 0);
  m.ghas[t] = 1;
}

std::vector<double> logits_of(const Model& m, int B) {
  const int t = m.ops.back().out;
  return std::vector<double>(m.act[t].begin(), m.act[t].begin() + (int64_t)B * m.classes);
}

// Logit gradients of sum_n scale * [ lambda * CE(z_clean_n, y_n) + KL(p(z_clean_n) || p(z_adv_n)) ] from the two
// passes' log-probabilities lp (clean) and lq (perturbed):
//   branch 0, d/dz_adv:   scale * (q - p)                       (the CE term does not depend on z_adv)
//   branch 1, d/dz_clean: scale * (lambda * (p - onehot(y)) + p .* (log p - log q - KL_n))
// kl[n] = KL_n.  y may be null when lambda is 0 or branch is 0.
void kl_logit_grad(const std::vector<double>& lp, const std::vector<double>& lq, const int32_t* y, int B, int nc, double lambda,
                   int branch, double scale, std::vector<double>& kl, std::vector<double>& dz) {
  kl.assign((size_t)B, 0.0);
  dz.resize((size_t)B * nc);
  for (int n = 0; n < B; ++n) {
    double s = 0.0;
    for (int c = 0; c < nc; ++c) { const int64_t i = (int64_t)n * nc + c; s += std::exp(lp[i]) * (lp[i] - lq[i]); }
    kl[n] = s;
  }
  if (branch == 0) {
    for (int64_t i = 0; i < (int64_t)B * nc; ++i) dz[i] = (std::exp(lq[i]) - std::exp(lp[i])) * scale;
    return;
  }
  for (int n = 0; n < B; ++n)
    for (int c = 0; c < nc; ++c) {
      const int64_t i = (int64_t)n * nc + c;
      const double pc = std::exp(lp[i]);
      const double ce = lambda != 0.0 ? lambda * (pc - (c == y[n] ? 1.0 : 0.0)) : 0.0;
      dz[i] = (ce + pc * (lp[i] - lq[i] - kl[n])) * scale;
    }
}

// The two network inputs are already in m's input format when `load` is null (fp64 entry).
struct RegResult { double loss_clean, loss_phi; };

// Core shared by the fp32 and the fp64 entry: `set_clean` / `set_adv` write the network input.
template <class SetClean, class SetAdv>
RegResult objective_and_grads(Model& m, int B, const int32_t* y, double lambda, int phi, bool want_gtheta, bool want_gadv,
                              SetClean set_clean, SetAdv set_adv, std::vector<double>& gtheta, std::vector<double>& gadv_in) {
  const int nc = m.classes;
  const double inv = 1.0 / B;
  RegResult r{0.0, 0.0};
  gtheta.assign(want_gtheta ? (size_t)m.d : 0, 0.0);
  auto add_gtheta = [&]() { for (int64_t i = 0; i < m.d; ++i) gtheta[i] += m.gtheta[i]; };
  if (phi == 0) {
    if (lambda != 0.0) {
      set_clean(); forward(m, B);
      r.loss_clean = ce_loss_and_grad(m, y, B, lambda * inv);
      if (want_gtheta) { backward(m, B, true); add_gtheta(); }
    }
    set_adv(); forward(m, B);
    r.loss_phi = ce_loss_and_grad(m, y, B, want_gadv && !want_gtheta ? 1.0 : inv);
    if (want_gtheta || want_gadv) {
      backward(m, B, want_gtheta);
      if (want_gtheta) add_gtheta();
      if (want_gadv) gadv_in = m.gact[0];
    }
    return r;
  }
  // TRADES: clean logits first
  set_clean(); forward(m, B);
  std::vector<double> lp, lq;
  softmax_rows(logits_of(m, B), B, nc, lp);
  set_adv(); forward(m, B);
  softmax_rows(logits_of(m, B), B, nc, lq);
  std::vector<double> kl, dz;
  // adversarial branch (activations of the x+delta pass are in place)
  const double sadv = (want_gadv && !want_gtheta) ? 1.0 : inv;   // the attack uses the sum over the batch
  kl_logit_grad(lp, lq, y, B, nc, lambda, 0, sadv, kl, dz);
  for (int n = 0; n < B; ++n) { r.loss_phi += kl[n] * inv; r.loss_clean += -lp[(int64_t)n * nc + y[n]] * inv; }
  if (want_gtheta || want_gadv) {
    install_logit_grad(m, dz);
    backward(m, B, want_gtheta);
    if (want_gtheta) add_gtheta();
    if (want_gadv) gadv_in = m.gact[0];
  }
  if (want_gtheta) {
    // clean branch: its activations were overwritten, run that pass again
    set_clean(); forward(m, B);
    kl_logit_grad(lp, lq, y, B, nc, lambda, 1, inv, kl, dz);
    install_logit_grad(m, dz);
    backward(m, B, true);
    add_gtheta();
  }
  return r;
}

}  // namespace

extern "C" {

// Worker gradient of the objective above at fp32 pixels x (clean) and xadv (= clip(x + delta)).
// grads: fp32 [d] (sum of the passes accumulated in fp64, rounded once).  losses[0] = mean clean CE
// (0 when lambda = 0 and phi = 0: that pass is not run), losses[1] = mean phi.
void orc_step_reg(void* h, const float* x, const float* xadv, const int32_t* y, int B, double lambda, int phi,
                  float* grads, double* losses) {
  Model* m = (Model*)h;
  prepare(*m, B);
  std::vector<double> gt, unused;
  RegResult r = objective_and_grads(*m, B, y, lambda, phi, true, false, [&]() { load_input(*m, x, B); },
                                    [&]() { load_input(*m, xadv, B); }, gt, unused);
  for (int64_t i = 0; i < m->d; ++i) grads[i] = (float)gt[i];
  if (losses) { losses[0] = r.loss_clean; losses[1] = r.loss_phi; }
}

// The logit gradients of the TRADES objective (kl_logit_grad above) from given fp32 logits of the two passes, for
// teacher-forced comparisons: dz fp32 [B][nc]; kl_mean = (1/B) sum_n KL_n.
void orc_kl_logit_grad(const float* z_clean, const float* z_adv, const int32_t* y, int B, int nc, double lambda, int branch,
                       double scale, float* dz, double* kl_mean) {
  std::vector<double> zc(z_clean, z_clean + (int64_t)B * nc), za(z_adv, z_adv + (int64_t)B * nc), lp, lq, kl, d;
  softmax_rows(zc, B, nc, lp);
  softmax_rows(za, B, nc, lq);
  kl_logit_grad(lp, lq, y, B, nc, lambda, branch, scale, kl, d);
  for (size_t i = 0; i < d.size(); ++i) dz[i] = (float)d[i];
  double s = 0.0;
  for (int n = 0; n < B; ++n) s += kl[n];
  if (kl_mean) *kl_mean = s / B;
}

// Gradient of sum_n phi_n w.r.t. the perturbed pixels (the clean pass is a constant): what the inner
// maximisation ascends.  gx: fp32 [B,H,W,3].  Returns mean phi.
double orc_phi_input_grad(void* h, const float* x, const float* xadv, const int32_t* y, int B, int phi, float* gx) {
  Model* m = (Model*)h;
  prepare(*m, B);
  std::vector<double> gt, gin;
  RegResult r = objective_and_grads(*m, B, y, 0.0, phi, false, true, [&]() { load_input(*m, x, B); },
                                    [&]() { load_input(*m, xadv, B); }, gt, gin);
  m->gact[0] = gin;
  pixel_grad(*m, B, gx);
  return r.loss_phi;
}

// fp64 end to end (parameters from theta64, pixels used as given, no storage rounding): returns
// F = lambda * mean CE + mean phi; optional gradients of F w.r.t. theta, and of sum_n phi_n w.r.t.
// xadv with the clean pass held constant.
double orc_objective_f64(void* h, const double* theta64, const double* x64, const double* xadv64, const int32_t* y, int B,
                         double lambda, int phi, double* gtheta64, double* gxadv64) {
  Model* m = (Model*)h;
  int saved = m->emu; m->emu = 0;
  prepare(*m, B);
  std::vector<double> keep = m->theta;
  std::copy(theta64, theta64 + m->d, m->theta.begin());
  const Shape s = m->in_shape;
  const int64_t rows = (int64_t)B * s.H * s.W;
  auto put = [&](const double* src) {
    for (int64_t i = 0; i < rows; ++i)
      for (int c = 0; c < s.C; ++c) {
        double v = src[i * s.C + c];
        if (m->normalize) v = (v - (double)m->mean[c]) * (double)m->inv_std[c];
        m->act[0][i * s.C + c] = v;
      }
  };
  std::vector<double> gt, gin;
  double F = 0.0;
  if (gxadv64) {
    RegResult r = objective_and_grads(*m, B, y, 0.0, phi, false, true, [&]() { put(x64); }, [&]() { put(xadv64); }, gt, gin);
    (void)r;
    for (int64_t i = 0; i < rows; ++i)
      for (int c = 0; c < s.C; ++c)
        gxadv64[i * s.C + c] = gin[i * s.C + c] * (m->normalize ? (double)m->inv_std[c] : 1.0);
  }
  {
    RegResult r = objective_and_grads(*m, B, y, lambda, phi, gtheta64 != nullptr, false, [&]() { put(x64); },
                                      [&]() { put(xadv64); }, gt, gin);
    F = lambda * r.loss_clean + r.loss_phi;   // loss_clean is 0 when that pass is not part of the objective
    if (gtheta64) std::copy(gt.begin(), gt.end(), gtheta64);
  }
  m->theta = keep; m->emu = saved;
  return F;
}

// Inner maximisation of phi = KL(p(x) || p(x + delta)) by the same projected sign ascent as orc_attack
// (no labels).  The clean logits are those of one forward pass on x and stay fixed.
void orc_attack_kl(void* h, const float* x, int B, float eps, float alpha, int K, int init_mode, uint64_t seed,
                   const float* delta0, float* delta, float* loss_per_step, float* delta_trace);

// delta0 for the three init modes: 0 zero, 1 uniform in the eps-ball from Philox stream 1
// (u -> (2u-1)*eps), 2 given.  Always followed by the clip that keeps x+delta in [0,1].
void orc_init_delta(const float* x, int64_t N, float eps, int mode, uint64_t seed,
                    const float* given, float* delta) {
  for (int64_t i = 0; i < N; ++i) {
    float d = 0.0f;
    if (mode == 1) { float u = uniform_at((uint64_t)i, seed, STREAM_INIT); float t = 2.0f * u - 1.0f; d = t * eps; }
    else if (mode == 2) d = clampf(given[i], -eps, eps);
    d = clampf(d, -x[i], 1.0f - x[i]);
    delta[i] = d;
  }
}

void orc_pgd_update(const float* x, const float* G, float* delta, int64_t N, float eps, float alpha) {
  pgd_update(x, G, delta, N, eps, alpha);
}

void orc_make_xadv(const float* x, const float* delta, float* xadv, int64_t N) { make_xadv(x, delta, xadv, N); }

// K-step attack for one batch.  Optional traces for teacher-forced comparisons:
//   loss_per_step[K+1]: mean CE at delta_0..delta_K;  delta_trace[(K+1)*N];  grad_trace[K*N].
void orc_attack(void* h, const float* x, const int32_t* y, int B, float eps, float alpha, int K,
                int init_mode, uint64_t seed, const float* delta0, float* delta,
                float* loss_per_step, float* delta_trace, float* grad_trace) {
  Model* m = (Model*)h;
  int64_t N = (int64_t)B * m->in_shape.numel();
  std::vector<float> xadv((size_t)N), G((size_t)N);
  orc_init_delta(x, N, eps, init_mode, seed, delta0, delta);
  if (delta_trace) std::copy(delta, delta + N, delta_trace);
  for (int k = 0; k < K; ++k) {
    make_xadv(x, delta, xadv.data(), N);
    double loss = orc_loss_grad(h, xadv.data(), y, B, 0, nullptr, G.data(), nullptr);
    if (loss_per_step) loss_per_step[k] = (float)loss;
    if (grad_trace) std::copy(G.begin(), G.end(), grad_trace + (int64_t)k * N);
    pgd_update(x, G.data(), delta, N, eps, alpha);
    if (delta_trace) std::copy(delta, delta + N, delta_trace + (int64_t)(k + 1) * N);
  }
  if (loss_per_step) {
    make_xadv(x, delta, xadv.data(), N);
    loss_per_step[K] = (float)orc_loss_grad(h, xadv.data(), y, B, 0, nullptr, nullptr, nullptr);
  }
}

// Outer step: g = (1/B) sum_n grad_theta CE(net(x_adv_n), y_n).
double orc_step(void* h, const float* xadv, const int32_t* y, int B, float* grads) {
  return orc_loss_grad(h, xadv, y, B, 1, nullptr, nullptr, grads);
}

void orc_attack_kl(void* h, const float* x, int B, float eps, float alpha, int K, int init_mode, uint64_t seed,
                   const float* delta0, float* delta, float* loss_per_step, float* delta_trace) {
  Model* m = (Model*)h;
  const int64_t N = (int64_t)B * m->in_shape.numel();
  std::vector<float> xadv((size_t)N), G((size_t)N);
  std::vector<int32_t> nolabel((size_t)B, 0);
  orc_init_delta(x, N, eps, init_mode, seed, delta0, delta);
  if (delta_trace) std::copy(delta, delta + N, delta_trace);
  for (int k = 0; k < K; ++k) {
    make_xadv(x, delta, xadv.data(), N);
    const double loss = orc_phi_input_grad(h, x, xadv.data(), nolabel.data(), B, 1, G.data());
    if (loss_per_step) loss_per_step[k] = (float)loss;
    pgd_update(x, G.data(), delta, N, eps, alpha);
    if (delta_trace) std::copy(delta, delta + N, delta_trace + (int64_t)(k + 1) * N);
  }
  if (loss_per_step) {
    make_xadv(x, delta, xadv.data(), N);
    loss_per_step[K] = (float)orc_phi_input_grad(h, x, xadv.data(), nolabel.data(), B, 1, G.data());
  }
}

void orc_sgd_update(void* h, const float* grads, float lr) {
  Model* m = (Model*)h;
  std::vector<float> p((size_t)m->d);
  for (int64_t i = 0; i < m->d; ++i) { float t = lr * grads[i]; p[i] = (float)m->master[i] - t; }
  orc_set_params(h, p.data());
}

// ----------------------------------------------------------------------------------------
// Randomized quantizer (appendix "Additional details on gradient quantization").
// Per tensor t: scale = max|g| (use_l2 = 0) or ||g||_2 (use_l2 = 1, the paper's literal
// choice); S levels per sign.  r = |g_i| * (S/scale); l = floor(r); the code magnitude is l
// with probability 1-(r-l) and l+1 with probability r-l (Eq. (xi) with s = S); the sign is
// carried by the code.  codes are int32 here; packing is a separate, trivial step.
// ----------------------------------------------------------------------------------------
void orc_quantize(const float* g, const int64_t* offsets, int num_tensors, int S, uint64_t seed,
                  int use_l2, int32_t* codes, float* scales) {
  for (int t = 0; t < num_tensors; ++t) {
    int64_t lo = offsets[t], hi = offsets[t + 1];
    float scale = 0.0f;
    if (use_l2) {
      double ss = 0.0;
      for (int64_t i = lo; i < hi; ++i) ss += (double)g[i] * (double)g[i];
      scale = (float)std::sqrt(ss);
    } else {
      for (int64_t i = lo; i < hi; ++i) scale = std::max(scale, std::fabs(g[i]));
    }
    scales[t] = scale;
    if (!(scale > 0.0f)) { for (int64_t i = lo; i < hi; ++i) codes[i] = 0; continue; }
    float inv = (float)S / scale;
    for (int64_t i = lo; i < hi; ++i) {
      float r = std::fabs(g[i]) * inv;
      float l = std::floor(r);
      float p = r - l;
      float u = uniform_at((uint64_t)i, seed, STREAM_QUANT);
      float mag = l + (u < p ? 1.0f : 0.0f);
      if (mag > (float)S) mag = (float)S;
      int32_t c = (int32_t)mag;
      codes[i] = g[i] < 0.0f ? -c : c;
    }
  }
}

void orc_dequantize(const int32_t* codes, const float* scales, const int64_t* offsets,
                    int num_tensors, int S, float* out) {
  for (int t = 0; t < num_tensors; ++t) {
    float step = scales[t] / (float)S;
    for (int64_t i = offsets[t]; i < offsets[t + 1]; ++i) out[i] = (float)codes[i] * step;
  }
}

// Wire packing: `bits`-bit two's-complement fields, little-endian: element i occupies bits
// [(i*bits) mod 8, ...) of byte floor(i*bits/8) (for bits = 4: element 2j in the low nibble of
// byte j; for bits = 16: low byte first).  bits in {2, 4, 8, 16}.
void orc_pack(const int32_t* codes, int64_t d, int bits, uint8_t* q) {
  int64_t nbytes = (d * bits + 7) / 8;
  for (int64_t j = 0; j < nbytes; ++j) q[j] = 0;
  for (int64_t i = 0; i < d; ++i) {
    uint32_t field = (uint32_t)codes[i] & ((1u << bits) - 1u);
    for (int b = 0; b < bits; ++b) {
      int64_t pos = i * bits + b;
      if ((field >> b) & 1u) q[pos / 8] |= (uint8_t)(1u << (pos % 8));
    }
  }
}

void orc_unpack(const uint8_t* q, int64_t d, int bits, int32_t* codes) {
  for (int64_t i = 0; i < d; ++i) {
    uint32_t field = 0;
    for (int b = 0; b < bits; ++b) {
      int64_t pos = i * bits + b;
      if ((q[pos / 8] >> (pos % 8)) & 1u) field |= 1u << b;
    }
    int32_t v = (int32_t)field;
    if (field & (1u << (bits - 1))) v -= (int32_t)(1u << bits);
    codes[i] = v;
  }
}

// ----------------------------------------------------------------------------------------
// Outer-minimisation oracle A(.): layer-wise adaptive learning rate, Eq. (3), with the descent
// direction u of LAMB, Alg. A2 (use_adam = 1), or u = g (use_adam = 0).  "Layer" = one tensor
// of the table.  Per element (Alg. A2): m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
// u = (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + zeta) [+ wd*theta: decoupled weight decay as in the
// cited LAMB; wd = 0 gives the listing as printed].  Per layer i (Eq. (3)):
//   theta_i <- theta_i - eta * tau(||theta_i||_2) / ||u_i||_2 * u_i,  tau(x) = min(max(x, c_l), c_u);
// a layer with ||u_i|| = 0 is left unchanged.  fp64 arithmetic on fp32 state.
void orc_lamb_update(float* theta, float* m, float* v, const float* g, const int64_t* offsets, int num_tensors,
                     int use_adam, double eta, double b1, double b2, double zeta, double wd, double c_l, double c_u,
                     int t) {
  const double bc1 = 1.0 - std::pow(b1, t), bc2 = 1.0 - std::pow(b2, t);
  for (int i = 0; i < num_tensors; ++i) {
    const int64_t lo = offsets[i], hi = offsets[i + 1];
    std::vector<double> u((size_t)(hi - lo));
    double nth = 0.0, nu = 0.0;
    for (int64_t e = lo; e < hi; ++e) {
      double ue;
      if (use_adam) {
        const double mm = b1 * (double)m[e] + (1.0 - b1) * (double)g[e];
        const double vv = b2 * (double)v[e] + (1.0 - b2) * (double)g[e] * (double)g[e];
        m[e] = (float)mm; v[e] = (float)vv;
        ue = ((double)m[e] / bc1) / (std::sqrt((double)v[e] / bc2) + zeta);
      } else {
        ue = (double)g[e];
      }
      ue += wd * (double)theta[e];
      u[(size_t)(e - lo)] = ue;
      nth += (double)theta[e] * (double)theta[e];
      nu += ue * ue;
    }
    nth = std::sqrt(nth); nu = std::sqrt(nu);
    if (!(nu > 0.0)) continue;
    const double tau = std::min(std::max(nth, c_l), c_u);
    const double rate = eta * tau / nu;
    for (int64_t e = lo; e < hi; ++e) theta[e] = (float)((double)theta[e] - rate * u[(size_t)(e - lo)]);
  }
}

// Server block, Eq. (grad_agg): g_hat = (1/M) sum_i Q(g^(i)), from M workers' codes and scales.
// fp32, one rounding per operation, workers added in index order:  acc = acc + code*step_i; out = acc / M.
void orc_aggregate(const int32_t* const* codes, const float* const* scales, int M, const int64_t* offsets,
                   int num_tensors, int S, float* out) {
  for (int t = 0; t < num_tensors; ++t)
    for (int64_t e = offsets[t]; e < offsets[t + 1]; ++e) {
      float acc = 0.0f;
      for (int i = 0; i < M; ++i) {
        const float step = scales[i][t] / (float)S;
        const float term = (float)codes[i][e] * step;
        acc = acc + term;
      }
      out[e] = acc / (float)M;
    }
}

void orc_philox(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
  U4 c; std::memcpy(c.v, ctr, 16);
  U4 r = philox4x32_10(c, key[0], key[1]);
  std::memcpy(out, r.v, 16);
}

void orc_uniform(uint64_t start, int64_t n, uint64_t seed, uint32_t stream, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = uniform_at(start + (uint64_t)i, seed, stream);
}

double orc_round_bf16(double v) { return round_bf16(v); }

// Single-layer entry points for adjoint / definition tests: a one-conv "model" on the fly.
void orc_conv_forward(const double* in, const double* W, double* out, int B, int H, int Wd, int Ci,
                      int Co, int k, int stride, int pad) {
  Model m; m.classes = 1; m.in_shape = {H, Wd, Ci}; m.add_tensor(m.in_shape);
  m.conv(0, Co, k, stride, pad);
  m.theta.assign(W, W + m.d); m.ghas.assign(m.tens.size(), 0);
  prepare(m, B);
  std::copy(in, in + (int64_t)B * m.in_shape.numel(), m.act[0].begin());
  conv_forward(m, m.ops[0], B);
  std::copy(m.act[1].begin(), m.act[1].end(), out);
}

void orc_conv_backward(const double* in, const double* W, const double* dout, double* din, double* dW,
                       int B, int H, int Wd, int Ci, int Co, int k, int stride, int pad) {
  Model m; m.classes = 1; m.in_shape = {H, Wd, Ci}; m.add_tensor(m.in_shape);
  m.conv(0, Co, k, stride, pad);
  m.theta.assign(W, W + m.d); m.ghas.assign(m.tens.size(), 0);
  prepare(m, B);
  std::copy(in, in + (int64_t)B * m.in_shape.numel(), m.act[0].begin());
  std::copy(dout, dout + (int64_t)B * m.tens[1].numel(), m.gact[1].begin());
  m.ghas[1] = 1;
  conv_backward(m, m.ops[0], B, true);
  std::copy(m.gact[0].begin(), m.gact[0].end(), din);
  std::copy(m.gtheta.begin(), m.gtheta.end(), dW);
}

// Single output elements of the three convolution contractions, straight from the definitions
// (fp32 inputs, fp64 sums), for spot checks on tensors too large to convolve whole.
//   forward:  idx = flat index into y[B][Ho][Wo][Co]
//   bwd data: idx = flat index into dx[B][H][W][Ci]
//   bwd weight: idx = flat index into dw[Co][k][k][Ci]
void orc_conv_forward_points(const float* x, const float* w, int B, int H, int Wd, int Ci, int Co, int k,
                             int stride, int pad, const int64_t* idx, int n, double* out) {
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
  (void)B;
  for (int q = 0; q < n; ++q) {
    int64_t p = idx[q];
    const int co = (int)(p % Co); p /= Co;
    const int wo = (int)(p % Wo); p /= Wo;
    const int ho = (int)(p % Ho); const int64_t b = p / Ho;
    double acc = 0.0;
    for (int r = 0; r < k; ++r) for (int s = 0; s < k; ++s) {
      const int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
      if (hi < 0 || hi >= H || wi < 0 || wi >= Wd) continue;
      for (int ci = 0; ci < Ci; ++ci)
        acc += (double)x[((b * H + hi) * Wd + wi) * Ci + ci] * (double)w[(((int64_t)co * k + r) * k + s) * Ci + ci];
    }
    out[q] = acc;
  }
}

void orc_conv_bwd_data_points(const float* dy, const float* w, int B, int H, int Wd, int Ci, int Co, int k,
                              int stride, int pad, const int64_t* idx, int n, double* out) {
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
  (void)B;
  for (int q = 0; q < n; ++q) {
    int64_t p = idx[q];
    const int ci = (int)(p % Ci); p /= Ci;
    const int wi = (int)(p % Wd); p /= Wd;
    const int hi = (int)(p % H); const int64_t b = p / H;
    double acc = 0.0;
    for (int ho = 0; ho < Ho; ++ho) for (int wo = 0; wo < Wo; ++wo) {
      const int r = hi - ho * stride + pad, s = wi - wo * stride + pad;   // tap that connects (ho,wo) to (hi,wi)
      if (r < 0 || r >= k || s < 0 || s >= k) continue;
      for (int co = 0; co < Co; ++co)
        acc += (double)dy[((b * Ho + ho) * Wo + wo) * Co + co] * (double)w[(((int64_t)co * k + r) * k + s) * Ci + ci];
    }
    out[q] = acc;
  }
}

void orc_conv_bwd_weight_points(const float* x, const float* dy, int B, int H, int Wd, int Ci, int Co, int k,
                                int stride, int pad, const int64_t* idx, int n, double* out) {
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
#pragma omp parallel for schedule(dynamic, 1)
  for (int q = 0; q < n; ++q) {
    int64_t p = idx[q];
    const int ci = (int)(p % Ci); p /= Ci;
    const int s = (int)(p % k); p /= k;
    const int r = (int)(p % k); const int co = (int)(p / k);
    double acc = 0.0;
    for (int64_t b = 0; b < B; ++b) for (int ho = 0; ho < Ho; ++ho) for (int wo = 0; wo < Wo; ++wo) {
      const int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
      if (hi < 0 || hi >= H || wi < 0 || wi >= Wd) continue;
      acc += (double)dy[((b * Ho + ho) * Wo + wo) * Co + co] * (double)x[((b * H + hi) * Wd + wi) * Ci + ci];
    }
    out[q] = acc;
  }
}

// ----------------------------------------------------------------------------------------
// Op-by-op stepping, for teacher-forced comparisons of another implementation's stored
// tensors with this reference.  Nothing below does arithmetic of the method: it runs the
// layer functions above one op at a time, copies tensors in and out, and counts differences.
//   which: 0 = activation tensors, 1 = their gradients.
// ----------------------------------------------------------------------------------------
int orc_num_ops(void* h) { return (int)((Model*)h)->ops.size(); }
int orc_num_act_tensors(void* h) { return (int)((Model*)h)->tens.size(); }

// info[10] = kind (0 conv, 1 bias+act, 2 BN+act, 3 max-pool, 4 global pool, 5 linear), in, out, res,
//            k, stride, pad, relu, p0, p1
void orc_op_info(void* h, int i, int32_t* info) {
  const Op& op = ((Model*)h)->ops[(size_t)i];
  const int32_t v[10] = {(int32_t)op.kind, op.in, op.out, op.res, op.k, op.stride, op.pad, op.relu, op.p0, op.p1};
  std::copy(v, v + 10, info);
}

void orc_tensor_shape(void* h, int t, int32_t* hwc) {
  const Shape s = ((Model*)h)->tens[(size_t)t];
  hwc[0] = s.H; hwc[1] = s.W; hwc[2] = s.C;
}

// Allocates the per-call state for batch B and loads the network input from pixels x.
void orc_begin(void* h, const float* x, int B) {
  Model* m = (Model*)h;
  prepare(*m, B);
  load_input(*m, x, B);
  std::fill(m->ghas.begin(), m->ghas.end(), 0);
}

void orc_forward_op(void* h, int i) {
  Model* m = (Model*)h;
  const Op& op = m->ops[(size_t)i];
  switch (op.kind) {
    case OP_CONV: conv_forward(*m, op, m->B); break;
    case OP_BIASACT: biasact_forward(*m, op, m->B); break;
    case OP_BNACT: bnact_forward(*m, i, m->B); break;
    case OP_MAXPOOL: maxpool_forward(*m, op, m->B); break;
    case OP_GAP: gap_forward(*m, op, m->B); break;
    case OP_FC: fc_forward(*m, op, m->B); break;
  }
}

// Installs the logit gradient of the cross-entropy (scale 1: sum over the batch, 1/B: mean) and
// clears every other gradient slot.  Returns the mean loss.
double orc_loss_backward_begin(void* h, const int32_t* y, double scale) {
  Model* m = (Model*)h;
  return ce_loss_and_grad(*m, y, m->B, scale);
}

void orc_backward_op(void* h, int i, int want_wgrad) {
  Model* m = (Model*)h;
  const Op& op = m->ops[(size_t)i];
  switch (op.kind) {
    case OP_CONV: conv_backward(*m, op, m->B, want_wgrad != 0); break;
    case OP_BIASACT: biasact_backward(*m, op, m->B); break;
    case OP_BNACT: bnact_backward(*m, i, m->B); break;
    case OP_MAXPOOL: maxpool_backward(*m, op, m->B); break;
    case OP_GAP: gap_backward(*m, op, m->B); break;
    case OP_FC: fc_backward(*m, op, m->B); break;
  }
}

int orc_grad_present(void* h, int t) { return ((Model*)h)->ghas[(size_t)t]; }

static std::vector<double>& tensor_of(Model* m, int which, int t) { return which ? m->gact[(size_t)t] : m->act[(size_t)t]; }

static inline double bf16_bits_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16; float f; std::memcpy(&f, &u, 4); return (double)f;
}

void orc_get_tensor(void* h, int which, int t, float* out) {
  Model* m = (Model*)h;
  const std::vector<double>& v = tensor_of(m, which, t);
  const int64_t n = (int64_t)m->B * m->tens[(size_t)t].numel();
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) out[i] = (float)v[(size_t)i];
}

// src: fp32 values (is_bf16 = 0) or bf16 bit patterns (is_bf16 = 1), B * numel(t) of them.
void orc_set_tensor(void* h, int which, int t, const void* src, int is_bf16) {
  Model* m = (Model*)h;
  std::vector<double>& v = tensor_of(m, which, t);
  const int64_t n = (int64_t)m->B * m->tens[(size_t)t].numel();
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i)
    v[(size_t)i] = is_bf16 ? bf16_bits_to_double(((const uint16_t*)src)[i]) : (double)((const float*)src)[i];
  if (which) m->ghas[(size_t)t] = 1;
}

// Element-by-element comparison of `got` (fp32 values or bf16 bit patterns) with tensor t:
// an element violates when |got - ref| > rel*|ref| + abs_frac*max|ref| (max over the tensor).
// stats[8] = { count, exactly equal, violations, max |got-ref| / tolerance, max|ref|, max|got-ref|,
//              non-finite values in got, index of the worst element }.
void orc_compare_tensor(void* h, int which, int t, const void* got, int is_bf16, double rel, double abs_frac, double* stats) {
  Model* m = (Model*)h;
  const std::vector<double>& v = tensor_of(m, which, t);
  const int64_t n = (int64_t)m->B * m->tens[(size_t)t].numel();
  double mx = 0.0;
#pragma omp parallel for schedule(static) reduction(max : mx)
  for (int64_t i = 0; i < n; ++i) mx = std::max(mx, std::fabs(v[(size_t)i]));
  int64_t exact = 0, viol = 0, bad = 0;
  double worst = 0.0, maxerr = 0.0; int64_t worst_i = -1;
#pragma omp parallel
  {
    int64_t le = 0, lv = 0, lb = 0; double lw = 0.0, lm = 0.0; int64_t li = -1;
#pragma omp for schedule(static) nowait
    for (int64_t i = 0; i < n; ++i) {
      const double g = is_bf16 ? bf16_bits_to_double(((const uint16_t*)got)[i]) : (double)((const float*)got)[i];
      const double r = v[(size_t)i];
      if (!(g == g) || std::isinf(g)) { ++lb; ++lv; continue; }
      const double e = std::fabs(g - r), tol = rel * std::fabs(r) + abs_frac * mx;
      if (e == 0.0) { ++le; continue; }
      if (e > tol) ++lv;
      const double ratio = tol > 0.0 ? e / tol : INFINITY;
      if (ratio > lw) { lw = ratio; li = i; }
      lm = std::max(lm, e);
    }
#pragma omp critical
    {
      exact += le; viol += lv; bad += lb; maxerr = std::max(maxerr, lm);
      if (lw > worst) { worst = lw; worst_i = li; }
    }
  }
  stats[0] = (double)n; stats[1] = (double)exact; stats[2] = (double)viol; stats[3] = worst;
  stats[4] = mx; stats[5] = maxerr; stats[6] = (double)bad; stats[7] = (double)worst_i;
}

// Batch statistics of BN op i from the last forward pass over it; parameter gradients accumulated so far.
void orc_get_bn_stats(void* h, int i, double* mean, double* rstd) {
  Model* m = (Model*)h;
  std::copy(m->bn_mean[(size_t)i].begin(), m->bn_mean[(size_t)i].end(), mean);
  std::copy(m->bn_rstd[(size_t)i].begin(), m->bn_rstd[(size_t)i].end(), rstd);
}

void orc_get_param_grads(void* h, double* out) {
  Model* m = (Model*)h;
  std::copy(m->gtheta.begin(), m->gtheta.end(), out);
}

void orc_pixel_grad(void* h, float* gx) { Model* m = (Model*)h; pixel_grad(*m, m->B, gx); }

int orc_threads() {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
