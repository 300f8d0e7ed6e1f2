/* dat.h -- C ABI of libdat: one worker's step of distributed adversarial training (DAT) on one
 * AMD MI355X (gfx950).
 *
 * The calls follow Algorithm A1 of Liu et al., "Distributed Adversarial Training to Robustify
 * Deep Neural Networks at Scale" (UAI 2022), worker block (steps 4-7):
 *   dat_attack      step 5, Eq. (inner_max_alg): per-sample inner maximisation under an l-inf ball
 *                   by K projected sign-gradient steps (K = 1: FGSM, K > 1: PGD; the unified
 *                   update of Sec. "Methodologies", paragraph on inner maximisation);
 *   dat_step        step 6, Eq. (stoch_grad_batch) with lambda = 0 and phi = cross-entropy:
 *                   batch-mean gradient w.r.t. the parameters at the perturbed samples;
 *   dat_quantize    step 7: randomized b-bit quantizer Q, Eqs. (rand_q) and (xi) of appendix
 *                   "Additional details on gradient quantization";
 *   dat_dequantize  the map back to fp32 that the aggregation of Eq. (grad_agg) applies.
 *
 * Conventions
 *   - Every call returns a dat_status, never throws or aborts; on an argument error nothing
 *     is launched and outputs are untouched.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The model object owns its parameters and workspace (allocated at
 *     dat_model_create for `max_batch`), freed by dat_model_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work on it and return without synchronising unless a host output (`loss`,
 *     `loss_per_step`) is requested; host outputs are written after an internal
 *     hipStreamSynchronize.
 *   - Images are NHWC fp32 with C = 3 and pixel values in [0,1]; eps, alpha, delta and the
 *     [0,1] clip live in pixel space.  A model created with mean/std applies
 *     (x - mean_c) * (1/std_c) as its first operation.
 *   - Parameters and gradients are one flat fp32 vector in tensor-table order (op order; conv:
 *     W[Cout][kh][kw][Cin] (then bias); batch-norm: gamma, beta; linear: W[out][in], b).
 *   - A DAT_BF16 model stores conv/linear weights, activations and activation gradients in
 *     bf16 and accumulates in fp32 on the matrix cores; a DAT_F32 model keeps everything in
 *     fp32.  Batch-norm runs in train mode (batch statistics) in every pass.
 *   - Non-finite values.  Device data is never inspected by the host, so a call without a host output cannot
 *     report them: a NaN input gradient counts as sign 0 (that coordinate of delta stays), a NaN or infinite
 *     per-tensor scale is written to scales[t] and that tensor's codes are zero.  A call asked for a host loss
 *     synchronises anyway and returns DAT_ERR_NONFINITE when a loss it fetched is NaN or infinite; its device
 *     outputs have been written by then (the one exception to "outputs untouched on error").
 *   - Calls on one model, or sharing one stream's buffers, must not overlap in time.
 */
#ifndef DAT_H
#define DAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dat_model dat_model;

typedef enum {
  DAT_OK = 0,
  DAT_ERR_ARG = 1,         /* null pointer, negative size, bad enum, misaligned buffer */
  DAT_ERR_SHAPE = 2,       /* batch larger than max_batch, unsupported image size       */
  DAT_ERR_NOMEM = 3,       /* device or host allocation failed                           */
  DAT_ERR_NONFINITE = 4,   /* a requested host loss value was NaN or Inf (see Conventions) */
  DAT_ERR_HIP = 5,         /* a HIP runtime call failed (see dat_last_error)             */
  DAT_ERR_UNSUPPORTED = 6  /* valid request that this build does not implement           */
} dat_status;

typedef enum {
  DAT_ARCH_TINYCNN = 0,         /* conv3x3(3-16)+b+ReLU, conv3x3(16-32,s2)+b+ReLU, GAP, FC        */
  DAT_ARCH_RESNET18_CIFAR = 1,  /* post-activation BasicBlocks [2,2,2,2], widths 64..512          */
  DAT_ARCH_WRN34_10 = 2,        /* pre-activation wide blocks, widths 160/320/640                 */
  DAT_ARCH_RESNET50 = 3,        /* Bottleneck [3,4,6,3], stride on the 3x3, 7x7 stem + max-pool   */
  DAT_ARCH_PREACT_RESNET18 = 4, /* pre-activation BasicBlocks [2,2,2,2], widths 64..512 (the      */
                                /* paper's CIFAR "ResNet-18", Sec. "Experiment setup")            */
  DAT_ARCH_WRN28_10 = 5,        /* pre-activation wide blocks, 4 per group (semi-supervised runs) */
  DAT_ARCH_TESTNET = 100        /* small net containing every op kind (for parity tests)          */
} dat_arch;

typedef enum { DAT_F32 = 0, DAT_BF16 = 1 } dat_dtype;

typedef enum { DAT_INIT_ZERO = 0, DAT_INIT_UNIFORM = 1, DAT_INIT_GIVEN = 2 } dat_init_mode;

/* Start point z_0 of the inner maximisation.  UNIFORM: i.i.d. U(-eps,eps) from Philox4x32-10
 * (counter = flat element index / 4, stream 1, key = seed).  GIVEN: `delta0` (device,
 * [B,H,W,3]) projected onto the eps-ball.  In all modes z_0 is then clipped to [-x, 1-x]. */
typedef struct {
  dat_init_mode mode;
  uint64_t seed;
  const float* delta0;
} dat_init;

/* ---- model ------------------------------------------------------------------------------ */

/* Builds `arch` for H x W x 3 inputs and `num_classes` outputs, allocates parameters (zero)
 * and a workspace for batches up to `max_batch` on the current device.  mean/stdv: host,
 * 3 floats each, or both NULL for no normalisation. */
dat_status dat_model_create(dat_arch arch, dat_dtype dtype, int max_batch, int H, int W,
                            int num_classes, const float* mean, const float* stdv,
                            dat_model** out);
dat_status dat_model_destroy(dat_model* m);

/* d = total parameter count, num_tensors = entries of the tensor table. */
dat_status dat_model_num_params(const dat_model* m, int64_t* d, int* num_tensors);

/* Host outputs: offsets[num_tensors+1] (element offsets into the flat vector), and optionally
 * fan_in[num_tensors], kind[num_tensors] (0 conv W, 1 conv bias, 2 BN gamma, 3 BN beta,
 * 4 linear W, 5 linear b, 6 gamma of the last BN of a residual branch).  The model also keeps a device copy of `offsets`, returned by
 * dat_model_offsets_device (int64, num_tensors+1 entries, owned by the model). */
dat_status dat_model_tensor_table(const dat_model* m, int64_t* offsets, int32_t* fan_in,
                                  int32_t* kind);
const int64_t* dat_model_offsets_device(const dat_model* m);

/* Flat fp32 parameter vector, host memory, d elements.  set: uploads and (bf16 models) rounds
 * conv/linear weights to nearest-even bf16 for the compute copy; synchronous. */
dat_status dat_model_set_params(dat_model* m, const float* host_flat);
dat_status dat_model_get_params(const dat_model* m, float* host_flat);

/* ---- the worker step --------------------------------------------------------------------- */

/* Inner maximisation (Alg. A1 step 5).  x, delta: device fp32 [B,H,W,3]; y: device int32 [B].
 *   z_0 per `init`;  for k = 1..K:  G = grad_x sum_n CE(net(x + z_{k-1}), y)
 *     z_k = clip(z_{k-1} + alpha*sign(G), -eps, eps), sign(0) = 0;  z_k = min(max(z_k, -x), 1-x)
 *   delta = z_K (K = 0 returns z_0).  loss_per_step: optional host array of K+1 floats, mean CE
 *   at z_0..z_K (costs one extra forward and a synchronisation).
 *   A label outside [0, num_classes) is not an error the host can see (labels are device memory): that sample
 *   gets a NaN loss and a logit gradient without the one-hot term, in every call that takes labels.
 *   DAT_INIT_GIVEN: delta0 must be 16-byte aligned like x and delta. */
dat_status dat_attack(dat_model* m, const float* x, const int32_t* y, int B, float eps,
                      float alpha, int K, dat_init init, float* delta, float* loss_per_step,
                      void* stream);

/* Outer gradient (Alg. A1 step 6): grads[d] (device fp32, tensor-table order) =
 * (1/B) sum_n grad_theta CE(net(x_adv_n), y_n).  x_adv: device fp32 [B,H,W,3] pixels (already
 * perturbed).  loss: optional host float, mean CE. */
dat_status dat_step(dat_model* m, const float* x_adv, const int32_t* y, int B, float* grads,
                    float* loss, void* stream);

/* The quantizer's per-tensor scales of the gradient dat_step has just written, max_i |g_i| for every tensor of the
 * table (Eq. (rand_q): the norm that scales the vector before rounding; per-tensor abs-max here): every kernel
 * that writes a parameter gradient also raises that tensor's maximum (compared through the bit pattern of |g|,
 * so the value is exact, independent of order, and a NaN or Inf surfaces as in dat_quantize), which saves the
 * quantizer's own pass over the gradient.  *scales_dev: device fp32 [num_tensors], owned by the model,
 * overwritten by the next dat_step; valid for work enqueued after dat_step on the same stream.
 * DAT_ERR_UNSUPPORTED when the last call on the model did not produce them (fp32 models, models with bias
 * layers, dat_step_reg with two passes, no dat_step yet): use dat_quantize then. */
dat_status dat_model_grad_scales(const dat_model* m, const float** scales_dev);

/* One backward-to-input pass: gx[B,H,W,3] (device fp32) = grad_x sum_n CE(net(x), y); logits
 * (optional, device fp32 [B,classes]).  The quantity whose sign drives dat_attack. */
dat_status dat_input_grad(dat_model* m, const float* x, const int32_t* y, int B, float* gx,
                          float* logits, float* loss, void* stream);

/* ---- the general worker objective (Eq. (prob_DAT)) ----------------------------------------------
 *   f = E[ lambda * l(theta; x, y) + max_{|delta|_inf <= eps} phi(theta, delta; x, y) ],  lambda >= 0.
 * phi = DAT_PHI_CE: phi = l(theta; x + delta, y), DAT with labeled data (lambda = 0 is dat_attack + dat_step).
 * phi = DAT_PHI_TRADES_KL: phi = KL(p(x; theta) || p(x + delta; theta)), p = softmax of the logits: the
 *   TRADES regulariser of "DAT with unlabeled data"; no label enters phi.
 * Every network evaluation is its own train-mode forward pass (batch statistics of that pass).
 *
 * dat_attack_kl: inner maximisation of the KL regulariser by the projected sign ascent of dat_attack:
 *   the logits of one forward pass on x stay fixed; for k = 1..K:  G = grad_delta sum_n KL(p(x_n) || p(x_n + z_{k-1})).
 *   A zero start is a fixed point (the gradient vanishes where the two passes coincide): use
 *   DAT_INIT_UNIFORM or DAT_INIT_GIVEN.  loss_per_step: optional host array of K+1 floats, mean KL.
 * dat_step_reg: grads[d] (device fp32) = grad_theta (1/B) sum_n [ lambda * l(theta; x_n, y_n) + phi_n ]
 *   at the given perturbed pixels x_adv (= clip(x + delta)); the gradient flows through every pass
 *   (for the KL regulariser through both the clean and the perturbed logits; the clean pass is run twice
 *   because the two passes share the activation buffers).  losses: optional host float[2] =
 *   { mean clean cross-entropy (0 when lambda = 0 and phi = CE: that pass is not run), mean phi }.
 *   x, x_adv: device fp32 [B,H,W,3], 16-byte aligned; y: device int32 [B].  Allocates a second gradient
 *   vector inside the model on first use. */
typedef enum { DAT_PHI_CE = 0, DAT_PHI_TRADES_KL = 1 } dat_phi;
dat_status dat_attack_kl(dat_model* m, const float* x, int B, float eps, float alpha, int K,
                         dat_init init, float* delta, float* loss_per_step, void* stream);
dat_status dat_step_reg(dat_model* m, const float* x, const float* x_adv, const int32_t* y, int B,
                        float lambda, dat_phi phi, float* grads, float* losses, void* stream);

/* The elementwise pieces of the attack on their own (also what dat_attack launches):
 * dat_pgd_init writes z_0; dat_pgd_update applies one projected sign step in place.
 * N = number of fp32 elements (B*H*W*3); all pointers device; buffers 16-byte aligned. */
dat_status dat_pgd_init(const float* x, int64_t N, float eps, dat_init init, float* delta,
                        void* stream);
dat_status dat_pgd_update(const float* x, const float* G, float* delta, int64_t N, float eps,
                          float alpha, void* stream);
/* The adversarial batch handed to dat_step (Alg. A1 step 6 evaluates the loss at x + delta):
 * x_adv = clip(x + delta, 0, 1), one single-rounded fp32 addition per element.  Same argument
 * conventions as above; x_adv may not alias x or delta.  DAT_ERR_ARG for null or misaligned pointers
 * or N not a multiple of 3; nothing is written on error. */
dat_status dat_make_xadv(const float* x, const float* delta, int64_t N, float* x_adv, void* stream);

/* Plain SGD on the fp32 master parameters: theta <- theta - lr * grads (then the bf16 compute
 * copy is refreshed).  The outer-minimisation oracle A(.) of Alg. A1 in its simplest form. */
dat_status dat_sgd_update(dat_model* m, const float* grads, float lr, void* stream);

/* ---- gradient quantizer (Alg. A1 step 7) ---------------------------------------------------
 * Per tensor t of the table: scale_t = max_i |g_i|;  S = 2^(bits-1) - 1;
 *   r = |g_i| * (S / scale_t);  l = floor(r);  code magnitude = l + [u_i < r - l] (capped at S),
 *   u_i = 24-bit uniform from Philox4x32-10 (counter = i/4, stream 0, key = seed, word i mod 4,
 *   i = flat element index);  the code carries the sign of g_i.  scale_t = 0 gives zero codes;
 *   a non-finite scale_t is written to scales[t] and that tensor's codes are zero.
 * Codes are `bits`-bit two's-complement fields packed little-endian (element i occupies bits
 * [(i*bits) mod 8, ...) of byte i*bits/8).  bits in {2,4,8,16}.
 *   grads: device fp32 [d], 16-byte aligned;  offsets_dev: device int64 [num_tensors+1];
 *   q: device, dat_quantized_bytes(d,bits) bytes, 4-byte aligned;  scales: device fp32
 *   [num_tensors].  Asynchronous on `stream`. */
dat_status dat_quantize(const float* grads, const int64_t* offsets_dev, int num_tensors,
                        int64_t d, int bits, uint64_t seed, uint8_t* q, float* scales,
                        void* stream);

/* The same with the per-tensor scales given instead of computed: `scales` (device fp32 [num_tensors], read only)
 * must hold max_i |g_i| of each tensor; only the encoder runs.  With the scales of dat_model_grad_scales the
 * codes are those dat_quantize would write. */
dat_status dat_quantize_scaled(const float* grads, const int64_t* offsets_dev, int num_tensors, int64_t d,
                               int bits, uint64_t seed, const float* scales, uint8_t* q, void* stream);

/* grads_out[i] = code_i * (scale_t / S), device fp32 [d], 16-byte aligned. */
dat_status dat_dequantize(const uint8_t* q, const float* scales, const int64_t* offsets_dev,
                          int num_tensors, int64_t d, int bits, float* grads_out, void* stream);

size_t dat_quantized_bytes(int64_t d, int bits);

/* ---- after the worker block (next steps of Alg. A1) ----------------------------------------------
 * dat_aggregate: the server's Eq. (grad_agg), g_hat = (1/M) sum_i Q(g^(i)), from M workers' packed
 * codes and per-tensor scales (as written by dat_quantize, same `bits` and tensor table):
 *   out[e] = (sum over i = 0..M-1, in this order, of code_i[e] * (scale_i[t] / S)) / M   in fp32, one
 *   rounding per operation.  q, scales: HOST arrays of M DEVICE pointers (M <= DAT_MAX_WORKERS);
 *   out: device fp32 [d].  A second, server-side quantization is dat_quantize applied to `out`.
 * dat_lamb_update: the outer-minimisation oracle A(.) on the model's fp32 master parameters, the
 *   layer-wise adaptive learning rate of Eq. (3) ("layer" = tensor of the table):
 *     theta_i <- theta_i - eta * tau(||theta_i||_2) / ||u_i||_2 * u_i,  tau(x) = min(max(x, c_l), c_u)
 *   with u = g + wd*theta (use_adam = 0) or the LAMB direction of Alg. A2 (use_adam = 1):
 *     m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;  u = (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + zeta) + wd*theta,
 *   t = 1, 2, ... the step number.  The moments live in the model (allocated on first use, zero).
 *   A layer with ||u_i|| = 0 is left unchanged.  grads: device fp32 [d].  The bf16 compute copies
 *   of the weights are refreshed afterwards. */
#define DAT_MAX_WORKERS 32
dat_status dat_aggregate(const uint8_t* const* q, const float* const* scales, int M,
                         const int64_t* offsets_dev, int num_tensors, int64_t d, int bits, float* out,
                         void* stream);
dat_status dat_lamb_update(dat_model* m, const float* grads, int use_adam, float eta, float beta1,
                           float beta2, float zeta, float weight_decay, float c_l, float c_u, int t,
                           void* stream);

/* ---- convolution kernels on their own (bf16 storage, fp32 accumulate on MFMA) --------------
 * The three contractions behind dat_attack / dat_step, exposed for per-shape parity tests and
 * timing.  Tensors are device bf16 (uint16 bit patterns): x [B,H,W,Cin], w [Cout,k,k,Cin],
 * y / dy [B,Ho,Wo,Cout], Ho = (H + 2*pad - k)/stride + 1; Cin and Cout multiples of 8.
 *   forward:         y = conv(x, w)
 *   backward_data:   dx = adjoint of forward w.r.t. x applied to dy
 *   backward_weight: dw (device fp32 [Cout,k,k,Cin]) = adjoint w.r.t. w applied to dy */
dat_status dat_conv_forward(const uint16_t* x, const uint16_t* w, uint16_t* y, int B, int H,
                            int W, int Cin, int Cout, int k, int stride, int pad, void* stream);
dat_status dat_conv_backward_data(const uint16_t* dy, const uint16_t* w, uint16_t* dx, int B,
                                  int H, int W, int Cin, int Cout, int k, int stride, int pad,
                                  void* stream);
dat_status dat_conv_backward_weight(const uint16_t* x, const uint16_t* dy, float* dw, int B,
                                    int H, int W, int Cin, int Cout, int k, int stride, int pad,
                                    void* stream);

/* The same backward-weight contraction for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops that must not call hipMalloc, harnesses that forbid it): it calls no hipMalloc, hipFree
 * or other allocating routine and does not synchronise.  The split partial sums of the contraction, which
 * dat_conv_backward_weight keeps in a workspace allocated per call, go to a buffer of
 * dat_conv_backward_weight_static_limit() = 32 MiB that is part of the library's device image (each GPU the
 * library runs on holds it until the process ends).  Same arguments, same kernels, same bits as
 * dat_conv_backward_weight.  Returns DAT_ERR_UNSUPPORTED (text in dat_last_error) when the shape's partial sums
 * (splits * Cout*k*k*Cin * 4 bytes; the split count grows with B*Ho*Wo) do not fit, and launches nothing then.
 * All calls on one GPU share that buffer: calls that overlap in time on one GPU (different streams or threads)
 * race; calls on one stream are ordered and safe.  Nothing in the buffer needs clearing between calls: every
 * partial sum a call reads was written by its own first launch. */
dat_status dat_conv_backward_weight_static(const uint16_t* x, const uint16_t* dy, float* dw, int B, int H,
                                           int W, int Cin, int Cout, int k, int stride, int pad,
                                           void* stream);
size_t dat_conv_backward_weight_static_limit(void);

/* ---- per-launch timing (for benchmarks; not part of the paper's method) ----------------------
 * While enabled, every launch group of dat_attack / dat_step / dat_input_grad on this model is
 * bracketed by a hipEvent pair on the caller's stream.  dat_profile_read synchronises the device
 * and returns, for one class, the summed event time (ms), the number of launch groups and their
 * summed algorithmic work: FLOPs (2 * B*Ho*Wo*Cout*k*k*Cin, the same count for the forward,
 * backward-data and backward-weight of a layer) for the convolution classes, bytes for the
 * others.  dat_profile_enable(m, 0/1) also clears the records. */
typedef enum {
  DAT_PROF_CONV_FWD = 0,       /* implicit-GEMM forward                                  */
  DAT_PROF_CONV_BWD_DATA = 1,  /* implicit-GEMM backward-data (same kernel as forward)   */
  DAT_PROF_CONV_WGRAD = 2,     /* backward-weight + its split reduction                  */
  DAT_PROF_BN = 3,             /* batch-norm statistics + apply, forward and backward    */
  DAT_PROF_PGD = 4,            /* fused projected sign step                              */
  DAT_PROF_CONV_BWD_DATA_BN = 5, /* backward-data passes that also form the batch-norm input
                                    gradient while loading (DAT_OPT_FUSE_BN_INPUT_GRAD)     */
  DAT_PROF_NUM_CLASSES = 6
} dat_prof_class;
dat_status dat_profile_enable(dat_model* m, int on);
dat_status dat_profile_read(dat_model* m, int cls, double* ms_total, int64_t* launches, double* work);

/* ---- execution options (for ablations and tests) ------------------------------------------------
 * DAT_OPT_FUSE_BN_INPUT_GRAD (default 1, bf16 models): in backward sweeps that need no weight
 * gradients (dat_attack, dat_input_grad, dat_attack_kl) the input gradient of a batch
 * normalisation that follows a 1x1 stride-1 convolution is not written to memory; that
 * convolution's backward-data pass forms it from d(out), the normalisation's input and the ReLU
 * mask while loading its operand.  0: always run the stand-alone pass.  Both settings evaluate the
 * same fp32 expression and round to bf16 once, so they give identical bits.
 * DAT_OPT_FUSE_BN_SUMS (default 1, bf16 models): the two per-channel sums of a batch normalisation's
 * backward pass (sum dy, sum dy*xhat) are accumulated by the epilogue of the backward-data
 * convolution whose launch completes d(out), from the tile it is storing.  0: a pass of its own
 * reads d(out) again.  The two orders of summation agree to fp32 rounding, not bit for bit.
 * DAT_OPT_FUSE_PGD_GRADIENT (default 1, bf16 models): the projected sign step of dat_attack /
 * dat_attack_kl reads the bf16 input gradient the backward pass leaves in the network-input layout
 * (only its sign enters the step; the normalisation scale 1/std is positive) instead of an fp32
 * pixel gradient made by a pass of its own.  0: make that copy first.  Identical bits either way.
 * DAT_OPT_SPARSE_SHORTCUT_GRADIENT (default 1, bf16 models): the input gradient of a strided 1x1
 * projection shortcut is non-zero at the pixels the projection reads only (even row, even column).
 * Its backward-data pass writes just those, and the backward-data pass of the block's first
 * convolution, which adds its own part to the same tensor, reads the stored values there and takes
 * zero elsewhere.  0: the projection's pass also writes the zeros and the other pass reads them
 * back.  Identical bits either way.
 * DAT_OPT_OVERLAP_WEIGHT_GRADIENTS (default 1, bf16 models): in dat_step / dat_step_reg the
 * backward-weight launches of the convolutions run on a stream owned by the model, each after an
 * event that marks its output gradient complete on the caller's stream, and the caller's stream
 * waits for them before the call's work on it ends (fork / join: the call stays asynchronous on
 * `stream`).  0: everything on the caller's stream.  Identical bits either way.
 * Returns DAT_ERR_ARG for an unknown option.
 * DAT_OPT_ABSORB_SHORTCUT_BN (default 1, bf16 models): the batch normalisation on a projection shortcut is
 * evaluated by the last normalisation of the residual branch (forward) and shares its pass over d(out)
 * (backward); neither its output nor its output gradient is stored.  0: it runs as passes of its own.
 * Identical bits either way (with DAT_OPT_FUSE_BN_SUMS = 0; that option's sums depend on the launch graph).
 * DAT_OPT_FUSE_STEM_POOL (default 1, bf16 models): a BN + ReLU read only by a 3x3/2 max-pool does not store its
 * output; one forward pass writes the pooled tensor, and the backward pass gathers d(out) from the pool's output
 * gradient.  0: the pool runs as passes of its own.  Identical bits either way.
 * DAT_OPT_GRADIENT_SCALES (default 1, bf16 models): the kernels that write parameter gradients in dat_step also
 * maintain the per-tensor abs-max that dat_model_grad_scales returns.  0: they do not (dat_model_grad_scales then
 * refuses).  The gradients are the same bits either way.
 * DAT_OPT_KEEP_BOTH_PASSES (default 1): dat_step_reg with the KL regulariser keeps the clean pass's activations,
 * batch statistics and masks in a second set of buffers (allocated on the first such call: as much device memory
 * again as the model's activations) while the perturbed pass runs, so each branch of the gradient finds its own
 * pass; 0, or when that allocation fails: one set, the clean pass is run a second time.  Identical bits either way.
 * Options may be changed between calls, not while a call on the model is in flight. */
typedef enum { DAT_OPT_FUSE_BN_INPUT_GRAD = 0, DAT_OPT_FUSE_BN_SUMS = 1, DAT_OPT_FUSE_PGD_GRADIENT = 2,
               DAT_OPT_SPARSE_SHORTCUT_GRADIENT = 3, DAT_OPT_OVERLAP_WEIGHT_GRADIENTS = 4,
               DAT_OPT_ABSORB_SHORTCUT_BN = 5, DAT_OPT_FUSE_STEM_POOL = 6, DAT_OPT_GRADIENT_SCALES = 7,
               DAT_OPT_KEEP_BOTH_PASSES = 8 } dat_option;
dat_status dat_model_set_option(dat_model* m, dat_option opt, int value);
/* Process-wide kernel selection (ablations and tests; an atomic flag, read at every convolution launch of every
 * model and of the dat_conv_* entry points).  DAT_KOPT_RING_KERNEL (default 1): layers that run as one round of
 * 256-channel tiles go through the multi-stage kernel; 0: through the 128x128 kernels.  The convolution outputs
 * are bit-identical, the grouping of the batch-norm partial sums differs (256 instead of 128 pixels per slab).
 * DAT_KOPT_TILE_160 (default 1): layers with 160 or 320 output channels (the wide ResNets)
 * run in 160-channel tiles; 0: in 128-channel tiles, the last one partly empty.  Bit-identical outputs.
 * DAT_KOPT_NARROW_UNDERFILLED (default 1): a layer with a contraction >= 1024 whose 128x128 tiles would number at
 * most 1.5 per compute unit runs in 32-channel tiles; 0: in 128-channel tiles.  Bit-identical outputs (the partial
 * sums of the batch statistics are grouped differently). */
typedef enum { DAT_KOPT_RING_KERNEL = 0, DAT_KOPT_TILE_160 = 1, DAT_KOPT_NARROW_UNDERFILLED = 2 } dat_kernel_option;
dat_status dat_set_kernel_option(dat_kernel_option opt, int value);

/* ---- introspection for parity tests (not part of the paper's method) --------------------------------
 * The layer graph and the tensors a model keeps on the device, so that a test can compare every stored
 * activation, activation gradient and batch statistic of the last pass with a reference element by element,
 * and restart the reference from the library's own tensors op by op (teacher forcing).
 *   dat_inspect_counts  number of ops and of activation tensors (tensor 0 = the network input).
 *   dat_inspect_op      info[10] = kind (0 conv, 1 bias+act, 2 BN+act, 3 max-pool, 4 global average pool,
 *                       5 linear), input tensor, output tensor, residual tensor or -1, k, stride, pad, relu,
 *                       first and second parameter tensor of the table or -1.
 *   dat_inspect_tensor  info[6] = H, W, C (channels as stored), bytes per element (2: bf16, 4: fp32),
 *                       act_stored, grad_stored.  act_stored = 0: the model never writes this tensor in plain
 *                       NHWC form (a fused pass consumes it, or it is the padded network input of a bf16
 *                       model).  grad_stored = 1: the last backward sweep left the complete gradient of this
 *                       tensor in memory (sweeps without parameter gradients skip some).
 *   dat_inspect_read    copies the B*H*W*C stored elements of tensor t (which = 0) or of its gradient
 *                       (which = 1) to host memory as they are; `bytes` must be exactly that size.
 *                       Synchronises the device.
 *   dat_inspect_bn      batch mean and 1/sqrt(var + 1e-5) of BN op `op` from the last forward pass, host
 *                       arrays of C floats.  DAT_ERR_ARG if `op` is not a batch normalisation. */
dat_status dat_inspect_counts(const dat_model* m, int* num_ops, int* num_tensors);
dat_status dat_inspect_op(const dat_model* m, int op, int32_t* info);
dat_status dat_inspect_tensor(const dat_model* m, int t, int32_t* info);
dat_status dat_inspect_read(dat_model* m, int which, int t, int B, void* host_dst, size_t bytes);
dat_status dat_inspect_bn(dat_model* m, int op, float* mean_host, float* rstd_host);

/* ---- misc ---------------------------------------------------------------------------------- */
const char* dat_status_string(dat_status s);
/* Text of the last HIP error seen by this thread's calls ("" if none). */
const char* dat_last_error(void);
/* Fills out[n] (device) with the library's Philox uniforms for flat indices start..start+n-1:
 * the stream the quantizer (stream_id 0) and the random init (stream_id 1) draw from. */
dat_status dat_philox_uniform(uint64_t start, int64_t n, uint64_t seed, uint32_t stream_id,
                              float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DAT_H */
