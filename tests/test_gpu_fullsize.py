"""Parity at the full benchmark sizes (ResNet-50, 224x224, batch 256, bf16), in the launch
configuration bench.py times.  The whole-network reference would take the CPU hours here, so:
  * the three convolution kernels are spot-checked at full layer shapes against single outputs the
    reference computes one by one from the definition;
  * the quantizer and the PGD update are compared bit for bit on the full 25.56 M / 38.5 M vectors;
  * dat_attack / dat_step are checked through properties that hold at any size: the l-inf ball and
    image box exactly, determinism, the batch-norm scale invariance <W, dL/dW> = 0 of every
    convolution that feeds a batch-norm, sum_c dL/db_c = 0 of the classifier bias, loss growth."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as syn

pytestmark = pytest.mark.gpu
MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)
B = 256

# full-size layers of ResNet-50 at batch 256 (H, Cin, Cout, k, stride, pad)
LAYERS = [
    (224, 8, 64, 7, 2, 3),       # stem (3 channels padded to 8)
    (56, 64, 64, 3, 1, 1),       # layer1 3x3
    (56, 256, 64, 1, 1, 0),      # layer1 reduce
    (56, 128, 128, 3, 2, 1),     # layer2 strided 3x3
    (28, 128, 512, 1, 1, 0),     # layer2 expand
    (28, 512, 1024, 1, 2, 0),    # layer3 projection shortcut
    (14, 256, 256, 3, 1, 1),     # layer3 3x3 (one round of 256x256 tiles: ring kernel)
    (14, 1024, 256, 1, 1, 0),    # layer3 reduce (ring kernel forward)
    (7, 2048, 512, 1, 1, 0),     # layer4 reduce (one round of 256x128 tiles: ring kernel)
    (7, 512, 512, 3, 1, 1),      # layer4 3x3 (ring kernel)
]


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _sample(rng, n, total, extra=()):
    idx = np.unique(np.concatenate([rng.integers(0, total, size=n), np.array(extra, np.int64)]))
    return idx.astype(np.int64)


@pytest.mark.parametrize("layer", LAYERS)
def test_conv_kernels_at_full_layer_shapes(dat, layer):
    H, Ci, Co, k, st, pad = layer
    g = torch.Generator(device="cuda"); g.manual_seed(H * 1000 + Ci)
    x = torch.randn(B, H, H, Ci, device="cuda", generator=g).to(torch.bfloat16)
    w = (torch.randn(Co, k, k, Ci, device="cuda", generator=g) / np.sqrt(Ci * k * k)).to(torch.bfloat16)
    y = dat.conv_forward(x, w, st, pad)
    Ho = y.shape[1]
    dy = torch.randn(B, Ho, Ho, Co, device="cuda", generator=g).to(torch.bfloat16)
    dx = dat.conv_backward_data(dy, w, (H, H), st, pad)
    dw = dat.conv_backward_weight(x, dy, k, st, pad)
    torch.cuda.synchronize()
    xh, wh, dyh = x.float().cpu().numpy(), w.float().cpu().numpy(), dy.float().cpu().numpy()
    rng = np.random.default_rng(H + Ci)
    # samples include the tensor's first and last elements and borders (padding paths, last tiles)
    iy = _sample(rng, 300, y.numel(), (0, y.numel() - 1, Co * Ho - 1))
    want = oracle.conv_forward_points(xh, wh, st, pad, iy)
    got = y.reshape(-1)[torch.from_numpy(iy).cuda()].float().cpu().numpy()
    scale = np.abs(want).max()
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-5 * scale), np.abs(got - want).max()
    ix = _sample(rng, 200, dx.numel(), (0, dx.numel() - 1, Ci * H + 1))
    want = oracle.conv_backward_data_points(dyh, wh, (H, H), st, pad, ix)
    got = dx.reshape(-1)[torch.from_numpy(ix).cuda()].float().cpu().numpy()
    scale = max(np.abs(want).max(), 1e-30)
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-5 * scale), np.abs(got - want).max()
    iw = _sample(rng, 24, dw.numel(), (0, dw.numel() - 1))
    want = oracle.conv_backward_weight_points(xh, dyh, k, st, pad, iw)
    got = dw.reshape(-1)[torch.from_numpy(iw).cuda()].cpu().numpy()
    # fp32 accumulation over B*Ho*Wo (up to 3.2 M) bf16 products
    assert np.abs(got - want).max() <= 3e-5 * np.abs(want).max() + 1e-3 * np.sqrt(B * Ho * Ho) * 2.0 ** -24 * 16, np.abs(got - want).max()


def test_quantizer_full_gradient_bit_exact(dat):
    """Config 5: b = 8 and b = 4 on the full 25.56 M-element gradient, 161 tensors."""
    ref = oracle.Model(oracle.ARCH_RESNET50, 1, 224, 224, 1000, MEAN, STD)
    g = syn.stress_gradient(5, ref.offsets)
    gd = torch.from_numpy(g).cuda()
    od = torch.from_numpy(ref.offsets).cuda()
    seed = syn.seed_for(5, "quantizer")
    for bits in (8, 4):
        S = oracle.levels(bits)
        codes, scales = oracle.quantize(g, ref.offsets, S, seed)
        q, sc = dat.quantize(gd, od, bits, seed)
        assert np.array_equal(sc.cpu().numpy(), scales)
        assert np.array_equal(q.cpu().numpy(), oracle.pack(codes, bits))
        out = dat.dequantize(q, sc, od, g.size, bits).cpu().numpy()
        assert np.array_equal(out, oracle.dequantize(codes, scales, ref.offsets, S))


def test_pgd_update_full_batch_bit_exact(dat):
    eps, alpha = 2 / 255, 0.5 / 255
    x = syn.images(6, B, 224, 224)
    xd = torch.from_numpy(x).cuda()
    seed = syn.seed_for(6, "attack_init")
    d0 = dat.pgd_init(xd, eps, oracle.INIT_UNIFORM, seed)
    want0 = oracle.init_delta(x, eps, oracle.INIT_UNIFORM, seed)
    assert np.array_equal(d0.cpu().numpy(), want0)
    G = np.random.default_rng(3).standard_normal(x.shape).astype(np.float32)
    got = dat.pgd_update(xd, torch.from_numpy(G).cuda(), d0, eps, alpha).cpu().numpy()
    assert np.array_equal(got, oracle.pgd_update(x, G, want0, eps, alpha))


@pytest.mark.parametrize("layer", [(14, 256, 256, 3, 1, 1), (14, 1024, 256, 1, 1, 0), (7, 512, 512, 3, 1, 1), (7, 2048, 512, 1, 1, 0),
                                   (28, 256, 256, 3, 2, 1)])
def test_ring_kernel_gives_the_bits_of_the_single_stage_kernel(dat, layer):
    """Layers that run as one round of 256-channel tiles through the multi-stage kernel: every accumulator sees the
    same k order as in the 128x128 kernel, so forward and backward-data outputs are identical bit for bit (the
    process-wide switch is read at every launch)."""
    H, Ci, Co, k, st, pad = layer
    g = torch.Generator(device="cuda"); g.manual_seed(H * 77 + Ci)
    x = torch.randn(B, H, H, Ci, device="cuda", generator=g).to(torch.bfloat16)
    w = (torch.randn(Co, k, k, Ci, device="cuda", generator=g) / np.sqrt(Ci * k * k)).to(torch.bfloat16)
    try:
        dat.set_kernel_option(dat.KOPT_RING_KERNEL, 1)
        y = dat.conv_forward(x, w, st, pad)
        dy = torch.randn_like(y)
        dx = dat.conv_backward_data(dy, w, (H, H), st, pad)
        dat.set_kernel_option(dat.KOPT_RING_KERNEL, 0)
        y0 = dat.conv_forward(x, w, st, pad)
        dx0 = dat.conv_backward_data(dy, w, (H, H), st, pad)
        torch.cuda.synchronize()
    finally:
        dat.set_kernel_option(dat.KOPT_RING_KERNEL, 1)
    assert torch.equal(y.view(torch.int16), y0.view(torch.int16))
    assert torch.equal(dx.view(torch.int16), dx0.view(torch.int16))
    assert float(y.float().abs().max()) > 0 and float(dx.float().abs().max()) > 0


def test_network_with_ring_kernel_agrees_with_single_stage_kernels(dat):
    """ResNet-50 224 at batch 256, forward pass with and without the multi-stage kernel.  The convolution outputs
    are the same bits; only the batch-norm partial sums are grouped by 256 pixels instead of 128.  So every tensor
    up to and including the output of the first convolution the multi-stage kernel runs is bit-identical in the
    two passes, and the batch statistics its epilogue produced agree to fp32 summation error (a wrong slab count
    or a wrong 512-thread epilogue would move them by O(1)); from there on single flipped bf16 roundings cascade,
    so the logits are only required to agree within the bf16 bar."""
    model = dat.Model(dat.ARCH_RESNET50, dat.BF16, B, 224, 224, 1000, MEAN, STD)
    model.set_params(syn.he_normal_params(7, model.offsets, model.fan_in, model.kind))
    xd = torch.from_numpy(syn.images(7, B, 224, 224)).cuda()
    yd = torch.from_numpy(syn.labels(7, B, 1000)).cuda()
    ops, info = model.inspect_ops(), model.inspect_tensors()
    # first layer the multi-stage kernel takes at this batch: contraction >= 1024 into a multiple of 256 channels on 14x14
    ring = next(i for i, o in enumerate(ops) if o["kind"] == 0 and info[o["out"]]["C"] % 256 == 0 and info[o["out"]]["H"] == 14
                and o["k"] * o["k"] * info[o["in"]]["C"] >= 1024)
    bn_after = next(i for i, o in enumerate(ops) if o["kind"] == 2 and o["in"] == ops[ring]["out"])
    runs = []
    try:
        for on in (1, 0):
            dat.set_kernel_option(dat.KOPT_RING_KERNEL, on)
            gx, logits, loss = model.input_grad(xd, yd)
            conv_out = model.inspect_read(0, ops[ring]["out"], B, info[ops[ring]["out"]])
            conv_in = model.inspect_read(0, ops[ring]["in"], B, info[ops[ring]["in"]])
            runs.append((conv_in, conv_out, model.inspect_bn(bn_after, info[ops[ring]["out"]]["C"]), logits.cpu().numpy().astype(np.float64), loss))
    finally:
        dat.set_kernel_option(dat.KOPT_RING_KERNEL, 1)
    (in1, out1, (mean1, rstd1), z1, l1), (in0, out0, (mean0, rstd0), z0, l0) = runs
    assert np.array_equal(in1, in0) and np.array_equal(out1, out0) and np.abs(out1.astype(np.int64)).max() > 0
    assert np.abs(mean1 - mean0).max() <= 1e-5 / rstd0.min() and np.abs(rstd1 / rstd0 - 1).max() <= 1e-5
    rel = np.linalg.norm(z1 - z0) / np.linalg.norm(z0)
    print("ring vs single-stage: logits rel %.3e, loss %.6f vs %.6f" % (rel, l1, l0))
    assert np.isfinite(z1).all() and rel < 2e-2 and abs(l1 - l0) < 2e-2 * abs(l0)
    model.close()


def test_attack_chains_its_own_gradient_exactly_at_full_size(dat):
    """dat_attack at ResNet-50 224x224 B = 256 against the reference's update rule applied to the library's own input
    gradient: z_{k+1} must equal, bit for bit, clip(clip(z_k + alpha sign(G_k), +-eps), -x, 1-x) with G_k the gradient
    dat_input_grad returns at clip(x + z_k) -- for the first step from a given start and for the second step, which
    starts from the network input the fused sign-step kernel wrote itself.  (What G_k is worth is the op-by-op
    test's business; this one pins the wiring of the iteration: start point, input formation, sign step read
    straight from the bf16 input gradient in its blocked layout, projection, next input.)"""
    eps, alpha = 4 / 255, 1 / 255
    model = dat.Model(dat.ARCH_RESNET50, dat.BF16, B, 224, 224, 1000, MEAN, STD)
    model.set_params(syn.he_normal_params(5, model.offsets, model.fan_in, model.kind))
    x, y = syn.images(5, B, 224, 224), syn.labels(5, B, 1000)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    z0 = oracle.init_delta(x, eps, oracle.INIT_UNIFORM, 91)
    z0d = torch.from_numpy(z0).cuda()
    z1 = model.attack(xd, yd, eps, alpha, 1, dat.INIT_GIVEN, delta0=z0d).cpu().numpy()
    z2 = model.attack(xd, yd, eps, alpha, 2, dat.INIT_GIVEN, delta0=z0d).cpu().numpy()
    for zk, zk1 in ((z0, z1), (z1, z2)):
        gx, _, _ = model.input_grad(torch.from_numpy(oracle.make_xadv(x, zk)).cuda(), yd, want_logits=False, want_loss=False)
        want = oracle.pgd_update(x, gx.cpu().numpy(), zk, eps, alpha)
        assert np.array_equal(zk1, want)
        assert (zk1 != zk).mean() > 0.5           # the step moved most coordinates
    model.close()


@pytest.mark.parametrize("B,eps,alpha,K", [
    (256, 4 / 255, 1 / 255, 3),          # config 5
    (85, 2 / 255, 1.25 / 255, 4),        # the paper's own ImageNet shape: 85 images per GPU, PGD-4 (odd batch: tile tails)
])
def test_attack_and_step_properties_at_full_size(dat, B, eps, alpha, K):
    model = dat.Model(dat.ARCH_RESNET50, dat.BF16, B, 224, 224, 1000, MEAN, STD)
    theta = syn.he_normal_params(5, model.offsets, model.fan_in, model.kind)
    model.set_params(theta)
    x = syn.images(5, B, 224, 224)
    y = syn.labels(5, B, 1000)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    seed = syn.seed_for(5, "attack_init")
    delta, losses = model.attack(xd, yd, eps, alpha, K, dat.INIT_UNIFORM, seed=seed, want_losses=True)
    d = delta.cpu().numpy()
    assert np.abs(d).max() <= np.float32(eps)                 # exact, fp32
    assert (x + d).min() >= 0.0 and (x + d).max() <= 1.0
    assert np.isfinite(losses).all() and losses[-1] > losses[0]
    # every step moves each coordinate by at most alpha from the clipped start
    d0 = oracle.init_delta(x, eps, oracle.INIT_UNIFORM, seed)
    assert np.abs(d - d0).max() <= K * np.float32(alpha) * (1 + 1e-6)
    # determinism: same inputs, same bits
    d2 = model.attack(xd, yd, eps, alpha, K, dat.INIT_UNIFORM, seed=seed).cpu().numpy()
    assert np.array_equal(d, d2)
    xadv = torch.from_numpy(oracle.make_xadv(x, d)).cuda()
    g, loss = model.step(xadv, yd, want_loss=True)
    # the per-tensor abs-max the gradient writers left behind is the quantizer's own, and so are the codes
    offs = (model.offsets_device(), model.num_tensors)
    fused = model.grad_scales_tensor()
    for bits in (8, 4):
        q_ref, sc_ref = dat.quantize(g, offs, bits, 77)
        q_fused = dat.quantize_scaled(g, offs, bits, 77, model.grad_scales())
        assert torch.equal(sc_ref.view(torch.int32), fused.view(torch.int32)) and torch.equal(q_ref, q_fused)
    assert float(fused.min()) > 0
    g = g.cpu().numpy()
    assert np.isfinite(g).all() and abs(loss - losses[-1]) < 2e-2 * abs(loss)
    off, kind = model.offsets, model.kind
    # classifier bias: sum_c dL/db_c = mean_n sum_c (softmax - onehot) = 0
    tb = int(np.where(kind == 5)[0][0])
    gb = g[off[tb]:off[tb + 1]]
    assert abs(gb.sum()) < 1e-5 and np.abs(gb).max() > 1e-5
    # every conv is followed by train-mode BN: the loss does not change when W is scaled, so
    # <W, dL/dW> = 0 up to bf16 rounding of the stored tensors
    worst = 0.0
    for t in np.where(kind == 0)[0]:
        wv, gv = theta[off[t]:off[t + 1]].astype(np.float64), g[off[t]:off[t + 1]].astype(np.float64)
        worst = max(worst, abs(wv @ gv) / (np.linalg.norm(wv) * np.linalg.norm(gv) + 1e-300))
    assert worst < 0.05, worst
    model.close()
