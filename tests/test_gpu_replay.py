"""Every stored tensor of the GPU library's forward and backward passes against the CPU reference, element
by element, op by op, with teacher forcing (tests/replay.py): the reference evaluates each op from the tensors
the GPU actually stored, so a comparison sees one op's rounding and not the cascade a deep ReLU / batch-norm
network makes of it.  Covered per case: every convolution output, every BN / ReLU / residual output, pooled
tensors, logits, batch statistics, every stored activation gradient of the sweep with weight gradients
(dat_step) and of the sweep without (dat_input_grad, where some BN input gradients are formed inside a
convolution and never stored), the pixel gradient and every parameter-gradient tensor -- in the launch
configuration the library picks for that size, fusions on.  The configured sizes of the benchmark configs
(CIFAR ResNet-18 batch 512, WRN-34-10 batch 256, ResNet-50 224x224 batch 256) run whole, and so do ResNet-50 with
the paper's 85 images per GPU and pre-activation ResNet-18 batch 512.

Bars (per element): bf16-stored tensors |gpu - ref| <= 2^-7 |ref| + 2e-5 max|ref| (one unit in the last place
of the stored format, plus fp32 accumulation error where a value is small through cancellation); fp32 tensors
and statistics 2e-5 relative; parameter gradients 1e-4 of the tensor's largest entry.  Statistics and parameter
gradients must meet their bar everywhere.  A stored tensor may miss it in a few elements (at most ACT_VIOL_FRAC
of an activation tensor, GRAD_VIOL_FRAC of a gradient tensor): where the comparison spans two roundings -- a
tensor the GPU fuses away between two stored ones, a gradient with several contributions that is re-rounded
after each -- a flipped rounding of the intermediate shows up relative to a final value that may be much
smaller through cancellation.  Where one op separates the two sides no element may miss the bar by more than a
factor WORST_CAP; where a never-stored tensor lies between them (the stem's activation ahead of the max-pool)
a window whose two largest values are one rounding apart may send its gradient to the other pixel on the two
sides, both valid, so only the fraction is bounded there.  (Measured at ResNet-50 224x224 batch 256: 99.98 % of
10.3 billion stored elements bit-equal, at most 4e-6 of any tensor over the bar, eight elements of the stem's
205 M re-routed; a kernel that writes zeros, garbage or a wrong sign misses the bar in most elements.)"""
import os
import time

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as syn
from tests import replay

pytestmark = pytest.mark.gpu
MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)
ACT_VIOL_FRAC, GRAD_VIOL_FRAC, WORST_CAP = 5e-5, 1e-3, 100.0
LOG = os.environ.get("DAT_REPLAY_LOG_DIR")     # per-tensor tables go to <dir>/replay.log when set; summaries are always printed


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _report(tag, rec, t0):
    s = rec.summary()
    line = "%s: %d comparisons, %d elements, exactly equal %.4f, over the bar %d (worst tensor %.2e of its elements), %.1f s" % (
        tag, s["items"], s["elements"], s["exact_frac"], s["viol"], s["max_viol_frac"], time.time() - t0)
    print(line, flush=True)
    try:
        if not LOG:
            return s
        os.makedirs(LOG, exist_ok=True)
        with open(os.path.join(LOG, "replay.log"), "a") as f:
            f.write(line + "\n")
            for r in rec:
                f.write("  %-60s n=%-10d exact=%.4f viol=%-8d worst=%.3g max_ref=%.3g max_err=%.3g\n" % (
                    r["name"], r["n"], r["exact"] / max(r["n"], 1), r["viol"], r["worst"], r["max_ref"], r["max_err"]))
    except OSError:
        pass
    return s


def _check(rec):
    replay.check(rec, ACT_VIOL_FRAC, GRAD_VIOL_FRAC, WORST_CAP)


def _oracle_bytes(ref, B):
    return sum(B * h * w * c for h, w, c in ref.tensor_shapes()) * 16


def _replay_case(dat, arch, bf16, B, H, W, classes, norm, cfg, perturbed, attack_sweep=True):
    mean, std = (MEAN, STD) if norm else (None, None)
    ref = oracle.Model(arch, bf16, H, W, classes, mean, std)
    need = _oracle_bytes(ref, B)
    try:
        import psutil
        avail = psutil.virtual_memory().available
    except Exception:  # pragma: no cover
        avail = 1 << 62
    if need * 1.25 > avail:
        pytest.skip("the reference needs %.0f GB of host memory for this case, %.0f GB available" % (need / 1e9, avail / 1e9))
    gpu = dat.Model(arch, dat.BF16 if bf16 else dat.F32, B, H, W, classes, mean, std)
    gen = syn.perturbed_params if perturbed else syn.he_normal_params
    theta = gen(cfg, ref.offsets, ref.fan_in, ref.kind)
    ref.set_params(theta); gpu.set_params(theta)
    assert [tuple(o[k] for k in ("kind", "in", "out", "res", "k", "stride", "pad", "relu", "p0", "p1")) for o in gpu.inspect_ops()] == \
           [tuple(o[k] for k in ("kind", "in", "out", "res", "k", "stride", "pad", "relu", "p0", "p1")) for o in ref.ops()]
    x, y = syn.images(cfg, B, H, W), syn.labels(cfg, B, classes)
    xd, yd = _cuda(x), _cuda(y)
    tag = "arch %d %s B=%d %dx%d" % (arch, "bf16" if bf16 else "fp32", B, H, W)
    # sweep with parameter gradients
    t0 = time.time()
    g_gpu, l_gpu = gpu.step(xd, yd, want_loss=True)
    src = replay.GpuSource(gpu, B)
    rec = replay.Record()
    own = replay.forward(ref, src, x, rec)
    s = _report(tag + " forward", rec, t0)
    _check(rec)
    t0 = time.time()
    recb = replay.Record()
    loss, _ = replay.backward(ref, src, y, 1.0 / B, True, recb, own_acts=own)
    replay.param_grads(ref, g_gpu.cpu().numpy(), recb)
    _report(tag + " backward (dat_step)", recb, t0)
    _check(recb)
    assert abs(l_gpu - loss) <= 2e-5 * abs(loss)
    if attack_sweep:
        # sweep without parameter gradients: same forward pass, other backward launches
        t0 = time.time()
        logits_step = src.act(ref.ops()[-1]["out"])
        gx, logits, l2 = gpu.input_grad(xd, yd)
        assert np.array_equal(logits.cpu().numpy().reshape(-1), logits_step)
        src.refresh()
        reca = replay.Record()
        _, spans = replay.backward(ref, src, y, 1.0, False, reca, own_acts=own)
        replay.pixel_grad(ref, gx.cpu().numpy(), reca, bool(bf16), spans)
        _report(tag + " backward (dat_input_grad)", reca, t0)
        _check(reca)
        stored = sum(1 for r in reca if " grad t" in r["name"])
        assert stored >= 3
    gpu.close()
    return s


SMALL = [
    # arch, bf16, B, H, W, classes, normalise
    (100, 1, 8, 16, 16, 5, True),
    (100, 0, 8, 16, 16, 5, True),
    (0, 0, 32, 32, 32, 10, False),     # config 1's network at its configured size
    (1, 1, 16, 16, 16, 10, False),
    (1, 0, 6, 16, 16, 10, False),
    (2, 1, 4, 16, 16, 10, False),
    (3, 1, 6, 96, 96, 12, True),
    (3, 1, 5, 64, 96, 1000, True),     # ragged tiles, the full classifier
    (3, 1, 3, 68, 70, 12, True),       # odd block counts per row (35) in the stem's 2x2-block layout
    (3, 0, 3, 64, 64, 12, True),
    (4, 1, 12, 16, 16, 10, False),
    (5, 1, 5, 8, 8, 10, False),
]


@pytest.mark.parametrize("arch,bf16,B,H,W,classes,norm", SMALL)
def test_every_stored_tensor_matches_the_reference_op_by_op(dat, arch, bf16, B, H, W, classes, norm):
    _replay_case(dat, arch, bf16, B, H, W, classes, norm, cfg=arch + 70 + bf16, perturbed=True)


def test_config2_resnet18_cifar_batch512_at_its_configured_size(dat):
    s = _replay_case(dat, 1, 1, 512, 32, 32, 10, False, cfg=2, perturbed=False)
    assert s["elements"] > 3e8


def test_config2_end_to_end_against_the_comparison_resolution(dat):
    """The same configuration WITHOUT teacher forcing: one forward + backward-to-input of the GPU against one of the
    reference, beside the reference against itself with its convolution sums jittered by 1e-7 (the resolution of any
    end-to-end comparison of two bf16 implementations).  Forward quantities meet the spec bar outright; for the
    gradients the printed numbers show that GPU-vs-reference and reference-vs-itself are the same size, and they are
    asserted only while 1.5 x the resolution stays below 0.1 (see tests/test_gpu_network.py)."""
    B, H, W, classes = 512, 32, 32, 10
    ref = oracle.Model(1, 1, H, W, classes)
    gpu = dat.Model(1, dat.BF16, B, H, W, classes)
    theta = syn.he_normal_params(2, ref.offsets, ref.fan_in, ref.kind)
    ref.set_params(theta); gpu.set_params(theta)
    x, y = syn.images(2, B, H, W), syn.labels(2, B, classes)
    r = ref.loss_grad(x, y, "sum")
    ref.set_accum_jitter(1e-7)
    rj = ref.loss_grad(x, y, "sum")
    gx, logits, loss = gpu.input_grad(_cuda(x), _cuda(y))
    gx, logits = gx.cpu().numpy().astype(np.float64), logits.cpu().numpy().astype(np.float64)

    def rel2(a, b):
        return float(np.linalg.norm(a - b) / np.linalg.norm(b))
    got = dict(logits=rel2(logits, r["logits"]), gx=rel2(gx, r["gx"]), sign=float((np.sign(gx) != np.sign(r["gx"])).mean()),
               loss=abs(loss - r["loss"]) / abs(r["loss"]))
    res = dict(logits=rel2(rj["logits"], r["logits"]), gx=rel2(rj["gx"], r["gx"]), sign=float((np.sign(rj["gx"]) != np.sign(r["gx"])).mean()))
    line = "config 2 end to end (B=512, 32x32): GPU vs reference %s; reference vs itself under 1e-7 jitter %s" % (got, res)
    print(line, flush=True)
    try:
        if LOG:
            with open(os.path.join(LOG, "replay.log"), "a") as f:
                f.write(line + "\n")
    except OSError:
        pass
    assert got["logits"] < 2e-2 and got["loss"] < 2e-2
    for k, bar in (("gx", 2e-2), ("sign", 1e-3)):
        bound = max(bar, 1.5 * res[k])
        if bound <= 0.1:
            assert got[k] < bound, (k, got[k], bound)
    gpu.close()


def test_config3_wrn34_10_batch256_at_its_configured_size(dat):
    s = _replay_case(dat, 2, 1, 256, 32, 32, 10, False, cfg=3, perturbed=False, attack_sweep=False)
    assert s["elements"] > 1e9


def test_config4_5_resnet50_224_batch256_at_its_configured_size(dat):
    s = _replay_case(dat, 3, 1, 256, 224, 224, 1000, True, cfg=4, perturbed=False)
    assert s["elements"] > 5e9


def test_imagenet_shape_of_the_papers_runs_resnet50_224_batch85(dat):
    """85 images per GPU: pixel counts that are no multiple of the kernels' tiles at 56x56 and below."""
    s = _replay_case(dat, 3, 1, 85, 224, 224, 1000, True, cfg=7, perturbed=False)
    assert s["elements"] > 1.5e9


def test_preact_resnet18_batch512_at_its_configured_size(dat):
    s = _replay_case(dat, 4, 1, 512, 32, 32, 10, False, cfg=8, perturbed=False)
    assert s["elements"] > 3e8
