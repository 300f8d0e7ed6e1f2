"""Pins for the CPU reference's network arithmetic (forward, backward to input, weight
gradients): library special cases, finite differences, adjoint identities, published sizes."""
import os

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as syn
from tests import torch_mirror

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)


def _rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


def test_param_counts_match_published():
    for line in open(os.path.join(GOLD, "param_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        arch, H, W, classes, d = map(int, line.split())
        assert oracle.Model(arch, 0, H, W, classes).d == d


def test_round_bf16_matches_library_conversion():
    rng = np.random.default_rng(1)
    v = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.uniform(-30, 30, 4000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40, -1e-45]]).astype(np.float32)
    want = torch.tensor(v).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.round_bf16(float(x)) for x in v], np.float32)
    assert np.array_equal(want, got)
    # exact ties go to the even neighbour; a value just above a tie (not representable in fp32) goes up
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7


@pytest.mark.parametrize("k,stride,pad,H,W", [(3, 1, 1, 7, 6), (3, 2, 1, 9, 8), (1, 2, 0, 7, 7), (7, 2, 3, 17, 15), (1, 1, 0, 5, 4)])
def test_conv_matches_library_and_adjoint(k, stride, pad, H, W):
    rng = np.random.default_rng(k * 100 + stride)
    B, Ci, Co = 2, 5, 4
    x = rng.standard_normal((B, H, W, Ci))
    w = rng.standard_normal((Co, k, k, Ci))
    out = oracle.conv_forward(x, w, stride, pad)
    xt = torch.tensor(x).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(w).permute(0, 3, 1, 2).requires_grad_(True)
    ot = torch.nn.functional.conv2d(xt, wt, None, stride, pad)
    assert _rel(out, ot.detach().permute(0, 2, 3, 1).numpy()) < 1e-13
    dout = rng.standard_normal(out.shape)
    din, dw = oracle.conv_backward(x, w, dout, stride, pad)
    ot.backward(torch.tensor(dout).permute(0, 3, 1, 2))
    assert _rel(din, xt.grad.permute(0, 2, 3, 1).numpy()) < 1e-13
    assert _rel(dw, wt.grad.permute(0, 2, 3, 1).numpy()) < 1e-13
    # adjoint identities <conv(x,w),dy> = <x,bwd_data(dy,w)> = <w,bwd_weight(x,dy)>
    lhs = (out * dout).sum()
    assert abs(lhs - (x * din).sum()) < 1e-10 * abs(lhs) + 1e-10
    assert abs(lhs - (w * dw).sum()) < 1e-10 * abs(lhs) + 1e-10


def _setup(arch, H, W, classes, B, cfg=7, norm=False):
    m = oracle.Model(arch, 0, H, W, classes, MEAN if norm else None, STD if norm else None)
    theta = syn.perturbed_params(cfg, m.offsets, m.fan_in, m.kind).astype(np.float64)
    x = syn.images(cfg, B, H, W).astype(np.float64)
    y = syn.labels(cfg, B, classes)
    return m, theta, x, y


@pytest.mark.parametrize("arch,H,W,classes,B,norm", [
    (100, 16, 16, 5, 4, True), (0, 8, 8, 10, 3, False), (1, 8, 8, 10, 4, False),
    (2, 8, 8, 10, 2, False), (3, 64, 64, 12, 3, True), (101, 2, 2, 2, 3, False),
    (4, 8, 8, 10, 4, False), (5, 8, 8, 10, 2, False)])
@pytest.mark.parametrize("reduction", ["sum", "mean"])
def test_network_matches_autograd_mirror(arch, H, W, classes, B, norm, reduction):
    if arch in (2, 3, 4, 5) and reduction == "mean":
        pytest.skip("one reduction is enough for the large nets")
    m, theta, x, y = _setup(arch, H, W, classes, B, norm=norm)
    loss, gx, gt = m.loss_f64(theta, x, y, reduction, want_grads=True)
    # the normalisation constants are fp32 values (mean_c, 1/std_c) in the reference
    mean = np.float32(MEAN).astype(np.float64) if norm else None
    std = 1.0 / (np.float32(1) / np.float32(STD)).astype(np.float64) if norm else None
    tl, tz, tgx, tgt = torch_mirror.loss_and_grads(arch, theta, x, y, classes, reduction, mean, std)
    assert abs(loss - tl) < 1e-9 * abs(tl)
    assert _rel(gx, tgx) < 1e-7
    assert _rel(gt, tgt) < 1e-7


@pytest.mark.parametrize("arch,H,W,classes,B", [(100, 16, 16, 5, 3), (0, 8, 8, 10, 2)])
def test_central_finite_differences(arch, H, W, classes, B):
    m, theta, x, y = _setup(arch, H, W, classes, B, cfg=11, norm=(arch == 100))
    loss, gx, gt = m.loss_f64(theta, x, y, "sum", want_grads=True)
    rng = np.random.default_rng(5)
    h = 1e-5
    # every parameter tensor gets probed at two coordinates
    idx = []
    for t in range(m.num_tensors):
        lo, hi = int(m.offsets[t]), int(m.offsets[t + 1])
        idx += list(rng.integers(lo, hi, size=2))
    for i in idx:
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h; tm[i] -= h
        fd = (m.loss_f64(tp, x, y, "sum") - m.loss_f64(tm, x, y, "sum")) / (2 * h)
        assert abs(fd - gt[i]) < 1e-6 * max(1.0, abs(gt[i])) + 2e-6 * np.abs(gt).max(), (i, fd, gt[i])
    flat = x.reshape(-1)
    for i in rng.integers(0, flat.size, size=25):
        xp, xm = flat.copy(), flat.copy()
        xp[i] += h; xm[i] -= h
        fd = (m.loss_f64(theta, xp.reshape(x.shape), y, "sum") - m.loss_f64(theta, xm.reshape(x.shape), y, "sum")) / (2 * h)
        assert abs(fd - gx.reshape(-1)[i]) < 2e-6 * np.abs(gx).max() + 1e-9, (i, fd, gx.reshape(-1)[i])


def test_fp32_entry_agrees_with_fp64_entry():
    m, theta, x, y = _setup(100, 16, 16, 5, 4, norm=True)
    m.set_params(theta.astype(np.float32))
    x32 = x.astype(np.float32)
    r = m.loss_grad(x32, y, "mean", want_gtheta=True)
    loss, gx, gt = m.loss_f64(theta.astype(np.float32).astype(np.float64), x32.astype(np.float64), y, "mean", want_grads=True)
    assert abs(r["loss"] - loss) < 1e-6
    assert _rel(r["gx"], gx) < 1e-5 and _rel(r["gtheta"], gt) < 1e-5


def test_gradient_is_a_batch_mean():
    # Eq. (stoch_grad_batch): duplicating the batch leaves the mean gradient unchanged (no BN here)
    m, theta, x, y = _setup(0, 8, 8, 10, 3)
    m.set_params(theta.astype(np.float32))
    g1, l1 = m.step(x.astype(np.float32), y)
    g2, l2 = m.step(np.concatenate([x, x]).astype(np.float32), np.concatenate([y, y]))
    assert abs(l1 - l2) < 1e-12 and _rel(g2, g1) < 1e-6


def test_bf16_storage_mode_rounds_and_stays_close():
    m32 = oracle.Model(100, 0, 16, 16, 5)
    m16 = oracle.Model(100, 1, 16, 16, 5)
    theta = syn.perturbed_params(3, m32.offsets, m32.fan_in, m32.kind)
    m32.set_params(theta); m16.set_params(theta)
    x, y = syn.images(3, 8, 16, 16), syn.labels(3, 8, 5)
    a = m32.loss_grad(x, y, "mean", want_gtheta=True)
    b = m16.loss_grad(x, y, "mean", want_gtheta=True)
    assert 0 < _rel(b["logits"], a["logits"]) < 0.05
    # gradients of a randomly initialised ReLU/BN net react strongly to 2^-9 storage rounding
    # (ReLU decisions flip); they stay well aligned with the fp64 gradient but not close
    for k in ("gx", "gtheta"):
        cos = float(np.dot(a[k].ravel(), b[k].ravel()) / (np.linalg.norm(a[k]) * np.linalg.norm(b[k])))
        assert 0.85 < cos < 1.0, (k, cos)
    # the input gradient is a stored bf16 tensor times 1/std-free scale: on the bf16 grid
    g = torch.tensor(b["gx"])
    assert torch.equal(g, g.to(torch.bfloat16).to(torch.float32))


def test_point_evaluators_agree_with_whole_tensor_convolution():
    rng = np.random.default_rng(9)
    for (k, stride, pad, H, W) in [(3, 1, 1, 6, 5), (3, 2, 1, 7, 8), (7, 2, 3, 12, 10), (1, 2, 0, 5, 5)]:
        B, Ci, Co = 2, 3, 4
        x = rng.standard_normal((B, H, W, Ci)).astype(np.float32)
        w = rng.standard_normal((Co, k, k, Ci)).astype(np.float32)
        y = oracle.conv_forward(x, w, stride, pad)
        dy = rng.standard_normal(y.shape).astype(np.float32)
        dx, dw = oracle.conv_backward(x, w, dy, stride, pad)
        for full, pts in ((y, oracle.conv_forward_points(x, w, stride, pad, np.arange(y.size))),
                          (dx, oracle.conv_backward_data_points(dy, w, (H, W), stride, pad, np.arange(dx.size))),
                          (dw, oracle.conv_backward_weight_points(x, dy, k, stride, pad, np.arange(dw.size)))):
            assert np.abs(full.reshape(-1) - pts).max() < 1e-12
