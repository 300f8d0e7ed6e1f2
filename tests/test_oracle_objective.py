"""Pins for the reference's general worker objective (Eq. (prob_DAT)): lambda * clean loss + phi, with
phi the adversarial cross-entropy or the TRADES KL regulariser.  Nothing here touches the GPU."""
import numpy as np
import pytest

import oracle
import synth_inputs as syn
from tests import torch_mirror

MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)


def _rel(a, b):
    return float(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)).max() / (np.abs(b).max() + 1e-300))


def _setup(arch, H, classes, B, cfg, norm=False, eps=8 / 255):
    m = oracle.Model(arch, 0, H, H, classes, MEAN if norm else None, STD if norm else None)
    theta = syn.perturbed_params(cfg, m.offsets, m.fan_in, m.kind).astype(np.float64)
    x = syn.images(cfg, B, H, H)
    y = syn.labels(cfg, B, classes)
    d = oracle.init_delta(x, eps, oracle.INIT_UNIFORM, seed=cfg)
    xadv = oracle.make_xadv(x, d)
    return m, theta, x.astype(np.float64), xadv.astype(np.float64), y


@pytest.mark.parametrize("arch,H,classes,B,norm", [(100, 16, 5, 4, True), (0, 8, 10, 3, False), (4, 8, 10, 4, False)])
@pytest.mark.parametrize("lam,phi", [(0.0, 0), (0.7, 0), (0.0, 1), (1.5, 1)])
def test_objective_matches_autograd_mirror(arch, H, classes, B, norm, lam, phi):
    m, theta, x, xadv, y = _setup(arch, H, classes, B, cfg=31, norm=norm)
    Fv, gt, gx = m.objective_f64(theta, x, xadv, y, lam, phi, want_gtheta=True, want_gxadv=True)
    mean = np.float32(MEAN).astype(np.float64) if norm else None
    std = 1.0 / (np.float32(1) / np.float32(STD)).astype(np.float64) if norm else None
    tF, tgt, tgx = torch_mirror.objective_and_grads(arch, theta, x, xadv, y, classes, lam, phi, mean, std)
    assert abs(Fv - tF) < 1e-9 * max(abs(tF), 1e-3)
    assert _rel(gt, tgt) < 1e-7
    assert _rel(gx, tgx) < 1e-7


def test_labeled_objective_without_clean_term_is_the_plain_step():
    # lambda = 0, phi = CE is Alg. A1 step 6 as it was
    m, theta, x, xadv, y = _setup(100, 16, 5, 4, cfg=32, norm=True)
    m.set_params(theta.astype(np.float32))
    g0, l0 = m.step(xadv.astype(np.float32), y)
    g1, losses = m.step_reg(x.astype(np.float32), xadv.astype(np.float32), y, 0.0, oracle.PHI_CE)
    assert np.array_equal(g0, g1) and abs(losses[1] - l0) < 1e-12 and losses[0] == 0.0


def test_objective_is_affine_in_lambda():
    m, theta, x, xadv, y = _setup(100, 16, 5, 4, cfg=33, norm=True)
    for phi in (0, 1):
        F0, g0, _ = m.objective_f64(theta, x, xadv, y, 0.0, phi, want_gtheta=True)
        F1, g1, _ = m.objective_f64(theta, x, xadv, y, 1.0, phi, want_gtheta=True)
        F3, g3, _ = m.objective_f64(theta, x, xadv, y, 3.0, phi, want_gtheta=True)
        clean, _, gclean = m.loss_f64(theta, x, y, "mean", want_grads=True)
        assert abs((F1 - F0) - clean) < 1e-12 * max(1.0, abs(clean))
        assert abs((F3 - F0) - 3 * clean) < 1e-11 * max(1.0, abs(clean))
        assert _rel(g1 - g0, gclean) < 1e-9 and _rel(g3 - g0, 3 * gclean) < 1e-9


def test_kl_regulariser_closed_forms():
    m, theta, x, xadv, y = _setup(100, 16, 5, 4, cfg=34, norm=True)
    # at delta = 0 the two passes coincide: phi = 0, and so is its gradient w.r.t. the perturbed pixels
    F, gt, gx = m.objective_f64(theta, x, x, y, 0.0, 1, want_gtheta=True, want_gxadv=True)
    assert F == 0.0 and np.abs(gx).max() == 0.0
    # ... and the parameter gradients of the two branches cancel
    assert np.abs(gt).max() < 1e-12
    # phi >= 0 (Gibbs) away from delta = 0
    F, _, _ = m.objective_f64(theta, x, xadv, y, 0.0, 1)
    assert F > 0.0


@pytest.mark.parametrize("phi,lam", [(1, 0.0), (1, 0.8), (0, 0.8)])
def test_objective_central_finite_differences(phi, lam):
    m, theta, x, xadv, y = _setup(100, 16, 5, 3, cfg=35, norm=True)
    F, gt, gx = m.objective_f64(theta, x, xadv, y, lam, phi, want_gtheta=True, want_gxadv=True)
    rng = np.random.default_rng(6)
    h = 1e-5
    idx = []
    for t in range(m.num_tensors):
        idx += list(rng.integers(int(m.offsets[t]), int(m.offsets[t + 1]), size=1))
    for i in idx:
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h; tm[i] -= h
        fd = (m.objective_f64(tp, x, xadv, y, lam, phi)[0] - m.objective_f64(tm, x, xadv, y, lam, phi)[0]) / (2 * h)
        assert abs(fd - gt[i]) < 1e-6 * max(1.0, abs(gt[i])) + 2e-6 * np.abs(gt).max(), (i, fd, gt[i])
    if phi == 1 and lam == 0.0:
        # derivative of sum_n phi_n w.r.t. the perturbed pixels; the clean pass does not depend on them
        flat = xadv.reshape(-1)
        B = x.shape[0]
        for i in rng.integers(0, flat.size, size=12):
            xp, xm = flat.copy(), flat.copy()
            xp[i] += h; xm[i] -= h
            fd = B * (m.objective_f64(theta, x, xp.reshape(x.shape), y, 0.0, 1)[0] -
                      m.objective_f64(theta, x, xm.reshape(x.shape), y, 0.0, 1)[0]) / (2 * h)
            assert abs(fd - gx.reshape(-1)[i]) < 2e-6 * np.abs(gx).max() + 1e-9, (i, fd, gx.reshape(-1)[i])


def test_kl_attack_invariants_and_ascent():
    m, theta, x, xadv, y = _setup(0, 8, 10, 4, cfg=36)
    m.set_params(theta.astype(np.float32))
    x32 = x.astype(np.float32)
    eps, alpha = np.float32(8 / 255), np.float32(2 / 255)
    d, tr = m.attack_kl(x32, eps, alpha, 5, oracle.INIT_UNIFORM, seed=3, trace=True)
    assert np.abs(d).max() <= eps and (x32 + d).min() >= 0 and (x32 + d).max() <= 1
    assert tr["loss"][-1] > tr["loss"][0] >= 0.0
    # every step is one application of the shared update to the KL input gradient
    for k in range(5):
        G, _ = m.phi_input_grad(x32, oracle.make_xadv(x32, tr["delta"][k]), y, oracle.PHI_TRADES_KL)
        assert np.array_equal(oracle.pgd_update(x32, G, tr["delta"][k], eps, alpha), tr["delta"][k + 1])
    # a zero start is a fixed point: the KL gradient vanishes where the two passes coincide
    d0 = m.attack_kl(x32, eps, alpha, 3, oracle.INIT_ZERO)
    assert np.abs(d0).max() == 0.0
