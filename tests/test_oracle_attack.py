"""Pins for the reference's inner maximisation (Eq. (1); unified PGD/FGSM update of Sec.
"Methodologies") and its fp32 perturbation arithmetic."""
import itertools

import numpy as np

import oracle
import synth_inputs as syn

EPS, ALPHA = 8 / 255, 2 / 255


def _tiny(B=6, H=8):
    m = oracle.Model(oracle.ARCH_TINYCNN, 0, H, H, 10)
    m.set_params(syn.perturbed_params(1, m.offsets, m.fan_in, m.kind))
    return m, syn.images(1, B, H, H), syn.labels(1, B, 10)


def test_invariants_linf_ball_and_valid_image():
    m, x, y = _tiny()
    x[0, :2] = 0.0          # pixels at the box boundary
    x[1, :2] = 1.0
    for init in (oracle.INIT_ZERO, oracle.INIT_UNIFORM):
        d = m.attack(x, y, EPS, ALPHA, 7, init, seed=3)
        assert np.abs(d).max() <= np.float32(EPS)               # exact, fp32
        assert (x + d).min() >= 0.0 and (x + d).max() <= 1.0
        assert np.abs(d).max() > 0.9 * EPS


def test_k0_returns_init_and_uniform_init_statistics():
    m, x, y = _tiny(B=64, H=8)
    x[:] = 0.5   # far from the [0,1] boundary: the init is not clipped
    d0 = m.attack(x, y, EPS, ALPHA, 0, oracle.INIT_ZERO)
    assert not d0.any()
    d = m.attack(x, y, EPS, ALPHA, 0, oracle.INIT_UNIFORM, seed=9)
    assert np.array_equal(d, oracle.init_delta(x, EPS, oracle.INIT_UNIFORM, 9))
    u = d / np.float32(EPS)                                       # ~ U(-1,1)
    n = u.size
    assert abs(u.mean()) < 4 / np.sqrt(3 * n) and abs(u.var() - 1 / 3) < 0.01
    assert u.min() >= -1 and u.max() < 1
    given = (syn.images(2, 64, 8, 8) - 0.5) * 0.2
    dg = m.attack(x, y, EPS, ALPHA, 0, oracle.INIT_GIVEN, delta0=given)
    assert np.array_equal(dg, np.clip(given, -np.float32(EPS), np.float32(EPS)))


def test_fgsm_is_one_step_pgd_from_zero():
    # K = 1, z0 = 0, alpha = eps: delta = eps * sign(grad), clipped to the image box
    m, x, y = _tiny()
    d = m.attack(x, y, EPS, EPS, 1, oracle.INIT_ZERO)
    g = m.loss_grad(x, y, "sum")["gx"]
    want = np.clip(np.float32(EPS) * np.sign(g), -x, np.float32(1) - x).astype(np.float32)
    assert np.array_equal(d, want)


def test_pgd_is_the_composition_of_single_steps():
    m, x, y = _tiny()
    d, tr = m.attack(x, y, EPS, ALPHA, 4, oracle.INIT_UNIFORM, seed=5, trace=True)
    cur = oracle.init_delta(x, EPS, oracle.INIT_UNIFORM, 5)
    for k in range(4):
        assert np.array_equal(tr["delta"][k], cur)
        g = m.loss_grad(oracle.make_xadv(x, cur), y, "sum")["gx"]
        assert np.array_equal(g, tr["grad"][k])
        nxt = np.clip(cur + np.float32(ALPHA) * np.sign(g), -np.float32(EPS), np.float32(EPS)).astype(np.float32)
        nxt = np.minimum(np.maximum(nxt, -x), np.float32(1) - x)
        cur = oracle.pgd_update(x, g, cur, EPS, ALPHA)
        assert np.array_equal(cur, nxt)
    assert np.array_equal(cur, d)
    # sign steps do not guarantee monotone ascent per sample; the batch loss does go up here
    assert tr["loss"][-1] > tr["loss"][0]


def test_sign_of_zero_gradient_leaves_delta():
    x = np.full((1, 2, 2, 3), 0.5, np.float32)
    g = np.zeros_like(x); g[0, 0, 0, 0] = 1.0; g[0, 0, 0, 1] = -1.0; g[0, 0, 0, 2] = -0.0
    d0 = np.full_like(x, 0.01)
    d = oracle.pgd_update(x, g, d0, EPS, ALPHA)
    assert d[0, 0, 0, 0] == np.float32(0.01) + np.float32(ALPHA)
    assert d[0, 0, 0, 1] == np.float32(0.01) - np.float32(ALPHA)
    assert np.array_equal(d.reshape(-1)[2:], d0.reshape(-1)[2:])


def test_linear_two_class_model_fgsm_is_exact_maximiser():
    # GAP + linear layer, 2 classes: the loss is monotone in a margin that is linear in delta,
    # so the box maximum sits at the corner eps*sign(grad).  Brute force over all 2^12 corners.
    m = oracle.Model(oracle.ARCH_LINEAR, 0, 2, 2, 2)
    theta = syn.perturbed_params(4, m.offsets, m.fan_in, m.kind)
    m.set_params(theta)
    x = (0.3 + 0.4 * syn.images(4, 1, 2, 2)).astype(np.float32)
    y = np.array([1], np.int32)
    d = m.attack(x, y, EPS, EPS, 1, oracle.INIT_ZERO)
    best = m.loss_grad(x + d, y, "sum", want_gx=False)["loss"]
    worst_gap = -1.0
    for corner in itertools.product((-1.0, 1.0), repeat=12):
        dd = (np.float32(EPS) * np.array(corner, np.float32)).reshape(x.shape)
        worst_gap = max(worst_gap, m.loss_grad(x + dd, y, "sum", want_gx=False)["loss"] - best)
    assert worst_gap <= 1e-12
    assert best > m.loss_grad(x, y, "sum", want_gx=False)["loss"]


def test_eps_zero_reduces_to_standard_training_gradient():
    # M = 1, lambda = 0, phi = l with eps = 0 is ordinary training (remark after Eq. (2))
    m, x, y = _tiny()
    d = m.attack(x, y, 0.0, 0.0, 3, oracle.INIT_UNIFORM, seed=1)
    assert not d.any()
    g_adv, _ = m.step(oracle.make_xadv(x, d), y)
    g_std = m.loss_grad(x, y, "mean", want_gtheta=True)["gtheta"]
    assert np.array_equal(g_adv, g_std)


def test_sgd_step_on_master_weights():
    m, x, y = _tiny()
    p0 = m.get_params()
    g, _ = m.step(x, y)
    m.sgd_update(g, 0.1)
    assert np.array_equal(m.get_params(), p0 - np.float32(0.1) * g)
