"""Pins for the reference's outer-minimisation oracle (LALR, Eq. (3); LAMB, Alg. A2) and the
server-side aggregation (Eq. (grad_agg))."""
import numpy as np

import oracle
import synth_inputs as syn


def _setup(T=7, cfg=2):
    off = syn.ragged_offsets(cfg, T, 300)
    rng = np.random.default_rng(cfg)
    d = int(off[-1])
    theta = rng.standard_normal(d).astype(np.float32) * 0.3
    g = rng.standard_normal(d).astype(np.float32) * 10.0 ** rng.uniform(-3, 0, d).astype(np.float32)
    return off, theta, g


def test_lalr_step_length_is_eta_times_tau():
    # Eq. (3): ||theta_{t+1,i} - theta_{t,i}|| = eta * tau(||theta_i||) exactly, whatever the gradient scale
    off, theta, g = _setup()
    theta[off[3]:off[4]] *= 100.0          # ||theta_i|| > c_u = 10: clipped from above
    eta = 0.05
    new, _, _ = oracle.lamb_update(theta, np.zeros_like(theta), np.zeros_like(theta), g, off, False, eta)
    for i in range(len(off) - 1):
        lo, hi = off[i], off[i + 1]
        step = np.linalg.norm(new[lo:hi].astype(np.float64) - theta[lo:hi])
        tau = min(max(np.linalg.norm(theta[lo:hi].astype(np.float64)), 0.0), 10.0)
        assert abs(step - eta * tau) < 1e-5 * eta * tau + 1e-9, i
        # direction is -g_i
        cos = -(new[lo:hi] - theta[lo:hi]).astype(np.float64) @ g[lo:hi] / (step * np.linalg.norm(g[lo:hi].astype(np.float64)) + 1e-300)
        assert cos > 1 - 1e-5


def test_lamb_first_step_is_sign_like_and_moments_follow_the_listing():
    off, theta, g = _setup()
    b1, b2, zeta, eta = 0.9, 0.999, 1e-6, 0.01
    new, m, v = oracle.lamb_update(theta, np.zeros_like(theta), np.zeros_like(theta), g, off, True, eta, b1, b2, zeta)
    assert np.allclose(m, (1 - b1) * g, rtol=1e-6) and np.allclose(v, (1 - b2) * g.astype(np.float64) ** 2, rtol=1e-6)
    # t = 1: bias-corrected m = g, v = g^2, so u = g/(|g| + zeta) ~ sign(g)
    for i in range(len(off) - 1):
        lo, hi = off[i], off[i + 1]
        u = g[lo:hi].astype(np.float64) / (np.abs(g[lo:hi].astype(np.float64)) + zeta)
        tau = min(np.linalg.norm(theta[lo:hi].astype(np.float64)), 10.0)
        want = theta[lo:hi] - eta * tau / np.linalg.norm(u) * u
        assert np.abs(new[lo:hi] - want).max() < 1e-6
    # second step against a straight numpy transcription with running moments
    g2 = np.roll(g, 5)
    new2, m2, v2 = oracle.lamb_update(new, m, v, g2, off, True, eta, b1, b2, zeta, t=2)
    mm = b1 * m.astype(np.float64) + (1 - b1) * g2
    vv = b2 * v.astype(np.float64) + (1 - b2) * g2.astype(np.float64) ** 2
    assert np.allclose(m2, mm, rtol=1e-6) and np.allclose(v2, vv, rtol=1e-6)
    u = (m2.astype(np.float64) / (1 - b1 ** 2)) / (np.sqrt(v2.astype(np.float64) / (1 - b2 ** 2)) + zeta)
    lo, hi = off[2], off[3]
    tau = min(np.linalg.norm(new[lo:hi].astype(np.float64)), 10.0)
    want = new[lo:hi] - eta * tau / np.linalg.norm(u[lo:hi]) * u[lo:hi]
    assert np.abs(new2[lo:hi] - want).max() < 1e-6


def test_zero_direction_leaves_layer_unchanged_and_weight_decay_enters_u():
    off, theta, g = _setup()
    g[off[1]:off[2]] = 0.0
    new, _, _ = oracle.lamb_update(theta, np.zeros_like(theta), np.zeros_like(theta), g, off, False, 0.1)
    assert np.array_equal(new[off[1]:off[2]], theta[off[1]:off[2]])
    new_wd, _, _ = oracle.lamb_update(theta, np.zeros_like(theta), np.zeros_like(theta), g, off, False, 0.1, wd=0.5)
    lo, hi = off[1], off[2]                                     # u = wd*theta: the layer shrinks along itself
    tau = min(np.linalg.norm(theta[lo:hi].astype(np.float64)), 10.0)
    want = theta[lo:hi].astype(np.float64) * (1 - 0.1 * tau / np.linalg.norm(theta[lo:hi].astype(np.float64)))
    assert np.abs(new_wd[lo:hi] - want).max() < 1e-6


def test_aggregate_is_mean_of_dequantized_and_unbiased():
    off, _, g = _setup(T=5, cfg=4)
    S = oracle.levels(8)
    M = 6
    cs, ss = zip(*[oracle.quantize(g * (1 + 0.1 * i), off, S, 100 + i) for i in range(M)])
    agg = oracle.aggregate(cs, ss, off, S)
    want = np.mean([oracle.dequantize(c, s, off, S).astype(np.float64) for c, s in zip(cs, ss)], axis=0)
    assert np.abs(agg - want).max() <= 1e-6 * np.abs(want).max()
    # M = 1 is plain dequantisation
    assert np.array_equal(oracle.aggregate(cs[:1], ss[:1], off, S), oracle.dequantize(cs[0], ss[0], off, S))
    # many workers holding the same gradient: the aggregate converges to it (Eq. E[Q(g)] = g)
    M2 = 16
    cs, ss = zip(*[oracle.quantize(g, off, oracle.levels(4), 500 + i) for i in range(M2)])
    agg = oracle.aggregate(cs, ss, off, oracle.levels(4))
    one = oracle.dequantize(cs[0], ss[0], off, oracle.levels(4))
    assert np.linalg.norm(agg - g) < 0.45 * np.linalg.norm(one - g)
