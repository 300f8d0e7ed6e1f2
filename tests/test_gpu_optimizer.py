"""GPU parity of the steps that follow the worker block: aggregation of M quantized gradients
(Eq. (grad_agg), bit exact) and the LALR / LAMB parameter update (Eq. (3), Alg. A2)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as syn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _cuda(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("bits,M", [(8, 6), (4, 3), (2, 2), (16, 1), (8, 32)])
def test_aggregate_bit_exact(dat, bits, M):
    off = syn.ragged_offsets(40 + bits, 23, 3000)
    g = syn.stress_gradient(40 + bits, off)
    d, S = g.size, oracle.levels(bits)
    od = _cuda(off)
    qs, scs, cs, ss = [], [], [], []
    for i in range(M):
        gi = (g * np.float32(1 + 0.07 * i)).astype(np.float32)
        c, s = oracle.quantize(gi, off, S, 900 + i)
        q, sc = dat.quantize(_cuda(gi), od, bits, 900 + i)
        assert np.array_equal(q.cpu().numpy(), oracle.pack(c, bits))
        qs.append(q); scs.append(sc); cs.append(c); ss.append(s)
    got = dat.aggregate(qs, scs, od, d, bits).cpu().numpy()
    assert np.array_equal(got, oracle.aggregate(cs, ss, off, S))


@pytest.mark.parametrize("use_adam", [False, True])
def test_lamb_update_matches_reference(dat, use_adam):
    model = dat.Model(dat.ARCH_TESTNET, dat.BF16, 2, 16, 16, 5)
    off = model.offsets
    theta = syn.perturbed_params(8, off, model.fan_in, model.kind)
    t_big = int(np.argmax(np.diff(off)))
    theta[off[t_big]:off[t_big + 1]] *= 40.0           # a layer with ||theta|| > c_u
    model.set_params(theta)
    rng = np.random.default_rng(0)
    ref_theta, m, v = theta.copy(), np.zeros_like(theta), np.zeros_like(theta)
    for step in (1, 2, 3):
        g = (rng.standard_normal(theta.size) * 10.0 ** rng.uniform(-4, 0, theta.size)).astype(np.float32)
        if step == 2:
            g[off[1]:off[2]] = 0.0
        model.lamb_update(_cuda(g), 0.02, use_adam=use_adam, weight_decay=1e-4, t=step)
        ref_theta, m, v = oracle.lamb_update(ref_theta, m, v, g, off, use_adam, 0.02, wd=1e-4, t=step)
        got = model.get_params()
        for t in range(len(off) - 1):
            lo, hi = off[t], off[t + 1]
            err = np.abs(got[lo:hi] - ref_theta[lo:hi]).max()
            assert err <= 2e-6 * max(np.abs(ref_theta[lo:hi]).max(), 1e-3), (step, t, err)
    model.close()
