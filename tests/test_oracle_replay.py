"""The op-by-op stepping interface of the CPU reference and the teacher-forced comparison built on it
(tests/replay.py), checked on the CPU: stepping reproduces the whole-network entry points bit for bit, a
faithful source passes with every element exactly equal, and planted mistakes of the kind a kernel bug would
produce (a zeroed input gradient, a flipped sign, a 2 % scale error, a dropped residual, wrong batch statistics)
are flagged at the tensor they were planted in."""
import numpy as np
import pytest

import oracle
import synth_inputs as syn
from tests import replay

MEAN, STD = (0.485, 0.456, 0.406), (0.229, 0.224, 0.225)
CASES = [(100, 8, 16, 16, 5), (3, 3, 64, 64, 12), (2, 4, 8, 8, 10)]


def _setup(arch, B, H, W, classes, bf16=1, cfg=61):
    def make():
        m = oracle.Model(arch, bf16, H, W, classes, MEAN, STD)
        m.set_params(syn.perturbed_params(cfg, m.offsets, m.fan_in, m.kind))
        return m
    return make, syn.images(cfg, B, H, W), syn.labels(cfg, B, classes)


@pytest.mark.parametrize("arch,B,H,W,classes", CASES)
def test_stepping_reproduces_the_whole_network_entry_points(arch, B, H, W, classes):
    make, x, y = _setup(arch, B, H, W, classes)
    whole = make().loss_grad(x, y, "mean", want_gtheta=True)
    m = make()
    m.begin(x)
    n = len(m.ops())
    for i in range(n):
        m.forward_op(i)
    loss = m.loss_backward_begin(y, 1.0 / B)
    for i in range(n - 1, -1, -1):
        m.backward_op(i, True)
    assert loss == whole["loss"]
    assert np.array_equal(m.get_tensor(0, m.ops()[-1]["out"]).reshape(B, classes), whole["logits"])
    assert np.array_equal(m.pixel_grad(x.shape), whole["gx"])
    assert np.array_equal(m.param_grads().astype(np.float32), whole["gtheta"])


@pytest.mark.parametrize("arch,B,H,W,classes", CASES)
@pytest.mark.parametrize("bf16", [0, 1])
def test_faithful_source_is_exactly_equal_everywhere(arch, B, H, W, classes, bf16):
    make, x, y = _setup(arch, B, H, W, classes, bf16)
    # the source also leaves out some tensors, as fused GPU passes do: the comparison then spans two ops
    src = replay.ReferenceSource(make(), x, y, 1.0, True, bool(bf16), missing={(0, 2), (1, 2), (1, 5)})
    ref = make()
    rec = replay.Record()
    replay.forward(ref, src, x, rec)
    loss, _ = replay.backward(ref, src, y, 1.0, True, rec)
    # (tensors kept in fp32 -- all of them in an fp32 model, pooled features and logits in a bf16 model -- are served
    # rounded once from fp64, so the reference restarts from slightly different values there)
    replay.param_grads(ref, src.m.param_grads(), rec, rel=1e-5, abs_frac=1e-5)
    assert abs(loss - src.loss) < 1e-6 * src.loss
    s = rec.summary()
    assert s["viol"] == 0 and s["nonfinite"] == 0 and s["items"] > 40
    if bf16:    # every bf16-stored tensor is reproduced exactly
        import re
        for r in rec:
            hit = re.search(r" t(\d+) ", r["name"])
            if hit and int(hit.group(1)) not in src.f32_tensors:
                assert r["exact"] == r["n"], r
    assert max(r["worst"] for r in rec) < 0.05


def _find(ops, kind, nth=0, **want):
    hits = [i for i, op in enumerate(ops) if op["kind"] == kind and all(op[k] == v for k, v in want.items())]
    return hits[nth]


def _flagged(rec, needle):
    rows = [r for r in rec if needle in r["name"]]
    assert rows, needle
    return max(r["viol"] / r["n"] for r in rows)


def test_planted_mistakes_are_flagged():
    arch, B, H, W, classes = 100, 8, 16, 16, 5
    make, x, y = _setup(arch, B, H, W, classes)
    ops = make().ops()
    bn_res = _find(ops, replay.KIND_BN, 0, relu=1, res=[op["res"] for op in ops if op["kind"] == replay.KIND_BN and op["res"] >= 0][0])
    conv3 = _find(ops, replay.KIND_CONV, 3)
    bn2 = _find(ops, replay.KIND_BN, 2)

    def run(tamper, want_wgrad=True):
        src = replay.ReferenceSource(make(), x, y, 1.0, want_wgrad, True, tamper=tamper)
        ref = make()
        rec = replay.Record()
        replay.forward(ref, src, x, rec)
        replay.backward(ref, src, y, 1.0, want_wgrad, rec)
        return rec

    # (1) the input gradient of a batch normalisation written as zeros
    t_in = ops[bn2]["in"]
    rec = run(lambda which, t, a: np.zeros_like(a) if (which, t) == (1, t_in) else a)
    assert _flagged(rec, "grad t%d " % t_in) > 0.5
    # (2) a convolution's input gradient with the wrong sign
    t_in = ops[conv3]["in"]
    rec = run(lambda which, t, a: -a if (which, t) == (1, t_in) else a)
    assert _flagged(rec, "grad t%d " % t_in) > 0.5
    # (3) an activation tensor off by 2 % (more than one bf16 unit in the last place); values stay bf16-exact
    t_out = ops[conv3]["out"]
    def scale(which, t, a):
        if (which, t) != (0, t_out):
            return a
        b = (a * np.float32(1.02)).view(np.uint32)
        return ((b + 0x8000) & 0xFFFF0000).astype(np.uint32).view(np.float32)
    rec = run(scale)
    assert _flagged(rec, "act t%d " % t_out) > 0.5
    # (4) the residual left out of a block's output: out = relu(bn(y)) instead of relu(bn(y) + r)
    t_out, t_res = ops[bn_res]["out"], ops[bn_res]["res"]
    keep = {}
    def no_res(which, t, a):
        if which == 0 and t == t_res:
            keep["r"] = a.copy()
        if (which, t) == (0, t_out):
            return np.maximum(a - keep["r"], 0).astype(np.float32)
        return a
    rec = run(no_res)
    assert _flagged(rec, "act t%d " % t_out) > 0.2
    # (5) untampered control: nothing is flagged
    rec = run(lambda which, t, a: a)
    assert rec.summary()["viol"] == 0


def test_wrong_batch_statistics_are_flagged():
    """Unbiased instead of biased variance moves rstd by 1/(2M): invisible in a bf16 output, caught by the
    comparison of the statistics themselves."""
    arch, B, H, W, classes = 100, 8, 16, 16, 5
    make, x, y = _setup(arch, B, H, W, classes)
    src = replay.ReferenceSource(make(), x, y, 1.0, False, True)
    ops = src.ops
    bn0 = _find(ops, replay.KIND_BN, 0)
    rows = B * H * W
    mean, rstd = src.stats[bn0]
    var = 1.0 / rstd ** 2 - 1e-5
    src.stats[bn0] = (mean, 1.0 / np.sqrt(var * rows / (rows - 1) + 1e-5))
    ref = make()
    rec = replay.Record()
    replay.forward(ref, src, x, rec)
    assert _flagged(rec, "op%d bn rstd" % bn0) == 1.0
    assert sum(r["viol"] for r in rec if "rstd" not in r["name"]) == 0


@pytest.mark.parametrize("arch,B,H,W,classes", [(100, 8, 16, 16, 5), (1, 6, 16, 16, 10)])
@pytest.mark.parametrize("lam", [0.0, 1.5])
def test_trades_objective_through_the_stepping_calls(arch, B, H, W, classes, lam):
    """The TRADES step is three forward and two backward sweeps with the logit gradients of kl_logit_grad installed:
    done through the stepping interface it reproduces step_reg (whose gradients are pinned in
    tests/test_oracle_objective.py), so a teacher-forced comparison may install these logit gradients."""
    make, x, y = _setup(arch, B, H, W, classes)
    xadv = oracle.make_xadv(x, oracle.init_delta(x, np.float32(8 / 255), oracle.INIT_UNIFORM, seed=3))
    g_whole, l_whole = make().step_reg(x, xadv, y, lam, 1)
    m = make()
    n, t = len(m.ops()), m.ops()[-1]["out"]

    def sweep(inp):
        m.begin(inp)
        for i in range(n):
            m.forward_op(i)
        return m.get_tensor(0, t).reshape(B, classes)

    def back(dz):
        m.loss_backward_begin(y, 1.0)
        m.set_tensor(1, t, dz.reshape(-1))
        for i in range(n - 1, -1, -1):
            m.backward_op(i, True)
        return m.param_grads()

    zc = sweep(x)
    za = sweep(xadv)
    dz0, kl = oracle.kl_logit_grad(zc, za, None, 0.0, 0, 1.0 / B)
    g = back(dz0)
    zc2 = sweep(x)
    assert np.array_equal(zc2, zc)
    dz1, _ = oracle.kl_logit_grad(zc, za, y, lam, 1, 1.0 / B)
    g = g + back(dz1)
    assert abs(kl - l_whole[1]) <= 1e-6 * abs(l_whole[1]) + 1e-12
    # (the logits pass through fp32 on the way into kl_logit_grad, the whole-network entry keeps them in fp64)
    err = np.abs(g - g_whole).max() / np.abs(g_whole).max()
    assert err < 2e-6, err
    # each branch matters: leaving one out is far outside the tolerance
    assert np.abs(back(dz1) - g_whole).max() / np.abs(g_whole).max() > 1e-2
