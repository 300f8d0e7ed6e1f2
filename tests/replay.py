"""Teacher-forced, op-by-op comparison of an implementation's stored tensors with the CPU reference.

A deep ReLU / batch-norm network at random initialisation amplifies a single flipped bf16 rounding into
percent-level changes of everything downstream, so an end-to-end comparison of two correct bf16
implementations cannot be tight.  Here every op is checked on its own: the reference evaluates op i from
the inputs the implementation under test actually had (its stored tensors are copied into the reference
after they have been compared), so each comparison sees one op's worth of rounding: the stored bf16
value is the rounding of an fp32 result that differs from the reference's fp64 result by accumulation
error only -- almost always the very same bf16 number, occasionally its neighbour.

`source` is any object with
    act(t)   -> stored activation tensor t as a flat array (uint16 bf16 bit patterns or float32), or None
    grad(t)  -> its gradient after the backward sweep, or None if the sweep did not leave it in memory
    bn(op)   -> (mean, rstd) float arrays of BN op `op`, or None
(the GPU library through its introspection calls, or a second reference instance in the CPU tests).
"""
import numpy as np

KIND_CONV, KIND_BIAS, KIND_BN, KIND_POOL, KIND_GAP, KIND_FC = range(6)

# Tolerances |got - ref| <= rel*|ref| + abs_frac*max|ref| per element.
#   bf16 tensors: one unit in the last place of an 8-bit significand is at most 2^-7 of the value; the absolute
#   term covers elements that are small only through cancellation (their fp32 accumulation error is
#   relative to the operands, not to the result).
TOL_BF16 = dict(rel=2.0 ** -7 * 1.001, abs_frac=2e-5)
#   fp32 tensors against fp64: accumulation error of sums of up to a few thousand terms.
TOL_F32 = dict(rel=2e-5, abs_frac=2e-6)


class Record(list):
    """Rows (name, n, exact, viol, worst, max_ref, max_err, nonfinite, composite).  composite: the comparison
    spans more than one op, because a tensor between two stored ones is never stored by the source; then ties
    (the arg-max of a pooling window between values one rounding apart) may legitimately fall differently."""

    def add(self, name, st, composite=False):
        self.append(dict(name=name, composite=bool(composite), **st))

    def worst(self, k=5):
        return sorted(self, key=lambda r: -r["viol"] / max(r["n"], 1))[:k]

    def summary(self):
        n = sum(r["n"] for r in self)
        return dict(items=len(self), elements=n, exact_frac=sum(r["exact"] for r in self) / max(n, 1),
                    viol=sum(r["viol"] for r in self), max_viol_frac=max((r["viol"] / max(r["n"], 1) for r in self), default=0.0),
                    nonfinite=sum(r["nonfinite"] for r in self))


def check(rec, act_viol_frac=5e-5, grad_viol_frac=1e-3, worst_cap=100.0):
    """The acceptance rule of the GPU comparisons: statistics and parameter gradients meet their bar everywhere; a
    stored activation (gradient) tensor may miss it in at most act_viol_frac (grad_viol_frac) of its elements, and
    where one op separates the two sides by no more than the factor worst_cap (tests/test_gpu_replay.py says why)."""
    def limit(r):
        if " act t" in r["name"]:
            return act_viol_frac * r["n"]
        if " grad t" in r["name"] or "gradient" in r["name"]:
            return grad_viol_frac * r["n"]
        return 0
    bad = [r for r in rec if r["nonfinite"] or r["viol"] > limit(r) or (r["worst"] > worst_cap and not r["composite"])]
    assert not bad, [(r["name"], r["n"], r["viol"], r["worst"]) for r in bad[:8]]


def _tol(arr):
    return TOL_BF16 if arr.dtype == np.uint16 else TOL_F32


def _cmp_small(got, ref, rel, abs_frac):
    """numpy version of the element-wise test for small vectors (statistics, parameter gradients)."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    mx = float(np.abs(ref).max()) if ref.size else 0.0
    err = np.abs(got - ref)
    tol = rel * np.abs(ref) + abs_frac * mx
    bad = ~np.isfinite(got)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(err > 0, err / tol, 0.0)
    return dict(n=int(ref.size), exact=int((err == 0).sum()), viol=int(((err > tol) | bad).sum()),
                worst=float(np.nanmax(ratio)) if ref.size else 0.0, max_ref=mx, max_err=float(err.max()) if ref.size else 0.0,
                nonfinite=int(bad.sum()), worst_index=int(np.nanargmax(ratio)) if ref.size else -1)


def forward(ref, source, x, rec, force=True):
    """Runs the reference forward op by op from pixels x; compares, then (force) adopts, every tensor the
    source has stored.  Batch statistics of every BN are compared too."""
    ref.begin(x)
    ops = ref.ops()
    shapes = ref.tensor_shapes()
    own = set()          # tensors the reference computed itself and the source could not replace
    for i, op in enumerate(ops):
        ref.forward_op(i)
        t = op["out"]
        composite = op["in"] in own or op["res"] in own
        if op["kind"] == KIND_BN:
            st = source.bn(i)
            if st is not None:
                mean, rstd = ref.bn_stats(i, shapes[op["in"]][2])
                # the mean is compared on the scale of the channel's spread (1/rstd)
                spread = 1.0 / rstd
                e = np.abs(np.asarray(st[0], np.float64) - mean) / spread
                rec.add("op%d bn mean" % i, dict(n=e.size, exact=int((e == 0).sum()), viol=int((e > 2e-5).sum()), worst=float(e.max() / 2e-5),
                                                 max_ref=float(np.abs(mean).max()), max_err=float(e.max()), nonfinite=int((~np.isfinite(st[0])).sum()), worst_index=int(e.argmax())))
                rec.add("op%d bn rstd" % i, _cmp_small(st[1], rstd, 2e-5, 0.0))
        got = source.act(t)
        if got is None:
            own.add(t)
            continue
        rec.add("op%d kind%d act t%d %s" % (i, op["kind"], t, shapes[t]), ref.compare_tensor(0, t, got, **_tol(got)), composite)
        if force:
            ref.set_tensor(0, t, got)
    return own


def backward(ref, source, y, scale, want_wgrad, rec, force=True, own_acts=(), logit_grad=None):
    """After `forward` (own_acts: what it returned): installs the loss gradient (scale 1 = sum over the batch,
    1/B = mean; or `logit_grad`, the expected gradient of another loss w.r.t. the logits, flat fp32), then runs the
    reference backward op by op.  A tensor's gradient is complete once every op that
    reads the tensor has run; at that point it is compared with the source's and (force) replaced by it.
    Returns (mean loss, whether the comparison of the pixel gradient spans more than one op)."""
    ops = ref.ops()
    own_acts = set(own_acts) - {0}
    own = set()          # gradients the source could not supply
    mixed = set()        # gradient tensors with a contribution computed from such a gradient or activation
    shapes = ref.tensor_shapes()
    first_reader = {}
    for i, op in enumerate(ops):
        for t in (op["in"], op["res"]):
            if t >= 0 and t not in first_reader:
                first_reader[t] = i
    loss = ref.loss_backward_begin(y, scale)
    if logit_grad is not None:
        ref.set_tensor(1, ops[-1]["out"], np.ascontiguousarray(logit_grad, np.float32).reshape(-1))

    def settle(t, name):
        got = source.grad(t) if t != 0 else None
        if got is None:
            own.add(t)
            return
        rec.add(name, ref.compare_tensor(1, t, got, **_tol(got)), t in mixed)
        if force:
            ref.set_tensor(1, t, got)

    settle(ops[-1]["out"], "logit gradient t%d" % ops[-1]["out"])
    for i in range(len(ops) - 1, -1, -1):
        op = ops[i]
        ref.backward_op(i, want_wgrad)
        if op["out"] in own or ({op["in"], op["out"], op["res"]} & own_acts):
            mixed.update({op["in"], op["res"]} - {-1})
        for t in sorted({op["in"], op["res"]} - {-1}):
            if first_reader[t] == i:
                settle(t, "op%d kind%d grad t%d %s" % (i, op["kind"], t, shapes[t]))
    return loss, (0 in mixed)


def param_grads(ref, got, rec, rel=1e-4, abs_frac=1e-4):
    """Per parameter tensor: the source's gradient vector against the reference's accumulated one."""
    want = ref.param_grads()
    got = np.asarray(got, np.float64)
    for t in range(ref.num_tensors):
        lo, hi = int(ref.offsets[t]), int(ref.offsets[t + 1])
        rec.add("param tensor %d kind %d (%d)" % (t, int(ref.kind[t]), hi - lo), _cmp_small(got[lo:hi], want[lo:hi], rel, abs_frac))


def pixel_grad(ref, gx_got, rec, bf16, composite=False):
    want = ref.pixel_grad(gx_got.shape)
    tol = TOL_BF16 if bf16 else TOL_F32
    rec.add("pixel gradient", _cmp_small(gx_got.reshape(-1), want.reshape(-1), **tol), composite)


class ReferenceSource:
    """A second reference instance posing as the implementation under test (CPU tests): runs an ordinary,
    unforced pass and serves its tensors in storage format.  `tamper(which, t, array)` may alter what is served."""

    def __init__(self, model, x, y, scale, want_wgrad, bf16, tamper=None, missing=()):
        self.m, self.bf16, self.tamper, self.missing = model, bf16, tamper, set(missing)
        model.begin(x)
        self.ops = model.ops()
        for i in range(len(self.ops)):
            model.forward_op(i)
        self.stats = {i: model.bn_stats(i, model.tensor_shapes()[op["in"]][2]) for i, op in enumerate(self.ops) if op["kind"] == KIND_BN}
        self.acts = {t: model.get_tensor(0, t) for t in range(len(model.tensor_shapes()))}
        self.loss = model.loss_backward_begin(y, scale)
        for i in range(len(self.ops) - 1, -1, -1):
            model.backward_op(i, want_wgrad)
        self.grads = {t: model.get_tensor(1, t) for t in range(len(model.tensor_shapes())) if model.grad_present(t)}
        self.f32_tensors = {self.ops[-1]["out"], self.ops[-1]["in"]}   # logits and pooled features stay fp32

    def _serve(self, which, t, a):
        if a is None or (which, t) in self.missing:
            return None
        a = a.copy()
        if self.tamper is not None:
            a = self.tamper(which, t, a)
        if self.bf16 and t not in self.f32_tensors:
            return (a.view(np.uint32) >> 16).astype(np.uint16)      # values are bf16-exact: truncation is exact
        return a

    def act(self, t):
        return self._serve(0, t, self.acts.get(t))

    def grad(self, t):
        return self._serve(1, t, self.grads.get(t))

    def bn(self, op):
        mean, rstd = self.stats[op]
        return mean.astype(np.float32), rstd.astype(np.float32)


class GpuSource:
    """The GPU library's stored tensors through its introspection calls."""

    def __init__(self, gpu, B):
        self.gpu, self.B = gpu, B
        self.refresh()

    def refresh(self):
        self.info = self.gpu.inspect_tensors()

    def act(self, t):
        return self.gpu.inspect_read(0, t, self.B, self.info[t]) if self.info[t]["act_stored"] else None

    def grad(self, t):
        return self.gpu.inspect_read(1, t, self.B, self.info[t]) if self.info[t]["grad_stored"] else None

    def bn(self, op):
        return self.gpu.inspect_bn(op, self.info[self.gpu.inspect_ops()[op]["in"]]["C"])
