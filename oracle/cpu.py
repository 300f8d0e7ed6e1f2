"""ctypes wrapper around oracle/libdat_oracle.so (argument marshalling only)."""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdat_oracle.so")

ARCH_TINYCNN, ARCH_RESNET18_CIFAR, ARCH_WRN34_10, ARCH_RESNET50, ARCH_TESTNET, ARCH_LINEAR = 0, 1, 2, 3, 100, 101
ARCH_PREACT_RESNET18, ARCH_WRN28_10 = 4, 5
INIT_ZERO, INIT_UNIFORM, INIT_GIVEN = 0, 1, 2
PHI_CE, PHI_TRADES_KL = 0, 1


def build(force=False):
    """Compile the reference with g++ (make); a no-op when it is up to date."""
    cmd = ["make", "-C", _HERE] + (["-B"] if force else [])
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL)


def _load():
    src = os.path.join(_HERE, "dat_oracle.cpp")
    if not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        build()
    return C.CDLL(_LIB_PATH)


_lib = _load()

_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")


def _sig(name, res, *args):
    f = getattr(_lib, name)
    f.restype = res
    f.argtypes = list(args)
    return f


_create = _sig("orc_model_create", C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p)
_destroy = _sig("orc_model_destroy", None, C.c_void_p)
_jitter = _sig("orc_set_accum_jitter", None, C.c_void_p, C.c_double)
_num_params = _sig("orc_num_params", C.c_int64, C.c_void_p)
_num_tensors = _sig("orc_num_tensors", C.c_int, C.c_void_p)
_table = _sig("orc_tensor_table", None, C.c_void_p, _i64p, _i32p, _i32p)
_set_params = _sig("orc_set_params", None, C.c_void_p, _f32p)
_get_params = _sig("orc_get_params", None, C.c_void_p, _f32p)
_loss_grad = _sig("orc_loss_grad", C.c_double, C.c_void_p, _f32p, _i32p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p)
_loss_f64 = _sig("orc_loss_f64", C.c_double, C.c_void_p, _f64p, _f64p, _i32p, C.c_int, C.c_int, C.c_void_p, C.c_void_p)
_init_delta = _sig("orc_init_delta", None, _f32p, C.c_int64, C.c_float, C.c_int, C.c_uint64, C.c_void_p, _f32p)
_pgd_update = _sig("orc_pgd_update", None, _f32p, _f32p, _f32p, C.c_int64, C.c_float, C.c_float)
_make_xadv = _sig("orc_make_xadv", None, _f32p, _f32p, _f32p, C.c_int64)
_attack = _sig("orc_attack", None, C.c_void_p, _f32p, _i32p, C.c_int, C.c_float, C.c_float, C.c_int, C.c_int,
               C.c_uint64, C.c_void_p, _f32p, C.c_void_p, C.c_void_p, C.c_void_p)
_step = _sig("orc_step", C.c_double, C.c_void_p, _f32p, _i32p, C.c_int, _f32p)
_step_reg = _sig("orc_step_reg", None, C.c_void_p, _f32p, _f32p, _i32p, C.c_int, C.c_double, C.c_int, _f32p, _f64p)
_phi_gx = _sig("orc_phi_input_grad", C.c_double, C.c_void_p, _f32p, _f32p, _i32p, C.c_int, C.c_int, _f32p)
_obj_f64 = _sig("orc_objective_f64", C.c_double, C.c_void_p, _f64p, _f64p, _f64p, _i32p, C.c_int, C.c_double, C.c_int,
                C.c_void_p, C.c_void_p)
_attack_kl = _sig("orc_attack_kl", None, C.c_void_p, _f32p, C.c_int, C.c_float, C.c_float, C.c_int, C.c_int, C.c_uint64,
                  C.c_void_p, _f32p, C.c_void_p, C.c_void_p)
_sgd = _sig("orc_sgd_update", None, C.c_void_p, _f32p, C.c_float)
_quant = _sig("orc_quantize", None, _f32p, _i64p, C.c_int, C.c_int, C.c_uint64, C.c_int, _i32p, _f32p)
_dequant = _sig("orc_dequantize", None, _i32p, _f32p, _i64p, C.c_int, C.c_int, _f32p)
_pack = _sig("orc_pack", None, _i32p, C.c_int64, C.c_int, _u8p)
_unpack = _sig("orc_unpack", None, _u8p, C.c_int64, C.c_int, _i32p)
_philox = _sig("orc_philox", None, _u32p, _u32p, _u32p)
_uniform = _sig("orc_uniform", None, C.c_uint64, C.c_int64, C.c_uint64, C.c_uint32, _f32p)
_rbf16 = _sig("orc_round_bf16", C.c_double, C.c_double)
_conv_f = _sig("orc_conv_forward", None, _f64p, _f64p, _f64p, *([C.c_int] * 8))
_conv_b = _sig("orc_conv_backward", None, _f64p, _f64p, _f64p, _f64p, _f64p, *([C.c_int] * 8))
_pts = [_sig(n, None, _f32p, _f32p, *([C.c_int] * 8), _i64p, C.c_int, _f64p)
        for n in ("orc_conv_forward_points", "orc_conv_bwd_data_points", "orc_conv_bwd_weight_points")]
_lamb = _sig("orc_lamb_update", None, _f32p, _f32p, _f32p, _f32p, _i64p, C.c_int, C.c_int, *([C.c_double] * 7), C.c_int)
_aggregate = _sig("orc_aggregate", None, C.c_void_p, C.c_void_p, C.c_int, _i64p, C.c_int, C.c_int, _f32p)
_threads = _sig("orc_threads", C.c_int)
_num_ops = _sig("orc_num_ops", C.c_int, C.c_void_p)
_num_act = _sig("orc_num_act_tensors", C.c_int, C.c_void_p)
_op_info = _sig("orc_op_info", None, C.c_void_p, C.c_int, _i32p)
_tshape = _sig("orc_tensor_shape", None, C.c_void_p, C.c_int, _i32p)
_begin = _sig("orc_begin", None, C.c_void_p, _f32p, C.c_int)
_fwd_op = _sig("orc_forward_op", None, C.c_void_p, C.c_int)
_loss_bwd = _sig("orc_loss_backward_begin", C.c_double, C.c_void_p, _i32p, C.c_double)
_bwd_op = _sig("orc_backward_op", None, C.c_void_p, C.c_int, C.c_int)
_grad_present = _sig("orc_grad_present", C.c_int, C.c_void_p, C.c_int)
_get_tensor = _sig("orc_get_tensor", None, C.c_void_p, C.c_int, C.c_int, _f32p)
_set_tensor = _sig("orc_set_tensor", None, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int)
_cmp_tensor = _sig("orc_compare_tensor", None, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_double, C.c_double, _f64p)
_bn_stats = _sig("orc_get_bn_stats", None, C.c_void_p, C.c_int, _f64p, _f64p)
_param_grads = _sig("orc_get_param_grads", None, C.c_void_p, _f64p)
_pixel_grad = _sig("orc_pixel_grad", None, C.c_void_p, _f32p)
_kl_dz = _sig("orc_kl_logit_grad", None, _f32p, _f32p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_int, C.c_double, _f32p, _f64p)


def _opt(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Model:
    """One network (architecture + parameters) of the reference."""

    def __init__(self, arch, bf16_storage, H, W, num_classes, mean=None, std=None):
        m = None if mean is None else np.asarray(mean, np.float32)
        s = None if std is None else np.asarray(std, np.float32)
        self._h = _create(arch, int(bool(bf16_storage)), H, W, num_classes, _opt(m), _opt(s))
        if not self._h:
            raise ValueError("unknown architecture %r" % (arch,))
        self.H, self.W, self.classes = H, W, num_classes
        self.d = int(_num_params(self._h))
        self.num_tensors = int(_num_tensors(self._h))
        self.offsets = np.zeros(self.num_tensors + 1, np.int64)
        self.fan_in = np.zeros(self.num_tensors, np.int32)
        self.kind = np.zeros(self.num_tensors, np.int32)
        _table(self._h, self.offsets, self.fan_in, self.kind)

    def __del__(self):
        if getattr(self, "_h", None):
            _destroy(self._h)
            self._h = None

    def set_accum_jitter(self, rel):
        """Relative pseudo-random factor applied to every convolution sum (summation-order model)."""
        _jitter(self._h, float(rel))

    def set_params(self, flat):
        flat = np.ascontiguousarray(flat, np.float32)
        assert flat.size == self.d
        _set_params(self._h, flat)

    def get_params(self):
        out = np.zeros(self.d, np.float32)
        _get_params(self._h, out)
        return out

    def loss_grad(self, x, y, reduction="sum", want_logits=True, want_gx=True, want_gtheta=False):
        x = np.ascontiguousarray(x, np.float32)
        y = np.ascontiguousarray(y, np.int32)
        B = x.shape[0]
        logits = np.zeros((B, self.classes), np.float32) if want_logits else None
        gx = np.zeros_like(x) if want_gx else None
        gt = np.zeros(self.d, np.float32) if want_gtheta else None
        loss = _loss_grad(self._h, x, y, B, 0 if reduction == "sum" else 1, _opt(logits), _opt(gx), _opt(gt))
        return dict(loss=loss, logits=logits, gx=gx, gtheta=gt)

    def loss_f64(self, theta, x, y, reduction="sum", want_grads=False):
        theta = np.ascontiguousarray(theta, np.float64)
        x = np.ascontiguousarray(x, np.float64)
        y = np.ascontiguousarray(y, np.int32)
        B = x.shape[0]
        gx = np.zeros_like(x) if want_grads else None
        gt = np.zeros(self.d, np.float64) if want_grads else None
        loss = _loss_f64(self._h, theta, x, y, B, 0 if reduction == "sum" else 1, _opt(gx), _opt(gt))
        return (loss, gx, gt) if want_grads else loss

    def attack(self, x, y, eps, alpha, K, init=INIT_ZERO, seed=0, delta0=None, trace=False):
        x = np.ascontiguousarray(x, np.float32)
        y = np.ascontiguousarray(y, np.int32)
        B = x.shape[0]
        delta = np.zeros_like(x)
        d0 = None if delta0 is None else np.ascontiguousarray(delta0, np.float32)
        losses = np.zeros(K + 1, np.float32) if trace else None
        dtr = np.zeros((K + 1,) + x.shape, np.float32) if trace else None
        gtr = np.zeros((K,) + x.shape, np.float32) if trace else None
        _attack(self._h, x, y, B, eps, alpha, K, init, seed, _opt(d0), delta, _opt(losses), _opt(dtr), _opt(gtr))
        if trace:
            return delta, dict(loss=losses, delta=dtr, grad=gtr)
        return delta

    def step(self, x_adv, y):
        x_adv = np.ascontiguousarray(x_adv, np.float32)
        y = np.ascontiguousarray(y, np.int32)
        g = np.zeros(self.d, np.float32)
        loss = _step(self._h, x_adv, y, x_adv.shape[0], g)
        return g, loss

    def step_reg(self, x, x_adv, y, lam, phi):
        """Worker gradient of lam*CE(x) + phi (batch mean); returns (grads, [mean clean CE, mean phi])."""
        x = np.ascontiguousarray(x, np.float32)
        x_adv = np.ascontiguousarray(x_adv, np.float32)
        y = np.ascontiguousarray(y, np.int32)
        g = np.zeros(self.d, np.float32)
        losses = np.zeros(2, np.float64)
        _step_reg(self._h, x, x_adv, y, x.shape[0], float(lam), int(phi), g, losses)
        return g, losses

    def phi_input_grad(self, x, x_adv, y, phi):
        """Gradient of sum_n phi_n w.r.t. the perturbed pixels (clean pass constant); returns (gx, mean phi)."""
        x = np.ascontiguousarray(x, np.float32)
        x_adv = np.ascontiguousarray(x_adv, np.float32)
        y = np.ascontiguousarray(y, np.int32)
        gx = np.zeros_like(x)
        loss = _phi_gx(self._h, x, x_adv, y, x.shape[0], int(phi), gx)
        return gx, loss

    def objective_f64(self, theta, x, x_adv, y, lam, phi, want_gtheta=False, want_gxadv=False):
        theta = np.ascontiguousarray(theta, np.float64)
        x = np.ascontiguousarray(x, np.float64)
        x_adv = np.ascontiguousarray(x_adv, np.float64)
        y = np.ascontiguousarray(y, np.int32)
        gt = np.zeros(self.d, np.float64) if want_gtheta else None
        gx = np.zeros_like(x) if want_gxadv else None
        F = _obj_f64(self._h, theta, x, x_adv, y, x.shape[0], float(lam), int(phi), _opt(gt), _opt(gx))
        return F, gt, gx

    def attack_kl(self, x, eps, alpha, K, init=INIT_UNIFORM, seed=0, delta0=None, trace=False):
        x = np.ascontiguousarray(x, np.float32)
        B = x.shape[0]
        delta = np.zeros_like(x)
        d0 = None if delta0 is None else np.ascontiguousarray(delta0, np.float32)
        losses = np.zeros(K + 1, np.float32) if trace else None
        dtr = np.zeros((K + 1,) + x.shape, np.float32) if trace else None
        _attack_kl(self._h, x, B, eps, alpha, K, init, seed, _opt(d0), delta, _opt(losses), _opt(dtr))
        if trace:
            return delta, dict(loss=losses, delta=dtr)
        return delta

    def sgd_update(self, grads, lr):
        _sgd(self._h, np.ascontiguousarray(grads, np.float32), lr)

    # ---- op-by-op stepping (teacher-forced comparisons); which: 0 activations, 1 gradients ----
    def ops(self):
        """List of dicts (kind, in, out, res, k, stride, pad, relu, p0, p1), in op order."""
        names = ("kind", "in", "out", "res", "k", "stride", "pad", "relu", "p0", "p1")
        out = []
        for i in range(int(_num_ops(self._h))):
            info = np.zeros(10, np.int32)
            _op_info(self._h, i, info)
            out.append(dict(zip(names, (int(v) for v in info))))
        return out

    def tensor_shapes(self):
        out = []
        for t in range(int(_num_act(self._h))):
            hwc = np.zeros(3, np.int32)
            _tshape(self._h, t, hwc)
            out.append(tuple(int(v) for v in hwc))
        return out

    def begin(self, x):
        x = np.ascontiguousarray(x, np.float32)
        self._B = x.shape[0]
        _begin(self._h, x, self._B)

    def forward_op(self, i):
        _fwd_op(self._h, i)

    def loss_backward_begin(self, y, scale):
        return float(_loss_bwd(self._h, np.ascontiguousarray(y, np.int32), float(scale)))

    def backward_op(self, i, want_wgrad):
        _bwd_op(self._h, i, int(bool(want_wgrad)))

    def grad_present(self, t):
        return int(_grad_present(self._h, t))

    def _numel(self, t):
        hwc = np.zeros(3, np.int32)
        _tshape(self._h, t, hwc)
        return self._B * int(hwc[0]) * int(hwc[1]) * int(hwc[2])

    def get_tensor(self, which, t):
        out = np.zeros(self._numel(t), np.float32)
        _get_tensor(self._h, which, t, out)
        return out

    def set_tensor(self, which, t, values):
        """values: float32 array, or uint16 array of bf16 bit patterns."""
        values = np.ascontiguousarray(values)
        assert values.size == self._numel(t) and values.dtype in (np.float32, np.uint16), (values.size, values.dtype)
        _set_tensor(self._h, which, t, values.ctypes.data_as(C.c_void_p), int(values.dtype == np.uint16))

    def compare_tensor(self, which, t, got, rel, abs_frac):
        """Element-wise |got - ref| <= rel*|ref| + abs_frac*max|ref|; returns a dict of counts and maxima."""
        got = np.ascontiguousarray(got)
        assert got.size == self._numel(t) and got.dtype in (np.float32, np.uint16), (got.size, got.dtype)
        st = np.zeros(8, np.float64)
        _cmp_tensor(self._h, which, t, got.ctypes.data_as(C.c_void_p), int(got.dtype == np.uint16), float(rel), float(abs_frac), st)
        return dict(n=int(st[0]), exact=int(st[1]), viol=int(st[2]), worst=float(st[3]), max_ref=float(st[4]),
                    max_err=float(st[5]), nonfinite=int(st[6]), worst_index=int(st[7]))

    def bn_stats(self, op_index, C_):
        mean, rstd = np.zeros(C_, np.float64), np.zeros(C_, np.float64)
        _bn_stats(self._h, op_index, mean, rstd)
        return mean, rstd

    def param_grads(self):
        out = np.zeros(self.d, np.float64)
        _param_grads(self._h, out)
        return out

    def pixel_grad(self, shape):
        out = np.zeros(shape, np.float32)
        _pixel_grad(self._h, out.reshape(-1))
        return out


def kl_logit_grad(z_clean, z_adv, y, lam, branch, scale):
    """Logit gradient of sum_n scale * [lam * CE(z_clean_n, y_n) + KL(p(z_clean_n) || p(z_adv_n))] w.r.t. the perturbed
    pass's logits (branch 0) or the clean pass's (branch 1), from given fp32 logits [B, classes].  Returns (dz, mean KL)."""
    zc = np.ascontiguousarray(z_clean, np.float32); za = np.ascontiguousarray(z_adv, np.float32)
    assert zc.ndim == 2 and zc.shape == za.shape
    yy = None if y is None else np.ascontiguousarray(y, np.int32)
    assert yy is not None or (lam == 0.0 or branch == 0)
    dz = np.zeros_like(zc)
    kl = np.zeros(1, np.float64)
    _kl_dz(zc, za, None if yy is None else yy.ctypes.data, zc.shape[0], zc.shape[1], float(lam), int(branch), float(scale), dz, kl)
    return dz, float(kl[0])


def init_delta(x, eps, mode, seed=0, given=None):
    x = np.ascontiguousarray(x, np.float32)
    out = np.zeros_like(x)
    g = None if given is None else np.ascontiguousarray(given, np.float32)
    _init_delta(x.reshape(-1), x.size, eps, mode, seed, _opt(g), out.reshape(-1))
    return out


def pgd_update(x, G, delta, eps, alpha):
    x = np.ascontiguousarray(x, np.float32)
    G = np.ascontiguousarray(G, np.float32)
    d = np.array(delta, np.float32, copy=True, order="C")
    _pgd_update(x.reshape(-1), G.reshape(-1), d.reshape(-1), x.size, eps, alpha)
    return d


def make_xadv(x, delta):
    x = np.ascontiguousarray(x, np.float32)
    delta = np.ascontiguousarray(delta, np.float32)
    out = np.zeros_like(x)
    _make_xadv(x.reshape(-1), delta.reshape(-1), out.reshape(-1), x.size)
    return out


def levels(bits):
    """Code magnitudes per sign for b-bit signed codes: S = 2^(b-1) - 1."""
    return (1 << (bits - 1)) - 1


def quantize(g, offsets, S, seed, use_l2=False):
    g = np.ascontiguousarray(g, np.float32)
    offsets = np.ascontiguousarray(offsets, np.int64)
    T = offsets.size - 1
    codes = np.zeros(g.size, np.int32)
    scales = np.zeros(T, np.float32)
    _quant(g, offsets, T, S, seed, int(use_l2), codes, scales)
    return codes, scales


def dequantize(codes, scales, offsets, S):
    codes = np.ascontiguousarray(codes, np.int32)
    scales = np.ascontiguousarray(scales, np.float32)
    offsets = np.ascontiguousarray(offsets, np.int64)
    out = np.zeros(codes.size, np.float32)
    _dequant(codes, scales, offsets, offsets.size - 1, S, out)
    return out


def pack(codes, bits):
    codes = np.ascontiguousarray(codes, np.int32)
    n = (codes.size * bits + 7) // 8
    q = np.zeros(n, np.uint8)
    _pack(codes, codes.size, bits, q)
    return q


def unpack(q, d, bits):
    q = np.ascontiguousarray(q, np.uint8)
    codes = np.zeros(d, np.int32)
    _unpack(q, d, bits, codes)
    return codes


def philox4x32_10(counter, key):
    c = np.ascontiguousarray(counter, np.uint32)
    k = np.ascontiguousarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    _philox(c, k, out)
    return out


def uniform(start, n, seed, stream):
    out = np.zeros(n, np.float32)
    _uniform(start, n, seed, stream, out)
    return out


def round_bf16(v):
    return float(_rbf16(float(v)))


def conv_forward(x, w, stride, pad):
    """x [B,H,W,Ci] fp64, w [Co,k,k,Ci] fp64 -> [B,Ho,Wo,Co]."""
    x = np.ascontiguousarray(x, np.float64)
    w = np.ascontiguousarray(w, np.float64)
    B, H, W, Ci = x.shape
    Co, k = w.shape[0], w.shape[1]
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    out = np.zeros((B, Ho, Wo, Co), np.float64)
    _conv_f(x, w, out, B, H, W, Ci, Co, k, stride, pad)
    return out


def conv_backward(x, w, dout, stride, pad):
    x = np.ascontiguousarray(x, np.float64)
    w = np.ascontiguousarray(w, np.float64)
    dout = np.ascontiguousarray(dout, np.float64)
    B, H, W, Ci = x.shape
    Co, k = w.shape[0], w.shape[1]
    din = np.zeros_like(x)
    dw = np.zeros_like(w)
    _conv_b(x, w, dout, din, dw, B, H, W, Ci, Co, k, stride, pad)
    return din, dw


def _points(which, a, b, geom, idx):
    a = np.ascontiguousarray(a, np.float32)
    b = np.ascontiguousarray(b, np.float32)
    idx = np.ascontiguousarray(idx, np.int64)
    out = np.zeros(idx.size, np.float64)
    _pts[which](a.reshape(-1), b.reshape(-1), *geom, idx, idx.size, out)
    return out


def conv_forward_points(x, w, stride, pad, idx):
    """Selected elements (flat indices into y[B,Ho,Wo,Co]) of conv(x, w), from the definition."""
    B, H, W, Ci = x.shape
    return _points(0, x, w, (B, H, W, Ci, w.shape[0], w.shape[1], stride, pad), idx)


def conv_backward_data_points(dy, w, in_hw, stride, pad, idx):
    """Selected elements (flat indices into dx[B,H,W,Ci]) of the adjoint w.r.t. the input."""
    B = dy.shape[0]
    return _points(1, dy, w, (B, in_hw[0], in_hw[1], w.shape[3], w.shape[0], w.shape[1], stride, pad), idx)


def conv_backward_weight_points(x, dy, k, stride, pad, idx):
    """Selected elements (flat indices into dw[Co,k,k,Ci]) of the adjoint w.r.t. the weights."""
    B, H, W, Ci = x.shape
    return _points(2, x, dy, (B, H, W, Ci, dy.shape[3], k, stride, pad), idx)


def lamb_update(theta, m, v, g, offsets, use_adam, eta, b1=0.9, b2=0.999, zeta=1e-6, wd=0.0, c_l=0.0, c_u=10.0, t=1):
    """In-place on copies: returns (theta, m, v) after one LALR/LAMB step (Eq. (3), Alg. A2)."""
    theta = np.array(theta, np.float32, copy=True); m = np.array(m, np.float32, copy=True); v = np.array(v, np.float32, copy=True)
    g = np.ascontiguousarray(g, np.float32); offsets = np.ascontiguousarray(offsets, np.int64)
    _lamb(theta, m, v, g, offsets, offsets.size - 1, int(use_adam), eta, b1, b2, zeta, wd, c_l, c_u, t)
    return theta, m, v


def aggregate(codes_list, scales_list, offsets, S):
    """g_hat = (1/M) sum_i dequantize(codes_i, scales_i)  (Eq. (grad_agg))."""
    M = len(codes_list)
    codes_list = [np.ascontiguousarray(c, np.int32) for c in codes_list]
    scales_list = [np.ascontiguousarray(s, np.float32) for s in scales_list]
    offsets = np.ascontiguousarray(offsets, np.int64)
    cp = (C.c_void_p * M)(*[c.ctypes.data for c in codes_list])
    sp = (C.c_void_p * M)(*[s.ctypes.data for s in scales_list])
    out = np.zeros(codes_list[0].size, np.float32)
    _aggregate(cp, sp, M, offsets, offsets.size - 1, S, out)
    return out


def threads():
    return int(_threads())
