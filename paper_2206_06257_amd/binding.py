"""ctypes binding of libdat.so with the same names as include/dat.h (without the dat_ prefix on
methods of Model).  Raises if the library has not been built: there is no fallback path."""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdat.so")

ARCH_TINYCNN, ARCH_RESNET18_CIFAR, ARCH_WRN34_10, ARCH_RESNET50, ARCH_TESTNET = 0, 1, 2, 3, 100
ARCH_PREACT_RESNET18, ARCH_WRN28_10 = 4, 5
PHI_CE, PHI_TRADES_KL = 0, 1
F32, BF16 = 0, 1
INIT_ZERO, INIT_UNIFORM, INIT_GIVEN = 0, 1, 2

EXPORTS = [
    "dat_model_create", "dat_model_destroy", "dat_model_num_params", "dat_model_tensor_table",
    "dat_model_offsets_device", "dat_model_set_params", "dat_model_get_params", "dat_attack", "dat_step",
    "dat_input_grad", "dat_pgd_init", "dat_pgd_update", "dat_sgd_update", "dat_quantize", "dat_dequantize",
    "dat_quantized_bytes", "dat_conv_forward", "dat_conv_backward_data", "dat_conv_backward_weight",
    "dat_status_string", "dat_last_error", "dat_philox_uniform", "dat_profile_enable", "dat_profile_read", "dat_aggregate", "dat_lamb_update",
    "dat_attack_kl", "dat_step_reg", "dat_model_set_option", "dat_make_xadv",
    "dat_conv_backward_weight_static", "dat_conv_backward_weight_static_limit", "dat_set_kernel_option", "dat_model_grad_scales", "dat_quantize_scaled",
    "dat_inspect_counts", "dat_inspect_op", "dat_inspect_tensor", "dat_inspect_read", "dat_inspect_bn",
]


class DatError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        msg = _lib.dat_status_string(status).decode()
        extra = _lib.dat_last_error().decode()
        super().__init__("%s: %s (%d)%s" % (where, msg, self.status, (" -- " + extra) if extra and self.status in (5, 6) else ""))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libdat.so is not built: run `python -m paper_2206_06257_amd.build` "
                          "(or __graft_entry__.build()) first; there is no CPU fallback")
    return C.CDLL(LIB_PATH)


_lib = _load()


class _Init(C.Structure):
    _fields_ = [("mode", C.c_int), ("seed", C.c_uint64), ("delta0", C.c_void_p)]


_vp, _i, _i64, _f, _u64 = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_uint64
_lib.dat_status_string.restype = C.c_char_p
_lib.dat_status_string.argtypes = [_i]
_lib.dat_last_error.restype = C.c_char_p
_lib.dat_model_create.argtypes = [_i, _i, _i, _i, _i, _i, _vp, _vp, C.POINTER(_vp)]
_lib.dat_model_destroy.argtypes = [_vp]
_lib.dat_model_num_params.argtypes = [_vp, C.POINTER(_i64), C.POINTER(_i)]
_lib.dat_model_tensor_table.argtypes = [_vp, _vp, _vp, _vp]
_lib.dat_model_offsets_device.restype = _vp
_lib.dat_model_offsets_device.argtypes = [_vp]
_lib.dat_model_set_params.argtypes = [_vp, _vp]
_lib.dat_model_get_params.argtypes = [_vp, _vp]
_lib.dat_attack.argtypes = [_vp, _vp, _vp, _i, _f, _f, _i, _Init, _vp, _vp, _vp]
_lib.dat_step.argtypes = [_vp, _vp, _vp, _i, _vp, _vp, _vp]
_lib.dat_input_grad.argtypes = [_vp, _vp, _vp, _i, _vp, _vp, _vp, _vp]
_lib.dat_pgd_init.argtypes = [_vp, _i64, _f, _Init, _vp, _vp]
_lib.dat_pgd_update.argtypes = [_vp, _vp, _vp, _i64, _f, _f, _vp]
_lib.dat_make_xadv.argtypes = [_vp, _vp, _i64, _vp, _vp]
_lib.dat_sgd_update.argtypes = [_vp, _vp, _f, _vp]
_lib.dat_quantize.argtypes = [_vp, _vp, _i, _i64, _i, _u64, _vp, _vp, _vp]
_lib.dat_dequantize.argtypes = [_vp, _vp, _vp, _i, _i64, _i, _vp, _vp]
_lib.dat_quantize_scaled.argtypes = [_vp, _vp, _i, _i64, _i, _u64, _vp, _vp, _vp]
_lib.dat_model_grad_scales.argtypes = [_vp, C.POINTER(_vp)]
_lib.dat_quantized_bytes.restype = C.c_size_t
_lib.dat_quantized_bytes.argtypes = [_i64, _i]
_lib.dat_conv_backward_weight_static_limit.restype = C.c_size_t
_lib.dat_conv_backward_weight_static_limit.argtypes = []
for _n in ("dat_conv_forward", "dat_conv_backward_data", "dat_conv_backward_weight", "dat_conv_backward_weight_static"):
    getattr(_lib, _n).argtypes = [_vp, _vp, _vp] + [_i] * 8 + [_vp]
_lib.dat_philox_uniform.argtypes = [_u64, _i64, _u64, C.c_uint32, _vp, _vp]
_lib.dat_aggregate.argtypes = [_vp, _vp, _i, _vp, _i, _i64, _i, _vp, _vp]
_lib.dat_lamb_update.argtypes = [_vp, _vp, _i, _f, _f, _f, _f, _f, _f, _f, _i, _vp]
_lib.dat_attack_kl.argtypes = [_vp, _vp, _i, _f, _f, _i, _Init, _vp, _vp, _vp]
_lib.dat_step_reg.argtypes = [_vp, _vp, _vp, _vp, _i, _f, _i, _vp, _vp, _vp]
_lib.dat_profile_enable.argtypes = [_vp, _i]
_lib.dat_inspect_counts.argtypes = [_vp, C.POINTER(_i), C.POINTER(_i)]
_lib.dat_inspect_op.argtypes = [_vp, _i, _vp]
_lib.dat_inspect_tensor.argtypes = [_vp, _i, _vp]
_lib.dat_inspect_read.argtypes = [_vp, _i, _i, _i, _vp, C.c_size_t]
_lib.dat_inspect_bn.argtypes = [_vp, _i, _vp, _vp]
_lib.dat_model_set_option.argtypes = [_vp, _i, _i]
OPT_FUSE_BN_INPUT_GRAD = 0
OPT_FUSE_BN_SUMS = 1
OPT_FUSE_PGD_GRADIENT = 2
OPT_SPARSE_SHORTCUT_GRADIENT = 3
OPT_OVERLAP_WEIGHT_GRADIENTS = 4
OPT_ABSORB_SHORTCUT_BN = 5
OPT_FUSE_STEM_POOL = 6
OPT_GRADIENT_SCALES = 7
OPT_KEEP_BOTH_PASSES = 8
KOPT_RING_KERNEL = 0
KOPT_TILE_160 = 1
KOPT_NARROW_UNDERFILLED = 2
_lib.dat_set_kernel_option.argtypes = [_i, _i]
_lib.dat_profile_read.argtypes = [_vp, _i, C.POINTER(C.c_double), C.POINTER(_i64), C.POINTER(C.c_double)]
PROF_CLASSES = ("conv_fwd", "conv_bwd_data", "conv_wgrad", "bn", "pgd", "conv_bwd_data_bn")


def _check(status, where):
    if status != 0:
        raise DatError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dev(t, dtype):
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, (t.device, t.dtype, dtype)
    return t


def _init(mode, seed, delta0):
    return _Init(int(mode), int(seed) & 0xFFFFFFFFFFFFFFFF, None if delta0 is None else delta0.data_ptr())


class Model:
    """dat_model handle: one architecture with its device parameters and workspace."""

    def __init__(self, arch, dtype, max_batch, H, W, num_classes, mean=None, std=None):
        h = _vp()
        m = None if mean is None else np.ascontiguousarray(mean, np.float32)
        s = None if std is None else np.ascontiguousarray(std, np.float32)
        _check(_lib.dat_model_create(arch, dtype, max_batch, H, W, num_classes,
                                     None if m is None else m.ctypes.data, None if s is None else s.ctypes.data,
                                     C.byref(h)), "dat_model_create")
        self._h = h
        self.arch, self.dtype, self.max_batch, self.H, self.W, self.classes = arch, dtype, max_batch, H, W, num_classes
        d, nt = _i64(), _i()
        _check(_lib.dat_model_num_params(h, C.byref(d), C.byref(nt)), "dat_model_num_params")
        self.d, self.num_tensors = d.value, nt.value
        self.offsets = np.zeros(self.num_tensors + 1, np.int64)
        self.fan_in = np.zeros(self.num_tensors, np.int32)
        self.kind = np.zeros(self.num_tensors, np.int32)
        _check(_lib.dat_model_tensor_table(h, self.offsets.ctypes.data, self.fan_in.ctypes.data, self.kind.ctypes.data),
               "dat_model_tensor_table")
        self.offsets_device_ptr = _lib.dat_model_offsets_device(h)

    def close(self):
        # (at interpreter shutdown the module globals may already be gone: the process is ending anyway)
        if getattr(self, "_h", None) and _lib is not None:
            _lib.dat_model_destroy(self._h)
            self._h = None

    __del__ = close

    def set_params(self, flat):
        flat = np.ascontiguousarray(flat, np.float32)
        assert flat.size == self.d
        _check(_lib.dat_model_set_params(self._h, flat.ctypes.data), "dat_model_set_params")

    def get_params(self):
        out = np.zeros(self.d, np.float32)
        _check(_lib.dat_model_get_params(self._h, out.ctypes.data), "dat_model_get_params")
        return out

    def attack(self, x, y, eps, alpha, K, init=INIT_ZERO, seed=0, delta0=None, delta=None, want_losses=False, stream=None):
        _dev(x, torch.float32); _dev(y, torch.int32)
        B = x.shape[0]
        if delta is None:
            delta = torch.empty_like(x)
        losses = np.zeros(K + 1, np.float32) if want_losses else None
        _check(_lib.dat_attack(self._h, _ptr(x), _ptr(y), B, eps, alpha, K, _init(init, seed, delta0), _ptr(delta),
                               None if losses is None else losses.ctypes.data, _stream(stream)), "dat_attack")
        return (delta, losses) if want_losses else delta

    def step(self, x_adv, y, grads=None, want_loss=False, stream=None):
        _dev(x_adv, torch.float32); _dev(y, torch.int32)
        if grads is None:
            grads = torch.empty(self.d, dtype=torch.float32, device=x_adv.device)
        loss = C.c_float(0.0)
        _check(_lib.dat_step(self._h, _ptr(x_adv), _ptr(y), x_adv.shape[0], _ptr(grads),
                             C.byref(loss) if want_loss else None, _stream(stream)), "dat_step")
        return (grads, loss.value) if want_loss else grads

    def attack_kl(self, x, eps, alpha, K, init=INIT_UNIFORM, seed=0, delta0=None, delta=None, want_losses=False, stream=None):
        _dev(x, torch.float32)
        if delta is None:
            delta = torch.empty_like(x)
        losses = np.zeros(K + 1, np.float32) if want_losses else None
        _check(_lib.dat_attack_kl(self._h, _ptr(x), x.shape[0], eps, alpha, K, _init(init, seed, delta0), _ptr(delta),
                                  None if losses is None else losses.ctypes.data, _stream(stream)), "dat_attack_kl")
        return (delta, losses) if want_losses else delta

    def step_reg(self, x, x_adv, y, lam, phi, grads=None, want_losses=False, stream=None):
        _dev(x, torch.float32); _dev(x_adv, torch.float32); _dev(y, torch.int32)
        if grads is None:
            grads = torch.empty(self.d, dtype=torch.float32, device=x.device)
        losses = np.zeros(2, np.float32) if want_losses else None
        _check(_lib.dat_step_reg(self._h, _ptr(x), _ptr(x_adv), _ptr(y), x.shape[0], lam, int(phi), _ptr(grads),
                                 None if losses is None else losses.ctypes.data, _stream(stream)), "dat_step_reg")
        return (grads, losses) if want_losses else grads

    def input_grad(self, x, y, want_logits=True, want_loss=True, stream=None):
        _dev(x, torch.float32); _dev(y, torch.int32)
        gx = torch.empty_like(x)
        logits = torch.empty(x.shape[0], self.classes, dtype=torch.float32, device=x.device) if want_logits else None
        loss = C.c_float(0.0)
        _check(_lib.dat_input_grad(self._h, _ptr(x), _ptr(y), x.shape[0], _ptr(gx), _ptr(logits),
                                   C.byref(loss) if want_loss else None, _stream(stream)), "dat_input_grad")
        return gx, logits, (loss.value if want_loss else None)

    def sgd_update(self, grads, lr, stream=None):
        _check(_lib.dat_sgd_update(self._h, _ptr(_dev(grads, torch.float32)), lr, _stream(stream)), "dat_sgd_update")

    def lamb_update(self, grads, eta, use_adam=True, beta1=0.9, beta2=0.999, zeta=1e-6, weight_decay=0.0, c_l=0.0, c_u=10.0,
                    t=1, stream=None):
        _check(_lib.dat_lamb_update(self._h, _ptr(_dev(grads, torch.float32)), int(bool(use_adam)), eta, beta1, beta2, zeta,
                                    weight_decay, c_l, c_u, int(t), _stream(stream)), "dat_lamb_update")

    def set_option(self, opt, value):
        _check(_lib.dat_model_set_option(self._h, int(opt), int(value)), "dat_model_set_option")

    def profile_enable(self, on=True):
        _check(_lib.dat_profile_enable(self._h, int(bool(on))), "dat_profile_enable")

    def profile_read(self):
        """{class: (ms_total, launches, algorithmic work)} since profile_enable(True)."""
        out = {}
        for i, name in enumerate(PROF_CLASSES):
            ms, n, w = C.c_double(), _i64(), C.c_double()
            _check(_lib.dat_profile_read(self._h, i, C.byref(ms), C.byref(n), C.byref(w)), "dat_profile_read")
            out[name] = (ms.value, n.value, w.value)
        return out

    def offsets_device(self):
        """int64 device pointer to the tensor table (owned by the model)."""
        return self.offsets_device_ptr

    def grad_scales(self):
        """Device pointer (int) to the per-tensor max |g| of the gradient the last step() wrote; raises if not produced."""
        p = _vp()
        _check(_lib.dat_model_grad_scales(self._h, C.byref(p)), "dat_model_grad_scales")
        return p.value

    def grad_scales_tensor(self):
        """A copy of those scales as a float32 CUDA tensor [num_tensors]."""
        class _View:
            pass
        v = _View()
        v.__cuda_array_interface__ = {"shape": (self.num_tensors,), "typestr": "<f4", "data": (self.grad_scales(), False),
                                      "version": 2, "strides": None}
        return torch.as_tensor(v, device="cuda").clone()

    # ---- introspection (parity tests) ----
    def inspect_ops(self):
        n_ops, n_t = _i(), _i()
        _check(_lib.dat_inspect_counts(self._h, C.byref(n_ops), C.byref(n_t)), "dat_inspect_counts")
        names = ("kind", "in", "out", "res", "k", "stride", "pad", "relu", "p0", "p1")
        ops = []
        for i in range(n_ops.value):
            info = np.zeros(10, np.int32)
            _check(_lib.dat_inspect_op(self._h, i, info.ctypes.data), "dat_inspect_op")
            ops.append(dict(zip(names, (int(v) for v in info))))
        return ops

    def inspect_tensors(self):
        n_ops, n_t = _i(), _i()
        _check(_lib.dat_inspect_counts(self._h, C.byref(n_ops), C.byref(n_t)), "dat_inspect_counts")
        names = ("H", "W", "C", "elem_bytes", "act_stored", "grad_stored")
        out = []
        for t in range(n_t.value):
            info = np.zeros(6, np.int32)
            _check(_lib.dat_inspect_tensor(self._h, t, info.ctypes.data), "dat_inspect_tensor")
            out.append(dict(zip(names, (int(v) for v in info))))
        return out

    def inspect_read(self, which, t, B, info):
        """Raw stored elements of tensor t (which = 0) or its gradient (1): uint16 bf16 bit patterns or float32."""
        n = B * info["H"] * info["W"] * info["C"]
        out = np.empty(n, np.uint16 if info["elem_bytes"] == 2 else np.float32)
        _check(_lib.dat_inspect_read(self._h, which, t, B, out.ctypes.data, out.nbytes), "dat_inspect_read")
        return out

    def inspect_bn(self, op, C_):
        mean, rstd = np.zeros(C_, np.float32), np.zeros(C_, np.float32)
        _check(_lib.dat_inspect_bn(self._h, op, mean.ctypes.data, rstd.ctypes.data), "dat_inspect_bn")
        return mean, rstd


def set_kernel_option(opt, value):
    _check(_lib.dat_set_kernel_option(int(opt), int(value)), "dat_set_kernel_option")


def pgd_init(x, eps, init=INIT_ZERO, seed=0, delta0=None, delta=None, stream=None):
    _dev(x, torch.float32)
    if delta is None:
        delta = torch.empty_like(x)
    _check(_lib.dat_pgd_init(_ptr(x), x.numel(), eps, _init(init, seed, delta0), _ptr(delta), _stream(stream)), "dat_pgd_init")
    return delta


def pgd_update(x, G, delta, eps, alpha, stream=None):
    _dev(x, torch.float32); _dev(G, torch.float32); _dev(delta, torch.float32)
    _check(_lib.dat_pgd_update(_ptr(x), _ptr(G), _ptr(delta), x.numel(), eps, alpha, _stream(stream)), "dat_pgd_update")
    return delta


def make_xadv(x, delta, out=None, stream=None):
    _dev(x, torch.float32); _dev(delta, torch.float32)
    if out is None:
        out = torch.empty_like(x)
    _dev(out, torch.float32)
    _check(_lib.dat_make_xadv(_ptr(x), _ptr(delta), x.numel(), _ptr(out), _stream(stream)), "dat_make_xadv")
    return out


def quantized_bytes(d, bits):
    return int(_lib.dat_quantized_bytes(d, bits))


def quantize(grads, offsets_dev, bits, seed, q=None, scales=None, stream=None):
    """offsets_dev: int64 CUDA tensor [T+1] or a raw device pointer with num_tensors given as (ptr, T)."""
    _dev(grads, torch.float32)
    if isinstance(offsets_dev, tuple):
        optr, T = C.c_void_p(offsets_dev[0]), offsets_dev[1]
    else:
        _dev(offsets_dev, torch.int64)
        optr, T = _ptr(offsets_dev), offsets_dev.numel() - 1
    d = grads.numel()
    if q is None:
        q = torch.empty(max(quantized_bytes(d, bits), 1), dtype=torch.uint8, device=grads.device)
    if scales is None:
        scales = torch.empty(T, dtype=torch.float32, device=grads.device)
    _check(_lib.dat_quantize(_ptr(grads), optr, T, d, bits, int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(q), _ptr(scales),
                             _stream(stream)), "dat_quantize")
    return q, scales


def quantize_scaled(grads, offsets_dev, bits, seed, scales, q=None, stream=None):
    """Encoder only: `scales` is a float32 CUDA tensor [T] or a raw device pointer (int) to the per-tensor max |g|."""
    _dev(grads, torch.float32)
    if isinstance(offsets_dev, tuple):
        optr, T = C.c_void_p(offsets_dev[0]), offsets_dev[1]
    else:
        optr, T = _ptr(offsets_dev), offsets_dev.numel() - 1
    d = grads.numel()
    if q is None:
        q = torch.empty(max(quantized_bytes(d, bits), 1), dtype=torch.uint8, device=grads.device)
    sp = C.c_void_p(scales) if isinstance(scales, int) else _ptr(_dev(scales, torch.float32))
    _check(_lib.dat_quantize_scaled(_ptr(grads), optr, T, d, bits, int(seed) & 0xFFFFFFFFFFFFFFFF, sp, _ptr(q),
                                    _stream(stream)), "dat_quantize_scaled")
    return q


def dequantize(q, scales, offsets_dev, d, bits, out=None, stream=None):
    if isinstance(offsets_dev, tuple):
        optr, T = C.c_void_p(offsets_dev[0]), offsets_dev[1]
    else:
        optr, T = _ptr(offsets_dev), offsets_dev.numel() - 1
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=q.device)
    sp = C.c_void_p(scales) if isinstance(scales, int) else _ptr(scales)     # tensor or raw device pointer
    _check(_lib.dat_dequantize(_ptr(q), sp, optr, T, d, bits, _ptr(out), _stream(stream)), "dat_dequantize")
    return out


def aggregate(q_list, scales_list, offsets_dev, d, bits, out=None, stream=None):
    """g_hat = (1/M) sum_i dequantize(q_i, scales_i): Eq. (grad_agg) for M workers' quantized gradients."""
    M = len(q_list)
    if isinstance(offsets_dev, tuple):
        optr, T = C.c_void_p(offsets_dev[0]), offsets_dev[1]
    else:
        optr, T = _ptr(offsets_dev), offsets_dev.numel() - 1
    qp = (C.c_void_p * M)(*[t.data_ptr() for t in q_list])
    sp = (C.c_void_p * M)(*[t.data_ptr() for t in scales_list])
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=q_list[0].device)
    _check(_lib.dat_aggregate(qp, sp, M, optr, T, d, bits, _ptr(out), _stream(stream)), "dat_aggregate")
    return out


def philox_uniform(start, n, seed, stream_id, device="cuda"):
    out = torch.empty(n, dtype=torch.float32, device=device)
    _check(_lib.dat_philox_uniform(start, n, seed, stream_id, _ptr(out), _stream(None)), "dat_philox_uniform")
    return out


def _conv_shapes(B, H, W, Cin, Cout, k, stride, pad):
    return (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1


def conv_forward(x, w, stride, pad, stream=None):
    """x [B,H,W,Cin] bf16, w [Cout,k,k,Cin] bf16 -> y [B,Ho,Wo,Cout] bf16."""
    _dev(x, torch.bfloat16); _dev(w, torch.bfloat16)
    B, H, W, Cin = x.shape
    Cout, k = w.shape[0], w.shape[1]
    Ho, Wo = _conv_shapes(B, H, W, Cin, Cout, k, stride, pad)
    y = torch.empty(B, Ho, Wo, Cout, dtype=torch.bfloat16, device=x.device)
    _check(_lib.dat_conv_forward(_ptr(x), _ptr(w), _ptr(y), B, H, W, Cin, Cout, k, stride, pad, _stream(stream)), "dat_conv_forward")
    return y


def conv_backward_data(dy, w, in_hw, stride, pad, stream=None):
    _dev(dy, torch.bfloat16); _dev(w, torch.bfloat16)
    B = dy.shape[0]
    Cout, k, Cin = w.shape[0], w.shape[1], w.shape[3]
    H, W = in_hw
    dx = torch.empty(B, H, W, Cin, dtype=torch.bfloat16, device=dy.device)
    _check(_lib.dat_conv_backward_data(_ptr(dy), _ptr(w), _ptr(dx), B, H, W, Cin, Cout, k, stride, pad, _stream(stream)), "dat_conv_backward_data")
    return dx


def conv_backward_weight(x, dy, k, stride, pad, stream=None, dw=None, static=False):
    """static: through dat_conv_backward_weight_static (no allocation inside the call; pass `dw`)."""
    _dev(x, torch.bfloat16); _dev(dy, torch.bfloat16)
    B, H, W, Cin = x.shape
    Cout = dy.shape[3]
    if dw is None:
        dw = torch.empty(Cout, k, k, Cin, dtype=torch.float32, device=x.device)
    fn, name = (_lib.dat_conv_backward_weight_static, "dat_conv_backward_weight_static") if static else \
               (_lib.dat_conv_backward_weight, "dat_conv_backward_weight")
    _check(fn(_ptr(x), _ptr(dy), _ptr(dw), B, H, W, Cin, Cout, k, stride, pad, _stream(stream)), name)
    return dw


def conv_backward_weight_static_limit():
    return int(_lib.dat_conv_backward_weight_static_limit())
