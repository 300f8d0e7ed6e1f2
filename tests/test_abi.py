"""The C-ABI library loads and exports every entry point that include/dat.h declares
(no compute calls: runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dat_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    path = os.path.join(ROOT, "paper_2206_06257_amd", "libdat.so")
    assert os.path.exists(path), "build first: python -m paper_2206_06257_amd.build"
    lib = ctypes.CDLL(path)
    names = _declared()
    assert len(names) >= 20
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing


def test_binding_lists_the_same_names():
    import paper_2206_06257_amd.binding as b
    assert sorted(b.EXPORTS) == _declared()


def test_host_only_calls_and_argument_errors():
    import paper_2206_06257_amd.binding as b
    lib = b._lib
    assert lib.dat_status_string(0) == b"ok"
    assert lib.dat_status_string(1) == b"invalid argument"
    assert b.quantized_bytes(1001, 8) == 1001 and b.quantized_bytes(1001, 4) == 501
    assert b.quantized_bytes(5, 2) == 2 and b.quantized_bytes(3, 16) == 6
    assert b.quantized_bytes(10, 3) == 0          # unsupported width
    # argument validation happens before any device work
    assert lib.dat_quantize(None, None, 1, 10, 8, 0, None, None, None) == 1
    assert lib.dat_dequantize(None, None, None, 1, 10, 8, None, None) == 1
    assert lib.dat_model_destroy(None) == 1
    assert lib.dat_attack(None, None, None, 1, 0.1, 0.1, 1, b._Init(0, 0, None), None, None, None) == 1
    assert lib.dat_step(None, None, None, 1, None, None, None) == 1
    assert lib.dat_conv_forward(None, None, None, 1, 8, 8, 8, 8, 3, 1, 1, None) == 1
    assert lib.dat_conv_backward_weight_static(None, None, None, 1, 8, 8, 8, 8, 3, 1, 1, None) == 1
    assert b.conv_backward_weight_static_limit() == 32 << 20
    assert lib.dat_quantize_scaled(None, None, 1, 10, 8, 0, None, None, None) == 1
    assert lib.dat_model_grad_scales(None, None) == 1
    assert lib.dat_set_kernel_option(99, 1) == 1 and lib.dat_set_kernel_option(b.KOPT_RING_KERNEL, 1) == 0
    assert lib.dat_inspect_counts(None, None, None) == 1 and lib.dat_inspect_read(None, 0, 0, 1, None, 0) == 1
    assert lib.dat_model_set_option(None, 0, 1) == 1
