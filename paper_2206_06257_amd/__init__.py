"""MI355X-native hot path of distributed adversarial training (DAT): thin Python binding of the
C ABI in include/dat.h.  Argument marshalling only -- every step runs in the HIP kernels of
libdat.so.  PyTorch supplies device memory and streams; tensors are passed by data_ptr().

The binding is loaded on first use so that `python -m paper_2206_06257_amd.build` can run
before the library exists; using any name of the package without a built library raises."""
import importlib

_binding = None


def __getattr__(name):
    global _binding
    if name.startswith("__"):
        raise AttributeError(name)
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    return getattr(_binding, name)
