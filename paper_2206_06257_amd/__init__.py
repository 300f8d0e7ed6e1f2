"""MI355X-native hot path of distributed adversarial training (DAT): thin Python binding of the
C ABI in include/dat.h.  Argument marshalling only -- every step runs in the HIP kernels of
libdat.so.  PyTorch supplies device memory and streams; tensors are passed by data_ptr()."""
from .binding import *  # noqa: F401,F403
