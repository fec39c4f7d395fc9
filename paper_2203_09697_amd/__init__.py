"""Python binding of the gpgnn HIP library (argument marshalling only).

Every computational step runs in the library's HIP kernels; this module loads
libgpgnn.so with ctypes, mirrors the C structs of include/gpgnn.h and passes
torch tensors' device pointers through.  torch is used for device memory and
streams only.  There is no CPU fallback: importing the package without a built
library raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
