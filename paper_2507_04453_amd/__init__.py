"""MI355X-native hot path of ESSA (arXiv 2507.04453): thin Python binding over libessa's C ABI.

Everything numerical runs in the HIP kernels of libessa.so; this package only marshals arguments
(torch tensors are used as device memory and for the stream).  There is no CPU fallback: if the
library is missing or cannot be loaded, importing the binding raises.
"""
from .essa import *  # noqa: F401,F403
from .essa import __all__  # noqa: F401
