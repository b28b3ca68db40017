"""MI355X-native split backward (2-stage backpropagation) for a LLaMa-like decoder stage.

The product is the HIP library `libtbp.so` (C ABI in include/tbp.h); this package is its thin Python
binding.  PyTorch is used for device memory and streams only.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
