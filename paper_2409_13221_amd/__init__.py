"""Fused generation + inference stage of RLHF (arXiv 2409.13221, Section 4) for one MI355X.

The product is the HIP shared library built from csrc/ (C ABI in include/rlhf.h); this
package is its thin Python binding.  Importing it does not load the library; the first call
does, and raises if the library has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import LIB_PATH, RlhfError, lib, model_cfg_of  # noqa: F401
