"""MI355X-native hot path of the Lazarus MoE layer (arXiv 2407.04656).

Thin binding over liblazarus_moe.so (hand-written HIP kernels behind a C ABI, see
include/lazarus_moe.h).  PyTorch is used for device memory and streams only; every
step of the path runs in the library's kernels.  There is no CPU fallback: importing
`binding` fails loudly if the shared library has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
