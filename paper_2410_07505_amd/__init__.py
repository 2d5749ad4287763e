"""MI355X-native CrossQuant activation-quantization hot path (arxiv 2410.07505).

The work is done by hand-written HIP kernels for gfx950 behind the C ABI declared in
``include/crossquant.h`` (``libcrossquant.so``, built in-tree by ``paper_2410_07505_amd.build``).
This package is only the argument-marshalling layer: torch supplies device memory and the
stream handle; every step of the path runs in the library's kernels.  There is no CPU or
eager fallback: if the shared library is missing, importing :mod:`binding` raises.
"""
from .binding import (  # noqa: F401
    LIB_PATH,
    CrossQuantError,
    crossquant_absmax,
    crossquant_kernel_analysis,
    crossquant_kernel_count,
    crossquant_quantize,
    crossquant_status_string,
    crossquant_version,
    crossquant_w8a8_linear,
    crossquant_weight_quantize,
    lib,
    raw,
)
