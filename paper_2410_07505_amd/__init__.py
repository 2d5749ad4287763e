"""MI355X-native CrossQuant activation-quantization hot path (arxiv 2410.07505).

The work is done by hand-written HIP kernels for gfx950 behind the C ABI declared in
``include/crossquant.h`` (``libcrossquant.so``, built in-tree by ``paper_2410_07505_amd.build``).
This package is only the argument-marshalling layer: torch supplies device memory and the
stream handle; every step of the path runs in the library's kernels.  There is no CPU or
eager fallback: the first use of any entry point loads the shared library and raises if it is
missing or stale (the binding is imported on first use so that ``python -m
paper_2410_07505_amd.build`` can run before the library exists).
"""
_EXPORTS = (
    "LIB_PATH", "CrossQuantError", "crossquant_absmax", "crossquant_absmax_batched", "crossquant_calib_copy", "crossquant_calib_mfma_i8", "crossquant_calib_mfma_f6", "crossquant_calib_read", "crossquant_absmax_quantize", "crossquant_absmax_quantize_single_read",
    "crossquant_kernel_analysis", "crossquant_kernel_analysis_static", "crossquant_kernel_count", "crossquant_pack_fp6", "crossquant_pack_fp6_weights", "crossquant_w4a4_linear",
    "crossquant_quantize", "crossquant_quantize_batched", "crossquant_quantize_fp6", "crossquant_quantize_linear_fused", "crossquant_status_string", "crossquant_unpack_int4", "crossquant_version", "crossquant_w8a8_linear",
    "crossquant_weight_quantize", "crossquant_weight_quantize_grouped", "lib", "raw",
)
__all__ = list(_EXPORTS)


def __getattr__(name):
    if name in _EXPORTS:
        from . import binding
        return getattr(binding, name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))
