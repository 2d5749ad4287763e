"""ctypes binding for libcrossquant.so: same names as the C ABI, argument marshalling only.

Each wrapper takes torch tensors that already live on the GPU, checks dtype / contiguity,
passes ``data_ptr()`` and the current HIP stream handle to the C entry point, and returns
(or fills) output tensors.  Output tensors can be passed in (``out=...``) so that a caller
such as the benchmark allocates nothing inside its timed region.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcrossquant.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libcrossquant.so is not built (%s). Run `python -m paper_2410_07505_amd.build`; "
        "there is no fallback path." % LIB_PATH)

lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _int, _f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
lib.crossquant_absmax.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp]
lib.crossquant_quantize.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _int, _vp, _vp, _vp, _vp, _vp, _vp]
lib.crossquant_absmax_quantize.argtypes = [_vp, _i64, _i64, _i64, _f32, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.crossquant_absmax_quantize_single_read.argtypes = lib.crossquant_absmax_quantize.argtypes
lib.crossquant_absmax_quantize_single_read.restype = _int
lib.crossquant_debug_set_barrier_polls.argtypes = [ctypes.c_uint]
lib.crossquant_debug_set_barrier_polls.restype = None
lib.crossquant_absmax_batched.argtypes = [_vp, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _vp]
lib.crossquant_quantize_batched.argtypes = [_vp, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _f32, _int, _vp, _vp, _vp, _vp, _vp, _vp]
lib.crossquant_calib_read.argtypes = [_vp, _i64, _vp, _vp]
lib.crossquant_calib_copy.argtypes = [_vp, _vp, _i64, _vp]
lib.crossquant_calib_mfma_i8.argtypes = [_int, _int, _vp, ctypes.POINTER(ctypes.c_double), _vp]
lib.crossquant_calib_mfma_f6.argtypes = [_int, _vp, ctypes.POINTER(ctypes.c_double), _vp]
lib.crossquant_calib_mfma_f6.restype = _int
lib.crossquant_fp6_packed_bytes.argtypes = [_i64, _i64]
lib.crossquant_fp6_packed_bytes.restype = ctypes.c_int64
lib.crossquant_fp6_packed_weight_bytes.argtypes = [_i64, _i64]
lib.crossquant_fp6_packed_weight_bytes.restype = ctypes.c_int64
lib.crossquant_pack_fp6.argtypes = [_vp, _int, _i64, _i64, _vp, _vp]
lib.crossquant_pack_fp6_weights.argtypes = [_vp, _int, _i64, _i64, _vp, _vp]
lib.crossquant_pack_fp6_weights.restype = _int
lib.crossquant_quantize_fp6.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _vp, _vp]
lib.crossquant_w4a4_linear.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _vp, _vp]
lib.crossquant_kernel_count.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _int, _vp, _vp, _vp, _vp]
lib.crossquant_kernel_analysis.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _int, _vp, _vp, _vp, _vp, _vp]
lib.crossquant_kernel_analysis_static.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _int, _vp, _vp, _vp]
lib.crossquant_kernel_analysis_static.restype = _int
lib.crossquant_unpack_int4.argtypes = [_vp, _i64, _i64, _vp, _vp]
lib.crossquant_weight_quantize.argtypes = [_vp, _i64, _i64, _vp, _int, _vp, _vp, _vp]
lib.crossquant_weight_quantize_grouped.argtypes = [_vp, _i64, _i64, _vp, _i64, _int, _vp, _vp, _vp, _vp]
lib.crossquant_w8a8_linear.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _vp, _vp]
lib.crossquant_quantize_linear_fused.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _f32, _int, _vp, _vp, _i64, _vp, _i64, _vp,
                                                 _vp, _vp, _vp]
lib.crossquant_quantize_linear_fused.restype = _int
for _n in ("crossquant_absmax", "crossquant_quantize", "crossquant_absmax_quantize", "crossquant_absmax_batched",
           "crossquant_quantize_batched", "crossquant_calib_read", "crossquant_calib_copy", "crossquant_calib_mfma_i8", "crossquant_pack_fp6",
           "crossquant_w4a4_linear", "crossquant_quantize_fp6", "crossquant_kernel_count", "crossquant_kernel_analysis", "crossquant_unpack_int4",
           "crossquant_weight_quantize", "crossquant_weight_quantize_grouped", "crossquant_w8a8_linear",
           "crossquant_version"):
    getattr(lib, _n).restype = _int
lib.crossquant_status_string.argtypes = [_int]
lib.crossquant_status_string.restype = ctypes.c_char_p
lib.crossquant_version.argtypes = []

raw = lib  # the unwrapped C entry points, for callers that marshal pointers themselves


class CrossQuantError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("crossquant: %s (status %d)" % (crossquant_status_string(status), status))


def crossquant_status_string(status: int) -> str:
    return lib.crossquant_status_string(int(status)).decode()


def crossquant_version() -> int:
    return int(lib.crossquant_version())


def _check(status: int) -> None:
    if status != 0:
        raise CrossQuantError(status)


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _req(t: torch.Tensor, dtype, name: str, ndim: int) -> None:
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must have dtype %s" % (name, dtype))
    if t.dim() != ndim:
        raise ValueError("%s must be %d-D" % (name, ndim))
    if ndim == 2:
        if t.stride(1) != 1 and t.shape[1] != 1:
            raise ValueError("%s must have unit stride along its last axis" % name)
    elif not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)


def _buf(ten: torch.Tensor, dtype, shape, name: str, like: torch.Tensor) -> None:
    """A caller-supplied buffer: exact dtype and shape, contiguous, on the same device as `like`.  The C ABI
    sees only pointers, so a buffer that is too short would be overrun on the device; it is refused here."""
    if not isinstance(ten, torch.Tensor):
        raise TypeError("%s must be a torch.Tensor" % name)
    if ten.dtype != dtype:
        raise TypeError("%s must have dtype %s, not %s" % (name, dtype, ten.dtype))
    if tuple(ten.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, not %s" % (name, tuple(shape), tuple(ten.shape)))
    if not ten.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if ten.device != like.device:
        raise ValueError("%s must be on %s, not %s" % (name, like.device, ten.device))


def _matrix(X: torch.Tensor, dtype, name: str) -> None:
    """A 2-D input with unit stride along its rows; the device check comes after the shape checks of the
    buffers that go with it, so that those can be exercised without a GPU."""
    if not isinstance(X, torch.Tensor) or X.dtype != dtype or X.dim() != 2:
        raise TypeError("%s must be a 2-D tensor of dtype %s" % (name, dtype))
    if X.stride(1) != 1 and X.shape[1] != 1:
        raise ValueError("%s must have unit stride along its last axis" % name)
    if X.shape[0] > 1 and X.stride(0) < X.shape[1]:
        raise ValueError("%s must not have overlapping rows" % name)


def _on_gpu(X: torch.Tensor, name: str) -> None:
    if not X.is_cuda:
        raise ValueError("%s must be a GPU tensor" % name)


def _code_shape(T: int, I: int, bits: int):
    if bits not in (4, 8):
        raise CrossQuantError(-3)
    if bits == 4 and I % 2:
        raise CrossQuantError(-3)
    return ((T, I), torch.int8) if bits == 8 else ((T, I // 2), torch.uint8)


def crossquant_absmax(X: torch.Tensor, *, t: torch.Tensor = None, c: torch.Tensor = None):
    """Row maxima t (float32 [T]) and column maxima c (float32 [I]) of |X| in one pass."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    if t is None:
        t = torch.empty(T, dtype=torch.float32, device=X.device)
    if c is None:
        c = torch.empty(I, dtype=torch.float32, device=X.device)
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    _on_gpu(X, "X")
    _check(lib.crossquant_absmax(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(), _stream(X)))
    return t, c


def _quant_buffers(X, T, I, t, c, codes, code_shape, code_dtype, xhat, row_scale, col_scale, zero_count) -> None:
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    _buf(codes, code_dtype, code_shape, "codes", X)
    if xhat is not None:
        _buf(xhat, torch.float16, (T, I), "xhat", X)
    _buf(row_scale, torch.float32, (T,), "row_scale", X)
    _buf(col_scale, torch.float32, (I,), "col_scale", X)
    if zero_count is not None:
        _buf(zero_count, torch.int64, (1,), "zero_count", X)
    _on_gpu(X, "X")


def crossquant_quantize(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, bits: int, *,
                        want_xhat: bool = True, want_count: bool = True, codes: torch.Tensor = None,
                        xhat: torch.Tensor = None, row_scale: torch.Tensor = None,
                        col_scale: torch.Tensor = None, zero_count: torch.Tensor = None):
    """CrossQuant codes (+ dequantized matrix, scale factors, zero count).

    Returns (codes, xhat_or_None, row_scale, col_scale, zero_count_or_None); zero_count is a
    one-element int64 tensor (the library's unsigned 64-bit counter)."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    dev = X.device
    code_shape, code_dtype = _code_shape(T, I, bits)
    if codes is None:
        codes = torch.empty(code_shape, dtype=code_dtype, device=dev)
    if xhat is None and want_xhat:
        xhat = torch.empty((T, I), dtype=torch.float16, device=dev)
    if row_scale is None:
        row_scale = torch.empty(T, dtype=torch.float32, device=dev)
    if col_scale is None:
        col_scale = torch.empty(I, dtype=torch.float32, device=dev)
    if zero_count is None and want_count:
        zero_count = torch.empty(1, dtype=torch.int64, device=dev)
    _quant_buffers(X, T, I, t, c, codes, code_shape, code_dtype, xhat, row_scale, col_scale, zero_count)
    _check(lib.crossquant_quantize(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(), float(alpha),
                                   int(bits), codes.data_ptr(), _ptr(xhat), row_scale.data_ptr(),
                                   col_scale.data_ptr(), _ptr(zero_count), _stream(X)))
    return codes, xhat, row_scale, col_scale, zero_count


def crossquant_absmax_quantize(X: torch.Tensor, alpha: float, bits: int, *, single_read: bool = False,
                               want_xhat: bool = True, want_count: bool = True, t: torch.Tensor = None, c: torch.Tensor = None,
                               codes: torch.Tensor = None, xhat: torch.Tensor = None,
                               row_scale: torch.Tensor = None, col_scale: torch.Tensor = None,
                               zero_count: torch.Tensor = None):
    """crossquant_absmax + crossquant_quantize as one call.

    Returns (t, c, codes, xhat_or_None, row_scale, col_scale, zero_count_or_None).
    single_read=True calls crossquant_absmax_quantize_single_read instead (one kernel that keeps X on
    chip): same results; raises CrossQuantError with status -6 when the matrix does not fit on chip or
    is not in the vector layout."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    dev = X.device
    code_shape, code_dtype = _code_shape(T, I, bits)
    if t is None:
        t = torch.empty(T, dtype=torch.float32, device=dev)
    if c is None:
        c = torch.empty(I, dtype=torch.float32, device=dev)
    if codes is None:
        codes = torch.empty(code_shape, dtype=code_dtype, device=dev)
    if xhat is None and want_xhat:
        xhat = torch.empty((T, I), dtype=torch.float16, device=dev)
    if row_scale is None:
        row_scale = torch.empty(T, dtype=torch.float32, device=dev)
    if col_scale is None:
        col_scale = torch.empty(I, dtype=torch.float32, device=dev)
    if zero_count is None and want_count:
        zero_count = torch.empty(1, dtype=torch.int64, device=dev)
    _quant_buffers(X, T, I, t, c, codes, code_shape, code_dtype, xhat, row_scale, col_scale, zero_count)
    call = lib.crossquant_absmax_quantize_single_read if single_read else lib.crossquant_absmax_quantize
    _check(call(X.data_ptr(), T, I, X.stride(0), float(alpha), int(bits), t.data_ptr(), c.data_ptr(),
                codes.data_ptr(), _ptr(xhat), row_scale.data_ptr(), col_scale.data_ptr(), _ptr(zero_count), _stream(X)))
    return t, c, codes, xhat, row_scale, col_scale, zero_count


def crossquant_absmax_quantize_single_read(X: torch.Tensor, alpha: float, bits: int, **kw):
    """crossquant_absmax_quantize(..., single_read=True)."""
    return crossquant_absmax_quantize(X, alpha, bits, single_read=True, **kw)


def _req3(X: torch.Tensor):
    if not isinstance(X, torch.Tensor) or not X.is_cuda:
        raise ValueError("X must be a CUDA/HIP tensor")
    if X.dtype != torch.float16 or X.dim() != 3 or (X.stride(2) != 1 and X.shape[2] != 1):
        raise ValueError("X must be a float16 [B][S][I] tensor with contiguous rows")


def crossquant_absmax_batched(X: torch.Tensor, *, t: torch.Tensor = None, c: torch.Tensor = None):
    """Per-token maxima t (float32 [B][S]) and per-sequence column maxima c (float32 [B][I])."""
    _req3(X)
    B, S, I = X.shape
    if t is None:
        t = torch.empty((B, S), dtype=torch.float32, device=X.device)
    if c is None:
        c = torch.empty((B, I), dtype=torch.float32, device=X.device)
    _buf(t, torch.float32, (B, S), "t", X)
    _buf(c, torch.float32, (B, I), "c", X)
    _check(lib.crossquant_absmax_batched(X.data_ptr(), B, S, I, X.stride(1), X.stride(0), t.data_ptr(), c.data_ptr(),
                                         _stream(X)))
    return t, c


def crossquant_quantize_batched(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, bits: int, *,
                                want_codes: bool = True, want_xhat: bool = True, want_count: bool = True):
    """Batched CrossQuant with per-sequence column factors.

    Returns (codes [B][S][I or I/2] or None, xhat or None, row_scale [B][S], col_scale [B][I],
    zero_count or None)."""
    _req3(X)
    B, S, I = X.shape
    dev = X.device
    codes = None
    if want_codes:
        codes = (torch.empty((B, S, I), dtype=torch.int8, device=dev) if bits == 8
                 else torch.empty((B, S, max(I // 2, 1)), dtype=torch.uint8, device=dev))
    xhat = torch.empty((B, S, I), dtype=torch.float16, device=dev) if (want_xhat and want_codes) else None
    row_scale = torch.empty((B, S), dtype=torch.float32, device=dev)
    col_scale = torch.empty((B, I), dtype=torch.float32, device=dev)
    zero_count = torch.empty(1, dtype=torch.int64, device=dev) if (want_count or not want_codes) else None
    for ten, n, name in ((t, B * S, "t"), (c, B * I, "c")):
        if (not isinstance(ten, torch.Tensor) or ten.dtype != torch.float32 or ten.numel() != n
                or not ten.is_contiguous() or ten.device != dev):
            raise ValueError("%s must hold %d contiguous float32 values on %s" % (name, n, dev))
    _check(lib.crossquant_quantize_batched(X.data_ptr(), B, S, I, X.stride(1), X.stride(0), t.data_ptr(), c.data_ptr(),
                                           float(alpha), int(bits), _ptr(codes), _ptr(xhat), row_scale.data_ptr(),
                                           col_scale.data_ptr(), _ptr(zero_count), _stream(X)))
    return codes, xhat, row_scale, col_scale, zero_count


def crossquant_pack_fp6(codes: torch.Tensor, *, packed: torch.Tensor = None, weights: bool = False) -> torch.Tensor:
    """INT4 codes -> FP6 fragments for crossquant_w4a4_linear.  codes: int8 [R][K] (values in
    [-7, 7]) or uint8 packed nibbles [R][K/2]; returns a uint8 tensor of the packed size.
    weights=True: the weight operand's row order (crossquant_pack_fp6_weights), for codes [O][K]."""
    if not codes.is_cuda or codes.dim() != 2 or not codes.is_contiguous():
        raise ValueError("codes must be a contiguous 2-D GPU tensor")
    if codes.dtype == torch.int8:
        fmt, (R, K) = 8, codes.shape
    elif codes.dtype == torch.uint8:
        fmt, R, K = 4, codes.shape[0], codes.shape[1] * 2
    else:
        raise TypeError("codes must be int8 (one code per byte) or uint8 (packed nibbles)")
    n = int((lib.crossquant_fp6_packed_weight_bytes if weights else lib.crossquant_fp6_packed_bytes)(R, K))
    if n < 0:
        raise CrossQuantError(-6)
    if packed is None:
        packed = torch.empty(n, dtype=torch.uint8, device=codes.device)
    elif packed.dtype != torch.uint8 or packed.numel() != n or not packed.is_contiguous():
        raise ValueError("packed must be a contiguous uint8 tensor of %d bytes" % n)
    pack = lib.crossquant_pack_fp6_weights if weights else lib.crossquant_pack_fp6
    _check(pack(codes.data_ptr(), fmt, R, K, packed.data_ptr(), _stream(codes)))
    return packed


def crossquant_pack_fp6_weights(codes: torch.Tensor, *, packed: torch.Tensor = None) -> torch.Tensor:
    """INT4 weight codes [O][K] -> the weight operand of crossquant_w4a4_linear (FP6 fragments with the rows of
    every group of 64 output channels interleaved four ways)."""
    return crossquant_pack_fp6(codes, packed=packed, weights=True)


def crossquant_quantize_fp6(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, *,
                            want_xhat: bool = False, want_count: bool = True, packed: torch.Tensor = None,
                            xhat: torch.Tensor = None, row_scale: torch.Tensor = None,
                            col_scale: torch.Tensor = None, zero_count: torch.Tensor = None):
    """INT4 CrossQuant codes written directly as FP6 fragments for crossquant_w4a4_linear.

    Returns (packed, xhat_or_None, row_scale, col_scale, zero_count_or_None)."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    dev = X.device
    n = int(lib.crossquant_fp6_packed_bytes(T, I))
    if n < 0:
        raise CrossQuantError(-6)
    if packed is None:
        packed = torch.zeros(n, dtype=torch.uint8, device=dev)
    elif packed.dtype != torch.uint8 or packed.numel() != n or not packed.is_contiguous():
        raise ValueError("packed must be a contiguous uint8 tensor of %d bytes" % n)
    if xhat is None and want_xhat:
        xhat = torch.empty((T, I), dtype=torch.float16, device=dev)
    if row_scale is None:
        row_scale = torch.empty(T, dtype=torch.float32, device=dev)
    if col_scale is None:
        col_scale = torch.empty(I, dtype=torch.float32, device=dev)
    if zero_count is None and want_count:
        zero_count = torch.empty(1, dtype=torch.int64, device=dev)
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    _buf(packed, torch.uint8, (n,), "packed", X)
    if xhat is not None:
        _buf(xhat, torch.float16, (T, I), "xhat", X)
    _buf(row_scale, torch.float32, (T,), "row_scale", X)
    _buf(col_scale, torch.float32, (I,), "col_scale", X)
    if zero_count is not None:
        _buf(zero_count, torch.int64, (1,), "zero_count", X)
    _on_gpu(X, "X")
    _check(lib.crossquant_quantize_fp6(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(), float(alpha),
                                       packed.data_ptr(), _ptr(xhat), row_scale.data_ptr(), col_scale.data_ptr(),
                                       _ptr(zero_count), _stream(X)))
    return packed, xhat, row_scale, col_scale, zero_count


def _linear_outputs(Y, acc_debug, T: int, O: int, like: torch.Tensor) -> None:
    """Y: float16 [T][O], rows may be padded (unit stride inside a row); acc_debug: int32 [T][O] contiguous."""
    if not isinstance(Y, torch.Tensor) or Y.dtype != torch.float16 or tuple(Y.shape) != (T, O):
        raise ValueError("Y must be a float16 tensor of shape (%d, %d)" % (T, O))
    if (O > 1 and Y.stride(1) != 1) or (T > 1 and Y.stride(0) < O) or Y.device != like.device:
        raise ValueError("Y must have unit stride inside a row, non-overlapping rows, and be on %s" % like.device)
    if acc_debug is not None:
        _buf(acc_debug, torch.int32, (T, O), "acc_debug", like)


def crossquant_w4a4_linear(qx_fp6: torch.Tensor, row_scale: torch.Tensor, qw_fp6: torch.Tensor, w_scale: torch.Tensor,
                           T: int, I: int, O: int, *, Y: torch.Tensor = None, acc_debug: torch.Tensor = None,
                           want_acc: bool = False):
    """A4W4 linear layer on FP6-packed INT4 codes (exact).  Returns (Y, acc_or_None)."""
    for ten, name in ((qx_fp6, "qx_fp6"), (qw_fp6, "qw_fp6")):
        if not ten.is_cuda or ten.dtype != torch.uint8 or not ten.is_contiguous():
            raise ValueError("%s must be a contiguous uint8 GPU tensor from crossquant_pack_fp6 / _weights" % name)
    if qx_fp6.numel() != lib.crossquant_fp6_packed_bytes(T, I) or qw_fp6.numel() != lib.crossquant_fp6_packed_weight_bytes(O, I):
        raise ValueError("packed operand sizes do not match T, I, O")
    _buf(row_scale, torch.float32, (T,), "row_scale", qx_fp6)
    _buf(w_scale, torch.float32, (O,), "w_scale", qx_fp6)
    if qw_fp6.device != qx_fp6.device:
        raise ValueError("qw_fp6 must be on %s" % qx_fp6.device)
    if Y is None:
        Y = torch.empty((T, O), dtype=torch.float16, device=qx_fp6.device)
    if acc_debug is None and want_acc:
        acc_debug = torch.empty((T, O), dtype=torch.int32, device=qx_fp6.device)
    _linear_outputs(Y, acc_debug, T, O, qx_fp6)
    _check(lib.crossquant_w4a4_linear(qx_fp6.data_ptr(), row_scale.data_ptr(), qw_fp6.data_ptr(), w_scale.data_ptr(),
                                      T, I, O, Y.data_ptr(), Y.stride(0), _ptr(acc_debug), _stream(qx_fp6)))
    return Y, acc_debug


def crossquant_calib_read(src: torch.Tensor) -> None:
    """Plain streaming read of a contiguous GPU tensor (roofline calibration)."""
    _check(lib.crossquant_calib_read(src.data_ptr(), src.numel() * src.element_size(), 0, _stream(src)))


def crossquant_calib_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    """Plain copy between two contiguous GPU tensors of the same size (roofline calibration)."""
    if src.numel() * src.element_size() != dst.numel() * dst.element_size():
        raise ValueError("src and dst must have the same size in bytes")
    _check(lib.crossquant_calib_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream(src)))


def crossquant_calib_mfma_i8(iters: int, data_mode: int) -> float:
    """MFMA-only loop on the current device and stream; returns the integer operations launched."""
    ops = ctypes.c_double(0.0)
    _check(lib.crossquant_calib_mfma_i8(int(iters), int(data_mode), 0, ctypes.byref(ops),
                                        torch.cuda.current_stream().cuda_stream))
    return float(ops.value)


def crossquant_calib_mfma_f6(iters: int) -> float:
    """FP6 MFMA loop fed from LDS on the current device and stream; returns the operations launched."""
    ops = ctypes.c_double(0.0)
    _check(lib.crossquant_calib_mfma_f6(int(iters), 0, ctypes.byref(ops), torch.cuda.current_stream().cuda_stream))
    return float(ops.value)


def crossquant_kernel_count(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, bits: int, *,
                            row_scale: torch.Tensor = None, col_scale: torch.Tensor = None,
                            zero_count: torch.Tensor = None) -> torch.Tensor:
    """Number of elements whose code is zero (one-element int64 tensor on the GPU).  row_scale / col_scale:
    optional buffers that receive the scale factors; without them the library uses none."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    dev = X.device
    if zero_count is None:
        zero_count = torch.empty(1, dtype=torch.int64, device=dev)
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    if (row_scale is None) != (col_scale is None):
        raise ValueError("row_scale and col_scale: pass both or neither")
    if row_scale is not None:
        _buf(row_scale, torch.float32, (T,), "row_scale", X)
        _buf(col_scale, torch.float32, (I,), "col_scale", X)
    _buf(zero_count, torch.int64, (1,), "zero_count", X)
    _on_gpu(X, "X")
    _check(lib.crossquant_kernel_count(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(),
                                       float(alpha), int(bits), _ptr(row_scale), _ptr(col_scale),
                                       zero_count.data_ptr(), _stream(X)))
    return zero_count


def crossquant_kernel_analysis(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, bits: int, *,
                               want_xrk: bool = True, xrk: torch.Tensor = None, row_scale: torch.Tensor = None,
                               col_scale: torch.Tensor = None, counters: torch.Tensor = None,
                               work_vectors: bool = True):
    """"Remove Kernel" matrix (float16 [T][I] or None) and a three-element int64 tensor
    {kernel size, #{c_j >= t_i}, #{B~_ij < B_ij}}.  row_scale / col_scale are the call's work vectors
    (allocated here when not given); work_vectors=False passes NULL for both instead."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    dev = X.device
    if xrk is None and want_xrk:
        xrk = torch.empty((T, I), dtype=torch.float16, device=dev)
    if work_vectors and row_scale is None and col_scale is None:
        row_scale = torch.empty(T, dtype=torch.float32, device=dev)
        col_scale = torch.empty(I, dtype=torch.float32, device=dev)
    if counters is None:
        counters = torch.empty(3, dtype=torch.int64, device=dev)
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    if xrk is not None:
        _buf(xrk, torch.float16, (T, I), "xrk", X)
    if (row_scale is None) != (col_scale is None):
        raise ValueError("row_scale and col_scale: pass both or neither")
    if row_scale is not None:
        _buf(row_scale, torch.float32, (T,), "row_scale", X)
        _buf(col_scale, torch.float32, (I,), "col_scale", X)
    _buf(counters, torch.int64, (3,), "counters", X)
    _on_gpu(X, "X")
    _check(lib.crossquant_kernel_analysis(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(),
                                          float(alpha), int(bits), _ptr(xrk), _ptr(row_scale),
                                          _ptr(col_scale), counters.data_ptr(), _stream(X)))
    return xrk, counters


def crossquant_kernel_analysis_static(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, bits: int, *,
                                      xrk: torch.Tensor = None, counters: torch.Tensor):
    """crossquant_kernel_analysis with the work vectors in the library's static device array: nothing is
    allocated here or in the library, so every buffer (xrk optional, counters required) comes from the caller."""
    _matrix(X, torch.float16, "X")
    T, I = X.shape
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    if xrk is not None:
        _buf(xrk, torch.float16, (T, I), "xrk", X)
    _buf(counters, torch.int64, (3,), "counters", X)
    _on_gpu(X, "X")
    _check(lib.crossquant_kernel_analysis_static(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(),
                                                 float(alpha), int(bits), _ptr(xrk), counters.data_ptr(), _stream(X)))
    return xrk, counters


def crossquant_unpack_int4(packed: torch.Tensor, *, codes: torch.Tensor = None) -> torch.Tensor:
    """Packed INT4 codes (uint8 [T][I/2]) -> int8 codes [T][I]."""
    _req(packed, torch.uint8, "packed", 2)
    if not packed.is_contiguous():
        raise ValueError("packed must be contiguous")
    T, half = packed.shape
    if codes is None:
        codes = torch.empty((T, 2 * half), dtype=torch.int8, device=packed.device)
    _buf(codes, torch.int8, (T, 2 * half), "codes", packed)
    _check(lib.crossquant_unpack_int4(packed.data_ptr(), T, 2 * half, codes.data_ptr(), _stream(packed)))
    return codes


def crossquant_weight_quantize(W: torch.Tensor, fold, bits: int, *, qw: torch.Tensor = None,
                               w_scale: torch.Tensor = None):
    """Per-output-channel weight codes qw (int8 [O][I]) and steps w_scale (float32 [O])."""
    _req(W, torch.float16, "W", 2)
    if not W.is_contiguous():
        raise ValueError("W must be contiguous")
    I, O = W.shape
    if qw is None:
        qw = torch.empty((O, I), dtype=torch.int8, device=W.device)
    if w_scale is None:
        w_scale = torch.empty(O, dtype=torch.float32, device=W.device)
    _buf(qw, torch.int8, (O, I), "qw", W)
    _buf(w_scale, torch.float32, (O,), "w_scale", W)
    if fold is not None:
        _buf(fold, torch.float32, (I,), "fold", W)
    _check(lib.crossquant_weight_quantize(W.data_ptr(), I, O, _ptr(fold), int(bits), qw.data_ptr(),
                                          w_scale.data_ptr(), _stream(W)))
    return qw, w_scale


def crossquant_weight_quantize_grouped(W: torch.Tensor, fold, group: int, bits: int, *, want_dq: bool = False,
                                       qw: torch.Tensor = None, w_scale: torch.Tensor = None,
                                       w_dq: torch.Tensor = None):
    """Group-wise weight codes qw (int8 [O][I]), steps (float32 [O][I/group]) and, optionally, the
    dequantized weights (float16 [I][O])."""
    _req(W, torch.float16, "W", 2)
    if not W.is_contiguous():
        raise ValueError("W must be contiguous")
    I, O = W.shape
    if group < 1 or I % group:
        raise ValueError("the group size must divide the number of input channels")
    if qw is None:
        qw = torch.empty((O, I), dtype=torch.int8, device=W.device)
    if w_scale is None:
        w_scale = torch.empty((O, I // group), dtype=torch.float32, device=W.device)
    if w_dq is None and want_dq:
        w_dq = torch.empty((I, O), dtype=torch.float16, device=W.device)
    _buf(qw, torch.int8, (O, I), "qw", W)
    _buf(w_scale, torch.float32, (O, I // group), "w_scale", W)
    if w_dq is not None:
        _buf(w_dq, torch.float16, (I, O), "w_dq", W)
    if fold is not None:
        _buf(fold, torch.float32, (I,), "fold", W)
    _check(lib.crossquant_weight_quantize_grouped(W.data_ptr(), I, O, _ptr(fold), int(group), int(bits),
                                                  qw.data_ptr(), w_scale.data_ptr(), _ptr(w_dq), _stream(W)))
    return qw, w_scale, w_dq


def crossquant_w8a8_linear(qx: torch.Tensor, row_scale: torch.Tensor, qw: torch.Tensor, w_scale: torch.Tensor, *,
                           Y: torch.Tensor = None, acc_debug: torch.Tensor = None, want_acc: bool = False):
    """Y = fl16(acc * row_scale_i * w_scale_k) with acc = qx . qw^T in int32.  Returns (Y, acc_or_None)."""
    _matrix(qx, torch.int8, "qx")
    _matrix(qw, torch.int8, "qw")
    if not qx.is_contiguous() or not qw.is_contiguous():
        raise ValueError("qx and qw must be contiguous")
    T, I = qx.shape
    O, I2 = qw.shape
    if I != I2:
        raise ValueError("qx is [T][I] and qw [O][I]: the contraction lengths differ (%d, %d)" % (I, I2))
    if qw.device != qx.device:
        raise ValueError("qw must be on %s" % qx.device)
    _buf(row_scale, torch.float32, (T,), "row_scale", qx)
    _buf(w_scale, torch.float32, (O,), "w_scale", qx)
    if Y is None:
        Y = torch.empty((T, O), dtype=torch.float16, device=qx.device)
    if acc_debug is None and want_acc:
        acc_debug = torch.empty((T, O), dtype=torch.int32, device=qx.device)
    _linear_outputs(Y, acc_debug, T, O, qx)
    _on_gpu(qx, "qx")
    _check(lib.crossquant_w8a8_linear(qx.data_ptr(), row_scale.data_ptr(), qw.data_ptr(), w_scale.data_ptr(),
                                      T, I, O, Y.data_ptr(), Y.stride(0), _ptr(acc_debug), _stream(qx)))
    return Y, acc_debug


def crossquant_quantize_linear_fused(X: torch.Tensor, t: torch.Tensor, c: torch.Tensor, alpha: float, bits: int,
                                     qw: torch.Tensor, w_scale: torch.Tensor, *, Y: torch.Tensor = None,
                                     row_scale: torch.Tensor = None, col_scale: torch.Tensor = None,
                                     acc_debug: torch.Tensor = None, want_acc: bool = False):
    """Quantize inside the GEMM's activation load: Y from X directly.  Returns (Y, row_scale, col_scale, acc_or_None)."""
    _matrix(X, torch.float16, "X")
    _matrix(qw, torch.int8, "qw")
    T, I = X.shape
    O, I2 = qw.shape
    if I != I2 or not qw.is_contiguous():
        raise ValueError("qw must be a contiguous [O][I] tensor with I = %d" % I)
    dev = X.device
    if row_scale is None:
        row_scale = torch.empty(T, dtype=torch.float32, device=dev)
    if col_scale is None:
        col_scale = torch.empty(I, dtype=torch.float32, device=dev)
    if Y is None:
        Y = torch.empty((T, O), dtype=torch.float16, device=dev)
    if acc_debug is None and want_acc:
        acc_debug = torch.empty((T, O), dtype=torch.int32, device=dev)
    _buf(t, torch.float32, (T,), "t", X)
    _buf(c, torch.float32, (I,), "c", X)
    _buf(row_scale, torch.float32, (T,), "row_scale", X)
    _buf(col_scale, torch.float32, (I,), "col_scale", X)
    _buf(w_scale, torch.float32, (O,), "w_scale", X)
    _linear_outputs(Y, acc_debug, T, O, X)
    if qw.device != dev:
        raise ValueError("qw must be on %s" % dev)
    _on_gpu(X, "X")
    _check(lib.crossquant_quantize_linear_fused(X.data_ptr(), T, I, X.stride(0), t.data_ptr(), c.data_ptr(), float(alpha),
                                                int(bits), qw.data_ptr(), w_scale.data_ptr(), O, Y.data_ptr(),
                                                Y.stride(0), row_scale.data_ptr(), col_scale.data_ptr(),
                                                _ptr(acc_debug), _stream(X)))
    return Y, row_scale, col_scale, acc_debug
