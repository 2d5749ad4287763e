"""CrossQuant CPU oracle (test infrastructure, not product code).

Thin numpy/ctypes marshalling around ``crossquant_oracle.c``, the plain C statement of the
paper's definitions (Eq. 1 per-token, Eq. 2 per-channel, Definition 1 quantization kernel, the
CrossQuant equation and the appendix fake-quant listing's dequantization).  Nothing here is
imported by the product package; only tests, the smoke check and the benchmark's cpu_baseline
leg use it.  It never touches a GPU.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "crossquant_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libcrossquant_oracle.so")
_lib = None

# -ffp-contract=off: no fused multiply-add, so every binary32 operation rounds on its own.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-fopenmp"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        tmp = _LIB_PATH + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *_CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.cq_oracle_half_to_float.restype = ctypes.c_float
        lib.cq_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.cq_oracle_float_to_half.restype = ctypes.c_uint16
        lib.cq_oracle_float_to_half.argtypes = [ctypes.c_float]
        lib.cq_oracle_num_threads.restype = ctypes.c_int
        for name in ("cq_oracle_absmax", "cq_oracle_scales", "cq_oracle_quantize",
                     "cq_oracle_kernel_count", "cq_oracle_weight_quantize", "cq_oracle_w8a8_linear",
                     "cq_oracle_kernel_analysis", "cq_oracle_weight_quantize_grouped"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _p(arr):
    return None if arr is None else ctypes.c_void_p(arr.ctypes.data)


def _i64(v):
    return ctypes.c_int64(int(v))


def _as_half_bits(x: np.ndarray) -> np.ndarray:
    if x.dtype != np.float16:
        raise TypeError("expected a float16 array")
    if x.ndim != 2 or x.strides[1] != 2 or x.strides[0] % 2:
        raise ValueError("expected a 2-D array with contiguous rows")
    return x.view(np.uint16)


def qmax(bits: int) -> int:
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    return 2 ** (bits - 1) - 1


def num_threads() -> int:
    return int(_load().cq_oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads used by the row loops from now on (timing only; results do not depend on it)."""
    lib = _load()
    lib.cq_oracle_set_num_threads.restype = None
    lib.cq_oracle_set_num_threads.argtypes = [ctypes.c_int]
    lib.cq_oracle_set_num_threads(int(n))


def half_to_float(h: int) -> float:
    return float(_load().cq_oracle_half_to_float(int(h)))


def float_to_half(f: float) -> int:
    return int(_load().cq_oracle_float_to_half(float(np.float32(f))))


def absmax(X: np.ndarray):
    """t_i = max_j |X_ij| (Eq. 1), c_j = max_i |X_ij| (CrossQuant equation); float32 vectors."""
    xb = _as_half_bits(X)
    T, I = X.shape
    t = np.empty(T, np.float32)
    c = np.empty(I, np.float32)
    _load().cq_oracle_absmax(_p(xb), _i64(T), _i64(I), _i64(X.strides[0] // 2), _p(t), _p(c))
    return t, c


def scales(t: np.ndarray, c: np.ndarray, alpha: float, bits: int):
    """a_i = t_i^alpha / q_max, b_j = c_j^(1-alpha): the CrossQuant step split in two factors."""
    qmax(bits)
    t = np.ascontiguousarray(t, np.float32)
    c = np.ascontiguousarray(c, np.float32)
    a = np.empty_like(t)
    b = np.empty_like(c)
    _load().cq_oracle_scales(_p(t), _p(c), _i64(t.size), _i64(c.size), ctypes.c_float(alpha),
                             ctypes.c_int(bits), _p(a), _p(b))
    return a, b


def quantize(X: np.ndarray, t: np.ndarray, c: np.ndarray, alpha: float, bits: int,
             want_xhat: bool = True):
    """CrossQuant codes, dequantized matrix, scale factors, kernel size and clamp-hit count.

    Returns a dict: codes (int8 [T][I], or uint8 [T][I/2] packed nibbles for bits=4), xhat
    (float16 or None), a, b (float32), Z (int), clamp_hits (int)."""
    qmax(bits)
    xb = _as_half_bits(X)
    T, I = X.shape
    if bits == 4 and I % 2:
        raise ValueError("INT4 packing needs an even number of channels")
    t = np.ascontiguousarray(t, np.float32)
    c = np.ascontiguousarray(c, np.float32)
    codes = np.zeros((T, I), np.int8) if bits == 8 else np.zeros((T, I // 2), np.uint8)
    xhat = np.empty((T, I), np.uint16) if want_xhat else None
    a = np.empty(T, np.float32)
    b = np.empty(I, np.float32)
    Z = ctypes.c_uint64(0)
    clamps = ctypes.c_uint64(0)
    _load().cq_oracle_quantize(_p(xb), _i64(T), _i64(I), _i64(X.strides[0] // 2), _p(t), _p(c),
                               ctypes.c_float(alpha), ctypes.c_int(bits), _p(codes), _p(xhat),
                               _p(a), _p(b), ctypes.byref(Z), ctypes.byref(clamps))
    return {"codes": codes, "xhat": None if xhat is None else xhat.view(np.float16), "a": a,
            "b": b, "Z": int(Z.value), "clamp_hits": int(clamps.value)}


def absmax_batched(X3: np.ndarray):
    """[B][S][I] tensor (the appendix listing's shape): per-token maxima t [B][S] and per-sequence
    column maxima c [B][I].  Each sequence is an independent S x I problem."""
    if X3.ndim != 3:
        raise ValueError("expected a [B][S][I] array")
    ts, cs = zip(*(absmax(X3[b]) for b in range(X3.shape[0])))
    return np.stack(ts), np.stack(cs)


def quantize_batched(X3: np.ndarray, t: np.ndarray, c: np.ndarray, alpha: float, bits: int):
    """CrossQuant applied to every sequence of a [B][S][I] tensor with that sequence's own t and c.
    Returns a dict like quantize(), arrays stacked along a leading batch axis, Z summed."""
    if X3.ndim != 3:
        raise ValueError("expected a [B][S][I] array")
    outs = [quantize(X3[b], t[b], c[b], alpha, bits) for b in range(X3.shape[0])]
    res = {k: np.stack([o[k] for o in outs]) for k in ("codes", "xhat", "a", "b")}
    res["Z"] = sum(o["Z"] for o in outs)
    res["clamp_hits"] = sum(o["clamp_hits"] for o in outs)
    return res


def kernel_count(X: np.ndarray, t: np.ndarray, c: np.ndarray, alpha: float, bits: int) -> int:
    """Size of the quantization kernel (Definition 1): number of elements with code 0."""
    qmax(bits)
    xb = _as_half_bits(X)
    T, I = X.shape
    t = np.ascontiguousarray(t, np.float32)
    c = np.ascontiguousarray(c, np.float32)
    a = np.empty(T, np.float32)
    b = np.empty(I, np.float32)
    Z = ctypes.c_uint64(0)
    _load().cq_oracle_kernel_count(_p(xb), _i64(T), _i64(I), _i64(X.strides[0] // 2), _p(t), _p(c),
                                   ctypes.c_float(alpha), ctypes.c_int(bits), _p(a), _p(b),
                                   ctypes.byref(Z))
    return int(Z.value)


def kernel_analysis(X: np.ndarray, t: np.ndarray, c: np.ndarray, alpha: float, bits: int,
                    want_xrk: bool = True):
    """"Remove Kernel" matrix and the Table 1 indicators.  Returns a dict: xrk (float16 or None),
    Z, n_col_ge_row (#{c_j >= t_i}), n_bound_smaller (#{B~_ij < B_ij}), a, b."""
    qmax(bits)
    xb = _as_half_bits(X)
    T, I = X.shape
    t = np.ascontiguousarray(t, np.float32)
    c = np.ascontiguousarray(c, np.float32)
    xrk = np.empty((T, I), np.uint16) if want_xrk else None
    a = np.empty(T, np.float32)
    b = np.empty(I, np.float32)
    counters = np.zeros(3, np.uint64)
    _load().cq_oracle_kernel_analysis(_p(xb), _i64(T), _i64(I), _i64(X.strides[0] // 2), _p(t), _p(c),
                                      ctypes.c_float(alpha), ctypes.c_int(bits), _p(xrk), _p(a), _p(b),
                                      _p(counters))
    return {"xrk": None if xrk is None else xrk.view(np.float16), "Z": int(counters[0]),
            "n_col_ge_row": int(counters[1]), "n_bound_smaller": int(counters[2]), "a": a, "b": b}


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    """Packed two's-complement nibbles [T][I/2] -> int8 [T][I] (even column = low nibble)."""
    lo = (packed & 0xF).astype(np.int8)
    hi = (packed >> 4).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo).astype(np.int8)
    hi = np.where(hi > 7, hi - 16, hi).astype(np.int8)
    out = np.empty((packed.shape[0], packed.shape[1] * 2), np.int8)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


def weight_quantize(W: np.ndarray, fold, bits: int):
    """Per-output-channel weight quantization (Eq. 2).  W float16 [I][O]; returns qw int8 [O][I]
    (transposed, contraction axis contiguous) and s float32 [O]."""
    qmax(bits)
    wb = np.ascontiguousarray(_as_half_bits(W))
    I, O = W.shape
    f = None if fold is None else np.ascontiguousarray(fold, np.float32)
    if f is not None and f.size != I:
        raise ValueError("fold must have one factor per input channel")
    qw = np.empty((O, I), np.int8)
    s = np.empty(O, np.float32)
    _load().cq_oracle_weight_quantize(_p(wb), _i64(I), _i64(O), _p(f), ctypes.c_int(bits), _p(qw), _p(s))
    return qw, s


def weight_quantize_grouped(W: np.ndarray, fold, group: int, bits: int, want_dq: bool = True):
    """Group-wise weight quantization along the input-channel axis.  Returns qw int8 [O][I],
    s float32 [O][I/group] and (optionally) the dequantized weights float16 [I][O]."""
    qmax(bits)
    wb = np.ascontiguousarray(_as_half_bits(W))
    I, O = W.shape
    if group < 1 or I % group:
        raise ValueError("the group size must divide the number of input channels")
    f = None if fold is None else np.ascontiguousarray(fold, np.float32)
    qw = np.empty((O, I), np.int8)
    s = np.empty((O, I // group), np.float32)
    wdq = np.empty((I, O), np.uint16) if want_dq else None
    _load().cq_oracle_weight_quantize_grouped(_p(wb), _i64(I), _i64(O), _p(f), _i64(group), ctypes.c_int(bits),
                                              _p(qw), _p(s), _p(wdq))
    return qw, s, (None if wdq is None else wdq.view(np.float16))


def w8a8_linear(qx: np.ndarray, a: np.ndarray, qw: np.ndarray, s: np.ndarray,
                want_acc: bool = True, want_y: bool = True):
    """Integer linear layer: acc = qx . qw^T (int32, exact), Y = fl16(acc * a_i * s_k)."""
    qx = np.ascontiguousarray(qx, np.int8)
    qw = np.ascontiguousarray(qw, np.int8)
    a = np.ascontiguousarray(a, np.float32)
    s = np.ascontiguousarray(s, np.float32)
    T, I = qx.shape
    O, I2 = qw.shape
    if I != I2 or a.size != T or s.size != O:
        raise ValueError("shape mismatch")
    acc = np.empty((T, O), np.int32) if want_acc else None
    Y = np.empty((T, O), np.uint16) if want_y else None
    _load().cq_oracle_w8a8_linear(_p(qx), _p(a), _p(qw), _p(s), _i64(T), _i64(I), _i64(O), _p(Y),
                                  _i64(O), _p(acc))
    return (None if Y is None else Y.view(np.float16)), acc
