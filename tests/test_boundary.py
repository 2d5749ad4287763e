"""Host-side checks of the C-ABI library: it loads, exports what the header declares, and
rejects bad arguments on the host before anything is launched (no GPU needed)."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "crossquant.h")
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))


@pytest.fixture(scope="module")
def cq():
    import paper_2410_07505_amd as pkg
    return pkg


def declared_functions(headers=None):
    names = set()
    for h in (HEADERS if headers is None else headers):
        src = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names.update(re.findall(r"\b(crossquant_\w+)\s*\(", src))
    return sorted(names)


def test_header_declares_the_four_named_calls():
    names = declared_functions([HEADER])
    for n in ("crossquant_absmax", "crossquant_quantize", "crossquant_kernel_count", "crossquant_w8a8_linear"):
        assert n in names
    # benchmark calibration and test hooks are not in the method's header
    assert not [n for n in names if "calib" in n or "debug" in n]
    assert len(HEADERS) >= 2 and any("calib" in n for n in declared_functions())


def test_library_exports_every_declared_symbol(cq):
    lib = ctypes.CDLL(cq.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_version_and_status_strings(cq):
    assert cq.crossquant_version() >= 100
    seen = set()
    for code in range(0, -9, -1):
        s = cq.crossquant_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert cq.crossquant_status_string(-99) == "unknown status"


# Fake, suitably aligned, non-null "device pointers": every call below must fail validation on
# the host, so none of them is ever dereferenced or passed to a launch.
P = 0x10000


def test_absmax_argument_errors(cq):
    f = cq.raw.crossquant_absmax
    assert f(0, 4, 8, 8, P, P, None) == -1
    assert f(P, 4, 8, 8, 0, P, None) == -1
    assert f(P, 4, 8, 8, P, 0, None) == -1
    assert f(P, 0, 8, 8, P, P, None) == -2
    assert f(P, 4, 0, 8, P, P, None) == -2
    assert f(P, 4, 8, 7, P, P, None) == -2            # ldx < I
    assert f(P, -1, 8, 8, P, P, None) == -2
    assert f(P, 1 << 25, 8, 8, P, P, None) == -2
    assert f(P + 1, 4, 8, 8, P, P, None) == -5         # binary16 needs 2-byte alignment
    assert f(P, 4, 8, 8, P + 2, P, None) == -5


def test_quantize_argument_errors(cq):
    f = cq.raw.crossquant_quantize

    def call(X=P, T=4, I=8, ldx=8, t=P, c=P, alpha=0.15, bits=8, codes=P, xhat=P, rs=P, cs=P, zc=P):
        return f(X, T, I, ldx, t, c, alpha, bits, codes, xhat, rs, cs, zc, None)

    assert call(X=0) == -1 and call(t=0) == -1 and call(c=0) == -1
    assert call(codes=0) == -1 and call(rs=0) == -1 and call(cs=0) == -1
    assert call(T=0) == -2 and call(I=0) == -2 and call(ldx=4) == -2
    assert call(bits=3) == -3 and call(bits=16) == -3 and call(bits=0) == -3
    assert call(bits=4, I=7, ldx=8) == -3              # INT4 packs two channels per byte
    assert call(alpha=-0.01) == -4 and call(alpha=1.01) == -4 and call(alpha=float("nan")) == -4
    assert call(zc=P + 4) == -5 and call(xhat=P + 1) == -5
    # the factors are written while t and c are still being read: no overlap allowed
    far = dict(t=P, c=P + 0x1000, rs=P + 0x2000, cs=P + 0x3000)
    assert call(**{**far, "rs": P}) == -8
    assert call(**{**far, "rs": P + 12}) == -8           # last element of t (T = 4)
    assert call(**{**far, "cs": P + 0x1000 + 28}) == -8  # last element of c (I = 8)
    assert call(**{**far, "cs": P + 0x1000 - 28}) == -8  # cs's last element is c's first


@pytest.mark.parametrize("entry", ["crossquant_absmax_quantize", "crossquant_absmax_quantize_single_read"])
def test_absmax_quantize_argument_errors(cq, entry):
    f = getattr(cq.raw, entry)

    def call(X=P, T=4, I=8, ldx=8, alpha=0.15, bits=8, t=P, c=P, codes=P, xhat=P, rs=P, cs=P, zc=P):
        return f(X, T, I, ldx, alpha, bits, t, c, codes, xhat, rs, cs, zc, None)

    assert call(X=0) == -1 and call(t=0) == -1 and call(c=0) == -1 and call(codes=0) == -1 and call(rs=0) == -1
    assert call(T=0) == -2 and call(ldx=4) == -2
    assert call(bits=5) == -3 and call(alpha=1.5) == -4
    assert call(zc=P + 4) == -5 and call(xhat=P + 1) == -5
    assert call(rs=P) == -8 and call(c=P + 0x100, cs=P + 0x100) == -8


def test_batched_argument_errors(cq):
    f = cq.raw.crossquant_absmax_batched
    assert f(0, 2, 4, 8, 8, 32, P, P, None) == -1 and f(P, 2, 4, 8, 8, 32, 0, P, None) == -1
    assert f(P, 0, 4, 8, 8, 32, P, P, None) == -2
    assert f(P, 2, 4, 8, 8, 31, P, P, None) == -2          # sequences would overlap
    assert f(P, 1 << 20, 1 << 10, 8, 8, 1 << 13, P, P, None) == -2   # B*S over the limit
    g = cq.raw.crossquant_quantize_batched

    def call(X=P, B=2, S=4, I=8, ldx=8, bs=32, t=P, c=P, alpha=0.15, bits=8, codes=P, xhat=P, rs=P, cs=P, zc=P):
        return g(X, B, S, I, ldx, bs, t, c, alpha, bits, codes, xhat, rs, cs, zc, None)

    assert call(t=0) == -1 and call(rs=0) == -1
    assert call(codes=0) == -1                              # count only, but xhat given
    assert call(codes=0, xhat=0, zc=0) == -1                # count only without a counter
    assert call(B=0) == -2 and call(bs=8) == -2
    assert call(bits=7) == -3 and call(bits=4, I=7, ldx=8) == -3 and call(alpha=-0.5) == -4
    assert call(zc=P + 4) == -5
    # a launch has to stay below 2^32 threads: one-token sequences take a block each
    far = dict(t=P, c=P + (1 << 27), rs=P + (2 << 27), cs=P + (3 << 27))
    assert call(B=1 << 23, S=1, I=1, ldx=1, bs=1, **far) == -2          # 512-thread blocks
    assert f(P, 1 << 24, 1, 1, 1, 1, P, P, None) == -2                  # 256-thread blocks
    assert call(t=P, c=P + 0x1000, rs=P + 28, cs=P + 0x3000) == -8     # B*S = 8 row factors
    assert call(t=P, c=P + 0x1000, rs=P + 0x2000, cs=P + 0x1000 + 60) == -8   # B*I = 16 column factors


def test_kernel_count_argument_errors(cq):
    f = cq.raw.crossquant_kernel_count

    def call(X=P, T=4, I=8, ldx=8, t=P, c=P, alpha=1.0, bits=8, rs=P, cs=P, zc=P):
        return f(X, T, I, ldx, t, c, alpha, bits, rs, cs, zc, None)

    assert call(zc=0) == -1 and call(X=0) == -1
    assert call(rs=0) == -1 and call(cs=0) == -1            # the two work vectors: both or neither
    assert call(rs=0, cs=0, T=0) == -2                      # neither is fine: the next check is reached
    assert call(T=0) == -2
    assert call(bits=5) == -3
    assert call(alpha=2.0) == -4
    assert call(t=P, c=P + 0x1000, rs=P, cs=P + 0x3000) == -8
    assert call(t=P, c=P + 0x1000, rs=P + 0x2000, cs=P + 0x1000) == -8


def test_kernel_analysis_argument_errors(cq):
    f = cq.raw.crossquant_kernel_analysis

    def call(X=P, T=4, I=8, ldx=8, t=P, c=P, alpha=0.15, bits=8, xrk=P, rs=P, cs=P, cnt=P):
        return f(X, T, I, ldx, t, c, alpha, bits, xrk, rs, cs, cnt, None)

    assert call(cnt=0) == -1 and call(X=0) == -1 and call(cs=0) == -1 and call(rs=0) == -1
    assert call(rs=0, cs=0, I=0) == -2                      # no work vectors: allowed
    assert call(I=0) == -2 and call(ldx=7) == -2
    assert call(bits=6) == -3
    assert call(alpha=-1.0) == -4
    assert call(cnt=P + 4) == -5 and call(xrk=P + 1) == -5
    far = dict(t=P, c=P + 0x1000, rs=P + 0x2000, cs=P + 0x3000)
    assert call(**{**far, "rs": P + 12}) == -8 and call(**{**far, "cs": P + 0x1000}) == -8


def test_weight_quantize_argument_errors(cq):
    f = cq.raw.crossquant_weight_quantize
    assert f(0, 8, 8, None, 8, P, P, None) == -1
    assert f(P, 8, 8, None, 8, 0, P, None) == -1
    assert f(P, 0, 8, None, 8, P, P, None) == -2
    assert f(P, 8, 8, None, 2, P, P, None) == -3
    assert f(P, 8, 8, P + 2, 8, P, P, None) == -5


def test_weight_quantize_grouped_argument_errors(cq):
    f = cq.raw.crossquant_weight_quantize_grouped
    assert f(0, 8, 8, None, 8, 8, P, P, None, None) == -1
    assert f(P, 8, 8, None, 8, 8, P, 0, None, None) == -1
    assert f(P, 8, 8, None, 3, 8, P, P, None, None) == -2       # group does not divide I
    assert f(P, 8, 8, None, 0, 8, P, P, None, None) == -2
    assert f(P, 8, 8, None, 16, 8, P, P, None, None) == -2
    assert f(P, 8, 8, None, 8, 7, P, P, None, None) == -3
    assert f(P, 8, 8, None, 8, 8, P, P, P + 1, None) == -5


def test_unpack_int4_argument_errors(cq):
    f = cq.raw.crossquant_unpack_int4
    assert f(0, 4, 8, P, None) == -1 and f(P, 4, 8, 0, None) == -1
    assert f(P, 0, 8, P, None) == -2 and f(P, 4, 7, P, None) == -2


def test_fp6_argument_errors(cq):
    n = cq.raw.crossquant_fp6_packed_bytes
    assert n(32, 128) == 32 * 128 * 6 // 8 and n(33, 128) == 64 * 128 * 6 // 8 and n(300, 256) == 320 * 256 * 6 // 8
    assert n(0, 128) == -1 and n(32, 64) == -1
    nw = cq.raw.crossquant_fp6_packed_weight_bytes          # whole groups of 64 output channels
    assert nw(64, 128) == n(64, 128) and nw(8, 128) == n(64, 128) and nw(65, 256) == n(128, 256) and nw(300, 256) == n(320, 256)
    assert nw(0, 128) == -1 and nw(64, 64) == -1
    for f in (cq.raw.crossquant_pack_fp6, cq.raw.crossquant_pack_fp6_weights):
        assert f(0, 8, 32, 128, P, None) == -1 and f(P, 8, 32, 128, 0, None) == -1
        assert f(P, 8, 0, 128, P, None) == -2 and f(P, 6, 32, 128, P, None) == -3
        assert f(P, 8, 32, 100, P, None) == -6 and f(P + 4, 8, 32, 128, P, None) == -5
    q = cq.raw.crossquant_quantize_fp6
    assert q(P, 4, 128, 128, P, P, 0.15, 0, None, P, P, None, None) == -1
    assert q(P, 4, 128, 100, P, P, 0.15, P, None, P, P, None, None) == -2
    assert q(P, 4, 128, 128, P, P, 1.5, P, None, P, P, None, None) == -4
    assert q(P, 4, 64, 64, P, P, 0.15, P, None, P, P, None, None) == -6
    assert q(P, 4, 128, 128, P, P, 0.15, P + 8, None, P, P, None, None) == -6
    assert q(P, 4, 128, 128, P, P + 0x1000, 0.15, P, None, P, P + 0x3000, None, None) == -8
    g = cq.raw.crossquant_w4a4_linear

    def call(qx=P, rs=P, qw=P, ws=P, T=4, I=128, O=8, Y=P, ldy=8, acc=None):
        return g(qx, rs, qw, ws, T, I, O, Y, ldy, acc, None)

    assert call(qx=0) == -1 and call(Y=0) == -1 and call(ws=0) == -1
    assert call(T=0) == -2 and call(ldy=4) == -2 and call(I=1 << 19) == -2
    assert call(Y=P + 1) == -5
    assert call(I=64) == -6 and call(O=12, ldy=16) == -6 and call(ldy=12) == -6 and call(qx=P + 8) == -6
    assert call(ldy=1 << 22) == -6


def test_calibration_argument_errors(cq):
    r, c, m = cq.raw.crossquant_calib_read, cq.raw.crossquant_calib_copy, cq.raw.crossquant_calib_mfma_i8
    assert r(0, 1024, None, None) == -1 and r(P, 0, None, None) == -2 and r(P, 1000, None, None) == -2
    assert r(P + 8, 1024, None, None) == -5
    assert c(P, 0, 1024, None) == -1 and c(P, P + 4096, 24, None) == -2 and c(P, P + 4, 1024, None) == -5
    assert m(0, 0, None, None, None) == -2 and m(10, 4, None, None, None) == -6
    m6 = cq.raw.crossquant_calib_mfma_f6
    assert m6(0, None, None, None) == -2 and m6(10, 2, None, None) == -5


def test_linear_argument_errors(cq):
    f = cq.raw.crossquant_w8a8_linear

    def call(qx=P, rs=P, qw=P, ws=P, T=4, I=16, O=8, Y=P, ldy=8, acc=None):
        return f(qx, rs, qw, ws, T, I, O, Y, ldy, acc, None)

    assert call(qx=0) == -1 and call(rs=0) == -1 and call(qw=0) == -1 and call(ws=0) == -1 and call(Y=0) == -1
    assert call(T=0) == -2 and call(O=0) == -2 and call(I=0) == -2
    assert call(ldy=7) == -2
    assert call(I=200000) == -2                         # accumulator could overflow int32
    assert call(Y=P + 1) == -5 and call(acc=P + 2) == -5


def test_quantize_linear_fused_argument_errors(cq):
    f = cq.raw.crossquant_quantize_linear_fused

    def call(X=P, T=4, I=128, ldx=128, t=P, c=P + 0x1000, alpha=0.15, bits=8, qw=P, ws=P, O=8, Y=P, ldy=8,
             rs=P + 0x2000, cs=P + 0x3000, acc=None):
        return f(X, T, I, ldx, t, c, alpha, bits, qw, ws, O, Y, ldy, rs, cs, acc, None)

    assert call(X=0) == -1 and call(t=0) == -1 and call(qw=0) == -1 and call(Y=0) == -1 and call(rs=0) == -1
    assert call(T=0) == -2 and call(O=0) == -2 and call(ldy=4) == -2 and call(ldx=64) == -2
    assert call(bits=6) == -3 and call(alpha=1.5) == -4
    assert call(Y=P + 1) == -5 and call(acc=P + 2) == -5
    assert call(rs=P) == -8 and call(cs=P + 0x1000) == -8
    assert call(I=64, ldx=64) == -6 and call(ldx=132) == -6 and call(X=P + 2) == -6 and call(cs=P + 0x3004) == -6


def test_python_wrappers_refuse_cpu_tensors(cq):
    import torch
    X = torch.zeros((4, 8), dtype=torch.float16)
    with pytest.raises(ValueError):
        cq.crossquant_absmax(X)


def test_python_wrappers_check_every_buffer_they_are_given(cq):
    """The C ABI sees pointers only, so the binding refuses buffers of the wrong length, shape, dtype or
    device before the library is called (CPU tensors reach these checks; a correct set fails later, on
    "must be a GPU tensor")."""
    import torch
    T, I, O = 4, 8, 16
    X = torch.zeros((T, I), dtype=torch.float16)
    f32 = lambda n: torch.zeros(n, dtype=torch.float32)
    t, c = f32(T), f32(I)
    with pytest.raises(ValueError, match="GPU"):
        cq.crossquant_absmax(X, t=t, c=c)
    with pytest.raises(ValueError, match="t must have shape"):
        cq.crossquant_absmax(X, t=c, c=t)                                  # swapped
    with pytest.raises(ValueError, match="c must have shape"):
        cq.crossquant_absmax(X, t=t, c=f32(I - 1))
    with pytest.raises(TypeError, match="t must have dtype"):
        cq.crossquant_absmax(X, t=torch.zeros(T, dtype=torch.float64), c=c)
    with pytest.raises(ValueError, match="contiguous"):
        cq.crossquant_absmax(X, t=f32(2 * T)[::2], c=c)
    for fn in (cq.crossquant_quantize, ):
        with pytest.raises(ValueError, match="t must have shape"):
            fn(X, c, t, 0.15, 8)
        with pytest.raises(ValueError, match="codes must have shape"):
            fn(X, t, c, 0.15, 8, codes=torch.zeros((T, I // 2), dtype=torch.int8))
        with pytest.raises(TypeError, match="codes must have dtype"):
            fn(X, t, c, 0.15, 4, codes=torch.zeros((T, I // 2), dtype=torch.int8))
        with pytest.raises(ValueError, match="xhat must have shape"):
            fn(X, t, c, 0.15, 8, xhat=torch.zeros((T, I - 1), dtype=torch.float16))
        with pytest.raises(ValueError, match="row_scale must have shape"):
            fn(X, t, c, 0.15, 8, row_scale=f32(I), col_scale=f32(I))
        with pytest.raises(ValueError, match="zero_count must have shape"):
            fn(X, t, c, 0.15, 8, zero_count=torch.zeros(2, dtype=torch.int64))
        with pytest.raises(TypeError, match="zero_count must have dtype"):
            fn(X, t, c, 0.15, 8, zero_count=torch.zeros(1, dtype=torch.int32))
    with pytest.raises(ValueError, match="c must have shape"):
        cq.crossquant_absmax_quantize(X, 0.15, 8, c=f32(T))
    with pytest.raises(ValueError, match="both or neither"):
        cq.crossquant_kernel_count(X, t, c, 1.0, 8, row_scale=f32(T))
    with pytest.raises(ValueError, match="t must have shape"):
        cq.crossquant_kernel_count(X, c, t, 1.0, 8)
    with pytest.raises(ValueError, match="counters must have shape"):
        cq.crossquant_kernel_analysis(X, t, c, 1.0, 8, counters=torch.zeros(2, dtype=torch.int64))
    with pytest.raises(ValueError, match="xrk must have shape"):
        cq.crossquant_kernel_analysis(X, t, c, 1.0, 8, xrk=torch.zeros((I, T), dtype=torch.float16))
    qx, qw = torch.zeros((T, I), dtype=torch.int8), torch.zeros((O, I), dtype=torch.int8)
    with pytest.raises(ValueError, match="row_scale must have shape"):
        cq.crossquant_w8a8_linear(qx, f32(O), qw, f32(O))
    with pytest.raises(ValueError, match="w_scale must have shape"):
        cq.crossquant_w8a8_linear(qx, f32(T), qw, f32(T))
    with pytest.raises(ValueError, match="Y must be a float16 tensor of shape"):
        cq.crossquant_w8a8_linear(qx, f32(T), qw, f32(O), Y=torch.zeros((T, O - 1), dtype=torch.float16))
    with pytest.raises(ValueError, match="Y must be a float16 tensor of shape"):
        cq.crossquant_w8a8_linear(qx, f32(T), qw, f32(O), Y=torch.zeros((T, O), dtype=torch.float32))
    with pytest.raises(ValueError, match="acc_debug must have shape"):
        cq.crossquant_w8a8_linear(qx, f32(T), qw, f32(O), acc_debug=torch.zeros((O, T), dtype=torch.int32))
    with pytest.raises(ValueError, match="contraction lengths"):
        cq.crossquant_w8a8_linear(qx, f32(T), torch.zeros((O, I + 1), dtype=torch.int8), f32(O))
