"""Pins for the CPU oracle: closed forms, brute force, special cases, invariants.

The oracle is what every GPU parity test is measured against, so it is first checked here
against things that are not itself: numpy's own binary16 conversions, exact rational arithmetic
(``fractions.Fraction``), an independently written per-token routine (Eq. 1), a float64
evaluation of the CrossQuant equation, hand-derived cases (``tests/golden/exact_cases.txt``;
the paper's own worked examples are figures and are not available as text) and the
inequalities the paper proves (kernel-size analysis, cases I and II).
"""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "exact_cases.txt")


# ----------------------------------------------------------------------------- helpers
def rne_fraction(q: Fraction) -> int:
    """Round an exact rational half-to-even."""
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def outlier_matrix(T, I, seed, n_out=3, scale=60.0, dist="normal"):
    return workloads.activation(T, I, dist=dist, n_outlier=n_out, scale_lo=scale, scale_hi=scale,
                                seed=seed)


def read_golden():
    cases, cur = [], {}
    for line in open(GOLDEN):
        line = line.strip()
        if line.startswith("#"):
            continue
        if not line:
            if cur:
                cases.append(cur)
                cur = {}
            continue
        k, v = line.split(":", 1)
        cur[k.strip()] = v.strip()
    if cur:
        cases.append(cur)

    def mat(s, dt):
        return np.array([[float(x) for x in row.split()] for row in s.split(";")]).astype(dt)

    out = []
    for c in cases:
        d = {"name": c["name"], "bits": int(c["bits"]), "alpha": float(c["alpha"]),
             "X": mat(c["X"], np.float16), "t": mat(c["t"], np.float32)[0],
             "c": mat(c["c"], np.float32)[0], "codes": mat(c["codes"], np.int8), "Z": int(c["Z"])}
        if "packed" in c:
            d["packed"] = mat(c["packed"], np.uint8)
        out.append(d)
    return out


# ----------------------------------------------------------------------------- binary16 conversions
def test_half_to_float_exhaustive_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], np.float32)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite].view(np.uint32), want[finite].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))


def test_float_to_half_vs_numpy():
    rng = np.random.default_rng(7)
    vals = [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25,
            2.0 ** -25 * 1.0001, 2.0 ** -14, 2.0 ** -14 * (1 - 2.0 ** -12), 1.0 + 2.0 ** -11,
            1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5, 6.1e-5, 5.9e-8, 3.0e-8, 2.9e-8]
    vals += list(rng.standard_normal(20000) * 10.0 ** rng.integers(-9, 5, 20000))
    # all midpoints between adjacent positive halfs (ties must go to even)
    h = np.arange(0, 0x7BFF, dtype=np.uint16).view(np.float16).astype(np.float64)
    h2 = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    vals += list(((h + h2) / 2)[::7])
    vals = np.array(vals, np.float32)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in vals], np.uint16)
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------- absmax
def test_absmax_is_the_textbook_definition():
    X = outlier_matrix(37, 53, seed=11)
    t, c = oracle.absmax(X)
    A = np.abs(X.astype(np.float64))
    assert np.array_equal(t.astype(np.float64), A.max(axis=1))
    assert np.array_equal(c.astype(np.float64), A.max(axis=0))
    # brute force, pure Python
    for i in (0, 17, 36):
        assert float(t[i]) == max(abs(float(v)) for v in X[i])
    for j in (0, 29, 52):
        assert float(c[j]) == max(abs(float(X[i, j])) for i in range(X.shape[0]))


def test_absmax_respects_leading_dimension_and_sign():
    base = outlier_matrix(16, 40, seed=3)
    view = base[:, 4:28]                       # ldx = 40 > I = 24
    t, c = oracle.absmax(view)
    t2, c2 = oracle.absmax(np.ascontiguousarray(view))
    assert np.array_equal(t, t2) and np.array_equal(c, c2)
    X = np.zeros((3, 4), np.float16)
    X[1, 2] = -9.0                              # a negative entry must count by magnitude
    t, c = oracle.absmax(X)
    assert t.tolist() == [0.0, 9.0, 0.0] and c.tolist() == [0.0, 0.0, 9.0, 0.0]


# ----------------------------------------------------------------------------- scales
@pytest.mark.parametrize("alpha", [0.0, 0.15, 0.5, 0.85, 1.0])
@pytest.mark.parametrize("bits", [4, 8])
def test_scales_match_float64_power(alpha, bits):
    X = outlier_matrix(64, 96, seed=5)
    t, c = oracle.absmax(X)
    a, b = oracle.scales(t, c, alpha, bits)
    al = float(np.float32(alpha))
    qm = 2 ** (bits - 1) - 1
    want_a = (np.power(t.astype(np.float64), al) / qm).astype(np.float32)
    want_b = np.power(c.astype(np.float64), 1.0 - al).astype(np.float32)
    assert np.array_equal(a, want_a) and np.array_equal(b, want_b)
    # product of the two factors is the CrossQuant step, to float32 accuracy
    step = np.power(t.astype(np.float64), al)[:, None] * np.power(c.astype(np.float64), 1 - al)[None] / qm
    rel = np.abs(a[:, None].astype(np.float64) * b[None].astype(np.float64) - step) / step
    assert rel.max() < 2.0 ** -22


def test_scales_closed_forms_at_alpha_0_and_1():
    t = np.array([0.0, 1.0, 3.5, 127.0, 60000.0], np.float32)
    c = np.array([0.0, 2.0, 0.007], np.float32)
    a, b = oracle.scales(t, c, 1.0, 8)
    assert np.array_equal(b, np.ones(3, np.float32))              # alpha = 1: per-token
    assert np.array_equal(a, (t.astype(np.float64) / 127).astype(np.float32))
    a, b = oracle.scales(t, c, 0.0, 4)
    assert np.array_equal(a, np.full(5, np.float32(1.0 / 7.0)))   # alpha = 0: pow(x, 0) = 1, also at 0
    assert np.array_equal(b, c)
    a, b = oracle.scales(t, c, 0.5, 8)
    assert a[0] == 0.0 and b[0] == 0.0                            # zero maxima give a zero step


# ----------------------------------------------------------------------------- codes
@pytest.mark.parametrize("case", read_golden(), ids=lambda c: c["name"])
def test_hand_derived_cases(case):
    X = case["X"]
    t, c = oracle.absmax(X)
    assert np.array_equal(t, case["t"]) and np.array_equal(c, case["c"])
    r = oracle.quantize(X, t, c, case["alpha"], case["bits"])
    codes = r["codes"] if case["bits"] == 8 else oracle.unpack_int4(r["codes"])
    assert np.array_equal(codes, case["codes"])
    assert r["Z"] == case["Z"] == oracle.kernel_count(X, t, c, case["alpha"], case["bits"])
    assert r["clamp_hits"] == 0
    if "packed" in case:
        assert np.array_equal(r["codes"], case["packed"])


@pytest.mark.parametrize("bits", [4, 8])
def test_maximum_elements_map_to_qmax(bits):
    qm = 2 ** (bits - 1) - 1
    X = outlier_matrix(48, 64, seed=21)
    t, c = oracle.absmax(X)
    A = np.abs(X.astype(np.float32))
    gi, gj = np.unravel_index(np.argmax(A), A.shape)
    for alpha in (0.0, 0.15, 0.5, 1.0):
        r = oracle.quantize(X, t, c, alpha, bits)
        codes = r["codes"] if bits == 8 else oracle.unpack_int4(r["codes"])
        assert r["clamp_hits"] == 0 and np.abs(codes).max() <= qm
        # the global maximum has t_i = c_j = |x|, so its step is |x|/q_max for every alpha
        assert codes[gi, gj] == qm * np.sign(float(X[gi, gj]))
        if alpha == 1.0:       # Eq. 1: each row's maximum sits on +-q_max
            rows = np.arange(X.shape[0])
            jm = A.argmax(axis=1)
            assert np.array_equal(np.abs(codes[rows, jm]), np.full(X.shape[0], qm))
        if alpha == 0.0:       # pure column step: each column's maximum sits on +-q_max
            cols = np.arange(X.shape[1])
            im = A.argmax(axis=0)
            assert np.array_equal(np.abs(codes[im, cols]), np.full(X.shape[1], qm))


@pytest.mark.parametrize("bits", [4, 8])
def test_alpha_one_is_per_token_quantization(bits):
    """Table 1's caption: alpha = 1 is per-token quantization.  Eq. 1 written independently."""
    qm = np.float32(2 ** (bits - 1) - 1)
    X = outlier_matrix(40, 72, seed=8)
    Xf = X.astype(np.float32)
    step = np.abs(Xf).max(axis=1) / qm                    # Delta_i = t_i / (2^(N-1)-1)
    want = np.rint(Xf / step[:, None]).astype(np.int8)    # numpy rint is half-to-even
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, 1.0, bits)
    codes = r["codes"] if bits == 8 else oracle.unpack_int4(r["codes"])
    assert np.array_equal(codes, want)
    assert r["Z"] == int((want == 0).sum())


@pytest.mark.parametrize("alpha", [0.0, 0.15, 0.5, 0.75])
def test_codes_agree_with_float64_crossquant_equation(alpha):
    """Exact-within-bound: against the CrossQuant equation in float64, a code may differ by one
    and only where the real quotient sits within float32 rounding of a rounding tie."""
    X = outlier_matrix(96, 128, seed=31, dist="student_t3")
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, alpha, 8)
    al = float(np.float32(alpha))
    step = (t.astype(np.float64) ** al)[:, None] * (c.astype(np.float64) ** (1 - al))[None] / 127.0
    quo = X.astype(np.float64) / step
    want = np.rint(quo)
    diff = r["codes"].astype(np.float64) - want
    bad = diff != 0
    assert np.abs(diff).max() <= 1
    assert bad.mean() < 1e-3
    dist_to_tie = np.abs(np.abs(quo - np.floor(quo)) - 0.5)
    assert np.all(dist_to_tie[bad] < 1e-4)


def test_sign_symmetry_and_permutation_equivariance():
    X = outlier_matrix(32, 48, seed=13)
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, 0.15, 8)
    Xn = (-X).astype(np.float16)
    tn, cn = oracle.absmax(Xn)
    rn = oracle.quantize(Xn, tn, cn, 0.15, 8)
    assert np.array_equal(rn["codes"], -r["codes"]) and rn["Z"] == r["Z"]
    rng = np.random.default_rng(2)
    pr, pc = rng.permutation(32), rng.permutation(48)
    Xp = np.ascontiguousarray(X[pr][:, pc])
    tp, cp = oracle.absmax(Xp)
    rp = oracle.quantize(Xp, tp, cp, 0.15, 8)
    assert np.array_equal(tp, t[pr]) and np.array_equal(cp, c[pc])
    assert np.array_equal(rp["codes"], r["codes"][pr][:, pc])
    assert np.array_equal(rp["xhat"].view(np.uint16), r["xhat"].view(np.uint16)[pr][:, pc])


def test_int4_packing_layout():
    X = outlier_matrix(8, 16, seed=4)
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, 0.15, 4)
    packed = r["codes"]
    assert packed.shape == (8, 8) and packed.dtype == np.uint8
    codes = oracle.unpack_int4(packed)
    for i in range(8):
        for j in range(0, 16, 2):
            assert packed[i, j // 2] == ((int(codes[i, j]) & 0xF) | ((int(codes[i, j + 1]) & 0xF) << 4))
    assert np.abs(codes).max() <= 7


# ----------------------------------------------------------------------------- brute force, exact rationals
@pytest.mark.parametrize("alpha,bits", [(1.0, 8), (0.0, 8), (1.0, 4), (0.0, 4), (0.5, 8)])
def test_tiny_matrix_bruteforce_with_exact_rationals(alpha, bits):
    """Codes and kernel size on an 8x8 matrix by a double loop in exact rational arithmetic.
    For alpha = 0.5 the entries are arranged so that t_i * c_j is a perfect square."""
    qm = 2 ** (bits - 1) - 1
    rng = np.random.default_rng(int(alpha * 10) + bits)
    if alpha == 0.5:
        # rows/cols dominated by perfect squares on the diagonal block: t_i, c_j in {4, 16, 64}
        X = (rng.integers(-15, 16, (8, 8)) / 8.0).astype(np.float16)
        sq = [4.0, 16.0, 64.0, 4.0, 16.0, 64.0, 4.0, 16.0]
        for k in range(8):
            X[k, :] = np.clip(X[k, :], -1.9, 1.9)
        for k in range(8):
            X[k, k] = sq[k]
    else:
        X = (rng.integers(-200, 201, (8, 8)) / 16.0).astype(np.float16)
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, alpha, bits)
    codes = r["codes"] if bits == 8 else oracle.unpack_int4(r["codes"])
    Z = 0
    near_tie = 0
    for i in range(8):
        ti = max(abs(Fraction(float(v))) for v in X[i])
        for j in range(8):
            cj = max(abs(Fraction(float(X[k, j]))) for k in range(8))
            if alpha == 1.0:
                step = ti / qm
            elif alpha == 0.0:
                step = cj / qm
            else:
                root = Fraction(int(round(float(ti * cj) ** 0.5)))
                assert root * root == ti * cj
                step = root / qm
            quo = Fraction(float(X[i, j])) / step
            want = rne_fraction(quo)
            frac = abs(quo - (quo.numerator // quo.denominator) - Fraction(1, 2))
            if frac < Fraction(1, 10 ** 5):
                near_tie += 1          # float32 rounding of the step may legitimately flip these
                continue
            assert codes[i, j] == want, (i, j, float(quo))
            Z += want == 0
    if near_tie == 0:
        assert r["Z"] == Z
    assert near_tie <= 4


# ----------------------------------------------------------------------------- dequantized output
@pytest.mark.parametrize("bits", [4, 8])
def test_dequantized_output(bits):
    X = outlier_matrix(64, 80, seed=17)
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, 0.15, bits)
    codes = (r["codes"] if bits == 8 else oracle.unpack_int4(r["codes"])).astype(np.float32)
    D = r["a"][:, None] * r["b"][None, :]
    # numpy's own float32 -> float16 rounding of code * step
    want = (codes * D).astype(np.float16)
    assert np.array_equal(r["xhat"].view(np.uint16), want.view(np.uint16))
    # reconstruction error at most half a step plus half an ulp of the binary16 result
    xh = r["xhat"].astype(np.float64)
    ulp = np.spacing(np.abs(r["xhat"])).astype(np.float64)
    err = np.abs(xh - X.astype(np.float64))
    assert np.all(err <= 0.5 * D.astype(np.float64) * (1 + 1e-6) + 0.5 * ulp)


# ----------------------------------------------------------------------------- quantization kernel
@pytest.mark.parametrize("alpha", [0.15, 1.0])
def test_kernel_count_equals_zero_bound_form(alpha):
    """Definition 1: code 0  <=>  |x| < B = 0.5 * step, up to exact ties |x| = B (which
    half-to-even also sends to 0) -- counted separately and added."""
    X = outlier_matrix(128, 96, seed=41)
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, alpha, 8)
    D = (r["a"][:, None] * r["b"][None, :]).astype(np.float64)
    A = np.abs(X.astype(np.float64))
    quo = np.abs((X.astype(np.float32) / (r["a"][:, None] * r["b"][None, :])).astype(np.float64))
    strictly_inside = int((quo < 0.5).sum())
    ties = int((quo == 0.5).sum())
    assert r["Z"] == strictly_inside + ties == int((r["codes"] == 0).sum())
    assert r["Z"] == oracle.kernel_count(X, t, c, alpha, 8)
    # the real-number form agrees except within float32 rounding of the bound
    real = int((A < 0.5 * D).sum())
    assert abs(real - r["Z"]) <= 2


def test_kernel_shrinks_from_per_token_to_crossquant_on_outlier_inputs():
    """The paper's headline observation (Fig. 4, Table 1, kernel-size analysis)."""
    for name in ("C1",):
        X = workloads.config_activation(name)
        t, c = oracle.absmax(X)
        z_pt = oracle.kernel_count(X, t, c, 1.0, 8)
        z_cq = oracle.kernel_count(X, t, c, 0.15, 8)
        assert z_cq < z_pt / 5
    X = outlier_matrix(256, 512, seed=9, n_out=3, scale=80.0, dist="student_t3")
    t, c = oracle.absmax(X)
    zs = [oracle.kernel_count(X, t, c, al, 8) for al in (0.0, 0.15, 0.5, 1.0)]
    assert zs[1] < zs[3] and zs[2] < zs[3]


def test_case_one_and_case_two_zero_bounds():
    """Kernel-size analysis: c_j < t_i  =>  B~_ij < B_ij ; c_j >= t_i  =>  B~_ij >= B_ij."""
    X = outlier_matrix(64, 64, seed=23)
    t, c = oracle.absmax(X)
    a1, b1 = oracle.scales(t, c, 1.0, 8)
    B = 0.5 * a1[:, None].astype(np.float64) * b1[None].astype(np.float64)
    for alpha in (0.0, 0.15, 0.75):
        a, b = oracle.scales(t, c, alpha, 8)
        Bt = 0.5 * a[:, None].astype(np.float64) * b[None].astype(np.float64)
        case1 = c[None, :] < t[:, None]
        margin = 1e-6 * B
        assert np.all(Bt[case1] < B[case1] + margin[case1])
        assert np.all(Bt[~case1] >= B[~case1] - margin[~case1])
        strict = case1 & (c[None, :] < 0.99 * t[:, None])
        assert np.all(Bt[strict] < B[strict])


def test_kernel_proportion_matches_gaussian_expectation():
    """Per-token on pure N(0,1) rows: P(code = 0) = 2*Phi(B) - 1 with B = t_i / 254."""
    from math import erf, sqrt
    X = workloads.activation(256, 1024, seed=77)
    t, c = oracle.absmax(X)
    z = oracle.kernel_count(X, t, c, 1.0, 8)
    expect = sum(erf((float(ti) / 254.0) / sqrt(2.0)) for ti in t) * X.shape[1]
    assert abs(z - expect) < 6 * sqrt(expect)


def test_all_zero_rows_and_columns():
    X = outlier_matrix(12, 16, seed=6)
    X[3, :] = 0
    X[:, 5] = 0
    t, c = oracle.absmax(X)
    assert t[3] == 0 and c[5] == 0
    for alpha in (0.0, 0.15, 1.0):
        r = oracle.quantize(X, t, c, alpha, 8)
        assert np.all(r["codes"][3] == 0) and np.all(r["codes"][:, 5] == 0)
        assert np.all(r["xhat"][3] == 0) and np.all(r["xhat"][:, 5] == 0)
        assert np.all(np.isfinite(r["xhat"].astype(np.float32)))
        assert r["Z"] == int((r["codes"] == 0).sum())


# ----------------------------------------------------------------------------- weights
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("use_fold", [False, True])
def test_weight_quantize_per_output_channel(bits, use_fold):
    qm = 2 ** (bits - 1) - 1
    W = workloads.weight(48, 20, seed=3)
    fold = None
    Wf = W.astype(np.float32)
    if use_fold:
        fold = np.random.default_rng(1).uniform(0.5, 4.0, 48).astype(np.float32)
        Wf = fold[:, None] * Wf                      # float32 product, one rounding
    qw, s = oracle.weight_quantize(W, fold, bits)
    assert qw.shape == (20, 48) and s.shape == (20,)
    m = np.abs(Wf).max(axis=0)
    want_s = m / np.float32(qm)
    assert np.array_equal(s, want_s)
    want_q = np.rint(Wf / want_s[None, :]).astype(np.int8).T     # Eq. 2, transposed storage
    assert np.array_equal(qw, want_q)
    # each output channel's largest weight sits on +-q_max
    jm = np.abs(Wf).argmax(axis=0)
    assert np.array_equal(np.abs(qw[np.arange(20), jm]), np.full(20, qm))


def test_weight_quantize_zero_channel():
    W = workloads.weight(8, 4, seed=5)
    W[:, 2] = 0
    qw, s = oracle.weight_quantize(W, None, 8)
    assert s[2] == 0 and np.all(qw[2] == 0)


# ----------------------------------------------------------------------------- linear
def test_linear_accumulators_are_the_integer_product():
    qx = workloads.int8_codes(13, 70, seed=1)
    qw = workloads.int8_codes(9, 70, seed=2)
    rng = np.random.default_rng(3)
    a = rng.uniform(1e-3, 1e-1, 13).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, 9).astype(np.float32)
    Y, acc = oracle.w8a8_linear(qx, a, qw, s)
    want = qx.astype(np.int64) @ qw.astype(np.int64).T
    assert np.array_equal(acc.astype(np.int64), want)
    y32 = (want.astype(np.float32) * a[:, None]) * s[None, :]
    assert np.array_equal(Y.view(np.uint16), y32.astype(np.float16).view(np.uint16))
    y64 = want.astype(np.float64) * a[:, None].astype(np.float64) * s[None].astype(np.float64)
    assert np.all(np.abs(Y.astype(np.float64) - y64) <= 1e-3 * np.abs(y64) + 1e-7)


def test_linear_extreme_accumulator():
    I = 8192
    qx = np.full((2, I), 127, np.int8)
    qx[1] = -127
    qw = np.full((3, I), 127, np.int8)
    _, acc = oracle.w8a8_linear(qx, np.ones(2, np.float32), qw, np.ones(3, np.float32), want_y=False)
    assert acc[0, 0] == 127 * 127 * I and acc[1, 2] == -127 * 127 * I


def test_end_to_end_linear_tracks_the_fp_product_and_crossquant_beats_per_token():
    """Folding b_j into W gives Y ~= X W; on outlier inputs alpha = 0.15 loses less than alpha = 1."""
    X = workloads.config_activation("C1")
    W = workloads.config_weight("C1")
    ref = X.astype(np.float64) @ W.astype(np.float64)
    t, c = oracle.absmax(X)
    errs = {}
    for alpha in (0.15, 1.0):
        r = oracle.quantize(X, t, c, alpha, 8, want_xhat=False)
        qw, s = oracle.weight_quantize(W, r["b"], 8)
        Y, _ = oracle.w8a8_linear(r["codes"], r["a"], qw, s)
        errs[alpha] = np.linalg.norm(Y.astype(np.float64) - ref) / np.linalg.norm(ref)
    assert errs[0.15] < 0.05 and errs[1.0] < 0.2
    assert errs[0.15] < errs[1.0]


# ----------------------------------------------------------------------------- Remove Kernel, Table 1 indicators
@pytest.mark.parametrize("alpha,bits", [(1.0, 8), (0.15, 8), (0.15, 4), (0.0, 8)])
def test_remove_kernel_matrix(alpha, bits):
    """Kernel elements become zero, all others keep their FP16 value (Fig. 1 caption)."""
    X = outlier_matrix(48, 96, seed=61)
    X[3, 7] = np.float16(-0.0)
    t, c = oracle.absmax(X)
    r = oracle.quantize(X, t, c, alpha, bits)
    codes = r["codes"] if bits == 8 else oracle.unpack_int4(r["codes"])
    an = oracle.kernel_analysis(X, t, c, alpha, bits)
    want = np.where(codes == 0, np.float16(0.0), X)
    assert np.array_equal(an["xrk"].view(np.uint16), want.view(np.uint16))
    assert an["Z"] == r["Z"] == int((an["xrk"].view(np.uint16) == 0).sum())
    assert np.array_equal(an["a"], r["a"]) and np.array_equal(an["b"], r["b"])
    # removing the kernel changes nothing that quantization would have kept
    r2 = oracle.quantize(an["xrk"], t, c, alpha, bits)
    assert np.array_equal(r2["codes"], r["codes"])


def test_table1_indicators_bruteforce():
    X = outlier_matrix(40, 56, seed=67)
    t, c = oracle.absmax(X)
    for alpha in (0.0, 0.15, 0.45, 0.75):
        an = oracle.kernel_analysis(X, t, c, alpha, 8, want_xrk=False)
        # case II count by a plain double loop
        ge = sum(1 for i in range(40) for j in range(56) if c[j] >= t[i])
        assert an["n_col_ge_row"] == ge == int((c[None, :] >= t[:, None]).sum())
        # zero bounds from an independent float64 evaluation; equality only possible at c_j == t_i
        al = float(np.float32(alpha))
        Bt = 0.5 * (t.astype(np.float64) ** al)[:, None] * (c.astype(np.float64) ** (1 - al))[None] / 127.0
        B = 0.5 * t.astype(np.float64)[:, None] / 127.0 * np.ones((1, 56))
        clear = np.abs(Bt - B) > 1e-6 * B
        lo = int(((Bt < B) & clear).sum())
        hi = lo + int((~clear).sum())
        assert lo <= an["n_bound_smaller"] <= hi
        # the kernel-size analysis: case I (c_j < t_i) <=> B~ < B, so the two indicators partition
        # the matrix except where c_j == t_i within rounding
        near_equal = int((np.abs(c[None, :] - t[:, None]) <= 1e-6 * t[:, None]).sum())
        assert abs(an["n_col_ge_row"] + an["n_bound_smaller"] - X.size) <= near_equal
    # alpha = 1 is per-token itself: no bound is strictly smaller (Table 1 leaves that cell empty)
    an = oracle.kernel_analysis(X, t, c, 1.0, 8, want_xrk=False)
    assert an["n_bound_smaller"] == 0


def test_indicators_on_outlier_inputs_follow_the_paper():
    """On outlier-channel inputs case II (c_j >= t_i) is rare (about 3 % in Table 1)."""
    X = workloads.config_activation("C1")
    t, c = oracle.absmax(X)
    an = oracle.kernel_analysis(X, t, c, 0.15, 8, want_xrk=False)
    assert an["n_col_ge_row"] / X.size < 0.05
    assert an["n_bound_smaller"] / X.size > 0.95


# ----------------------------------------------------------------------------- group-wise weights
@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("group", [8, 32, 96])
def test_grouped_weight_quantize(bits, group):
    qm = 2 ** (bits - 1) - 1
    I, O = 96, 20
    W = workloads.weight(I, O, seed=9)
    W[8:16, 5] = 0                                       # one all-zero group
    fold = np.random.default_rng(4).uniform(0.5, 3.0, I).astype(np.float32)
    for f in (None, fold):
        qw, s, wdq = oracle.weight_quantize_grouped(W, f, group, bits)
        Wf = W.astype(np.float32) if f is None else f[:, None] * W.astype(np.float32)
        G = Wf.reshape(I // group, group, O)             # [group index][j in group][k]
        m = np.abs(G).max(axis=1)                        # [I/g][O]
        want_s = (m / np.float32(qm)).T                  # [O][I/g]
        assert np.array_equal(s, want_s)
        step = np.repeat(want_s.T, group, axis=0)        # [I][O]
        with np.errstate(divide="ignore", invalid="ignore"):
            q = np.where(step == 0, 0, np.rint(Wf / step)).astype(np.int8)
        assert np.array_equal(qw, q.T)
        assert np.array_equal(wdq.view(np.uint16), (q.astype(np.float32) * step).astype(np.float16).view(np.uint16))
        # every group's largest weight sits on +-q_max; the reconstruction error is at most half a step
        nz = want_s.T > 0
        assert np.all(np.abs(q.reshape(I // group, group, O)).max(axis=1)[nz] == qm)
        assert np.all(np.abs(wdq.astype(np.float64) - Wf) <= 0.5 * step * (1 + 1e-6) + 1e-3 * np.abs(Wf) + 1e-9)
    if group == 96:                                       # one group per channel = Eq. 2 per-channel
        qw_pc, s_pc = oracle.weight_quantize(W, None, bits)
        qw, s, _ = oracle.weight_quantize_grouped(W, None, 96, bits, want_dq=False)
        assert np.array_equal(qw, qw_pc) and np.array_equal(s[:, 0], s_pc)


def test_weight_crossquant_is_the_activation_routine_on_the_stored_weight():
    """CrossQuant on weights (Appendix B.1, alpha_W): the same equation applied to the weight
    matrix stored output-channel-major; alpha_W = 1 is per-channel quantization (Eq. 2)."""
    W = workloads.weight(40, 24, seed=2)
    Wt = np.ascontiguousarray(W.T)                       # [O][I], one row per output channel
    t, c = oracle.absmax(Wt)
    r = oracle.quantize(Wt, t, c, 1.0, 8)
    qw_pc, s_pc = oracle.weight_quantize(W, None, 8)
    assert np.array_equal(r["codes"], qw_pc) and np.array_equal(r["a"], s_pc)
    r0 = oracle.quantize(Wt, t, c, 0.0, 8)               # alpha_W = 0: one step per input channel
    im = np.abs(Wt.astype(np.float32)).argmax(axis=0)
    assert np.array_equal(np.abs(r0["codes"][im, np.arange(40)]), np.full(40, 127))


def test_batched_tensor_has_per_sequence_column_maxima():
    """[B][S][I] input (the appendix listing's dims: row maximum over the last axis, column
    maximum over the second to last): every sequence is its own S x I problem."""
    B, S, I = 3, 20, 48
    X3 = np.stack([workloads.activation(S, I, n_outlier=2, scale_lo=30 * (b + 1), scale_hi=30 * (b + 1), seed=40 + b)
                   for b in range(B)])
    t, c = oracle.absmax_batched(X3)
    A = np.abs(X3.astype(np.float32))
    assert np.array_equal(t, A.max(axis=2)) and np.array_equal(c, A.max(axis=1))
    r = oracle.quantize_batched(X3, t, c, 0.15, 8)
    assert r["codes"].shape == (B, S, I) and r["a"].shape == (B, S) and r["b"].shape == (B, I)
    # B = 1 is the plain 2-D routine
    r1 = oracle.quantize_batched(X3[:1], t[:1], c[:1], 0.15, 8)
    r2 = oracle.quantize(X3[0], t[0], c[0], 0.15, 8)
    assert np.array_equal(r1["codes"][0], r2["codes"]) and r1["Z"] == r2["Z"]
    # sequences do not influence each other ...
    Y3 = X3.copy()
    Y3[1] *= np.float16(0.5)
    ty, cy = oracle.absmax_batched(Y3)
    ry = oracle.quantize_batched(Y3, ty, cy, 0.15, 8)
    assert np.array_equal(ry["codes"][0], r["codes"][0]) and np.array_equal(ry["codes"][2], r["codes"][2])
    # ... (halving a sequence halves its steps: same codes) ...
    assert np.array_equal(ry["codes"][1], r["codes"][1])
    # ... unlike the flattened [B*S][I] reading, whose shared column maxima couple them
    Xf = X3.reshape(B * S, I)
    tf, cf = oracle.absmax(Xf)
    rf = oracle.quantize(Xf, tf, cf, 0.15, 8)
    assert np.array_equal(cf, c.max(axis=0))
    assert not np.array_equal(rf["codes"].reshape(B, S, I)[0], r["codes"][0])
    assert r["Z"] == sum(int((r["codes"][b] == 0).sum()) for b in range(B))
