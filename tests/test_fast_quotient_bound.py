"""The error bound the quantize kernel's fast quotient relies on, checked on the CPU.

The kernel replaces fl32(x / fl32(a * b)) by x * (ra * rb) with ra, rb reciprocals accurate to
1 ulp, and falls back to the exact division whenever |frac| + (|q| + 1) * 2^-19 >= 1/2.  That is sound
if the approximation stays within 2^-19 (relative) of the correctly rounded quotient; the
analysis gives 2^-20 (two reciprocals at up to 1.5 * 2^-23 each as modelled here, three roundings
at 2^-24, and the quotient's own).  Here the bound is measured with numpy binary32 arithmetic, with
the correctly rounded reciprocals perturbed by +-1 ulp in every combination (the hardware
reciprocal is within 1 ulp of the true value; its exact rounding is not specified).

This file MODELS the kernel's shortcut in numpy; it does not run the kernel, and the 1-ulp
reciprocal is an assumption about the hardware, not something measured here.  It says that the
margin is wide enough if that assumption holds.  What pins the shortcut on the device is the GPU
parity suite: `test_quotients_just_off_a_rounding_tie` (quotients 2^-24 ... 2^-10 away from a tie,
every one compared with the oracle's division) and the exact-tie cases of
`test_quantize_rounding_ties` in tests/test_gpu_parity.py."""
from __future__ import annotations

import numpy as np


def ulp_shift(v: np.ndarray, k: int) -> np.ndarray:
    return (v.view(np.int32) + np.int32(k)).view(np.float32)


def test_fast_quotient_stays_within_the_fallback_margin():
    rng = np.random.default_rng(123)
    n = 400_000
    # x: binary16 values; a, b: positive binary32 scale factors over many magnitudes
    x = rng.standard_normal(n).astype(np.float16).astype(np.float32) * np.float32(8.0)
    a = np.exp(rng.uniform(-12, 4, n)).astype(np.float32)
    b = np.exp(rng.uniform(-6, 6, n)).astype(np.float32)
    D = (a * b).astype(np.float32)
    exact = (x.astype(np.float64) / D.astype(np.float64))          # the real quotient by fl32(a*b)
    rounded = (x / D).astype(np.float32).astype(np.float64)        # what the oracle rounds
    ra0 = (np.float32(1.0) / a).astype(np.float32)
    rb0 = (np.float32(1.0) / b).astype(np.float32)
    worst = 0.0
    for da in (-1, 0, 1):
        for db in (-1, 0, 1):
            ra, rb = ulp_shift(ra0, da), ulp_shift(rb0, db)
            approx = (x * (ra * rb).astype(np.float32)).astype(np.float32).astype(np.float64)
            nz = exact != 0
            rel = np.abs(approx[nz] - rounded[nz]) / np.abs(exact[nz])
            worst = max(worst, float(rel.max()))
    assert worst <= 2.0 ** -20, worst            # the analysed bound (measured: 2^-20.97)
    assert worst <= 2.0 ** -19 / 2               # at most half of the kernel's fallback margin


def test_rounding_can_only_differ_near_a_tie():
    """The kernel rounds the approximate quotient p = x * (ra * rb) straight to an integer q (one
    fma against 1.5 * 2^23), forms p - q with a second fma and falls back to the exact division when
    |p - q| + (|q| + 1) * 2^-19 >= 1/2.  If |p - exact| <= 2^-20 * |exact| (the bound above) then
    q != rne(exact) implies that the test fires: brute force on quotients around every tie,
    including the first one, where q may be 0."""
    ks = np.arange(0, 127, dtype=np.float64) + 0.5
    tol = 2.0 ** -19
    for eps in (2.0 ** -20, -(2.0 ** -20), 2.0 ** -22, -(2.0 ** -22)):
        for off in np.linspace(-3e-5, 3e-5, 241):
            exact = ks * (1 + off)
            p = exact * (1 + eps)                              # the product inside the fma is exact
            q = np.rint(p)
            differs = q != np.rint(exact)
            f = (p - q).astype(np.float32).astype(np.float64)  # the second fma rounds once
            fires = np.abs(f) + np.abs(q) * tol >= 0.5 - tol
            assert not np.any(differs & ~fires)


def test_count_only_sign_test_agrees_with_the_exact_code_unless_flagged():
    """The count-only kernel decides "code == 0" from the sign of d = fma(|x|, rb, -a/2) and takes
    the exact division whenever |d| <= (a/2) * 2^-19.  Model of that test in numpy (the fma is
    formed exactly in binary64 and rounded once), with the reciprocal perturbed by +-1 ulp, on
    inputs steered towards the boundary quotient 1/2: wherever the flag is not raised the sign
    test must agree with rne(fl32(x / fl32(a b))) == 0."""
    rng = np.random.default_rng(321)
    n = 300_000
    a = np.exp(rng.uniform(-10, 3, n)).astype(np.float32)
    b = np.exp(rng.uniform(-5, 5, n)).astype(np.float32)
    D = (a * b).astype(np.float32)
    # |x| / D close to 1/2: relative offsets from 2^-26 to 2^-12 on either side, and exact halves
    off = np.exp(rng.uniform(np.log(2.0 ** -26), np.log(2.0 ** -12), n)) * rng.choice([-1.0, 1.0], n)
    off[: n // 20] = 0.0
    x = (0.5 * D.astype(np.float64) * (1.0 + off)).astype(np.float32)      # binary32 stands in for the data grid
    q_exact = np.rint((x / D).astype(np.float32).astype(np.float64))        # rint: ties to even, as the kernel
    is_zero = q_exact == 0
    rb0 = (np.float32(1.0) / b).astype(np.float32)
    ha = (np.float32(0.5) * a).astype(np.float32)
    tol = (ha * np.float32(2.0 ** -19)).astype(np.float32)
    flagged_total = 0
    for db in (-1, 0, 1):
        rb = ulp_shift(rb0, db)
        d = (np.abs(x).astype(np.float64) * rb.astype(np.float64) - ha.astype(np.float64)).astype(np.float32)
        flagged = np.abs(d) <= tol
        says_zero = ~(d > 0)
        wrong = (says_zero != is_zero) & ~flagged
        assert not wrong.any(), (int(wrong.sum()), db)
        flagged_total += int(flagged.sum())
    # the flag is a narrow band, not a catch-all: offsets beyond 2^-17 never raise it
    far = np.abs(off) > 2.0 ** -17
    d = (np.abs(x).astype(np.float64) * rb0.astype(np.float64) - ha.astype(np.float64)).astype(np.float32)
    assert not (np.abs(d[far]) <= tol[far]).any()
    assert flagged_total > 0
