"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer, byte and index results (maxima, scale factors, codes, packed nibbles, zero
counts, int32 accumulators) must be bit-exact; binary16 outputs are produced with the same
operation order and are also compared bit for bit (the stated tolerance, max relative error
1e-3, is asserted as well and is far looser)."""
from __future__ import annotations

import sys

import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cq():
    import torch
    assert torch.cuda.is_available()
    import paper_2410_07505_amd as pkg
    return pkg


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def gpu(arr):
    import torch
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def bits16(a):
    return np.ascontiguousarray(a).view(np.uint16)


def bits32(a):
    return np.ascontiguousarray(a).view(np.uint32)


def outliers(T, I, seed, n_out=3, scale=60.0, dist="normal"):
    return workloads.activation(T, I, dist=dist, n_outlier=min(n_out, I), scale_lo=scale, scale_hi=scale,
                                seed=seed)


# ----------------------------------------------------------------------------- absmax
ABSMAX_SHAPES = [(1, 1), (1, 8), (3, 5), (37, 53), (64, 256), (130, 1000), (129, 512), (257, 1537), (1000, 24)]


@pytest.mark.parametrize("T,I", ABSMAX_SHAPES)
def test_absmax_small_and_ragged(cq, T, I):
    say("absmax T=%d I=%d" % (T, I))
    X = outliers(T, I, seed=T * 1000 + I)
    t_ref, c_ref = oracle.absmax(X)
    t, c = cq.crossquant_absmax(gpu(X))
    assert np.array_equal(bits32(host(t)), bits32(t_ref))
    assert np.array_equal(bits32(host(c)), bits32(c_ref))


def test_absmax_strided_and_misaligned_views(cq):
    say("absmax strided / misaligned")
    base = outliers(70, 200, seed=5)
    g = gpu(base)
    for lo, hi in ((0, 96), (8, 136), (1, 130), (3, 200)):       # the last two start off 16-byte alignment
        view = g[:, lo:hi]
        t, c = cq.crossquant_absmax(view)
        t_ref, c_ref = oracle.absmax(base[:, lo:hi])
        assert np.array_equal(host(t), t_ref) and np.array_equal(host(c), c_ref), (lo, hi)


def test_absmax_overwrites_stale_outputs_and_handles_zeros(cq):
    import torch
    say("absmax stale outputs")
    X = np.zeros((40, 72), np.float16)
    X[7, 9] = -3.0
    t = torch.full((40,), 99.0, device="cuda")
    c = torch.full((72,), 99.0, device="cuda")
    cq.crossquant_absmax(gpu(X), t=t, c=c)
    t_ref, c_ref = oracle.absmax(X)
    assert np.array_equal(host(t), t_ref) and np.array_equal(host(c), c_ref)


def test_absmax_calls_in_a_row_clear_for_themselves(cq):
    """The vector-layout call clears t and c inside its one launch (the launch's first blocks store the zeros, the
    others wait for them before their atomics).  Many calls in a row on one stream, into the same output vectors,
    with data whose maxima shrink from call to call: a maximum left over from an earlier call would survive."""
    import torch
    say("absmax: 40 calls in a row, shrinking maxima, two shapes alternating")
    rng = np.random.default_rng(5)
    shapes = [(300, 1536), (64, 520 * 8)]
    t_buf = {s_: torch.empty(s_[0], dtype=torch.float32, device="cuda") for s_ in shapes}
    c_buf = {s_: torch.empty(s_[1], dtype=torch.float32, device="cuda") for s_ in shapes}
    pending = []
    for it in range(40):
        T, I = shapes[it % 2]
        X = (rng.standard_normal((T, I)) * (100.0 / (it + 1))).astype(np.float16)
        Xg = gpu(X)
        cq.crossquant_absmax(Xg, t=t_buf[(T, I)], c=c_buf[(T, I)])
        pending.append((X, t_buf[(T, I)].clone(), c_buf[(T, I)].clone()))      # clones are ordered on the stream
    torch.cuda.synchronize()
    for X, t, c in pending:
        t_ref, c_ref = oracle.absmax(X)
        assert np.array_equal(bits32(host(t)), bits32(t_ref)) and np.array_equal(bits32(host(c)), bits32(c_ref))


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_absmax_full_configs(cq, name):
    say("absmax config %s" % name)
    X = workloads.config_activation(name)
    t_ref, c_ref = oracle.absmax(X)
    t, c = cq.crossquant_absmax(gpu(X))
    assert np.array_equal(bits32(host(t)), bits32(t_ref))
    assert np.array_equal(bits32(host(c)), bits32(c_ref))


# ----------------------------------------------------------------------------- scale factors
@pytest.mark.parametrize("alpha", [0.0, 0.15, 0.45, 0.5, 0.75, 1.0])
@pytest.mark.parametrize("bits", [8, 4])
def test_scale_factors_for_every_binary16_maximum(cq, alpha, bits):
    """t and c are maxima of binary16 values, so there are only 31744 possible positive finite
    inputs (plus zero): check the device's scale factors for all of them."""
    import torch
    say("scale factors alpha=%g bits=%d" % (alpha, bits))
    vals = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)   # 0 .. 65504
    n = vals.size
    a_ref, _ = oracle.scales(vals, vals[:8], alpha, bits)
    _, b_ref = oracle.scales(vals[:8], vals, alpha, bits)
    # rows: T = n, I = 8
    X = torch.zeros((n, 8), dtype=torch.float16, device="cuda")
    t = gpu(vals)
    c = gpu(vals[:8].copy())
    _, _, a, _, _ = cq.crossquant_quantize(X, t, c, alpha, bits, want_xhat=False)
    bad_a = int((bits32(host(a)) != bits32(a_ref)).sum())
    # columns: T = 8, I = n
    X2 = torch.zeros((8, n), dtype=torch.float16, device="cuda")
    _, _, _, b, _ = cq.crossquant_quantize(X2, c, t, alpha, bits, want_xhat=False)
    bad_b = int((bits32(host(b)) != bits32(b_ref)).sum())
    assert bad_a == 0 and bad_b == 0, (bad_a, bad_b)


# ----------------------------------------------------------------------------- quantize
def check_quantize(cq, X, alpha, bits, Xg=None, label=""):
    say("quantize %s shape=%s alpha=%g bits=%d" % (label, X.shape, alpha, bits))
    Xg = gpu(X) if Xg is None else Xg
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, alpha, bits)
    t, c = cq.crossquant_absmax(Xg)
    codes, xhat, a, b, zc = cq.crossquant_quantize(Xg, t, c, alpha, bits)
    # scale factors first: a mismatch here would be a pow() disagreement, not a kernel bug
    assert np.array_equal(bits32(host(a)), bits32(ref["a"])), "row scale factors differ"
    assert np.array_equal(bits32(host(b)), bits32(ref["b"])), "column scale factors differ"
    got = host(codes)
    assert got.shape == ref["codes"].shape and got.dtype == ref["codes"].dtype
    neq = got != ref["codes"]
    assert not neq.any(), "%d codes differ, first at %s" % (neq.sum(), np.argwhere(neq)[:4].tolist())
    assert int(host(zc)[0]) == ref["Z"]
    xh = host(xhat)
    assert np.array_equal(bits16(xh), bits16(ref["xhat"]))
    # the stated floating-point bar (implied by bit equality, kept explicit)
    r64, g64 = ref["xhat"].astype(np.float64), xh.astype(np.float64)
    assert np.all(np.abs(g64 - r64) <= 1e-3 * np.abs(r64))
    assert ref["clamp_hits"] == 0
    # codes-only and count-only variants give the same codes / count
    codes2, none_xhat, _, _, zc2 = cq.crossquant_quantize(Xg, t, c, alpha, bits, want_xhat=False)
    assert none_xhat is None and np.array_equal(host(codes2), ref["codes"]) and int(host(zc2)[0]) == ref["Z"]
    zc3 = cq.crossquant_kernel_count(Xg, t, c, alpha, bits)          # no work vectors (NULL, NULL)
    assert int(host(zc3)[0]) == ref["Z"] == oracle.kernel_count(X, t_ref, c_ref, alpha, bits)
    a4, b4 = a.clone().fill_(-1.0), b.clone().fill_(-1.0)            # with them: they receive the factors
    zc4 = cq.crossquant_kernel_count(Xg, t, c, alpha, bits, row_scale=a4, col_scale=b4)
    assert int(host(zc4)[0]) == ref["Z"]
    assert np.array_equal(bits32(host(a4)), bits32(ref["a"])) and np.array_equal(bits32(host(b4)), bits32(ref["b"]))
    return ref


QUANT_SHAPES = [(1, 2), (3, 6), (37, 54), (64, 256), (130, 1000), (129, 520), (200, 1538)]


@pytest.mark.parametrize("T,I", QUANT_SHAPES)
@pytest.mark.parametrize("bits", [8, 4])
def test_quantize_small_and_ragged(cq, T, I, bits):
    X = outliers(T, I, seed=T + I)
    for alpha in (0.15, 1.0):
        check_quantize(cq, X, alpha, bits)


def test_quantize_odd_channel_count_int8(cq):
    X = outliers(33, 77, seed=12)
    check_quantize(cq, X, 0.15, 8)


@pytest.mark.parametrize("alpha", [0.0, 0.15, 0.5, 1.0])
def test_quantize_tiny_config_all_alphas(cq, alpha):
    X = workloads.config_activation("C1")
    for bits in (8, 4):
        check_quantize(cq, X, alpha, bits, label="C1")


def test_quantize_strided_and_misaligned_input(cq):
    base = outliers(50, 300, seed=77)
    g = gpu(base)
    for lo, hi in ((8, 264), (1, 257), (5, 299)):
        view = base[:, lo:hi]
        check_quantize(cq, view, 0.15, 8, Xg=g[:, lo:hi], label="view[%d:%d]" % (lo, hi))


def test_quantize_zero_rows_columns_and_all_zero_matrix(cq):
    X = outliers(40, 96, seed=3)
    X[5, :] = 0
    X[:, 17] = 0
    X[9, 4] = np.float16(-0.0)
    for alpha in (0.0, 0.15, 1.0):
        ref = check_quantize(cq, X, alpha, 8, label="zero row/col")
        assert np.all(ref["codes"][5] == 0) and np.all(ref["codes"][:, 17] == 0)
    Z = np.zeros((20, 64), np.float16)
    ref = check_quantize(cq, Z, 0.15, 8, label="all zero")
    assert ref["Z"] == Z.size


def test_quantize_rounding_ties(cq):
    """Quotients that sit exactly on k + 1/2 (steps that are powers of two): the fast quotient
    must hand these to the exact division, and half-to-even must decide them."""
    rng = np.random.default_rng(5)
    T, I = 96, 512
    X = (rng.integers(-250, 251, (T, I)) / 2.0).astype(np.float16)        # multiples of 1/2
    X[:, 0] = 127.0                                                        # t_i = 127 -> step 1 at alpha = 1
    X[::2, 0] = -127.0
    check_quantize(cq, X, 1.0, 8, label="ties alpha=1")
    X4 = (rng.integers(-13, 14, (T, I)) / 2.0).astype(np.float16)
    X4[0, :] = 7.0                                                         # c_j = 7 -> step ~1 at alpha = 0
    check_quantize(cq, X4, 0.0, 4, label="ties alpha=0 int4")
    check_quantize(cq, X4, 0.0, 8, label="ties alpha=0 int8")


def test_quotients_just_off_a_rounding_tie(cq):
    """Calibrated maxima chosen so that every element of row i has the quotient (k_i + 1/2)(1 + d_i)
    with |d_i| from 2^-24 to 2^-10 on either side: the band in which the fast quotient (and the
    count-only sign test, for k = 0) must either be right or hand over to the exact division."""
    import torch
    ks = np.array([0, 0, 1, 2, 5, 31, 63, 100, 126], dtype=np.float64)
    ds = np.concatenate([[0.0], 2.0 ** -np.arange(10, 25), -(2.0 ** -np.arange(10, 25))])
    rows = [(k, d) for k in ks for d in ds]
    T, I = len(rows), 72
    rng = np.random.default_rng(11)
    X = np.full((T, I), 3.0, np.float16)
    X[:, ::3] = -3.0
    X[:, 5] = rng.standard_normal(T).astype(np.float16)                  # some ordinary elements too
    t_cal = np.array([127.0 * 3.0 / ((k + 0.5) * (1.0 + d)) for k, d in rows]).astype(np.float32)
    c_cal = np.full(I, 3.0, np.float32)
    Xg = gpu(X)
    for alpha, tt, cc in ((1.0, t_cal, c_cal), (0.5, t_cal, (c_cal * c_cal / t_cal.mean()).astype(np.float32))):
        ref = oracle.quantize(X, tt, cc, alpha, 8)
        say("near ties alpha=%g: %d distinct codes in the reference" % (alpha, len(np.unique(ref["codes"]))))
        codes, xhat, _, _, zc = cq.crossquant_quantize(Xg, gpu(tt), gpu(cc), alpha, 8)
        neq = host(codes) != ref["codes"]
        assert not neq.any(), (alpha, int(neq.sum()), np.argwhere(neq)[:4].tolist())
        assert np.array_equal(bits16(host(xhat)), bits16(ref["xhat"])) and int(host(zc)[0]) == ref["Z"]
        zc2 = cq.crossquant_kernel_count(Xg, gpu(tt), gpu(cc), alpha, 8)
        assert int(host(zc2)[0]) == ref["Z"] == oracle.kernel_count(X, tt, cc, alpha, 8)


def test_quantize_subnormal_binary16_data(cq):
    """Every element a subnormal binary16 value (multiples of 2^-24 below 2^-14), and a mix of subnormal
    and ordinary rows: conversions, reciprocals and the mixed-precision fmas must treat them exactly."""
    rng = np.random.default_rng(17)
    sub = (rng.integers(-1023, 1024, (70, 600)).astype(np.float64) * 2.0 ** -24).astype(np.float16)
    assert np.all(np.abs(sub.astype(np.float64)) < 2.0 ** -14)
    for alpha in (0.0, 0.15, 1.0):
        check_quantize(cq, sub, alpha, 8, label="subnormal")
    mixed = sub.copy()
    mixed[::3] = outliers(24, 600, seed=18)
    check_quantize(cq, mixed, 0.15, 8, label="subnormal + ordinary rows")
    check_quantize(cq, mixed, 0.5, 4, label="subnormal + ordinary rows")
    check_analysis(cq, mixed, 0.15, 8, label="subnormal + ordinary rows")


def test_quantize_golden_cases(cq):
    from test_oracle_pins import read_golden
    for case in read_golden():
        X = case["X"]
        Xg = gpu(X)
        t, c = cq.crossquant_absmax(Xg)
        codes, _, _, _, zc = cq.crossquant_quantize(Xg, t, c, case["alpha"], case["bits"])
        got = host(codes)
        if case["bits"] == 4:
            assert np.array_equal(got, case["packed"])
            got = oracle.unpack_int4(got)
        assert np.array_equal(got, case["codes"]) and int(host(zc)[0]) == case["Z"]


def test_quantize_with_calibrated_maxima_clamps(cq):
    """t and c smaller than the data's maxima (e.g. calibrated elsewhere): codes saturate at
    +-q_max exactly as in the oracle."""
    X = outliers(48, 128, seed=9)
    t_ref, c_ref = oracle.absmax(X)
    t_small = (t_ref * 0.25).astype(np.float32)
    c_small = (c_ref * 0.5).astype(np.float32)
    for bits in (8, 4):
        ref = oracle.quantize(X, t_small, c_small, 0.15, bits)
        assert ref["clamp_hits"] > 0
        codes, xhat, _, _, zc = cq.crossquant_quantize(gpu(X), gpu(t_small), gpu(c_small), 0.15, bits)
        assert np.array_equal(host(codes), ref["codes"])
        assert np.array_equal(bits16(host(xhat)), bits16(ref["xhat"])) and int(host(zc)[0]) == ref["Z"]
        zc2 = cq.crossquant_kernel_count(gpu(X), gpu(t_small), gpu(c_small), 0.15, bits)
        assert int(host(zc2)[0]) == ref["Z"]
    # a zero maximum handed in for non-zero data: the step is 0 and every code of that row / column is 0
    t0, c0 = t_ref.copy(), c_ref.copy()
    t0[3] = 0.0
    c0[5] = 0.0
    ref = oracle.quantize(X, t0, c0, 0.15, 8)
    assert np.all(ref["codes"][3] == 0) and np.all(ref["codes"][:, 5] == 0)
    codes, _, _, _, zc = cq.crossquant_quantize(gpu(X), gpu(t0), gpu(c0), 0.15, 8)
    zc2 = cq.crossquant_kernel_count(gpu(X), gpu(t0), gpu(c0), 0.15, 8)
    assert np.array_equal(host(codes), ref["codes"]) and int(host(zc)[0]) == ref["Z"] == int(host(zc2)[0])


def test_quantize_with_absurdly_small_calibrated_maxima(cq):
    """Maxima so small that a * b underflows (to a subnormal, or to zero: then every code is 0 by
    definition) or 1/a * 1/b overflows: the quotient shortcut must hand these to the exact division."""
    X = outliers(24, 64, seed=19)
    for tv, cv, alpha in ((1e-30, 1e-30, 0.5), (1e-42, 1e-42, 0.5), (3e-39, 2e-38, 0.15), (1e-44, 1.0, 0.5), (1e-44, 1e-44, 0.5),
                          (1.0, 1e-44, 0.15), (1e-20, 1e-36, 0.5)):
        t = np.full(24, tv, np.float32)
        c = np.full(64, cv, np.float32)
        for bits in (8, 4):
            ref = oracle.quantize(X, t, c, alpha, bits)
            codes, xhat, a, b, zc = cq.crossquant_quantize(gpu(X), gpu(t), gpu(c), alpha, bits)
            assert np.array_equal(bits32(host(a)), bits32(ref["a"])) and np.array_equal(bits32(host(b)), bits32(ref["b"]))
            assert np.array_equal(host(codes), ref["codes"]), (tv, cv, alpha, bits)
            assert int(host(zc)[0]) == ref["Z"]
            assert np.array_equal(bits16(host(xhat)), bits16(ref["xhat"]))
            zc2 = cq.crossquant_kernel_count(gpu(X), gpu(t), gpu(c), alpha, bits)
            assert int(host(zc2)[0]) == ref["Z"]


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5"])
def test_quantize_full_configs(cq, name):
    cfg = workloads.CONFIGS[name]
    X = workloads.config_activation(name)
    Xg = gpu(X)
    z = {}
    for alpha in cfg.alphas + ((1.0,) if 1.0 not in cfg.alphas else ()):
        ref = check_quantize(cq, X, alpha, cfg.bits, Xg=Xg, label=name)
        z[alpha] = ref["Z"]
    # direction of the paper's kernel-proportion result on outlier-channel inputs
    assert z[0.15] < z[1.0]
    say("%s kernel proportion: %s" % (name, {k: round(v / X.size, 4) for k, v in z.items()}))


def test_quantize_is_deterministic(cq):
    X = workloads.config_activation("C2")
    Xg = gpu(X)
    t, c = cq.crossquant_absmax(Xg)
    r1 = cq.crossquant_quantize(Xg, t, c, 0.15, 8)
    r2 = cq.crossquant_quantize(Xg, t, c, 0.15, 8)
    import torch
    assert torch.equal(r1[0], r2[0]) and torch.equal(r1[1], r2[1]) and torch.equal(r1[4], r2[4])


@pytest.mark.parametrize("T,I", [(3, 70000), (60000, 8), (5, 65536), (20000, 24), (2, 131080)])
def test_extreme_aspect_ratios(cq, T, I):
    """Very wide and very tall matrices: many column chunks with few rows, and many row chunks
    with one partly filled column chunk."""
    X = outliers(T, I, seed=T % 97 + I % 89)
    check_quantize(cq, X, 0.15, 8, label="aspect")
    check_quantize(cq, X, 0.5, 4, label="aspect")
    check_analysis(cq, X, 0.15, 8, label="aspect")


@pytest.mark.parametrize("T,I", [(4010, 8200), (6010, 8200), (2500, 16390)])
def test_row_counts_per_block_that_are_not_powers_of_two(cq, T, I):
    """The launchers pick the rows per block from the block count: these shapes give 5, 7 and 6 batches per
    wave (the layer-shaped configurations give 2, 3 and 4), each with a partly filled last row chunk and a
    column chunk of 8 columns."""
    X = outliers(T, I, seed=T % 89 + I % 97)
    check_quantize(cq, X, 0.15, 8, label="rows per block")
    check_analysis(cq, X, 0.15, 8, label="rows per block")


@pytest.mark.parametrize("T,I", [(270000, 8), (4, 262200)])
def test_very_long_maxima_vectors(cq, T, I):
    """More than 2^18 rows, or columns: thousands of row chunks / column chunks in one launch."""
    X = outliers(T, I, seed=3 + T % 11)
    check_quantize(cq, X, 0.15, 8, label="long vectors")


def test_calls_overlapping_on_many_streams(cq):
    """Calls on different streams may run at the same time; each stream has its own word of the
    library-owned zero-count accumulators (more streams than words: the rest clear the caller's
    counter with a kernel first).  Everything is enqueued first, then checked."""
    import torch
    say("20 streams, absmax + quantize + count enqueued without waiting")
    n = 20
    streams = [torch.cuda.Stream() for _ in range(n)]
    Xs = [outliers(200 + 37 * k, 600 + 130 * k, seed=700 + k) for k in range(n)]
    Xg = [gpu(X) for X in Xs]
    torch.cuda.synchronize()
    out = []
    for rep in range(2):                      # second round: every stream reuses its piece
        for k, st in enumerate(streams):
            with torch.cuda.stream(st):
                t, c = cq.crossquant_absmax(Xg[k])
                res = cq.crossquant_quantize(Xg[k], t, c, 0.15, 8)
                zc = cq.crossquant_kernel_count(Xg[k], t, c, 1.0, 8)
            if rep == 1:
                out.append((t, c, res, zc))
    torch.cuda.synchronize()
    for k in range(n):
        t_ref, c_ref = oracle.absmax(Xs[k])
        ref = oracle.quantize(Xs[k], t_ref, c_ref, 0.15, 8)
        t, c, (codes, xhat, a, b, z), zc = out[k]
        assert np.array_equal(bits32(host(t)), bits32(t_ref)) and np.array_equal(bits32(host(c)), bits32(c_ref)), k
        assert np.array_equal(host(codes), ref["codes"]) and int(host(z)[0]) == ref["Z"], k
        assert np.array_equal(bits16(host(xhat)), bits16(ref["xhat"])), k
        assert int(host(zc)[0]) == oracle.kernel_count(Xs[k], t_ref, c_ref, 1.0, 8), k


def test_more_than_2_to_31_elements(cq):
    """70 000 x 65 544 = 4.59e9 elements (9.2 GB of binary16): every element offset past row 32 767
    needs more than 32 bits.  The oracle computes the maxima of the whole matrix; codes and
    dequantized values are checked on sampled rows from the beginning, the middle and the very end;
    the zero count against the zero codes of the whole output."""
    import torch
    T, I = 70000, 65544
    say("quantizer on %d x %d (%.1f GB)" % (T, I, T * I * 2 / 1e9))
    gen = torch.Generator(device="cuda").manual_seed(4591)
    Xg = torch.empty((T, I), dtype=torch.float16, device="cuda")
    for r0 in range(0, T, 5000):                                   # in slabs: no large temporary
        Xg[r0:r0 + 5000].normal_(generator=gen)
    Xg[:, 1000::9973] *= 60.0                                      # a few outlier channels
    X = host(Xg)
    t_ref, c_ref = oracle.absmax(X)
    t, c = cq.crossquant_absmax(Xg)
    assert np.array_equal(bits32(host(t)), bits32(t_ref)) and np.array_equal(bits32(host(c)), bits32(c_ref))
    codes, xhat, a, b, zc = cq.crossquant_quantize(Xg, t, c, 0.15, 8)
    zc2 = cq.crossquant_kernel_count(Xg, t, c, 0.15, 8)
    n_zero = sum(int((codes[r0:r0 + 5000] == 0).sum().item()) for r0 in range(0, T, 5000))
    assert int(host(zc)[0]) == n_zero == int(host(zc2)[0])
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([np.arange(40), np.arange(32760, 32776), np.arange(T - 40, T), rng.integers(0, T, 60)]))
    ref = oracle.quantize(np.ascontiguousarray(X[rows]), t_ref[rows], c_ref, 0.15, 8)
    ri = torch.from_numpy(rows).cuda()
    assert np.array_equal(bits32(host(a[ri])), bits32(ref["a"])) and np.array_equal(bits32(host(b)), bits32(ref["b"]))
    assert np.array_equal(host(codes[ri]), ref["codes"])
    assert np.array_equal(bits16(host(xhat[ri])), bits16(ref["xhat"]))
    del codes
    # the analysis call on the same matrix: the kept elements on the sampled rows against the oracle, the
    # kernel size against the count above, the two indicators against their definitions evaluated with
    # library routines on the device (same binary32 operations)
    xrk, counters = cq.crossquant_kernel_analysis(Xg, t, c, 0.15, 8, xrk=xhat)
    ref_a = oracle.kernel_analysis(np.ascontiguousarray(X[rows]), t_ref[rows], c_ref, 0.15, 8)
    assert np.array_equal(bits16(host(xrk[ri])), bits16(ref_a["xrk"]))
    got = [int(v) for v in host(counters)]
    assert got[0] == n_zero
    c_sorted = torch.sort(c).values
    assert got[1] == int((I - torch.searchsorted(c_sorted, t.contiguous(), right=False)).sum().item())   # #{c_j >= t_i}
    pt = t / 127.0
    n_smaller = 0
    for r0 in range(0, T, 2000):
        n_smaller += int(((a[r0:r0 + 2000, None] * b[None, :]) < pt[r0:r0 + 2000, None]).sum().item())
    assert got[2] == n_smaller


def test_batched_tensor_with_more_than_2_to_31_elements(cq):
    """64 sequences of 8192 x 8200 (4.3e9 elements): sequence offsets past 2^31.  The first, one from the
    middle and the last sequence against the oracle; the zero count against the zero codes of the whole output."""
    import torch
    B, S, I = 64, 8192, 8200
    say("batched %d x %d x %d" % (B, S, I))
    gen = torch.Generator(device="cuda").manual_seed(77)
    Xg = torch.empty((B, S, I), dtype=torch.float16, device="cuda")
    for b0 in range(B):
        Xg[b0].normal_(generator=gen)
        Xg[b0, :, 17 * (b0 + 1)] *= 40.0 + b0                       # a different outlier channel per sequence
    t, c = cq.crossquant_absmax_batched(Xg)
    codes, xhat, a, b, zc = cq.crossquant_quantize_batched(Xg, t, c, 0.15, 8)
    n_zero = sum(int((codes.view(B, S, I)[b0] == 0).sum().item()) for b0 in range(B))
    assert int(host(zc)[0]) == n_zero
    for b0 in (0, 31, B - 1):
        Xs = host(Xg[b0])
        t_ref, c_ref = oracle.absmax(Xs)
        ref = oracle.quantize(Xs, t_ref, c_ref, 0.15, 8)
        assert np.array_equal(bits32(host(t.view(B, S)[b0])), bits32(t_ref)), b0
        assert np.array_equal(bits32(host(c.view(B, I)[b0])), bits32(c_ref)), b0
        assert np.array_equal(host(codes.view(B, S, I)[b0]), ref["codes"]), b0
        assert np.array_equal(bits16(host(xhat.view(B, S, I)[b0])), bits16(ref["xhat"])), b0


def test_weights_with_more_than_2_to_31_elements(cq):
    """8200 x 270 000 weights (2.2e9 elements): output-channel offsets past 2^31 in the transposed codes.
    Output channels are independent, so the oracle checks a sample of them (first, last, random)."""
    import torch
    I, O = 8200, 270000
    say("weights %d x %d" % (I, O))
    gen = torch.Generator(device="cuda").manual_seed(78)
    Wg = torch.empty((I, O), dtype=torch.float16, device="cuda")
    for j0 in range(0, I, 1025):
        Wg[j0:j0 + 1025].normal_(std=0.02, generator=gen)
    rng = np.random.default_rng(79)
    fold = rng.uniform(0.5, 4.0, I).astype(np.float32)
    qw, ws = cq.crossquant_weight_quantize(Wg, gpu(fold), 8)
    cols = np.unique(np.concatenate([np.arange(70), np.arange(O - 70, O), rng.integers(0, O, 120)]))
    ci = torch.from_numpy(cols).cuda()
    qw_ref, s_ref = oracle.weight_quantize(host(Wg[:, ci]), fold, 8)
    assert np.array_equal(bits32(host(ws[ci])), bits32(s_ref))
    assert np.array_equal(host(qw[ci]), qw_ref)
    # every channel's largest code is +-127 (the channel's own maximum), wherever it lies
    peak = qw.view(O, I).abs().amax(dim=1)
    assert bool((peak == 127).all())


def test_linear_output_with_more_than_2_to_31_elements(cq):
    """32 768 x 65 544 outputs (4.3 GB of binary16) from a short contraction: output offsets past
    2^31.  Sampled rows against the oracle; an integer checksum over every output against the exact
    value sum_k (sum_i qx_i) . qw_k computed on the host."""
    import torch
    T, I, O = 32768, 128, 65544
    say("linear %d x %d x %d" % (T, I, O))
    qx = workloads.int8_codes(T, I, seed=71)
    qw = workloads.int8_codes(O, I, seed=72)
    rng = np.random.default_rng(73)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y, acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), want_acc=True)
    rows = np.unique(np.concatenate([np.arange(8), np.arange(32760 // 2 - 4, 32760 // 2 + 4), np.arange(T - 8, T),
                                     rng.integers(0, T, 16)]))
    Y_ref, acc_ref = oracle.w8a8_linear(qx[rows], a[rows], qw, s)
    ri = torch.from_numpy(rows).cuda()
    assert np.array_equal(host(acc[ri]), acc_ref)
    assert np.array_equal(bits16(host(Y[ri])), bits16(Y_ref))
    total = int(acc.sum(dtype=torch.int64).item())
    expect = int(qx.astype(np.int64).sum(axis=0) @ qw.astype(np.int64).sum(axis=0))
    assert total == expect


def test_wide_leading_dimension(cq):
    """A narrow window of a very wide matrix: rows 64 KiB apart."""
    import torch
    base = outliers(40, 32768, seed=31)
    g = gpu(base)
    for lo, hi in ((1024, 1280), (8191, 8191 + 300)):
        check_quantize(cq, base[:, lo:hi], 0.15, 8, Xg=g[:, lo:hi], label="window[%d:%d]" % (lo, hi))


# ----------------------------------------------------------------------------- single-read fused call
def check_fused(cq, X, alpha, bits, Xg=None, label="", want_xhat=True, single_read=False):
    say("absmax_quantize%s %s shape=%s alpha=%g bits=%d xhat=%s" % ("_single_read" if single_read else "", label, X.shape,
                                                                  alpha, bits, want_xhat))
    import torch
    Xg = gpu(X) if Xg is None else Xg
    T, I = X.shape
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, alpha, bits)
    # stale contents everywhere: the call must overwrite all of it
    stale = dict(t=torch.full((T,), 7.0, device="cuda"), c=torch.full((I,), 9.0, device="cuda"),
                 zero_count=torch.full((1,), 12345, dtype=torch.int64, device="cuda"))
    t, c, codes, xhat, a, b, zc = cq.crossquant_absmax_quantize(Xg, alpha, bits, want_xhat=want_xhat,
                                                                single_read=single_read, **stale)
    assert np.array_equal(bits32(host(t)), bits32(t_ref)) and np.array_equal(bits32(host(c)), bits32(c_ref))
    assert np.array_equal(bits32(host(a)), bits32(ref["a"])), "row scale factors differ"
    assert np.array_equal(bits32(host(b)), bits32(ref["b"])), "column scale factors differ"
    got = host(codes)
    neq = got != ref["codes"]
    assert not neq.any(), "%d codes differ, first at %s" % (neq.sum(), np.argwhere(neq)[:4].tolist())
    assert int(host(zc)[0]) == ref["Z"]
    if want_xhat:
        xh = host(xhat)
        assert np.array_equal(bits16(xh), bits16(ref["xhat"]))
        r64, g64 = ref["xhat"].astype(np.float64), xh.astype(np.float64)
        assert np.all(np.abs(g64 - r64) <= 1e-3 * np.abs(r64))
    else:
        assert xhat is None
    return ref


FUSED_SHAPES = [(1, 8), (3, 16), (37, 56), (64, 256), (130, 1000), (129, 520), (257, 1544), (300, 2048), (1000, 4104)]


@pytest.mark.parametrize("T,I", FUSED_SHAPES)
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("single_read", [False, True])
def test_fused_small_and_ragged(cq, T, I, bits, single_read):
    X = outliers(T, I, seed=T + I)
    check_fused(cq, X, 0.15, bits, single_read=single_read)
    check_fused(cq, X, 1.0, bits, want_xhat=False, single_read=single_read)


@pytest.mark.parametrize("single_read", [False, True])
def test_fused_zero_rows_columns_ties_and_strided(cq, single_read):
    X = outliers(40, 96, seed=3)
    X[5, :] = 0
    X[:, 17] = 0
    for alpha in (0.0, 0.15, 1.0):
        check_fused(cq, X, alpha, 8, label="zero row/col", single_read=single_read)
    check_fused(cq, np.zeros((20, 64), np.float16), 0.15, 8, label="all zero", single_read=single_read)
    rng = np.random.default_rng(5)
    Xt = (rng.integers(-250, 251, (96, 512)) / 2.0).astype(np.float16)
    Xt[:, 0] = 127.0
    check_fused(cq, Xt, 1.0, 8, label="ties", single_read=single_read)
    base = outliers(50, 304, seed=77)
    g = gpu(base)
    check_fused(cq, base[:, 8:264], 0.15, 8, Xg=g[:, 8:264], label="view[8:264]", single_read=single_read)


def test_single_read_reports_unsupported_requests(cq):
    """Layouts the register-resident kernel does not take, and matrices that do not fit on the
    chip, come back as CQ_ERR_UNSUPPORTED with nothing enqueued; crossquant_absmax_quantize serves them."""
    import torch
    base = outliers(50, 304, seed=78)
    g = gpu(base)
    for view in (g[:, 1:257], g[:, 0:54]):                     # misaligned rows; I % 8 != 0
        with pytest.raises(cq.CrossQuantError) as e:
            cq.crossquant_absmax_quantize_single_read(view, 0.15, 8)
        assert e.value.status == -6
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    rows = 256 * (n_cu // 16) + 1                              # one row block too many at I = 8192
    big = torch.zeros((rows, 8192), dtype=torch.float16, device="cuda")
    with pytest.raises(cq.CrossQuantError) as e:
        cq.crossquant_absmax_quantize_single_read(big, 0.15, 8)
    assert e.value.status == -6
    torch.cuda.synchronize()


def test_single_read_barrier_gives_up_cleanly(cq):
    """The grid barrier's bounded wait, forced from the host: with a poll limit of 0 every block
    gives up at once, the kernel ends normally, flags the failure with NaN scale factors and
    writes no codes; with the default limit the same call is correct again."""
    import torch
    X = outliers(300, 1024, seed=55)
    Xg = gpu(X)
    codes = torch.full((300, 1024), 99, dtype=torch.int8, device="cuda")
    try:
        cq.raw.crossquant_debug_set_barrier_polls(0)
        _, _, codes_out, _, a, b, _ = cq.crossquant_absmax_quantize_single_read(Xg, 0.15, 8, codes=codes)
        torch.cuda.synchronize()
    finally:
        cq.raw.crossquant_debug_set_barrier_polls(1 << 22)
    assert bool(torch.isnan(a).all()) and bool(torch.isnan(b).all())
    assert bool((codes_out == 99).all())
    check_fused(cq, X, 0.15, 8, Xg=Xg, label="after the forced failure", single_read=True)


def test_fused_call_takes_every_layout_and_size(cq):
    """Misaligned rows, a channel count that is not a multiple of 8, a very tall matrix: the one call serves
    every layout and size the two calls serve."""
    import torch
    base = outliers(50, 304, seed=78)
    g = gpu(base)
    for lo, hi in ((1, 257), (0, 54)):                         # misaligned rows; I % 8 != 0
        check_fused(cq, base[:, lo:hi], 0.15, 8, Xg=g[:, lo:hi], label="view[%d:%d]" % (lo, hi))
    say("one call on 266 240 x 2048")
    T, I = 512 * 520, 2048
    rng = np.random.default_rng(9)
    X = np.zeros((T, I), dtype=np.float16)
    X[:, :64] = rng.standard_normal((T, 64)).astype(np.float16)
    X[::1000, 100] = 300.0
    check_fused(cq, X, 0.15, 8, label="tall", want_xhat=False)
    torch.cuda.synchronize()


def test_fused_call_many_times_and_on_many_streams(cq):
    """Calls in a row on one stream, with maxima that shrink from call to call (the absmax launch clears for
    itself, against a counter that only grows), and calls that overlap on several streams."""
    import torch
    rng = np.random.default_rng(12)
    T, I = 300, 1024
    outs = []
    for it in range(12):
        X = (rng.standard_normal((T, I)) * (50.0 / (it + 1))).astype(np.float16)
        outs.append((X, cq.crossquant_absmax_quantize(gpu(X), 0.15, 8)))
    streams = [torch.cuda.Stream() for _ in range(6)]
    par = []
    for i, st in enumerate(streams):
        X = outliers(257 + i, 520 + 8 * i, seed=90 + i)
        Xg = gpu(X)
        st.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(st):
            for _ in range(3):
                res = cq.crossquant_absmax_quantize(Xg, 0.45, 4)
        par.append((X, res))
    torch.cuda.synchronize()
    for X, (t, c, codes, xhat, a, b, zc) in outs:
        t_ref, c_ref = oracle.absmax(X)
        ref = oracle.quantize(X, t_ref, c_ref, 0.15, 8)
        assert np.array_equal(bits32(host(t)), bits32(t_ref)) and np.array_equal(bits32(host(c)), bits32(c_ref))
        assert np.array_equal(host(codes), ref["codes"]) and int(host(zc)[0]) == ref["Z"]
        assert np.array_equal(bits16(host(xhat)), bits16(ref["xhat"]))
    for X, (t, c, codes, xhat, a, b, zc) in par:
        t_ref, c_ref = oracle.absmax(X)
        ref = oracle.quantize(X, t_ref, c_ref, 0.45, 4)
        assert np.array_equal(bits32(host(c)), bits32(c_ref)) and np.array_equal(host(codes), ref["codes"])
        assert int(host(zc)[0]) == ref["Z"]


@pytest.mark.parametrize("name", ["C2", "C3", "C5"])
def test_fused_full_configs(cq, name):
    import torch
    cfg = workloads.CONFIGS[name]
    X = workloads.config_activation(name)
    Xg = gpu(X)
    T, I = X.shape
    check_fused(cq, X, 0.15, 8, Xg=Xg, label=name)
    check_fused(cq, X, 0.15, 4, Xg=Xg, label=name, want_xhat=False)
    # same inputs twice: identical outputs (the atomics' order must not matter)
    r1 = cq.crossquant_absmax_quantize(Xg, 0.15, 8)
    r2 = cq.crossquant_absmax_quantize(Xg, 0.15, 8)
    assert all(torch.equal(x, y) for x, y in zip(r1, r2))
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    if ((T + 255) // 256) * ((I + 511) // 512) <= n_cu:        # fits on chip: the single-read kernel as well
        check_fused(cq, X, 0.15, 8, Xg=Xg, label=name, single_read=True)
        check_fused(cq, X, 0.15, 4, Xg=Xg, label=name, want_xhat=False, single_read=True)
        r3 = cq.crossquant_absmax_quantize_single_read(Xg, 0.15, 8)
        assert all(torch.equal(x, y) for x, y in zip(r1, r3))


# ----------------------------------------------------------------------------- batched [B][S][I]
def batch_tensor(B, S, I, seed):
    return np.stack([workloads.activation(S, I, n_outlier=min(2, I), scale_lo=20.0 * (b + 1), scale_hi=20.0 * (b + 1),
                                          seed=seed + b) for b in range(B)])


def check_batched(cq, X3, alpha, bits, Xg=None, label=""):
    say("batched %s shape=%s alpha=%g bits=%d" % (label, X3.shape, alpha, bits))
    Xg = gpu(X3) if Xg is None else Xg
    t_ref, c_ref = oracle.absmax_batched(X3)
    ref = oracle.quantize_batched(X3, t_ref, c_ref, alpha, bits)
    t, c = cq.crossquant_absmax_batched(Xg)
    assert np.array_equal(bits32(host(t)), bits32(t_ref)) and np.array_equal(bits32(host(c)), bits32(c_ref))
    codes, xhat, a, b, zc = cq.crossquant_quantize_batched(Xg, t, c, alpha, bits)
    assert np.array_equal(bits32(host(a)), bits32(ref["a"])) and np.array_equal(bits32(host(b)), bits32(ref["b"]))
    assert np.array_equal(host(codes), ref["codes"])
    assert np.array_equal(bits16(host(xhat)), bits16(ref["xhat"]))
    assert int(host(zc)[0]) == ref["Z"]
    none_codes, none_xhat, _, _, zc2 = cq.crossquant_quantize_batched(Xg, t, c, alpha, bits, want_codes=False)
    assert none_codes is None and none_xhat is None and int(host(zc2)[0]) == ref["Z"]
    return ref


@pytest.mark.parametrize("B,S,I", [(1, 5, 16), (3, 37, 54), (4, 64, 256), (2, 130, 1000), (5, 33, 1538), (7, 1, 8),
                                   (6, 200, 520)])
@pytest.mark.parametrize("bits", [8, 4])
def test_batched_small_and_ragged(cq, B, S, I, bits):
    X3 = batch_tensor(B, S, I, seed=B * 1000 + S + I)
    check_batched(cq, X3, 0.15, bits)


def test_batched_launch_at_the_grid_size_limit(cq):
    """2^23 - 5 one-token sequences, one block each: the largest grid a launch of 512-thread blocks
    can have (its thread count has to stay below 2^32), and nearly the most the zero-count word's
    block field counts.  The oracle takes minutes for that many sequences, so it checks a sample of
    them (first, last and random ones: sequences are independent); the count is checked against
    the zero codes of the whole output.  Eight sequences more and the call is refused."""
    import torch
    B = (1 << 23) - 5
    say("batched, %d sequences of 1 x 1" % B)
    rng = np.random.default_rng(23)
    X3 = rng.standard_normal((B + 8, 1, 1)).astype(np.float16)
    X3[::7, 0, 0] = 0
    Xbig = gpu(X3)
    Xg = Xbig[:B]
    t, c = cq.crossquant_absmax_batched(Xg)
    codes, xhat, a, b, zc = cq.crossquant_quantize_batched(Xg, t, c, 0.15, 8)
    _, _, _, _, zc2 = cq.crossquant_quantize_batched(Xg, t, c, 0.15, 8, want_codes=False)
    n_zero = int((codes == 0).sum().item())
    assert int(host(zc)[0]) == n_zero == int(host(zc2)[0]) == int((X3[:B] == 0).sum())
    idx = np.unique(np.concatenate([np.arange(1500), np.arange(B - 1500, B), rng.integers(0, B, 1000)]))
    Xs = np.ascontiguousarray(X3[idx])
    t_ref, c_ref = oracle.absmax_batched(Xs)
    ref = oracle.quantize_batched(Xs, t_ref, c_ref, 0.15, 8)
    ti = torch.from_numpy(idx).cuda()
    assert np.array_equal(bits32(host(t.view(B, 1)[ti]).ravel()), bits32(t_ref.ravel()))
    assert np.array_equal(bits32(host(c.view(B, 1)[ti]).ravel()), bits32(c_ref.ravel()))
    assert np.array_equal(host(codes.view(B, 1)[ti]).ravel(), ref["codes"].ravel())
    assert np.array_equal(bits16(host(xhat.view(B, 1)[ti]).ravel()), bits16(ref["xhat"].ravel()))
    # 2^23 + 3 sequences: the maxima still fit (256-thread blocks), the quantize launch does not
    t2, c2 = cq.crossquant_absmax_batched(Xbig)
    assert np.array_equal(bits32(host(t2[:B])), bits32(host(t)))
    with pytest.raises(cq.CrossQuantError) as err:
        cq.crossquant_quantize_batched(Xbig, t2, c2, 0.15, 8)
    assert err.value.status == -2


def test_batched_views_with_padding_between_sequences(cq):
    base = batch_tensor(3, 40, 304, seed=9)
    g = gpu(base)
    for (s0, s1, lo, hi) in ((0, 40, 8, 264), (3, 35, 0, 304), (2, 39, 1, 257)):
        view = np.ascontiguousarray(base[:, s0:s1, lo:hi])
        check_batched(cq, view, 0.15, 8, Xg=g[:, s0:s1, lo:hi], label="view[%d:%d,%d:%d]" % (s0, s1, lo, hi))


def test_batched_equals_separate_calls_at_layer_scale(cq):
    """32 sequences of 128 tokens x 4096 channels: one launch each for the maxima and the
    quantizer, compared with the oracle on sampled sequences and with per-sequence GPU calls."""
    import torch
    B, S, I = 32, 128, 4096
    X3 = batch_tensor(B, S, I, seed=77)
    Xg = gpu(X3)
    t, c = cq.crossquant_absmax_batched(Xg)
    codes, xhat, a, b, zc = cq.crossquant_quantize_batched(Xg, t, c, 0.15, 8)
    z = 0
    for bi in range(B):
        t1, c1 = cq.crossquant_absmax(Xg[bi])
        q1, x1, a1, b1, z1 = cq.crossquant_quantize(Xg[bi], t1, c1, 0.15, 8)
        assert torch.equal(t1, t[bi]) and torch.equal(c1, c[bi]) and torch.equal(q1, codes[bi])
        assert torch.equal(x1, xhat[bi]) and torch.equal(a1, a[bi]) and torch.equal(b1, b[bi])
        z += int(z1.item())
    assert z == int(zc.item())
    for bi in (0, 17, 31):
        tr, cr = oracle.absmax(X3[bi])
        ref = oracle.quantize(X3[bi], tr, cr, 0.15, 8)
        assert np.array_equal(host(codes[bi]), ref["codes"]) and np.array_equal(bits16(host(xhat[bi])), bits16(ref["xhat"]))


# ----------------------------------------------------------------------------- Remove Kernel, Table 1 indicators
def check_analysis(cq, X, alpha, bits, Xg=None, label=""):
    say("analysis %s shape=%s alpha=%g bits=%d" % (label, X.shape, alpha, bits))
    Xg = gpu(X) if Xg is None else Xg
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.kernel_analysis(X, t_ref, c_ref, alpha, bits)
    t, c = cq.crossquant_absmax(Xg)
    xrk, counters = cq.crossquant_kernel_analysis(Xg, t, c, alpha, bits)
    got = host(counters)
    assert [int(v) for v in got] == [ref["Z"], ref["n_col_ge_row"], ref["n_bound_smaller"]]
    assert np.array_equal(bits16(host(xrk)), bits16(ref["xrk"]))
    none_xrk, counters2 = cq.crossquant_kernel_analysis(Xg, t, c, alpha, bits, want_xrk=False)
    assert none_xrk is None and np.array_equal(host(counters2), got)
    # without work vectors (NULL, NULL): the kernel forms the factors itself
    xrk3, counters3 = cq.crossquant_kernel_analysis(Xg, t, c, alpha, bits, work_vectors=False)
    assert np.array_equal(host(counters3), got) and np.array_equal(bits16(host(xrk3)), bits16(ref["xrk"]))
    return ref


@pytest.mark.parametrize("T,I", [(1, 1), (3, 6), (37, 54), (130, 1000), (129, 520), (200, 1537)])
def test_analysis_small_and_ragged(cq, T, I):
    X = outliers(T, I, seed=T * 7 + I)
    if T > 2 and I > 5:
        X[1, :] = 0
        X[:, 4] = 0
        X[2, 3] = np.float16(-0.0)
    for alpha, bits in ((1.0, 8), (0.15, 8), (0.15, 4), (0.0, 8)):
        check_analysis(cq, X, alpha, bits)


def test_analysis_strided_input(cq):
    base = outliers(40, 300, seed=19)
    g = gpu(base)
    for lo, hi in ((8, 264), (3, 259)):
        check_analysis(cq, base[:, lo:hi], 0.15, 8, Xg=g[:, lo:hi], label="view[%d:%d]" % (lo, hi))


@pytest.mark.parametrize("name", ["C1", "C3", "C5"])
def test_analysis_full_configs(cq, name):
    cfg = workloads.CONFIGS[name]
    X = workloads.config_activation(name)
    Xg = gpu(X)
    for alpha in (0.15, 1.0):
        ref = check_analysis(cq, X, alpha, cfg.bits, Xg=Xg, label=name)
        say("%s alpha=%g: kernel %.4f, c_j>=t_i %.4f, B~<B %.4f" % (
            name, alpha, ref["Z"] / X.size, ref["n_col_ge_row"] / X.size, ref["n_bound_smaller"] / X.size))


# ----------------------------------------------------------------------------- weights
WEIGHT_SHAPES = [(1, 1), (8, 8), (70, 45), (64, 64), (256, 256), (130, 1000), (1000, 130), (513, 520)]


@pytest.mark.parametrize("I,O", WEIGHT_SHAPES)
@pytest.mark.parametrize("bits", [8, 4])
def test_weight_quantize_small_and_ragged(cq, I, O, bits):
    say("weight quantize I=%d O=%d bits=%d" % (I, O, bits))
    W = workloads.weight(I, O, seed=I + O)
    if I > 4 and O > 4:
        W[:, 3] = 0                                             # an all-zero output channel
    fold = np.random.default_rng(I).uniform(0.05, 8.0, I).astype(np.float32)
    for f in (None, fold):
        qw_ref, s_ref = oracle.weight_quantize(W, f, bits)
        qw, s = cq.crossquant_weight_quantize(gpu(W), None if f is None else gpu(f), bits)
        assert np.array_equal(bits32(host(s)), bits32(s_ref))
        assert np.array_equal(host(qw), qw_ref)


@pytest.mark.parametrize("I,O,group", [(8, 8, 8), (96, 20, 32), (96, 20, 8), (256, 256, 128), (384, 130, 128),
                                         (130, 77, 10), (1024, 520, 64), (70, 45, 70)])
@pytest.mark.parametrize("bits", [8, 4])
def test_weight_quantize_grouped(cq, I, O, group, bits):
    say("grouped weight quantize I=%d O=%d g=%d bits=%d" % (I, O, group, bits))
    W = workloads.weight(I, O, seed=I * 3 + O)
    if I >= 2 * group and O > 3:
        W[group:2 * group, 2] = 0                                  # an all-zero group
    fold = np.random.default_rng(O).uniform(0.05, 8.0, I).astype(np.float32)
    for f in (None, fold):
        qw_ref, s_ref, dq_ref = oracle.weight_quantize_grouped(W, f, group, bits)
        qw, s, dq = cq.crossquant_weight_quantize_grouped(gpu(W), None if f is None else gpu(f), group, bits,
                                                          want_dq=True)
        assert np.array_equal(bits32(host(s)), bits32(s_ref))
        assert np.array_equal(host(qw), qw_ref)
        assert np.array_equal(bits16(host(dq)), bits16(dq_ref))
        qw2, s2, none_dq = cq.crossquant_weight_quantize_grouped(gpu(W), None if f is None else gpu(f), group, bits)
        assert none_dq is None and np.array_equal(host(qw2), qw_ref) and np.array_equal(host(s2), s_ref)


def test_weight_quantize_grouped_at_layer_scale(cq):
    """The paper's W4-g128 setting on the low-bit configuration's 4096 x 4096 weight."""
    W = workloads.config_weight("C4")
    qw_ref, s_ref, dq_ref = oracle.weight_quantize_grouped(W, None, 128, 4)
    qw, s, dq = cq.crossquant_weight_quantize_grouped(gpu(W), None, 128, 4, want_dq=True)
    assert np.array_equal(bits32(host(s)), bits32(s_ref)) and np.array_equal(host(qw), qw_ref)
    assert np.array_equal(bits16(host(dq)), bits16(dq_ref))


def test_weight_crossquant_through_the_activation_calls(cq):
    """CrossQuant on weights (alpha_W): the activation calls applied to the weight stored
    output-channel-major; alpha_W = 1 reproduces per-channel quantization (Eq. 2)."""
    say("weight crossquant")
    W = workloads.weight(512, 384, seed=5)
    Wt = np.ascontiguousarray(W.T)
    Wg = gpu(Wt)
    t, c = cq.crossquant_absmax(Wg)
    for alpha_w in (1.0, 0.55, 0.0):
        t_ref, c_ref = oracle.absmax(Wt)
        ref = oracle.quantize(Wt, t_ref, c_ref, alpha_w, 8)
        codes, what, u, v, _ = cq.crossquant_quantize(Wg, t, c, alpha_w, 8)
        assert np.array_equal(host(codes), ref["codes"]) and np.array_equal(bits16(host(what)), bits16(ref["xhat"]))
        assert np.array_equal(host(u), ref["a"]) and np.array_equal(host(v), ref["b"])
    qw_pc, s_pc = cq.crossquant_weight_quantize(gpu(W), None, 8)
    codes, _, u, _, _ = cq.crossquant_quantize(Wg, t, c, 1.0, 8, want_xhat=False)
    import torch
    assert torch.equal(codes, qw_pc) and torch.equal(u, s_pc)


# ----------------------------------------------------------------------------- linear
LINEAR_SHAPES = [(1, 16, 1), (5, 32, 7), (100, 200, 300), (64, 256, 256), (256, 128, 256), (300, 208, 270),
                 (256, 1024, 512), (513, 384, 257), (33, 100, 65),
                 # ragged token / channel counts on the MFMA fast path (I % 128 == 0, O % 8 == 0)
                 (1, 128, 8), (300, 256, 520), (257, 384, 264), (513, 1024, 1000), (700, 512, 776), (255, 128, 248)]


@pytest.mark.parametrize("T,I,O", LINEAR_SHAPES)
def test_linear_small_and_ragged(cq, T, I, O):
    say("linear T=%d I=%d O=%d" % (T, I, O))
    qx = workloads.int8_codes(T, I, seed=T)
    qw = workloads.int8_codes(O, I, seed=O + 7)
    rng = np.random.default_rng(T + O)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    Y, acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), want_acc=True)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(bits16(host(Y)), bits16(Y_ref))
    Y2, none_acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s))
    assert none_acc is None and np.array_equal(bits16(host(Y2)), bits16(Y_ref))


@pytest.mark.parametrize("T,I,O", [(2304, 256, 10240),     # 9 x 40 = 360 tiles = 1.41 rounds of 256: 104 tiles run as halves
                                   (2250, 256, 10248),     # 9 x 41 = 369 tiles, ragged: the last tile column is 8 wide
                                   (1280, 384, 5120),      # 100 tiles, less than half a round: every tile runs as two halves
                                   (300, 128, 392),        # 4 tiles; the last one's second half is empty
                                   (256, 128, 128)])       # one tile that is a single half
def test_linear_with_a_partly_filled_last_round_of_tiles(cq, T, I, O):
    """One block fills a CU, so output tiles run in rounds of 256; a last round that is at most half full is run as
    256 x 128 half tiles.  Every accumulator and output against the oracle."""
    say("linear, half-tile round: T=%d I=%d O=%d" % (T, I, O))
    qx = workloads.int8_codes(T, I, seed=T + 1)
    qw = workloads.int8_codes(O, I, seed=O + 11)
    rng = np.random.default_rng(T + O)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    Y, acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), want_acc=True)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(bits16(host(Y)), bits16(Y_ref))
    # without the raw accumulators a block requests its next (half) tile's first operands before its epilogue
    for _ in range(2):
        Y2, none_acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s))
        assert none_acc is None and np.array_equal(bits16(host(Y2)), bits16(Y_ref))


@pytest.mark.parametrize("T,I,O", [(5120, 128, 5120),      # 400 tiles = 1.56 rounds, taken whole: 144 blocks walk two tiles; one K step
                                   (5120, 384, 5120),      # the same with three K steps
                                   (4100, 256, 7688),      # 17 x 31 = 527 tiles, ragged on both edges: two whole rounds + 15 tiles as halves
                                   (8192, 128, 6144)])     # 768 tiles = three whole rounds
def test_linear_blocks_walk_several_tiles(cq, T, I, O):
    """With more output tiles than CUs a block works through several of them, and (when the raw accumulators are not
    asked for) requests the next tile's first operands before it scales and stores the current one.  Every output of
    both forms against the oracle, twice in a row into the same buffer."""
    say("linear, several tiles per block: T=%d I=%d O=%d" % (T, I, O))
    qx = workloads.int8_codes(T, I, seed=T + 3)
    qw = workloads.int8_codes(O, I, seed=O + 13)
    rng = np.random.default_rng(T + O)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    gx, ga, gw, gs = gpu(qx), gpu(a), gpu(qw), gpu(s)
    Y, none_acc = cq.crossquant_w8a8_linear(gx, ga, gw, gs)
    assert none_acc is None and np.array_equal(bits16(host(Y)), bits16(Y_ref))
    Y.zero_()
    cq.crossquant_w8a8_linear(gx, ga, gw, gs, Y=Y)
    assert np.array_equal(bits16(host(Y)), bits16(Y_ref))
    Y2, acc = cq.crossquant_w8a8_linear(gx, ga, gw, gs, want_acc=True)
    assert np.array_equal(host(acc), acc_ref) and np.array_equal(bits16(host(Y2)), bits16(Y_ref))


def test_linear_extreme_accumulators(cq):
    say("linear extremes")
    T, I, O = 256, 8192, 256
    qx = np.full((T, I), 127, np.int8)
    qx[1::2] = -127
    qw = np.full((O, I), 127, np.int8)
    qw[::3] = -127
    a = np.full(T, 2.0 ** -20, np.float32)
    s = np.full(O, 2.0 ** -6, np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx[:4], a[:4], qw, s)
    Y, acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), want_acc=True)
    acc = host(acc)
    assert np.array_equal(acc[:4], acc_ref) and abs(int(acc[0, 1])) == 127 * 127 * I
    assert np.array_equal(acc[0::2], np.broadcast_to(acc[0], (T // 2, O)))
    assert np.array_equal(acc[1::2], np.broadcast_to(acc[1], (T // 2, O)))
    assert np.array_equal(bits16(host(Y))[:4], bits16(Y_ref))


def test_linear_strided_output(cq):
    import torch
    say("linear ldy > O")
    T, I, O = 70, 64, 40
    qx, qw = workloads.int8_codes(T, I, seed=1), workloads.int8_codes(O, I, seed=2)
    a = np.full(T, 0.01, np.float32)
    s = np.full(O, 0.001, np.float32)
    Y_ref, _ = oracle.w8a8_linear(qx, a, qw, s)
    buf = torch.full((T, 64), 7.0, dtype=torch.float16, device="cuda")
    cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), Y=buf[:, :O])
    out = host(buf)
    assert np.array_equal(bits16(out[:, :O]), bits16(Y_ref)) and np.all(out[:, O:] == 7.0)


def test_linear_ragged_fast_path_writes_nothing_outside_its_output(cq):
    """Ragged T and O on the MFMA fast path (edge tiles read clamped rows and drop the surplus
    outputs): rows past T and columns past O of the surrounding buffer must stay untouched."""
    import torch
    say("linear ragged fast path, guarded buffer")
    T, I, O = 300, 256, 520
    qx, qw = workloads.int8_codes(T, I, seed=3), workloads.int8_codes(O, I, seed=4)
    rng = np.random.default_rng(6)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    buf = torch.full((T + 20, 640), 7.0, dtype=torch.float16, device="cuda")
    accbuf = torch.full((T + 20, O), -5, dtype=torch.int32, device="cuda")
    cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), Y=buf[:T, :O], acc_debug=accbuf[:T])
    out, acc = host(buf), host(accbuf)
    assert np.array_equal(bits16(out[:T, :O]), bits16(Y_ref)) and np.array_equal(acc[:T], acc_ref)
    assert np.all(out[:T, O:] == 7.0) and np.all(out[T:] == 7.0) and np.all(acc[T:] == -5)


def test_end_to_end_tiny_config(cq):
    """C1 through every call: absmax -> quantize -> weight quantize (folded) -> linear."""
    say("end to end C1")
    X, W = workloads.config_activation("C1"), workloads.config_weight("C1")
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, 0.15, 8)
    qw_ref, s_ref = oracle.weight_quantize(W, ref["b"], 8)
    Y_ref, acc_ref = oracle.w8a8_linear(ref["codes"], ref["a"], qw_ref, s_ref)
    Xg, Wg = gpu(X), gpu(W)
    t, c = cq.crossquant_absmax(Xg)
    codes, _, a, b, _ = cq.crossquant_quantize(Xg, t, c, 0.15, 8, want_xhat=False)
    qw, s = cq.crossquant_weight_quantize(Wg, b, 8)
    Y, acc = cq.crossquant_w8a8_linear(codes, a, qw, s, want_acc=True)
    assert np.array_equal(host(qw), qw_ref) and np.array_equal(bits32(host(s)), bits32(s_ref))
    assert np.array_equal(host(acc), acc_ref) and np.array_equal(bits16(host(Y)), bits16(Y_ref))
    full = X.astype(np.float64) @ W.astype(np.float64)
    rel = np.linalg.norm(host(Y).astype(np.float64) - full) / np.linalg.norm(full)
    assert rel < 0.05


@pytest.mark.parametrize("T,I", [(1, 2), (3, 6), (37, 54), (64, 256), (129, 1030)])
def test_unpack_int4(cq, T, I):
    say("unpack int4 T=%d I=%d" % (T, I))
    packed = np.random.default_rng(T + I).integers(0, 256, (T, I // 2), dtype=np.uint8)
    got = host(cq.crossquant_unpack_int4(gpu(packed)))
    assert np.array_equal(got, oracle.unpack_int4(packed))


def test_end_to_end_a4w4_config(cq):
    """C4 (4096 x 4096, A4 W4): packed INT4 activations, expanded to bytes, through the INT8 GEMM."""
    import torch
    say("end to end C4 (A4W4)")
    cfg = workloads.CONFIGS["C4"]
    X, W = workloads.config_activation("C4"), workloads.config_weight("C4")
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, 0.15, 4, want_xhat=False)
    qx_ref = oracle.unpack_int4(ref["codes"])
    qw_ref, s_ref = oracle.weight_quantize(W, ref["b"], 4)
    Xg, Wg = gpu(X), gpu(W)
    t, c = cq.crossquant_absmax(Xg)
    packed, _, a, b, zc = cq.crossquant_quantize(Xg, t, c, 0.15, 4, want_xhat=False)
    z_pt = cq.crossquant_kernel_count(Xg, t, c, 1.0, 4)
    qx = cq.crossquant_unpack_int4(packed)
    qw, s = cq.crossquant_weight_quantize(Wg, b, 4)
    Y, acc = cq.crossquant_w8a8_linear(qx, a, qw, s, want_acc=True)
    assert np.array_equal(host(packed), ref["codes"]) and np.array_equal(host(qx), qx_ref)
    assert np.array_equal(host(qw), qw_ref) and np.array_equal(bits32(host(s)), bits32(s_ref))
    assert int(np.abs(host(qx)).max()) <= 7 and int(np.abs(host(qw)).max()) <= 7
    rows = np.array([0, 1, 255, 256, 1000, 4095])
    Yr, accr = oracle.w8a8_linear(qx_ref[rows], ref["a"][rows], qw_ref, s_ref)
    ridx = torch.from_numpy(rows).cuda()
    assert np.array_equal(host(acc[ridx]), accr) and np.array_equal(bits16(host(Y[ridx])), bits16(Yr))
    want_k = (qw_ref.astype(np.float64) @ qx_ref.astype(np.int64).sum(axis=0).astype(np.float64)).astype(np.int64)
    assert np.array_equal(host(acc.sum(dim=0, dtype=torch.int64)), want_k)
    # zero-count reported against the per-token baseline, as the low-bit configuration asks
    z, zp = int(host(zc)[0]), int(host(z_pt)[0])
    assert z == ref["Z"] and zp == oracle.kernel_count(X, t_ref, c_ref, 1.0, 4) and z < zp
    say("C4 kernel proportion: crossquant %.4f per-token %.4f" % (z / X.size, zp / X.size))


@pytest.mark.parametrize("name", ["C2", "C3", "C5"])
def test_end_to_end_full_config_sampled(cq, name):
    """Full-size run in the benchmark's launch configuration.  Weight codes and steps are
    compared in full; accumulators and outputs on sampled rows and columns the oracle recomputes
    one by one, plus exact integer checksums that cover every output in aggregate."""
    import torch
    say("end to end %s" % name)
    cfg = workloads.CONFIGS[name]
    X, W = workloads.config_activation(name), workloads.config_weight(name)
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, 0.15, 8, want_xhat=False)
    qw_ref, s_ref = oracle.weight_quantize(W, ref["b"], 8)
    say("oracle side ready")
    Xg, Wg = gpu(X), gpu(W)
    t, c = cq.crossquant_absmax(Xg)
    codes, _, a, b, _ = cq.crossquant_quantize(Xg, t, c, 0.15, 8, want_xhat=False)
    qw, s = cq.crossquant_weight_quantize(Wg, b, 8)
    assert np.array_equal(host(codes), ref["codes"])
    assert np.array_equal(bits32(host(s)), bits32(s_ref))
    assert torch.equal(qw.cpu(), torch.from_numpy(qw_ref))
    Y, acc = cq.crossquant_w8a8_linear(codes, a, qw, s, want_acc=True)
    torch.cuda.synchronize()
    say("gpu side done")
    rng = np.random.default_rng(11)
    # at least 64 whole rows and 256 whole columns, tile edges included
    rows = np.sort(rng.choice(cfg.T, 64, replace=False))
    rows = np.unique(np.concatenate([rows, [0, cfg.T - 1, 255, 256]]))
    cols = np.sort(rng.choice(cfg.O, 256, replace=False))
    cols = np.unique(np.concatenate([cols, [0, cfg.O - 1, 255, 256]]))
    Yr, accr = oracle.w8a8_linear(ref["codes"][rows], ref["a"][rows], qw_ref, s_ref)
    assert np.array_equal(host(acc[torch.from_numpy(rows).cuda()]), accr)
    assert np.array_equal(bits16(host(Y[torch.from_numpy(rows).cuda()])), bits16(Yr))
    Yc, accc = oracle.w8a8_linear(ref["codes"], ref["a"], qw_ref[cols], s_ref[cols])
    assert np.array_equal(host(acc[:, torch.from_numpy(cols).cuda()]), accc)
    assert np.array_equal(bits16(host(Y[:, torch.from_numpy(cols).cuda()])), bits16(Yc))
    # checksums: sum_i acc_ik = sum_j (sum_i q_ij) qw_kj ; sum_k acc_ik = sum_j q_ij (sum_k qw_kj)
    col_sum = ref["codes"].astype(np.int64).sum(axis=0)
    row_sum_w = qw_ref.astype(np.int64).sum(axis=0)
    want_k = (qw_ref.astype(np.float64) @ col_sum.astype(np.float64)).astype(np.int64)   # exact: < 2^53
    want_i = (ref["codes"].astype(np.float64) @ row_sum_w.astype(np.float64)).astype(np.int64)
    assert np.array_equal(host(acc.sum(dim=0, dtype=torch.int64)), want_k)
    assert np.array_equal(host(acc.sum(dim=1, dtype=torch.int64)), want_i)
    # every output equals its own accumulator through the epilogue (checked on the GPU tensors)
    y_from_acc = ((acc.to(torch.float32) * a[:, None]) * s[None, :]).to(torch.float16)
    assert torch.equal(y_from_acc.view(torch.int16), Y.view(torch.int16))


# ----------------------------------------------------------------------------- quantize inside the GEMM's activation load
@pytest.mark.parametrize("T,I,O,bits,alpha", [(1, 128, 8, 8, 0.15), (37, 128, 70, 8, 0.0), (300, 256, 520, 8, 0.15),
                                              (257, 384, 264, 4, 0.15), (513, 1024, 1000, 8, 1.0), (64, 256, 256, 4, 0.5)])
def test_quantize_inside_the_gemm_equals_the_two_calls_and_the_oracle(cq, T, I, O, bits, alpha):
    say("fused quantize + linear T=%d I=%d O=%d bits=%d alpha=%g" % (T, I, O, bits, alpha))
    X = outliers(T, I, seed=T + I + O)
    if T > 2:
        X[1, :] = 0                      # a zero row: a_i = 0
        X[:, 5] = 0                      # a zero column: b_j = 0 (alpha < 1)
    W = workloads.weight(I, O, seed=O)
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, alpha, bits, want_xhat=False)
    codes_ref = ref["codes"] if bits == 8 else oracle.unpack_int4(ref["codes"])
    qw_ref, s_ref = oracle.weight_quantize(W, ref["b"], bits)
    Y_ref, acc_ref = oracle.w8a8_linear(codes_ref, ref["a"], qw_ref, s_ref)
    Xg = gpu(X)
    t, c = cq.crossquant_absmax(Xg)
    Y, a, b, acc = cq.crossquant_quantize_linear_fused(Xg, t, c, alpha, bits, gpu(qw_ref), gpu(s_ref), want_acc=True)
    assert np.array_equal(bits32(host(a)), bits32(ref["a"])) and np.array_equal(bits32(host(b)), bits32(ref["b"]))
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(bits16(host(Y)), bits16(Y_ref))


def test_quantize_inside_the_gemm_rounding_ties_and_layer_scale(cq):
    """Exact ties (the fast quotient must hand over to the division inside the GEMM's loader too) and a
    full-size layer, against the two calls."""
    import torch
    say("fused quantize + linear: ties, then C4 against the two calls")
    T, I, O = 128, 128, 64
    X = np.zeros((T, I), dtype=np.float16)
    X[:, 0] = 127.0                              # every row and column maximum 127 -> D = 1 at any alpha
    X[0, :] = 127.0
    X[1:, 1:] = (np.arange((T - 1) * (I - 1)).reshape(T - 1, I - 1) % 253 - 126 + 0.5).astype(np.float16)   # k + 1/2
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, 0.5, 8, want_xhat=False)
    qw = workloads.int8_codes(O, I, seed=3)
    s = np.full(O, 1e-3, np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(ref["codes"], ref["a"], qw, s)
    Xg = gpu(X)
    t, c = cq.crossquant_absmax(Xg)
    Y, a, b, acc = cq.crossquant_quantize_linear_fused(Xg, t, c, 0.5, 8, gpu(qw), gpu(s), want_acc=True)
    assert np.array_equal(host(acc), acc_ref) and np.array_equal(bits16(host(Y)), bits16(Y_ref))
    cfg = workloads.CONFIGS["C4"]
    Xg, Wg = gpu(workloads.config_activation("C4")), gpu(workloads.config_weight("C4"))
    t, c = cq.crossquant_absmax(Xg)
    nib, _, a2, b2, _ = cq.crossquant_quantize(Xg, t, c, 0.15, 4, want_xhat=False)
    qw4, ws4 = cq.crossquant_weight_quantize(Wg, b2, 4)
    Y2, acc2 = cq.crossquant_w8a8_linear(cq.crossquant_unpack_int4(nib), a2, qw4, ws4, want_acc=True)
    Y, a, b, acc = cq.crossquant_quantize_linear_fused(Xg, t, c, 0.15, 4, qw4, ws4, want_acc=True)
    assert torch.equal(acc, acc2) and torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
    assert torch.equal(a, a2) and torch.equal(b, b2)


# ----------------------------------------------------------------------------- HIP graph replay
def test_whole_path_replays_from_a_hip_graph(cq):
    """The calls allocate nothing, never synchronise and clear their accumulators with kernels, so
    the whole path can be captured once and replayed.  Every replay (with eager work and
    synchronisations in between, and new input values each time) must equal the eager result."""
    import torch
    T, I, O = 300, 1024, 520
    W = workloads.weight(I, O, seed=5)
    Wg = gpu(W)
    Xg = torch.empty((T, I), dtype=torch.float16, device="cuda")
    t = torch.empty(T, device="cuda"); c = torch.empty(I, device="cuda")
    a = torch.empty(T, device="cuda"); b = torch.empty(I, device="cuda")
    a1 = torch.empty(T, device="cuda"); b1 = torch.empty(I, device="cuda")
    codes = torch.empty((T, I), dtype=torch.int8, device="cuda")
    xhat = torch.empty((T, I), dtype=torch.float16, device="cuda")
    zc = torch.empty(1, dtype=torch.int64, device="cuda"); zc1 = torch.empty(1, dtype=torch.int64, device="cuda")
    qw = torch.empty((O, I), dtype=torch.int8, device="cuda"); ws = torch.empty(O, device="cuda")
    Y = torch.empty((T, O), dtype=torch.float16, device="cuda")

    def path():
        cq.crossquant_absmax(Xg, t=t, c=c)
        cq.crossquant_quantize(Xg, t, c, 0.15, 8, codes=codes, xhat=xhat, row_scale=a, col_scale=b, zero_count=zc)
        cq.crossquant_kernel_count(Xg, t, c, 1.0, 8, row_scale=a1, col_scale=b1, zero_count=zc1)
        cq.crossquant_weight_quantize(Wg, b, 8, qw=qw, w_scale=ws)
        cq.crossquant_w8a8_linear(codes, a, qw, ws, Y=Y)

    Xg.copy_(gpu(outliers(T, I, seed=100)))
    path()                                             # warm up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            path()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        X = outliers(T, I, seed=200 + rep)
        say("graph replay %d" % rep)
        Xg.copy_(gpu(X))
        for buf in (t, c, a, b, codes, xhat, zc, zc1, Y):       # stale contents before every replay
            buf.fill_(1)
        graph.replay()
        torch.cuda.synchronize()
        got = [host(x).copy() for x in (t, c, a, b, codes, xhat, zc, zc1, qw, ws, Y)]
        t_ref, c_ref = oracle.absmax(X)
        ref = oracle.quantize(X, t_ref, c_ref, 0.15, 8)
        assert np.array_equal(got[4], ref["codes"]) and int(got[6][0]) == ref["Z"]
        assert int(got[7][0]) == oracle.kernel_count(X, t_ref, c_ref, 1.0, 8)
        path()                                         # eager, same inputs
        torch.cuda.synchronize()
        eager = [host(x) for x in (t, c, a, b, codes, xhat, zc, zc1, qw, ws, Y)]
        for g_, e_ in zip(got, eager):
            assert np.array_equal(g_.view(np.uint8), e_.view(np.uint8))


# ----------------------------------------------------------------------------- roofline calibration kernels
def test_calibration_kernels_run_and_copy_is_exact(cq):
    import torch
    n = (3 << 20) + 16 * 7                                  # not a multiple of the grid's stride
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    cq.crossquant_calib_copy(src, dst)
    cq.crossquant_calib_read(src)
    ops = cq.crossquant_calib_mfma_i8(10, 1)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    assert ops == n_cu * 4 * 10 * 16 * 65536.0
    ops_lds = cq.crossquant_calib_mfma_i8(10, 2)            # the loop fed from LDS: 8 waves x 32 instructions (16 x 16 x 64) a step
    ops_16 = cq.crossquant_calib_mfma_i8(10, 3)             # the same instruction on operands in registers: 8 waves
    torch.cuda.synchronize()
    assert ops_lds == n_cu * 8 * 10 * 32 * 32768.0 and ops_16 == n_cu * 8 * 10 * 32 * 32768.0
    ops_f6 = cq.crossquant_calib_mfma_f6(10)                # the FP6 loop fed from LDS: 8 waves x 32 instructions (16 x 16 x 128)
    torch.cuda.synchronize()
    assert ops_f6 == n_cu * 8 * 10 * 32 * 65536.0


# ----------------------------------------------------------------------------- seeded random shapes
def test_random_shapes_quantizer(cq):
    """Sixty seeded random problems (shape, alpha, bits, distribution) through absmax, quantize,
    count and, where the layout allows, the single-read call."""
    rng = np.random.default_rng(2024)
    for case in range(60):
        T = int(rng.integers(1, 700))
        I = int(rng.integers(1, 2100))
        bits = int(rng.choice([4, 8]))
        if bits == 4:
            I += I & 1
        alpha = float(rng.choice([0.0, 0.05, 0.15, 0.3, 0.55, 0.85, 1.0]))
        dist = str(rng.choice(["normal", "student_t3"]))
        X = outliers(T, I, seed=1000 + case, n_out=int(rng.integers(0, 4)), scale=float(rng.uniform(5, 200)), dist=dist)
        check_quantize(cq, X, alpha, bits, label="random %d" % case)
        if I % 8 == 0:
            check_fused(cq, X, alpha, bits, label="random %d" % case)


def test_random_shapes_linear(cq):
    """Forty seeded random GEMM shapes, half of them on the MFMA fast path's conditions."""
    rng = np.random.default_rng(4048)
    for case in range(40):
        T = int(rng.integers(1, 900))
        if case % 2:
            I = 128 * int(rng.integers(1, 9))
            O = 8 * int(rng.integers(1, 120))
        else:
            I = int(rng.integers(1, 1100))
            O = int(rng.integers(1, 900))
        say("random linear %d: T=%d I=%d O=%d" % (case, T, I, O))
        qx = workloads.int8_codes(T, I, seed=5000 + case)
        qw = workloads.int8_codes(O, I, seed=6000 + case)
        a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
        s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
        Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
        Y, acc = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s), want_acc=True)
        assert np.array_equal(host(acc), acc_ref)
        assert np.array_equal(bits16(host(Y)), bits16(Y_ref))


# ----------------------------------------------------------------------------- A4W4 on the FP6 matrix instruction
E2M3 = np.array([0, 8, 16, 20, 24, 26, 28, 30], np.uint8)      # bit patterns of 0..7 (1 sign, 2 exponent, 3 mantissa)


def fp6_fragments(codes):
    """The operand format written out with numpy: [ceil(R/32)][K/64] fragments; lane l = row l & 31,
    columns [32 (l >> 5), +32), element j in bits [6j, 6j+6) of the lane's 192-bit stream; a
    fragment is 64 lanes x 16 bytes (bits 0..127) followed by 64 lanes x 8 bytes (bits 128..191)."""
    R, K = codes.shape
    RB, KB = (R + 31) // 32, K // 64
    padded = np.zeros((RB * 32, K), np.int64)
    padded[:R] = np.clip(codes.astype(np.int64), -7, 7)
    pat = E2M3[np.abs(padded)].astype(np.uint64) | np.where(padded < 0, 32, 0).astype(np.uint64)
    lanes = pat.reshape(RB, 32, KB, 2, 32).transpose(0, 2, 3, 1, 4).reshape(RB, KB, 64, 32)   # [rb][kb][lane][j]
    words = np.zeros((RB, KB, 64, 3), np.uint64)                                              # three 64-bit words per lane
    for j in range(32):
        bit = 6 * j
        p, sh = bit // 64, bit % 64
        words[..., p] |= (lanes[..., j] << np.uint64(sh)) & np.uint64(0xFFFFFFFFFFFFFFFF)
        if sh > 58:
            words[..., p + 1] |= lanes[..., j] >> np.uint64(64 - sh)
    lo = np.ascontiguousarray(words[..., 0:2]).reshape(RB, KB, 64 * 2)
    hi = np.ascontiguousarray(words[..., 2]).reshape(RB, KB, 64)
    return np.concatenate([lo, hi], axis=2).reshape(-1).view(np.uint8)


def fp6_weight_fragments(codes):
    """The weight operand: the same fragments over the rows in interleaved order -- inside every group of 64 output
    channels, stored row 16 n + f holds channel 4 f + n (channels past O are zero rows)."""
    O, K = codes.shape
    padded = np.zeros(((O + 63) // 64 * 64, K), codes.dtype)
    padded[:O] = codes
    stored = np.arange(padded.shape[0])
    source = (stored // 64) * 64 + 4 * (stored % 16) + (stored % 64) // 16
    return fp6_fragments(padded[source])


def int4_codes(R, K, seed):
    return np.random.default_rng(seed).integers(-7, 8, (R, K)).astype(np.int8)


def nibbles(codes):
    c = codes.astype(np.uint8) & 0xF
    return (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)


@pytest.mark.parametrize("R,K", [(1, 128), (32, 128), (45, 256), (300, 384), (64, 1024)])
def test_fp6_packing(cq, R, K):
    codes = int4_codes(R, K, seed=R + K)
    want = fp6_fragments(codes)
    got8 = host(cq.crossquant_pack_fp6(gpu(codes)))
    got4 = host(cq.crossquant_pack_fp6(gpu(nibbles(codes))))
    assert got8.shape == want.shape and np.array_equal(got8, want)
    assert np.array_equal(got4, want)
    # codes outside the INT4 range saturate
    wide = (codes.astype(np.int16) * 3).clip(-128, 127).astype(np.int8)
    assert np.array_equal(host(cq.crossquant_pack_fp6(gpu(wide))), fp6_fragments(wide))
    # the weight operand's row order
    want_w = fp6_weight_fragments(codes)
    got_w8 = host(cq.crossquant_pack_fp6_weights(gpu(codes)))
    assert got_w8.shape == want_w.shape and np.array_equal(got_w8, want_w)
    assert np.array_equal(host(cq.crossquant_pack_fp6(gpu(nibbles(codes)), weights=True)), want_w)


@pytest.mark.parametrize("T,I,O", [(1, 128, 8), (32, 128, 32), (256, 256, 256), (300, 256, 520), (257, 384, 264),
                                   (513, 1024, 1000), (700, 512, 776), (64, 2048, 128)])
def test_w4a4_linear_fp6(cq, T, I, O):
    say("w4a4 fp6 T=%d I=%d O=%d" % (T, I, O))
    qx, qw = int4_codes(T, I, seed=T), int4_codes(O, I, seed=O + 7)
    rng = np.random.default_rng(T + O)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    px, pw = cq.crossquant_pack_fp6(gpu(nibbles(qx))), cq.crossquant_pack_fp6_weights(gpu(qw))
    Y, acc = cq.crossquant_w4a4_linear(px, gpu(a), pw, gpu(s), T, I, O, want_acc=True)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(bits16(host(Y)), bits16(Y_ref))
    Y8, _ = cq.crossquant_w8a8_linear(gpu(qx), gpu(a), gpu(qw), gpu(s))          # the integer path agrees
    assert np.array_equal(bits16(host(Y8)), bits16(host(Y)))


@pytest.mark.parametrize("T,I,O", [(5120, 128, 5120),      # 400 tiles: 144 blocks walk two tiles; one K step
                                   (5120, 256, 5120),      # two K steps
                                   (4100, 384, 7688),      # 527 tiles, ragged on both edges; three K steps
                                   (8192, 512, 6144)])     # 768 tiles = three whole rounds; four K steps
def test_w4a4_linear_fp6_blocks_walk_several_tiles(cq, T, I, O):
    """More output tiles than CUs: a block works through several of them and requests the next tile's first operands
    before it scales and stores the current one (not when the raw accumulators are asked for).  Every output of both
    forms against the oracle, twice in a row into the same buffer."""
    say("w4a4 fp6, several tiles per block: T=%d I=%d O=%d" % (T, I, O))
    qx, qw = int4_codes(T, I, seed=T + 5), int4_codes(O, I, seed=O + 17)
    rng = np.random.default_rng(T + O)
    a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
    s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    px, pw = cq.crossquant_pack_fp6(gpu(nibbles(qx))), cq.crossquant_pack_fp6_weights(gpu(qw))
    ga, gs = gpu(a), gpu(s)
    Y, none_acc = cq.crossquant_w4a4_linear(px, ga, pw, gs, T, I, O)
    assert none_acc is None and np.array_equal(bits16(host(Y)), bits16(Y_ref))
    Y.zero_()
    cq.crossquant_w4a4_linear(px, ga, pw, gs, T, I, O, Y=Y)
    assert np.array_equal(bits16(host(Y)), bits16(Y_ref))
    Y2, acc = cq.crossquant_w4a4_linear(px, ga, pw, gs, T, I, O, want_acc=True)
    assert np.array_equal(host(acc), acc_ref) and np.array_equal(bits16(host(Y2)), bits16(Y_ref))


def test_w4a4_linear_fp6_extreme_accumulators_and_guarded_output(cq):
    """All codes at +-7 over 4096 channels (|acc| = 49 * 4096, exact in binary32), written into a
    window of a larger buffer whose surroundings must stay untouched."""
    import torch
    T, I, O = 70, 4096, 72
    qx = np.full((T, I), 7, np.int8)
    qx[::2] = -7
    qw = np.full((O, I), -7, np.int8)
    qw[::3] = 7
    a = np.full(T, 0.01, np.float32)
    s = np.full(O, 0.001, np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    assert np.abs(acc_ref).max() == 49 * I
    buf = torch.full((T + 5, 96), 7.0, dtype=torch.float16, device="cuda")
    px, pw = cq.crossquant_pack_fp6(gpu(qx)), cq.crossquant_pack_fp6_weights(gpu(qw))
    _, acc = cq.crossquant_w4a4_linear(px, gpu(a), pw, gpu(s), T, I, O, Y=buf[:T, :O], want_acc=True)
    out = host(buf)
    assert np.array_equal(host(acc), acc_ref) and np.array_equal(bits16(out[:T, :O]), bits16(Y_ref))
    assert np.all(out[:T, O:] == 7.0) and np.all(out[T:] == 7.0)


def test_w4a4_linear_fp6_longest_contraction(cq):
    """I = 2^18, the documented limit: |acc| reaches 49 * 2^18 = 12 845 056 < 2^24, still exact."""
    T, I, O = 3, 1 << 18, 8
    qx = np.full((T, I), 7, np.int8)
    qx[1] = -7
    qx[2, ::2] = 3
    qw = np.full((O, I), 7, np.int8)
    qw[1::2] = -7
    qw[3, 5::7] = -2
    a = np.array([1e-6, 2e-6, 3e-6], np.float32)
    s = np.full(O, 1e-3, np.float32)
    Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
    assert np.abs(acc_ref).max() == 49 * I
    px, pw = cq.crossquant_pack_fp6(gpu(qx)), cq.crossquant_pack_fp6_weights(gpu(qw))
    Y, acc = cq.crossquant_w4a4_linear(px, gpu(a), pw, gpu(s), T, I, O, want_acc=True)
    assert np.array_equal(host(acc), acc_ref) and np.array_equal(bits16(host(Y)), bits16(Y_ref))


@pytest.mark.parametrize("T,I", [(1, 128), (32, 128), (45, 256), (300, 640), (257, 1024), (64, 2048)])
def test_quantize_straight_to_fp6(cq, T, I):
    """INT4 CrossQuant codes leaving the quantizer already as FP6 fragments: same bytes as
    quantize (bits = 4) followed by the packing kernel, same zero count, same dequantized matrix."""
    X = outliers(T, I, seed=T * 7 + I)
    Xg = gpu(X)
    t_ref, c_ref = oracle.absmax(X)
    for alpha in (0.15, 1.0):
        ref = oracle.quantize(X, t_ref, c_ref, alpha, 4)
        want = fp6_fragments(oracle.unpack_int4(ref["codes"]))
        t, c = cq.crossquant_absmax(Xg)
        packed, xhat, a, b, zc = cq.crossquant_quantize_fp6(Xg, t, c, alpha, want_xhat=True)
        assert np.array_equal(host(packed), want)
        assert int(host(zc)[0]) == ref["Z"] and np.array_equal(bits16(host(xhat)), bits16(ref["xhat"]))
        assert np.array_equal(bits32(host(a)), bits32(ref["a"])) and np.array_equal(bits32(host(b)), bits32(ref["b"]))
        nib, _, _, _, _ = cq.crossquant_quantize(Xg, t, c, alpha, 4, want_xhat=False)
        assert np.array_equal(host(cq.crossquant_pack_fp6(nib)), want)


def test_end_to_end_a4w4_fp6_config(cq):
    """The low-bit configuration end to end with the FP6 linear layer: CrossQuant INT4 activation
    codes (packed nibbles) and INT4 per-channel weights, compared with the oracle on sampled rows
    and in full with the integer path."""
    import torch
    cfg = workloads.CONFIGS["C4"]
    X, W = workloads.config_activation("C4"), workloads.config_weight("C4")
    t_ref, c_ref = oracle.absmax(X)
    ref = oracle.quantize(X, t_ref, c_ref, 0.15, 4, want_xhat=False)
    qw_ref, s_ref = oracle.weight_quantize(W, ref["b"], 4)
    Xg, Wg = gpu(X), gpu(W)
    t, c = cq.crossquant_absmax(Xg)
    packed, _, a, b, _ = cq.crossquant_quantize(Xg, t, c, 0.15, 4, want_xhat=False)
    qw, s = cq.crossquant_weight_quantize(Wg, b, 4)
    px, pw = cq.crossquant_pack_fp6(packed), cq.crossquant_pack_fp6_weights(qw)
    px_direct, _, a_d, _, _ = cq.crossquant_quantize_fp6(Xg, t, c, 0.15)
    assert torch.equal(px, px_direct) and torch.equal(a, a_d)
    Y, acc = cq.crossquant_w4a4_linear(px, a, pw, s, cfg.T, cfg.I, cfg.O, want_acc=True)
    Y8, acc8 = cq.crossquant_w8a8_linear(cq.crossquant_unpack_int4(packed), a, qw, s, want_acc=True)
    assert torch.equal(acc, acc8) and torch.equal(Y.view(torch.int16), Y8.view(torch.int16))
    rows = np.array([0, 255, 256, 1777, cfg.T - 1])
    Yr, accr = oracle.w8a8_linear(oracle.unpack_int4(ref["codes"])[rows], ref["a"][rows], qw_ref, s_ref)
    assert np.array_equal(host(acc[torch.from_numpy(rows).cuda()]), accr)
    assert np.array_equal(bits16(host(Y[torch.from_numpy(rows).cuda()])), bits16(Yr))


def test_random_shapes_w4a4_fp6(cq):
    """Thirty seeded random shapes for the FP6 linear layer (I a multiple of 128, O of 8, any T),
    including contractions of one, two and three K steps (the pipeline's start-up cases)."""
    rng = np.random.default_rng(8096)
    for case in range(30):
        T = int(rng.integers(1, 700))
        I = 128 * int(rng.integers(1, 13)) if case >= 6 else 128 * (1 + case % 3)
        O = 8 * int(rng.integers(1, 100))
        say("random w4a4 %d: T=%d I=%d O=%d" % (case, T, I, O))
        qx, qw = int4_codes(T, I, seed=9000 + case), int4_codes(O, I, seed=9500 + case)
        a = rng.uniform(1e-3, 1e-1, T).astype(np.float32)
        s = rng.uniform(1e-5, 1e-3, O).astype(np.float32)
        Y_ref, acc_ref = oracle.w8a8_linear(qx, a, qw, s)
        px, pw = cq.crossquant_pack_fp6(gpu(nibbles(qx))), cq.crossquant_pack_fp6_weights(gpu(qw))
        Y, acc = cq.crossquant_w4a4_linear(px, gpu(a), pw, gpu(s), T, I, O, want_acc=True)
        assert np.array_equal(host(acc), acc_ref)
        assert np.array_equal(bits16(host(Y)), bits16(Y_ref))
