#!/usr/bin/env python3
"""Benchmark of the CrossQuant hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, all resident in HBM:
  absmax (row + column maxima)  ->  quantize (codes + dequantized matrix + zero count)
  ->  kernel count at alpha = 1 (the per-token baseline)  ->  W8A8 linear (INT8 MFMA GEMM).
Weight quantization is weight preparation and happens once, outside the timed region.

Prints one JSON line.  `value` is the quantizer's throughput (absmax + quantize stages:
algorithmic bytes / summed stage time); the W8A8 linear's TOPS is reported beside it.  The
`roofline` object describes the dominant kernel (the GEMM); `roofline_quantize` the fused
quantize kernel.  Stage times come from HIP events recorded on the stream the kernels run on.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense INT8 MFMA, published (5.0 POP/s)
FP6_PEAK_TOPS = 10100.0      # MI355X dense FP6 / FP4 MFMA, published (10.1 PFLOP/s): the A4W4 path
METRIC = "CrossQuant quantize GB/s (% HBM peak) + W8A8 linear TOPS (% INT8 MFMA peak)"

# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain copy of known size (profiles/bench_c5_hbm_traffic_pmc.txt).  Measured
# once per workload; null for workloads that have not been profiled.
MEASURED_TRAFFIC_BYTES = {
    "C5": {"gemm": (1344.9 + 224.0) * 2 ** 20, "quantize": (64.4 + 96.1) * 2 ** 20},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="C5", help="workload: C2, C3 or C5 (INT8 configurations)")
    ap.add_argument("--alpha", type=float, default=0.15)
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a captured HIP graph and report its time per step")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed step loop: no single-read / warm / calibration / A4W4 comparisons "
                         "(the form the committed profiles are taken with)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the plain read / copy / MFMA-only calibration kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stages", default="all",
                    help="all, or a comma list of absmax,quantize,count,linear (for profiling one stage)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of known size (calibrates HBM byte counters under "
                         "rocprofv3 --pmc) and exit")
    return ap.parse_args()


def cpu_baseline(cfg, X, W, alpha):
    """The CPU oracle, as it stands, timed on the host cores on a bounded sample of the same
    workload: the full activation matrix for absmax / quantize / count, a 2048-row slab of the
    linear layer (full I x O) scaled to T rows."""
    import numpy as np
    import oracle
    T, I, O = cfg.T, cfg.I, cfg.O
    t0 = time.perf_counter()
    t, c = oracle.absmax(X)
    t1 = time.perf_counter()
    ref = oracle.quantize(X, t, c, alpha, cfg.bits, want_xhat=True)
    t2 = time.perf_counter()
    oracle.kernel_count(X, t, c, 1.0, cfg.bits)
    t3 = time.perf_counter()
    slab = min(2048, T)
    Wslab_cols = O
    qw, s = oracle.weight_quantize(W[:, :Wslab_cols], ref["b"], cfg.bits)
    t4 = time.perf_counter()
    oracle.w8a8_linear(ref["codes"][:slab], ref["a"][:slab], qw, s)
    t5 = time.perf_counter()
    n = T * I
    q_bytes = 2 * n + (2 + 1 + 2) * n            # absmax read + quantize read/codes/xhat
    q_time = (t1 - t0) + (t2 - t1)
    lin_time = (t5 - t4) * (T / slab)
    # the same quantizer on one thread (the definition as a scalar loop), on a quarter of the rows
    n_thr = oracle.num_threads()
    oracle.set_num_threads(1)
    Xq = X[: max(T // 4, 1)]
    s0 = time.perf_counter()
    t1t, c1t = oracle.absmax(Xq)
    oracle.quantize(Xq, t1t, c1t, alpha, cfg.bits, want_xhat=True)
    s1 = time.perf_counter()
    oracle.set_num_threads(n_thr)
    single_gbs = 7 * Xq.size / (s1 - s0) / 1e9
    return {
        "value": q_bytes / q_time / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "full %dx%d activation for absmax+quantize+count; linear layer on a %d-row slab "
                  "(full %dx%d weights), time scaled by T/%d" % (T, I, slab, I, O, slab),
        "absmax_s": t1 - t0, "quantize_s": t2 - t1, "count_s": t3 - t2,
        "linear_s_extrapolated": lin_time, "w8a8_linear_tops": 2.0 * T * I * O / lin_time / 1e12,
        "single_thread_value": single_gbs, "single_thread_sample": "absmax + quantize on the first %d rows" % Xq.shape[0],
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (value is the one GPU's "
              "throughput)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.copy_calibration:
        # 20 copies of a 256 MiB buffer: reads 256 MiB and writes 256 MiB per launch
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 256 << 20, "bytes_written": 256 << 20, "launches": 20}}))
        return

    import paper_2410_07505_amd as cq     # raises if libcrossquant.so is missing: no fallback
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU available", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = workloads.CONFIGS[args.config]
    bits = cfg.bits                 # 8: W8A8 on the INT8 kernel; 4: A4W4 on the FP6 kernel (codes packed per step)
    T, I, O = cfg.T, cfg.I, cfg.O
    alpha = args.alpha
    stages = ("absmax", "quantize", "count", "linear") if args.stages == "all" else tuple(args.stages.split(","))

    X = workloads.config_activation(args.config)
    W = workloads.config_weight(args.config)
    Xg = torch.from_numpy(X).to(dev)
    Wg = torch.from_numpy(W).to(dev)

    # every buffer the step touches is allocated here, once
    t = torch.empty(T, dtype=torch.float32, device=dev)
    c = torch.empty(I, dtype=torch.float32, device=dev)
    a = torch.empty(T, dtype=torch.float32, device=dev)
    b = torch.empty(I, dtype=torch.float32, device=dev)
    a_pt = torch.empty(T, dtype=torch.float32, device=dev)
    b_pt = torch.empty(I, dtype=torch.float32, device=dev)
    codes = (torch.empty((T, I), dtype=torch.int8, device=dev) if bits == 8
             else torch.empty((T, I // 2), dtype=torch.uint8, device=dev))
    xhat = torch.empty((T, I), dtype=torch.float16, device=dev)
    zc = torch.zeros(1, dtype=torch.int64, device=dev)
    zc_pt = torch.zeros(1, dtype=torch.int64, device=dev)
    Y = torch.empty((T, O), dtype=torch.float16, device=dev)
    qw = torch.empty((O, I), dtype=torch.int8, device=dev)
    ws = torch.empty(O, dtype=torch.float32, device=dev)

    # weight preparation (once): needs the column factors of this activation
    cq.crossquant_absmax(Xg, t=t, c=c)
    cq.crossquant_quantize(Xg, t, c, alpha, bits, codes=codes, xhat=xhat, row_scale=a, col_scale=b, zero_count=zc)
    cq.crossquant_weight_quantize(Wg, b, bits, qw=qw, w_scale=ws)
    px = pw = None
    if bits == 4:
        pw = cq.crossquant_pack_fp6(qw)
        px = cq.crossquant_pack_fp6(codes)
    torch.cuda.synchronize()
    del Wg

    def step(ev=None, single_read=False):
        if ev is not None:
            ev[0].record()
        if single_read:
            cq.crossquant_absmax_quantize(Xg, alpha, bits, t=t, c=c, codes=codes, xhat=xhat, row_scale=a,
                                          col_scale=b, zero_count=zc)
        elif "absmax" in stages:
            cq.crossquant_absmax(Xg, t=t, c=c)
        if ev is not None:
            ev[1].record()
        if "quantize" in stages and not single_read:
            if bits == 8:
                cq.crossquant_quantize(Xg, t, c, alpha, 8, codes=codes, xhat=xhat, row_scale=a, col_scale=b,
                                       zero_count=zc)
            else:       # INT4 codes leave the quantizer already in the FP6 kernel's operand format
                cq.crossquant_quantize_fp6(Xg, t, c, alpha, packed=px, xhat=xhat, row_scale=a, col_scale=b,
                                           zero_count=zc)
        if ev is not None:
            ev[2].record()
        if "count" in stages:
            cq.crossquant_kernel_count(Xg, t, c, 1.0, bits, row_scale=a_pt, col_scale=b_pt, zero_count=zc_pt)
        if ev is not None:
            ev[3].record()
        if "linear" in stages:
            if bits == 8:
                cq.crossquant_w8a8_linear(codes, a, qw, ws, Y=Y)
            else:
                cq.crossquant_w4a4_linear(px, a, pw, ws, T, I, O, Y=Y)
        if ev is not None:
            ev[4].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    stage_ms = np.zeros(4)
    for ev in events:
        for s_ in range(4):
            stage_ms[s_] += ev[s_].elapsed_time(ev[s_ + 1])
    stage_ms /= args.steps
    ms_per_step = wall * 1e3 / args.steps

    n = T * I
    bytes_absmax = 2 * n + 4 * (T + I)
    code_bytes = 1.0 if bits == 8 else 0.75     # int8 codes, or 6-bit fields of the FP6 fragments
    bytes_quant = (2 + code_bytes + 2) * n + 4 * (T + I)
    bytes_count = 2 * n
    ops_linear = 2.0 * T * I * O
    # a stage that was switched off (--stages) only measures the gap between two event records
    ran = {name: (name in stages) for name in ("absmax", "quantize", "count", "linear")}
    for idx, name in enumerate(("absmax", "quantize", "count", "linear")):
        if not ran[name]:
            stage_ms[idx] = 0.0
    quant_gbs = (bytes_absmax + bytes_quant) / ((stage_ms[0] + stage_ms[1]) * 1e-3) / 1e9 \
        if (ran["absmax"] and ran["quantize"]) else None
    tops = ops_linear / (stage_ms[3] * 1e-3) / 1e12 if ran["linear"] else None
    mfma_peak = INT8_PEAK_TOPS if bits == 8 else FP6_PEAK_TOPS

    z, z_pt = int(zc.item()), int(zc_pt.item())

    # The single-read variant of absmax + quantize (same outputs), timed after the main loop, both
    # inside the same step (X cold: the linear layer has just swept the caches) and back to back
    # (X still in the Infinity Cache).  It is not part of `value`, which stays on the two named calls.
    fused = None
    if args.stages == "all" and not args.no_extras and bits == 8:
        try:
            for _ in range(max(args.warmup, 3)):
                step(single_read=True)
            torch.cuda.synchronize()
            n_f = max(args.steps // 2, 1)
            ev_f = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_f)]
            for i in range(n_f):
                step(ev_f[i], single_read=True)
            torch.cuda.synchronize()
            in_step_ms = sum(ev[0].elapsed_time(ev[2]) for ev in ev_f) / n_f
            z_f = int(zc.item())
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n_f):
                cq.crossquant_absmax_quantize(Xg, alpha, bits, t=t, c=c, codes=codes, xhat=xhat, row_scale=a,
                                              col_scale=b, zero_count=zc)
            e1.record()
            torch.cuda.synchronize()
            warm_ms = e0.elapsed_time(e1) / n_f
            f_bytes = (2 + code_bytes + 2) * n + 8 * (T + I)
            fused = {"in_step_ms": in_step_ms, "in_step_algorithmic_GBs": f_bytes / (in_step_ms * 1e-3) / 1e9,
                     "back_to_back_ms": warm_ms, "two_call_in_step_ms": float(stage_ms[0] + stage_ms[1]),
                     "zero_count_matches": z_f == z}
        except cq.CrossQuantError as e:
            fused = {"unsupported": str(e)}

    def event_ms(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # the same two quantizer calls back to back (X stays in the memory-side cache): the warm rate
    warm_ms = None
    if ran["absmax"] and ran["quantize"] and not args.no_extras:
        def quantizer():
            cq.crossquant_absmax(Xg, t=t, c=c)
            if bits == 8:
                cq.crossquant_quantize(Xg, t, c, alpha, 8, codes=codes, xhat=xhat, row_scale=a, col_scale=b,
                                       zero_count=zc)
            else:
                cq.crossquant_quantize_fp6(Xg, t, c, alpha, packed=px, xhat=xhat, row_scale=a, col_scale=b,
                                           zero_count=zc)
        event_ms(quantizer, 5)
        warm_ms = event_ms(quantizer, max(args.steps // 2, 1))

    # what the device sustains on a plain read, a plain copy and an MFMA-only loop
    achievable = None
    if not args.no_ceilings and not args.no_extras:
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)       # 1 GiB: far beyond the caches
        big.fill_(1)
        half = 512 << 20
        event_ms(lambda: cq.crossquant_calib_read(big), 2)
        read_ms = event_ms(lambda: cq.crossquant_calib_read(big), 10)
        event_ms(lambda: cq.crossquant_calib_copy(big[:half], big[half:]), 2)
        copy_ms = event_ms(lambda: cq.crossquant_calib_copy(big[:half], big[half:]), 10)
        del big
        mf = {}
        for mode, name in ((0, "zero_operands"), (1, "code_like_operands")):
            ops_ = cq.crossquant_calib_mfma_i8(2000, mode)
            ms_ = event_ms(lambda: cq.crossquant_calib_mfma_i8(2000, mode), 5)
            mf[name] = ops_ / (ms_ * 1e-3) / 1e12
        achievable = {
            "hbm_read_GBs": (1 << 30) / (read_ms * 1e-3) / 1e9,
            "hbm_copy_GBs_read_plus_write": 2 * half / (copy_ms * 1e-3) / 1e9,
            "mfma_i8_TOPs": mf,
            "quantizer_frac_of_copy": (quant_gbs / (2 * half / (copy_ms * 1e-3) / 1e9)) if quant_gbs else None,
            "w8a8_linear_frac_of_mfma_loop": (tops / mf["code_like_operands"]) if (tops and bits == 8) else None,
        }

    # The same layer in the paper's W4A4 setting: INT4 codes of the same X and W, multiplied on the
    # FP6 matrix instruction (exact) and, for comparison, unpacked to int8 on the INT8 kernel.
    a4w4 = None
    if args.stages == "all" and not args.no_extras and bits == 8:
        Wg4 = torch.from_numpy(W).to(dev)
        nib, _, a4, b4, _ = cq.crossquant_quantize(Xg, t, c, alpha, 4, want_xhat=False)
        qw4, ws4 = cq.crossquant_weight_quantize(Wg4, b4, 4)
        del Wg4
        px, pw = cq.crossquant_pack_fp6(nib), cq.crossquant_pack_fp6(qw4)
        q8 = cq.crossquant_unpack_int4(nib)
        event_ms(lambda: cq.crossquant_w4a4_linear(px, a4, pw, ws4, T, I, O, Y=Y), 10)
        fp6_ms = event_ms(lambda: cq.crossquant_w4a4_linear(px, a4, pw, ws4, T, I, O, Y=Y), max(args.steps // 4, 1))
        y6 = Y.clone()
        event_ms(lambda: cq.crossquant_w8a8_linear(q8, a4, qw4, ws4, Y=Y), 10)
        i8_ms = event_ms(lambda: cq.crossquant_w8a8_linear(q8, a4, qw4, ws4, Y=Y), max(args.steps // 4, 1))
        pack_ms = event_ms(lambda: cq.crossquant_pack_fp6(nib, packed=px), 10)
        a4w4 = {"fp6_ms": fp6_ms, "fp6_TOPs": ops_linear / (fp6_ms * 1e-3) / 1e12, "int8_path_ms": i8_ms,
                "int8_path_TOPs": ops_linear / (i8_ms * 1e-3) / 1e12, "pack_activations_ms": pack_ms,
                "identical_outputs": bool(torch.equal(y6.view(torch.int16), Y.view(torch.int16)))}
        del px, pw, q8, nib, qw4, y6
        cq.crossquant_w8a8_linear(codes, a, qw, ws, Y=Y)      # leave Y as the W8A8 result

    graph_ms = None
    if args.graph and args.stages == "all":
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg) * 1e3 / args.steps

    out = {
        "metric": METRIC,
        "value": quant_gbs, "unit": "GB/s",
        "quantize_frac_hbm_peak": quant_gbs / HBM_PEAK_GBS if quant_gbs else None,
        "w8a8_linear_tops": tops if bits == 8 else None,
        "w8a8_linear_frac_int8_peak": (tops / INT8_PEAK_TOPS) if (tops and bits == 8) else None,
        "a4w4_linear_tops": tops if bits == 4 else None,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("fp16 in, fp32 scale arithmetic, int8 codes, int32 accumulate" if bits == 8 else
                  "fp16 in, fp32 scale arithmetic, int4 codes as fp6 (exact), fp32 accumulate (exact)"),
        "data": "synthetic (seeded N(0,1) activations with outlier channels, N(0,0.02) weights)",
        "config": {"workload": "%s: %s" % (cfg.name, cfg.label), "T": T, "I": I, "O": O, "bits": bits,
                   "alpha": alpha, "stages": list(stages)},
        "stage_ms": {"absmax": stage_ms[0], "quantize": stage_ms[1], "count_per_token": stage_ms[2],
                     ("w8a8_linear" if bits == 8 else "a4w4_linear"): stage_ms[3]},
        "stage_rate": {
            "absmax_GBs": bytes_absmax / (stage_ms[0] * 1e-3) / 1e9 if stage_ms[0] > 0 else None,
            "quantize_GBs": bytes_quant / (stage_ms[1] * 1e-3) / 1e9 if stage_ms[1] > 0 else None,
            "count_GBs": bytes_count / (stage_ms[2] * 1e-3) / 1e9 if stage_ms[2] > 0 else None,
        },
        "kernel_proportion": {"crossquant": z / n, "per_token": z_pt / n},
        "absmax_quantize_single_read": fused,
        "graph_replay_ms_per_step": graph_ms,
        "quantizer_warm": {"ms": warm_ms, "GBs": (bytes_absmax + bytes_quant) / (warm_ms * 1e-3) / 1e9} if warm_ms else None,
        "achievable": achievable,
        "a4w4_linear": a4w4,
        "roofline": {"kernel": ("gemm_i8_ring_kernel (W8A8 linear)" if bits == 8 else
                                "gemm_f6_ring_kernel (A4W4 linear)"),
                     "bound": "mfma", "achieved": tops, "peak": mfma_peak, "unit": "TOP/s",
                     "frac": tops / mfma_peak if tops else None,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("gemm")},
        "roofline_quantize": {"kernel": "quantize_kernel (scale factors + codes + xhat + zero count)",
                              "bound": "hbm",
                              "achieved": bytes_quant / (stage_ms[1] * 1e-3) / 1e9 if stage_ms[1] > 0 else None,
                              "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": (bytes_quant / (stage_ms[1] * 1e-3) / 1e9 / HBM_PEAK_GBS)
                              if stage_ms[1] > 0 else None,
                              "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("quantize")},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, X, W, alpha)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
