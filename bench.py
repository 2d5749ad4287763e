#!/usr/bin/env python3
"""Benchmark of the CrossQuant hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, all resident in HBM:
  absmax (row + column maxima)  ->  quantize (codes + dequantized matrix + zero count)
  ->  kernel count at alpha = 1 (the per-token baseline)  ->  linear layer on the codes
      (W8A8 on the INT8 matrix instruction; the INT4 configuration: A4W4 on the FP6 one).
Weight quantization is weight preparation and happens once, outside the timed region.

Prints one JSON line.  The headline workload is C5 (the 70B-shaped layer): `value` is its
quantizer throughput = algorithmic bytes of absmax + quantize / the sum of the two stage times,
each stage time the MEDIAN over the timed steps of the HIP-event interval around the stage (events
recorded on the stream the kernels run on; they are timing-only events, created with
hipEventDisableSystemFence, so that recording one does not add a system-scope cache release to the
stage it closes -- `with_default_events` repeats the loop with torch.cuda.Event, which does, and shows
the difference).  `roofline` describes the dominant kernel (the GEMM),
`roofline_quantize` the fused quantize kernel.  `event_free` gives the same step timed by the wall
clock with no event in it, with and without the two quantizer calls: what the event packets between
the stages cost can be read off the difference.  `configs` repeats the step loop on the other
configurations (C1-C4), `cpu_baseline` times the CPU oracle on this machine's host cores.
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
STAGES = ("absmax", "quantize", "count", "linear")

# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a plain copy of known size (profiles/bench_hbm_traffic_pmc.txt).  Measured once per
# workload with the commands given in that profile ("linear": the matrix kernel of the workload's linear
# layer; "quantize": its quantize kernel); null for workloads that have not been profiled (C1).
MEASURED_TRAFFIC_BYTES = {
    "C2": {"quantize": (16.4 + 24.0) * 2 ** 20, "linear": (160.5 + 43.0) * 2 ** 20},
    "C3": {"quantize": (40.5 + 60.0) * 2 ** 20, "linear": (600.6 + 160.0) * 2 ** 20},
    "C4": {"quantize": (32.5 + 44.0) * 2 ** 20, "linear": (72.3 + 32.0) * 2 ** 20},
    "C5": {"quantize": (64.5 + 96.1) * 2 ** 20, "linear": (1344.8 + 224.0) * 2 ** 20},
}


class _TimingEvent:
    """A HIP event for timing only, created with hipEventDisableSystemFence: recording it does not make the stream
    perform a system-scope release (a write-back of the caches for the host's benefit), which a default event --
    torch.cuda.Event is one -- adds to whatever it brackets.  Recorded on torch's current stream, the stream the
    library's calls are enqueued on."""
    DISABLE_SYSTEM_FENCE = 0x20000000
    _hip = None

    @classmethod
    def library(cls):
        if cls._hip is None:
            import ctypes
            hip = ctypes.CDLL("libamdhip64.so")          # the runtime torch has loaded already
            vp = ctypes.c_void_p
            hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(vp), ctypes.c_uint]
            hip.hipEventRecord.argtypes = [vp, vp]
            hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), vp, vp]
            hip.hipEventDestroy.argtypes = [vp]
            cls._hip = hip
        return cls._hip

    def __init__(self, torch):
        import ctypes
        self._h = self.library()
        self._e = ctypes.c_void_p()
        self._stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if self._h.hipEventCreateWithFlags(ctypes.byref(self._e), self.DISABLE_SYSTEM_FENCE) != 0:
            raise RuntimeError("hipEventCreateWithFlags failed")

    def record(self):
        if self._h.hipEventRecord(self._e, self._stream) != 0:
            raise RuntimeError("hipEventRecord failed")

    def elapsed_time(self, other):
        import ctypes
        ms = ctypes.c_float()
        if self._h.hipEventElapsedTime(ctypes.byref(ms), self._e, other._e) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value

    def __del__(self):
        try:
            if getattr(self, "_e", None) is not None and self._e.value:
                self._h.hipEventDestroy(self._e)
                self._e = None
        except Exception:                                   # interpreter shutdown: the runtime may be gone already
            pass


EVENT_KINDS = set()     # what make_events handed out in this run, for the JSON line


def make_events(torch, n, timing_only=True):
    """n events for bracketing stages: timing-only HIP events, or torch's default ones (also when the HIP runtime
    cannot be reached through ctypes; the JSON line says which kind was used)."""
    if timing_only:
        try:
            ev = [_TimingEvent(torch) for _ in range(n)]
            EVENT_KINDS.add("hipEventDisableSystemFence")
            return ev
        except (OSError, AttributeError, RuntimeError):
            pass
        EVENT_KINDS.add("torch.cuda.Event (fallback)")
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)      # the part takes ~50 steps (35 ms) to settle into its clocks
    ap.add_argument("--config", default="C5", help="headline workload (C1 ... C5); C5 is the one the metric is quoted on")
    ap.add_argument("--alpha", type=float, default=0.15)
    ap.add_argument("--graph", action="store_true",
                    help="also replay the step from a captured HIP graph and report its time per step")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed step loop of the headline workload: no other configurations, no "
                         "event-free / single-read / warm / calibration / A4W4 / vendor comparisons (the form the "
                         "committed kernel-trace profiles are taken with)")
    ap.add_argument("--no-configs", action="store_true", help="skip the step loops of the other configurations")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the plain read / copy / MFMA-only calibration kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stages", default="all",
                    help="all, or a comma list of absmax,quantize,count,linear (for profiling one stage)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of known size (calibrates HBM byte counters under "
                         "rocprofv3 --pmc) and exit")
    return ap.parse_args()


def median_time(fn, reps):
    """Median wall time of fn() over reps calls, and the value of the last call."""
    import statistics
    ts, out = [], None
    for _ in range(reps):
        t0 = time.perf_counter()
        out = fn()
        ts.append(time.perf_counter() - t0)
    return statistics.median(ts), out


def cpu_baseline(cfg, X, W, alpha):
    """The CPU oracle, as it stands, on the host cores, on a bounded sample of the headline workload: the
    full activation matrix for absmax / quantize / count, a 512-row slab of the linear layer (full I x O)
    scaled to T rows.  Every leg is run three times and the median reported."""
    import oracle
    T, I, O = cfg.T, cfg.I, cfg.O
    reps = 3
    absmax_s, (t, c) = median_time(lambda: oracle.absmax(X), reps)
    quant_s, ref = median_time(lambda: oracle.quantize(X, t, c, alpha, cfg.bits, want_xhat=True), reps)
    count_s, _ = median_time(lambda: oracle.kernel_count(X, t, c, 1.0, cfg.bits), reps)
    slab = min(512, T)
    qw, s = oracle.weight_quantize(W, ref["b"], cfg.bits)
    q_slab = ref["codes"][:slab] if cfg.bits == 8 else oracle.unpack_int4(ref["codes"][:slab])
    lin_slab_s, _ = median_time(lambda: oracle.w8a8_linear(q_slab, ref["a"][:slab], qw, s), reps)
    n = T * I
    q_bytes = 2 * n + (2 + 1 + 2) * n            # absmax read + quantize read/codes/xhat
    lin_time = lin_slab_s * (T / slab)
    # the same quantizer on one thread (the definition as a scalar loop), on a quarter of the rows
    n_thr = oracle.num_threads()
    oracle.set_num_threads(1)
    Xq = X[: max(T // 4, 1)]

    def single():
        t1, c1 = oracle.absmax(Xq)
        oracle.quantize(Xq, t1, c1, alpha, cfg.bits, want_xhat=True)
    single_s, _ = median_time(single, reps)
    oracle.set_num_threads(n_thr)
    return {
        "value": q_bytes / (absmax_s + quant_s) / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "full %dx%d activation for absmax+quantize+count; linear layer on a %d-row slab (full %dx%d "
                  "weights), time scaled by T/%d; every leg the median of %d runs" % (T, I, slab, I, O, slab, reps),
        "absmax_s": absmax_s, "quantize_s": quant_s, "count_s": count_s,
        "linear_s_extrapolated": lin_time, "w8a8_linear_tops": 2.0 * T * I * O / lin_time / 1e12,
        "single_thread_value": 7 * Xq.size / single_s / 1e9,
        "single_thread_sample": "absmax + quantize on the first %d rows, median of %d runs" % (Xq.shape[0], reps),
    }


class Workload:
    """Everything one configuration's step touches, allocated once; `step` enqueues one pass."""

    def __init__(self, name, alpha, stages):
        import torch
        import paper_2410_07505_amd as cq
        import workloads
        self.cq, self.torch = cq, torch
        self.cfg = cfg = workloads.CONFIGS[name]
        self.alpha, self.stages = alpha, stages
        self.bits = bits = cfg.bits     # 8: W8A8 on the INT8 kernel; 4: A4W4 on the FP6 kernel
        T, I, O = cfg.T, cfg.I, cfg.O
        dev = torch.device("cuda:0")
        self.X = workloads.config_activation(name)
        self.W = workloads.config_weight(name)
        self.Xg = torch.from_numpy(self.X).to(dev)
        Wg = torch.from_numpy(self.W).to(dev)
        f32 = lambda n_: torch.empty(n_, dtype=torch.float32, device=dev)
        self.t, self.c, self.a, self.b, self.a_pt, self.b_pt = f32(T), f32(I), f32(T), f32(I), f32(T), f32(I)
        self.codes = (torch.empty((T, I), dtype=torch.int8, device=dev) if bits == 8
                      else torch.empty((T, I // 2), dtype=torch.uint8, device=dev))
        self.xhat = torch.empty((T, I), dtype=torch.float16, device=dev)
        self.zc = torch.zeros(1, dtype=torch.int64, device=dev)
        self.zc_pt = torch.zeros(1, dtype=torch.int64, device=dev)
        self.Y = torch.empty((T, O), dtype=torch.float16, device=dev)
        self.qw = torch.empty((O, I), dtype=torch.int8, device=dev)
        self.ws = f32(O)
        # weight preparation (once): needs the column factors of this activation
        cq.crossquant_absmax(self.Xg, t=self.t, c=self.c)
        cq.crossquant_quantize(self.Xg, self.t, self.c, alpha, bits, codes=self.codes, xhat=self.xhat, row_scale=self.a,
                               col_scale=self.b, zero_count=self.zc)
        cq.crossquant_weight_quantize(Wg, self.b, bits, qw=self.qw, w_scale=self.ws)
        self.px = self.pw = None
        if bits == 4:
            self.pw = cq.crossquant_pack_fp6_weights(self.qw)
            self.px = cq.crossquant_pack_fp6(self.codes)
        torch.cuda.synchronize()
        del Wg

    def quantizer(self):
        cq = self.cq
        cq.crossquant_absmax(self.Xg, t=self.t, c=self.c)
        self.quantize()

    def quantize(self):
        cq = self.cq
        if self.bits == 8:
            cq.crossquant_quantize(self.Xg, self.t, self.c, self.alpha, 8, codes=self.codes, xhat=self.xhat,
                                   row_scale=self.a, col_scale=self.b, zero_count=self.zc)
        else:       # INT4 codes leave the quantizer already in the FP6 kernel's operand format
            cq.crossquant_quantize_fp6(self.Xg, self.t, self.c, self.alpha, packed=self.px, xhat=self.xhat,
                                       row_scale=self.a, col_scale=self.b, zero_count=self.zc)

    def step(self, ev=None, single_read=False, stages=None):
        """single_read: False = the named calls; "call" = crossquant_absmax_quantize; "kernel" = the single-read kernel."""
        cq, cfg = self.cq, self.cfg
        stages = self.stages if stages is None else stages
        if ev is not None:
            ev[0].record()
        if single_read:
            cq.crossquant_absmax_quantize(self.Xg, self.alpha, self.bits, single_read=(single_read == "kernel"),
                                          t=self.t, c=self.c, codes=self.codes, xhat=self.xhat, row_scale=self.a,
                                          col_scale=self.b, zero_count=self.zc)
        elif "absmax" in stages:
            cq.crossquant_absmax(self.Xg, t=self.t, c=self.c)
        if ev is not None:
            ev[1].record()
        if "quantize" in stages and not single_read:
            self.quantize()
        if ev is not None:
            ev[2].record()
        if "count" in stages:
            cq.crossquant_kernel_count(self.Xg, self.t, self.c, 1.0, self.bits, zero_count=self.zc_pt)
        if ev is not None:
            ev[3].record()
        if "linear" in stages:
            if self.bits == 8:
                cq.crossquant_w8a8_linear(self.codes, self.a, self.qw, self.ws, Y=self.Y)
            else:
                cq.crossquant_w4a4_linear(self.px, self.a, self.pw, self.ws, cfg.T, cfg.I, cfg.O, Y=self.Y)
        if ev is not None:
            ev[4].record()

    def timed_steps(self, steps, warmup, timing_only_events=True, **kw):
        """Stage times in ms (median and mean over the steps of each HIP-event interval) and the wall time per step."""
        import numpy as np
        torch = self.torch
        for _ in range(warmup):
            self.step(**kw)
        torch.cuda.synchronize()
        events = [make_events(torch, 5, timing_only_events) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(events[i], **kw)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per = np.array([[ev[s].elapsed_time(ev[s + 1]) for s in range(4)] for ev in events])
        return np.median(per, axis=0), per.mean(axis=0), wall * 1e3 / steps

    def wall_ms_per_step(self, steps, warmup, stages):
        """The step with no event in it, timed by the host clock around `steps` of them."""
        torch = self.torch
        for _ in range(warmup):
            self.step(stages=stages)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(stages=stages)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def figures(self, stage_ms):
        """Rates of one configuration from its stage times (ms)."""
        cfg, bits = self.cfg, self.bits
        T, I, O = cfg.T, cfg.I, cfg.O
        n = T * I
        code_bytes = 1.0 if bits == 8 else 0.75     # int8 codes, or 6-bit fields of the FP6 fragments
        bytes_absmax = 2 * n + 4 * (T + I)
        bytes_quant = (2 + code_bytes + 2) * n + 4 * (T + I)
        ran = {name: (name in self.stages) for name in STAGES}
        ms = {name: (float(stage_ms[i]) if ran[name] else 0.0) for i, name in enumerate(STAGES)}
        quant_gbs = ((bytes_absmax + bytes_quant) / ((ms["absmax"] + ms["quantize"]) * 1e-3) / 1e9
                     if (ran["absmax"] and ran["quantize"]) else None)
        tops = 2.0 * T * I * O / (ms["linear"] * 1e-3) / 1e12 if ran["linear"] else None
        rate = lambda b_, m_: (b_ / (m_ * 1e-3) / 1e9) if m_ > 0 else None
        return {"ms": ms, "quant_gbs": quant_gbs, "tops": tops, "bytes_absmax": bytes_absmax, "bytes_quant": bytes_quant,
                "absmax_gbs": rate(bytes_absmax, ms["absmax"]), "quantize_gbs": rate(bytes_quant, ms["quantize"]),
                "count_gbs": rate(2 * n, ms["count"]), "peak_tops": INT8_PEAK_TOPS if bits == 8 else FP6_PEAK_TOPS}

    def inside_gemm(self, reps=3):
        """The quantize step inside the GEMM's activation load (one call: X -> Y) against the two calls it replaces
        (quantize without the dequantized matrix, then the linear layer), each timed back to back."""
        cq, torch, cfg = self.cq, self.torch, self.cfg
        qw8 = self.qw                       # int8 codes; for the INT4 configuration the codes are in [-7, 7]

        def timed(fn):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        fused_ms = timed(lambda: cq.crossquant_quantize_linear_fused(self.Xg, self.t, self.c, self.alpha, self.bits, qw8,
                                                                     self.ws, Y=self.Y, row_scale=self.a, col_scale=self.b))
        y_fused = self.Y.clone()

        def two_calls():
            if self.bits == 8:
                cq.crossquant_quantize(self.Xg, self.t, self.c, self.alpha, 8, codes=self.codes, want_xhat=False,
                                       row_scale=self.a, col_scale=self.b, want_count=False)
                cq.crossquant_w8a8_linear(self.codes, self.a, qw8, self.ws, Y=self.Y)
            else:
                cq.crossquant_quantize_fp6(self.Xg, self.t, self.c, self.alpha, packed=self.px, row_scale=self.a,
                                           col_scale=self.b, want_count=False)
                cq.crossquant_w4a4_linear(self.px, self.a, self.pw, self.ws, cfg.T, cfg.I, cfg.O, Y=self.Y)
        two_ms = timed(two_calls)
        same = bool(torch.equal(y_fused.view(torch.int16), self.Y.view(torch.int16)))
        return {"one_call_ms": fused_ms, "two_calls_ms": two_ms, "column_tiles": (cfg.O + 255) // 256,
                "slowdown": fused_ms / two_ms, "identical_outputs": same}

    def settle(self, seconds=0.05):
        """Untimed steps for `seconds` of wall time: a loop that starts on an idle part runs slower for its first
        ~35 ms, which is longer than the whole loop of a small configuration."""
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(10):
                self.step()
            self.torch.cuda.synchronize()

    def summary(self, steps, warmup):
        """The per-configuration object of the `configs` section."""
        self.settle()
        med, _, wall_ms = self.timed_steps(steps, warmup)
        f = self.figures(med)
        n = self.cfg.T * self.cfg.I
        lin = "w8a8_linear" if self.bits == 8 else "a4w4_linear_fp6"
        return {
            "workload": "%s: %s" % (self.cfg.name, self.cfg.label), "bits": self.bits, "steps": steps,
            "ms_per_step": wall_ms,
            "stage_ms_median": {"absmax": f["ms"]["absmax"], "quantize": f["ms"]["quantize"],
                                "count_per_token": f["ms"]["count"], lin: f["ms"]["linear"]},
            "quantizer_GBs": f["quant_gbs"], "quantizer_frac_hbm_peak": f["quant_gbs"] / HBM_PEAK_GBS,
            "absmax_GBs": f["absmax_gbs"], "quantize_GBs": f["quantize_gbs"], "count_GBs": f["count_gbs"],
            "linear_TOPs": f["tops"], "linear_peak_TOPs": f["peak_tops"], "linear_frac_peak": f["tops"] / f["peak_tops"],
            "traffic_bytes": MEASURED_TRAFFIC_BYTES.get(self.cfg.name),
            "kernel_proportion": {"crossquant": int(self.zc.item()) / n, "per_token": int(self.zc_pt.item()) / n},
            "quantize_inside_gemm": self.inside_gemm(),
        }

    def release(self):
        for k in list(self.__dict__):
            if k not in ("cfg", "bits", "alpha", "stages", "cq", "torch"):
                delattr(self, k)
        self.torch.cuda.empty_cache()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (value is the one GPU's "
              "throughput)" % args.gpus, file=sys.stderr)
        sys.exit(2)

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

    if not torch.cuda.is_available():
        print("bench.py: no GPU available", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    stages = STAGES if args.stages == "all" else tuple(args.stages.split(","))
    full = args.stages == "all"
    extras = full and not args.no_extras

    wl = Workload(args.config, args.alpha, stages)
    cfg, bits, alpha = wl.cfg, wl.bits, args.alpha
    T, I, O = cfg.T, cfg.I, cfg.O
    n = T * I

    # ---- the timed region: exactly `steps` steps after `warmup` untimed ones
    med, mean, ms_per_step = wl.timed_steps(args.steps, args.warmup)
    f = wl.figures(med)
    f_mean = wl.figures(mean)
    # The same loop with default events (torch.cuda.Event), which make the stream release to system scope at every
    # record: about 1.5 us on each stage that the stage's kernels do not spend.  Reported beside the headline.
    med_d, _, ms_per_step_d = wl.timed_steps(args.steps, min(args.warmup, 3), timing_only_events=False)
    f_d = wl.figures(med_d)
    default_events = {"stage_ms": dict(zip(("absmax", "quantize", "count_per_token", "w8a8_linear"), map(float, med_d))),
                      "ms_per_step": ms_per_step_d, "quantizer_GBs": f_d["quant_gbs"],
                      "quantizer_frac_hbm_peak": (f_d["quant_gbs"] / HBM_PEAK_GBS) if f_d["quant_gbs"] else None,
                      "w8a8_linear_TOPs": f_d["tops"]}
    quant_gbs, tops, mfma_peak = f["quant_gbs"], f["tops"], f["peak_tops"]
    z, z_pt = int(wl.zc.item()), int(wl.zc_pt.item())

    def event_ms(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def median_ms(fn, reps):
        """Median of the calls' own event intervals (each call bracketed by timing-only events), as for the stages."""
        import statistics
        ev = [make_events(torch, 2) for _ in range(reps)]
        for e0, e1 in ev:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        return statistics.median(e0.elapsed_time(e1) for e0, e1 in ev)

    # ---- the same step with no event in it (host clock around the loop), with and without the two
    # quantizer calls: their difference is what absmax + quantize cost inside the step when nothing
    # but kernels is on the stream; `value` keeps the event-bracketed definition.
    event_free = None
    if extras:
        # The linear layer's time drifts by a per cent or two over seconds (it is limited by power), which is as
        # much as the two quantizer calls take: the two loops therefore alternate in short runs, and the figure
        # is the median of the per-round differences.  (The second loop leaves t, c, a, b, codes as the first
        # one wrote them, so the count and the linear layer see the same operands.)
        # Three loops: all stages; without quantize (the count still follows absmax and reads X from the
        # memory-side cache, as in the full step, so the difference is the quantize call alone); without absmax and
        # quantize (here the count reads X cold, which lengthens this loop by a few microseconds: the difference to
        # the full step understates the two calls by that much).
        import statistics
        rounds = 8
        per_round = max(args.steps // rounds, 5)
        alls, no_q, rests = [], [], []
        for _ in range(rounds):
            alls.append(wl.wall_ms_per_step(per_round, 2, STAGES))
            no_q.append(wl.wall_ms_per_step(per_round, 2, ("absmax", "count", "linear")))
            rests.append(wl.wall_ms_per_step(per_round, 2, ("count", "linear")))
        w_all, w_rest = statistics.median(alls), statistics.median(rests)
        d_ms = statistics.median([x - y for x, y in zip(alls, rests)])
        q_ms = statistics.median([x - y for x, y in zip(alls, no_q)])
        event_free = {"ms_per_step_all_stages": w_all, "ms_per_step_without_absmax_quantize": w_rest,
                      "rounds": rounds, "steps_per_round": per_round,
                      "quantize_ms": q_ms,
                      "absmax_plus_quantize_ms": d_ms,
                      "quantizer_GBs": (f["bytes_absmax"] + f["bytes_quant"]) / (d_ms * 1e-3) / 1e9 if d_ms > 0 else None,
                      "with_events_ms_per_step": ms_per_step,
                      "event_bracketed_absmax_plus_quantize_ms": f["ms"]["absmax"] + f["ms"]["quantize"]}

    # ---- the single-call variant of absmax + quantize (same outputs), both inside the same step (X cold:
    # the linear layer has just swept the caches) and back to back (X still in the memory-side cache).
    # It is not part of `value`, which stays on the two named calls.
    def one_call_figures(kind):
        try:
            n_f = max(args.steps // 2, 1)
            med_f, _, _ = wl.timed_steps(n_f, max(args.warmup, 3), single_read=kind)
            z_f = int(wl.zc.item())
            single = lambda: cq.crossquant_absmax_quantize(wl.Xg, alpha, bits, single_read=(kind == "kernel"), t=wl.t,
                                                           c=wl.c, codes=wl.codes, xhat=wl.xhat, row_scale=wl.a,
                                                           col_scale=wl.b, zero_count=wl.zc)
            event_ms(single, 3)
            warm_f = event_ms(single, n_f)
            in_step_ms = float(med_f[0] + med_f[1])
            # one read of X for the single-read kernel, two for the call that enqueues the two kernels
            f_bytes = ((2 if kind == "kernel" else 4) + 1 + 2) * n + 8 * (T + I)
            return {"in_step_ms": in_step_ms, "in_step_algorithmic_GBs": f_bytes / (in_step_ms * 1e-3) / 1e9,
                    "back_to_back_ms": warm_f, "two_call_in_step_ms": f["ms"]["absmax"] + f["ms"]["quantize"],
                    "zero_count_matches": z_f == z}
        except cq.CrossQuantError as e:
            return {"unsupported": str(e)}

    fused = one_call_figures("call") if extras and bits == 8 else None
    single_read = one_call_figures("kernel") if extras and bits == 8 else None

    # the same two quantizer calls back to back (X stays in the memory-side cache): the warm rate
    warm_ms = None
    if extras:
        event_ms(wl.quantizer, 5)
        warm_ms = event_ms(wl.quantizer, max(args.steps // 2, 1))

    # what the device sustains on a plain read, a plain copy and an MFMA-only loop
    achievable = None
    if extras and not args.no_ceilings:
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)       # 1 GiB: far beyond the caches
        big.fill_(1)
        half = 512 << 20
        event_ms(lambda: cq.crossquant_calib_read(big), 2)
        read_ms = event_ms(lambda: cq.crossquant_calib_read(big), 10)
        event_ms(lambda: cq.crossquant_calib_copy(big[:half], big[half:]), 2)
        copy_ms = event_ms(lambda: cq.crossquant_calib_copy(big[:half], big[half:]), 10)
        del big
        mf = {}
        # modes 0, 1: v_mfma_i32_32x32x32_i8 on operands in registers; mode 3: the 16 x 16 x 64 instruction the linear
        # kernel uses; mode 2: that instruction with the code-like operands re-read from LDS every step at the
        # kernel's own ratio, two waves per SIMD -- its inner loop without global loads, barriers and epilogue
        for mode, name, it_ in ((0, "zero_operands", 2000), (1, "code_like_operands", 2000),
                                (3, "code_like_operands_16x16x64", 1000), (2, "code_like_operands_fed_from_lds", 1000)):
            ops_ = cq.crossquant_calib_mfma_i8(it_, mode)
            ms_ = event_ms(lambda: cq.crossquant_calib_mfma_i8(it_, mode), 5)
            mf[name] = ops_ / (ms_ * 1e-3) / 1e12
        f6_it = 1000
        f6_ops = cq.crossquant_calib_mfma_f6(f6_it)
        f6_loop = f6_ops / (event_ms(lambda: cq.crossquant_calib_mfma_f6(f6_it), 5) * 1e-3) / 1e12
        achievable = {
            "hbm_read_GBs": (1 << 30) / (read_ms * 1e-3) / 1e9,
            "hbm_copy_GBs_read_plus_write": 2 * half / (copy_ms * 1e-3) / 1e9,
            "mfma_i8_TOPs": mf,
            "mfma_fp6_TOPs_int4_like_operands_fed_from_lds": f6_loop,
            "quantizer_frac_of_copy": (quant_gbs / (2 * half / (copy_ms * 1e-3) / 1e9)) if quant_gbs else None,
            "w8a8_linear_frac_of_mfma_loop": (tops / mf["code_like_operands_16x16x64"]) if (tops and bits == 8) else None,
            "w8a8_linear_frac_of_lds_fed_mfma_loop": (tops / mf["code_like_operands_fed_from_lds"]) if (tops and bits == 8) else None,
        }

    # The same layer in the paper's W4A4 setting: INT4 codes of the same X and W, multiplied on the
    # FP6 matrix instruction (exact) and, for comparison, unpacked to int8 on the INT8 kernel; and the
    # vendor library's int8 GEMM (torch._int_mm, int32 output, no epilogue) on the same W8A8 codes.
    a4w4 = vendor = None
    if extras and bits == 8:
        ops_linear = 2.0 * T * I * O
        reps = max(args.steps // 4, 1)
        try:
            acc32 = torch.empty((T, O), dtype=torch.int32, device=dev)
            qwt = wl.qw.t()
            vend = lambda: torch._int_mm(wl.codes, qwt, out=acc32)
            event_ms(vend, 3)
            v_ms = median_ms(vend, reps)
            vendor = {"what": "torch._int_mm on the same int8 codes (int32 output, no scale epilogue)", "ms": v_ms,
                      "TOPs": ops_linear / (v_ms * 1e-3) / 1e12, "this_kernel_ms": f["ms"]["linear"]}
            del acc32
        except Exception as e:                      # not every build of the vendor library takes this layout
            vendor = {"unavailable": repr(e)[:200]}
        Wg4 = torch.from_numpy(wl.W).to(dev)
        nib, _, a4, b4, _ = cq.crossquant_quantize(wl.Xg, wl.t, wl.c, alpha, 4, want_xhat=False)
        qw4, ws4 = cq.crossquant_weight_quantize(Wg4, b4, 4)
        del Wg4
        px, pw = cq.crossquant_pack_fp6(nib), cq.crossquant_pack_fp6_weights(qw4)
        q8 = cq.crossquant_unpack_int4(nib)
        event_ms(lambda: cq.crossquant_w4a4_linear(px, a4, pw, ws4, T, I, O, Y=wl.Y), 10)
        fp6_ms = median_ms(lambda: cq.crossquant_w4a4_linear(px, a4, pw, ws4, T, I, O, Y=wl.Y), reps)
        y6 = wl.Y.clone()
        event_ms(lambda: cq.crossquant_w8a8_linear(q8, a4, qw4, ws4, Y=wl.Y), 10)
        i8_ms = median_ms(lambda: cq.crossquant_w8a8_linear(q8, a4, qw4, ws4, Y=wl.Y), reps)
        pack_ms = event_ms(lambda: cq.crossquant_pack_fp6(nib, packed=px), 10)
        a4w4 = {"fp6_ms": fp6_ms, "fp6_TOPs": ops_linear / (fp6_ms * 1e-3) / 1e12, "int8_path_ms": i8_ms,
                "int8_path_TOPs": ops_linear / (i8_ms * 1e-3) / 1e12, "pack_activations_ms": pack_ms,
                "identical_outputs": bool(torch.equal(y6.view(torch.int16), wl.Y.view(torch.int16)))}
        if achievable:
            a4w4["fp6_frac_of_lds_fed_mfma_loop"] = a4w4["fp6_TOPs"] / achievable["mfma_fp6_TOPs_int4_like_operands_fed_from_lds"]
        del px, pw, q8, nib, qw4, y6
        cq.crossquant_w8a8_linear(wl.codes, wl.a, wl.qw, wl.ws, Y=wl.Y)      # leave Y as the W8A8 result

    inside = wl.inside_gemm() if extras else None

    # ---- the calls built beyond the four named ones, on the headline shapes (medians of event intervals, the
    # calls back to back): the kernel-size analysis, weight preparation per channel and per group of 128, and the
    # batched form on 32 sequences of 128 tokens.  GB/s are algorithmic bytes over the call's time.
    next_rows = None
    if extras and bits == 8:
        reps = max(args.steps // 4, 3)
        xrk = torch.empty_like(wl.xhat)
        cnt3 = torch.empty(3, dtype=torch.int64, device=dev)
        an = lambda: cq.crossquant_kernel_analysis(wl.Xg, wl.t, wl.c, alpha, bits, xrk=xrk, counters=cnt3,
                                                   work_vectors=False)
        event_ms(an, 3)
        an_ms = event_ms(an, reps)
        del xrk
        Wg = torch.from_numpy(wl.W).to(dev)
        wq = lambda: cq.crossquant_weight_quantize(Wg, wl.b, bits, qw=wl.qw, w_scale=wl.ws)
        event_ms(wq, 2)
        wq_ms = event_ms(wq, max(reps // 4, 3))
        gs = torch.empty((O, I // 128), dtype=torch.float32, device=dev)
        qg = torch.empty_like(wl.qw)
        wg = lambda: cq.crossquant_weight_quantize_grouped(Wg, wl.b, 128, 4, qw=qg, w_scale=gs)
        event_ms(wg, 2)
        wg_ms = event_ms(wg, max(reps // 4, 3))
        del qg, gs
        wq()                                                    # wl.qw / wl.ws as the step expects them
        del Wg
        Bq, Sq = 32, 128
        X3 = wl.Xg[:Bq * Sq].view(Bq, Sq, I)
        def batched():
            t3, c3 = cq.crossquant_absmax_batched(X3)
            return cq.crossquant_quantize_batched(X3, t3, c3, alpha, bits)
        event_ms(batched, 3)
        b_ms = event_ms(batched, reps)
        nb3 = Bq * Sq * I
        next_rows = {
            "kernel_analysis": {"what": "Remove-Kernel matrix + the three indicator counts, one call", "ms": an_ms,
                                "GBs": 4 * n / (an_ms * 1e-3) / 1e9},
            "weight_quantize": {"what": "per-output-channel INT8 codes of diag(b) W (%d x %d)" % (I, O), "ms": wq_ms,
                                "GBs_3_bytes_per_weight": 3.0 * I * O / (wq_ms * 1e-3) / 1e9},
            "weight_quantize_grouped": {"what": "INT4 codes with one step per group of 128 input channels", "ms": wg_ms,
                                        "GBs_3_bytes_per_weight": 3.0 * I * O / (wg_ms * 1e-3) / 1e9},
            "batched_absmax_quantize": {"what": "[%d][%d][%d] tensor, per-sequence column maxima, two calls incl. their "
                                                "output allocation" % (Bq, Sq, I), "ms": b_ms,
                                        "GBs": 7.0 * nb3 / (b_ms * 1e-3) / 1e9},
        }
    if extras:
        wl.step()                            # leave every buffer as the step writes it

    graph_ms = None
    if args.graph and full:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                wl.step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - tg) * 1e3 / args.steps

    lin_name = "w8a8_linear" if bits == 8 else "a4w4_linear"
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
        "stage_time_statistic": "median over the timed steps of each stage's HIP-event interval",
        "stage_events": ("timing-only HIP events (hipEventDisableSystemFence) on the launch stream; the same loop with "
                         "default events is under with_default_events"),
        "with_default_events": default_events,
        "stage_ms": {"absmax": f["ms"]["absmax"], "quantize": f["ms"]["quantize"], "count_per_token": f["ms"]["count"],
                     lin_name: f["ms"]["linear"]},
        "stage_ms_mean": {"absmax": f_mean["ms"]["absmax"], "quantize": f_mean["ms"]["quantize"],
                          "count_per_token": f_mean["ms"]["count"], lin_name: f_mean["ms"]["linear"]},
        "stage_rate": {"absmax_GBs": f["absmax_gbs"], "quantize_GBs": f["quantize_gbs"], "count_GBs": f["count_gbs"]},
        "kernel_proportion": {"crossquant": z / n, "per_token": z_pt / n},
        "event_free": event_free,
        "absmax_quantize_single_call": fused,
        "absmax_quantize_single_read": single_read,
        "graph_replay_ms_per_step": graph_ms,
        "quantizer_warm": {"ms": warm_ms, "GBs": (f["bytes_absmax"] + f["bytes_quant"]) / (warm_ms * 1e-3) / 1e9} if warm_ms else None,
        "achievable": achievable,
        "vendor_int8_gemm": vendor,
        "quantize_inside_gemm": inside,
        "next_rows": next_rows,
        "a4w4_linear": a4w4,
        "roofline": {"kernel": ("gemm_i8_ring_kernel (W8A8 linear)" if bits == 8 else
                                "gemm_f6_ring_kernel (A4W4 linear)"),
                     "bound": "mfma", "achieved": tops, "peak": mfma_peak, "unit": "TOP/s",
                     "frac": tops / mfma_peak if tops else None,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("linear")},
        "roofline_quantize": {"kernel": "quantize_stream_kernel (scale factors + codes + xhat + zero count)",
                              "bound": "hbm", "achieved": f["quantize_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": (f["quantize_gbs"] / HBM_PEAK_GBS) if f["quantize_gbs"] else None,
                              "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("quantize")},
    }

    X_head, W_head = wl.X, wl.W
    # ---- the other configurations: the same step loop (parity cases for the tests, bench lines here so
    # that every shape's rates are on record); fewer steps each, the headline stays the long run
    if extras and not args.no_configs:
        wl.release()
        out["configs"] = {}
        for name in ("C1", "C2", "C3", "C4", "C5"):
            if name == cfg.name:
                continue
            w2 = Workload(name, alpha, STAGES)
            out["configs"][name] = w2.summary(min(args.steps, 100), min(args.warmup, 10))
            w2.release()
            del w2

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, X_head, W_head, alpha)
    out["stage_event_kinds"] = sorted(EVENT_KINDS)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
