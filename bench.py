#!/usr/bin/env python3
"""Benchmark of the MXFP4 linear-layer hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input: for the
Llama-3.1-8B fused QKV projection (M=8192 tokens, K=4096, N=6144) the three training GEMMs
Fprop, Dgrad and Wgrad, each preceded by the deterministic 32-point Hadamard rotation and the
MXFP4 quantisation of both operands.  The timed step is the training pair mxfp4_linear_fwd_save +
mxfp4_linear_bwd_saved: X, W and dY are each read once and quantised along both axes (2 quantiser
launches, X and W sharing one, producing the 6 quantised operands; 3 GEMM launches).  The same work through
mxfp4_linear_fwd + mxfp4_linear_bwd (5 quantiser launches) is timed as well and reported as
`separate_calls_ms_per_step`.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` = 3 * 2*M*N*K flop / step time, i.e. GEMM TFLOP/s including the
rotation and quantisation time; the timed region of `--steps` steps is repeated 7 times after the warm-up
and the median repetition is reported (minimum and maximum beside it), after the per-kernel legs have
already run, so that clocks still ramping at the start of the process cannot move it.  `roofline` describes
the dominant kernel (the FP4 GEMM) against the dense MXFP4 MFMA peak, with the shader clock sampled
during a sustained run of that kernel; `quantizer` the fused rotate+quantise kernels against peak
HBM bandwidth (measured on a rotation of buffers larger than the 256 MB last-level cache), for no
rotation, H16 and H32; `configs` the totals of the other four benchmark configurations;
`cpu_baseline` the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

M, K, N = 8192, 4096, 6144
PEAK_FP4_TFLOPS = 10100.0  # MI355X dense MXFP4 MFMA peak
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E peak
BYTES_PER_ELEM = 2.0 + 0.5 + 1.0 / 32.0  # bf16 read + packed codes + scale byte per element
BYTES_PER_ELEM_DUAL = 2.0 + 2 * (0.5 + 1.0 / 32.0)  # one read, both quantisations written

# Bytes crossing the L2's outward port in one launch of the step's longest kernel (Dgrad and Wgrad side by side):
# not measured in this run but taken from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised in the file named
# below (FETCH_SIZE x 2.0 after calibration against a 256 MiB copy): 421.23 MiB read + 160.01 MiB written.  They
# include what the 256 MB Infinity Cache serves.
GEMM_TRAFFIC_BYTES = 609.5e6
GEMM_TRAFFIC_SOURCE = "profiles/qkv_traffic_counters.md"
# operands once + outputs once: Dgrad (dY and W^T quantised, dX bf16) + Wgrad (dY^T and X^T quantised, dW fp32)
GEMM_ALGORITHMIC_BYTES = (M * N + K * N) * 0.53125 + M * K * 2 + (N * M + K * M) * 0.53125 + N * K * 4
REPEATS = 7  # repetitions of the timed region; the median is reported


def event_time_ms(fn, iters, torch):
    """Average duration of fn() in ms measured with events on the current stream."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


class ClockSampler:
    """Samples the shader clock (MHz) and the socket power (W) from sysfs a few times a second in a thread while
    a leg runs (the boxes do not let an ordinary user pin clocks, so the clock the kernel actually ran at is
    reported beside the spec-peak fraction)."""

    def __init__(self, period_s=0.05):
        import glob
        self.period = period_s
        self.sclk_files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.power_files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average") +
                                  glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.sclk, self.power = [], []
        self._stop = False
        self._th = None

    def _read(self):
        try:
            for line in open(self.sclk_files[0]):
                if line.rstrip().endswith("*"):
                    self.sclk.append(float(line.split(":")[1].strip().rstrip("*").strip().lower().replace("mhz", "")))
        except Exception:
            pass
        try:
            self.power.append(float(open(self.power_files[0]).read()) * 1e-6)
        except Exception:
            pass

    def __enter__(self):
        import threading

        def loop():
            while not self._stop:
                self._read()
                time.sleep(self.period)
        self._th = threading.Thread(target=loop, daemon=True)
        self._th.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._th.join()

    @staticmethod
    def _median(v):
        v = sorted(v)
        return v[len(v) // 2] if v else None

    def summary(self):
        return {"sclk_mhz_median": self._median(self.sclk), "sclk_mhz_min": min(self.sclk) if self.sclk else None,
                "sclk_mhz_max": max(self.sclk) if self.sclk else None, "samples": len(self.sclk),
                "power_w_median": self._median(self.power)}


def power_probe(args, torch, mx) -> int:
    """Shader clock and socket power while the tiled GEMM runs back to back on the headline shape, for operand
    codes that are (a) all zero, (b) uniformly random bytes, (c) the quantised N(0,1) / N(0,0.02) tensors of the
    benchmark: plain text, one block per case (the evidence behind `frac_at_measured_clock`)."""
    from paper_2605_09825_amd import synth
    dev = torch.device("cuda:0")
    Ra, Rb, C = M, N, K
    out = torch.empty((Ra, Rb), dtype=torch.bfloat16, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)

    def operands(kind):
        if kind == "zero codes":
            aq = torch.zeros((Ra, C // 2), dtype=torch.uint8, device=dev)
            bq = torch.zeros((Rb, C // 2), dtype=torch.uint8, device=dev)
        elif kind == "random codes":
            aq = torch.randint(0, 256, (Ra, C // 2), dtype=torch.uint8, device=dev, generator=gen)
            bq = torch.randint(0, 256, (Rb, C // 2), dtype=torch.uint8, device=dev, generator=gen)
        else:
            x = synth.normal(Ra, C, 1.0, 0, synth.STREAM_X).to(dev)
            w = synth.normal(Rb, C, 0.02, 0, synth.STREAM_W).to(dev)
            aq, as_ = mx.mxfp4_quantize(x, mx.AXIS_LAST, mx.HAD_DET)
            bq, bs = mx.mxfp4_quantize(w, mx.AXIS_LAST, mx.HAD_DET)
            return aq, as_, bq, bs
        as_ = torch.full((Ra, C // 32), 127, dtype=torch.uint8, device=dev)
        bs = torch.full((Rb, C // 32), 127, dtype=torch.uint8, device=dev)
        return aq, as_, bq, bs

    print(f"# tiled MXFP4 GEMM {Ra} x {Rb} x {C}, bf16 out, back-to-back launches for {args.probe_seconds} s per case;")
    print("# shader clock from pp_dpm_sclk, socket power from hwmon, one sample every 50 ms")
    for kind in ("zero codes", "random codes", "quantised benchmark tensors (H32, RNE)"):
        aq, as_, bq, bs = operands(kind)
        for _ in range(50):
            mx.mxfp4_gemm(aq, as_, bq, bs, out=out, out_dtype=mx.OUT_BF16)
        torch.cuda.synchronize()
        n = 0
        with ClockSampler() as cs:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            t0 = time.perf_counter()
            while time.perf_counter() - t0 < args.probe_seconds:
                for _ in range(200):
                    mx.mxfp4_gemm(aq, as_, bq, bs, out=out, out_dtype=mx.OUT_BF16)
                torch.cuda.synchronize()
                n += 200
            e1.record()
            e1.synchronize()
        us = e0.elapsed_time(e1) / n * 1e3
        tf = 2.0 * Ra * Rb * C / us / 1e6
        c = cs.summary()
        sclk = c["sclk_mhz_median"]
        at_clock = tf / (PEAK_FP4_TFLOPS * sclk / 2400.0) if sclk else float("nan")
        print(f"{kind}: {us:.1f} us per GEMM = {tf:.0f} TFLOP/s = {tf / PEAK_FP4_TFLOPS:.3f} of the 10.1 PFLOP/s peak; "
              f"sclk median {sclk} MHz (min {c['sclk_mhz_min']}, max {c['sclk_mhz_max']}, {c['samples']} samples), "
              f"power median {c['power_w_median']} W; fraction of the peak at that clock {at_clock:.3f}")
        k = max(1, len(cs.sclk) // 12)
        print("    sclk MHz:", " ".join(f"{v:.0f}" for v in cs.sclk[::k]))
        print("    power W: ", " ".join(f"{v:.0f}" for v in cs.power[::k]))
    return 0


def other_config(args, torch, mx, synth, emit=True):
    """Timing of the benchmark configurations other than the headline one (1, 3, 4, 5): one JSON line each,
    same conventions (inputs resident, rotation and quantisation inside the timed region)."""
    dev = torch.device("cuda:0")

    def time_calls(fn):
        for _ in range(max(args.warmup // 5, 3)):
            fn()
        torch.cuda.synchronize()
        n = max(args.steps // 10, 5)
        reps = []
        for _ in range(3):  # median of three repetitions of the timed region
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            reps.append((time.perf_counter() - t0) * 1e3 / n)
        return sorted(reps)[1]

    def layer(Ml, Kl, Nl, had, rnd, x, w, dy, stages="fdw"):
        cfg = mx.make_cfg(had, rnd, 2024, y_dtype=mx.OUT_BF16, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32)
        ws_f = torch.empty(mx.mxfp4_linear_workspace_bytes(Ml, Nl, Kl, cfg, False), dtype=torch.uint8, device=dev)
        ws_b = torch.empty(mx.mxfp4_linear_workspace_bytes(Ml, Nl, Kl, cfg, True), dtype=torch.uint8, device=dev)
        y = torch.empty((Ml, Nl), dtype=torch.bfloat16, device=dev)
        dx = torch.empty((Ml, Kl), dtype=torch.bfloat16, device=dev)
        dw = torch.empty((Nl, Kl), dtype=torch.float32, device=dev)
        if stages == "f":
            return time_calls(lambda: mx.mxfp4_linear_fwd(x, w, cfg, y=y, workspace=ws_f)), 1
        if stages == "w":
            return time_calls(lambda: mx.mxfp4_linear_bwd(dy, x, None, cfg, dw=dw, need_dx=False, workspace=ws_b)), 1
        saved = torch.empty(mx.mxfp4_linear_saved_bytes(Ml, Nl, Kl), dtype=torch.uint8, device=dev)

        def both():
            mx.mxfp4_linear_fwd_save(x, w, cfg, y=y, workspace=ws_f, saved=saved)
            mx.mxfp4_linear_bwd_saved(dy, saved, Kl, cfg, dx=dx, dw=dw, workspace=ws_b)
        return time_calls(both), 3

    rows = []
    if args.config == 1:
        x = synth.normal(256, 512, 1.0, 0, synth.STREAM_X).to(dev)
        w = synth.normal(512, 512, 0.02, 0, synth.STREAM_W).to(dev)
        ms, g = layer(256, 512, 512, mx.HAD_NONE, mx.RNE, x, w, None, "f")
        rows.append(("fprop 256x512x512 no-H RNE", ms, g * 2.0 * 256 * 512 * 512))
        workload = "config 1: single linear Fprop, M=256 K=512 N=512, no rotation, RNE (launch-latency bound)"
    elif args.config == 3:
        for name, Kl, Nl, sd in (("gate/up", 4096, 28672, 0), ("down", 14336, 4096, 1)):
            x = synth.normal_with_outlier_channels(8192, Kl, sd, synth.STREAM_X).to(dev)
            w = synth.normal(Nl, Kl, 0.02, sd, synth.STREAM_W).to(dev)
            dy = synth.normal(8192, Nl, 1e-3, sd, synth.STREAM_DY).to(dev)
            for had, hn in ((mx.HAD_DET, "H32"), (mx.HAD_NONE, "no-H")):
                ms, g = layer(8192, Kl, Nl, had, mx.RNE, x, w, dy)
                rows.append((f"{name} {hn} fwd+bwd", ms, g * 2.0 * 8192 * Kl * Nl))
            del x, w, dy
        workload = "config 3: Llama-3.1-8B MLP (gate/up K=4096 N=28672, down K=14336 N=4096), M=8192, outlier channels"
    elif args.config == 4:
        Ml, Nl, Kl = 16384, 4096, 14336
        dy = synth.student_t3(Ml, Nl, 1e-3, 0, synth.STREAM_DY).to(dev)
        x = synth.normal(Ml, Kl, 1.0, 0, synth.STREAM_X).to(dev)
        for had, rnd, nm in ((mx.HAD_DET, mx.RNE, "det-H RNE"), (mx.HAD_RANDSIGN, mx.RNE, "random-sign-H RNE"),
                             (mx.HAD_NONE, mx.SR, "no-H SR")):
            ms, g = layer(Ml, Kl, Nl, had, rnd, x, None, dy, "w")
            rows.append((f"wgrad {nm}", ms, g * 2.0 * Ml * Kl * Nl))
        workload = "config 4: Wgrad stress, dW[4096,14336] = dY^T X over M=16384 tokens, both operands column-wise"
    else:
        for name, Kl, Nl in (("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
                             ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096)):
            x = synth.normal(8192, Kl, 1.0, 5, synth.STREAM_X).to(dev)
            w = synth.normal(Nl, Kl, 0.02, 5, synth.STREAM_W).to(dev)
            dy = synth.normal(8192, Nl, 1e-3, 5, synth.STREAM_DY).to(dev)
            ms, g = layer(8192, Kl, Nl, mx.HAD_DET, mx.RNE, x, w, dy)
            rows.append((f"{name} K={Kl} N={Nl} fwd+bwd", ms, g * 2.0 * 8192 * Kl * Nl))
            del x, w, dy
        workload = "config 5: the 7 linears of one Llama-3.1-8B decoder layer, M=8192, det-H32 RNE, fwd+bwd (21 GEMMs)"
        # the same layer the way training stacks lay it out: q, k, v as one N=6144 projection and gate, up as one
        # N=28672 projection (one quantisation of the shared X each); same flops, 12 GEMMs; reported beside the total
        fused_ms = 0.0
        for name, Kl, Nl in (("qkv", 4096, 6144), ("o", 4096, 4096), ("gate_up", 4096, 28672), ("down", 14336, 4096)):
            x = synth.normal(8192, Kl, 1.0, 5, synth.STREAM_X).to(dev)
            w = synth.normal(Nl, Kl, 0.02, 5, synth.STREAM_W).to(dev)
            dy = synth.normal(8192, Nl, 1e-3, 5, synth.STREAM_DY).to(dev)
            fused_ms += layer(8192, Kl, Nl, mx.HAD_DET, mx.RNE, x, w, dy)[0]
            del x, w, dy
        fused = {"what": "same layer with q,k,v fused (N=6144) and gate,up fused (N=28672): 4 linears, 12 GEMMs",
                 "ms": round(fused_ms, 4),
                 "tflops_incl_quant": round(sum(r[2] for r in rows) / (fused_ms * 1e-3) / 1e12, 1)}
    total_ms = sum(r[1] for r in rows)
    total_flop = sum(r[2] for r in rows)
    out = {
        "metric": "mxfp4_linear_gemm_tflops_incl_hadamard_quantize",
        "value": round(total_flop / (total_ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": max(args.steps // 10, 5), "warmup": max(args.warmup // 5, 3), "ms_per_step": round(total_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp4", "data": "synthetic",
        "config": {"workload": workload},
        "pct_of_fp4_peak_incl_quant": round(100.0 * total_flop / (total_ms * 1e-3) / 1e12 / PEAK_FP4_TFLOPS, 2),
        "parts": [{"what": n, "ms": round(ms, 4), "tflops_incl_quant": round(f / (ms * 1e-3) / 1e12, 1)}
                  for n, ms, f in rows],
    }
    if args.config == 5:
        out["fused_projections"] = fused
    if not emit:
        return out
    print(json.dumps(out))
    return 0


def ladder(args, torch, mx, synth) -> int:
    """The stage-wise enablement ladder of Table 1 at kernel level: the headline layer (fwd+bwd, training pair)
    with MXFP4 in none, one, two or all three of its GEMMs and MXFP8 in the others.  One JSON line."""
    dev = torch.device("cuda:0")
    x = synth.normal(M, K, 1.0, 0, synth.STREAM_X).to(dev)
    w = synth.normal(N, K, 0.02, 0, synth.STREAM_W).to(dev)
    dy = synth.normal(M, N, 1e-3, 0, synth.STREAM_DY).to(dev)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    dw = torch.empty((N, K), dtype=torch.float32, device=dev)
    rows = []
    E2, E4 = mx.FMT_E2M1, mx.FMT_E4M3
    for name, fm in (("all GEMMs MXFP8", (E4, E4, E4)), ("Fprop MXFP4", (E2, E4, E4)),
                     ("Fprop + Dgrad MXFP4", (E2, E2, E4)), ("Fprop + Dgrad + Wgrad MXFP4", (E2, E2, E2))):
        cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 0, y_dtype=mx.OUT_BF16, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32,
                          fprop_format=fm[0], dgrad_format=fm[1], wgrad_format=fm[2])
        ws_f = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, False), dtype=torch.uint8, device=dev)
        ws_b = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, True), dtype=torch.uint8, device=dev)
        saved = torch.empty(mx.mxfp4_linear_saved_bytes(M, N, K, cfg), dtype=torch.uint8, device=dev)

        def step():
            mx.mxfp4_linear_fwd_save(x, w, cfg, y=y, workspace=ws_f, saved=saved)
            mx.mxfp4_linear_bwd_saved(dy, saved, K, cfg, dx=dx, dw=dw, workspace=ws_b)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        rows.append((name, (time.perf_counter() - t0) * 1e3 / args.steps))
    base = rows[0][1]
    out = {
        "metric": "linear_fwd_bwd_ms_by_stage_recipe", "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "higher_is_better": False, "dtype": "fp4/fp8", "data": "synthetic",
        "config": {"workload": "Llama-3.1-8B fused QKV linear, M=8192 K=4096 N=6144, fwd+bwd, deterministic H32 on the "
                               "MXFP4 GEMMs, RNE; stages not in MXFP4 run in MXFP8 (E4M3)"},
        "ladder": [{"recipe": n, "ms_per_step": round(ms, 4), "speedup_vs_all_mxfp8": round(base / ms, 3),
                    "tflops_incl_quant": round(3 * 2.0 * M * N * K / (ms * 1e-3) / 1e12, 1)} for n, ms in rows],
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--ladder", action="store_true",
                    help="time the headline layer under the stage-wise recipes of Table 1 (MXFP4 in 0..3 of the "
                         "GEMMs, MXFP8 in the others) instead of the headline benchmark")
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="benchmark configuration; 2 (the default) is the headline workload with the full report")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the totals of configurations 1, 3, 4 and 5 (the `configs` array)")
    ap.add_argument("--power-probe", action="store_true",
                    help="print shader clock and socket power sampled while the GEMM runs on zero, random and "
                         "benchmark operands (text, no JSON)")
    ap.add_argument("--probe-seconds", type=float, default=3.0)
    ap.add_argument("--counter-run", action="store_true",
                    help="for rocprofv3 --pmc: one 256 MiB device copy (known traffic) followed by one "
                         "step through the training pair and one through the separate calls, no timing, "
                         "no JSON")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2605_09825_amd as mx
    from paper_2605_09825_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    mx.lib()  # fail loudly now if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.power_probe:
        return power_probe(args, torch, mx)
    if args.ladder:
        return ladder(args, torch, mx, synth)
    if args.config != 2:
        return other_config(args, torch, mx, synth)

    x_cpu = synth.normal(M, K, 1.0, 0, synth.STREAM_X)
    w_cpu = synth.normal(N, K, 0.02, 0, synth.STREAM_W)
    dy_cpu = synth.normal(M, N, 1e-3, 0, synth.STREAM_DY)
    x, w, dy = x_cpu.to(dev), w_cpu.to(dev), dy_cpu.to(dev)

    cfg = mx.make_cfg(mx.HAD_DET, mx.RNE, 0, y_dtype=mx.OUT_BF16, dx_dtype=mx.OUT_BF16, dw_dtype=mx.OUT_FP32)
    ws_f = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(mx.mxfp4_linear_workspace_bytes(M, N, K, cfg, True), dtype=torch.uint8, device=dev)
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
    dw = torch.empty((N, K), dtype=torch.float32, device=dev)

    saved = torch.empty(mx.mxfp4_linear_saved_bytes(M, N, K), dtype=torch.uint8, device=dev)

    def step():
        mx.mxfp4_linear_fwd_save(x, w, cfg, y=y, workspace=ws_f, saved=saved)
        mx.mxfp4_linear_bwd_saved(dy, saved, K, cfg, dx=dx, dw=dw, workspace=ws_b)

    def step_separate():
        mx.mxfp4_linear_fwd(x, w, cfg, y=y, workspace=ws_f)
        mx.mxfp4_linear_bwd(dy, x, w, cfg, dx=dx, dw=dw, workspace=ws_b)

    if args.counter_run:
        ref = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(ref)
        ref.zero_()
        torch.cuda.synchronize()
        dst.copy_(ref)  # reference dispatch: reads 256 MiB, writes 256 MiB
        step()
        step_separate()
        torch.cuda.synchronize()
        print("counter run done: reference copy 268435456 bytes each way, then 2 steps")
        return 0

    flop_step = 3 * 2.0 * M * N * K

    # ---- per-kernel durations, live, with events on the launch stream -------------------------
    # (torch's current stream is the stream every call above was launched on)
    off_f = mx.mxfp4_linear_workspace_layout(M, N, K, False)
    off_b = mx.mxfp4_linear_workspace_layout(M, N, K, True)

    def view(ws, off, R, C, k):
        q = ws[off[2 * k]: off[2 * k] + R * C // 2].view(R, C // 2)
        s = ws[off[2 * k + 1]: off[2 * k + 1] + R * C // 32].view(R, C // 32)
        return q, s

    xq, xs = view(ws_f, off_f, M, K, 0)
    wq, wsc = view(ws_f, off_f, N, K, 1)
    gq, gs = view(ws_b, off_b, M, N, 0)
    wtq, wts = view(ws_b, off_b, K, N, 1)
    gtq, gts = view(ws_b, off_b, N, M, 2)
    xtq, xts = view(ws_b, off_b, K, M, 3)
    off_s = mx.mxfp4_linear_saved_layout(M, N, K)
    sv_wtq = saved[off_s[0]: off_s[0] + K * N // 2].view(K, N // 2)
    sv_wts = saved[off_s[1]: off_s[1] + K * N // 32].view(K, N // 32)
    sv_xtq = saved[off_s[2]: off_s[2] + K * M // 2].view(K, M // 2)
    sv_xts = saved[off_s[3]: off_s[3] + K * M // 32].view(K, M // 32)

    def q_rows(t, q, s):
        mx.mxfp4_quantize(t, mx.AXIS_LAST, mx.HAD_DET, mx.RNE, 0, q=q, s=s)

    def q_cols(t, q, s):
        mx.mxfp4_quantize(t, mx.AXIS_FIRST, mx.HAD_DET, mx.RNE, 0, q=q, s=s)

    L = mx.lib()
    st = torch.cuda.current_stream().cuda_stream

    def q_dual(t, ql, sl, qf, sf):
        rc = L.mxfp4_quantize_dual(t.data_ptr(), t.shape[0], t.shape[1], t.shape[1], mx.HAD_DET, mx.RNE, 0,
                                   ql.data_ptr(), sl.data_ptr(), qf.data_ptr(), sf.data_ptr(), st)
        assert rc == mx.OK

    # The launches of one step, in the step's order and on the step's buffers, issued through the single-operation
    # entry points so that an event pair can bracket every kernel: a second timed region of the same work.
    launches = [
        ("x_dual", lambda: q_dual(x, xq, xs, sv_xtq, sv_xts)),
        ("w_dual", lambda: q_dual(w, wq, wsc, sv_wtq, sv_wts)),
        ("fprop", lambda: mx.mxfp4_gemm(xq, xs, wq, wsc, out=y, out_dtype=mx.OUT_BF16)),
        ("dy_dual", lambda: q_dual(dy, gq, gs, gtq, gts)),
        ("dgrad+wgrad", lambda: mx.mxfp4_gemm_pair((gq, gs), (sv_wtq, sv_wts), dx, (gtq, gts), (sv_xtq, sv_xts), dw)),
    ]
    single = {  # the two backward products as launches of their own (what the separate calls enqueue)
        "dgrad": lambda: mx.mxfp4_gemm(gq, gs, sv_wtq, sv_wts, out=dx, out_dtype=mx.OUT_BF16),
        "wgrad": lambda: mx.mxfp4_gemm(gtq, gts, sv_xtq, sv_xts, out=dw, out_dtype=mx.OUT_FP32),
    }
    n_inst = min(args.steps, 100)
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in launches]
          for _ in range(n_inst)]
    for _ in range(3):
        for _, fn in launches:
            fn()
    torch.cuda.synchronize()
    for i in range(n_inst):
        for k, (_, fn) in enumerate(launches):
            ev[i][k][0].record()
            fn()
            ev[i][k][1].record()
    torch.cuda.synchronize()
    t_k = {name: sum(ev[i][k][0].elapsed_time(ev[i][k][1]) for i in range(n_inst)) / n_inst
           for k, (name, _) in enumerate(launches)}
    # Each bracket also holds the dispatch gap to the previous kernel (the event records serialise the queue), so
    # the kernel's own duration is taken from back-to-back launches of the same GEMM on the same operands, which
    # is what a kernel trace reports as well; both are printed.
    iters = min(max(5, args.steps), 50)
    t_fprop = event_time_ms(launches[2][1], iters, torch)
    t_pair = event_time_ms(launches[4][1], iters, torch)
    t_dgrad = event_time_ms(single["dgrad"], iters, torch)
    t_wgrad = event_time_ms(single["wgrad"], iters, torch)
    # the step's longest launch, Dgrad and Wgrad side by side (two GEMMs' flops), is the kernel of the roofline
    pair_tflops = 2 * 2.0 * M * N * K / (t_pair * 1e-3) / 1e12
    single_tflops = 2.0 * M * N * K / ((t_fprop + t_dgrad + t_wgrad) / 3.0 * 1e-3) / 1e12
    t_quant_total = t_k["x_dual"] + t_k["w_dual"] + t_k["dy_dual"]

    # the single-axis kernels on the same (cache-warm) operands, back to back
    t_q = {
        "x_rows": event_time_ms(lambda: q_rows(x, xq, xs), iters, torch),
        "w_rows": event_time_ms(lambda: q_rows(w, wq, wsc), iters, torch),
        "dy_rows": event_time_ms(lambda: q_rows(dy, gq, gs), iters, torch),
        "w_cols": event_time_ms(lambda: q_cols(w, wtq, wts), iters, torch),
        "dy_cols": event_time_ms(lambda: q_cols(dy, gtq, gts), iters, torch),
        "x_cols": event_time_ms(lambda: q_cols(x, xtq, xts), iters, torch),
    }
    elems = {"x_rows": M * K, "w_rows": N * K, "dy_rows": M * N, "w_cols": N * K, "dy_cols": M * N, "x_cols": M * K}
    t_q.update({k: t_k[k] for k in ("x_dual", "w_dual", "dy_dual")})

    # HBM-resident rate: rotate over 10 distinct X-sized inputs (640 MiB > the 256 MB last-level cache)
    rot = [x] + [torch.empty_like(x).copy_(x) for _ in range(9)]
    state = {"i": 0}

    def q_rot(fn):
        def run():
            fn(rot[state["i"] % len(rot)], xq if fn is q_rows else xtq, xs if fn is q_rows else xts)
            state["i"] += 1
        return run

    def dual_rot():
        q_dual(rot[state["i"] % len(rot)], xq, xs, xtq, xts)
        state["i"] += 1

    x8q = torch.empty((M, K), dtype=torch.uint8, device=dev)   # MXFP8 outputs (row-wise [M][K], column-wise [K][M])

    def fp8_rot(axis):
        def run():
            t = rot[state["i"] % len(rot)]
            rc = L.mxfp4_quantize_fp8(t.data_ptr(), M, K, K, axis, mx.HAD_NONE, 0, x8q.data_ptr(),
                                      (xs if axis == mx.AXIS_LAST else xts).data_ptr(), st)
            assert rc == mx.OK
            state["i"] += 1
        return run

    def dual_2d_rot():  # the 32 x 32 geometry, both outputs, no rotation
        t = rot[state["i"] % len(rot)]
        rc = L.mxfp4_quantize_2d(t.data_ptr(), M, K, K, mx.HAD_NONE, mx.RNE, 0, xq.data_ptr(), xs.data_ptr(),
                                 xtq.data_ptr(), xts.data_ptr(), st)
        assert rc == mx.OK
        state["i"] += 1

    n_rot = 2 * len(rot)
    q_rot(q_rows)()
    q_rot(q_cols)()
    dual_rot()
    t_rows_cold = event_time_ms(q_rot(q_rows), n_rot, torch)
    t_cols_cold = event_time_ms(q_rot(q_cols), n_rot, torch)
    t_dual_cold = event_time_ms(dual_rot, n_rot, torch)
    dual_2d_rot()
    t_2d_cold = event_time_ms(dual_2d_rot, n_rot, torch)
    fp8_rot(mx.AXIS_LAST)()
    fp8_rot(mx.AXIS_FIRST)()
    t_fp8_rows = event_time_ms(fp8_rot(mx.AXIS_LAST), n_rot, torch)
    t_fp8_cols = event_time_ms(fp8_rot(mx.AXIS_FIRST), n_rot, torch)
    gbs = lambda n_el, ms, bpe=BYTES_PER_ELEM: n_el * bpe / (ms * 1e-3) / 1e9

    # the same three kernels under each rotation size (Table 1 note: H16 against H32), HBM-resident
    def rot_call(kind, had):
        def run():
            t = rot[state["i"] % len(rot)]
            state["i"] += 1
            if kind == "rows":
                mx.mxfp4_quantize(t, mx.AXIS_LAST, had, mx.RNE, 0, q=xq, s=xs)
            elif kind == "cols":
                mx.mxfp4_quantize(t, mx.AXIS_FIRST, had, mx.RNE, 0, q=xtq, s=xts)
            else:
                rc = L.mxfp4_quantize_dual(t.data_ptr(), M, K, K, had, mx.RNE, 0, xq.data_ptr(), xs.data_ptr(),
                                           xtq.data_ptr(), xts.data_ptr(), st)
                assert rc == mx.OK
        return run

    by_rotation = {}
    for kind, bpe in (("rows", BYTES_PER_ELEM), ("cols", BYTES_PER_ELEM), ("dual", BYTES_PER_ELEM_DUAL)):
        by_rotation[kind] = {}
        for name, had in (("none", mx.HAD_NONE), ("h16", mx.HAD_DET16), ("h32", mx.HAD_DET)):
            fn = rot_call(kind, had)
            fn()
            ms = event_time_ms(fn, n_rot, torch)
            by_rotation[kind][name] = {"launch_ms": round(ms, 4), "achieved": round(gbs(M * K, ms, bpe), 1),
                                       "frac": round(gbs(M * K, ms, bpe) / PEAK_HBM_GBS, 4)}
        by_rotation[kind]["h16_speedup_over_h32"] = round(by_rotation[kind]["h32"]["launch_ms"] /
                                                          by_rotation[kind]["h16"]["launch_ms"], 3)
    del rot
    quant_rows_gbs, quant_cols_gbs = gbs(M * K, t_rows_cold), gbs(M * K, t_cols_cold)
    quant_dual_gbs = gbs(M * K, t_dual_cold, BYTES_PER_ELEM_DUAL)
    quant_2d_gbs = gbs(M * K, t_2d_cold, BYTES_PER_ELEM_DUAL)
    bpe8 = 2.0 + 1.0 + 1.0 / 32.0  # bf16 read + one E4M3 byte + scale byte per element
    fp8_rows_gbs, fp8_cols_gbs = gbs(M * K, t_fp8_rows, bpe8), gbs(M * K, t_fp8_cols, bpe8)

    # ---- shader clock during a sustained run of the dominant kernel ---------------------------------------
    # (about a second of back-to-back launches of the step's GEMM kernels on the step's operands: Fprop, then
    # Dgrad and Wgrad side by side)
    def gemm_round():
        launches[2][1]()
        launches[4][1]()
    for _ in range(20):
        gemm_round()
    torch.cuda.synchronize()
    with ClockSampler() as cs:
        t0 = time.perf_counter()
        n_rounds = 0
        while time.perf_counter() - t0 < 1.0:
            for _ in range(100):
                gemm_round()
            torch.cuda.synchronize()
            n_rounds += 100
        t_sustained = (time.perf_counter() - t0) * 1e3 / (3 * n_rounds)
    clock = cs.summary()
    sclk = clock["sclk_mhz_median"]
    gemm_tflops_sustained = 2.0 * M * N * K / (t_sustained * 1e-3) / 1e12
    peak_at_clock = PEAK_FP4_TFLOPS * sclk / 2400.0 if sclk else None

    # ---- the headline: the whole step, timed last (the legs above have brought the chip to its working state) --
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    reps = []
    for _ in range(REPEATS):
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        reps.append((time.perf_counter() - t0) * 1e3 / args.steps)
    ms_per_step = sorted(reps)[REPEATS // 2]
    for _ in range(5):
        step_separate()
    torch.cuda.synchronize()
    reps_sep = []
    for _ in range(3):
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_separate()
        torch.cuda.synchronize()
        reps_sep.append((time.perf_counter() - t0) * 1e3 / args.steps)
    ms_separate = sorted(reps_sep)[1]
    tflops_incl = flop_step / (ms_per_step * 1e-3) / 1e12

    out = {
        "metric": "mxfp4_linear_gemm_tflops_incl_hadamard_quantize",
        "value": round(tflops_incl, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "repeats": REPEATS,
        "ms_per_step_min": round(min(reps), 4),
        "ms_per_step_max": round(max(reps), 4),
        "timing": f"median of {REPEATS} repetitions of the timed region of `steps` steps, after `warmup` steps; "
                  "the per-kernel legs run before it",
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp4",
        "data": "synthetic",
        "config": {
            "workload": "config 2: Llama-3.1-8B fused QKV linear, Fprop+Dgrad+Wgrad, M=8192 K=4096 N=6144, "
                        "deterministic H32 + MXFP4 RNE on both operands of each GEMM; y,dx bf16, dw fp32",
            "M": M, "K": K, "N": N, "launches_per_step": 4,
            "calls": "mxfp4_linear_fwd_save + mxfp4_linear_bwd_saved",
        },
        "separate_calls_ms_per_step": round(ms_separate, 4),
        "pct_of_fp4_peak_incl_quant": round(100.0 * tflops_incl / PEAK_FP4_TFLOPS, 2),
        "roofline": {
            "kernel": "gemm_tile_pair_kernel: Dgrad 8192x4096x6144 (bf16 out) and Wgrad 6144x4096x8192 (fp32 out) side "
                      "by side in one launch, the longest kernel of the step",
            "bound": "mfma",
            "achieved": round(pair_tflops, 2),
            "peak": PEAK_FP4_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(pair_tflops / PEAK_FP4_TFLOPS, 4),
            "flop_per_launch": 2 * 2.0 * M * N * K,
            "single_launches": {"what": "Fprop, Dgrad and Wgrad as launches of their own, mean",
                                "achieved": round(single_tflops, 2),
                                "frac": round(single_tflops / PEAK_FP4_TFLOPS, 4)},
            "traffic": GEMM_TRAFFIC_BYTES,
            "traffic_source": GEMM_TRAFFIC_SOURCE + " (rocprofv3 FETCH_SIZE + WRITE_SIZE at the L2's outward port, "
                              "Infinity Cache hits included; not measured in this run)",
            "algorithmic_bytes": round(GEMM_ALGORITHMIC_BYTES),
            "traffic_over_algorithmic": round(GEMM_TRAFFIC_BYTES / GEMM_ALGORITHMIC_BYTES, 2),
            "sclk_mhz": sclk,
            "clock_samples": clock,
            "sustained_tflops": round(gemm_tflops_sustained, 2),
            "peak_at_measured_clock": round(peak_at_clock, 1) if peak_at_clock else None,
            "frac_at_measured_clock": round(gemm_tflops_sustained / peak_at_clock, 4) if peak_at_clock else None,
            "launch_ms": {"dgrad+wgrad": round(t_pair, 4), "fprop": round(t_fprop, 4), "dgrad": round(t_dgrad, 4),
                          "wgrad": round(t_wgrad, 4)},
            "in_step_bracket_ms": {k: round(t_k[k], 4) for k in ("fprop", "dgrad+wgrad")},
        },
        "quantizer": {
            "bound": "hbm",
            "unit": "GB/s",
            "peak": PEAK_HBM_GBS,
            "bytes_per_element": BYTES_PER_ELEM,
            "rows_hbm_resident": {"achieved": round(quant_rows_gbs, 1), "frac": round(quant_rows_gbs / PEAK_HBM_GBS, 4),
                                  "launch_ms": round(t_rows_cold, 4)},
            "cols_hbm_resident": {"achieved": round(quant_cols_gbs, 1), "frac": round(quant_cols_gbs / PEAK_HBM_GBS, 4),
                                  "launch_ms": round(t_cols_cold, 4)},
            "dual_hbm_resident": {"achieved": round(quant_dual_gbs, 1), "frac": round(quant_dual_gbs / PEAK_HBM_GBS, 4),
                                  "launch_ms": round(t_dual_cold, 4), "bytes_per_element": BYTES_PER_ELEM_DUAL},
            "dual_2d_hbm_resident": {"achieved": round(quant_2d_gbs, 1), "frac": round(quant_2d_gbs / PEAK_HBM_GBS, 4),
                                     "launch_ms": round(t_2d_cold, 4), "bytes_per_element": BYTES_PER_ELEM_DUAL},
            "mxfp8_rows_hbm_resident": {"achieved": round(fp8_rows_gbs, 1), "frac": round(fp8_rows_gbs / PEAK_HBM_GBS, 4),
                                        "launch_ms": round(t_fp8_rows, 4), "bytes_per_element": bpe8},
            "mxfp8_cols_hbm_resident": {"achieved": round(fp8_cols_gbs, 1), "frac": round(fp8_cols_gbs / PEAK_HBM_GBS, 4),
                                        "launch_ms": round(t_fp8_cols, 4), "bytes_per_element": bpe8},
            "by_rotation_hbm_resident": by_rotation,
            "in_step_ms": {k: round(v, 4) for k, v in t_q.items()},
            "in_step_gbs_cache_warm": {k: round(gbs(elems[k], t_q[k]), 1) for k in elems},
        },
        "breakdown_ms": {"gemm_total": round(t_k["fprop"] + t_k["dgrad+wgrad"], 4),
                         "quantize_total": round(t_quant_total, 4),
                         "note": "event brackets inside a second timed region; each includes the dispatch gap"},
    }

    if not args.no_other_configs:
        # totals of the other benchmark configurations, same conventions (free the headline's buffers first)
        del x, w, dy, y, dx, dw, ws_f, ws_b, saved, xq, xs, wq, wsc, gq, gs, wtq, wts, gtq, gts, xtq, xts
        del sv_wtq, sv_wts, sv_xtq, sv_xts, launches, single
        torch.cuda.empty_cache()
        out["configs"] = []
        for c in (1, 3, 4, 5):
            args.config = c
            r = other_config(args, torch, mx, synth, emit=False)
            out["configs"].append({"config": c, "workload": r["config"]["workload"], "ms": r["ms_per_step"],
                                   "tflops_incl_quant": r["value"],
                                   "pct_of_fp4_peak_incl_quant": r["pct_of_fp4_peak_incl_quant"], "parts": r["parts"]})
            if "fused_projections" in r:
                out["configs"][-1]["fused_projections"] = r["fused_projections"]
            torch.cuda.empty_cache()
        args.config = 2

    if not args.no_cpu_baseline:
        import oracle
        Ms = 4096  # the first 4096 of the 8192 tokens; all of N and K; all three stages
        xb, wb, dyb = synth.as_u16(x_cpu[:Ms]), synth.as_u16(w_cpu), synth.as_u16(dy_cpu[:Ms])
        c0 = time.perf_counter()
        oracle.linear_fwd(xb, wb, oracle.HAD_DET)
        oracle.linear_bwd(dyb, xb, wb, oracle.HAD_DET)
        c1 = time.perf_counter()
        out["cpu_baseline"] = {
            "value": round(3 * 2.0 * Ms * N * K / (c1 - c0) / 1e12, 6),
            "unit": "TFLOP/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"first {Ms} of {M} tokens, full N and K, Fprop+Dgrad+Wgrad with rotation and "
                      f"quantisation; {round(c1 - c0, 2)} s",
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
