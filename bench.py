#!/usr/bin/env python3
"""Throughput of one pipeline stage's micro-batched training step on one MI355X.

A step is one mini-batch on the stage: grad_accum_reset, M forwards (boundary
activation kept only), then M recompute+backward calls with fp32 gradient
accumulation -- all through the C ABI, inputs resident in HBM before timing.
Prints ONE JSON line (metric, value, roofline of the dominant kernel measured
with HIP events, and the fp64 oracle timed on the host cores as cpu_baseline).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", help="C1..C5 (default: the largest stage, C5)")
    ap.add_argument("--micro-batches", type=int, default=0, help="override M (default: the config's)")
    ap.add_argument("--wgrad-group", type=int, default=8,
                    help="micro-batches per weight-gradient GEMM (library knob; 1 = per micro-batch)")
    ap.add_argument("--stage", choices=("middle", "last"), default="middle",
                    help="middle: M forwards then M recompute+backward calls (the headline step); last: the "
                         "last pipeline stage's step, M times forward_keep + backward_stored, no recompute")
    ap.add_argument("--calibrate", default="",
                    help="comma-separated micro-batch sizes m: instead of the step benchmark, print F(m), "
                         "recompute+backward(m), keeping-forward(m) and stored-backward(m) per m and the m picked")
    ap.add_argument("--pipeline-stages", type=int, default=0,
                    help="with --calibrate: also feed the measured times of the picked m into the schedule simulator "
                         "for a pipeline of this many stages (the config's M micro-batches) and print the estimates")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout probability on attention probabilities and both residual branches (the headline "
                         "workload has none; this measures what the counter-based masks cost)")
    ap.add_argument("--tail", action="store_true",
                    help="instead of the step benchmark, time the mini-batch tail (gradient statistics + Adam "
                         "step over the stage's parameters) and print its HBM roofline")
    ap.add_argument("--ceiling", action="store_true",
                    help="instead of the step benchmark, measure what the matrix cores sustain when fed from registers "
                         "only (v_mfma_f32_32x32x16_bf16 on normally distributed and on all-zero operands)")
    ap.add_argument("--energy", action="store_true",
                    help="instead of the step benchmark, measure energy per FLOP (the GPU's accumulated-energy counter "
                         "read through rocm-smi over windows of several seconds) of the register-only MFMA loop, of this "
                         "library's forward GEMM on two C5 shapes, and of the vendor library's GEMM as a reference point")
    ap.add_argument("--no-ungrouped", action="store_true",
                    help="skip the second measurement of the same step with wgrad_group=1 (the configuration as "
                         "specified: weight gradients accumulated after every micro-batch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-profile", action="store_true")
    return ap.parse_args()


def cpu_baseline(cfg):
    """The fp64 oracle as it stands on ONE micro-batch of the benchmarked stage (all layers,
    full sequence): forward + backward = 3 of the 4 forward units a GPU micro-batch costs."""
    import numpy as np
    from oracle import stage_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    h, f, s, b = cfg.hidden, cfg.mlp_hidden, cfg.seq_len, cfg.micro_batch
    sh = O.StageShape(cfg.n_layers, h, cfg.n_heads, s, b, f, cfg.causal, cfg.ln_eps)
    rng = np.random.default_rng(cfg.seed)
    params = []
    for _ in range(cfg.n_layers):
        p = {k: rng.standard_normal(shp) * cfg.w_std for k, shp in O.param_shapes(sh).items()}
        p["ln1_g"] += 1.0
        p["ln2_g"] += 1.0
        params.append(p)
    x = rng.standard_normal((sh.tokens, h))
    dy = rng.standard_normal((sh.tokens, h))
    t0 = time.perf_counter()
    y, caches = O.stage_forward(x, params, sh)
    O.stage_backward(dy, params, caches, sh)
    dt = time.perf_counter() - t0
    attn = 4.0 * sh.tokens * s * h * (0.5 if cfg.causal else 1.0)
    useful = 3.0 * cfg.n_layers * (2.0 * sh.tokens * h * (4 * h + 2 * f) + attn)
    return {
        "value": useful / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "sample": f"fp64 numpy oracle, one whole micro-batch of {cfg.name} ({cfg.n_layers} layers, micro-batch {b} x seq {s}), "
                  f"forward+backward = 3 forward units, {dt:.1f} s wall = {dt * 1e3:.0f} ms per micro-batch",
        "seconds": dt, "ms_per_micro_batch": dt * 1e3, "host_cpus": os.cpu_count(),
    }


class GpuSensors:
    """Samples the GPU's own power and clock sensors (hwmon files of the amdgpu driver, read-only)
    from a host thread while a timed region runs: the evidence for what clock the chip holds
    under a given load.  Reports nulls if the box exposes no such files."""

    def __init__(self, period_s=0.05):
        import glob
        self.period = period_s
        self.files = {}
        for d in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
            for key, names in (("power_uw", ("power1_average", "power1_input")), ("sclk_hz", ("freq1_input",)),
                               ("cap_uw", ("power1_cap",))):
                for n in names:
                    f = os.path.join(d, n)
                    if key not in self.files and os.path.exists(f):
                        self.files[key] = f
            if self.files:
                break
        self.samples = {"power_uw": [], "sclk_hz": []}
        self._stop = None
        self._thread = None

    @staticmethod
    def _read(path):
        try:
            with open(path) as fh:
                return float(fh.read().strip())
        except (OSError, ValueError):
            return None

    def __enter__(self):
        import threading
        self.samples = {"power_uw": [], "sclk_hz": []}
        self._stop = threading.Event()

        def loop():
            while not self._stop.is_set():
                for k in self.samples:
                    if k in self.files:
                        v = self._read(self.files[k])
                        if v is not None:
                            self.samples[k].append(v)
                self._stop.wait(self.period)
        self._thread = threading.Thread(target=loop, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()

    def summary(self):
        def mean(v):
            return sum(v) / len(v) if v else None
        p, c = self.samples["power_uw"], self.samples["sclk_hz"]
        cap = self._read(self.files["cap_uw"]) if "cap_uw" in self.files else None
        return {"power_w_mean": None if not p else mean(p) / 1e6, "power_w_max": None if not p else max(p) / 1e6,
                "power_cap_w": None if cap is None else cap / 1e6,
                "sclk_mhz_mean": None if not c else mean(c) / 1e6, "sclk_mhz_min": None if not c else min(c) / 1e6,
                "samples": len(p) or len(c)}


def bench_ceiling(args):
    """Register-only MFMA rate on normally distributed and on all-zero operands, one and two
    waves per SIMD: the measured ceiling beside the nominal 2.5 PFLOP/s."""
    import torch
    from paper_2111_04007_amd import binding as B, flops
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    props = torch.cuda.get_device_properties(dev)
    gen = torch.Generator(device=dev).manual_seed(20211104)
    n = 1 << 23
    data = {"normal(0,1)": torch.empty(n, device=dev, dtype=torch.float32).normal_(generator=gen).to(torch.bfloat16),
            "normal(0,0.02)": (torch.empty(n, device=dev, dtype=torch.float32).normal_(generator=gen) * 0.02).to(torch.bfloat16),
            "zeros": torch.zeros(n, device=dev, dtype=torch.bfloat16)}
    sink = torch.empty(props.multi_processor_count * 2 * 256, device=dev, dtype=torch.float32)
    stream = torch.cuda.current_stream()
    iters = 200000      # about 0.1 s per launch
    rows = []
    cases = [(name, wps, 0) for name in data for wps in (1, 2)] + [("normal(0,1)", 2, pat) for pat in (1, 2, 3, 4, 5, 6, 7)]
    for name, wps, pat in cases:
        t = data[name]
        if True:
            rates = []
            sens = GpuSensors(0.01)
            for rep in range(args.warmup + args.steps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                if rep == args.warmup:
                    sens.__enter__()
                e0.record(stream)
                fl = B.probe_mfma_rate(t, wps, iters, sink, pat, stream)
                e1.record(stream)
                torch.cuda.synchronize()
                if rep >= args.warmup:
                    rates.append(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
            sens.__exit__()
            rates.sort()
            rows.append({"operands": name, "waves_per_simd": wps, "operand_pattern": pat, "tflops_median": rates[len(rates) // 2],
                         "tflops_min": rates[0], "tflops_max": rates[-1],
                         "frac_of_nominal_peak": rates[len(rates) // 2] * 1e12 / flops.MI355X_BF16_DENSE_PEAK,
                         "implied_clock_mhz": rates[len(rates) // 2] * 1e12 / flops.MI355X_BF16_DENSE_PEAK * 2400.0,
                         "sensors": sens.summary()})
    best_real = max(r["tflops_median"] for r in rows if r["operands"] == "normal(0,1)" and r["operand_pattern"] == 0)
    return {"metric": "register-only v_mfma_f32_32x32x16_bf16 rate (measured ceiling beside the nominal peak; operand patterns 6 and 7 are the 16x16x32 shape)",
            "value": best_real, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "higher_is_better": True, "dtype": "bf16", "data": "synthetic", "vs_baseline": None,
            "config": {"workload": "MFMA-only loop, no LDS or memory traffic", "device": props.name,
                       "compute_units": props.multi_processor_count, "iters_per_launch": iters,
                       "nominal_peak_tflops": flops.MI355X_BF16_DENSE_PEAK / 1e12},
            "rows": rows}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the stage step; this build has no multi-GPU path "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2111_04007_amd import CONFIGS, binding as B, flops, synth

    cfg = CONFIGS[args.config]
    if args.calibrate:
        from paper_2111_04007_amd import calibrate
        ms = [int(v) for v in args.calibrate.split(",")]
        torch.cuda.set_device(0)
        rows = calibrate.sweep(cfg, ms, n_mb=args.micro_batches or 4, reps=max(1, args.steps))
        pick = calibrate.pick_micro_batch([r["m"] for r in rows], [r["F_per_example_ms"] for r in rows])
        sim = None
        if args.pipeline_stages > 1:
            from paper_2111_04007_amd import schedule_sim
            r = next(r for r in rows if r["m"] == pick)
            sim = schedule_sim.estimate(args.pipeline_stages, cfg.n_micro_batches, r["F_ms"], r["RB_ms"], r["Fkeep_ms"], r["B_ms"])
            sim.update({"pipeline_stages": args.pipeline_stages, "n_micro_batches": cfg.n_micro_batches, "m": pick,
                        "note": "compute only: send latency and all-reduce set to 0 (one GPU is measured)"})
        print(json.dumps({"schedule_estimate": sim, "metric": "calibration: stage compute time per micro-batch size m (ms)", "unit": "ms",
                          "n_gpus": 1, "dtype": cfg.dtype, "data": "synthetic",
                          "config": {"workload": cfg.name + " swept over micro_batch", "n_layers": cfg.n_layers,
                                     "hidden": cfg.hidden, "seq_len": cfg.seq_len},
                          "rows": rows, "picked_m": pick, "rule": "lowest m whose F(m)/m no larger m beats by > 3 %"}))
        return
    if args.tail:
        print(json.dumps(bench_tail(cfg, args)))
        return
    if args.ceiling:
        print(json.dumps(bench_ceiling(args)))
        return
    if args.energy:
        print(json.dumps(bench_energy(args)))
        return
    if args.micro_batches:
        cfg = cfg.replace(n_micro_batches=args.micro_batches)
    cfg = cfg.replace(wgrad_group=max(1, args.wgrad_group), dropout_p=args.dropout)
    M = cfg.n_micro_batches
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    props = torch.cuda.get_device_properties(dev)

    params, xs, dys = synth.device_random_stage(cfg, dev)
    st = B.Stage(cfg, dev, params_flat=params)
    st.set_side_stream(torch.cuda.Stream(dev))   # the caller's second stream for the bias-gradient sums
    if cfg.dropout_p > 0:
        st.set_dropout_seed(20211104)
    ys = torch.empty_like(xs)
    dxs = torch.empty_like(xs)
    stream = torch.cuda.current_stream()

    last = args.stage == "last"

    def step():
        st.grad_accum_reset(stream)
        if last:
            for m in range(M):
                st.forward_keep(m, xs[m], ys[m], stream)
                st.backward_stored(m, dys[m], dxs[m], stream)
        else:
            for m in range(M):
                st.forward(m, xs[m], ys[m], stream)
            for m in range(M):
                st.backward_recompute(m, dys[m], dxs[m], stream)
        st.grad_flush(stream)

    for _ in range(args.warmup):
        step()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    sensors = GpuSensors()
    with sensors:
        t0 = time.perf_counter()
        for i in range(args.steps):
            marks[i].record(stream)     # per-step spread (median, min); the headline is the wall time of all steps
            step()
        marks[args.steps].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    ms_mb = ms_step / M
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_step_median = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    ms_step_min = per_step[0]

    # separate forward / (recompute+)backward timing with events on the same stream
    st.grad_accum_reset(stream)
    if last:
        evs = []
        for m in range(M):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record(stream)
            st.forward_keep(m, xs[m], ys[m], stream)
            e[1].record(stream)
            st.backward_stored(m, dys[m], dxs[m], stream)
            e[2].record(stream)
            evs.append(e)
        st.grad_flush(stream)
        torch.cuda.synchronize()
        ms_f = sum(e[0].elapsed_time(e[1]) for e in evs) / M
        ms_rb = sum(e[1].elapsed_time(e[2]) for e in evs) / M
    else:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record(stream)
        for m in range(M):
            st.forward(m, xs[m], ys[m], stream)
        ev[1].record(stream)
        for m in range(M):
            st.backward_recompute(m, dys[m], dxs[m], stream)
        st.grad_flush(stream)
        ev[2].record(stream)
        torch.cuda.synchronize()
        ms_f = ev[0].elapsed_time(ev[1]) / M
        ms_rb = ev[1].elapsed_time(ev[2]) / M

    # FLOP accounting.  Middle stage: 4 forward units per micro-batch (causal-aware), minus the
    # last layer's MLP2 GEMM that the recompute pass does not need and does not run.  Last stage:
    # 3 forward units (no recompute).
    useful_flops_mb = flops.useful_flops_per_microbatch(cfg)
    if last:
        hw_flops_mb = useful_flops_mb
    else:
        skipped = 2.0 * cfg.tokens * cfg.hidden * cfg.mlp_hidden
        hw_flops_mb = flops.step_flops_per_microbatch(cfg) - skipped
    tflops = hw_flops_mb * M / (ms_step * 1e-3) / 1e12
    frac_peak = tflops * 1e12 / flops.MI355X_BF16_DENSE_PEAK

    roofline = None
    classes = None
    if not args.no_kernel_profile:
        st.profile_enable(True)
        tot = {}
        for _ in range(args.steps):
            st.grad_accum_reset(stream)
            for m in range(M):
                if last:
                    st.forward_keep(m, xs[m], ys[m], stream)
                else:
                    st.forward(m, xs[m], ys[m], stream)
                if last or m % 8 == 7 or m == M - 1:
                    _acc(tot, st.profile_collect())
                if last:
                    st.backward_stored(m, dys[m], dxs[m], stream)
                    _acc(tot, st.profile_collect())
            for m in range(M if not last else 0):
                st.backward_recompute(m, dys[m], dxs[m], stream)
                _acc(tot, st.profile_collect())
            st.grad_flush(stream)
            _acc(tot, st.profile_collect())
        st.profile_enable(False)
        classes = {k: {"ms_per_step": v["ms"] / args.steps, "launches_per_step": v["launches"] // args.steps,
                       "tflops": (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["ms"] > 0 and v["flops"] > 0 else None,
                       "gbps": (v["bytes"] / (v["ms"] * 1e-3) / 1e9) if v["ms"] > 0 else None}
                   for k, v in tot.items() if v["launches"]}
        dom = max(tot.items(), key=lambda kv: kv[1]["ms"])
        name, v = dom
        if v["flops"] > 0:
            is_f32 = cfg.dtype == "f32"
            peak = 157.3 if is_f32 else flops.MI355X_BF16_DENSE_PEAK / 1e12
            ach = v["flops"] / (v["ms"] * 1e-3) / 1e12
            roofline = {"kernel": name, "bound": "alu" if is_f32 else "mfma", "achieved": ach, "peak": peak,
                        "unit": "TFLOP/s", "frac": ach / peak, "traffic": None,
                        "avg_launch_ms": v["ms"] / v["launches"], "launches": v["launches"] // args.steps}
        else:
            ach = v["bytes"] / (v["ms"] * 1e-3) / 1e9
            roofline = {"kernel": name, "bound": "hbm", "achieved": ach, "peak": flops.MI355X_HBM_PEAK / 1e9,
                        "unit": "GB/s", "frac": ach / (flops.MI355X_HBM_PEAK / 1e9), "traffic": None,
                        "avg_launch_ms": v["ms"] / v["launches"], "launches": v["launches"] // args.steps}

    # HBM traffic of the dominant kernel class: rocprofv3 --pmc counters cannot be read from inside
    # this process, so the figure is the committed summary of two counter runs of this same command
    # (profiles/hbm_traffic.json names the runs and the kernel sources they measured); null if that
    # file has no entry for this workload and kernel class.
    if roofline is not None:
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
                entry = json.load(fh)[cfg.name][roofline["kernel"]]
            roofline["traffic"] = entry["hbm_bytes_per_launch"]
            roofline["traffic_source"] = entry.get("source")
        except (OSError, KeyError, ValueError):
            roofline["traffic"] = None

    # The same step with weight gradients accumulated after every micro-batch (wgrad_group = 1:
    # no operand of a second micro-batch is ever held), reported beside the headline.
    ungrouped = None
    workspace_bytes = B.query_sizes(cfg)[3]
    if cfg.wgrad_group > 1 and not args.no_ungrouped and not last:
        cfg1 = cfg.replace(wgrad_group=1)
        st.close()
        del st
        torch.cuda.empty_cache()
        st = B.Stage(cfg1, dev, params_flat=params)
        st.set_side_stream(torch.cuda.Stream(dev))
        n1 = max(2, min(args.steps, 5))
        step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(n1):
            step()
        torch.cuda.synchronize()
        ms1 = (time.perf_counter() - t1) * 1e3 / n1
        tf1 = hw_flops_mb * M / (ms1 * 1e-3) / 1e12
        ungrouped = {"wgrad_group": 1, "steps": n1, "ms_per_step": ms1, "ms_per_micro_batch": ms1 / M, "tflops": tf1,
                     "frac_of_bf16_mfma_peak": tf1 * 1e12 / flops.MI355X_BF16_DENSE_PEAK,
                     "workspace_bytes": B.query_sizes(cfg1)[3]}

    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg)

    out = {
        "metric": ("stage fwd+bwd TFLOP/s, last stage without recompute" if last else
                   "stage fwd+recompute+bwd TFLOP/s") + " (ms/micro-batch and % of bf16 MFMA peak in config)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {
            "workload": cfg.name + (" (last-stage variant: no recompute)" if last else "") +
                        (f" with dropout {cfg.dropout_p}" if cfg.dropout_p > 0 else ""), "n_layers": cfg.n_layers, "hidden": cfg.hidden, "n_heads": cfg.n_heads,
            "seq_len": cfg.seq_len, "micro_batch": cfg.micro_batch, "n_micro_batches": M,
            "mlp_hidden": cfg.mlp_hidden, "causal": cfg.causal, "wgrad_group": cfg.wgrad_group, "dropout_p": cfg.dropout_p,
            "workspace_bytes": workspace_bytes, "same_step_ungrouped": ungrouped,
            "gpu_sensors_during_timed_steps": sensors.summary(),
            "ms_per_micro_batch": ms_mb, "ms_per_step_median": ms_step_median, "ms_per_step_min": ms_step_min,
            "ms_forward_per_micro_batch": ms_f,
            ("ms_backward_per_micro_batch" if last else "ms_recompute_backward_per_micro_batch"): ms_rb,
            "frac_of_bf16_mfma_peak": frac_peak, "peak_tflops_used": flops.MI355X_BF16_DENSE_PEAK / 1e12,
            "useful_tflops_paper_convention": useful_flops_mb * M / (ms_step * 1e-3) / 1e12,
            "flops_per_micro_batch_executed": hw_flops_mb,
            "device": props.name, "compute_units": props.multi_processor_count,
            "kernel_classes": classes,
        },
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    st.close()
    print(json.dumps(out))


def _energy_joules():
    """The GPU's accumulated-energy counter in joules, or None (rocm-smi missing or no such counter)."""
    import subprocess
    try:
        out = subprocess.run(["rocm-smi", "--showenergycounter", "--json"], capture_output=True, text=True, timeout=20).stdout
        card = next(iter(json.loads(out).values()))
        for k, v in card.items():
            if "uJ" in k:
                return float(v) * 1e-6
    except Exception:
        pass
    return None


def bench_energy(args):
    """Energy per FLOP under the board power limit.  Every kernel here runs the chip into its power
    cap on normally distributed operands, so its rate is set by the energy it spends per product;
    the counter is read before and after a window of `--steps` seconds of back-to-back launches."""
    import torch
    from paper_2111_04007_amd import binding as B, flops
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    window = float(max(4, args.steps))
    gen = torch.Generator(device=dev).manual_seed(20211104)
    dt = torch.bfloat16
    rows = []

    def run(label, fn, fl):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, t0, n = _energy_joules(), time.perf_counter(), 0
        while time.perf_counter() - t0 < window:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
            n += 20
        t1, e1 = time.perf_counter(), _energy_joules()
        row = {"kernel": label, "tflops": fl * n / (t1 - t0) / 1e12, "seconds": t1 - t0}
        if e0 is not None and e1 is not None:
            row.update({"watts": (e1 - e0) / (t1 - t0), "pj_per_flop": (e1 - e0) / (fl * n) * 1e12})
        rows.append(row)

    src = torch.empty(1 << 23, device=dev, dtype=torch.float32).normal_(generator=gen).to(dt)
    sink = torch.empty(torch.cuda.get_device_properties(dev).multi_processor_count * 2 * 256, device=dev)
    fl_probe = B.probe_mfma_rate(src, 2, 20000, sink, 0)
    run("register-only MFMA loop, normal(0,1)", lambda: B.probe_mfma_rate(src, 2, 20000, sink, 0), fl_probe)
    for name, (M, N, K) in (("QKV", (2048, 24576, 8192)), ("MLP2", (2048, 8192, 32768))):
        a = torch.empty(M, K, device=dev, dtype=torch.float32).normal_(generator=gen).to(dt)
        b = (torch.empty(N, K, device=dev, dtype=torch.float32).normal_(generator=gen) * 0.01).to(dt)
        bias = torch.zeros(N, device=dev, dtype=dt)
        out = torch.empty(M, N, device=dev, dtype=dt)
        fl = 2.0 * M * N * K
        run(f"forward GEMM {name} {M}x{N}x{K}, this library (library's choice of kernel)",
            lambda: B.op_gemm(B.OP_FWD, 0, a, b, out, bias=bias, variant=0, M=M, N=N, K=K), fl)
        run(f"forward GEMM {name} {M}x{N}x{K}, 256x256 tile on 8 waves with two stages (variant 5)",
            lambda: B.op_gemm(B.OP_FWD, 0, a, b, out, bias=bias, variant=5, M=M, N=N, K=K), fl)
        run(f"same product through torch.matmul (vendor library; reference point only)",
            lambda: torch.matmul(a, b.t(), out=out), fl)
    return {"metric": "energy per FLOP at the board power limit", "value": rows[1].get("pj_per_flop"), "unit": "pJ/FLOP",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "dtype": "bf16",
            "data": "synthetic", "vs_baseline": None,
            "config": {"workload": "C5 forward GEMM shapes, back-to-back launches", "window_seconds": window,
                       "nominal_peak_tflops": flops.MI355X_BF16_DENSE_PEAK / 1e12}, "rows": rows}


def bench_tail(cfg, args):
    """Gradient statistics + Adam step over all parameters of the stage, timed with events."""
    import torch
    from paper_2111_04007_amd import binding as B, flops, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = cfg.replace(n_micro_batches=1, wgrad_group=1)
    params, _, _ = synth.device_random_stage(cfg, dev, 1)
    st = B.Stage(cfg, dev, params_flat=params)
    n = st.grads.numel()
    st.grads.normal_(0.0, 1.0)
    master = st.params.to(torch.float32)
    m = torch.zeros(n, device=dev)
    v = torch.zeros(n, device=dev)
    out = torch.zeros(2, device=dev)
    stream = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_stats = t_adam = 0.0
    for it in range(args.warmup + args.steps):
        ev[0].record(stream)
        st.grad_stats(out, stream)
        ev[1].record(stream)
        st.adam_step(master, m, v, it + 1, lr=1e-4, grad_scale=1.0 / 32, skip=out[1:], stream=stream)
        ev[2].record(stream)
        torch.cuda.synchronize()
        if it >= args.warmup:
            t_stats += ev[0].elapsed_time(ev[1])
            t_adam += ev[1].elapsed_time(ev[2])
    t_stats /= args.steps
    t_adam /= args.steps
    es = 4 if cfg.dtype == "f32" else 2
    bytes_adam = (28.0 + es) * n      # read g, w, m, v; write w, m, v, param
    bytes_stats = 4.0 * n
    ach = bytes_adam / (t_adam * 1e-3) / 1e9
    res = {"metric": "mini-batch tail: gradient statistics + Adam step (ms)", "value": t_stats + t_adam, "unit": "ms",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "dtype": "f32",
           "data": "synthetic", "vs_baseline": None,
           "config": {"workload": cfg.name + " mini-batch tail", "parameters": n, "ms_grad_stats": t_stats,
                      "ms_adam": t_adam, "grad_stats_gbps": bytes_stats / (t_stats * 1e-3) / 1e9},
           "roofline": {"kernel": "adam_kernel", "bound": "hbm", "achieved": ach, "peak": flops.MI355X_HBM_PEAK / 1e9,
                        "unit": "GB/s", "frac": ach / (flops.MI355X_HBM_PEAK / 1e9), "traffic": None}}
    st.close()
    return res


def _acc(tot, part):
    for k, v in part.items():
        t = tot.setdefault(k, {"ms": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0})
        for kk in t:
            t[kk] += v[kk]


if __name__ == "__main__":
    main()
