#!/usr/bin/env python3
"""Benchmark of the fused attention forward + JVP on one MI355X.

A "step" is one call of attn_jvp_fwd (the whole hot path: Q/tQ load, KV streaming, six contractions,
online softmax, epilogue) on one batch of synthetic input already resident in HBM.
Prints ONE JSON line: attention+JVP TFLOP/s counting 12*Lq*Lkv*d flops per head, the roofline of the
dominant kernel (the sweep; timed by HIP events the library records around it) against the bf16 dense MFMA
peak, and the fp64 CPU oracle timed on a bounded row sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 MFMA: 256 CU x 2.4 GHz x 4096 flop/clk/CU


PEAK_FP32_TFLOPS = 157.3     # MI355X dense fp32 MFMA
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E


def bench_rmsnorm(args, cfg, dev):
    """RMSNorm + JVP over every (batch, head, token) row of the workload's q and tq: reads x, tx, writes y, ty."""
    import numpy as np
    import torch
    from paper_2510_08431_amd import binding
    from paper_2510_08431_amd.workloads import make_inputs
    t = make_inputs(cfg)
    x, tx = t["q"].to(dev), t["tq"].to(dev)
    w = (1.0 + 0.1 * torch.randn(cfg.d, generator=torch.Generator().manual_seed(7))).to(dev)
    y, ty = torch.empty_like(x), torch.empty_like(tx)
    eps = 1e-6
    rows = x.numel() // cfg.d
    nbytes = 4 * x.numel() * x.element_size()

    def step():
        binding.attn_jvp_rmsnorm_fwd(x, tx, w, eps, out=(y, ty))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in evs:          # one kernel per step, launched on torch's current stream: the events bracket it
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in evs]
    ms_per_step = wall * 1e3 / args.steps
    gbs = nbytes / (ms_per_step * 1e-3) / 1e9
    kern_gbs = nbytes / (float(np.mean(kern_ms)) * 1e-3) / 1e9
    out = {
        "metric": "RMSNorm+JVP GB/s (x, tx read, y, ty written once)", "value": round(gbs, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"qk-norm of {cfg.name}", "rows": rows, "d": cfg.d},
        "roofline": {"bound": "hbm", "achieved": round(kern_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(kern_gbs / PEAK_HBM_GBS, 4), "traffic": None, "kernel": "rmsnorm_jvp_kernel",
                     "kernel_ms_avg": round(float(np.mean(kern_ms)), 4), "kernel_ms_min": round(float(np.min(kern_ms)), 4)},
    }
    if not args.no_cpu_baseline:
        from oracle.rmsnorm_jvp_ref import rmsnorm_jvp_ref
        n = min(rows, 2_000_000)
        xs = t["q"].reshape(-1, cfg.d)[:n].double().numpy()
        txs = t["tq"].reshape(-1, cfg.d)[:n].double().numpy()
        ws = w.cpu().double().numpy()
        c0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - c0 < 10.0:
            rmsnorm_jvp_ref(xs, txs, ws, eps)
            reps += 1
        cpu_s = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(reps * 4 * n * cfg.d * x.element_size() / cpu_s / 1e9, 3), "unit": "GB/s",
                               "cores": torch.get_num_threads(), "kind": "oracle",
                               "sample": f"{n} rows x {reps} repetitions, fp64 numpy, {cpu_s:.1f} s "
                                         "(bytes counted as for the bf16 kernel)"}
    print(json.dumps(out))


def sustained_mfma_rates(torch, binding, dev, iters=150000, with_gemm=False):
    """What the chip at hand sustains on back-to-back dense 8-pass MFMAs (the library's rate probe: one wave per SIMD
    on every compute unit, nothing else in the loop), by operand VALUES: all-zero operands run at the full clock,
    N(0,1) operands at the clock the power limit leaves.  TFLOP/s each; optionally the same comparison on a library
    GEMM (torch.matmul, 8192^3)."""
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    out = torch.empty(256 * cus, dtype=torch.float32, device=dev)
    g = torch.Generator(device="cpu")
    g.manual_seed(4242)
    vals = torch.randn(8 * 256 * 8, generator=g)
    ops = {"bf16_zero_operands": (torch.zeros(8 * 256 * 8, dtype=torch.bfloat16), 0),
           "bf16_normal_operands": (vals.to(torch.bfloat16), 0),
           "fp16_normal_operands": (vals.to(torch.float16), 1)}
    res = {}
    for name, (x, f16) in ops.items():
        x = x.to(dev)
        binding.attn_jvp_mfma_rate_probe(x, out, f16, 2000)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = binding.attn_jvp_mfma_rate_probe(x, out, f16, iters)
        e1.record()
        torch.cuda.synchronize()
        res[name + "_tflops"] = round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    if with_gemm:
        n = 8192
        for dt, nm in ((torch.bfloat16, "bf16"), (torch.float16, "fp16")):
            for kind in ("zero", "normal"):
                a = torch.zeros(n, n, device=dev, dtype=dt) if kind == "zero" else torch.randn(n, n, device=dev).to(dt)
                b = a if kind == "zero" else torch.randn(n, n, device=dev).to(dt)
                for _ in range(5):
                    a @ b
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(60):
                    a @ b
                e1.record()
                torch.cuda.synchronize()
                res[f"library_gemm_8192_{nm}_{kind}_operands_tflops"] = round(2.0 * n ** 3 * 60 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (default 3: video-DiT self-attention); 6: the same shape at head dimension 64 (24 heads)")
    ap.add_argument("--variant", choices=["default", "bf16-pairs", "fast"], default="default",
                    help="MFMA kernel variant: default (workspace lent by the binding: fp16 value path from 2048 keys, or 256 with many query tiles, "
                         "on, bf16 pairs below), bf16-pairs (no workspace), fast (single bf16 weights; outside the "
                         "tolerance on peaked rows)")
    ap.add_argument("--fast", action="store_true", help="same as --variant fast")
    ap.add_argument("--null-kv-tangents", action="store_true",
                    help="pass tk = tv = NULL instead of the tensors (only meaningful where they are zero: config 4); "
                         "the kernel then executes 8*Lq*Lkv*d flop per head, the metric still counts 12")
    ap.add_argument("--layout", choices=["bhld", "blhd"], default="bhld",
                    help="memory layout of the eight tensors: [B,H,L,d] (default) or [B,L,H,d]")
    ap.add_argument("--input-dtype", choices=["config", "fp32"], default="config",
                    help="fp32: hold the workload's inputs (the same values) in fp32, which takes the fp32 matrix-core kernel; "
                         "priced against the fp32 MFMA peak")
    ap.add_argument("--op", choices=["attention", "rmsnorm"], default="attention",
                    help="attention (default: the headline metric) or rmsnorm: the RMSNorm + JVP kernel on the q tensor "
                         "of the chosen workload (its QK-normalisation), an HBM-bound second workload with its own line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy (known traffic) for scaling HBM counters")
    ap.add_argument("--mfma-calibration", action="store_true",
                    help="run only the sustained-MFMA-rate measurement (the library's rate probe with all-zero and N(0,1) "
                         "operands, and a library GEMM on the same two kinds of data) and print it as one JSON line")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "hbm_traffic.json"),
                    help="optional file with measured HBM bytes per launch, {workload: bytes}")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_08431_amd import binding
    from paper_2510_08431_amd.workloads import CONFIGS, make_inputs, make_head, sample_rows

    if args.copy_calibration:
        # a plain copy of known size: reads 1 GiB, writes 1 GiB per launch
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(3)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dst.copy_(src)
        e0.record()
        for _ in range(3):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        # (the rate is context for the HBM-bound kernels: what a plain library copy reaches on this machine)
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 4,
                          "copy_GBps_read_plus_write": round(2.0 * n * 3 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)}))
        return

    binding.load_library()          # fails loudly when the HIP library is missing
    cfg = CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.mfma_calibration:
        print(json.dumps({"mfma_sustained": sustained_mfma_rates(torch, binding, dev, iters=400000, with_gemm=True),
                          "published_peak_tflops": PEAK_BF16_TFLOPS}))
        return
    if args.op == "rmsnorm":
        bench_rmsnorm(args, cfg, dev)
        return
    t = {n: x.to(dev) for n, x in make_inputs(cfg).items()}
    B, H, Lq, Lkv, d = cfg.B, cfg.H, cfg.Lq, cfg.Lkv, cfg.d
    f32 = cfg.dtype != "bf16" or args.input_dtype == "fp32"
    if f32:
        t = {n: x.float() for n, x in t.items()}
    workload = cfg.name + ("-as-fp32" if f32 and cfg.dtype == "bf16" else "")
    layout = binding.LAYOUT_BHLD
    if args.layout == "blhd":
        t = {n: x.permute(0, 2, 1, 3).contiguous() for n, x in t.items()}
        layout = binding.LAYOUT_BLHD
    o = torch.empty(t["q"].shape, dtype=torch.float32, device=dev)
    to = torch.empty_like(o)
    lse = torch.empty(B, H, Lq, dtype=torch.float32, device=dev)
    if args.fast:
        args.variant = "fast"
    flags = {"default": 0, "bf16-pairs": binding.FLAG_NO_F16, "fast": binding.FLAG_FAST}[args.variant]

    if args.null_kv_tangents and (t["tk"].any() or t["tv"].any()):
        print("bench.py: --null-kv-tangents needs a workload whose tk and tv are zero (config 4)", file=sys.stderr)
        sys.exit(2)
    tk, tv = (None, None) if args.null_kv_tangents else (t["tk"], t["tv"])

    def step(events=None):
        binding.attn_jvp_fwd_ex(t["q"], t["k"], t["v"], t["tq"], tk, tv, cfg.scale, out=(o, to, lse),
                                flags=flags, timing_events=events, layout=layout)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # whole-job wall clock over exactly K steps (pre-pass kernels of the fp16 value path included), plus HIP events
    # that the library records on the launch stream right before and after the dominant kernel of every step
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in evs:          # create the underlying HIP events outside the timed region
        a.record()
        b.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for ev in evs:
        step(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [a.elapsed_time(b) for a, b in evs]
    ms_per_step = wall * 1e3 / args.steps
    kern_avg_ms = float(np.mean(kern_ms))
    tflops = cfg.flops / (ms_per_step * 1e-3) / 1e12
    kern_tflops = cfg.flops / (kern_avg_ms * 1e-3) / 1e12

    # Outside the timed region: the same K steps once more without the event pairs, whose records sit between the
    # pre-pass and the sweep and cost short workloads a noticeable share of a step (nothing on the 15 ms headline)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_plain = (time.perf_counter() - t0) * 1e3 / args.steps

    # Outside the timed region: the same workload through the two entry points that take no workspace from the caller.
    # attn_jvp_fwd (the plain 15-argument call) runs the hi + lo bf16-pair kernel; attn_jvp_fwd_static runs the same
    # kernels as the timed steps on the library's static scratch array (if the shape fits it).
    other_entries = {}
    if not f32 and args.variant == "default" and layout == binding.LAYOUT_BHLD and not args.null_kv_tangents:
        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - c0) * 1e3 / reps
            tf = cfg.flops / (ms * 1e-3) / 1e12
            return {"ms_per_call": round(ms, 4), "tflops": round(tf, 2), "pct_of_bf16_mfma_peak": round(100 * tf / PEAK_BF16_TFLOPS, 2)}
        reps = max(2, min(args.steps, 5))
        with torch.cuda.stream(torch.cuda.default_stream(dev)):
            other_entries["attn_jvp_fwd"] = dict(timed(lambda: binding.attn_jvp_fwd(
                t["q"], t["k"], t["v"], t["tq"], tk, tv, cfg.scale, out=(o, to, lse)), reps), workspace="none (bf16 pairs)")
        if binding.attn_jvp_workspace_bytes(B, H, Lq, Lkv, d) <= binding.attn_jvp_static_scratch_bytes():
            other_entries["attn_jvp_fwd_static"] = dict(timed(lambda: binding.attn_jvp_fwd_static(
                t["q"], t["k"], t["v"], t["tq"], tk, tv, cfg.scale, out=(o, to, lse)), reps), workspace="library's static array")

    traffic = None
    try:
        with open(args.traffic_json) as f:
            traffic = json.load(f).get(workload)
    except OSError:
        pass

    peak = PEAK_FP32_TFLOPS if f32 else PEAK_BF16_TFLOPS
    # what the path computes in (inputs; matrix products; accumulation), by the route the library takes for this call
    if f32:
        arithmetic = "f32 (fp32 MFMA, fp32 accumulate)" if d in (32, 64, 96, 128) else "f32 (vector ALU)"
    elif not (d in (32, 64, 96, 128) and cfg.scale > 0):
        arithmetic = "bf16 in, f32 vector ALU"
    elif args.variant == "fast":
        arithmetic = "bf16 in, bf16 MFMA (single bf16 weights), f32 accumulate"
    elif args.variant == "bf16-pairs" or not (Lkv >= 2048 or (Lkv >= 256 and B * H * ((Lq + 127) // 128) >= 4 * 256)):   # the library's rule
        arithmetic = "bf16 in, bf16 MFMA (weights as hi+lo bf16 pairs in the value products), f32 accumulate"
    else:
        arithmetic = "bf16 in, bf16 score MFMA + fp16 value MFMA (fp16 weights, V and tV as scaled fp16 copies), f32 accumulate"
    if f32:
        kernel_name = "attn_jvp_mfma_f32_kernel" if d in (32, 64, 96, 128) else "attn_jvp_fp32_kernel"
    else:
        kernel_name = "attn_jvp_mfma_kernel" if d in (32, 64, 96, 128) and cfg.scale > 0 else "attn_jvp_fp32_kernel"
    out = {
        "metric": f"attention+JVP TFLOP/s ({'fp32' if f32 else 'bf16'}, 12*Lq*Lkv*d/head)", "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": arithmetic, "data": "synthetic",
        "config": {"workload": workload, "B": B, "H": H, "Lq": Lq, "Lkv": Lkv, "d": d,
                   "variant": args.variant, "kv_tangents": "null" if args.null_kv_tangents else "tensors", "layout": args.layout},
        "pct_of_bf16_mfma_peak": round(100 * tflops / PEAK_BF16_TFLOPS, 2),
        # the same K steps without the HIP event pairs around the sweep kernel (not the headline: `value` is the timed region)
        "ms_per_step_without_kernel_events": round(ms_per_step_plain, 4),
        "tflops_without_kernel_events": round(cfg.flops / (ms_per_step_plain * 1e-3) / 1e12, 2),
        # counted: 12 Lq Lkv d per head (all six products); with tk = tv = NULL four of the six are executed
        "tflops_executed": round(tflops * (8.0 / 12.0 if args.null_kv_tangents else 1.0), 2),
        "roofline": {"bound": "mfma", "achieved": round(kern_tflops, 2), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(kern_tflops / peak, 4), "traffic": traffic,
                     "kernel": kernel_name,
                     "kernel_ms_avg": round(kern_avg_ms, 4), "kernel_ms_min": round(float(np.min(kern_ms)), 4),
                     "kernel_ms_median": round(float(np.median(kern_ms)), 4)},
    }

    if other_entries:
        out["entry_points_without_caller_workspace"] = other_entries
    if not f32 and kernel_name == "attn_jvp_mfma_kernel":
        # Outside the timed region: the rate this chip sustains on nothing but dense MFMAs, by operand values.  `frac`
        # above stays against the published peak; this says how much of that peak is reachable on real data here.
        sus = sustained_mfma_rates(torch, binding, dev)
        fp16_path = arithmetic.startswith("bf16 in, bf16 score MFMA + fp16")
        ref = (2.0 / (1.0 / sus["bf16_normal_operands_tflops"] + 1.0 / sus["fp16_normal_operands_tflops"])
               if fp16_path else sus["bf16_normal_operands_tflops"])     # half the products of the fp16 path are fp16 MFMAs
        sus["same_mix_of_mfma_types_tflops"] = round(ref, 1)
        out["mfma_sustained"] = sus
        out["roofline"]["frac_of_sustained_mfma_rate"] = round(kern_tflops / ref, 4)

    if not args.no_cpu_baseline:
        # the fp64 oracle, as it stands, on a bounded sample of the same workload: a seeded set of query rows
        # (all keys) of the first few heads, sized for roughly 10-20 s of host work
        from oracle.attn_jvp_ref import attn_jvp_ref
        rows_per_head = min(Lq, max(16, int(5.0e11 / (12.0 * Lkv * d))))
        rows = sample_rows(cfg, rows_per_head)[:rows_per_head]
        n_heads = min(B * H, max(6, int(5.0e11 / (12.0 * len(rows) * Lkv * d))))     # short sequences: more heads
        heads = [{n: x[None, None] for n, x in make_head(cfg, i // H, i % H).items()} for i in range(n_heads)]
        attn_jvp_ref(*(heads[0][n] for n in ("q", "k", "v", "tq", "tk", "tv")), cfg.scale, rows=rows[:8])
        c0 = time.perf_counter()
        for hd in heads:
            attn_jvp_ref(hd["q"], hd["k"], hd["v"], hd["tq"], hd["tk"], hd["tv"], cfg.scale, rows=rows)
        cpu_s = time.perf_counter() - c0
        n_eval = len(rows) * n_heads
        cpu_tflops = 12.0 * n_eval * Lkv * d / cpu_s / 1e12
        out["cpu_baseline"] = {"value": round(cpu_tflops, 5), "unit": "TFLOP/s", "cores": torch.get_num_threads(),
                               "kind": "oracle",
                               "sample": f"{len(rows)} query rows x all {Lkv} keys of each of {n_heads} heads, fp64 numpy, {cpu_s:.1f} s",
                               "full_workload_s_extrapolated": round(cfg.flops / (cpu_tflops * 1e12), 1)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
