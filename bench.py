#!/usr/bin/env python3
"""Benchmark of the 2:4 Squared-ReLU FFN hot path on one MI355X.

A step is one forward + backward of the 2:4 FFN (all kernels of the path) on one batch of seeded synthetic
inputs that are resident in HBM before the clock starts.  Prints ONE JSON line:
  value     dense-equivalent TFLOP/s of the step (12 T D F flops per step)
  roofline  the dominant kernel (largest share of the step) against the published MFMA peak, from HIP events
            recorded inside the library on the launch stream
  cpu_baseline  the CPU oracle timed on a bounded token slice of the same workload on this host
plus the dense-MFMA FFN timed the same way (speed-up) and every kernel's own rate.
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

PEAK_BF16_DENSE = 2500.0   # TFLOP/s, MI355X published dense bf16 MFMA peak
PEAK_FP8_DENSE = 5000.0    # TFLOP/s, published dense fp8 MFMA peak
# What this chip's matrix pipes sustain with operands already in registers (no memory traffic at all), measured once
# with a probe kernel: the clocks settle at 1.5-1.9 GHz under matrix load, the published peaks assume 2.4 GHz.
# TFLOP/s executed (a sparse op executes half of its dense equivalent): dense bf16, sparse bf16, dense fp8, sparse fp8.
REGISTER_RESIDENT = {("bf16", False): 1580.0, ("bf16", True): 1815.0, ("fp8", False): 4350.0, ("fp8", True): 3780.0}
# executed MFMA flops per kernel, in units of T*D*F (dense GEMM = 2, sparse GEMM executes half of its dense equivalent)
KERNEL_FLOPS = {"up_prune24": 2.0, "down_sp": 1.0, "dh_gather": 2.0, "dx_sp": 1.0, "dw2_sp": 1.0, "dw1_sp": 1.0,
                "dense_up": 2.0, "dense_down": 2.0, "dense_dh": 2.0, "dense_dx": 2.0, "dense_dw2": 2.0, "dense_dw1": 2.0}
SPARSE = {"down_sp", "dx_sp", "dw2_sp", "dw1_sp"}


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, each
    scaled by what the same counter reads for a 1 GiB copy); None if no summary covers this kernel and workload."""
    path = os.path.join(ROOT, "profiles", f"ffn24_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith(f"hbm_bytes_per_launch {kernel} ="):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def run_c3(args) -> int:
    """Workload c3: four independent forward FFN layers at the 7B dims, each with its own seed and sparsity
    (85 / 90 / 95 / 98 % zeros); per-layer time of the 2:4 FFN against the dense MFMA FFN."""
    import torch
    from paper_2503_16672_amd import ffn24, synth
    layers = {}
    tot24 = totd = 0.0
    for name in ("c3_85", "c3_90", "c3_95", "c3_98"):
        w = synth.WORKLOADS[name]
        T, D, F = w.T, w.D, w.F
        inp = synth.make_workload(name)
        dev = {k: torch.from_numpy(inp[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2")}
        b1 = torch.from_numpy(inp["b1"]).cuda()
        ctx = ffn24.Context(T, D, F, ffn24.FFN24_DENSE)
        ctx.prepare_weights(dev["W1"], dev["W2"])      # inference: the weight pass runs once, outside the timed region
        Y = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / args.steps
        s24 = timed(lambda: ctx.ffn24_fwd(dev["X"], None, b1, None, Y))
        sd = timed(lambda: ctx.ffn_fwd(dev["X"], None, b1, None, Y))
        fl = 4.0 * T * D * F
        layers[name] = {"sparsity": w.sparsity, "ms": round(s24 * 1e3, 4), "tflops": round(fl / s24 / 1e12, 1),
                        "dense_ms": round(sd * 1e3, 4), "speedup_vs_dense_ffn": round(sd / s24, 4)}
        tot24 += s24; totd += sd
        ctx.close()
        del dev, Y
    w = synth.WORKLOADS["c3_90"]
    fl = 4 * 4.0 * w.T * w.D * w.F
    print(json.dumps({"metric": "FFN fwd dense-equiv TFLOP/s", "value": round(fl / tot24 / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(tot24 * 1e3, 4), "higher_is_better": True,
                      "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "c3: four 2:4 Squared-ReLU FFN layers, fwd, T=16384 d_model=4096 d_ff=16384, 85/90/95/98 % zeros, weights prepared once",
                                 "parallelism": "single GPU"},
                      "speedup_vs_dense_ffn": round(totd / tot24, 4), "layers": layers}))
    return 0


def run_split_sweep(args) -> int:
    """Weight-gradient stage (dW2 and dW1, K = tokens) against the number of hidden features kept dense: the split
    GEMM of the paper's second kernel benchmark (operand 90 % zeros).  Each point times, from HIP events inside the
    library, everything the split adds or changes: partition, feature-wise kernel, sparse + dense GEMMs, dW1 transpose."""
    import torch
    from paper_2503_16672_amd import ffn24, synth
    w = synth.WORKLOADS[args.workload]
    T, D, F = w.T, w.D, w.F
    inp = synth.make_workload(args.workload, with_dy=True)
    dev = {k: torch.from_numpy(inp[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2", "dY")}
    b1 = torch.from_numpy(inp["b1"]).cuda()
    ctx = ffn24.Context(T, D, F, ffn24.FFN24_TRAINING | ffn24.FFN24_DENSE | ffn24.FFN24_SPLIT)
    Y = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    grads = (torch.empty((T, D), dtype=torch.bfloat16, device="cuda"), torch.empty((D, F), dtype=torch.bfloat16, device="cuda"),
             torch.empty((F, D), dtype=torch.bfloat16, device="cuda"))
    ctx.set_profiling(True)
    flops = 4.0 * T * D * F            # dense-equivalent flops of the two weight-gradient GEMMs
    points = []
    for nd in [0, 256, 512, 1024, 2048, 4096]:
        if nd > F // 4:
            continue
        ctx.set_split(nd)
        ids = [4, 5, 6] + ([15, 16] if nd else [])
        acc = {k: 0.0 for k in ids}
        up = 0.0
        for it in range(args.warmup + args.steps):
            ctx.ffn24_fwd(dev["X"], dev["W1"], b1, dev["W2"], Y)
            ctx.ffn24_bwd(dev["dY"], grads)
            torch.cuda.synchronize()
            if it >= args.warmup:
                up += ctx.kernel_ms(0)
                for k in ids:
                    acc[k] += ctx.kernel_ms(k)
        ms = {ffn24.KERNEL_NAMES[k]: round(v / args.steps, 4) for k, v in acc.items()}
        gemm_ms = sum(v for n, v in ms.items() if n in ("dw2_sp", "dw1_sp"))
        stage_ms = sum(ms.values())
        points.append({"n_dense": nd, "dense_fraction": round(nd / F, 4), "gemms_ms": round(gemm_ms, 4), "gemms_tflops": round(flops / gemm_ms / 1e9, 1),
                       "stage_ms": round(stage_ms, 4), "up_prune24_ms": round(up / args.steps, 4), "kernels": ms})
    dd = 0.0
    for it in range(args.warmup + args.steps):
        ctx.ffn_fwd(dev["X"], dev["W1"], b1, dev["W2"], Y)
        ctx.ffn_bwd(dev["dY"], grads)
        torch.cuda.synchronize()
        if it >= args.warmup:
            dd += ctx.kernel_ms(11) + ctx.kernel_ms(12)
    dense_ms = dd / args.steps
    ctx.close()
    print(json.dumps({"metric": "split weight-gradient GEMMs, dense-equiv TFLOP/s", "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"{w.name}: dW2 + dW1 of the 2:4 FFN, T={T} d_model={D} d_ff={F}, target sparsity {w.sparsity}"},
                      "fully_dense_gemms": {"ms": round(dense_ms, 4), "tflops": round(flops / dense_ms / 1e9, 1)}, "points": points}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", help="c1, c2, c3 (four forward layers), c3_85..c3_98, c4 (default: forward+backward at the 7B FFN dims), c5 (fp8 forward)")
    ap.add_argument("--fwd-only", action="store_true", help="time the forward pass only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-tokens", type=int, default=4096, help="token slice the CPU oracle is timed on (about 15 s of CPU work at the default workload)")
    ap.add_argument("--split", type=int, default=0, help="keep this many hidden features (multiple of 256, <= d_ff/4) out of the "
                    "feature-wise 2:4: split weight-gradient GEMMs (bf16 fwd+bwd workloads)")
    ap.add_argument("--rowwise", action="store_true", help="fp8 workload with row-wise instead of per-tensor scales (no dense baseline in this mode)")
    ap.add_argument("--permute", action="store_true", help="run the bf16 workload with a fixed token permutation around the FFN")
    ap.add_argument("--telemetry", action="store_true", help="bf16 workloads: count sparsity and 2:4 drops while running (reported under \"telemetry\")")
    ap.add_argument("--split-sweep", action="store_true", help="time the weight-gradient stage over a range of split sizes")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy before the steps (the known-size kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2503_16672_amd import ffn24, synth

    ffn24.lib()  # fails loudly if libffn24.so is not built; there is no fallback path
    if args.workload == "c3":
        return run_c3(args)
    if args.split_sweep:
        return run_split_sweep(args)
    w = synth.WORKLOADS[args.workload]
    T, D, F = w.T, w.D, w.F
    fp8 = args.workload == "c5"
    bwd = not (args.fwd_only or fp8)
    rowwise = fp8 and args.rowwise
    if rowwise:
        inp = synth.make_inputs_fp8_rowwise(T, D, F, w.sparsity, w.seed)
        dev = {k: torch.from_numpy(inp[k]).cuda() for k in ("X", "W1", "W2", "sx", "sw1", "sw2")}
        ctx = ffn24.Context(T, D, F, ffn24.FFN24_ROWWISE, dtype=ffn24.FFN24_FP8_E4M3)
        ctx.set_row_scales(dev["sx"], dev["sw1"], dev["sw2"])
    elif fp8:
        inp = synth.make_inputs_fp8(T, D, F, w.sparsity, w.seed)
        dev = {k: torch.from_numpy(inp[k]).cuda() for k in ("X", "W1", "W2")}
        ctx = ffn24.Context(T, D, F, ffn24.FFN24_DENSE, dtype=ffn24.FFN24_FP8_E4M3)
        ctx.set_scales(inp["sx"], inp["sw1"], inp["sh"], inp["sw2"])
    else:
        inp = synth.make_workload(args.workload, with_dy=True)
        dev = {k: torch.from_numpy(inp[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2", "dY")}
        ctx = ffn24.Context(T, D, F, (ffn24.FFN24_TRAINING if bwd else 0) | ffn24.FFN24_DENSE | (ffn24.FFN24_SPLIT if args.split and bwd else 0)
                            | (ffn24.FFN24_PERMUTE if args.permute else 0) | (ffn24.FFN24_TELEMETRY if args.telemetry else 0))
        if args.split and bwd:
            ctx.set_split(args.split)
        if args.permute:
            ctx.set_token_permutation(synth.token_permutation(T, w.seed + 1))
    b1 = torch.from_numpy(inp["b1"]).cuda()
    peak = PEAK_FP8_DENSE if fp8 else PEAK_BF16_DENSE
    Y = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
    grads = (torch.empty((T, D), dtype=torch.bfloat16, device="cuda"), torch.empty((D, F), dtype=torch.bfloat16, device="cuda"),
             torch.empty((F, D), dtype=torch.bfloat16, device="cuda"))

    # forward-only workloads are inference: the weights do not change between calls, so their re-arrangement runs
    # once, outside the timed region (for the 2:4 FFN and the dense one alike); a training step re-arranges them
    prepared = not bwd
    if prepared:
        ctx.prepare_weights(dev["W1"], dev["W2"])
    W1a, W2a = (None, None) if prepared else (dev["W1"], dev["W2"])

    def step24():
        ctx.ffn24_fwd(dev["X"], W1a, b1, W2a, Y)
        if bwd:
            ctx.ffn24_bwd(dev["dY"], grads)

    def step_dense():
        ctx.ffn_fwd(dev["X"], W1a, b1, W2a, Y)
        if bwd:
            ctx.ffn_bwd(dev["dY"], grads)

    def timed(fn, warmup, steps):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ctx.set_profiling(True)   # event pairs around every kernel, on the launch stream; no synchronisation added
    sec24 = timed(step24, args.warmup, args.steps)
    # per-kernel durations: average over the same number of steps, reading the events after each step
    k24 = list(range(0, 7 if bwd else 2)) + ([13, 14] if bwd else []) + ([15, 16] if args.split and bwd else []) + ([17] if rowwise else [])
    kd = [] if rowwise else list(range(7, 13 if bwd else 9))
    acc = {k: 0.0 for k in k24 + kd}
    for _ in range(args.steps):
        step24()
        torch.cuda.synchronize()
        for k in k24:
            acc[k] += ctx.kernel_ms(k)
    sec_dense = timed(step_dense, args.warmup, args.steps) if not rowwise else float("nan")
    for _ in range(args.steps if not rowwise else 0):
        step_dense()
        torch.cuda.synchronize()
        for k in kd:
            acc[k] += ctx.kernel_ms(k)
    ctx.set_profiling(False)
    telemetry = None
    if args.telemetry and not fp8:
        step24()
        t = ctx.telemetry()
        telemetry = {"zeros": round(1 - t["nonzero"] / t["elements"], 5), "dropped_tokenwise": round(1 - t["kept_tokenwise"] / t["nonzero"], 6),
                     "dropped_featurewise_on_top": round(1 - t["kept_featurewise"] / t["kept_tokenwise"], 6) if t["kept_featurewise"] else None,
                     "use_sparse_at_0.85": ctx.policy_use_sparse(0.85), "counts": t}
    kernel_ms = {ffn24.KERNEL_NAMES[k]: acc[k] / args.steps for k in acc}

    # standalone 2:4 compression of a dense [T, F] activation with the workload's sparsity (HBM-bound streaming kernel;
    # launched on torch's current stream, so torch events bracket it)
    sparsify = None
    if not fp8:
        g = torch.Generator(device="cuda"); g.manual_seed(w.seed)
        keep = 1.0 - (w.sparsity if isinstance(w.sparsity, float) else 0.915)
        Hs = torch.randn((T, F), generator=g, device="cuda")
        Hs = torch.where(torch.rand((T, F), generator=g, device="cuda") < keep, Hs * Hs, torch.zeros((), device="cuda")).to(torch.bfloat16)
        for _ in range(3):
            ffn24.sparsify24(Hs)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        vals = torch.empty((T, F // 2), dtype=torch.bfloat16, device="cuda"); meta = torch.empty((T, F // 8), dtype=torch.uint8, device="cuda")
        e0.record()
        for _ in range(args.steps):
            ffn24.sparsify24(Hs, vals, meta)
        e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        gbs = 3.125 * T * F / (ms * 1e-3) / 1e9      # read 2, write 1 + 1/8 bytes per element
        sparsify = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / 8000.0, 4)}
        del Hs, vals, meta

    tdf = float(T) * D * F
    flops_step = (12.0 if bwd else 4.0) * tdf
    value = flops_step / sec24 / 1e12
    kernels = {}
    for name, ms in kernel_ms.items():
        if name in KERNEL_FLOPS:
            tf = KERNEL_FLOPS[name] * tdf / (ms * 1e-3) / 1e12
            kernels[name] = {"ms": round(ms, 4), "tflops_executed": round(tf, 1), "frac_of_dense_mfma_peak": round(tf / peak, 4),
                             "frac_of_register_resident_rate": round(tf / REGISTER_RESIDENT[("fp8" if fp8 else "bf16", name in SPARSE)], 4)}
            if name in SPARSE:
                kernels[name]["tflops_dense_equivalent"] = round(2 * tf, 1)
        else:
            # streaming kernels: feature-wise re-compression moves 4.25 bytes per element of [T, F]; a transpose pair
            # reads and writes 2 x 2 bytes per element of its two matrices
            # (the weight pass also writes panel-form copies of W1 and W2 when the context trains: 12 D F bytes then)
            es = 1.0 if fp8 else 2.0
            if name == "quantise_rows":     # reads the bf16 kept values + metadata, writes codes + metadata (+ one scale per token)
                gbs = (1.0 + 0.125 + 0.5 + 0.125) * T * F / (ms * 1e-3) / 1e9
                kernels[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / 8000.0, 4)}
                continue
            if name == "split_partition":
                kernels[name] = {"ms": round(ms, 4)}
                continue
            nbytes = {"featurewise24": 4.25 * T * F, "transpose_weights": (6.0 if bwd else 4.0) * es * D * F, "transpose_acts": 8.0 * T * D,
                      "transpose_dw1": 4.0 * D * F}[name]
            gbs = nbytes / (ms * 1e-3) / 1e9
            kernels[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / 8000.0, 4)}
    dom = max((n for n in kernel_ms if n in KERNEL_FLOPS and not n.startswith("dense_")), key=lambda n: kernel_ms[n])
    achieved = KERNEL_FLOPS[dom] * tdf / (kernel_ms[dom] * 1e-3) / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 1), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": measured_traffic(dom, w.name),
                "note": "executed MFMA flops of the launch / its HIP-event duration; a sparse kernel executes half its dense-equivalent flops"}

    cpu = None
    if not args.no_cpu:
        from oracle import ffn24_oracle as O
        Ts = min(args.cpu_tokens, T)
        t0 = time.perf_counter()
        if rowwise:
            O.ffn24_fwd_fp8_rowwise_codes(inp["X"][:Ts], inp["sx"][:Ts], inp["W1"], inp["sw1"], inp["b1"], inp["W2"], inp["sw2"])
        elif fp8:
            O.ffn24_fwd_fp8_codes(inp["X"][:Ts], inp["W1"], inp["b1"], inp["W2"], inp["sx"], inp["sw1"], inp["sh"], inp["sw2"])
        else:
            sl = {k: inp[k][:Ts] if k in ("X", "dY") else inp[k] for k in inp}
            f = O.ffn24_fwd(sl["X"], sl["W1"], sl["b1"], sl["W2"])
            if bwd:
                O.ffn24_bwd(f, sl["dY"])
        dt = time.perf_counter() - t0
        cpu = {"value": round((12.0 if bwd else 4.0) * Ts * D * F / dt / 1e12, 5), "unit": "TFLOP/s", "cores": len(os.sched_getaffinity(0)),
               "kind": "oracle", "sample": f"first {Ts} of {T} tokens of the same workload, float64 numpy, {dt:.1f} s"}

    out = {
        "metric": "FFN fwd+bwd dense-equiv TFLOP/s" if bwd else "FFN fwd dense-equiv TFLOP/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec24 * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if fp8 else "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: 2:4 Squared-ReLU FFN {'fwd+bwd' if bwd else 'fwd'}, T={T} d_model={D} d_ff={F}, target sparsity {w.sparsity}"
                               + (f", {args.split} dense features in the weight gradients" if args.split and bwd else "")
                               + (", row-wise fp8 scales" if rowwise else "") + (", fixed token permutation" if args.permute and not fp8 else "")
                               + (", weights prepared once" if prepared else ""),
                   "T": T, "d_model": D, "d_ff": F, "parallelism": "single GPU"},
        "frac_of_sparse_mfma_peak": round(value / (2 * peak), 4),
        "dense_ffn": None if rowwise else {"ms_per_step": round(sec_dense * 1e3, 4), "tflops": round(flops_step / sec_dense / 1e12, 2)},
        "speedup_vs_dense_ffn": None if rowwise else round(sec_dense / sec24, 4),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "sparsify24_standalone": sparsify,
    }
    if telemetry:
        out["telemetry"] = telemetry
    ctx.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
