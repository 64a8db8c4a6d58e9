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
NOMINAL_MHZ = 2400.0       # the clock the published peaks assume; under matrix load the chip runs well below it
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


def _time_steps(torch, fn, warmup, steps):
    """Mean wall-clock seconds per call over `steps` calls bracketed by device synchronisation, then -- in a second pass of
    the same length -- every call timed on its own with events on the launch stream (median, min)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    mean = (time.perf_counter() - t0) / steps
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    each = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(steps))
    return mean, each[len(each) // 2], each[0]


def run_c3(args) -> int:
    """Workload c3: four independent forward FFN layers at the 7B dims, each with its own seed, weights, buffers and
    sparsity (85 / 90 / 95 / 98 % zeros).  A step is one pass over the four layers in turn, so that between two calls of
    a layer the other three (0.8 GB of operands and intermediates each) have gone through the 256 MB last-level cache:
    no layer finds its operands cached, and no explicit cache flush is used.  Per-layer times come from events around
    each layer's call inside those same steps."""
    import torch
    from paper_2503_16672_amd import ffn24, synth
    names = ("c3_85", "c3_90", "c3_95", "c3_98")
    L = []
    for name in names:
        w = synth.WORKLOADS[name]
        inp = synth.make_workload(name)
        dev = {k: torch.from_numpy(inp[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2")}
        dev["b1"] = torch.from_numpy(inp["b1"]).cuda()
        ctx = ffn24.Context(w.T, w.D, w.F, ffn24.FFN24_DENSE)
        ctx.prepare_weights(dev["W1"], dev["W2"])      # inference: the weight pass runs once, outside the timed region
        dev["Y"] = torch.empty((w.T, w.D), dtype=torch.bfloat16, device="cuda")
        L.append((name, w, dev, ctx))
        del inp
    w = L[0][1]
    T, D, F = w.T, w.D, w.F

    def run(dense: bool):
        per = {name: [] for name in names}
        evs = []

        def step(record):
            for name, _, dev, ctx in L:
                if record:
                    e0 = torch.cuda.Event(enable_timing=True); e0.record()
                (ctx.ffn_fwd if dense else ctx.ffn24_fwd)(dev["X"], None, dev["b1"], None, dev["Y"])
                if record:
                    e1 = torch.cuda.Event(enable_timing=True); e1.record()
                    evs.append((name, e0, e1))
        for _ in range(args.warmup):
            step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(False)
        torch.cuda.synchronize()
        mean = (time.perf_counter() - t0) / args.steps
        for _ in range(args.steps):
            step(True)
        torch.cuda.synchronize()
        for name, e0, e1 in evs:
            per[name].append(e0.elapsed_time(e1))
        return mean, {k: sorted(v) for k, v in per.items()}
    s24, per24 = run(False)
    sd, perd = run(True)
    fl = 4.0 * T * D * F
    layers = {}
    for name, wl, _, ctx in L:
        a, b = per24[name], perd[name]
        layers[name] = {"sparsity": wl.sparsity, "ms_median": round(a[len(a) // 2], 4), "ms_min": round(a[0], 4),
                        "tflops": round(fl / (a[len(a) // 2] * 1e-3) / 1e12, 1), "dense_ms_median": round(b[len(b) // 2], 4),
                        "speedup_vs_dense_ffn": round(b[len(b) // 2] / a[len(a) // 2], 4)}
        ctx.close()
    print(json.dumps({"metric": "FFN fwd dense-equiv TFLOP/s", "value": round(4 * fl / s24 / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(s24 * 1e3, 4), "higher_is_better": True,
                      "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "c3: four 2:4 Squared-ReLU FFN layers, fwd, T=16384 d_model=4096 d_ff=16384, 85/90/95/98 % zeros, "
                                             "weights prepared once, layers cycled (separate buffers, no cache flush)",
                                 "parallelism": "single GPU"},
                      "dense_ffn": {"ms_per_step": round(sd * 1e3, 4)}, "speedup_vs_dense_ffn": round(sd / s24, 4), "layers": layers}))
    return 0


def run_vendor_gemms(args) -> int:
    """Context for the dense baseline: the six GEMMs of a dense fwd+bwd at the workload's shapes through torch.matmul (the vendor's
    GEMM library), unfused, on operands with the workload's statistics.  Not part of the product or of its baseline."""
    import torch
    from paper_2503_16672_amd import synth
    w = synth.WORKLOADS[args.workload if args.workload in ("c2", "c4") else "c4"]
    T, D, F = w.T, w.D, w.F
    inp = synth.make_workload(w.name, with_dy=True)
    X, W1, W2, dY = (torch.from_numpy(inp[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2", "dY"))
    b1 = torch.from_numpy(inp["b1"]).cuda()
    H = (torch.clamp((X @ W1).float() + b1, min=0) ** 2).to(torch.bfloat16)
    dZ = ((dY @ W2.t()).float() * 2 * torch.sqrt(H.float())).to(torch.bfloat16)
    cases = (("up X W1", X, W1), ("down H W2", H, W2), ("dH dY W2^T", dY, W2.t()), ("dX dZ W1^T", dZ, W1.t()), ("dW2 H^T dY", H.t(), dY), ("dW1 X^T dZ", X.t(), dZ))
    out = {"vendor_gemms": f"torch.matmul, bf16, {w.name}: T={T} d_model={D} d_ff={F}", "gemms": {}}
    total = 0.0
    for name, a, b in cases:
        for _ in range(5):
            a @ b
        ts = []
        for _ in range(20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); a @ b; e1.record(); torch.cuda.synchronize(); ts.append(e0.elapsed_time(e1))
        ts.sort()
        out["gemms"][name] = {"ms_median": round(ts[10], 4), "ms_min": round(ts[0], 4), "tflops": round(2.0 * T * D * F / ts[10] / 1e9, 1)}
        total += ts[10]
    out["sum_ms"] = round(total, 4)
    print(json.dumps(out))
    return 0


def run_probe(args) -> int:
    """What the machine delivers, measured with the library's own probe kernels: register-resident matrix-op rates, the
    GEMM core with ingredients of its main loop removed (at the workload's sparse-GEMM and up-projection shapes), and a
    plain streaming copy."""
    from paper_2503_16672_amd import ffn24, synth
    w = synth.WORKLOADS[args.workload if args.workload in synth.WORKLOADS else "c4"]
    T, D, F = w.T, w.D, w.F
    out = {"probe": "machine rates", "workload_shapes": {"T": T, "d_model": D, "d_ff": F}, "mfma_register_resident": {}, "gemm_decomposition": {}}
    for kind, name in enumerate(ffn24.MFMA_KINDS):
        r = ffn24.probe_mfma_rate(kind)
        out["mfma_register_resident"][name] = {k: round(v, 2) for k, v in r.items()}
    for label, sparse, (M, N, K) in (("sparse_down T x d_model over d_ff", True, (T, D, F)), ("dense_down T x d_model over d_ff", False, (T, D, F)),
                                     ("dense_up d_ff x T over d_model", False, (F, T, D))):
        rows = {}
        for vname, v in ffn24.GEMM_PROBE_VARIANTS.items():
            if v == 512 and not sparse:
                continue   # a sparse-loop variant
            r = ffn24.probe_gemm(sparse, v, M, N, K)
            rows[vname] = {"ms": round(r["ms"], 4), "mhz": round(r["mhz"]), "tflops_dense_equivalent": round(2.0 * M * N * K / (r["ms"] * 1e-3) / 1e12, 1)}
        out["gemm_decomposition"][label] = rows
        # global->LDS fill of a CU: what one 1024-cycle stage of the loop needs (sparse: 16 KiB stored values + 2 KiB metadata +
        # 32 KiB of B for 64 k; dense: 16 + 16 KiB for 32 k) against what the stream alone delivers when every line hits the L2
        stage_bytes, stage_k = (51200, 64) if sparse else (32768, 32)
        per_cu = (M // 256) * (N // 256) / 256.0 * (K // stage_k) * stage_bytes
        alone = rows["dma_only_l2_hits"]
        out.setdefault("lds_fill_bytes_per_clk_per_cu", {})[label] = {
            "needed_at_full_matrix_rate": round(stage_bytes / 1024.0, 1),
            "stream_alone_all_l2_hits": round(per_cu / (alone["ms"] * 1e-3 * alone["mhz"] * 1e6), 1),
            "stream_alone_all_l2_hits_GBps_per_cu": round(per_cu / (alone["ms"] * 1e-3) / 1e9, 1),
            "product_loop": round(per_cu / (rows["all"]["ms"] * 1e-3 * rows["all"]["mhz"] * 1e6), 1)}
    # the same loop under other tile walks (rocprofv3 --pmc FETCH_SIZE on this command gives each walk's L2 fills: the
    # kernels differ in their last template argument)
    out["tile_walks"] = {}
    for label, sparse, (M, N, K) in (("sparse_down", True, (T, D, F)), ("dense_up", False, (F, T, D))):
        out["tile_walks"][label] = {wname: round(ffn24.probe_gemm(sparse, v, M, N, K)["ms"], 4) for wname, v in ffn24.GEMM_PROBE_WALKS.items()}
    nbytes = 1 << 30
    ms = ffn24.probe_copy(nbytes)
    out["copy_1GiB"] = {"ms": round(ms, 4), "GBps_read_plus_write": round(2 * nbytes / (ms * 1e-3) / 1e9, 1)}
    print(json.dumps(out))
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


def run_fwd_sweep(args) -> int:
    """FFN forward, 2:4 against dense, over model dimensions and token counts (what the paper's forward-speed-up figure plots:
    larger models and larger batches gain more), in the paper's precision recipe (fp8 with row-wise scales) and in bf16; d_ff = 4
    d_model, 90 % zeros, weights prepared once (inference).  Synthetic inputs by the workloads' recipe."""
    import torch
    from paper_2503_16672_amd import ffn24, synth
    points = []
    for D in (2048, 4096, 8192):
        F = 4 * D
        for T in (4096, 8192, 16384):
            row = {"T": T, "d_model": D, "d_ff": F}
            for mode in ("fp8_rowwise", "bf16"):
                if mode == "bf16":
                    inp = synth.make_inputs(T, D, F, 0.9, seed=7000 + D + T)
                    dev = {k: torch.from_numpy(inp[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2")}
                    ctx = ffn24.Context(T, D, F, ffn24.FFN24_DENSE)
                else:
                    inp = synth.make_inputs_fp8_rowwise(T, D, F, 0.9, seed=7000 + D + T)
                    dev = {k: torch.from_numpy(inp[k]).cuda() for k in ("X", "W1", "W2", "sx", "sw1", "sw2")}
                    ctx = ffn24.Context(T, D, F, ffn24.FFN24_ROWWISE | ffn24.FFN24_DENSE, dtype=ffn24.FFN24_FP8_E4M3)
                    ctx.set_row_scales(dev["sx"], dev["sw1"], dev["sw2"])
                b1 = torch.from_numpy(inp["b1"]).cuda()
                Y = torch.empty((T, D), dtype=torch.bfloat16, device="cuda")
                ctx.prepare_weights(dev["W1"], dev["W2"])
                _, m24, _ = _time_steps(torch, lambda: ctx.ffn24_fwd(dev["X"], None, b1, None, Y), args.warmup, args.steps)
                _, md, _ = _time_steps(torch, lambda: ctx.ffn_fwd(dev["X"], None, b1, None, Y), args.warmup, args.steps)
                row[mode] = {"ms_24": round(m24 * 1e3, 4), "ms_dense": round(md * 1e3, 4), "speedup": round(md / m24, 4),
                             "tflops_dense_equivalent": round(4.0 * T * D * F / m24 / 1e12, 1)}
                ctx.close()
                del dev, ctx
                torch.cuda.empty_cache()
            points.append(row)
            print(f"# T={T} d_model={D}: {row}", file=sys.stderr, flush=True)
    print(json.dumps({"metric": "FFN fwd speed-up over the dense FFN", "unit": "x", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "data": "synthetic", "config": {"workload": "forward sweep: d_ff = 4 d_model, 90 % zeros, weights prepared once; median of per-call event times"},
                      "points": points}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--vendor-gemms", action="store_true", help="context only: time the six GEMMs of a dense fwd+bwd through torch.matmul (the vendor library)")
    ap.add_argument("--probe", action="store_true", help="print the machine rates the probe kernels measure (matrix-op issue rate, GEMM "
                    "main-loop decomposition, copy rate) instead of running the workload")
    ap.add_argument("--workload", default="c4", help="c1, c2, c3 (four forward layers), c3_85..c3_98, c4 (default: forward+backward at the 7B FFN dims), c5 (fp8 forward)")
    ap.add_argument("--fwd-only", action="store_true", help="time the forward pass only")
    ap.add_argument("--fp8-bwd", action="store_true", help="workload c5: time forward + backward in fp8 (per-tensor scales), 2:4 FFN and dense fp8 baseline")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--cpu-tokens", type=int, default=4096, help="token slice the CPU oracle is timed on (about 15 s of CPU work at the default workload)")
    ap.add_argument("--split", type=int, default=0, help="keep this many hidden features (multiple of 256, <= d_ff/4) out of the "
                    "feature-wise 2:4: split weight-gradient GEMMs (bf16 fwd+bwd workloads, and c5 with --fp8-bwd --rowwise)")
    ap.add_argument("--rowwise", action="store_true", help="fp8 workload with row-wise instead of per-tensor scales (2:4 FFN and dense baseline alike); with --fp8-bwd: forward and backward with every GEMM scaled row-wise, 2:4 FFN and dense baseline")
    ap.add_argument("--permute", action="store_true", help="run the bf16 workload (or c5 with --fp8-bwd --rowwise) with a fixed token permutation around the FFN")
    ap.add_argument("--telemetry", action="store_true", help="bf16 workloads: count sparsity and 2:4 drops while running (reported under \"telemetry\")")
    ap.add_argument("--split-sweep", action="store_true", help="time the weight-gradient stage over a range of split sizes")
    ap.add_argument("--fwd-sweep", action="store_true", help="forward speed-up over the dense FFN across model dimensions and token counts (fp8 row-wise and bf16)")
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
    if args.probe:
        return run_probe(args)
    if args.vendor_gemms:
        return run_vendor_gemms(args)
    if args.workload == "c3":
        return run_c3(args)
    if args.split_sweep:
        return run_split_sweep(args)
    if args.fwd_sweep:
        return run_fwd_sweep(args)
    w = synth.WORKLOADS[args.workload]
    T, D, F = w.T, w.D, w.F
    fp8 = args.workload == "c5"
    bwd = not args.fwd_only and (not fp8 or args.fp8_bwd)
    rowwise = fp8 and args.rowwise and not bwd
    rowwise_bwd = fp8 and args.rowwise and bwd     # row-wise scaling in every GEMM of the forward and the backward (2:4 FFN only)
    no_dense = False
    if rowwise_bwd:
        inp = synth.make_inputs_fp8_rowwise(T, D, F, w.sparsity, w.seed)
        bwo = synth.make_bwd_operands_fp8_rowwise(T, D, F, w.sparsity, w.seed)
        dev = {k: torch.from_numpy(inp[k]).cuda() for k in ("X", "W1", "W2", "sx", "sw1", "sw2")}
        devb = {k: torch.from_numpy(v).cuda() for k, v in bwo.items()}
        ctx = ffn24.Context(T, D, F, ffn24.FFN24_ROWWISE | ffn24.FFN24_TRAINING | ffn24.FFN24_DENSE | (ffn24.FFN24_SPLIT if args.split else 0)
                            | (ffn24.FFN24_PERMUTE if args.permute else 0), dtype=ffn24.FFN24_FP8_E4M3)
        ctx.set_row_scales(dev["sx"], dev["sw1"], dev["sw2"])
        if args.split:
            ctx.set_split(args.split)
        if args.permute:
            ctx.set_token_permutation(synth.token_permutation(T, w.seed + 1))
    elif rowwise:
        inp = synth.make_inputs_fp8_rowwise(T, D, F, w.sparsity, w.seed)
        dev = {k: torch.from_numpy(inp[k]).cuda() for k in ("X", "W1", "W2", "sx", "sw1", "sw2")}
        ctx = ffn24.Context(T, D, F, ffn24.FFN24_ROWWISE | ffn24.FFN24_DENSE, dtype=ffn24.FFN24_FP8_E4M3)
        ctx.set_row_scales(dev["sx"], dev["sw1"], dev["sw2"])
    elif fp8:
        inp = synth.make_inputs_fp8(T, D, F, w.sparsity, w.seed)
        if bwd:   # incoming gradient ~ N(0, 1) quantised per tensor; static dZ scale with the same headroom as the activation's
            dY = np.random.Generator(np.random.Philox(w.seed + 7)).standard_normal((T, D), dtype=np.float32)
            inp["sdy"] = float(np.abs(dY).max() / 448.0)
            inp["dY"] = torch.from_numpy(dY / np.float32(inp["sdy"])).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            inp["sdz"] = 8.0 * 4.0 / 448.0      # |dH| up to about 4, derivative 2 max(0, z) up to about 8
            del dY
        dev = {k: torch.from_numpy(inp[k]).cuda() for k in ("X", "W1", "W2") + (("dY",) if bwd else ())}
        ctx = ffn24.Context(T, D, F, (ffn24.FFN24_TRAINING if bwd else 0) | ffn24.FFN24_DENSE, dtype=ffn24.FFN24_FP8_E4M3)
        ctx.set_scales(inp["sx"], inp["sw1"], inp["sh"], inp["sw2"])
        if bwd:
            ctx.set_bwd_scales(inp["sdy"], inp["sdz"])
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
        if rowwise_bwd:
            ctx.ffn24_bwd_rowwise(devb["dY8r"], devb["sdy_t"], devb["dY8c"], devb["sdy_d"], devb["X8c"], devb["sx_d"], devb["W2_8r"], devb["sw2_f"],
                                  devb["W1_8c"], devb["sw1_d"], out=grads)
        elif bwd:
            ctx.ffn24_bwd(dev["dY"], grads)

    def step_dense():
        ctx.ffn_fwd(dev["X"], W1a, b1, W2a, Y)
        if rowwise_bwd:
            ctx.ffn_bwd_rowwise(devb["dY8r"], devb["sdy_t"], devb["dY8c"], devb["sdy_d"], devb["X8c"], devb["sx_d"], devb["W2_8r"], devb["sw2_f"],
                                devb["W1_8c"], devb["sw1_d"], out=grads)
        elif bwd:
            ctx.ffn_bwd(dev["dY"], grads)

    if args.calib_copy:
        ffn24.probe_copy(1 << 30, 1)

    # what the matrix pipes of THIS chip sustain right now with operands in registers (no memory traffic): the live
    # denominator beside the published peak
    reg = {}
    for kind in ((2, 3) if fp8 else (0, 1)):
        reg[kind & 1] = ffn24.probe_mfma_rate(kind, 8000)

    # timed region: profiling off, nothing but the steps
    sec24, med24, min24 = _time_steps(torch, step24, args.warmup, args.steps)
    sec_dense, med_dense, min_dense = (_time_steps(torch, step_dense, args.warmup, args.steps) if not no_dense else (float("nan"),) * 3)
    # separate pass: event pairs around every kernel (on the launch stream) and a clock sample in every GEMM kernel
    ctx.set_profiling(True)
    k24 = list(range(0, 7 if bwd else 2)) + ([13, 14] if bwd else []) + ([15, 16] if args.split and bwd else []) + ([17] if rowwise or rowwise_bwd else []) + ([18, 19, 20] if rowwise_bwd else []) + ([21] if fp8 else [])
    kd = [] if no_dense else list(range(7, 13 if bwd else 9))      # (the dense row-wise quantisation kernel shares id 17 with the 2:4 one)
    acc = {k: [] for k in k24 + kd}
    mhz = {k: [] for k in k24 + kd}
    for fn, ids in ((step24, k24), (step_dense, kd)):
        for _ in range(min(args.steps, 20) if ids else 0):
            fn()
            torch.cuda.synchronize()
            for k in ids:
                acc[k].append(ctx.kernel_ms(k))
                m = ctx.kernel_mhz(k)
                if m:
                    mhz[k].append(m)
    ctx.set_profiling(False)
    telemetry = None
    if args.telemetry and not fp8:
        step24()
        t = ctx.telemetry()
        telemetry = {"zeros": round(1 - t["nonzero"] / t["elements"], 5), "dropped_tokenwise": round(1 - t["kept_tokenwise"] / t["nonzero"], 6),
                     "dropped_featurewise_on_top": round(1 - t["kept_featurewise"] / t["kept_tokenwise"], 6) if t["kept_featurewise"] else None,
                     "use_sparse_at_0.85": ctx.policy_use_sparse(0.85), "counts": t}
    kernel_ms = {ffn24.KERNEL_NAMES[k]: sum(v) / len(v) for k, v in acc.items()}
    kernel_mhz = {ffn24.KERNEL_NAMES[k]: sum(v) / len(v) for k, v in mhz.items() if v}

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

    # what the caller of the row-wise recipe does before a step (not part of the step, the same for the 2:4 and the dense FFN): the
    # eight row-wise / column-wise quantisations of its bf16 tensors, with the library's quantiser
    operand_quant = None
    if rowwise_bwd:
        fl = synth.make_inputs(T, D, F, w.sparsity, w.seed, with_dy=True)
        m16 = {k: torch.from_numpy(fl[k]).to(torch.bfloat16).cuda() for k in ("X", "W1", "W2", "dY")}
        del fl
        jobs = (("X", 1), ("W1", 0), ("W2", 0), ("dY", 1), ("dY", 0), ("X", 0), ("W2", 1), ("W1", 1))
        outs = [(torch.empty(m16[k].shape, dtype=torch.uint8, device="cuda"), torch.empty((m16[k].shape[0] if ax == 1 else m16[k].shape[1],), dtype=torch.float32, device="cuda"))
                for k, ax in jobs]
        def quant_all():
            for (k, ax), (cd, sc_) in zip(jobs, outs):
                ffn24.quantise_e4m3(m16[k], ax, cd, sc_)
        for _ in range(3):
            quant_all()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            quant_all()
        e1.record(); torch.cuda.synchronize()
        qms = e0.elapsed_time(e1) / 10
        qbytes = sum((3.0 if ax == 1 else 5.0) * m16[k].numel() for k, ax in jobs)      # rows: read 2, write 1; columns: read 2 twice, write 1
        operand_quant = {"ms": round(qms, 4), "GBps": round(qbytes / (qms * 1e-3) / 1e9, 1),
                         "what": "X per row, W1 and W2 per column (forward); dY per row and per column, X per column, W2 and W1 per row (backward), from bf16"}
        del m16, outs

    tdf = float(T) * D * F
    flops_step = (12.0 if bwd else 4.0) * tdf
    value = flops_step / sec24 / 1e12
    kernels = {}
    for name, ms in kernel_ms.items():
        if name in KERNEL_FLOPS:
            tf = KERNEL_FLOPS[name] * tdf / (ms * 1e-3) / 1e12
            sp = name in SPARSE
            rr = reg[1 if sp else 0]["tflops_dense_equivalent"] / (2.0 if sp else 1.0)      # executed flops of the register-resident loop
            kernels[name] = {"ms": round(ms, 4), "tflops_executed": round(tf, 1), "frac_of_dense_mfma_peak": round(tf / peak, 4),
                             "frac_of_register_resident_rate": round(tf / rr, 4)}
            if name in kernel_mhz:
                kernels[name]["sclk_mhz"] = round(kernel_mhz[name])
                kernels[name]["frac_of_peak_at_that_clock"] = round(tf / (peak * kernel_mhz[name] / NOMINAL_MHZ), 4)
            if name in SPARSE:
                kernels[name]["tflops_dense_equivalent"] = round(2 * tf, 1)
        else:
            # streaming kernels: feature-wise re-compression moves 4.25 bytes per element of [T, F]; a transpose pair
            # reads and writes 2 x 2 bytes per element of its two matrices
            # (the weight pass also writes panel-form copies of W1 and W2 when the context trains: 12 D F bytes then)
            es = 1.0 if fp8 else 2.0
            if name in ("quantise_rows", "quantise_dz_rows", "quantise_transposed"):
                # reads the bf16 kept values + metadata, writes codes + metadata (+ one scale per row); the transposed pair runs twice
                gbs = (2.0 if name == "quantise_transposed" else 1.0) * (1.0 + 0.125 + 0.5 + 0.125) * T * F / (ms * 1e-3) / 1e9
                kernels[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / 8000.0, 4)}
                continue
            if name == "split_partition":
                kernels[name] = {"ms": round(ms, 4)}
                continue
            nbytes = {"panelise_bwd_weights": 2.0 * D * F + 2.0 * T * D, "panelise_x": 2.0 * T * D, "featurewise24": (2.0 * (2.0 if rowwise_bwd else es) + 0.25) * T * F, "transpose_weights": (6.0 if bwd and not rowwise_bwd else 4.0) * es * D * F,
                      # (per-tensor fp8: the pass over dY8 also leaves its panel-form copy)
                      "transpose_acts": (5.0 if fp8 and not rowwise_bwd else 4.0) * es * T * D, "transpose_dw1": 4.0 * D * F}[name]
            gbs = nbytes / (ms * 1e-3) / 1e9
            kernels[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / 8000.0, 4)}
    dom = max((n for n in kernel_ms if n in KERNEL_FLOPS and not n.startswith("dense_")), key=lambda n: kernel_ms[n])
    achieved = KERNEL_FLOPS[dom] * tdf / (kernel_ms[dom] * 1e-3) / 1e12
    traffic = measured_traffic(dom, w.name)
    es = 1.0 if fp8 else 2.0
    # algorithmic HBM bytes of a launch of the dominant kernel (an up-projection or dH GEMM): both operands once, the
    # compressed activation (values + metadata) written, and for the dH GEMM the saved activation read as well
    alg = es * (D * F + T * D) + (es / 2 + 0.125) * T * F + ((1.0 + 0.125) * T * F if dom == "dh_gather" else 0.0)
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 1), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": traffic,
                "algorithmic_bytes": alg, "traffic_over_algorithmic": round(traffic / alg, 2) if traffic else None,
                "sclk_mhz": round(kernel_mhz[dom]) if dom in kernel_mhz else None,
                "frac_of_peak_at_that_clock": round(achieved / (peak * kernel_mhz[dom] / NOMINAL_MHZ), 4) if dom in kernel_mhz else None,
                "note": "executed MFMA flops of the launch / its HIP-event duration (a sparse kernel executes half its dense-equivalent flops); "
                        "peak is the published one at 2.4 GHz, sclk_mhz the clock the kernel really ran at"}

    cpu = None
    if not args.no_cpu:
        from oracle import ffn24_oracle as O
        Ts = min(args.cpu_tokens, T)
        t0 = time.perf_counter()
        if rowwise or rowwise_bwd:
            f8 = O.ffn24_fwd_fp8_rowwise_codes(inp["X"][:Ts], inp["sx"][:Ts], inp["W1"], inp["sw1"], inp["b1"], inp["W2"], inp["sw2"])
            if rowwise_bwd:
                O.ffn24_bwd_fp8_rowwise_codes(f8, bwo["dY8r"][:Ts], bwo["sdy_t"][:Ts], bwo["W2_8r"], bwo["sw2_f"], bwo["W1_8c"], bwo["sw1_d"],
                                              bwo["dY8c"][:Ts], bwo["sdy_d"], bwo["X8c"][:Ts], bwo["sx_d"])
        elif fp8:
            f8 = O.ffn24_fwd_fp8_codes(inp["X"][:Ts], inp["W1"], inp["b1"], inp["W2"], inp["sx"], inp["sw1"], inp["sh"], inp["sw2"])
            if bwd:
                O.ffn24_bwd_fp8_codes(f8, inp["X"][:Ts], inp["W1"], inp["W2"], inp["dY"][:Ts], inp["sx"], inp["sw1"], inp["sh"], inp["sw2"], inp["sdy"], inp["sdz"])
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
        "ms_per_step": round(sec24 * 1e3, 4), "ms_per_step_median": round(med24 * 1e3, 4), "ms_per_step_min": round(min24 * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if fp8 else "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: 2:4 Squared-ReLU FFN {'fwd+bwd' if bwd else 'fwd'}, T={T} d_model={D} d_ff={F}, target sparsity {w.sparsity}"
                               + (f", {args.split} dense features in the weight gradients" if args.split and bwd else "")
                               + (", row-wise fp8 scales" if rowwise or rowwise_bwd else "") + (", fixed token permutation" if args.permute and (not fp8 or rowwise_bwd) else "")
                               + (", weights prepared once" if prepared else ""),
                   "T": T, "d_model": D, "d_ff": F, "parallelism": "single GPU"},
        "frac_of_sparse_mfma_peak": round(value / (2 * peak), 4),
        "dense_ffn": None if no_dense else {"ms_per_step": round(sec_dense * 1e3, 4), "ms_per_step_median": round(med_dense * 1e3, 4),
                                           "ms_per_step_min": round(min_dense * 1e3, 4), "tflops": round(flops_step / sec_dense / 1e12, 2)},
        "register_resident_mfma": {("sparse" if k else "dense"): {a: round(b, 2) for a, b in v.items()} for k, v in reg.items()},
        "speedup_vs_dense_ffn": None if no_dense else round(sec_dense / sec24, 4),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "sparsify24_standalone": sparsify,
    }
    if telemetry:
        out["telemetry"] = telemetry
    if operand_quant:
        out["operand_quantisation_outside_the_step"] = operand_quant
    ctx.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
