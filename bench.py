#!/usr/bin/env python3
"""Benchmark of the compression step on one MI355X.

One step = one full L-C compression step (condensa_lc_step) over the large-model stress workload:
64 fp32 matrices of 4096x4608 (1.2 G weights) with multipliers, mu = 1e-3, density 0.1 -- global
selection on w - lambda/mu, theta, lambda' and the penalty gradient written out.  Inputs are seeded
synthetic tensors already resident in HBM when the timed region starts.

Prints ONE JSON line: whole-step throughput in weights/s, the roofline of the dominant kernel
(measured with HIP events on the launch stream, inside the timed region) and the CPU oracle timed on a
bounded sample of the same workload.
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

HBM_PEAK_GBPS = 8000.0           # MI355X published HBM3E peak

# HBM traffic of one k_window_fused launch on the full workload, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# calibrated with a plain copy (profiles/lc_step_large_model_hbm_counters.md).  Reported only while the
# kernel's sources still hash to what was measured, and only for the full 64-tensor workload without mask.
MEASURED_TRAFFIC = {"bytes": 24522131159, "tensors": 64,
                    "sources_sha256": "210d2707da11f78d9cde1bc77bf679492131162df606c7cce6e9c2642ce7f5f6"}
KERNEL_SOURCES = ("paper_1911_02497_amd/csrc/common.h", "paper_1911_02497_amd/csrc/k_fused.h")


def kernel_sources_hash():
    import hashlib
    m = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, f), "rb") as fh:
            m.update(fh.read())
    return m.hexdigest()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--tensors", type=int, default=64, help="number of 4096x4608 matrices (64 = the full workload)")
    ap.add_argument("--mask", action="store_true", help="also write the byte mask (+N bytes per step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tensors", type=int, default=6,
                    help="the oracle is timed on the first this-many tensors (6: ~12 s of one host core)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch plain device copies of one tensor (known bytes) for counter calibration")
    ap.add_argument("--apply-threads", type=int, default=0, help="workgroup size of the apply sweep (0 = default)")
    ap.add_argument("--all-phases", action="store_true",
                    help="time every phase with events (adds ~10 us of idle gap per event); default: the apply sweep only")
    ap.add_argument("--workload", default="lc_stress",
                    choices=["lc_stress", "prune_stress", "filter_stress", "block_stress", "single_prune_fp16", "vgg_thresholds", "vgg_masks", "resnet_filter_global",
                             "resnet_filter_per_tensor", "transformer_block8", "transformer_block32"],
                    help="lc_stress is the benchmark; *_stress run the other entry points on the same weights, the rest are the small parity workloads, timed for reference")
    ap.add_argument("--select-path", type=int, default=0, help="0 auto, 1 radix levels only, 2 sampled window")
    ap.add_argument("--window-margin", type=int, default=80,
                    help="half-width of the sampled window in 1/16 standard deviations (default 80 = 5 sigma)")
    ap.add_argument("--two-sweeps", action="store_true",
                    help="window path: separate selection and apply sweeps (default: one sweep does both)")
    return ap.parse_args()


def run_small_workload(args, P, workloads, torch, np, dev):
    """The small workloads (launch- and cache-bound): same JSON shape, step = one call of the entry point."""
    import oracle
    name = args.workload
    up = lambda arrs: P.tensor_table([torch.from_numpy(a).to(dev) for a in arrs])  # noqa: E731  (marshalled once)
    cfg = P.condensa_config(select_path=args.select_path, fused_sweep=1 if args.two_sweeps else 0,
                            window_margin=args.window_margin)
    prev = [None]                                # the first call allocates the outputs, later ones reuse them
    if name == "prune_stress":
        # global magnitude pruning of the large-model weights (no multipliers): theta + mask at density 0.1
        host, _ = workloads.lc_stress(indices=range(args.tensors), threads=16)
        d = up(host)
        call = lambda: P.condensa_prune(d, [0.1], workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
        op, F, J, bytes_per_elem, desc = P.binding.OP_PRUNE, 0, 1, 13, "global prune d=0.1, theta + mask"
        cpu = lambda: oracle.prune(host[:2], [0.1])  # noqa: E731
    elif name in ("filter_stress", "block_stress"):
        # structure pruning of the large-model weights: the matrices as 4096 filters of 512x3x3, or 8x8 blocks
        host, _ = workloads.lc_stress(indices=range(args.tensors), threads=16)
        if name == "filter_stress":
            host = [h.reshape(h.shape[0], h.shape[1] // 9, 3, 3) for h in host]
            d = up(host)
            call = lambda: P.condensa_filter_prune(d, 0.5, P.SCOPE_GLOBAL, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
            op, F, desc = P.binding.OP_FILTER_PRUNE, sum(t.shape[0] for t in host), "global filter prune d=0.5, theta + mask"
            cpu = lambda: oracle.filter_prune(host[:8], 0.5, P.SCOPE_GLOBAL)  # noqa: E731
        else:
            d = up(host)
            call = lambda: P.condensa_block_prune(d, 8, 8, 0.5, P.SCOPE_GLOBAL, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
            op, F = P.binding.OP_BLOCK_PRUNE, sum((t.shape[0] // 8) * (t.shape[1] // 8) for t in host)
            desc = "global block prune 8x8 d=0.5, theta + mask"
            cpu = lambda: oracle.block_prune(host[:8], 8, 8, 0.5, P.SCOPE_GLOBAL)  # noqa: E731
        J, bytes_per_elem = 1, 13                 # the weights are read twice (aggregate, apply): 4 + 4 + 4 theta + 1 mask
    elif name == "single_prune_fp16":
        host = workloads.single_matrix()
        d = up(host)
        call = lambda: P.condensa_prune(d, [0.02], theta=False, theta_f16=True, mask=True, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
        op, F, J, bytes_per_elem, desc = P.binding.OP_PRUNE, 0, 1, 11, "prune d=0.02 fused with fp16 theta + mask"
        cpu = lambda: oracle.quantize_f16(oracle.prune(host, [0.02])[0]["theta"][0])  # noqa: E731
    elif name in ("vgg_thresholds", "vgg_masks"):
        host = workloads.vgg19_cifar()
        d = up(host)
        ds = workloads.search_densities()
        if name == "vgg_thresholds":
            call = lambda: P.condensa_prune(d, ds, theta=False, mask=False, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
            bytes_per_elem, desc = 4, "thresholds of 10 densities from one sweep"
        else:
            call = lambda: P.condensa_prune(d, ds, theta=False, mask=True, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
            bytes_per_elem, desc = 4 + 4 + 10, "10 densities, one selection sweep + one apply sweep writing 10 masks"
        op, F, J = P.binding.OP_PRUNE, 0, len(ds)
        cpu = lambda: oracle.prune(host, ds)  # noqa: E731
    elif name.startswith("resnet_filter"):
        host = workloads.resnet56_cifar_convs()
        d = up(host)
        scope, dens = (P.SCOPE_GLOBAL, 0.3) if name.endswith("global") else (P.SCOPE_PER_TENSOR, 0.5)
        call = lambda: P.condensa_filter_prune(d, dens, scope, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
        op, F, J, bytes_per_elem = P.binding.OP_FILTER_PRUNE, sum(t.shape[0] for t in host), 1, 13
        desc = f"filter prune density {dens}, theta + mask"
        cpu = lambda: oracle.filter_prune(host, dens, scope)  # noqa: E731
    else:
        host = workloads.transformer_base()
        d = up(host)
        b = 8 if name.endswith("block8") else 32
        call = lambda: P.condensa_block_prune(d, b, b, 0.25, P.SCOPE_GLOBAL, workspace=ws, outputs=prev[0], config=cfg)  # noqa: E731
        op, F, J, bytes_per_elem = P.binding.OP_BLOCK_PRUNE, sum((t.shape[0] // b) * (t.shape[1] // b) for t in host), 1, 13
        desc = f"block prune {b}x{b} density 0.25, theta + mask"
        cpu = lambda: oracle.block_prune(host, b, b, 0.25, P.SCOPE_GLOBAL)  # noqa: E731
    N = sum(t.size for t in host)
    scope_ws = P.SCOPE_PER_TENSOR if name == "resnet_filter_per_tensor" else P.SCOPE_GLOBAL
    ws = torch.empty(max(P.condensa_workspace_bytes(op, N, F, len(host), J, scope_ws, cfg), 256), dtype=torch.uint8, device=dev)
    prev[0] = call()
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    if name == "prune_stress":
        # one sweep (window path, default) reads the weights once: 4 + 4 theta + 1 mask; two sweeps read them twice
        path = P.select_records(prev[0]["results"])[0]["path"]
        one_sweep = path == 2 and not args.two_sweeps
        bytes_per_elem = 9 if one_sweep else (13 if path == 2 else 21)
        desc += f" ({'1 sweep' if one_sweep else '2 sweeps' if path == 2 else 'radix levels'} over the weights)"
    gbps = bytes_per_elem * N / (ms * 1e-3) / 1e9
    cpu_rec = None
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        cpu()
        dt = time.perf_counter() - t0
        n_sample = {"prune_stress": 2, "filter_stress": 8, "block_stress": 8}.get(name, len(host))
        n_cpu = sum(t.size for t in host[:n_sample])
        cpu_rec = {"value": round(n_cpu / dt, 1), "unit": "weights/s", "cores": 1, "kind": "oracle",
                   "sample": (f"the first {n_sample} tensors" if name.endswith("_stress") else "the whole workload") + f" once, {dt:.2f} s",
                   "host_cpus": os.cpu_count()}
    print(json.dumps({
        "metric": "weights pruned/sec and achieved HBM GB/s (% of peak) per compression step",
        "value": round(N / (ms * 1e-3), 1), "unit": "weights/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "config": {"workload": f"{name}: {len(host)} tensors, {N} weights, {desc}",
                                        "note": "wall time per call, outputs preallocated; includes the Python binding's marshalling"},
        "roofline": {"bound": "hbm", "kernel": "whole call", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": bytes_per_elem * N},
        "cpu_baseline": cpu_rec}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: the path runs on ONE GPU only (no sharding or collectives exist); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1911_02497_amd as P
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    P.library()                                     # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload != "lc_stress":
        run_small_workload(args, P, workloads, torch, np, dev)
        return

    rows, cols, T = 4096, 4608, args.tensors
    mu, density = workloads.LC_MU, workloads.LC_DENSITY

    # ---- inputs: generated on the host from the seeded recipe, then made resident -------------------
    t0 = time.time()
    w_dev, lam_dev, cpu_w, cpu_l = [], [], [], []
    batch = 8
    for b in range(0, T, batch):
        idx = list(range(b, min(b + batch, T)))
        ws, ls = workloads.lc_stress(indices=idx, n_tensors=T, rows=rows, cols=cols, threads=16)
        for i, w, l in zip(idx, ws, ls):
            w_dev.append(torch.from_numpy(w).to(dev))
            lam_dev.append(torch.from_numpy(l).to(dev))
            if i < args.cpu_sample_tensors and not args.no_cpu_baseline:
                cpu_w.append(w)
                cpu_l.append(l)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    N = sum(t.numel() for t in w_dev)

    outputs = {
        "theta": [torch.empty_like(t) for t in w_dev],
        "grad": [torch.empty_like(t) for t in w_dev],
        "lambda": [torch.empty_like(t) for t in w_dev],
        "results": torch.zeros((1, 8), dtype=torch.int64, device=dev),
    }
    if args.mask:
        outputs["mask"] = [torch.empty(t.shape, dtype=torch.uint8, device=dev) for t in w_dev]
    cfg = P.condensa_config(select_path=args.select_path, apply_threads=args.apply_threads,
                            fused_sweep=1 if args.two_sweeps else 0, window_margin=args.window_margin)
    ws_bytes = P.condensa_workspace_bytes(P.binding.OP_LC_STEP, N, 0, T, 1, P.SCOPE_GLOBAL, cfg)
    workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step():
        return P.condensa_lc_step(w_dev, lam_dev, mu, density, outputs=outputs, mask=args.mask,
                                  workspace=workspace, config=cfg)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    if args.calibrate_copy:                         # 4 copies, each reads and writes rows*cols*4 bytes
        for i in range(4):
            outputs["theta"][i].copy_(w_dev[i])
        torch.cuda.synchronize()

    P.condensa_profile_reset()
    cfg.profile = 0x1F if args.all_phases else ((1 << 3) | (1 << 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    cfg.profile = 0
    phases = P.condensa_profile_read()

    ms_per_step = elapsed * 1e3 / args.steps
    rec = P.select_records(outputs["results"])[0]
    assert rec["k"] == int(np.floor(density * N + 0.5)) and rec["n"] == N, rec

    # ---- roofline of the dominant kernel --------------------------------------------------------------
    # One-sweep window path (default): k_window_fused reads w, lambda (8 B) and writes theta, lambda', g
    # (12 B) [+1 mask] per weight, and that is also all the step needs.  Two sweeps (radix path, or
    # --two-sweeps): k_lc_apply moves the same 20 B and the selection reads w, lambda once more (28 B a step).
    one_sweep = rec["path"] == 2 and not args.two_sweeps
    kernel_bytes_per_elem = 20 + (1 if args.mask else 0)
    step_bytes_per_elem = kernel_bytes_per_elem + (0 if one_sweep else 8)
    kernel_name, phase = ("k_window_fused", "sweep") if one_sweep else ("k_lc_apply", "apply")
    kp = phases[phase]
    kernel_ms = kp["ms"] / max(kp["intervals"], 1)
    achieved = kernel_bytes_per_elem * N / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    traffic = None
    if (T == MEASURED_TRAFFIC["tensors"] and not args.mask and one_sweep
            and kernel_sources_hash() == MEASURED_TRAFFIC["sources_sha256"]):
        traffic = MEASURED_TRAFFIC["bytes"]
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "avg_launch_ms": round(kernel_ms, 4), "algorithmic_bytes_per_launch": kernel_bytes_per_elem * N}
    step_gbps = step_bytes_per_elem * N / (ms_per_step * 1e-3) / 1e9
    phase_ms = {k: round(v["ms"] / args.steps, 4) for k, v in phases.items() if v["intervals"]}

    # ---- CPU oracle on a bounded sample of the same workload -----------------------------------------
    cpu = None
    if not args.no_cpu_baseline and cpu_w:
        import oracle
        t0 = time.perf_counter()
        oracle.lc_step(cpu_w, cpu_l, mu, density)
        dt = time.perf_counter() - t0
        n_cpu = sum(t.size for t in cpu_w)
        cpu = {"value": round(n_cpu / dt, 1), "unit": "weights/s", "cores": 1, "kind": "oracle",
               "sample": f"first {len(cpu_w)} of the {T} tensors ({n_cpu} weights), one L-C step, {dt:.1f} s",
               "host_cpus": os.cpu_count()}

    out = {
        "metric": "weights pruned/sec and achieved HBM GB/s (% of peak) per compression step",
        "value": round(N / (ms_per_step * 1e-3), 1),
        "unit": "weights/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"L-C compression step, {T} fp32 tensors of {rows}x{cols} ({N} weights) + multipliers, "
                               f"mu={mu}, density={density}, outputs theta/lambda'/grad" + ("/mask" if args.mask else ""),
                   "select_path": {1: "radix", 2: "window"}.get(rec["path"], str(rec["path"])),
                   "sweeps_over_the_weights": 1 if one_sweep else (2 if rec["path"] == 2 else 4),
                   "threshold_key": rec["threshold_key"], "n_tie": rec["n_tie"]},
        "step_algorithmic_GBps": round(step_gbps, 1),
        "step_frac_of_hbm_peak": round(step_gbps / HBM_PEAK_GBPS, 4),
        "step_bytes_per_weight": step_bytes_per_elem,
        # the same time against the 28 B/weight of a select-then-apply step (weights and multipliers read twice)
        "step_GBps_at_two_read_accounting": round((28 + (1 if args.mask else 0)) * N / (ms_per_step * 1e-3) / 1e9, 1),
        "phase_ms_per_step": phase_ms,
        "input_generation_s": round(gen_s, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
