#!/usr/bin/env python3
"""Benchmark of the compression step on one MI355X.

One step = one full L-C compression step (condensa_lc_step) over the large-model stress workload:
64 fp32 matrices of 4096x4608 (1.2 G weights) with multipliers, mu = 1e-3, density 0.1 -- global
selection on w - lambda/mu, theta, lambda' and the penalty gradient written out.  Inputs are seeded
synthetic tensors already resident in HBM when the timed region starts.

Prints ONE JSON line: whole-step throughput in weights/s (mean over the timed steps, with median and
minimum beside it), the roofline of the dominant kernel (measured with HIP events on the launch stream,
inside the timed region), the CPU oracle timed on bounded samples of the same workload, and under
"extras" the other half of the target on the same resident weights -- global magnitude pruning at
density 0.1 with its own roofline -- plus the four small workloads (wall time per call, launches,
oracle time).

Other modes: --workload NAME times one entry point alone (what the rocprofv3 runs wrap), and
--summarize-* turn rocprofv3 output into the short summaries kept under profiles/.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X published HBM3E peak
METRIC = "weights pruned/sec and achieved HBM GB/s (% of peak) per compression step"
N_STRESS = 64 * 4096 * 4608

# The HBM-counter summary that `roofline.traffic` is read from, and the sources whose hash ties it to the
# kernel it was taken from (reported as null once they differ).
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "lc_step_large_model_hbm_counters.md")
PRUNE_TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "prune_large_model_hbm_counters.md")
KERNEL_SOURCES = ("paper_1911_02497_amd/csrc/common.h", "paper_1911_02497_amd/csrc/k_fused.h")
SMALL_WORKLOADS = ("single_prune_fp16", "vgg_thresholds", "vgg_masks", "resnet_filter_global",
                   "resnet_filter_per_tensor", "transformer_block8", "transformer_block32")


def kernel_sources_hash():
    m = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, f), "rb") as fh:
            m.update(fh.read())
    return m.hexdigest()


def measured_traffic(kernel, tensors, other_outputs, profile=TRAFFIC_PROFILE):
    """HBM bytes per launch of `kernel` from the committed counter summary, or None when the summary is
    missing, describes another workload, or was taken from other kernel sources."""
    try:
        text = open(profile).read()
        rec = json.loads(text.split("```json", 1)[1].split("```", 1)[0])
    except (OSError, IndexError, ValueError):
        return None
    if rec.get("sources_sha256") != kernel_sources_hash() or rec.get("tensors") != tensors or other_outputs:
        return None
    return next((v for k, v in rec.get("traffic_bytes_per_launch", {}).items() if kernel.startswith(k)), None)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--tensors", type=int, default=64, help="number of 4096x4608 matrices (64 = the full workload)")
    ap.add_argument("--mask", action="store_true", help="also write the byte mask (+N bytes per step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="time the L-C step only")
    ap.add_argument("--cpu-sample-tensors", type=int, nargs=2, default=[3, 6],
                    help="the oracle is timed on the first A and the first B tensors (3 and 6: ~6 s + ~13 s of one core)")
    ap.add_argument("--cpu-all-cores", action="store_true",
                    help="also run one independent oracle step per host core at once (reported, never a target)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch plain device copies of one tensor (known bytes) for counter calibration")
    ap.add_argument("--apply-threads", type=int, default=0, help="workgroup size of the apply sweep (0 = default)")
    ap.add_argument("--all-phases", action="store_true",
                    help="time every phase with events (adds ~10 us of idle gap per event); default: the dominant kernel only")
    ap.add_argument("--workload", default="lc_stress",
                    choices=["lc_stress", "prune_stress", "filter_stress", "block_stress", "lc_pq_stress"] + list(SMALL_WORKLOADS),
                    help="lc_stress is the benchmark; *_stress run the other entry points on the same weights, the rest are "
                         "the small parity workloads, timed for reference")
    ap.add_argument("--select-path", type=int, default=0, help="0 auto, 1 radix levels only, 2 sampled window")
    ap.add_argument("--window-margin", type=int, default=80,
                    help="half-width of the sampled window in 1/16 standard deviations (default 80 = 5 sigma)")
    ap.add_argument("--two-sweeps", action="store_true",
                    help="window path: separate selection and apply sweeps (default: one sweep does both)")
    ap.add_argument("--summarize-trace", metavar="DIR", nargs="+",
                    help="rocprofv3 --kernel-trace --stats output directories (several: one section each, named after the "
                         "directory, with {W} in --command standing for that name)")
    ap.add_argument("--summarize-pmc", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="output directories of the rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs")
    ap.add_argument("--summarize-counters", metavar="DIR", help="output directory of a rocprofv3 --pmc run: per-kernel averages of every counter")
    ap.add_argument("--title", default="", help="summaries: heading")
    ap.add_argument("--command", default="", help="summaries: the profiled command, quoted in the file")
    ap.add_argument("--bytes-per-launch", action="append", default=[], metavar="KERNEL=BYTES",
                    help="summaries: algorithmic bytes of one launch of a kernel (substring of its name)")
    ap.add_argument("--out", help="summaries: file to write (under profiles/)")
    return ap.parse_args()


# ---- timing ----------------------------------------------------------------------------------------------

def timed_calls(call, steps, warmup, torch, before_timed=None):
    """warmup untimed calls, then `steps` calls between two synchronisations (the mean), with one event
    after every call on the launch stream (median and minimum of the per-call intervals)."""
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    if before_timed:
        before_timed()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        call()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    return {"mean": wall_ms / steps, "median": statistics.median(per), "min": min(per)}


def host_info():
    ram_gb = None
    try:
        with open("/proc/meminfo") as fh:
            for line in fh:
                if line.startswith("MemTotal:"):
                    ram_gb = round(int(line.split()[1]) / 2 ** 20, 1)
    except OSError:
        pass
    return {"host_cpus": os.cpu_count(), "host_ram_GiB": ram_gb}


# ---- the small workloads and the other entry points on the stress weights ---------------------------------------

def make_workload(name, args, P, workloads, torch, dev, resident=None):
    """Returns (call, info) for one workload: `call()` enqueues one call of the entry point with every output
    and the workspace preallocated; info carries the sizes, the algorithmic bytes and the oracle call."""
    import oracle
    up = lambda arrs: P.tensor_table([torch.from_numpy(a).to(dev) for a in arrs])  # noqa: E731  (marshalled once)
    cfg = P.condensa_config(select_path=args.select_path, fused_sweep=1 if args.two_sweeps else 0,
                            window_margin=args.window_margin, apply_threads=args.apply_threads,
                            profile=(1 << 1) if name == "prune_stress" else 0)
    prev, ws = [None], [None]
    F, J, scope_ws, sample, host = 0, 1, P.SCOPE_GLOBAL, None, None
    if name.endswith("_stress") and resident is None:
        host, _ = workloads.lc_stress(indices=range(args.tensors), threads=16)
    if name == "prune_stress":
        # global magnitude pruning of the large-model weights (no multipliers): theta + mask at density 0.1
        d = resident if resident is not None else up(host)
        call = lambda: P.condensa_prune(d, [0.1], workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
        op, bytes_per_elem, desc = P.binding.OP_PRUNE, 9, "global prune d=0.1, theta + mask"
        sample = lambda: workloads.lc_stress(indices=range(2), threads=2)[0]  # noqa: E731
        cpu = lambda hs: oracle.prune(hs, [0.1])  # noqa: E731
    elif name in ("filter_stress", "block_stress"):
        # structure pruning of the large-model weights: the matrices as 4096 filters of 512x3x3, or 8x8 blocks
        as_filters = lambda t: t.reshape(t.shape[0], t.shape[1] // 9, 3, 3)  # noqa: E731  (a view, on the host and on the device)
        if name == "filter_stress":
            d = P.tensor_table([as_filters(t) for t in resident]) if resident is not None else up([as_filters(h) for h in host])
            call = lambda: P.condensa_filter_prune(d, 0.5, P.SCOPE_GLOBAL, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
            op, F, desc = P.binding.OP_FILTER_PRUNE, sum(t.shape[0] for t in d), "global filter prune d=0.5, theta + mask"
            cpu = lambda hs: oracle.filter_prune([as_filters(h) for h in hs], 0.5, P.SCOPE_GLOBAL)  # noqa: E731
        else:
            d = resident if resident is not None else up(host)
            call = lambda: P.condensa_block_prune(d, 8, 8, 0.5, P.SCOPE_GLOBAL, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
            op, F = P.binding.OP_BLOCK_PRUNE, sum((t.shape[0] // 8) * (t.shape[1] // 8) for t in d)
            desc = "global block prune 8x8 d=0.5, theta + mask"
            cpu = lambda hs: oracle.block_prune(hs, 8, 8, 0.5, P.SCOPE_GLOBAL)  # noqa: E731
        n_cpu = 8 if resident is None else 2
        head = host[:n_cpu] if host is not None else None
        sample = (lambda: head) if head is not None else (lambda: workloads.lc_stress(indices=range(n_cpu), threads=2)[0])  # noqa: E731
        bytes_per_elem = 13                       # the weights are read twice (aggregate, apply): 4 + 4 + 4 theta + 1 mask
    elif name == "single_prune_fp16":
        host = workloads.single_matrix()
        d = up(host)
        call = lambda: P.condensa_prune(d, [0.02], theta=False, theta_f16=True, mask=True, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
        op, bytes_per_elem, desc = P.binding.OP_PRUNE, 11, "prune d=0.02 fused with fp16 theta + mask"
        cpu = lambda hs: oracle.quantize_f16(oracle.prune(hs, [0.02])[0]["theta"][0])  # noqa: E731
    elif name in ("vgg_thresholds", "vgg_masks"):
        host = workloads.vgg19_cifar()
        d = up(host)
        ds = workloads.search_densities()
        if name == "vgg_thresholds":
            call = lambda: P.condensa_prune(d, ds, theta=False, mask=False, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
            bytes_per_elem, desc = 4, "thresholds of 10 densities from one sweep"
        else:
            call = lambda: P.condensa_prune(d, ds, theta=False, mask=True, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
            bytes_per_elem, desc = 4 + 4 + 10, "10 densities, one selection sweep + one apply sweep writing 10 masks"
        op, J = P.binding.OP_PRUNE, len(ds)
        cpu = lambda hs: oracle.prune(hs, ds)  # noqa: E731
    elif name.startswith("resnet_filter"):
        host = workloads.resnet56_cifar_convs()
        d = up(host)
        scope, dens = (P.SCOPE_GLOBAL, 0.3) if name.endswith("global") else (P.SCOPE_PER_TENSOR, 0.5)
        scope_ws = scope
        call = lambda: P.condensa_filter_prune(d, dens, scope, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
        op, F, bytes_per_elem = P.binding.OP_FILTER_PRUNE, sum(t.shape[0] for t in host), 13
        desc = f"filter prune density {dens}, theta + mask"
        cpu = lambda hs: oracle.filter_prune(hs, dens, scope)  # noqa: E731
    elif name.startswith("transformer_block"):
        host = workloads.transformer_base()
        d = up(host)
        b = 8 if name.endswith("block8") else 32
        call = lambda: P.condensa_block_prune(d, b, b, 0.25, P.SCOPE_GLOBAL, workspace=ws[0], outputs=prev[0], config=cfg)  # noqa: E731
        op, F, bytes_per_elem = P.binding.OP_BLOCK_PRUNE, sum((t.shape[0] // b) * (t.shape[1] // b) for t in host), 13
        desc = f"block prune {b}x{b} density 0.25, theta + mask"
        cpu = lambda hs: oracle.block_prune(hs, b, b, 0.25, P.SCOPE_GLOBAL)  # noqa: E731
    else:
        raise ValueError(name)
    N = sum(t.numel() for t in d)
    ws[0] = torch.empty(max(P.condensa_workspace_bytes(op, N, F, len(d), J, scope_ws, cfg), 256), dtype=torch.uint8, device=dev)
    prev[0] = call()                              # the first call allocates the outputs, later ones reuse them
    if sample is None:
        whole = host
        sample = lambda: whole  # noqa: E731
    return call, {"N": N, "tensors": len(d), "bytes_per_elem": bytes_per_elem, "desc": desc, "cpu": cpu,
                  "sample": sample, "result": prev, "whole_sample": not name.endswith("_stress")}


def time_workload(name, args, P, workloads, torch, dev, steps, warmup, resident=None, with_oracle=True):
    call, info = make_workload(name, args, P, workloads, torch, dev, resident)
    torch.cuda.synchronize()
    l0 = P.condensa_launch_count()
    call()
    launches = P.condensa_launch_count() - l0
    torch.cuda.synchronize()
    if args.calibrate_copy and name.endswith("_stress"):     # 4 plain copies of one 4096x4608 fp32 tensor, for the counters
        src = torch.empty((4096, 4608), dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
    t = timed_calls(call, steps, warmup, torch, before_timed=P.condensa_profile_reset)
    phases = P.condensa_profile_read()
    N, bpe = info["N"], info["bytes_per_elem"]
    if name == "prune_stress":
        # one sweep (window path, default) reads the weights once: 4 + 4 theta + 1 mask; two sweeps read them twice
        path = P.select_records(info["result"][0]["results"])[0]["path"]
        one_sweep = path == 2 and not args.two_sweeps
        bpe = 9 if one_sweep else (13 if path == 2 else 21)
        info["desc"] += f" ({'1 sweep' if one_sweep else '2 sweeps' if path == 2 else 'radix levels'} over the weights)"
    gbps = bpe * N / (t["mean"] * 1e-3) / 1e9
    rec = {"workload": f"{name}: {info['tensors']} tensors, {N} weights, {info['desc']}",
           "ms_per_call": round(t["mean"], 4), "ms_per_call_median": round(t["median"], 4), "ms_per_call_min": round(t["min"], 4),
           "kernel_launches_per_call": launches, "weights_per_s": round(N / (t["mean"] * 1e-3), 1),
           "algorithmic_bytes_per_call": bpe * N, "algorithmic_GBps": round(gbps, 1),
           "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    if name == "prune_stress" and phases["sweep"]["intervals"]:
        k_ms = phases["sweep"]["ms"] / phases["sweep"]["intervals"]
        k_bpe = 9 if bpe == 9 else 4
        k_gbps = k_bpe * N / (k_ms * 1e-3) / 1e9
        rec["roofline"] = {"bound": "hbm", "kernel": "k_window_fused<prune>" if bpe == 9 else "selection sweep(s)",
                           "achieved": round(k_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                           "frac": round(k_gbps / HBM_PEAK_GBPS, 4),
                           "traffic": measured_traffic("k_window_fused", info["tensors"], False, PRUNE_TRAFFIC_PROFILE) if bpe == 9 else None,
                           "avg_launch_ms": round(k_ms, 4),
                           "launches_averaged": phases["sweep"]["intervals"], "algorithmic_bytes_per_launch": k_bpe * N}
    if with_oracle:
        hs = info["sample"]()
        t0 = time.perf_counter()
        info["cpu"](hs)
        dt = time.perf_counter() - t0
        n_cpu = sum(h.size for h in hs)
        rec["cpu_oracle"] = {"value": round(n_cpu / dt, 1), "unit": "weights/s", "ms": round(dt * 1e3, 2), "cores": 1,
                             "kind": "oracle",
                             "sample": ("the whole workload" if info["whole_sample"] else f"the first {len(hs)} tensors") + ", once"}
    return rec, t


def time_other_entry_points(P, torch, w_dev, dev):
    """The remaining entry points on the resident stress weights (or on a part of them): codecs, the non-zero
    count, the L-step update, thinning of one VGG-sized layer.  Kernel time by events on the stream the calls
    use, outputs allocated by the binding (torch's caching allocator: no device allocation after the first call)."""
    out = []

    def timed(name, fn, nbytes, n, reps=5):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbps = nbytes / (ms * 1e-3) / 1e9
        out.append({"entry_point": name, "elements": n, "ms_per_call": round(ms, 4), "algorithmic_bytes_per_call": nbytes,
                    "algorithmic_GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)})

    ws = list(w_dev)
    N = sum(t.numel() for t in ws)
    flat = torch.cat([w.reshape(-1) for w in ws[:16]])        # 302 M weights as one tensor
    n1 = flat.numel()
    timed("condensa_quantize (binary16 codes + values)", lambda: P.condensa_quantize(flat), 10 * n1, n1)
    timed("condensa_quantize (binary16 codes only)", lambda: P.condensa_quantize(flat, want_dq=False), 6 * n1, n1)
    q16 = P.condensa_quantize(flat, want_dq=False)[0]
    timed("condensa_dequantize (binary16)", lambda: P.condensa_dequantize(q16), 6 * n1, n1)
    timed("condensa_quantize_bf16 (codes + values)", lambda: P.condensa_quantize_bf16(flat), 10 * n1, n1)
    timed("condensa_quantize_fp8 E4M3 (codes + values)", lambda: P.condensa_quantize_fp8(flat, P.FP8_E4M3), 9 * n1, n1)
    q8 = P.condensa_quantize_fp8(flat, P.FP8_E4M3, want_dq=False)[0]
    timed("condensa_dequantize_fp8 E4M3", lambda: P.condensa_dequantize_fp8(q8, P.FP8_E4M3), 5 * n1, n1)
    del flat, q16, q8
    timed("condensa_count_nonzero (fp32)", lambda: P.condensa_count_nonzero(w_dev), 4 * N, N)
    half = [w.clone() for w in ws[:32]]                       # the update writes the weights: work on copies
    gl = [torch.randn_like(w) for w in half]
    th = [torch.zeros_like(w) for w in half]
    lam = [torch.zeros_like(w) for w in half]
    buf = [torch.zeros_like(w) for w in half]
    n2 = sum(w.numel() for w in half)
    timed("condensa_lc_sgd_step", lambda: P.condensa_lc_sgd_step(half, gl, th, lam, buf, 1e-3, 0.01, 0.9), 28 * n2, n2)
    del half, gl, th, lam, buf
    conv = torch.randn(512, 512, 3, 3, device=dev)
    keep = torch.arange(0, 512, 2, dtype=torch.int32, device=dev)
    n3 = 256 * 256 * 9
    timed("condensa_thin (512x512x3x3 -> 256x256x3x3)", lambda: P.condensa_thin(conv, keep, keep), 8 * n3, n3, reps=20)
    return out


def run_single_workload(args, P, workloads, torch, dev):
    """One entry point alone, same JSON shape as the benchmark line (what the profiler runs wrap)."""
    rec, t = time_workload(args.workload, args, P, workloads, torch, dev, args.steps, args.warmup,
                           with_oracle=not args.no_cpu_baseline)
    cpu = rec.pop("cpu_oracle", None)
    if cpu:
        cpu.update(host_info())
    roof = rec.pop("roofline", None) or {
        "bound": "hbm", "kernel": "whole call", "achieved": rec["algorithmic_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": rec["frac_of_hbm_peak"], "traffic": None, "algorithmic_bytes_per_launch": rec["algorithmic_bytes_per_call"]}
    print(json.dumps({
        "metric": METRIC, "value": rec["weights_per_s"], "unit": "weights/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": rec["ms_per_call"], "ms_per_step_median": rec["ms_per_call_median"],
        "ms_per_step_min": rec["ms_per_call_min"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": rec["workload"], "kernel_launches_per_call": rec["kernel_launches_per_call"],
                   "note": "wall time per call, outputs preallocated; includes the Python binding's marshalling"},
        "call_algorithmic_GBps": rec["algorithmic_GBps"], "call_frac_of_hbm_peak": rec["frac_of_hbm_peak"],
        "roofline": roof, "cpu_baseline": cpu}))


# ---- CPU oracle beside the L-C step ----------------------------------------------------------------------

def oracle_baseline(args, workloads, mu, density, T):
    """The oracle's L-C step, as it stands, on two bounded samples of the workload (the first A and the first
    B tensors).  The sort makes its cost grow as n log n: the two timings give the per-key cost of the sort
    and of the linear passes, and the model's figure for the full workload is quoted beside the sample's."""
    import math

    import oracle
    a_t, b_t = sorted(args.cpu_sample_tensors)
    runs = []
    for n_t in (a_t, b_t):
        ws, ls = workloads.lc_stress(indices=range(n_t), n_tensors=T, threads=8)
        t0 = time.perf_counter()
        oracle.lc_step(ws, ls, mu, density)
        dt = time.perf_counter() - t0
        runs.append((sum(w.size for w in ws), dt))
        del ws, ls
    (n1, t1), (n2, t2) = runs
    # t = a n log2 n + b n  through the two samples
    det = n1 * math.log2(n1) * n2 - n2 * math.log2(n2) * n1
    a = (t1 * n2 - t2 * n1) / det if det else 0.0
    b = (t1 - a * n1 * math.log2(n1)) / n1
    full = a * N_STRESS * math.log2(N_STRESS) + b * N_STRESS if a > 0 and b > 0 else None
    # whatever the split between the sort and the linear passes: between "all linear" and "all n log n" from the larger sample
    bounds = [t2 * N_STRESS / n2, t2 * N_STRESS * math.log2(N_STRESS) / (n2 * math.log2(n2))]
    rec = {"value": round(n2 / t2, 1), "unit": "weights/s", "cores": 1, "kind": "oracle",
           "sample": f"one L-C step of the oracle on the first {b_t} of the {T} tensors ({n2} weights): {t2:.1f} s; "
                     f"on the first {a_t} ({n1} weights): {t1:.1f} s = {n1 / t1:.0f} weights/s",
           "model": "t = a n log2 n + b n through the two samples" if full else "the two samples do not separate the sort from the linear passes",
           "full_workload_estimate_s": round(full, 1) if full else None,
           "full_workload_estimate_weights_per_s": round(N_STRESS / full, 1) if full else None,
           "full_workload_bounds_s": [round(bounds[0], 1), round(bounds[1], 1)]}
    rec.update(host_info())
    if args.cpu_all_cores:
        from concurrent.futures import ThreadPoolExecutor
        cores = os.cpu_count() or 1
        ws, ls = workloads.lc_stress(indices=range(a_t), n_tensors=T, threads=8)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as ex:       # the C oracle runs outside the interpreter lock
            list(ex.map(lambda _: oracle.lc_step(ws, ls, mu, density), range(cores)))
        dt = time.perf_counter() - t0
        rec["all_cores"] = {"value": round(cores * n1 / dt, 1), "unit": "weights/s", "cores": cores,
                            "kind": f"{cores} independent oracle steps at once, each on the first {a_t} tensors, {dt:.1f} s"}
    return rec


# ---- summaries of rocprofv3 output (profiles/*.md) ---------------------------------------------------------

def _short(name):
    name = name.replace("condensa::", "").replace("void ", "")
    if name.startswith("at::") or "at::native" in name:
        return "at::native elementwise / fill (torch)"
    return name.split("(")[0]


def _trace_section(directory, command, bytes_per_launch, top):
    files = glob.glob(os.path.join(directory, "**", "*kernel_stats.csv"), recursive=True)
    if not files:
        sys.exit(f"no *kernel_stats.csv under {directory}")
    rows = list(csv.DictReader(open(sorted(files)[0])))
    lines = ["    " + command, "",
             "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---:|---:|---:|---:|---:|"]
    for r in rows[:top]:
        lines.append("| `%s` | %s | %.1f | %.1f | %.1f | %.2f |" % (
            _short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
            float(r["Percentage"])))
    if rows and "TotalDurationNs" in rows[0]:
        ours = [r for r in rows if "condensa::" in r["Name"]]
        calls = max((int(r["Calls"]) for r in ours if "k_prepare" in r["Name"]), default=0)
        total_us = sum(float(r["TotalDurationNs"]) for r in ours) / 1e3
        if calls:
            lines += ["", f"The library's kernels: {sum(int(r['Calls']) for r in ours) / calls:.0f} launches and {total_us / calls:.1f} us "
                          f"of kernel time per call ({calls} calls in the run)."]
    for spec in bytes_per_launch:
        kernel, nbytes = spec.rsplit("=", 1)
        hit = [r for r in rows if kernel in r["Name"]]
        if not hit:
            continue
        us = float(hit[0]["AverageNs"]) / 1e3
        gbps = int(nbytes) / (us * 1e-6) / 1e9
        lines += ["", f"`{_short(hit[0]['Name'])}`: {us:.1f} us average for {int(nbytes):,} algorithmic bytes per launch -> "
                      f"{gbps:.0f} GB/s = {100 * gbps / HBM_PEAK_GBPS:.1f} % of the 8 TB/s peak."]
    return lines


def summarize_trace(args):
    dirs = args.summarize_trace
    lines = [f"# rocprofv3 kernel-trace summary: {args.title}", "",
             "Per-kernel statistics (`*_kernel_stats.csv`) of one MI355X; commands run from /tmp with TMPDIR=/tmp, "
             "$R = repository root.", ""]
    for d in dirs:
        name = os.path.basename(os.path.normpath(d))
        if len(dirs) > 1:
            lines += [f"## {name}", ""]
        lines += _trace_section(d, args.command.replace("{W}", name), args.bytes_per_launch, 24 if len(dirs) == 1 else 8) + [""]
    open(args.out, "w").write("\n".join(lines))
    print("wrote", args.out)


def _pmc_averages(directory, counter):
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        sys.exit(f"no *counter_collection.csv under {directory}")
    acc = {}
    for r in csv.DictReader(open(sorted(files)[0])):
        if r.get("Counter_Name") != counter:
            continue
        acc.setdefault(_short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    out = {}
    for k, v in acc.items():
        if "copybuffer" in k.lower():               # the table upload of a call is a copy too: keep the big ones only
            v = [x for x in v if x >= 0.5 * max(v)]
        out[k] = (sum(v) / len(v), len(v))
    return out


def summarize_pmc(args):
    """FETCH_SIZE / WRITE_SIZE per dispatch, scaled by what the same counters read for plain device copies of
    one 4096x4608 fp32 tensor (75 497 472 B read and written each; `--calibrate-copy`)."""
    fetch = _pmc_averages(args.summarize_pmc[0], "FETCH_SIZE")
    write = _pmc_averages(args.summarize_pmc[1], "WRITE_SIZE")
    copy_kib = 4096 * 4608 * 4 / 1024.0
    copy = [k for k in fetch if "copybuffer" in k.lower()]
    if not copy or copy[0] not in write:
        sys.exit("calibration copies not found: run bench.py with --calibrate-copy under the profiler")
    f_scale = copy_kib / fetch[copy[0]][0]
    w_scale = copy_kib / write[copy[0]][0]
    lines = [f"# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: {args.title}", "",
             "Commands (from /tmp with TMPDIR=/tmp; $R = repository root), one counter per run:", ""]
    lines += ["    " + c for c in args.command.split(" && ")]
    lines += ["", f"Calibration: `--calibrate-copy` launches four device-to-device copies of one 4096x4608 fp32 tensor "
                  f"(`{copy[0]}`; smaller dispatches of that kernel, the calls' table uploads, are left out), each "
                  f"reading and writing 75 497 472 B = {copy_kib:,.0f} KiB.  FETCH_SIZE reads "
                  f"{fetch[copy[0]][0]:,.1f} for them -> scale factor {f_scale:.5f}; WRITE_SIZE reads {write[copy[0]][0]:,.1f} "
                  f"-> factor {w_scale:.5f}.", "",
              "| kernel | dispatches | FETCH_SIZE raw (avg) | fetched bytes (scaled) | WRITE_SIZE raw (avg) | written bytes (scaled) | traffic / launch | algorithmic bytes / launch |",
              "|---|---:|---:|---:|---:|---:|---:|---:|"]
    alg = {}
    for spec in args.bytes_per_launch:
        kernel, nbytes = spec.rsplit("=", 1)
        alg[kernel] = int(nbytes)
    traffic = {}
    for k in sorted(fetch, key=lambda k: -fetch[k][0] - write.get(k, (0, 0))[0])[:12]:
        fb = fetch[k][0] * f_scale * 1024
        wb = write.get(k, (0.0, 0))[0] * w_scale * 1024
        key = next((key for key in alg if key in k), None)
        if key:
            traffic[key] = int(round(fb + wb))
        lines.append(f"| `{k}` | {fetch[k][1]} | {fetch[k][0]:,.1f} | {fb:,.0f} | {write.get(k, (0.0, 0))[0]:,.1f} | {wb:,.0f} | "
                     f"{fb + wb:,.0f} | {f'{alg[key]:,}' if key else '-'} |")
    for key, t in traffic.items():
        lines += ["", f"`{key}` moves {t / alg[key]:.3f}x its algorithmic bytes."]
    lines += ["", "Machine-readable (bench.py reads `roofline.traffic` from here while the kernel sources still hash to "
                  "`sources_sha256`):", "", "```json",
              json.dumps({"traffic_bytes_per_launch": traffic, "tensors": args.tensors, "fetch_scale": round(f_scale, 5),
                          "write_scale": round(w_scale, 5), "sources": list(KERNEL_SOURCES),
                          "sources_sha256": kernel_sources_hash()}, indent=1), "```"]
    open(args.out, "w").write("\n".join(lines) + "\n")
    print("wrote", args.out)


def summarize_counters(args):
    """Per-kernel averages of whatever counters one rocprofv3 --pmc run collected, plus the ratios that the
    design notes quote: LDS bank-conflict cycles per LDS-active cycle and mean waves per SIMD."""
    files = glob.glob(os.path.join(args.summarize_counters, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        sys.exit(f"no *counter_collection.csv under {args.summarize_counters}")
    acc, order = {}, []
    for r in csv.DictReader(open(sorted(files)[0])):
        k, c = _short(r["Kernel_Name"]), r["Counter_Name"]
        if c not in order:
            order.append(c)
        acc.setdefault(k, {}).setdefault(c, []).append(float(r["Counter_Value"]))
    lines = [f"# rocprofv3 --pmc summary: {args.title}", "",
             "Command (from /tmp with TMPDIR=/tmp; $R = repository root):", "", "    " + args.command, "",
             "Averages per dispatch, one MI355X (256 compute units, 4 SIMDs each, at most 8 waves per SIMD):", "",
             "| kernel | dispatches | " + " | ".join(order) + " | LDS conflict cycles / LDS active cycles | mean waves per SIMD |",
             "|---|---:|" + "---:|" * (len(order) + 2)]
    def avg(k, c):
        v = acc[k].get(c)
        return sum(v) / len(v) if v else None
    for k in sorted(acc, key=lambda k: -(avg(k, "SQ_BUSY_CYCLES") or 0))[:16]:
        n = len(next(iter(acc[k].values())))
        conf, act = avg(k, "SQ_LDS_BANK_CONFLICT"), avg(k, "SQ_LDS_IDX_ACTIVE")
        wc, gui = avg(k, "SQ_WAVE_CYCLES"), avg(k, "GRBM_GUI_ACTIVE")
        ratio = f"{conf / act:.3f}" if conf is not None and act else "-"
        # OccupancyPercent = 400 SQ_WAVE_CYCLES / GRBM_GUI_ACTIVE / CU_NUM / 32 of at most 8 waves per SIMD
        occ = f"{wc / gui / 256:.2f}" if wc is not None and gui else "-"
        lines.append(f"| `{k}` | {n} | " + " | ".join(f"{avg(k, c):,.0f}" if avg(k, c) is not None else "-" for c in order) +
                     f" | {ratio} | {occ} |")
    open(args.out, "w").write("\n".join(lines) + "\n")
    print("wrote", args.out)


# ---- the benchmark ---------------------------------------------------------------------------------------------

def main():
    args = parse()
    if args.summarize_trace:
        return summarize_trace(args)
    if args.summarize_pmc:
        return summarize_pmc(args)
    if args.summarize_counters:
        return summarize_counters(args)
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

    if args.workload not in ("lc_stress", "lc_pq_stress"):
        run_single_workload(args, P, workloads, torch, dev)
        return
    pq = args.workload == "lc_pq_stress"

    rows, cols, T = 4096, 4608, args.tensors
    mu, density = workloads.LC_MU, workloads.LC_DENSITY

    # ---- inputs: generated on the host from the seeded recipe, then made resident -------------------
    t0 = time.time()
    w_dev, lam_dev = [], []
    batch = 8
    for b in range(0, T, batch):
        idx = list(range(b, min(b + batch, T)))
        ws, ls = workloads.lc_stress(indices=idx, n_tensors=T, rows=rows, cols=cols, threads=16)
        for w, l in zip(ws, ls):
            w_dev.append(torch.from_numpy(w).to(dev))
            lam_dev.append(torch.from_numpy(l).to(dev))
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    w_dev = P.tensor_table(w_dev)
    N = sum(t.numel() for t in w_dev)

    outputs = {
        "theta": [torch.empty_like(t) for t in w_dev],
        "grad": [torch.empty_like(t) for t in w_dev],
        "lambda": [torch.empty_like(t) for t in w_dev],
        "results": torch.zeros((1, 8), dtype=torch.int64, device=dev),
    }
    if args.mask:
        outputs["mask"] = [torch.empty(t.shape, dtype=torch.uint8, device=dev) for t in w_dev]
    if pq:
        outputs["theta_f16"] = [torch.empty(t.shape, dtype=torch.int16, device=dev) for t in w_dev]
    def make_cfg(profile):
        return P.condensa_config(select_path=args.select_path, apply_threads=args.apply_threads,
                                 fused_sweep=1 if args.two_sweeps else 0, window_margin=args.window_margin,
                                 profile=profile)
    cfg = make_cfg(0)
    ws_bytes = P.condensa_workspace_bytes(P.binding.OP_LC_STEP, N, 0, T, 1, P.SCOPE_GLOBAL, cfg)
    workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def step():
        return P.condensa_lc_step(w_dev, lam_dev, mu, density, outputs=outputs, mask=args.mask,
                                  workspace=workspace, config=cfg, pq=pq, nnz=pq)

    l0 = P.condensa_launch_count()
    step()
    launches = P.condensa_launch_count() - l0
    torch.cuda.synchronize()
    # phase events inside the timed region bracket the dominant kernel only (every event pair costs the step a
    # few microseconds): the sweep on the one-sweep path, the apply otherwise; the untimed call above tells which
    first_path = P.select_records(outputs["results"])[0]["path"]
    cfg = make_cfg(0x1F if args.all_phases else ((1 << 1) if first_path == 2 and not args.two_sweeps else (1 << 3)))
    if args.calibrate_copy:                         # 4 copies, each reads and writes rows*cols*4 bytes
        for i in range(4):
            outputs["theta"][i].copy_(w_dev[i])
        torch.cuda.synchronize()

    t = timed_calls(step, args.steps, args.warmup, torch, before_timed=P.condensa_profile_reset)
    phases = P.condensa_profile_read()           # the event pairs recorded inside the timed region
    n_timed = args.steps

    ms_per_step = t["mean"]
    rec = P.select_records(outputs["results"])[0]
    assert rec["k"] == int(np.floor(density * N + 0.5)) and rec["n"] == N, rec

    # ---- roofline of the dominant kernel --------------------------------------------------------------
    # One-sweep window path (default): k_window_fused reads w, lambda (8 B) and writes theta, lambda', g
    # (12 B) [+1 mask, +2 binary16 codes] per weight, and that is also all the step needs.  Two sweeps (radix
    # path, or --two-sweeps): k_lc_apply moves the same bytes and the selection reads w, lambda once more.
    one_sweep = rec["path"] == 2 and not args.two_sweeps
    kernel_bytes_per_elem = 20 + (1 if args.mask else 0) + (2 if pq else 0)
    step_bytes_per_elem = kernel_bytes_per_elem + (0 if one_sweep else 8)
    kernel_name, phase = ("k_window_fused<LC>", "sweep") if one_sweep else ("k_lc_apply", "apply")
    kp = phases[phase]
    kernel_ms = kp["ms"] / max(kp["intervals"], 1)
    achieved = kernel_bytes_per_elem * N / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    traffic = measured_traffic(kernel_name, T, args.mask or pq) if one_sweep else None
    roofline = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "avg_launch_ms": round(kernel_ms, 4), "launches_averaged": kp["intervals"],
                "algorithmic_bytes_per_launch": kernel_bytes_per_elem * N}
    step_gbps = step_bytes_per_elem * N / (ms_per_step * 1e-3) / 1e9
    phase_ms = {k: round(v["ms"] / n_timed, 4) for k, v in phases.items() if v["intervals"]}

    # ---- the other half of the target and the small workloads, on the same device ---------------------------
    extras = None
    if not args.no_extras and not pq and T == 64:
        # the L-C step of the composed prune + binary16 scheme with the footprint objective counted inside it
        # (22 B/weight: the binary16 codes are written too)
        outputs["theta_f16"] = [torch.empty(t.shape, dtype=torch.int16, device=dev) for t in w_dev]
        cfg_pq = P.condensa_config(select_path=args.select_path, apply_threads=args.apply_threads,
                                   fused_sweep=1 if args.two_sweeps else 0, window_margin=args.window_margin)
        res_pq = [None]

        def step_pq():
            res_pq[0] = P.condensa_lc_step(w_dev, lam_dev, mu, density, outputs=outputs, mask=False, workspace=workspace,
                                           config=cfg_pq, pq=True, nnz=True)
        tpq = timed_calls(step_pq, args.steps, args.warmup, torch)
        outputs["nnz"] = res_pq[0]["nnz"]
        pq_bytes = (22 if one_sweep else 30) * N
        pq_rec = {"workload": "L-C step of Compose([Prune, Quantize(float16)]) on the same tensors, theta_f16 and the non-zero count written too",
                  "ms_per_step": round(tpq["mean"], 4), "ms_per_step_median": round(tpq["median"], 4), "ms_per_step_min": round(tpq["min"], 4),
                  "nonzero_codes": int(res_pq[0]["nnz"].item()), "kept": rec["k"],
                  "algorithmic_bytes_per_step": pq_bytes, "algorithmic_GBps": round(pq_bytes / (tpq["mean"] * 1e-3) / 1e9, 1),
                  "frac_of_hbm_peak": round(pq_bytes / (tpq["mean"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        # the same step keeping theta only as binary16 codes (what a P+Q pipeline stores): 8 read + 2 + 4 + 4 written
        def step_pq_codes():
            P.condensa_lc_step(w_dev, lam_dev, mu, density, outputs=outputs, theta=False, mask=False, workspace=workspace,
                               config=cfg_pq, pq=True, nnz=True)
        tpc = timed_calls(step_pq_codes, args.steps, args.warmup, torch)
        pc_bytes = (18 if one_sweep else 26) * N
        pq_rec["codes_only"] = {"workload": "the same step without the fp32 theta (theta as binary16 codes only)",
                                "ms_per_step": round(tpc["mean"], 4), "ms_per_step_median": round(tpc["median"], 4),
                                "ms_per_step_min": round(tpc["min"], 4), "algorithmic_bytes_per_step": pc_bytes,
                                "algorithmic_GBps": round(pc_bytes / (tpc["mean"] * 1e-3) / 1e9, 1),
                                "frac_of_hbm_peak": round(pc_bytes / (tpc["mean"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
        del outputs["theta_f16"], res_pq
        del outputs["grad"], outputs["lambda"]      # 9.7 GB back; the weights stay resident for the pruning call
        prune_rec, _ = time_workload("prune_stress", args, P, workloads, torch, dev, args.steps, args.warmup,
                                     resident=w_dev, with_oracle=not args.no_cpu_baseline)
        structure = []
        for name in ("filter_stress", "block_stress"):
            r, _ = time_workload(name, args, P, workloads, torch, dev, args.steps, args.warmup, resident=w_dev,
                                 with_oracle=not args.no_cpu_baseline)
            structure.append(r)
        small = []
        for name in SMALL_WORKLOADS:
            r, _ = time_workload(name, args, P, workloads, torch, dev, 50, 5, with_oracle=not args.no_cpu_baseline)
            small.append(r)
        others = time_other_entry_points(P, torch, w_dev, dev)
        extras = {"global_prune": prune_rec, "lc_step_pq": pq_rec, "structure_prune": structure, "small_workloads": small,
                  "other_entry_points": others,
                  "note": "global_prune: condensa_prune (theta + mask, d = 0.1) on the weights the L-C step ran on; "
                          "structure_prune: the same weights as 262144 filters of 512x3x3 and as 18.9 M blocks of 8x8, d = 0.5, "
                          "against 13 B/weight (the block call reads the weights once and moves 9.3 B/weight); "
                          "small_workloads: wall time per call through the binding (50 calls after 5), launch- and cache-bound"}

    # ---- CPU oracle on bounded samples of the same workload ---------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline and T == 64:
        cpu = oracle_baseline(args, workloads, mu, density, T)

    out = {
        "metric": METRIC,
        "value": round(N / (ms_per_step * 1e-3), 1),
        "unit": "weights/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(t["median"], 4),
        "ms_per_step_min": round(t["min"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"L-C compression step{' with prune + binary16 (P+Q)' if pq else ''}, {T} fp32 tensors of {rows}x{cols} ({N} weights) + multipliers, "
                               f"mu={mu}, density={density}, outputs theta/lambda'/grad" + ("/theta_f16" if pq else "") + ("/mask" if args.mask else ""),
                   "select_path": {1: "radix", 2: "window"}.get(rec["path"], str(rec["path"])),
                   "sweeps_over_the_weights": 1 if one_sweep else (2 if rec["path"] == 2 else 4),
                   "kernel_launches_per_step": launches,
                   "threshold_key": rec["threshold_key"], "n_tie": rec["n_tie"]},
        "step_algorithmic_GBps": round(step_gbps, 1),
        "step_frac_of_hbm_peak": round(step_gbps / HBM_PEAK_GBPS, 4),
        "step_bytes_per_weight": step_bytes_per_elem,
        # the same time against the bytes of a select-then-apply step (weights and multipliers read twice)
        "step_GBps_at_two_read_accounting": round((step_bytes_per_elem + (8 if one_sweep else 0)) * N / (ms_per_step * 1e-3) / 1e9, 1),
        "phase_ms_per_step": phase_ms,
        "input_generation_s": round(gen_s, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
