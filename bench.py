#!/usr/bin/env python3
"""Benchmark of the fused-tile forward + backward + gradient-sum pass on one MI355X.

One step = ftp_forward, ftp_backward, ftp_reduce_wgrad over one batch of synthetic input that is
already resident in HBM.  Prints ONE JSON line: whole-job images/s, the roofline of the dominant
kernel (timed live with HIP events inside the timed region), the kernels below the ridge against the HBM
roof, the bf16 workload with its layer-grouping sweep, and the CPU oracle timed on the host.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
# Plain vector fp32 of this build: 256 CUs x 4 SIMDs x 16 lanes x 2 FLOP (one FMA) x 2.4 GHz = 78.6 TFLOP/s.  The
# published 157.3 TFLOP/s needs packed fp32 (two FMAs per lane and clock), which this build switches off.
PEAK_ALU_TFLOPS = 78.6
SWEEP_GROUP_SIZES = (1, 2, 4, 8, 16)


def pick_config(name, group_size):
    from ftp_synth import configs as C
    if name == "cfg5":
        return C.config5(group_size)
    return C.ALL[name]()


def cpu_baseline(cfg, budget_images):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload."""
    from ftp_synth import configs as C
    from oracle import reference as O
    n = min(cfg.batch, budget_images)
    x, ws, bs, dy = C.make_tensors(cfg, images=list(range(n)))
    bf = cfg.dtype == "bf16"
    t0 = time.perf_counter()
    acts, args = O.forward(cfg.layers, x, ws, None, bf16_store=bf)
    O.backward(cfg.layers, acts, args, ws, dy, bf16_store=bf, want_db=False)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "images/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": "%d of %d images of the same workload, forward + backward, %.1f s" % (n, cfg.batch, dt)}


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc runs kept under profiles/ (None if not measured)."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def pooled_by_kernel(recs):
    """Per kernel symbol: summed duration, launches and algorithmic work of all the layers that run it."""
    by_kernel = {}
    for r in recs:
        k = by_kernel.setdefault(r["kernel"], {"ms": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0, "executed": 0.0, "layers": set()})
        k["executed"] += r["executed_flops_per_launch"] * r["launches"]
        k["ms"] += r["total_ms"]
        k["launches"] += r["launches"]
        k["flops"] += r["flops_per_launch"] * r["launches"]
        k["bytes"] += r["bytes_per_launch"] * r["launches"]
        k["layers"].add(r["layer"])
    return by_kernel


def roofline_of(name, k, dtype, workload, step_ms_total):
    """Roofline block of one kernel symbol: achieved = algorithmic work of its launches / their summed duration,
    i.e. average algorithmic work per launch / average launch duration (what rocprofv3 --stats reports per symbol)."""
    ai = k["flops"] / max(k["bytes"], 1.0)
    ridge = PEAK_MFMA_TFLOPS[dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    sec = k["ms"] * 1e-3
    if "mfma" in name and ai >= ridge:
        roof = {"bound": "mfma", "achieved": k["flops"] / sec / 1e12, "peak": PEAK_MFMA_TFLOPS[dtype], "unit": "TFLOP/s"}
    elif "mfma" not in name and ai >= PEAK_ALU_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        # a kernel of plain vector arithmetic above the ridge of the vector units
        roof = {"bound": "alu", "achieved": k["flops"] / sec / 1e12, "peak": PEAK_ALU_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": k["bytes"] / sec / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(workload, name)
    roof["kernel"] = name
    roof["layers"] = sorted(k["layers"])
    roof["launches"] = k["launches"]
    roof["avg_launch_ms"] = k["ms"] / k["launches"]
    roof["share_of_step"] = k["ms"] / step_ms_total
    # the same kernel on the FLOPs it really executed (halo recompute inside a group included): what the kernel
    # achieves as a kernel, next to `achieved`, which credits the untiled layer only
    roof["executed_tflops"] = k["executed"] / sec / 1e12
    return roof


def run_workload(cfg, steps, warmup, with_update=False, overlap=False, per_kernel=False, extras=True):
    """Times `steps` steps of one workload (inputs resident in HBM) with the per-kernel HIP events on.
    Returns the fields of the JSON line that describe this workload."""
    import torch
    from ftp_synth import configs as C
    import paper_2409_09083_amd as F
    from paper_2409_09083_amd.harness import Session

    x, ws, bs, dy = C.make_tensors(cfg)
    s = Session(cfg.layers, cfg.batch, cfg.in_c, cfg.in_h, cfg.in_w, cfg.grid, cfg.group_ends, cfg.dtype)
    s.load(x=x, weights=ws, dy=dy)
    del x, dy
    if overlap:
        s.set_overlap(True)
    torch.cuda.synchronize()
    # lr = 0 keeps the weights (and with them every step's work) unchanged while the update kernels run in full
    one_step = (lambda: s.train_step(0.0)) if with_update else s.step
    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    F.ftp_profile(s.plan, True)
    # (every step is also bracketed by two events on the stream the kernels run on: median and minimum over steps)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        one_step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    F.ftp_profile(s.plan, False)
    recs = F.ftp_profile_read(s.plan)
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]

    if per_kernel:
        for r in sorted(recs, key=lambda r: (r["layer"], r["pass"])):
            ms = r["total_ms"] / r["launches"]
            print("%-14s layer %2d  %8.3f ms  %7.2f TFLOP/s (executed %7.2f)  %7.1f GB/s  %s" % (
                r["pass"], r["layer"], ms, r["flops_per_launch"] / ms / 1e9, r["executed_flops_per_launch"] / ms / 1e9,
                r["bytes_per_launch"] / ms / 1e6, r["kernel"]), file=sys.stderr)
    ms_per_step = dt * 1e3 / steps
    by_kernel = pooled_by_kernel(recs)
    name, dom = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
    roof = roofline_of(name, dom, cfg.dtype, cfg.name, dt * 1e3)
    # the kernels below the ridge of their arithmetic unit (first layer, 1x1 bottlenecks, lone pools, dy scaling, gradient
    # sum): achieved algorithmic GB/s against the HBM roof, each kernel symbol pooled over its layers
    below = []
    for kn, k in sorted(by_kernel.items(), key=lambda kv: -kv[1]["ms"]):
        r = roofline_of(kn, k, cfg.dtype, cfg.name, dt * 1e3)
        if r["bound"] == "hbm":
            below.append({"kernel": kn, "layers": r["layers"], "achieved": r["achieved"], "unit": "GB/s", "frac": r["frac"],
                          "tflops": k["flops"] / (k["ms"] * 1e-3) / 1e12, "avg_launch_ms": r["avg_launch_ms"],
                          "share_of_step": r["share_of_step"], "traffic": r["traffic"]})
    phases = {}
    for r in recs:
        phases[r["pass"]] = phases.get(r["pass"], 0.0) + r["total_ms"] / steps
    work = s.work
    out = {
        "value": cfg.batch * steps / dt, "ms_per_step": ms_per_step,
        "ms_per_step_median": statistics.median(per_step), "ms_per_step_min": min(per_step),
        "config": {"workload": cfg.name, "batch": cfg.batch, "input": [cfg.in_c, cfg.in_h, cfg.in_w],
                   "primitive_layers": cfg.n_layers, "grid": list(cfg.grid), "group_ends": list(cfg.group_ends)},
        "roofline": roof,
        "memory_bound_kernels": below,
        "useful_tflops": 2.0 * work["useful_macs"] / (ms_per_step * 1e-3) / 1e12,
        "executed_over_useful_macs": work["executed_macs"] / work["useful_macs"],
        "halo_bytes_per_step": [work["halo_bytes_fwd"], work["halo_bytes_bwd"]],
        "phases_ms_per_step": phases,
    }
    if extras:
        if not overlap:
            # the same K steps once more with the two-stream backward pass (ftp_set_overlap) and without per-kernel events:
            # reported beside `value`, which stays the single-stream figure the roofline above belongs to
            s.set_overlap(True)
            for _ in range(min(warmup, 2)):
                one_step()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(steps):
                one_step()
            torch.cuda.synchronize()
            dt2 = time.perf_counter() - t1
            s.set_overlap(False)
            out["two_stream_backward"] = {"value": cfg.batch * steps / dt2, "unit": "images/s", "ms_per_step": dt2 * 1e3 / steps}
        # forward inference alone (ftp_forward), for reference
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            s.forward()
        torch.cuda.synchronize()
        dt3 = time.perf_counter() - t2
        out["forward_only"] = {"value": cfg.batch * steps / dt3, "unit": "images/s", "ms_per_pass": dt3 * 1e3 / steps}
    s.close()
    del s
    torch.cuda.empty_cache()
    return out


def cfg5_sweep(steps, warmup):
    """The bf16-storage workload (config 5: batch 32, 8 x 8 tiles) at every group size of its sweep: the trade-off between
    halo recompute (executed / useful MACs) and boundary exchange (halo bytes), Sec. 4.2."""
    from ftp_synth import configs as C
    out = {"unit": "images/s", "dtype": "bf16", "steps": steps, "warmup": warmup, "by_group_size": {}}
    for g in SWEEP_GROUP_SIZES:
        r = run_workload(C.config5(g), steps, warmup, extras=False)
        e = {"value": r["value"], "ms_per_step": r["ms_per_step"], "ms_per_step_median": r["ms_per_step_median"],
             "ms_per_step_min": r["ms_per_step_min"], "group_ends": r["config"]["group_ends"],
             "executed_over_useful_macs": r["executed_over_useful_macs"], "halo_bytes_per_step": r["halo_bytes_per_step"],
             "useful_tflops": r["useful_tflops"]}
        if g == 4:
            e["roofline"] = r["roofline"]
            e["memory_bound_kernels"] = r["memory_bound_kernels"]
            e["phases_ms_per_step"] = r["phases_ms_per_step"]
        out["by_group_size"][str(g)] = e
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg4", choices=["tiny", "cfg2_perblock", "cfg2_fused", "cfg3", "cfg4", "cfg5", "gen_stem"])
    ap.add_argument("--group-size", type=int, default=4, help="layers per group (cfg5 sweep)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (batch-size sweeps; 0 = as configured)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="leave out the config-5 grouping sweep (cfg5_sweep)")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the legs that follow the timed region (two-stream backward, forward only): profiler "
                         "runs then see the timed region's launches only")
    ap.add_argument("--with-update", action="store_true",
                    help="close every step with the fused gradient sum + filter update (lr 0) instead of the plain gradient sum")
    ap.add_argument("--overlap", action="store_true",
                    help="run the filter gradients on a second stream beside the delta back-propagation (ftp_set_overlap); "
                         "the per-kernel records then show overlapped, hence longer, launches")
    ap.add_argument("--per-kernel", action="store_true", help="print the per-kernel timing table to stderr")
    ap.add_argument("--cpu-images", type=int, default=0, help="images for the oracle timing (0 = automatic)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain device copy of 256 MiB (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    cfg = pick_config(args.config, args.group_size)
    if args.batch:
        cfg = cfg.with_(batch=args.batch)
    if args.traffic_probe:
        probe = torch.empty(2, 64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        probe[0].normal_()
        torch.cuda.synchronize()
        probe[1].copy_(probe[0])            # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del probe
    r = run_workload(cfg, args.steps, args.warmup, args.with_update, args.overlap, args.per_kernel, extras=not args.no_extras)
    out = {
        "metric": "train images/sec (fwd+bwd, fused-tile early layers)",
        "value": r.pop("value"), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
    }
    out.update(r)
    if args.config == "cfg4" and not args.batch and not args.no_sweep:
        out["cfg5_sweep"] = cfg5_sweep(max(3, args.steps // 2), min(args.warmup, 2))
    if not args.no_cpu_baseline:
        # about 10-20 s of oracle time: 12 images of the large workloads (the oracle is linear in the batch)
        n_img = args.cpu_images or (12 if cfg.name.startswith(("cfg4", "cfg5")) else cfg.batch)
        out["cpu_baseline"] = cpu_baseline(cfg, n_img)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
