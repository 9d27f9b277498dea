#!/usr/bin/env python3
"""Benchmark of the fused-tile forward + backward + gradient-sum pass on one MI355X.

One step = ftp_forward, ftp_backward, ftp_reduce_wgrad over one batch of synthetic input that is
already resident in HBM.  Prints ONE JSON line: whole-job images/s, the roofline of the dominant
kernel (timed live with HIP events inside the timed region) and the CPU oracle timed on the host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PEAK_ALU_TFLOPS = 157.3          # fp32 vector FMA, 256 CUs x 4 SIMD x 64 lanes x 2 x 2.4 GHz


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg4", choices=["tiny", "cfg2_perblock", "cfg2_fused", "cfg3", "cfg4", "cfg5", "gen_stem"])
    ap.add_argument("--group-size", type=int, default=4, help="layers per group (cfg5 sweep)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (batch-size sweeps; 0 = as configured)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    from ftp_synth import configs as C
    import paper_2409_09083_amd as F
    from paper_2409_09083_amd.harness import Session

    cfg = pick_config(args.config, args.group_size)
    if args.batch:
        cfg = cfg.with_(batch=args.batch)
    x, ws, bs, dy = C.make_tensors(cfg)
    s = Session(cfg.layers, cfg.batch, cfg.in_c, cfg.in_h, cfg.in_w, cfg.grid, cfg.group_ends, cfg.dtype)
    s.load(x=x, weights=ws, dy=dy)
    del x, dy
    if args.overlap:
        s.set_overlap(True)
    torch.cuda.synchronize()

    if args.traffic_probe:
        probe = torch.empty(2, 64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        probe[0].normal_()
        torch.cuda.synchronize()
        probe[1].copy_(probe[0])            # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del probe
    # lr = 0 keeps the weights (and with them every step's work) unchanged while the update kernels run in full
    one_step = (lambda: s.train_step(0.0)) if args.with_update else s.step
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    F.ftp_profile(s.plan, True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    F.ftp_profile(s.plan, False)
    recs = F.ftp_profile_read(s.plan)

    if args.per_kernel:
        for r in sorted(recs, key=lambda r: (r["layer"], r["pass"])):
            ms = r["total_ms"] / r["launches"]
            print("%-14s layer %2d  %8.3f ms  %7.2f TFLOP/s  %7.1f GB/s  %s" % (
                r["pass"], r["layer"], ms, r["flops_per_launch"] / ms / 1e9, r["bytes_per_launch"] / ms / 1e6, r["kernel"]), file=sys.stderr)
    ms_per_step = dt * 1e3 / args.steps
    images_per_s = cfg.batch * args.steps / dt

    # roofline of the dominant kernel: the kernel symbol with the largest share of the timed region.  Its launches
    # (one per layer that runs it) are pooled: achieved = algorithmic work of those launches / their summed duration,
    # i.e. average algorithmic work per launch / average launch duration (what rocprofv3 --stats reports per symbol).
    by_kernel = {}
    for r in recs:
        k = by_kernel.setdefault(r["kernel"], {"ms": 0.0, "launches": 0, "flops": 0.0, "bytes": 0.0, "layers": set()})
        k["ms"] += r["total_ms"]
        k["launches"] += r["launches"]
        k["flops"] += r["flops_per_launch"] * r["launches"]
        k["bytes"] += r["bytes_per_launch"] * r["launches"]
        k["layers"].add(r["layer"])
    name, dom = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
    avg_ms = dom["ms"] / dom["launches"]
    ai = dom["flops"] / max(dom["bytes"], 1.0)
    ridge = PEAK_MFMA_TFLOPS[cfg.dtype] * 1e12 / (PEAK_HBM_GBS * 1e9)
    if "mfma" in name and ai >= ridge:
        peak = PEAK_MFMA_TFLOPS[cfg.dtype]
        roof = {"bound": "mfma", "achieved": dom["flops"] / (dom["ms"] * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s"}
    elif "mfma" not in name and ai >= PEAK_ALU_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        # a kernel of plain vector arithmetic above the ridge of the vector units
        roof = {"bound": "alu", "achieved": dom["flops"] / (dom["ms"] * 1e-3) / 1e12, "peak": PEAK_ALU_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": dom["bytes"] / (dom["ms"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(cfg.name, name)
    roof["kernel"] = name
    roof["layers"] = sorted(dom["layers"])
    roof["launches"] = dom["launches"]
    roof["avg_launch_ms"] = avg_ms
    roof["share_of_step"] = dom["ms"] / (dt * 1e3)

    phases = {}
    for r in recs:
        phases[r["pass"]] = phases.get(r["pass"], 0.0) + r["total_ms"] / args.steps
    work = s.work
    useful_flops = 2.0 * work["useful_macs"]
    out = {
        "metric": "train images/sec (fwd+bwd, fused-tile early layers)",
        "value": images_per_s, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.batch, "input": [cfg.in_c, cfg.in_h, cfg.in_w],
                   "primitive_layers": cfg.n_layers, "grid": list(cfg.grid), "group_ends": list(cfg.group_ends)},
        "roofline": roof,
        "useful_tflops": useful_flops / (ms_per_step * 1e-3) / 1e12,
        "executed_over_useful_macs": work["executed_macs"] / work["useful_macs"],
        "halo_bytes_per_step": [work["halo_bytes_fwd"], work["halo_bytes_bwd"]],
        "phases_ms_per_step": phases,
    }
    if not args.overlap:
        # the same K steps once more with the two-stream backward pass (ftp_set_overlap) and without per-kernel events:
        # reported beside `value`, which stays the single-stream figure the roofline above belongs to
        s.set_overlap(True)
        for _ in range(min(args.warmup, 2)):
            one_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t1
        s.set_overlap(False)
        out["two_stream_backward"] = {"value": cfg.batch * args.steps / dt2, "unit": "images/s", "ms_per_step": dt2 * 1e3 / args.steps}
    # forward inference alone (ftp_forward), for reference
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        s.forward()
    torch.cuda.synchronize()
    dt3 = time.perf_counter() - t2
    out["forward_only"] = {"value": cfg.batch * args.steps / dt3, "unit": "images/s", "ms_per_pass": dt3 * 1e3 / args.steps}
    if not args.no_cpu_baseline:
        # about 10-20 s of oracle time: 12 images of the large workloads (the oracle is linear in the batch)
        n_img = args.cpu_images or (12 if cfg.name.startswith(("cfg4", "cfg5")) else cfg.batch)
        out["cpu_baseline"] = cpu_baseline(cfg, n_img)
    s.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
