"""Per-stack memory of a partition plan against the unpartitioned network (Sec. 5, memory experiment: a device
holds only its own stack, so feature and delta maps shrink with the number of tiles while every device keeps a
full copy of the filters and of its partial gradients).

Host only: builds plans for a series of tile grids and prints what one stack has to hold, as the planner accounts
it (largest stack; forward maps kept for back-propagation incl. recomputed halo, the two delta maps alive at a
time, filters + own partial gradient set, decision codes).

    python -m paper_2409_09083_amd.memory_report --config cfg4 [--grids 1 2 3 4 6 8] [--group-size 4]

prints one JSON object.
"""
import argparse
import json

from . import binding as B


def per_stack_memory(layers, batch, in_c, in_h, in_w, grid, group_ends, dtype="f32"):
    """{'feature_maps', 'delta_maps', 'filters_and_gradients', 'decision_codes', 'total'} in bytes for one stack."""
    plan = B.ftp_plan(list(layers), batch, in_c, in_h, in_w, grid[0], grid[1], list(group_ends),
                      B.FTP_BF16 if dtype == "bf16" else B.FTP_F32)
    try:
        f, d, w, o = B.ftp_plan_sizes(plan)["per_stack_split"]
    finally:
        B.ftp_plan_destroy(plan)
    return {"feature_maps": f, "delta_maps": d, "filters_and_gradients": w, "decision_codes": o, "total": f + d + w + o}


def report(cfg, grids, group_ends=None):
    ends = tuple(cfg.group_ends if group_ends is None else group_ends)
    rows = []
    base = per_stack_memory(cfg.layers, cfg.batch, cfg.in_c, cfg.in_h, cfg.in_w, (1, 1), ends, cfg.dtype)
    for n in grids:
        try:
            m = per_stack_memory(cfg.layers, cfg.batch, cfg.in_c, cfg.in_h, cfg.in_w, (n, n), ends, cfg.dtype)
        except B.FtpError as e:
            rows.append({"grid": [n, n], "error": str(e)})
            continue
        m["grid"] = [n, n]
        m["maps_vs_unpartitioned"] = (base["feature_maps"] + base["delta_maps"]) / float(m["feature_maps"] + m["delta_maps"])
        m["total_vs_unpartitioned"] = base["total"] / float(m["total"])
        rows.append(m)
    return {"workload": cfg.name, "batch": cfg.batch, "group_ends": list(ends), "unpartitioned": base, "per_stack": rows}


def main():
    from ftp_synth import configs as C
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg4", choices=sorted(C.ALL))
    ap.add_argument("--grids", type=int, nargs="+", default=[1, 2, 3, 4, 6, 8])
    ap.add_argument("--group-size", type=int, default=0, help="uniform groups of this many layers (0: as configured)")
    args = ap.parse_args()
    cfg = C.ALL[args.config]()
    ends = C.uniform_groups(cfg.n_layers, args.group_size) if args.group_size else None
    print(json.dumps(report(cfg, args.grids, ends)))


if __name__ == "__main__":
    main()
