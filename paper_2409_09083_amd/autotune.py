"""Grouping-profile search (Sec. 4.2: layers are combined into groups; larger groups exchange less boundary
data but recompute more halo, and the best profile depends on the machine).

The paper describes the trade-off and leaves the search to a technical report that is not part of it.  This
module does the search empirically on the GPU: the cost of a group (s, e) does not depend on how the other layers
are grouped (groups meet at whole maps), so every contiguous group up to a maximum length is timed on its own as
a one-group network, and a dynamic programme picks the partition of the layer list with the smallest total time.
That sum is a model (launch tails and cache state of neighbouring groups are not in it), so the partition it proposes
is then timed as a whole network next to the uniform profiles and the configured one, and the search returns the
fastest profile it has measured, never one it has only predicted.

    python -m paper_2409_09083_amd.autotune --config cfg4 [--max-group 8] [--steps 3]

prints one JSON object.  Timing inputs are random device tensors (the kernels' run time does not depend on the
values); no arithmetic of the method happens here.
"""
import argparse
import json
import sys
import time

import torch

from . import binding as B
from .harness import Session


def _fill(s, seed=1):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    s.x.copy_(torch.rand(s.in_shape, generator=g, device="cuda").to(s.tdtype))
    s.dy.copy_(torch.randn(s.out_shape, generator=g, device="cuda").to(s.tdtype))
    s.weights = []
    for ly in s.layers:
        if ly.kind != 0:
            s.weights.append(None)
            continue
        std = (2.0 / (ly.cin * ly.k * ly.k)) ** 0.5
        s.weights.append((torch.randn((ly.cout, ly.cin, ly.k, ly.k), generator=g, device="cuda") * std).to(s.tdtype))


def time_network(layers, batch, in_c, in_h, in_w, grid, group_ends, dtype, steps=3, warmup=1):
    """Milliseconds per forward + backward + gradient sum of one network / grouping."""
    s = Session(layers, batch, in_c, in_h, in_w, grid, group_ends, dtype)
    _fill(s)
    for _ in range(warmup):
        s.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        s.step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    s.close()
    del s
    torch.cuda.empty_cache()
    return ms


def boundary_shapes(cfg):
    """(C, H, W) of every boundary 0..L, as the library's planner computes them (any stride, odd maps)."""
    plan = B.ftp_plan(list(cfg.layers), cfg.batch, cfg.in_c, cfg.in_h, cfg.in_w, cfg.grid[0], cfg.grid[1],
                      list(cfg.group_ends), B.FTP_BF16 if cfg.dtype == "bf16" else B.FTP_F32)
    try:
        return [B.ftp_plan_map_shape(plan, b) for b in range(len(cfg.layers) + 1)]
    finally:
        B.ftp_plan_destroy(plan)


def candidate_profiles(L, searched, configured):
    """Profiles that are timed as whole networks: the dynamic programme's, the configured one, the uniform ones."""
    out = {"searched": tuple(searched), "as configured": tuple(configured)}
    for g in sorted({1, 2, 4, 8, 16, L}):
        if g <= L:
            out["uniform %d" % g] = tuple(list(range(g, L, g)) + [L])
    return out


def search(cfg, max_group=8, steps=3, log=None):
    """Returns (group ends, ms per step, details): the fastest profile among those timed on the whole network.
    details = {"predicted_ms", "group_cost", "profiles": {name: {"group_ends", "ms_per_step" | "error"}}, "chosen"}."""
    layers = list(cfg.layers)
    L = len(layers)
    shapes = boundary_shapes(cfg)
    cost = {}
    for s0 in range(L):
        for e0 in range(s0 + 1, min(L, s0 + max_group) + 1):
            c, h, w = shapes[s0]
            try:
                cost[(s0, e0)] = time_network(layers[s0:e0], cfg.batch, c, h, w, cfg.grid, (e0 - s0,), cfg.dtype, steps)
            except B.FtpError:
                continue                 # e.g. a tile would own no pixel of this group's output
            if log:
                log("group (%d, %d): %.3f ms" % (s0, e0, cost[(s0, e0)]))
    ends, predicted = best_partition(cost, L, max_group)
    measured = {}
    for name, pe in candidate_profiles(L, ends, cfg.group_ends).items():
        try:
            measured[name] = {"group_ends": list(pe),
                              "ms_per_step": time_network(layers, cfg.batch, cfg.in_c, cfg.in_h, cfg.in_w, cfg.grid, pe,
                                                          cfg.dtype, max(steps, 5), 2)}
        except B.FtpError as e:
            measured[name] = {"group_ends": list(pe), "error": str(e)}
        if log:
            log("profile %s %s: %s" % (name, list(pe), measured[name].get("ms_per_step", measured[name].get("error"))))
    timed = {k: v for k, v in measured.items() if "ms_per_step" in v}
    chosen = min(timed, key=lambda k: timed[k]["ms_per_step"])
    details = {"predicted_ms": predicted, "group_cost": {"%d-%d" % k: v for k, v in cost.items()}, "profiles": measured, "chosen": chosen}
    return tuple(timed[chosen]["group_ends"]), timed[chosen]["ms_per_step"], details


def best_partition(cost, L, max_group):
    """Partition of layers 0..L-1 into contiguous groups (s, e) with minimal summed cost[(s, e)]; groups without a
    cost entry are not allowed.  Returns (group ends, total)."""
    best = [0.0] + [float("inf")] * L
    cut = [0] * (L + 1)
    for e0 in range(1, L + 1):
        for s0 in range(max(0, e0 - max_group), e0):
            if (s0, e0) in cost and best[s0] + cost[(s0, e0)] < best[e0]:
                best[e0] = best[s0] + cost[(s0, e0)]
                cut[e0] = s0
    if best[L] == float("inf"):
        raise ValueError("no admissible partition")
    ends, e0 = [], L
    while e0 > 0:
        ends.append(e0)
        e0 = cut[e0]
    return tuple(reversed(ends)), best[L]


def main():
    from ftp_synth import configs as C
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg4", choices=["cfg2_fused", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--max-group", type=int, default=8)
    ap.add_argument("--steps", type=int, default=3)
    args = ap.parse_args()
    cfg = C.ALL[args.config]
    cfg = cfg() if callable(cfg) else cfg
    ends, ms, details = search(cfg, args.max_group, args.steps, log=lambda m: print(m, file=sys.stderr, flush=True))
    print(json.dumps({"workload": cfg.name, "batch": cfg.batch, "grid": list(cfg.grid), "max_group": args.max_group,
                      "group_ends": list(ends), "ms_per_step": ms, "chosen": details["chosen"],
                      "predicted_ms": details["predicted_ms"], "profiles": details["profiles"]}))


if __name__ == "__main__":
    main()
