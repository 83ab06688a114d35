#!/usr/bin/env python3
"""Benchmark: specs solved per second for the full lattice fill + compression, one MI355X.

A step = one pass of the whole hot path over one synthetic workload: for each
lattice of the configuration (config 5: MatmulAccum, bias-add+ReLU, fused) the
bottom-up fill of the memo table and the compression into the two box lists.
Inputs (target and lattice descriptors, a few hundred bytes) and all tables are
resident in HBM; nothing crosses PCIe in the timed region except counters.

Prints ONE JSON line: metric, value, roofline of the fill, CPU baseline (the oracle).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
FILL_BYTES_PER_SPEC = 18       # write cost (8) + argmin (2), read each cost once (8)


def measured_traffic(config, table, n_launch):
    """HBM bytes per fill launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a 1 GiB copy in the same run); None if there is no summary."""
    path = os.path.join(ROOT, "profiles", "fill_traffic_config%d_%s.json" % (config, table))
    try:
        with open(path) as f:
            t = json.load(f)
        return (t["fetch_bytes_per_solve"] + t["write_bytes_per_solve"]) / n_launch
    except (OSError, KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--scratch-gb", type=float, default=8.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the lattice fill is a single-GPU path); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_01637_amd import binding as B
    from paper_2505_01637_amd import workloads as W
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = torch.device("cuda", 0)

    cfg = W.config(args.config, seed=args.seed)
    target = B.Target(cfg["target"])
    scratch = torch.empty(int(args.scratch_gb * (1 << 30)), dtype=torch.uint8, device=dev)
    bufs = {}
    for label, lat, _ in cfg["lattices"]:
        cb, ab, _ = B.table_bytes(target, lat)
        bufs[label] = (torch.empty(cb, dtype=torch.uint8, device=dev), torch.empty(ab, dtype=torch.uint8, device=dev))

    def step():
        # every lattice gets its own slice of the scratch buffer: a solved table keeps its box
        # lists there while later lattices are solved.  One call for all lattices: those that do
        # not depend on each other (M and E) are in flight together, and F starts when the fills of
        # M and E are queued, while these two are still to be compressed.
        return B.solve_lattices(target, cfg["lattices"],
                                buffers={l: (bufs[l][0], bufs[l][1], scratch_of[l]) for l in bufs})

    # split the scratch buffer between the lattices: the small ones get their worst-case need,
    # the others share the rest in proportion to their size
    sizes = {label: W.n_specs(cfg["target"], lat) for label, lat, _ in cfg["lattices"]}
    total_specs = sum(sizes.values())
    need = {label: B.table_bytes(target, lat)[2] for label, lat, _ in cfg["lattices"]}
    small = {l for l in sizes if need[l] <= (512 << 20)}
    rest = scratch.numel() - sum(need[l] for l in small)
    rest_specs = sum(sizes[l] for l in sizes if l not in small) or 1
    scratch_of, off = {}, 0
    for label in sizes:
        share = need[label] if label in small else int(rest * sizes[label] / rest_specs)
        share = min((share + 255) // 256 * 256, scratch.numel() - off)
        scratch_of[label] = scratch[off:off + share]
        off += share

    if args.copy_calibration:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fill_ms = {l: 0.0 for l in sizes}
    comp_ms = {l: 0.0 for l in sizes}
    for _ in range(args.steps):
        tabs = step()
        for l, t in tabs.items():
            fill_ms[l] += t.stats.fill_ms
            comp_ms[l] += t.stats.compress_ms
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    stats = {l: t.stats.as_dict() for l, t in tabs.items()}
    n_rewrites = sum(s["n_rewrites"] for s in stats.values())

    # dominant kernel: the fill kernel of the largest lattice (HIP events on the solve's stream)
    big = max(sizes, key=sizes.get)
    big_fill_ms = fill_ms[big] / args.steps
    big_kind = next(lat["kind"] for label, lat, _ in cfg["lattices"] if label == big)
    n_launch = stats[big]["n_levels_run"]
    kernel_text = ("fill of table %s: plan_kernel (which also streams the (INF, NONE) pre-fill), sort_work_kernel, "
                   "fill_kernel / fill_big_kernel per dependency level" % big)
    if big_kind == W.KIND_MATMUL_BOUNDED:
        # one launch per diagonal: dependency level of shapes + rank (sum of the three operand levels)
        n_launch += 3 * (cfg["target"]["n_levels"] - 1)
        kernel_text = "fill of table %s: fill_bounded_kernel, one launch per diagonal of (dependency level, rank)" % big
    algo_bytes_per_launch = FILL_BYTES_PER_SPEC * sizes[big] / n_launch
    avg_launch_ms = big_fill_ms / n_launch
    achieved = algo_bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9

    out = {
        "metric": "specs solved/sec (full lattice fill + compression, 1 GPU)",
        "value": total_specs / (ms_per_step * 1e-3),
        "unit": "specs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": "config %d: %s" % (args.config, ", ".join("%s %d specs" % (l, n) for l, n in sizes.items())),
                   "seed": args.config if args.seed is None else args.seed},
        "rewrites_per_s": n_rewrites / (ms_per_step * 1e-3),
        "fill_specs_per_s": total_specs / (sum(fill_ms.values()) / args.steps * 1e-3),
        "detail": {l: {"specs": sizes[l], "fill_ms": fill_ms[l] / args.steps, "compress_ms": comp_ms[l] / args.steps,
                       "admissible": stats[l]["n_admissible"], "rewrites": stats[l]["n_rewrites"],
                       "launches": stats[l]["n_levels_run"],
                       "decision_boxes": stats[l]["n_decision_boxes"], "cost_boxes": stats[l]["n_cost_boxes"],
                       "scratch_used": stats[l]["scratch_used"]} for l in sizes},
        "roofline": {"bound": "hbm", "kernel": kernel_text,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(args.config, big, n_launch),
                     "launches_per_step": n_launch, "avg_launch_ms": avg_launch_ms,
                     "algorithmic_bytes_per_launch": algo_bytes_per_launch},
    }
    # the same table's other fractions of the 8 TB/s: measured bytes of the fill over its time, and
    # the compulsory bytes of fill + compression (18 + 10 B/spec) over the time of both
    traffic = out["roofline"]["traffic"]
    big_both_ms = big_fill_ms + comp_ms[big] / args.steps
    out["roofline"]["measured_traffic_frac"] = (None if traffic is None else
                                                traffic * n_launch / (big_fill_ms * 1e-3) / 1e9 / HBM_PEAK_GBS)
    out["roofline"]["fill_and_compress_frac"] = 28 * sizes[big] / (big_both_ms * 1e-3) / 1e9 / HBM_PEAK_GBS

    if not args.no_cpu_baseline:
        from oracle import oracle as O
        sample_max = {5: 128, 7: 16}.get(args.config)
        scfg = W.config(args.config, seed=args.seed, max_size=sample_max)
        t1 = time.perf_counter()
        res = O.solve_config(scfg)
        t_fill = time.perf_counter() - t1
        for label, lat, _ in scfg["lattices"]:
            O.compress_table(scfg["target"], lat, res[label]["cost"], res[label]["argmin"])
        t_all = time.perf_counter() - t1
        n_s = sum(len(r["cost"]) for r in res.values())
        out["cpu_baseline"] = {"value": n_s / t_all, "unit": "specs/s", "cores": 1, "kind": "oracle",
                               "sample": "config %d with sizes <= %s: %d specs, fill + both box lists, %.1f s"
                                         % (args.config, sample_max, n_s, t_all),
                               "fill_only_value": n_s / t_fill}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
