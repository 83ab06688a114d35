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


def source_hash():
    """Hash of the kernel sources: a committed counter summary names the sources it was taken
    with, so that a stale one is not passed off as this build's traffic."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2505_01637_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def method_bytes(n, n_adm, fused):
    """HBM bytes the method itself has to move to fill a dense table of n Specs of which n_adm are
    admissible: every entry is written once (cost 8 + rewrite id 2: 10 B), every admissible Spec's
    cost is read at least once by a Spec that rewrites to it (8 B), and an admissible fused Spec
    reads the two entries its bufferize rewrite is made of (16 B).  Entries of Specs that do not
    fit their levels are written and never read."""
    return 10 * n + 8 * n_adm + (16 * n_adm if fused else 0)


def measured_traffic(config, table):
    """(HBM bytes per solve, stale?) of the fill from the committed rocprofv3 --pmc summary
    (FETCH_SIZE and WRITE_SIZE runs, each scaled by a streaming kernel of known size in the same
    run); (None, None) if there is no summary."""
    path = os.path.join(ROOT, "profiles", "fill_traffic_config%d_%s.json" % (config, table))
    try:
        with open(path) as f:
            t = json.load(f)
        return t["fetch_bytes_per_solve"] + t["write_bytes_per_solve"], t.get("source_hash") != source_hash()
    except (OSError, KeyError, ValueError):
        return None, None


def bench_slabs(args, cfg, target, torch, B, W, dev):
    """The fused lattice in slabs along k (no rewrite of a fused Spec changes k): M and E as usual,
    then one mrl_solve per slab into the same table and scratch buffers; a slab's box lists are
    what is kept of it.  Reports the time of a step and the device memory the tables and the
    scratch buffers take, beside what the whole fused table would take."""
    lats = {label: lat for label, lat, _ in cfg["lattices"]}
    assert set(lats) == {"M", "E", "F"}, "--slabs needs the three tables of config 5"
    ks = lats["F"]["sizes"][2]
    per = -(-len(ks) // args.slabs)
    slabs = [dict(lats["F"], sizes=[lats["F"]["sizes"][0], lats["F"]["sizes"][1], ks[lo:lo + per], lats["F"]["sizes"][3]])
             for lo in range(0, len(ks), per)]
    n_slab = max(W.n_specs(cfg["target"], sl) for sl in slabs)
    bufs = {}
    for label in ("M", "E"):
        cb, ab, sb = B.table_bytes(target, lats[label])
        bufs[label] = tuple(torch.empty(x, dtype=torch.uint8, device=dev) for x in (cb, ab, min(sb, 1 << 30)))
    slab_scratch = int(args.scratch_gb * (1 << 30))
    slab_bufs = (torch.empty(8 * n_slab, dtype=torch.uint8, device=dev), torch.empty(2 * n_slab, dtype=torch.uint8, device=dev),
                 torch.empty(slab_scratch, dtype=torch.uint8, device=dev))
    sizes = {label: W.n_specs(cfg["target"], lats[label]) for label in lats}

    def step():
        tabs = B.solve_lattices(target, [j for j in cfg["lattices"] if j[0] != "F"], buffers=bufs)
        out = []
        for sl in slabs:
            t = B.solve(target, sl, deps=(tabs["M"], tabs["E"]), buffers=slab_bufs)
            out.append(t.stats.as_dict())
            t.close()
        return out

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        stats = step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    total = sum(sizes.values())
    print(json.dumps({
        "metric": "specs solved/sec (full lattice fill + compression, 1 GPU)", "value": total / (ms * 1e-3), "unit": "specs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "config %d, the fused table in %d slabs along k: %s" % (
            args.config, len(slabs), ", ".join("%s %d specs" % (l, n) for l, n in sizes.items())), "seed": args.config},
        "slabs": {"n": len(slabs), "specs_of_largest": n_slab,
                  "fused_table_and_scratch_bytes": 10 * n_slab + max(s["scratch_used"] for s in stats),
                  "whole_fused_table_bytes": 10 * sizes["F"],
                  "fill_ms": sum(s["fill_ms"] for s in stats), "compress_ms": sum(s["compress_ms"] for s in stats),
                  "decision_boxes": sum(s["n_decision_boxes"] for s in stats), "cost_boxes": sum(s["n_cost_boxes"] for s in stats)},
        "roofline": None, "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--scratch-gb", type=float, default=8.0)
    ap.add_argument("--max-size", type=int, default=None,
                    help="drop the allowed sizes above this (a smaller lattice of the same structure)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-only", action="store_true",
                    help="time the oracle on the smaller sample of the workload only (about 15 s instead of 2 minutes)")
    ap.add_argument("--slabs", type=int, default=0,
                    help="config 5 only: solve the fused lattice in this many slabs along k, one after the other into the "
                         "same buffers (a lattice too large for one table); prints that run's line instead of the default one")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a 1 GiB read-only kernel, a 1 GiB fill and a 1 GiB copy (to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
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

    cfg = W.config(args.config, seed=args.seed, max_size=args.max_size)
    target = B.Target(cfg["target"])
    if args.slabs:
        return bench_slabs(args, cfg, target, torch, B, W, dev)
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
        # kernels of known traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE: a read-only
        # streaming kernel (a sum over 1 GiB), a write-only one (a fill of 1 GiB) and a copy of 1 GiB
        src = torch.zeros(1 << 27, dtype=torch.int64, device=dev)
        torch.cuda.synchronize()
        total = src.sum()
        torch.cuda.synchronize()
        dst = torch.empty_like(src)
        dst.fill_(3)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst, total
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fill_ms = {l: 0.0 for l in sizes}
    prefill_ms = {l: 0.0 for l in sizes}
    comp_ms = {l: 0.0 for l in sizes}
    for _ in range(args.steps):
        tabs = step()
        for l, t in tabs.items():
            fill_ms[l] += t.stats.fill_ms
            prefill_ms[l] += t.stats.prefill_ms
            comp_ms[l] += t.stats.compress_ms
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    stats = {l: t.stats.as_dict() for l, t in tabs.items()}
    n_rewrites = sum(s["n_rewrites"] for s in stats.values())

    # dominant kernel group: the fill of the largest lattice (HIP events on the solve's stream)
    big = max(sizes, key=sizes.get)
    big_fill_ms = fill_ms[big] / args.steps
    big_prefill_ms = prefill_ms[big] / args.steps
    big_kind = next(lat["kind"] for label, lat, _ in cfg["lattices"] if label == big)
    fused = big_kind in (W.KIND_FUSED_MM_ADD_RELU, W.KIND_FUSED_BOUNDED, W.KIND_MATMUL_CHAIN)    # two reads for the bufferize
    n_launch = stats[big]["n_levels_run"]
    has_deps = any(deps for label, _, deps in cfg["lattices"] if label == big)
    kernel_text = ("fill of table %s: plan_kernel, sort_work_kernel, the (INF, NONE) pre-fill (%s), "
                   "fill_kernel / fill_big_kernel per dependency level"
                   % (big, "fill_ones_short_kernel, beside the fills of the tables it reads" if has_deps else "inside plan_kernel"))
    if big_kind in W.BOUNDED_KINDS + (W.KIND_MOVE, W.KIND_MATMUL_MOVES):
        # one launch per diagonal: dependency level of shapes + rank (sum of the operand levels)
        n_launch += W.n_operands(big_kind) * (cfg["target"]["n_levels"] - 1)
        kernel_text = "fill of table %s: fill_bounded_kernel, one launch per diagonal of (dependency level, rank)" % big
    n_big, adm_big = sizes[big], stats[big]["n_admissible"]
    algo_bytes = method_bytes(n_big, adm_big, fused)
    algo_bytes_per_launch = algo_bytes / n_launch
    avg_launch_ms = big_fill_ms / n_launch
    achieved = algo_bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    traffic, stale = measured_traffic(args.config, big)
    n_adm_total = sum(s["n_admissible"] for s in stats.values())

    def frac(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS if ms > 0 else None

    out = {
        "metric": "specs solved/sec (full lattice fill + compression, 1 GPU)",
        "value": total_specs / (ms_per_step * 1e-3),
        "unit": "specs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": "config %d%s: %s" % (args.config, "" if args.max_size is None else " with sizes <= %d" % args.max_size,
                                                      ", ".join("%s %d specs" % (l, n) for l, n in sizes.items())),
                   "seed": args.config if args.seed is None else args.seed},
        # the lattice points of the metric are mostly Specs that do not fit their levels, whose
        # whole cost is a streaming store; the work of the method is in the admissible ones
        "admissible_specs_per_s": n_adm_total / (ms_per_step * 1e-3),
        "rewrites_per_s": n_rewrites / (ms_per_step * 1e-3),
        "detail": {l: {"specs": sizes[l], "fill_ms": fill_ms[l] / args.steps, "prefill_ms": prefill_ms[l] / args.steps,
                       "compress_ms": comp_ms[l] / args.steps,
                       "admissible": stats[l]["n_admissible"], "rewrites": stats[l]["n_rewrites"],
                       "launches": stats[l]["n_levels_run"],
                       "decision_boxes": stats[l]["n_decision_boxes"], "cost_boxes": stats[l]["n_cost_boxes"],
                       "scratch_used": stats[l]["scratch_used"]} for l in sizes},
        "roofline": {"bound": "hbm", "kernel": kernel_text,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None if traffic is None or stale else traffic / n_launch,
                     "launches_per_step": n_launch, "avg_launch_ms": avg_launch_ms,
                     "algorithmic_bytes_per_launch": algo_bytes_per_launch,
                     "algorithmic_bytes": "10 B per Spec + 8 B per admissible Spec%s" % (" + 16 B per admissible fused Spec" if fused else ""),
                     "traffic_summary_stale": stale},
    }
    R = out["roofline"]
    # the same fill against other byte counts: what the counters measured, and the dense formula
    # (18 B for every Spec, as if every cost were read back), which over-counts this workload
    R["measured_traffic_frac"] = None if traffic is None or stale else frac(traffic, big_fill_ms)
    R["frac_dense_formula"] = frac(18 * n_big, big_fill_ms)
    # the two kernel groups of that fill: the streaming pre-fill (with the work lists), and the
    # level kernels, which read and write the admissible Specs only
    big_levels_ms = big_fill_ms - big_prefill_ms
    R["groups"] = {
        "prefill": {"ms": big_prefill_ms, "bytes": 10 * n_big, "frac": frac(10 * n_big, big_prefill_ms)},
        "levels": {"ms": big_levels_ms, "bytes": algo_bytes - 10 * n_big + 10 * adm_big,
                   "frac": frac(algo_bytes - 10 * n_big + 10 * adm_big, big_levels_ms),
                   "what": "reads of the admissible Specs' sub-Spec costs and the second write of their entries"},
    }
    # fill + compression of that table: the compression has to read the entries of the Specs that
    # fit (10 B each) and a bit per Spec saying which those are
    big_both_ms = big_fill_ms + comp_ms[big] / args.steps
    R["fill_and_compress_frac"] = frac(algo_bytes + 10 * adm_big + n_big // 8, big_both_ms)

    if not args.no_cpu_baseline:
        # the oracle as it stands (one thread, gcc -O2, no -march=native: the library is built on
        # another machine than the one it runs on), on the whole workload; beside it the sample of
        # the same workload with sizes up to 128, which takes a tenth of the time
        from oracle import oracle as O

        def timed(c):
            t1 = time.perf_counter()
            res = O.solve_config(c)
            t_fill = time.perf_counter() - t1
            for label, lat, _ in c["lattices"]:
                O.compress_table(c["target"], lat, res[label]["cost"], res[label]["argmin"])
            t_all = time.perf_counter() - t1
            return sum(len(r["cost"]) for r in res.values()), t_fill, t_all

        legs = {}
        sample_max = {5: 128, 7: 16, 8: 4, 9: 12}.get(args.config)
        if not args.cpu_sample_only:
            legs["full"] = timed(cfg)
        if sample_max is not None and (args.max_size is None or sample_max < args.max_size):
            legs["sample"] = timed(W.config(args.config, seed=args.seed, max_size=sample_max))
        main_leg = "full" if "full" in legs else "sample"
        n_s, t_fill, t_all = legs[main_leg]
        what = {"full": "config %d, the whole workload" % args.config,
                "sample": "config %d with sizes <= %s" % (args.config, sample_max)}
        out["cpu_baseline"] = {"value": n_s / t_all, "unit": "specs/s", "cores": 1, "host_cores": os.cpu_count(),
                               "kind": "oracle",
                               "sample": "%s: %d specs, fill + both box lists, %.1f s on one thread" % (what[main_leg], n_s, t_all),
                               "fill_only_value": n_s / t_fill}
        if main_leg == "full" and "sample" in legs:
            n2, f2, a2 = legs["sample"]
            out["cpu_baseline"]["smaller_sample"] = {"value": n2 / a2, "fill_only_value": n2 / f2,
                                                     "sample": "%s: %d specs, %.1f s" % (what["sample"], n2, a2)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
