"""Benchmark of the batched strategy-search DP on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]
                    [--mode bp|nobp|bp-general|nobp-general] [--also nobp,bp-general]
                    [--also-configs 0,1,2,4]

A step is one pass of the whole hot path over one batch whose inputs are already resident
in HBM: strategy enumeration, cost-table builder (model workloads), batched forward DP,
final reductions and the backtrace of the best instance.  Prints ONE JSON line: the main
workload (configs[3]) at the top level, the other four configurations under `other_configs`,
every block with its own latency and roofline (vector ALU, HBM and LDS fractions).
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

# Vector-ALU peak for the instructions this path uses (plain fp32 add / compare / select,
# one result per lane per issue, no packed or fused forms):
# 256 CUs x 4 SIMDs x 16 lanes per clock x 2.4 GHz.  The published 157.3 TFLOP/s is the
# same machine counting a packed (x2) fused multiply-add (x2) on every lane.
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
HBM_PEAK_GBS = 8000.0
# LDS: 128 bytes per clock and compute unit (4-byte accesses), 256 CUs, 2.4 GHz
LDS_PEAK_TBS = 256 * 128 * 2.4e9 / 1e12
# HBM and LDS bytes per launch as the profiler counted them (rocprofv3 --pmc, scaled by a
# copy and an LDS kernel of known size), written by paper_2504_21411_amd.profile_summary
PROFILED = os.path.join(ROOT, "profiles", "traffic.json")


def ops_per_relaxation(kernel: str, mode: str, S: int) -> float:
    """Vector-ALU instructions per relaxation that the kernel's algorithm needs.

    min only: one add and half of a three-input minimum.  Flat argmin (push and generic
    kernels): add, compare, two selects.  Two-level argmin (tile kernel): per chunk of
    eight candidates eight adds, four minimum instructions, one compare and two selects
    (15/8), plus the second look at one chunk per target state (8 adds, 8 compares,
    8 selects = 24 per S relaxations).
    """
    if mode == "nobp":
        return 1.5
    if kernel in ("k_dp_tile", "k_dp_wide"):
        return 15.0 / 8.0 + 24.0 / S
    return 4.0


def class_ops_per_row(S: int, nc: int, maxlen: int, nobp: bool) -> float:
    """Vector-ALU (and LDS-minimum) operations per lane that the class kernel's algorithm
    needs for one source row: rebuilding C from the compact plane (one add per strategy),
    the class minima (one minimum per strategy), nc x nc relaxations priced as in the
    general kernels (1.5 min-only, 15/8 with the two-level argmin), and per target class the
    second look at one chunk of eight classes (24) and at the members of one class (3 each).
    """
    ops = 2.0 * S
    if nobp:
        return ops + 1.5 * nc * nc
    return ops + 15.0 / 8.0 * nc * nc + nc * (24.0 + 3.0 * maxlen)


def load_profiled():
    try:
        with open(PROFILED) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def cpu_baseline(w, cfg_index, target_relax=3.0e10):
    """The oracle as it stands on a bounded sample of the same workload: the first instances
    one after the other on one core (about target_relax relaxations, at least one instance,
    layers cut off if one instance alone is more than that), and as independent
    single-threaded solves side by side on up to 16 cores.  Returns (one, many or None)."""
    import oracle
    E0 = int(w.budget[0])
    per_layer = (E0 + 1) * w.S * w.S
    Ls = int(max(2, min(w.L, 1 + target_relax // per_layer)))
    n1 = int(max(1, min(w.B, target_relax // max(1, (Ls - 1) * per_layer))))
    P = int(min(16, os.cpu_count() or 1, w.B))
    nP = int(min(w.B, P * n1))
    n = max(n1, nP)
    if w.kind == "model":
        desc = oracle.enumerate_strategies(**w.enum)
        T, O, R = oracle.build_tables(desc, w.layer[:n], w.hw, w.rmodel, w.M)
    else:
        T, O, R = w.T[:n], w.O[:n], w.R
    relax_of = lambda k: float(sum((Ls - 1) * (int(e) + 1) * w.S * w.S for e in w.budget[:k]))

    def timed(k, threads):
        t0 = time.perf_counter()
        oracle.solve_batch(T[:k, :Ls], O[:k, :Ls], R, w.r_index[:k, :Ls], w.budget[:k],
                           threads=threads)
        return time.perf_counter() - t0

    dt = timed(n1, 1)
    what = f"first {Ls} of {w.L} layers" if Ls < w.L else f"all {w.L} layers"
    one = {"value": relax_of(n1) / dt / 1e9, "unit": "Grelax/s", "cores": 1, "kind": "oracle",
           "sample": f"instances 0..{n1 - 1} of cfg{cfg_index} one after the other, {what}, "
                     f"{relax_of(n1) / 1e9:.2f} G relaxations in {dt:.1f} s"}
    if P < 2:
        return one, None
    dt = timed(nP, P)
    many = {"value": relax_of(nP) / dt / 1e9, "unit": "Grelax/s", "cores": P, "kind": "oracle",
            "sample": f"instances 0..{nP - 1} of cfg{cfg_index}, {P} independent single-threaded "
                      f"solves side by side, {what}, {relax_of(nP) / 1e9:.2f} G relaxations in "
                      f"{dt:.1f} s"}
    return one, many


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--mode", choices=["bp", "nobp", "bp-general", "nobp-general"], default="bp")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--min-warmup-seconds", type=float, default=0.5,
                    help="keep warming up at least this long (0 for short profiling runs)")
    ap.add_argument("--also", default="nobp,bp-general",
                    help="comma list of extra modes to time on the main workload ('' for none)")
    ap.add_argument("--also-configs", default="0,1,2,4",
                    help="comma list of further configs to time, with backpointers, and report "
                         "beside the main line ('' for none)")
    ap.add_argument("--instance-groups", type=int, default=0,
                    help="force this many chains of launches (0: the library's choice)")
    ap.add_argument("--fronts", type=int, default=-1,
                    help="class kernel: layer fronts per launch (knob 'fronts'; 0: one launch per "
                         "front; default: the library's choice)")
    ap.add_argument("--no-single-chain", action="store_true",
                    help="do not time the one-chain variant beside a multi-chain forward pass")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (reference for HBM byte counters)")
    ap.add_argument("--lds-calibration", action="store_true",
                    help="only run LDS kernels of known size (reference for LDS counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (the batch would shard over "
                 "GPUs by instance; no multi-GPU path exists). Use --gpus 1.")

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    from paper_2504_21411_amd import binding, runner, workloads
    binding.load_library()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_per_launch": int(src.numel() * 4),
                          "launches": 5}))
        return
    if args.lds_calibration:
        out = {}
        for mode, name in enumerate(("load_b32", "load_b128", "store_b32", "atomic_b32")):
            for _ in range(5):
                out[name] = binding.gsearch_lds_calibration(mode, 4096)
            torch.cuda.synchronize()
        print(json.dumps({"lds_calibration_bytes_per_launch": out, "launches_each": 5}))
        return

    profiled = load_profiled()

    def time_mode(mode, w, dw, cfg_index, steps, groups_forced=0, single_chain=True):
        relax = w.relaxations()
        # "bp" / "nobp": with or without a backpointer stream; "-general": the layout classes
        # of the strategies are withheld from the solve, so the general kernels run
        classes = not mode.endswith("-general")
        nobp = mode.startswith("nobp")
        flags = binding.GSEARCH_FLAG_NO_BACKPOINTERS if nobp else 0
        with runner.make_context(w, flags=flags) as ctx:
            ctx.gsearch_set_profiling(True)
            if groups_forced:
                ctx.gsearch_set_instance_groups(groups_forced)
            if args.fronts >= 0:
                ctx.gsearch_set_knob("fronts", args.fronts)
            # W untimed steps, and in any case half a second of them: on the test box the
            # first launch phase that starts 0.1-0.2 s after a context's first solve has been
            # seen to stall on the host for about 40 ms, once per context
            tw = time.perf_counter()
            done = 0
            while done < args.warmup or time.perf_counter() - tw < args.min_warmup_seconds:
                runner.run_step(ctx, dw, backtrace="best", classes=classes)
                torch.cuda.synchronize()
                done += 1
            torch.cuda.synchronize()
            fwd = []
            t0 = time.perf_counter()
            for _ in range(steps):
                out = runner.run_step(ctx, dw, backtrace="best", classes=classes)
                fwd.append(ctx.gsearch_forward_ms())      # waits for this step's forward pass
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            assert ctx.gsearch_data_status() == 0
            best = int(out["best_instance"].cpu()[0])
            kernel = ctx.gsearch_forward_kernel()
            groups = max(1, ctx.gsearch_instance_groups())
            # what follows the search on the same context (host wall time, synchronised):
            # best cost for every budget at once, and the pipeline-aware outer reduction
            extras = {}
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(5):
                ctx.gsearch_budget_curve()
            torch.cuda.synchronize()
            extras["budget_curve_ms"] = (time.perf_counter() - t1) * 1e3 / 5
            meta = getattr(w, "meta", None) or {}
            if meta.get("groups") is not None:
                # (pipeline degree, split, micro-batch count) candidates of the outer search:
                # CSR offsets, member instances, micro-batch counts
                go, gm, gk = (torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()
                              for a in meta["groups"][:3])
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(5):
                    ctx.gsearch_pipeline_reduce(go, gm, gk)
                torch.cuda.synchronize()
                extras["pipeline_reduce_ms"] = (time.perf_counter() - t1) * 1e3 / 5
                extras["pipeline_candidates"] = int(gk.numel())
            # Share of the (layer, budget row) pairs the forward kernels really computed:
            # source rows below the prefix sum of the per-layer minimum memory hold +inf and
            # are filled without being computed (64-row tile granularity); source rows above
            # E minus the suffix sum of the remaining layers' minimum memory lead to no
            # complete plan within the budget and are skipped.  Reporting only.
            O = (out["O"] if "O" in out else dw.O).cpu().numpy().astype(np.int64)
            mo = np.minimum(O.min(axis=2), w.M + 1)
            low = np.minimum(np.cumsum(mo, axis=1), w.M + 1)
            top = np.minimum(np.cumsum(mo[:, ::-1], axis=1)[:, ::-1], w.M + 1)  # layers l..L-1
            rows = w.budget.astype(np.int64)[:, None] + 1
            skipped = np.minimum(low[:, :-1] // 64 * 64, rows)
            upper = np.maximum(rows - top[:, 1:], 0)          # useful source rows of front l
            active = np.maximum(upper - np.minimum(skipped, upper), 0)
            executed = float(active.sum()) / float((rows * (w.L - 1)).sum())
            if not kernel.startswith(("k_dp_push", "k_dp_tile", "k_dp_wide", "k_dp_class")):
                executed = 1.0
            n_class = int(out["n_class"].cpu()[0]) if "n_class" in out else None
            computed = float(active.sum()) / (w.L - 1)
            if kernel.startswith("k_dp_class"):
                # Compact planes: a front reads and writes one float per computed source
                # row and CLASS (plus one backpointer byte).
                rc = out["r_class"].cpu().numpy()
                max_len = int(np.bincount(rc).max())
                class_rows = computed
                front_bytes = class_rows * n_class * (8.0 if nobp else 9.0)
            else:
                # algorithmic HBM bytes of one layer front: every computed source row is
                # read once (4 B per state) and every useful target row (those the next front,
                # or the result, reads) written once (4 B per state); backpointers: 1 B per
                # target state
                nxt = np.concatenate([top[:, 2:], np.zeros((top.shape[0], 1), np.int64)], axis=1)
                targets = float(np.maximum(rows - nxt, 0).sum()) / (w.L - 1)
                front_bytes = (computed * 4.0 + targets * 4.0) * w.S
                if not nobp:
                    front_bytes += targets * w.S
            if kernel == "k_dp_small":
                front_bytes = 0.0 if nobp else float(rows.sum()) * w.S   # planes stay in LDS
        ms_step = dt * 1e3 / steps
        fwd_ms = sum(fwd) / len(fwd)
        # The batch runs as `groups` chains of L-1 launches side by side (one stream each);
        # every chain spans the forward time, so a launch lasts fwd/(L-1) on average and
        # works on 1/groups of a layer front while the other chains' launches share the chip.
        # (k_dp_small runs all fronts in ONE launch and k_dp_class_fronts 64 per launch: a
        # "launch" below is then a layer front's share of it.)
        launches = w.L - 1
        launch_s = fwd_ms * 1e-3 / launches
        key = f"{cfg_index}/{mode}" + (f"/groups{groups_forced}" if groups_forced else "") \
            + ("/perfront" if kernel == "k_dp_class" and args.fronts == 0 else "")
        prof = dict((profiled.get("entries") or {}).get(key) or {})
        fronts_per_launch = 1.0
        if kernel == "k_dp_class_fronts" and prof.get("calls") and prof.get("solves"):
            # a launch of this kernel covers up to 64 layer fronts: the profile's per-dispatch
            # figures are brought to one layer front (dispatches per solve / (L - 1))
            fronts_per_launch = (w.L - 1) / (prof["calls"] / prof["solves"])
            for name in ("avg_us", "traffic_bytes", "lds_bytes", "fetch_bytes", "write_bytes"):
                if prof.get(name) is not None:
                    prof[name] = prof[name] / fronts_per_launch
        common = {"kernel": kernel, "concurrent_launches": groups,
                  "layer_fronts_per_launch": fronts_per_launch,
                  "traffic": prof.get("traffic_bytes"),
                  "traffic_profiled_kernel": prof.get("kernel")}
        if kernel.startswith("k_dp_class"):
            # With the transition classes the arithmetic shrinks to one minimum per class
            # and one relaxation per pair of classes, and with the compact planes the
            # traffic to 2 floats per row and class.
            opr_row = class_ops_per_row(w.S, n_class, max_len, nobp)
            ops = opr_row * class_rows / groups
            per_launch = ops / launch_s / 1e12
            alu_frac = per_launch * groups / ALU_PEAK_TLANEOPS
            executed_nominal = executed * (n_class * n_class + w.S) / float(w.S * w.S)
            extra = dict(classes=n_class, longest_class=max_len, ops_per_row=opr_row)
        else:
            opr = ops_per_relaxation(kernel, "nobp" if nobp else "bp", w.S)
            ops = opr * relax * executed / launches / groups        # executed, per launch
            per_launch = ops / launch_s / 1e12
            alu_frac = per_launch * groups / ALU_PEAK_TLANEOPS
            executed_nominal = executed
            extra = dict(ops_per_relaxation=opr)
        hbm_gbs = front_bytes / launch_s / 1e9                  # same launches, bytes moved
        hbm_frac = hbm_gbs / HBM_PEAK_GBS
        lds = None
        if prof.get("lds_bytes") is not None:
            # LDS bytes per launch as profiled (all concurrent launches together) over the
            # live launch duration
            lds_tbs = prof["lds_bytes"] * groups / launch_s / 1e12
            lds = {"achieved": lds_tbs, "peak": LDS_PEAK_TBS, "unit": "TB/s",
                   "frac": lds_tbs / LDS_PEAK_TBS, "bytes_per_launch_profiled": prof["lds_bytes"]}
        if hbm_frac > alu_frac:
            # few strategies per state (min-only pass of the outer-search batch): the plane
            # traffic, not the arithmetic, is the tighter roof
            roof = dict(common, bound="hbm", achieved=hbm_gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=hbm_frac, achieved_per_launch=hbm_gbs / groups)
        else:
            roof = dict(common, bound="alu", achieved=per_launch * groups,
                        peak=ALU_PEAK_TLANEOPS, unit="Tlaneop/s", frac=alu_frac,
                        achieved_per_launch=per_launch)
        roof.update(alu_frac=alu_frac, hbm_frac=hbm_frac, hbm_gbs=hbm_gbs, lds=lds,
                    algorithmic_bytes_per_launch=front_bytes / groups,
                    executed_fraction_of_nominal_relaxations=executed_nominal, **extra)
        roof["frac_is"] = ("one chain of launches, HIP events over the forward pass" if groups == 1
                           else f"{groups} chains of launches overlapping on parallel streams, "
                                "HIP events over the forward pass (a profiler serialises them: "
                                "see frac_single_chain)")
        if prof.get("avg_us") is not None:
            # the same algorithmic work per launch over the kernel-trace average of the
            # profile (dispatches serialised, about a microsecond of tracing each): the figure
            # that profiles/ alone reproduces
            roof["profiled_kernel_avg_us"] = prof["avg_us"]
            if roof["bound"] == "alu":
                roof["frac_at_profiled_duration"] = ops / (prof["avg_us"] * 1e-6) / 1e12 \
                    / ALU_PEAK_TLANEOPS
            else:
                roof["frac_at_profiled_duration"] = front_bytes / groups / (prof["avg_us"] * 1e-6) \
                    / 1e9 / HBM_PEAK_GBS
        res = {"mode": mode, "ms_per_step": ms_step, "forward_ms": fwd_ms,
               "grelax_per_s": relax / (ms_step * 1e-3) / 1e9,
               "forward_grelax_per_s": relax / (fwd_ms * 1e-3) / 1e9,
               "executed_grelax_per_s": relax * executed_nominal / (ms_step * 1e-3) / 1e9,
               "kernel_avg_us": fwd_ms * 1e3 / launches,
               "roofline": roof, "best_instance": best, **extras}
        if groups > 1 and single_chain and not args.no_single_chain:
            # the same forward pass as ONE chain of launches: what a kernel trace can confirm
            one = time_mode(mode, w, dw, cfg_index, max(3, steps // 2), groups_forced=1,
                            single_chain=False)
            roof["frac_single_chain"] = one["roofline"]["frac"]
            roof["single_chain_kernel_avg_us"] = one["kernel_avg_us"]
            roof["single_chain_forward_ms"] = one["forward_ms"]
            roof["single_chain_profiled_kernel_avg_us"] = \
                one["roofline"].get("profiled_kernel_avg_us")
            roof["frac_single_chain_at_profiled_duration"] = \
                one["roofline"].get("frac_at_profiled_duration")
        return res

    w = workloads.get_config(args.config)
    dw = runner.DeviceWorkload(w)
    main_res = time_mode(args.mode, w, dw, args.config, args.steps, args.instance_groups)
    also = [m for m in args.also.split(",") if m and m != args.mode]
    if w.kind != "model":       # table workloads state no classes: "-general" is the same run
        also = [m for m in also if not m.endswith("-general")]
    extra = [time_mode(m, w, dw, args.config, args.steps, args.instance_groups) for m in also]
    relax = w.relaxations()
    others = []
    for c in [int(x) for x in args.also_configs.split(",") if x and int(x) != args.config]:
        wc = workloads.get_config(c)
        res = time_mode("bp", wc, runner.DeviceWorkload(wc), c, args.steps)
        res["workload"] = f"configs[{c}] {wc.name}: B={wc.B} L={wc.L} S={wc.S} M={wc.M}"
        res["relaxations_per_step"] = wc.relaxations()
        others.append(res)

    general = next((e for e in extra if e["mode"] == "bp-general"), None)
    line = {
        "metric": "G DP relaxations/sec (min-plus updates) + batch search latency, 1 MI355X",
        "value": main_res["grelax_per_s"], "unit": "Grelax/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {w.name}: B={w.B} L={w.L} S={w.S} "
                               f"M={w.M}", "mode": args.mode,
                   "relaxations_per_step": relax},
        # `value` counts the NOMINAL relaxations of the metric's definition (B (L-1) (E+1) S^2);
        # with the layout classes of the strategies the kernel executes this share of them
        # for bit-identical results, and with the classes withheld (a general R) it runs at
        # general_r_grelax_per_s
        "executed_fraction": main_res["roofline"]["executed_fraction_of_nominal_relaxations"],
        "executed_grelax_per_s": main_res["executed_grelax_per_s"],
        "general_r_grelax_per_s": general["grelax_per_s"] if general else None,
        "target_50pct_of_roofline_met": bool(main_res["roofline"]["frac"] >= 0.5),
        "search_latency_ms": main_res["ms_per_step"],
        "forward_ms": main_res["forward_ms"],
        "forward_grelax_per_s": main_res["forward_grelax_per_s"],
        "kernel_avg_us": main_res["kernel_avg_us"],
        "budget_curve_ms": main_res.get("budget_curve_ms"),
        "roofline": main_res["roofline"],
        "traffic_commit": profiled.get("commit"),
    }
    if extra:
        line["other_modes"] = extra
    if others:
        line["other_configs"] = others
        for o in others:
            if "pipeline_reduce_ms" in o:
                line["pipeline_reduce_ms"] = o["pipeline_reduce_ms"]
    if not args.no_cpu_baseline:
        line["cpu_baseline"], many = cpu_baseline(w, args.config)
        if many:
            line["cpu_baseline_all_cores"] = many
    print(json.dumps(line))


if __name__ == "__main__":
    main()
