"""Turns rocprofv3 result databases of bench.py runs into profiles/traffic.json.

    python -m paper_2504_21411_amd.profile_summary --root <dir> --commit <hash> \
        [--out profiles/traffic.json] [--markdown-dir profiles] [--notes profiles/notes.json]
    python -m paper_2504_21411_amd.profile_summary --from-json profiles/traffic.json \
        --markdown-dir profiles [--notes profiles/notes.json]

<dir> holds one folder per measured run, named like the key bench.py looks up
("3_bp", "3_bp-general_groups1", "1_bp", ...: configuration, mode, forced instance groups), and
one folder "calib".  Inside a run folder, one sub-folder per rocprofv3 pass, each with the
*_results.db that `rocprofv3 -d <sub-folder>` wrote:

    kt      --kernel-trace --stats
    fetch   --pmc FETCH_SIZE
    write   --pmc WRITE_SIZE
    sq      --pmc SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_SALU
                  SQ_WAIT_INST_ANY SQ_INSTS_SMEM SQ_INSTS_LDS
    lds     --pmc SQ_INSTS_LDS_LOAD SQ_INSTS_LDS_STORE SQ_INSTS_LDS_ATOMIC
                  SQ_INSTS_LDS_LOAD_BANDWIDTH SQ_INSTS_LDS_STORE_BANDWIDTH
                  SQ_INSTS_LDS_ATOMIC_BANDWIDTH SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS

and "calib" holds copy_fetch / copy_write (bench.py --copy-calibration under FETCH_SIZE /
WRITE_SIZE) and lds (bench.py --lds-calibration under the lds counter set).  Counters are
averaged per dispatch of the forward kernel (the gs::k_dp_* kernel with the largest total time
of the run).  HBM bytes = FETCH_SIZE and WRITE_SIZE scaled by what the same counters read for a
plain copy of known size; LDS bytes = the three LDS bandwidth counters scaled by what they read
for LDS kernels of known size (four-byte loads, stores and atomics; the sixteen-byte load
factor is recorded beside them).  Only reads the databases and writes the two files: no
measurement happens here.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sqlite3
import time


def _dbs(folder):
    return sorted(glob.glob(os.path.join(folder, "**", "*_results.db"), recursive=True))


def _tables(cur):
    return [r[0] for r in cur.execute("select name from sqlite_master where type in ('view','table')")]


def kernel_times(folder):
    """{kernel name: (calls, avg_us, min_us, max_us, total_ms)} of a kernel-trace pass."""
    out = {}
    for path in _dbs(folder):
        cur = sqlite3.connect(path).cursor()
        if "kernels" not in _tables(cur):
            continue
        for name, n, avg, mn, mx, tot in cur.execute(
                "select name, count(*), avg(end-start), min(end-start), max(end-start), "
                "sum(end-start) from kernels group by name"):
            out[name] = (int(n), avg / 1e3, mn / 1e3, mx / 1e3, tot / 1e6)
    return out


def counters(folder):
    """{kernel name: {counter: average per dispatch}} of a --pmc pass."""
    out = {}
    for path in _dbs(folder):
        cur = sqlite3.connect(path).cursor()
        if "counters_collection" not in _tables(cur):
            continue
        for kname, cname, avg in cur.execute(
                "select kernel_name, counter_name, avg(value) from counters_collection "
                "group by kernel_name, counter_name"):
            out.setdefault(kname, {})[cname] = float(avg)
    return out


def short(name):
    return name.replace("gs::", "").split("(")[0]


def forward_kernel(times):
    best = None
    for name, t in times.items():
        if "k_dp_" in name and (best is None or t[4] > times[best][4]):
            best = name
    return best


NAMES = {"0": "cfg0_single_decoder", "1": "cfg1_batch_decoder", "2": "cfg2_hetero_encdec",
         "3": "cfg3_large_dense", "4": "cfg4_outer_search"}
SHAPES = {"0": "B=1, L=24, S=12, M=256", "1": "B=64, L=48, S=44, M=2048", "2": "B=256, L=32, S=44, M=4096, K=4",
          "3": "B=8, L=128, S=96, M=16384", "4": "B=2048, L=32, S=24, M=2048"}
SQ = "SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_SALU SQ_WAIT_INST_ANY SQ_INSTS_SMEM SQ_INSTS_LDS"
LDS = "SQ_INSTS_LDS_LOAD SQ_INSTS_LDS_STORE SQ_INSTS_LDS_ATOMIC SQ_INSTS_LDS_LOAD_BANDWIDTH SQ_INSTS_LDS_STORE_BANDWIDTH SQ_INSTS_LDS_ATOMIC_BANDWIDTH SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS"


def write_markdown(d, folder, notes):
    """One short summary per kernel and workload, written from the same document as
    traffic.json; older *.md files in the folder are removed."""
    commit = d["commit"]
    cal = d["calibration"]
    for old in os.listdir(folder):
        if old.endswith(".md"):
            os.remove(os.path.join(folder, old))
    groups = {}
    for key, e in d["entries"].items():
        cfg = key.split("/")[0]
        kern = e["kernel"].replace("void ", "").split("<")[0]
        groups.setdefault((kern, cfg), []).append((key, e))
    for (kern, cfg), items in sorted(groups.items()):
        path = os.path.join(folder, f"{kern}_{NAMES[cfg]}.md")
        out = []
        out.append(f"# {kern} on configs[{cfg}] ({SHAPES[cfg]}) — rocprofv3 summary, MI355X\n")
        out.append(f"Measured at commit `{commit}` ({d['written']}); figures per dispatch of the forward kernel, "
                   f"averaged over the run. Written from `profiles/traffic.json` "
                   f"(`python -m paper_2504_21411_amd.profile_summary`).\n")
        out.append("Commands (from /tmp with TMPDIR=/tmp; `bench.py` is the repository's; `<B>` below):\n")
        for key, e in items:
            parts = key.split("/")
            extra = " --instance-groups 1" if "groups1" in parts else (" --fronts 0" if "perfront" in parts else "")
            out.append(f"    <B {key}> = python3 bench.py --config {parts[0]} --mode {parts[1]} --also= --also-configs= "
                       f"--no-cpu-baseline --no-single-chain --min-warmup-seconds 0.3 --warmup 3{extra}")
        out.append("")
        out.append("    rocprofv3 --kernel-trace --stats -d <dir>/kt -o r -- <B> --steps 8")
        out.append("    rocprofv3 --pmc FETCH_SIZE -d <dir>/fetch -o r -- <B> --steps 3")
        out.append("    rocprofv3 --pmc WRITE_SIZE -d <dir>/write -o r -- <B> --steps 3")
        out.append(f"    rocprofv3 --pmc {SQ} -d <dir>/sq -o r -- <B> --steps 3")
        out.append(f"    rocprofv3 --pmc {LDS} -d <dir>/lds -o r -- <B> --steps 3")
        out.append("    rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) -d <dir>/calib/copy_fetch -o c -- python3 bench.py --copy-calibration")
        out.append(f"    rocprofv3 --pmc <the LDS set> -d <dir>/calib/lds -o c -- python3 bench.py --lds-calibration\n")
        out.append("| run | kernel | calls | avg µs | min | max | HBM fetch MB | write MB | total MB | LDS MB | VALU wave-insts | SALU | SMEM | LDS insts | waves |")
        out.append("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        for key, e in items:
            c = e["counters"]
            g = lambda k: f"{c[k] / 1e6:.2f} M" if k in c else "-"
            out.append(f"| {key} | `{e['kernel'].replace('void ', '')}` | {e['calls']} | {e['avg_us']:.2f} | {e['min_us']:.2f} | {e['max_us']:.2f} | "
                       f"{e.get('fetch_bytes', 0) / 1e6:.2f} | {e.get('write_bytes', 0) / 1e6:.2f} | {e.get('traffic_bytes', 0) / 1e6:.2f} | "
                       f"{e.get('lds_bytes', 0) / 1e6:.1f} | {g('SQ_INSTS_VALU')} | {g('SQ_INSTS_SALU')} | {g('SQ_INSTS_SMEM')} | {g('SQ_INSTS_LDS')} | {int(c.get('SQ_WAVES', 0))} |")
        out.append("")
        out.append(f"Calibration: a 1 GiB device copy reads FETCH_SIZE = {cal['FETCH_SIZE_of_a_1GiB_copy']:.0f} and "
                   f"WRITE_SIZE = {cal['WRITE_SIZE_of_a_1GiB_copy']:.0f} per dispatch, so one unit is "
                   f"{cal['FETCH_SIZE_bytes_per_unit']:.0f} and {cal['WRITE_SIZE_bytes_per_unit']:.0f} bytes. LDS bytes = "
                   f"LOAD / STORE / ATOMIC_BANDWIDTH units x {cal['lds_load_b32_bytes_per_unit']:.0f} / "
                   f"{cal['lds_store_b32_bytes_per_unit']:.0f} / {cal['lds_atomic_b32_bytes_per_unit']:.0f} bytes (what the counters "
                   f"read for 2^30 four-byte loads, stores and float-minimum atomics of `gsearch_lds_calibration`; a sixteen-byte "
                   f"load reads {cal['lds_load_b128_bytes_per_unit']:.0f} bytes per unit, so kernels with wide LDS loads move up to "
                   f"twice the LDS bytes listed).\n")
        for key, e in items:
            if "k_dp_class_fronts" in e["kernel"] and e.get("solves"):
                out.append(f"Run {key}: one dispatch of this kernel covers up to 64 layer fronts "
                           f"({e['calls']} dispatches in {e['solves']} solves); divide the per-dispatch "
                           f"figures by the fronts per dispatch for one front.")
        for key, e in items:
            ok = e.get("other_kernels", [])[:6]
            out.append(f"Other kernels of run {key}: " + ", ".join(f"`{o['kernel'].replace('void ', '')}` {o['calls']} x {o['avg_us']:.1f} µs" for o in ok) + ".")
        note = notes.get(f"{kern}|{cfg}")
        if note:
            out.append("")
            out.append(note)
        open(path, "w").write("\n".join(out) + "\n")
        print(path, os.path.getsize(path))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--root", default=None)
    ap.add_argument("--commit", default="unknown")
    ap.add_argument("--out", default=os.path.join("profiles", "traffic.json"))
    ap.add_argument("--text", default=None)
    ap.add_argument("--from-json", default=None,
                    help="skip the databases: rewrite the *.md summaries from this traffic.json")
    ap.add_argument("--markdown-dir", default=None, help="write one *.md summary per kernel here")
    ap.add_argument("--notes", default=None,
                    help="JSON {\"<kernel>|<config>\": \"remark\"} appended to the summaries")
    args = ap.parse_args()
    notes = json.load(open(args.notes)) if args.notes else {}
    if args.from_json:
        write_markdown(json.load(open(args.from_json)), args.markdown_dir or "profiles", notes)
        return

    calib = {}
    cdir = os.path.join(args.root, "calib")
    copy_bytes = float(1 << 30)
    for what, counter in (("copy_fetch", "FETCH_SIZE"), ("copy_write", "WRITE_SIZE")):
        vals = [v[counter] for k, v in counters(os.path.join(cdir, what)).items()
                if counter in v and v[counter] > 0.25 * copy_bytes / 1024 / 4]
        if vals:
            # the copy kernel is the dispatch that moves about 1 GiB each way
            calib[counter + "_bytes_per_unit"] = copy_bytes / max(vals)
            calib[counter + "_of_a_1GiB_copy"] = max(vals)
    lds_known = {"0": ("load_b32", 4), "1": ("load_b128", 16), "2": ("store_b32", 4),
                 "3": ("atomic_b32", 4)}
    for kname, v in counters(os.path.join(cdir, "lds")).items():
        if "k_lds_calibration" not in kname:
            continue
        mode = kname.split("<")[1].split(">")[0].strip()
        label, width = lds_known[mode]
        known = 1024 * 256 * 4096 * width
        c = {"load_b32": "SQ_INSTS_LDS_LOAD_BANDWIDTH", "load_b128": "SQ_INSTS_LDS_LOAD_BANDWIDTH",
             "store_b32": "SQ_INSTS_LDS_STORE_BANDWIDTH",
             "atomic_b32": "SQ_INSTS_LDS_ATOMIC_BANDWIDTH"}[label]
        calib["lds_" + label + "_counters"] = {k: v[k] for k in sorted(v)}
        if v.get(c, 0) > 0:
            calib["lds_" + label + "_bytes_per_unit"] = known / v[c]

    entries = {}
    text = []
    for run in sorted(os.listdir(args.root)):
        folder = os.path.join(args.root, run)
        if run == "calib" or not os.path.isdir(folder):
            continue
        key = run.replace("_", "/")
        times = kernel_times(os.path.join(folder, "kt"))
        fk = forward_kernel(times)
        if fk is None:
            continue
        e = {"kernel": short(fk), "calls": times[fk][0], "avg_us": times[fk][1],
             "min_us": times[fk][2], "max_us": times[fk][3]}
        # solves of the kernel-trace pass: every solve launches the prepare kernel once
        solves = [t[0] for n, t in times.items() if "k_bin_unit" in n]
        if solves:
            e["solves"] = solves[0]
        merged = {}
        for sub in ("fetch", "write", "sq", "lds"):
            c = counters(os.path.join(folder, sub))
            hit = [k for k in c if short(k) == short(fk)]
            if hit:
                merged.update(c[hit[0]])
        e["counters"] = {k: merged[k] for k in sorted(merged)}
        if "FETCH_SIZE" in merged and "FETCH_SIZE_bytes_per_unit" in calib:
            e["fetch_bytes"] = merged["FETCH_SIZE"] * calib["FETCH_SIZE_bytes_per_unit"]
        if "WRITE_SIZE" in merged and "WRITE_SIZE_bytes_per_unit" in calib:
            e["write_bytes"] = merged["WRITE_SIZE"] * calib["WRITE_SIZE_bytes_per_unit"]
        if "fetch_bytes" in e and "write_bytes" in e:
            e["traffic_bytes"] = e["fetch_bytes"] + e["write_bytes"]
        lds = 0.0
        have = False
        for counter, label in (("SQ_INSTS_LDS_LOAD_BANDWIDTH", "load_b32"),
                               ("SQ_INSTS_LDS_STORE_BANDWIDTH", "store_b32"),
                               ("SQ_INSTS_LDS_ATOMIC_BANDWIDTH", "atomic_b32")):
            f = calib.get("lds_" + label + "_bytes_per_unit")
            if counter in merged and f:
                lds += merged[counter] * f
                have = True
        if have:
            e["lds_bytes"] = lds
        others = sorted(((t[4], short(n), t[0], t[1]) for n, t in times.items() if n != fk),
                        reverse=True)[:8]
        e["other_kernels"] = [{"kernel": n, "calls": c, "avg_us": a} for _, n, c, a in others]
        entries[key] = e
        text.append(f"{key}: {e['kernel']} calls {e['calls']} avg {e['avg_us']:.2f} us "
                    f"(min {e['min_us']:.2f}, max {e['max_us']:.2f}); "
                    f"HBM {e.get('traffic_bytes', float('nan')) / 1e6:.2f} MB "
                    f"(fetch {e.get('fetch_bytes', float('nan')) / 1e6:.2f}, "
                    f"write {e.get('write_bytes', float('nan')) / 1e6:.2f}), "
                    f"LDS {e.get('lds_bytes', float('nan')) / 1e6:.2f} MB per launch")
    doc = {"commit": args.commit, "written": time.strftime("%Y-%m-%d"), "device": "MI355X (gfx950)",
           "calibration": calib, "entries": entries}
    with open(args.out, "w") as f:
        json.dump(doc, f, indent=1, sort_keys=True)
        f.write("\n")
    if args.text:
        with open(args.text, "w") as f:
            f.write("\n".join(text) + "\n")
    print("\n".join(text))
    if args.markdown_dir:
        write_markdown(doc, args.markdown_dir, notes)


if __name__ == "__main__":
    main()
