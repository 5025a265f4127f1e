"""Turns the CSV output of three rocprofv3 runs of bench.py on one workload into a short
text summary and a record of measured HBM traffic.

The three runs (same bench.py arguments, which must include ``--copy-probe MIB`` so that a
device copy of known size is in each counter run):

    rocprofv3 --kernel-trace --stats --output-format csv -d RUN/trace -- python3 bench.py ARGS
    rocprofv3 --pmc FETCH_SIZE       --output-format csv -d RUN/fetch -- python3 bench.py ARGS
    rocprofv3 --pmc WRITE_SIZE       --output-format csv -d RUN/write -- python3 bench.py ARGS

with the trace run's stdout (bench.py's JSON line) saved as RUN/bench.json.  Then

    python -m paper_2605_14438_amd.profile_summary --run RUN --name NAME --args "ARGS"

writes profiles/NAME.md (per-kernel durations, traffic per forward of the two expert GEMM
stages against their algorithmic bytes) and adds the traffic of those stages to
profiles/traffic.json, keyed by workload and by a hash of the kernel sources, which is
where bench.py reads ``roofline.traffic`` from.

The counters are in KiB per dispatch up to a factor that depends on the machine; the
factor is taken from the copy in the same run (its size is known), one for FETCH_SIZE and
one for WRITE_SIZE, and stated in the summary.
"""
import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = "paper_2605_14438_amd/csrc"
COPY_KERNEL = "__amd_rocclr_copyBuffer"


def stage_of(kernel):
    """'gate_up' / 'down' for the kernels of the two expert GEMM stages, else None."""
    if "ffn_tile_kernel<" in kernel:
        targs = kernel.split("ffn_tile_kernel<", 1)[1].split(">", 1)[0].split(",")
        return "gate_up" if targs[3].strip() in ("true", "1") else "down"
    if "gate_up" in kernel:
        return "gate_up"
    if re.search(r"\bdown_", kernel) or "::down" in kernel:
        return "down"
    return None


def sources_of(kernels):
    files = {f"{CSRC}/common.hpp"}
    for k in kernels:
        if "stream" in k:
            files.add(f"{CSRC}/ffn_stream.hip")
        elif "tile" in k:
            files.add(f"{CSRC}/ffn_tiled.hip")
        else:
            files.add(f"{CSRC}/ffn_generic.hip")
    return sorted(files)


def sha16(paths):
    h = hashlib.sha256()
    for p in paths:
        with open(os.path.join(ROOT, p), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def one_csv(run, sub, suffix):
    hits = glob.glob(os.path.join(run, sub, "**", "*" + suffix), recursive=True)
    if not hits:
        raise SystemExit(f"{run}/{sub}: no *{suffix}")
    if len(hits) > 1:      # output of an earlier run left in the folder: the newest file counts
        hits.sort(key=os.path.getmtime)
        print(f"{run}/{sub}: {len(hits)} files *{suffix}, taking the newest", file=sys.stderr)
    return hits[-1]


def short(kernel):
    k = kernel.split("(")[0].replace("void ", "")
    return k if len(k) <= 70 else k[:67] + "..."


def read_stats(run):
    rows = []
    for r in csv.DictReader(open(one_csv(run, "trace", "kernel_stats.csv"))):
        rows.append({"name": r["Name"], "calls": int(r["Calls"]), "mean": float(r["AverageNs"]),
                     "min": float(r["MinNs"]), "max": float(r["MaxNs"]),
                     "total": float(r["TotalDurationNs"])})
    return rows


def read_counter(run, sub, counter):
    """kernel -> [dispatches, sum of the counter]; and the per-dispatch values of the copies"""
    agg = collections.defaultdict(lambda: [0, 0.0])
    copies = []
    for r in csv.DictReader(open(one_csv(run, sub, "counter_collection.csv"))):
        if r["Counter_Name"] != counter:
            continue
        a = agg[r["Kernel_Name"]]
        a[0] += 1
        a[1] += float(r["Counter_Value"])
        if COPY_KERNEL in r["Kernel_Name"]:
            copies.append(float(r["Counter_Value"]))
    return agg, copies


def copy_scale(copies, copy_kib, what):
    """The probe's copies are the largest in the run (pass a --copy-probe size above that of
    one weight tensor): mean over the dispatches within 2 % of the largest reading."""
    if not copies:
        raise SystemExit(f"no {COPY_KERNEL} dispatch in the {what} run: pass --copy-probe to bench.py")
    top = [c for c in copies if c >= 0.98 * max(copies)]
    raw = sum(top) / len(top)
    return copy_kib / raw, raw


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    ap.add_argument("--run", required=True, help="folder with trace/, fetch/, write/, bench.json")
    ap.add_argument("--name", required=True, help="profiles/NAME.md")
    ap.add_argument("--args", required=True, help="the bench.py arguments of the three runs")
    ap.add_argument("--title", default=None)
    a = ap.parse_args()

    m = re.search(r"--copy-probe[ =](\d+)", a.args)
    if not m:
        raise SystemExit("--args must contain --copy-probe MIB")
    copy_kib = int(m.group(1)) * 1024.0

    rec = None
    for line in open(os.path.join(a.run, "bench.json")):
        if line.startswith("{"):
            rec = json.loads(line)
    if rec is None:
        raise SystemExit("bench.json holds no JSON line")
    wl = rec["config"]["workload"]
    key = rec["config"]["point"]     # bench.py's label of the point: what it looks traffic up by

    stats = read_stats(a.run)
    fetch, fetch_copies = read_counter(a.run, "fetch", "FETCH_SIZE")
    write, write_copies = read_counter(a.run, "write", "WRITE_SIZE")
    fs, fraw = copy_scale(fetch_copies, copy_kib, "FETCH_SIZE")
    ws, wraw = copy_scale(write_copies, copy_kib, "WRITE_SIZE")

    ours = [s for s in stats if "beam::" in s["name"] and "probe" not in s["name"]
            and "pack_" not in s["name"]]
    forwards = max((s["calls"] for s in ours if "topk_mask" in s["name"]), default=0)
    if forwards == 0:
        raise SystemExit("no routing kernel in the trace: was this a forward run?")

    out = []
    out.append(f"# {a.title or key}: per-kernel time and HBM traffic")
    out.append("")
    out.append(f"Workload: `{wl}`, {rec['config']['kept_pairs']} kept pairs on "
               f"{rec['config']['experts_touched']} experts, weights {rec['config']['weights']}, "
               f"{rec['config']['weight_sets_rotated']} rotating copies of the expert weights.  "
               f"MI355X, ROCm 7.2, {forwards} forwards in the trace.")
    out.append("")
    out.append("Commands (from /tmp with TMPDIR=/tmp; `$R` = repo root, `$D` = an output folder):")
    out.append("")
    out.append(f"    rocprofv3 --kernel-trace --stats --output-format csv -d $D/trace -- python3 $R/bench.py {a.args} > $D/bench.json")
    out.append(f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $D/fetch -- python3 $R/bench.py {a.args}")
    out.append(f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $D/write -- python3 $R/bench.py {a.args}")
    out.append(f"    python -m paper_2605_14438_amd.profile_summary --run $D --name {a.name} --args \"{a.args}\"")
    out.append("")
    out.append("## Kernel trace (`kernel_stats.csv`)")
    out.append("")
    out.append("| kernel | calls | mean ns | min ns | max ns | per forward us |")
    out.append("|---|---|---|---|---|---|")
    layer_us = 0.0
    for s in sorted(ours, key=lambda s: -s["total"]):
        per_fwd = s["total"] / forwards / 1e3
        layer_us += per_fwd
        out.append(f"| {short(s['name'])} | {s['calls']} | {s['mean']:.0f} | {s['min']:.0f} | "
                   f"{s['max']:.0f} | {per_fwd:.1f} |")
    out.append("")
    ku = rec["layer"]["kernel_us"]
    out.append(f"Sum of the kernels: {layer_us:.1f} us per forward.  bench.py in the same run "
               f"(HIP events, under the profiler): {rec['us_per_layer']:.1f} us per layer, "
               f"`kernel_us` " + ", ".join(f"{k} {v:.1f}" for k, v in ku.items()) + ".")
    out.append("")
    out.append("## HBM traffic (`--pmc`, per forward)")
    out.append("")
    out.append(f"Calibration on the {copy_kib / 1024:.0f} MiB device copy of `--copy-probe` "
               f"(`{COPY_KERNEL}`): FETCH_SIZE reads {fraw:.1f} per copy, WRITE_SIZE {wraw:.1f}, "
               f"so **FETCH_SIZE x {fs:.3f} and WRITE_SIZE x {ws:.3f}** give KiB on this box.")
    out.append("")
    out.append("| stage | kernels | fetched MB | written MB | algorithmic MB | traffic / algorithmic | mean us | of peak |")
    out.append("|---|---|---|---|---|---|---|---|")

    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    table = json.load(open(tpath)) if os.path.exists(tpath) else {"records": []}
    commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"],
                            capture_output=True, text=True).stdout.strip() or "unknown"
    alg = rec["layer"]["stage_algorithmic"]
    for stage in ("gate_up", "down"):
        ks = sorted({k for k in list(fetch) + list(write) if stage_of(k) == stage})
        if not ks:
            continue
        fb = sum(fetch[k][1] for k in ks if k in fetch) / max(1, _forwards(fetch, forwards)) * fs * 1024
        wb = sum(write[k][1] for k in ks if k in write) / max(1, _forwards(write, forwards)) * ws * 1024
        us = sum(s["total"] for s in stats if stage_of(s["name"]) == stage) / forwards / 1e3
        ab, fl = alg[stage]["bytes"], alg[stage]["flops"]
        t_b, t_f = ab / 8e12, fl / 2.5e15
        peak = (f"{ab / (us * 1e-6) / 8e12:.3f} of HBM" if t_b >= t_f
                else f"{fl / (us * 1e-6) / 2.5e15:.3f} of MFMA")
        out.append(f"| {stage} | {', '.join(short(k) for k in ks)} | {fb / 1e6:.1f} | {wb / 1e6:.1f} | "
                   f"{ab / 1e6:.1f} | {(fb + wb) / ab:.3f} | {us:.1f} | {peak} |")
        files = sources_of(ks)
        table["records"] = [r for r in table["records"]
                            if not (r["workload"] == key and r["kernel"] == stage)]
        table["records"].append({
            "workload": key, "kernel": stage, "fetch_bytes": round(fb), "write_bytes": round(wb),
            "fetch_scale": round(fs, 4), "write_scale": round(ws, 4), "forwards": forwards,
            "mean_us": round(us, 2), "source_files": files, "source_sha16": sha16(files),
            "commit": commit, "profile": f"profiles/{a.name}.md"})
    out.append("")
    rf = rec["roofline"]
    out.append(f"Roofline of the dominant kernel as bench.py reports it in this run: bound {rf['bound']}, "
               f"{rf['achieved']:.0f} {rf['unit']} of {rf['peak']:.0f} = **{rf['frac']:.3f}** "
               f"(duration {rf['duration_us']:.1f} us from HIP events; the trace's mean is in the table).")
    out.append("")
    table["records"].sort(key=lambda r: (r["workload"], r["kernel"]))
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    with open(os.path.join(ROOT, "profiles", a.name + ".md"), "w") as f:
        f.write("\n".join(out))
    with open(tpath, "w") as f:
        json.dump(table, f, indent=1)
        f.write("\n")
    print("\n".join(out))


def _forwards(agg, fallback):
    n = max((v[0] for k, v in agg.items() if "topk_mask" in k), default=0)
    return n or fallback


if __name__ == "__main__":
    main()
