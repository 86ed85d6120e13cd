#!/usr/bin/env python3
"""rocprofv3 evidence for bench.py: collects a kernel trace and the HBM traffic counters of one
workload on the GPU machine, and turns them into the short summary kept under profiles/.

    python bench_profile.py collect  <workload> [--lazy]     on an MI355X; raw output -> <raw>/prof_<tag>/
    python bench_profile.py summarize <workload> [--lazy]    anywhere; <raw>/prof_<tag>/ -> profiles/ef_step_<tag>.md

<raw> is the folder named by EF_PROFILE_RAW (default: an untracked scratch folder of the checkout).

`collect` starts three rocprofv3 runs of bench.py as child processes, the program itself after
`--`, counters in runs of their own: --kernel-trace --stats, --pmc FETCH_SIZE, --pmc WRITE_SIZE.
Each run also executes a torch add kernel of known size (bench.py --calib), whose counter values
give the scale of the counters.  `summarize` writes, per kernel of the library: calls, average
duration, the algorithmic bytes one launch must move (layout arithmetic only), the achieved rate
against the 8 TB/s HBM peak, and the measured bytes per launch; the last go into a
`traffic-json:` line that bench.py reads for `roofline.traffic`.

Measurement infrastructure: nothing here is used by the library, the tests or the timed path.
"""
import argparse
import collections
import csv
import glob
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
TILE = 4096
HBM_PEAK = 8.0e12
RAW = os.environ.get("EF_PROFILE_RAW") or os.path.join(ROOT, "gpurun_out")      # raw profiler output (not tracked)
CALIB_KIB = 1048576.0           # the calibration kernel reads 2^28 floats and writes 2^28 floats


VARIANT = "sgdm"                # bench.py --variant of the run being collected or summarized


def tag_of(workload, lazy):
    return workload + ("_deferred" if lazy else "") + ("" if VARIANT == "sgdm" else "_" + VARIANT)


def bench_args(workload, lazy, steps):
    a = ["python3", os.path.join(ROOT, "bench.py"), "--workload", workload, "--steps", str(steps), "--warmup", "1",
         "--no-cpu", "--no-others", "--calib", "--variant", VARIANT]
    return a + (["--lazy"] if lazy else ["--no-deferred"])


def commands(workload, lazy):
    out = os.path.join(RAW, "prof_" + tag_of(workload, lazy))
    return out, [
        ["rocprofv3", "--kernel-trace", "--stats", "--output-format", "csv", "-d", os.path.join(out, "kt"), "-o", "kt", "--"]
        + bench_args(workload, lazy, 5),
        ["rocprofv3", "--pmc", "FETCH_SIZE", "--output-format", "csv", "-d", os.path.join(out, "fetch"), "-o", "f", "--"]
        + bench_args(workload, lazy, 3),
        ["rocprofv3", "--pmc", "WRITE_SIZE", "--output-format", "csv", "-d", os.path.join(out, "write"), "-o", "w", "--"]
        + bench_args(workload, lazy, 3),
    ]


def collect(workload, lazy):
    out, cmds = commands(workload, lazy)
    os.makedirs(out, exist_ok=True)
    env = dict(os.environ, TMPDIR="/tmp")
    for cmd in cmds:
        print("[bench_profile] " + " ".join(cmd), flush=True)
        with open(os.path.join(out, "last_run.log"), "w") as log:
            rc = subprocess.call(cmd, cwd="/tmp", env=env, stdout=log, stderr=subprocess.STDOUT, timeout=600)
        if rc != 0:
            print(open(os.path.join(out, "last_run.log")).read()[-3000:])
            sys.exit(rc)
    # the commit the tree was at: from git, or from EF_COMMIT where the tree travels without its history
    head = os.environ.get("EF_COMMIT") or subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"],
                                                         capture_output=True, text=True).stdout.strip()
    with open(os.path.join(out, "meta.json"), "w") as f:
        json.dump({"commit": head or None}, f)


# --------------------------------------------------------------- summarize ---

def short(name):
    """Kernel name as the library spells it, without arguments; None for kernels of other origin
    (except the calibration add)."""
    if "CUDAFunctorOnSelf_add" in name:
        return "torch add (calibration, 1 GiB -> 1 GiB)"
    name = name.replace("void ", "")
    if not name.startswith("ef::"):
        return None
    depth, out = 0, []
    for ch in name:                 # cut at the argument list, keeping template arguments
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            break
        out.append(ch)
    return "".join(out)


def layout_counts(w):
    offs = w.offsets
    ntiles = (w.d + TILE - 1) // TILE
    import numpy as np
    first = np.searchsorted(offs, np.arange(ntiles, dtype=np.int64) * TILE, side="right") - 1
    last_el = np.minimum((np.arange(ntiles, dtype=np.int64) + 1) * TILE, w.d) - 1
    last = np.searchsorted(offs, last_el, side="right") - 1
    full = (np.arange(ntiles, dtype=np.int64) + 1) * TILE <= w.d
    whole = (first == last) & full
    n_whole = int(whole.sum())
    el_whole = n_whole * TILE
    return dict(ntiles=int(ntiles), n_whole=n_whole, n_mixed=int(ntiles - n_whole), el_whole=el_whole,
                el_mixed=int(w.d - el_whole))


def algorithmic(kernel, w, c):
    """Bytes one launch of `kernel` must move on workload w (what the method itself needs: state read
    once and written once, sign bits, scales); None where no simple count applies."""
    d, B, M = w.d, w.B, w.M
    if kernel.startswith("ef::k_worker_tiles<false"):       # Algorithm 3: no momentum buffer
        return M * (12.125 * d + 4.0 * B)
    if kernel.startswith("ef::k_worker_tiles"):
        return M * (20.125 * d + 4.0 * B)
    if kernel.startswith("ef::k_worker_uniform"):
        return M * 20.125 * c["el_whole"]
    if kernel.startswith("ef::k_worker_mixed"):
        return M * (20.125 * c["el_mixed"] + 4.0 * B)
    if kernel.startswith("ef::k_server_tiles"):
        return 8.0 * d + (M + 1) * d / 8.0 + 4.0 * B * (M + 1)
    if kernel == "ef::k_apply":
        return 8.125 * d + 4.0 * B
    if kernel == "ef::k_apply_wd":
        return 16.125 * d + 4.0 * B
    if kernel == "ef::k_quality_tiles":                     # one read of every vector
        return 4.0 * d * M
    if kernel in ("ef::k_probe_stream", "ef::k_probe_grouped"):
        return 20.0 * (M * ((d + 3) // 4 * 4) // TILE) * TILE
    return None


def summarize(workload, lazy):
    import ef_workloads as wl
    w = wl.get(workload)
    tag = tag_of(workload, lazy)
    out, cmds = commands(workload, lazy)
    meta = json.load(open(os.path.join(out, "meta.json"))) if os.path.exists(os.path.join(out, "meta.json")) else {}
    c = layout_counts(w)

    def one(pattern):
        hits = glob.glob(os.path.join(out, pattern), recursive=True)
        if not hits:
            sys.exit("no %s under %s: run `collect` on the GPU box first" % (pattern, out))
        return hits[0]

    stats = {}
    for r in csv.DictReader(open(one("kt/**/*kernel_stats.csv"))):
        s = short(r["Name"])
        if s:
            stats[s] = (int(r["Calls"]), float(r["AverageNs"]) * 1e-9, float(r["TotalDurationNs"]) * 1e-9)
    counters = collections.defaultdict(list)
    for which, pattern, col in (("fetch", "fetch/**/*counter_collection.csv", "FETCH_SIZE"),
                                ("write", "write/**/*counter_collection.csv", "WRITE_SIZE")):
        for r in csv.DictReader(open(one(pattern))):
            if r["Counter_Name"] == col:
                s = short(r["Kernel_Name"])
                if s:
                    counters[(which, s)].append(float(r["Counter_Value"]))
    mean = {k: sum(v) / len(v) for k, v in counters.items()}
    cal = "torch add (calibration, 1 GiB -> 1 GiB)"
    f_scale, w_scale = CALIB_KIB / mean[("fetch", cal)], CALIB_KIB / mean[("write", cal)]

    lines = ["# rocprofv3 summary: %s%s%s (d = %d, B = %d, M = %d), MI355X" %
             (workload, ", deferred-correction mode" if lazy else "",
              "" if VARIANT == "sgdm" else ", bench.py --variant " + VARIANT, w.d, w.B, w.M), "",
             "Layout: %d tiles of 4096 elements, %d whole (inside one block), %d mixed.  Measured at commit %s."
             % (c["ntiles"], c["n_whole"], c["n_mixed"], meta.get("commit")),
             "Commands (from /tmp with TMPDIR=/tmp; `python bench_profile.py collect %s%s%s` runs them):" %
             (workload, " --lazy" if lazy else "", "" if VARIANT == "sgdm" else " --variant " + VARIANT), ""]
    lines += ["    " + " ".join(cmd).replace(ROOT, "$R") for cmd in cmds]
    lines += ["", "bench.py here runs 1 warm-up step, the timed steps, one untimed diagnostic worker + server call and, last, the",
              "two bandwidth probes (1 warm-up + 3 timed passes each); `achieved` = algorithmic bytes / average duration.", "",
              "## Kernel trace and HBM roofline", "",
              "| kernel | calls | average ms | algorithmic GB per launch | achieved TB/s | % of 8 TB/s |", "|---|---|---|---|---|---|"]
    for s, (calls, avg, tot) in sorted(stats.items(), key=lambda kv: -kv[1][2]):
        alg = algorithmic(s, w, c)
        if alg is None:
            lines.append("| %s | %d | %.4f | - | - | - |" % (s, calls, avg * 1e3))
        else:
            lines.append("| %s | %d | %.4f | %.4f | %.2f | %.1f |" % (s, calls, avg * 1e3, alg / 1e9, alg / avg / 1e12,
                                                                     100.0 * alg / avg / HBM_PEAK))
    lines += ["", "## HBM traffic counters (KiB per dispatch, averages)", "",
              "Calibration: the torch add kernel reads 2^28 floats (1 048 576 KiB) and writes as many; it shows FETCH_SIZE = %.1f"
              % mean[("fetch", cal)],
              "and WRITE_SIZE = %.1f, so the counters are scaled by %.5f (fetch) and %.5f (write)." %
              (mean[("write", cal)], f_scale, w_scale), "",
              "| kernel | FETCH_SIZE | WRITE_SIZE | read GB | written GB | total GB | algorithmic GB | ratio |", "|---|---|---|---|---|---|---|---|"]
    record = {"workload": workload, "mode": ("deferred" if lazy else "default") + ("" if VARIANT == "sgdm" else "/" + VARIANT),
              "commit": meta.get("commit"), "kernels": {}}
    for s in sorted(stats, key=lambda k: -stats[k][2]):
        if s == cal or ("fetch", s) not in mean or ("write", s) not in mean:
            continue
        rd = mean[("fetch", s)] * f_scale * 1024.0
        wr = mean[("write", s)] * w_scale * 1024.0
        alg = algorithmic(s, w, c)
        ratio = (rd + wr) / alg if alg else None
        lines.append("| %s | %.1f | %.1f | %.4f | %.4f | %.4f | %s | %s |" %
                     (s, mean[("fetch", s)], mean[("write", s)], rd / 1e9, wr / 1e9, (rd + wr) / 1e9,
                      "%.4f" % (alg / 1e9) if alg else "-", "%.3f" % ratio if ratio else "-"))
        record["kernels"][s] = {"traffic_bytes": int(round(rd + wr)), "ratio": round(ratio, 4) if ratio else None}
    lines += ["", "traffic-json: " + json.dumps(record, sort_keys=True), ""]
    path = os.path.join(ROOT, "profiles", "ef_step_%s.md" % tag)
    with open(path, "w") as f:
        f.write("\n".join(lines))
    print("wrote", path)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["collect", "summarize"])
    ap.add_argument("workload")
    ap.add_argument("--lazy", action="store_true", help="the deferred-correction mode (ef_plan_set_lazy)")
    ap.add_argument("--variant", default="sgdm", choices=["sgdm", "sgd", "wd", "quality"], help="bench.py --variant")
    args = ap.parse_args()
    global VARIANT
    VARIANT = args.variant
    (collect if args.what == "collect" else summarize)(args.workload, args.lazy)


if __name__ == "__main__":
    main()
