#!/usr/bin/env python3
"""Regenerates bench_traffic.json (the measured HBM bytes that bench.py reports its roofline on) and the
rocprofv3 summaries under profiles/ from rocprofv3 runs of bench.py.

Two steps, both run from the repository root:

  on the MI355X machine (writes raw rocprofv3 output under gpurun_out/traffic/<tag>/):
      cd /tmp && export TMPDIR=/tmp && python3 $GRAFT_REPO_ROOT/bench_traffic.py collect [tag ...]
  afterwards, anywhere (reads gpurun_out/traffic/, writes bench_traffic.json and profiles/*.md):
      python3 bench_traffic.py fold

`collect` starts, per workload, one plain run of bench.py, one `rocprofv3 --kernel-trace --stats` run and
two `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE: counters in runs of their own, nothing else
traced with them).  It never touches the GPU itself; every run is a child process under a time limit,
and the first failure ends the collection.

`fold` scales each counter by what it reads for bench.py's copy probe (device-to-device copies of a
known size in the same run), averages per kernel symbol and per step, and stamps the table with the
fingerprint of the sources it was measured on (bench.source_fingerprint); bench.py ignores a table
whose fingerprint differs from the sources it runs.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(ROOT, "gpurun_out", "traffic")
PROBE_MIB = 1024

# tag -> extra bench.py arguments (the workload's own batch, semiring and pass unless overridden)
RUNS = collections.OrderedDict([
    ("layered_3m_fwd_bwd", []),
    ("layered_3m_fwd_bwd_chains", ["--unary-chains"]),
    ("layered_1m_log", ["--workload", "layered_1m"]),
    ("layered_1m_real", ["--workload", "layered_1m", "--semiring", "real"]),
    ("layered_1m_real_fwd_bwd", ["--workload", "layered_1m", "--semiring", "real", "--backward", "on"]),
    ("layered_1m_b1", ["--workload", "layered_1m", "--batch", "1"]),
    ("powerlaw_10m", ["--workload", "powerlaw_10m"]),
    ("powerlaw_1m_nodes", ["--workload", "powerlaw_1m_nodes"]),
    ("layered_100k", ["--workload", "layered_100k"]),
    ("tiny_ddnnf", ["--workload", "tiny_ddnnf"]),
])
KT_STEPS = ["--steps", "10", "--warmup", "3"]
PMC_STEPS = ["--steps", "2", "--warmup", "1"]


def run(cmd, log, limit):
    print("[bench_traffic] " + " ".join(cmd), flush=True)
    t0 = time.time()
    with open(log, "w") as fh:
        rc = subprocess.call(["timeout", "-s", "KILL", str(limit)] + cmd, stdout=fh, stderr=subprocess.STDOUT)
    print("[bench_traffic]   rc=%d in %.0f s" % (rc, time.time() - t0), flush=True)
    if rc != 0:
        sys.exit("bench_traffic: %s failed (see %s)" % (cmd[0], log))


def collect(tags):
    bench = os.path.join(ROOT, "bench.py")
    for tag in tags:
        d = os.path.join(OUT, tag)
        os.makedirs(d, exist_ok=True)
        extra = RUNS[tag] + ["--no-cpu-baseline", "--copy-probe-mib", str(PROBE_MIB)]
        run(["python3", bench] + KT_STEPS + extra, os.path.join(d, "plain.log"), 300)
        run(["rocprofv3", "--kernel-trace", "--stats", "--output-format", "csv", "-d", os.path.join(d, "kt"), "-o", "kt",
             "--", "python3", bench] + KT_STEPS + extra, os.path.join(d, "kt.log"), 300)
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            sub = counter.split("_")[0].lower()
            run(["rocprofv3", "--pmc", counter, "--output-format", "csv", "-d", os.path.join(d, sub), "-o", sub,
                 "--", "python3", bench] + PMC_STEPS + extra, os.path.join(d, sub + ".log"), 300)


def symbol(name):
    m = re.search(r"klay::(?:f64::)?\w+(?:<[^>]*>)?", name)
    if m:
        return m.group(0)
    if "copyBuffer" in name:
        return "copy_probe"
    return None


def bench_line(log):
    for line in open(log):
        if line.startswith("{"):
            return json.loads(line)
    raise SystemExit("no bench line in " + log)


def counter_means(path, counter):
    per = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        s = symbol(r["Kernel_Name"])
        if s:
            per[s].append(float(r["Counter_Value"]))
    return per


def fold():
    sys.path.insert(0, ROOT)
    from bench import source_fingerprint
    # the fingerprint that bench.py printed in the measured runs; all runs of a table must share it
    table = {"fingerprint": None, "peak_GBs": 8000.0, "probe_mib": PROBE_MIB, "runs": {}}
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    for tag in RUNS:
        d = os.path.join(OUT, tag)
        if not os.path.exists(os.path.join(d, "write", "write_counter_collection.csv")):
            print("fold: no data for", tag)
            continue
        plain, traced = bench_line(os.path.join(d, "plain.log")), bench_line(os.path.join(d, "kt.log"))
        cfg = plain["config"]
        if table["fingerprint"] is None:
            table["fingerprint"] = cfg["sources_fingerprint"]
        if cfg["sources_fingerprint"] != table["fingerprint"] or traced["config"]["sources_fingerprint"] != table["fingerprint"]:
            print("fold: %s was measured on other sources (%s), left out" % (tag, cfg["sources_fingerprint"]))
            continue
        backward = cfg["pass"] == "forward+backward"
        chains = cfg["layerization"].startswith("unary")
        key = "%s|B=%d|%s|%s|%s" % (cfg["workload"], cfg["batch"], cfg["semiring"], "fwd+bwd" if backward else "fwd",
                                    "chains" if chains else "default")
        # kernel trace
        stats = {}
        for r in csv.DictReader(open(os.path.join(d, "kt", "kt_kernel_stats.csv"))):
            s = symbol(r["Name"])
            if s and s != "copy_probe":
                stats[s] = (int(r["Calls"]), float(r["TotalDurationNs"]), float(r["AverageNs"]))
        kt_steps = 10 + 3 + min(10, 5)
        total_ns = sum(v[1] for v in stats.values())
        # counters, scaled by the copy probe of the same run
        fetch = counter_means(os.path.join(d, "fetch", "fetch_counter_collection.csv"), "FETCH_SIZE")
        write = counter_means(os.path.join(d, "write", "write_counter_collection.csv"), "WRITE_SIZE")
        probe_kib = PROBE_MIB * 1024.0
        scale_f = probe_kib / (sum(fetch["copy_probe"]) / len(fetch["copy_probe"]))
        scale_w = probe_kib / (sum(write["copy_probe"]) / len(write["copy_probe"]))
        pmc_steps = 2 + 1 + 2
        per_kernel, step_bytes = {}, 0.0
        for s in sorted(set(fetch) | set(write)):
            if s == "copy_probe":
                continue
            fv, wv = fetch.get(s, []), write.get(s, [])
            fb = sum(fv) / max(1, len(fv)) * scale_f * 1024.0
            wb = sum(wv) / max(1, len(wv)) * scale_w * 1024.0
            n = max(len(fv), len(wv)) / pmc_steps
            per_kernel[s] = {"fetch_bytes": round(fb), "write_bytes": round(wb), "launches_per_step": round(n, 2),
                             "avg_us_rocprof": round(stats[s][2] / 1e3, 2) if s in stats else None}
            step_bytes += (fb + wb) * n
        table["runs"][key] = {"tag": tag, "ms_per_step": round(plain["ms_per_step"], 4), "step_bytes": round(step_bytes),
                              "fetch_scale": round(scale_f, 4), "write_scale": round(scale_w, 4), "per_kernel": per_kernel}
        # summary
        ms = plain["ms_per_step"]
        roof = plain["roofline"]
        dom = max(stats, key=lambda s: stats[s][1])
        args = " ".join(RUNS[tag] + ["--no-cpu-baseline", "--copy-probe-mib", str(PROBE_MIB)])
        out = ["# rocprofv3 summary: bench.py %s" % " ".join(RUNS[tag]) if RUNS[tag] else "# rocprofv3 summary: bench.py (headline workload)",
               "",
               "Workload %s, B = %d, %s semiring, %s, %s; layered circuit %d nodes / %d edges in %d layers." % (
                   cfg["workload"], cfg["batch"], cfg["semiring"], cfg["pass"], cfg["layerization"], cfg["layered_nodes"],
                   cfg["layered_edges"], cfg["layers"]),
               "Sources fingerprint %s.  Written by `python3 bench_traffic.py fold` from the raw output of" % table["fingerprint"],
               "`cd /tmp && export TMPDIR=/tmp && python3 $GRAFT_REPO_ROOT/bench_traffic.py collect %s`, which ran:" % tag,
               "",
               "    python3 bench.py %s %s" % (" ".join(KT_STEPS), args),
               "    rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/traffic/%s/kt -o kt -- python3 bench.py %s %s" % (tag, " ".join(KT_STEPS), args),
               "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/traffic/%s/fetch -o fetch -- python3 bench.py %s %s" % (tag, " ".join(PMC_STEPS), args),
               "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/traffic/%s/write -o write -- python3 bench.py %s %s" % (tag, " ".join(PMC_STEPS), args),
               "",
               "Untraced: %.4f ms per step = %.3e edge-evals/s; under the kernel tracer %.4f ms per step." % (
                   ms, plain["value"], traced["ms_per_step"]),
               "Copy probe (%d MiB device-to-device, `__amd_rocclr_copyBuffer`): %.0f GB/s read + write; it calibrates the counters:" % (
                   PROBE_MIB, plain["copy_probe"]["read_plus_write_GBs"]),
               "FETCH_SIZE x %.3f and WRITE_SIZE x %.3f give KiB." % (scale_f, scale_w),
               "",
               "## Kernel trace (%d steps traced: 3 warm-up + 10 timed + 5 with per-launch HIP events)" % kt_steps,
               "",
               "| kernel | calls/step | avg us | ms/step | % of kernel time |", "|---|---|---|---|---|"]
        for s in sorted(stats, key=lambda s: -stats[s][1]):
            c, t, a = stats[s]
            out.append("| %s | %.1f | %.2f | %.4f | %.1f |" % (s.replace("klay::", ""), c / kt_steps, a / 1e3, t / 1e6 / kt_steps, 100 * t / total_ns))
        out += ["", "Sum of kernel time: %.4f ms per step." % (total_ns / 1e6 / kt_steps), "",
                "## HBM traffic (FETCH_SIZE / WRITE_SIZE, %d steps per run)" % pmc_steps, "",
                "| kernel | launches/step | fetch MB/launch | write MB/launch | traffic GB/step | GB/s at the traced avg | of 8 TB/s |",
                "|---|---|---|---|---|---|---|"]
        for s in sorted(per_kernel, key=lambda s: -(per_kernel[s]["fetch_bytes"] + per_kernel[s]["write_bytes"]) * per_kernel[s]["launches_per_step"]):
            k = per_kernel[s]
            tb = k["fetch_bytes"] + k["write_bytes"]
            rate = tb / (k["avg_us_rocprof"] * 1e-6) / 1e9 if k["avg_us_rocprof"] else float("nan")
            out.append("| %s | %.1f | %.2f | %.2f | %.4f | %.0f | %.3f |" % (
                s.replace("klay::", ""), k["launches_per_step"], k["fetch_bytes"] / 1e6, k["write_bytes"] / 1e6,
                tb * k["launches_per_step"] / 1e9, rate, rate / 8000.0))
        ws = roof["whole_step"]
        out += ["",
                "Whole step: %.3f GB of HBM traffic in %.4f ms = %.0f GB/s = %.3f of the 8 TB/s peak; the compulsory bytes" % (
                    step_bytes / 1e9, ms, step_bytes / ms / 1e6, step_bytes / ms / 1e6 / 8000.0),
                "(every distinct row once per pass) are %.3f GB (%.3f of peak over the same time), the no-reuse model" % (
                    ws["compulsory_bytes"] / 1e9, ws["compulsory_frac"]),
                "(every index entry fetches its row from memory) %.3f GB (%.3f: a model, it counts L2 hits as traffic)." % (
                    ws["no_reuse_model_bytes"] / 1e9, ws["model_no_reuse_frac"]),
                "Dominant kernel by time: %s, %.2f us average under the tracer; bench.py's HIP events give %s %.2f us." % (
                    dom.replace("klay::", ""), stats[dom][2] / 1e3, roof["kernel"].replace("klay::", ""), roof["kernel_avg_launch_us"]),
                ""]
        # named for the kernel that dominates the run and for the workload
        dom_name = re.sub(r"<.*", "", dom.replace("klay::", ""))
        name = "%s_%s_b%d_%s_%s%s.md" % (dom_name, cfg["workload"], cfg["batch"], cfg["semiring"],
                                         "fwd_bwd" if backward else "fwd", "_chains" if chains else "")
        with open(os.path.join(ROOT, "profiles", name), "w") as fh:
            fh.write("\n".join(out))
        print("fold:", key, "->", "profiles/" + name, "step %.3f GB" % (step_bytes / 1e9))
    if table["fingerprint"] != source_fingerprint():
        print("fold: WARNING the runs were measured on sources %s, the tree is now %s: bench.py will ignore the table" % (
            table["fingerprint"], source_fingerprint()))
    with open(os.path.join(ROOT, "bench_traffic.json"), "w") as fh:
        json.dump(table, fh, indent=1, sort_keys=True)
        fh.write("\n")


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "collect":
        tags = sys.argv[2:] or list(RUNS)
        for t in tags:
            if t not in RUNS:
                sys.exit("unknown tag %s (known: %s)" % (t, ", ".join(RUNS)))
        collect(tags)
    elif len(sys.argv) == 2 and sys.argv[1] == "fold":
        fold()
    else:
        sys.exit(__doc__)
