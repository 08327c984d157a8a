#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: forward + backward of the layered circuit evaluator
on the headline workload (3e6-node, 1e7-edge random layered circuit, depth 60, V=8192, B=256,
fp32 log semiring), reported as edge-evaluations per second with the roofline of the dominant
kernel and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Prints ONE JSON line.  A "step" is one klay_forward + klay_backward over one batch that is already
resident in device memory; klay_build (host layerization + upload) is outside the timed region.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
TRAFFIC_TABLE = os.path.join(ROOT, "bench_traffic.json")
FINGERPRINT_FILES = ("paper_2410_11415_amd/csrc/klay_api.hip", "paper_2410_11415_amd/csrc/klay_kernels.hip.h",
                     "paper_2410_11415_amd/csrc/layerize.cpp", "paper_2410_11415_amd/csrc/layerize.h",
                     "klay_synth/circuits.py", "klay_synth/configs.py", "klay_synth/weights.py")


def source_fingerprint() -> str:
    """Hash of the sources that decide what the kernels move (kernels, launch plans, node order, input
    generators).  The measured-traffic table carries the fingerprint it was measured at; figures from a
    table with another fingerprint are reported as null."""
    import hashlib
    h = hashlib.sha256()
    for f in FINGERPRINT_FILES:
        with open(os.path.join(ROOT, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def load_traffic(workload, batch, semiring, backward, chains):
    """HBM bytes per dispatch and per step from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs that
    bench_traffic.py folded into bench_traffic.json; None unless measured on these very sources."""
    try:
        with open(TRAFFIC_TABLE) as fh:
            table = json.load(fh)
    except (OSError, ValueError):
        return None
    if table.get("fingerprint") != source_fingerprint():
        return None
    key = "%s|B=%d|%s|%s|%s" % (workload, batch, semiring, "fwd+bwd" if backward else "fwd", "chains" if chains else "default")
    return table.get("runs", {}).get(key)


def kernel_symbol(cls, B, edges=False, fused_op=10):
    """rocprofv3's name for the kernel behind a profiling class (template arguments as it prints them)."""
    vec = 4 if B > 128 else (2 if B > 64 else 1)
    ops = {"fwd_sum": 0, "bwd_sum": 0, "fwd_prod": 1, "fwd_lse": 2, "bwd_softmax": 3, "fwd_max": 4, "bwd_prod": 5,
           "bwd_sum_enc": 6, "bwd_softmax_one": 7, "bwd_sum_mul": 8, "bwd_prod_mul": 9}
    if cls in ops:
        if B > 32:
            return "klay::stream_kernel<%d, %d>" % (ops[cls], vec)
        w = 1
        while w < B:
            w *= 2
        return ("klay::edge_kernel<%d, %d>" if edges else "klay::pass_kernel<%d, 1, %d>") % (ops[cls], w)
    w_small = 1
    while w_small < B:
        w_small *= 2
    ct = 1
    while ct < 8 and (B + ct - 1) // ct > 256:
        ct *= 2
    fixed = {"tail_fwd": "klay::slab_fwd_kernel<%d>" % ct, "tail_bwd": "klay::slab_bwd_kernel<%d>" % ct,
             "leaf": "klay::leaf_fwd_kernel" if B > 32 else "klay::leaf_fwd_small_kernel", "bwd_leaf": "klay::leaf_bwd_kernel", "root": "klay::root_out_kernel",
             "seed": "klay::seed_kernel", "split": "klay::pass_kernel<*> (segments of split rows)",
             "combine": "klay::combine_kernel<*>" if B > 32 else "klay::pass_kernel<*> (combine rows of split rows)",
             "main_combine": "klay::stream_combine_kernel<*>",
             "fwd_or_fused": "klay::stream_kernel<%d, %d>" % (fused_op, vec),
             "prod_edges": "klay::prod_parent_kernel<%d, %d>" % (vec, 64 if B > 32 else w_small)}
    return fixed.get(cls, cls)


class HipEvents:
    """hipEvent timing on an explicit stream, straight from the HIP runtime."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        e = ctypes.c_void_p()
        assert self.hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.hip.hipEventRecord(e, ctypes.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        assert self.hip.hipEventSynchronize(b) == 0
        ms = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return float(ms.value)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="layered_3m_fwd_bwd")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--semiring", choices=("log", "real", "maxlog"), default=None,
                    help="default: log where the workload lists it; maxlog = (max, +), forward only")
    ap.add_argument("--backward", choices=("on", "off"), default=None, help="default: as the workload specifies")
    ap.add_argument("--no-tail", action="store_true", help="one launch per layer also for the narrow top layers")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph (torch.cuda.graph) and time its replays")
    ap.add_argument("--unary-chains", action="store_true",
                    help="the paper's layerization throughout (one unary chain node per node and layer an edge skips) "
                         "instead of the default, which is padding-free below the narrow top of the circuit")
    ap.add_argument("--no-fusion", action="store_true",
                    help="every forward pass writes the value of every AND node (for comparison; by default a forward "
                         "pass that no backward pass follows leaves out the AND rows that the OR rows above can "
                         "evaluate themselves)")
    ap.add_argument("--small-batch-edges", action="store_true",
                    help="B <= 32: the lanes = edges kernel instead of a lane group per row (for comparison)")
    ap.add_argument("--f64", action="store_true",
                    help="also time the double-precision kernels on the same workload (extra object \"f64\")")
    ap.add_argument("--cpu-columns", type=int, default=0, help="oracle sample size in batch columns (0: auto)")
    ap.add_argument("--copy-probe-mib", type=int, default=1024,
                    help="first run 5 plain device-to-device copies of this many MiB: the achievable copy rate of "
                         "this box, and the dispatches that calibrate the rocprofv3 FETCH_SIZE / WRITE_SIZE counters "
                         "(0: skip)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (batch columns are independent, so more GPUs "
              "would each take a slice of the batch with no exchange); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2410_11415_amd as pkg
    from klay_synth import as_inputs, make_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    pkg.load()                                    # no fallback: fails if the HIP library is missing
    torch.cuda.set_device(0)

    copy_probe = None
    if args.copy_probe_mib > 0:
        n = args.copy_probe_mib * (1 << 20) // 4
        a = torch.empty(n, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 5
        copy_probe = {"mib": args.copy_probe_mib, "read_plus_write_GBs": round(2 * n * 4 / dt / 1e9, 1),
                      "what": "device-to-device copy, bytes read + bytes written over wall time"}
        del a, b
        torch.cuda.empty_cache()

    t0 = time.perf_counter()
    circ, p, spec = make_config(args.workload, seed=args.seed, batch=args.batch)
    t_gen = time.perf_counter() - t0
    B = p.shape[0]
    backward = bool(spec["backward"]) if args.backward is None else args.backward == "on"
    if args.semiring is not None:
        semiring = {"log": pkg.KLAY_LOG, "real": pkg.KLAY_REAL, "maxlog": pkg.KLAY_MAXLOG}[args.semiring]
    else:
        semiring = pkg.KLAY_LOG if "log" in spec["semirings"] else pkg.KLAY_REAL
    if semiring == pkg.KLAY_MAXLOG:
        backward = False
    semiring_name = {pkg.KLAY_LOG: "log", pkg.KLAY_REAL: "real", pkg.KLAY_MAXLOG: "maxlog"}[semiring]
    w32 = as_inputs(p, semiring != pkg.KLAY_REAL)

    t0 = time.perf_counter()
    k = pkg.Circuit(*circ.arrays(), device=0, no_tail=args.no_tail, unary_chains=args.unary_chains,
                    small_batch_edges=args.small_batch_edges, no_fusion=args.no_fusion)
    t_build = time.perf_counter() - t0
    info = k.info()
    E, N = info["num_edges"], info["num_nodes"]

    stream = torch.cuda.current_stream()
    w = torch.from_numpy(w32).cuda()
    out = torch.empty((B, k.num_roots), dtype=torch.float32, device="cuda")
    dout = torch.ones((B, k.num_roots), dtype=torch.float32, device="cuda")
    dleaf = torch.empty((B, k.num_vars), dtype=torch.float32, device="cuda")

    def step():
        k.forward(w, semiring, out=out, stream=stream)
        if backward:
            k.backward(dout, dleaf=dleaf, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    eager_step = step
    if args.graph:
        # the library only enqueues kernels on the given stream (no allocation once the workspace
        # exists, no host synchronisation), so a whole step can be captured and replayed
        side = torch.cuda.Stream()
        stream = side
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            eager_step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                eager_step()
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()

        def step():
            graph.replay()
        for _ in range(3):
            step()
        torch.cuda.synchronize()

    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev.record(e0, stream.cuda_stream)
    for _ in range(args.steps):
        step()
    ev.record(e1, stream.cuda_stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_events = ev.elapsed_ms(e0, e1)
    ms_per_step = wall * 1e3 / args.steps
    value = B * E * args.steps / wall

    # per-kernel-class durations: the same steps again with HIP events around every launch group
    step = eager_step
    k.set_profiling(True)
    classes = {}
    prof_steps = max(1, min(args.steps, 5))
    t0 = time.perf_counter()
    for _ in range(prof_steps):
        step()
        torch.cuda.synchronize()
        for name, rec in k.get_profile().items():
            c = classes.setdefault(name, {"ms": 0.0, "launches": 0, "alg_bytes": 0.0, "min_bytes": 0.0})
            for f in c:
                c[f] += rec[f]
    k.set_profiling(False)
    # ---- roofline: the kernel that takes most time, by symbol (a symbol can serve several classes:
    # the log-domain AND layers forward and backward are both stream_kernel<OP_SUM>)
    by_symbol = {}
    for name, c in classes.items():
        if not c["launches"]:
            continue
        g = by_symbol.setdefault(kernel_symbol(name, B, args.small_batch_edges, {pkg.KLAY_LOG: 10, pkg.KLAY_MAXLOG: 11, pkg.KLAY_REAL: 12}[semiring]), {"ms": 0.0, "launches": 0, "alg_bytes": 0.0, "min_bytes": 0.0,
                                                          "classes": []})
        for f in ("ms", "launches", "alg_bytes", "min_bytes"):
            g[f] += c[f]
        g["classes"].append(name)
    dom = max(by_symbol, key=lambda n: by_symbol[n]["ms"])
    d = by_symbol[dom]
    kernel_ms_total = sum(c["ms"] for c in classes.values()) / prof_steps
    alg_bytes_step = sum(c["alg_bytes"] for c in classes.values()) / prof_steps
    min_bytes_step = sum(c["min_bytes"] for c in classes.values()) / prof_steps
    measured = None
    if not args.no_tail and not args.graph and not args.small_batch_edges and not args.no_fusion:
        measured = load_traffic(args.workload, B, semiring_name, backward, bool(args.unary_chains))
    per_launch_s = d["ms"] * 1e-3 / max(1, d["launches"])
    traffic = None
    if measured and dom in measured["per_kernel"]:
        traffic = measured["per_kernel"][dom]["fetch_bytes"] + measured["per_kernel"][dom]["write_bytes"]
    no_reuse_GBs = d["alg_bytes"] / max(1, d["launches"]) / per_launch_s / 1e9 if per_launch_s > 0 else 0.0
    compulsory_GBs = d["min_bytes"] / max(1, d["launches"]) / per_launch_s / 1e9 if per_launch_s > 0 else 0.0
    if traffic is not None:
        achieved, basis = traffic / per_launch_s / 1e9, \
            "HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (bench_traffic.json) over the HIP-event launch time"
    else:
        achieved, basis = compulsory_GBs, \
            "compulsory bytes per launch (no counter figures for these sources: lower bound on the traffic)"
    step_s = ms_per_step * 1e-3
    step_traffic = measured["step_bytes"] if measured else None

    def per_kernel_entry(sym, g):
        t = g["ms"] * 1e-3
        e = {"classes": g["classes"], "ms_per_step": round(g["ms"] / prof_steps, 4), "launches_per_step": g["launches"] // prof_steps,
             "no_reuse_model_GBs": round(g["alg_bytes"] / t / 1e9) if t > 0 else None,
             "compulsory_GBs": round(g["min_bytes"] / t / 1e9) if t > 0 else None, "traffic_GBs": None}
        if measured and sym in measured["per_kernel"] and t > 0:
            m = measured["per_kernel"][sym]
            e["traffic_GBs"] = round((m["fetch_bytes"] + m["write_bytes"]) * g["launches"] / t / 1e9)
        if e["no_reuse_model_GBs"] and e["no_reuse_model_GBs"] > HBM_PEAK_GBS:
            e["note"] = "the no-reuse model counts L2 hits as memory reads: above the HBM peak, so not a traffic figure"
        return e

    roofline = {
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "basis": basis,
        "kernel": dom, "kernel_classes": d["classes"],
        "kernel_avg_launch_us": round(per_launch_s * 1e6, 2),
        "kernel_launches_per_step": d["launches"] // prof_steps,
        "kernel_share_of_kernel_time": round(d["ms"] / prof_steps / kernel_ms_total, 3) if kernel_ms_total > 0 else None,
        "kernel_no_reuse_bytes_per_launch": round(d["alg_bytes"] / max(1, d["launches"])),
        "kernel_compulsory_bytes_per_launch": round(d["min_bytes"] / max(1, d["launches"])),
        "model_no_reuse_frac": round(no_reuse_GBs / HBM_PEAK_GBS, 4),
        "compulsory_frac": round(compulsory_GBs / HBM_PEAK_GBS, 4),
        "achievable_GBs": copy_probe["read_plus_write_GBs"] if copy_probe else None,
        "traffic_table": None if measured is None else {"fingerprint": source_fingerprint(), "measured_ms_per_step": measured.get("ms_per_step")},
        "whole_step": {"kernel_ms": round(kernel_ms_total, 3),
                       "traffic_bytes": step_traffic,
                       "traffic_frac": None if step_traffic is None else round(step_traffic / step_s / 1e9 / HBM_PEAK_GBS, 4),
                       "no_reuse_model_bytes": round(alg_bytes_step),
                       "model_no_reuse_frac": round(alg_bytes_step / step_s / 1e9 / HBM_PEAK_GBS, 4),
                       "compulsory_bytes": round(min_bytes_step),
                       "compulsory_frac": round(min_bytes_step / step_s / 1e9 / HBM_PEAK_GBS, 4)},
        "per_kernel": {sym: per_kernel_entry(sym, g) for sym, g in sorted(by_symbol.items(), key=lambda kv: -kv[1]["ms"])},
    }

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        host = {"os_cpu_count": os.cpu_count(), "affinity": len(os.sched_getaffinity(0)), "omp_max_threads": oracle.max_threads()}
        threads = max(1, min(host["omp_max_threads"], host["affinity"], 16))
        # a bounded sample: about 1.3e9 edge evaluations, 10-20 s for the oracle on 16 threads
        cols = args.cpu_columns or max(threads, int(1.3e9 / max(1, E)) // threads * threads)
        cols = min(cols, B)
        sample = np.ascontiguousarray(w32[:cols]).astype(np.float64)
        oracle_semiring = {pkg.KLAY_LOG: oracle.LOG, pkg.KLAY_REAL: oracle.REAL, pkg.KLAY_MAXLOG: oracle.MAXLOG}[semiring]
        arrays = circ.arrays()
        ones = np.ones((cols, k.num_roots))

        def oracle_pass(x, nthreads):
            # one evaluation of the workload: forward, or forward + reverse sweep (the oracle's backward
            # evaluates the column forward itself before it sweeps back)
            t0 = time.perf_counter()
            if backward:
                r = oracle.backward(*arrays, x, oracle_semiring, ones[:x.shape[0]], nthreads=nthreads)
            else:
                r = oracle.forward(*arrays, x, oracle_semiring, nthreads=nthreads)
            return r, time.perf_counter() - t0
        # the oracle sorts the DAG (post-order) inside every call; like klay_build on the GPU side the sort is
        # not part of an evaluation, so it is timed by itself and taken out
        t0 = time.perf_counter()
        oracle.postorder(*arrays[1:])
        t_sort = time.perf_counter() - t0
        res, t_all = oracle_pass(sample, threads)
        cols1 = max(1, cols // 16)
        _, t_one = oracle_pass(sample[:cols1], 1)
        t_all_eval, t_one_eval = max(t_all - t_sort, 1e-9), max(t_one - t_sort, 1e-9)
        ref = oracle.forward(*arrays, sample, oracle_semiring, nthreads=threads) if backward else res
        got = out[:cols].cpu().numpy()
        err = float(np.abs(got - ref).max())
        cpu_baseline = {
            "value": cols * E / t_all_eval, "unit": "edge-evals/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d batch columns of the same workload, %s, fp64 post-order over the unlayered DAG "
                      "(%d nodes, %d edges); counted in layered edges like the GPU figure; %.1f s of evaluation "
                      "(+ %.2f s for the oracle's own topological sort, excluded like klay_build)" % (
                          cols, B, "forward+backward" if backward else "forward", info["dag_nodes"],
                          info["dag_edges"], t_all_eval, t_sort),
            "single_thread": {"value": cols1 * E / t_one_eval, "columns": cols1, "seconds": round(t_one_eval, 2)},
            "host": host,
            "max_abs_err_vs_gpu": err,
        }
        if backward:
            gerr = np.abs(dleaf[:cols].cpu().numpy() - res) / np.maximum(1.0, np.abs(res))
            cpu_baseline["max_grad_err_vs_gpu"] = float(gerr.max())
        cpu_baseline["max_abs_log_ref"] = float(np.abs(ref[np.isfinite(ref)]).max())

    result = {
        "metric": "edge-evals/sec (batch x edges/s) fwd+bwd at B=256; % of HBM roofline"
                  if backward else "edge-evals/sec (batch x edges/s) forward",
        "value": value, "unit": "edge-evals/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_hip_events": ms_events / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "semiring": semiring_name,
                   "pass": "forward+backward" if backward else "forward", "seed": args.seed,
                   "launch": "hip graph replay" if args.graph else "eager",
                   "layerization": "unary chain nodes per (node, layer) throughout" if args.unary_chains else
                                   "padding-free up to layer %d of %d, unary chain nodes above" % (
                                       info["alias_top_layer"], info["num_layers"]),
                   "padding_free_layers": info["alias_top_layer"],
                   "fused_and_rows": 0 if (args.no_fusion or backward or B <= 64) else info["num_fused_rows"],
                   "layers": info["num_layers"], "layered_nodes": N, "layered_edges": E,
                   "dag_nodes": info["dag_nodes"], "dag_edges": info["dag_edges"],
                   "pad_nodes": info["num_pad_nodes"], "num_vars": info["num_vars"], "num_roots": info["num_roots"],
                   "max_fan_in": info["max_fan_in"], "max_fan_out": info["max_fan_out"],
                   "build_seconds": round(t_build, 2), "generate_seconds": round(t_gen, 2),
                   "sources_fingerprint": source_fingerprint()},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }
    if args.f64:
        # the double-precision accuracy build: same launch plans, 8-byte values (not profiled per class)
        w64 = w.double()
        d64 = torch.ones((B, k.num_roots), dtype=torch.float64, device="cuda")
        bwd64 = backward and semiring == pkg.KLAY_LOG

        def step64():
            o = k.forward_f64(w64, semiring)
            if bwd64:
                k.backward_f64(d64)
            return o
        for _ in range(2):
            o64 = step64()
        torch.cuda.synchronize()
        n64 = max(2, args.steps // 4)
        t0 = time.perf_counter()
        for _ in range(n64):
            step64()
        torch.cuda.synchronize()
        t64 = (time.perf_counter() - t0) / n64
        fwd_share = 1.0 if (bwd64 or not backward) else None
        result["f64"] = {"ms_per_step": t64 * 1e3, "value": B * E / t64, "pass": "forward+backward" if bwd64 else "forward",
                         "max_abs_diff_fp32_vs_f64": float((out.double() - o64).abs().nan_to_num(0.0).max()),
                         "achieved_GBs": None if fwd_share is None else round(2 * alg_bytes_step / t64 / 1e9, 1),
                         "frac": None if fwd_share is None else round(2 * alg_bytes_step / t64 / 1e9 / HBM_PEAK_GBS, 4)}
    if copy_probe:
        result["copy_probe"] = copy_probe
    print(json.dumps(result))


if __name__ == "__main__":
    main()
