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

# HBM bytes per launch of a kernel class, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script (scaled by the copy probe: FETCH_SIZE x 2.000, WRITE_SIZE x 1.000), see
# profiles/stream_kernels_layered_3m_fwd_bwd_hbm_traffic.md.  Keyed by (workload, batch, class).
MEASURED_TRAFFIC_PER_LAUNCH = {
    ("layered_3m_fwd_bwd", 256, "bwd_softmax"): 422.9e6,    # 331.7 MB fetched + 91.2 MB written
    ("layered_3m_fwd_bwd", 256, "fwd_lse"): 236.6e6,        # 161.2 MB fetched + 75.4 MB written
}


# HBM bytes of a whole step from the same counter runs (sum over all dispatches of one step), keyed by
# (workload, batch, forward+backward?, alias_chains?)
MEASURED_TRAFFIC_PER_STEP = {
    ("layered_3m_fwd_bwd", 256, True, False): 25.5e9,
}


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
    ap.add_argument("--alias-chains", action="store_true",
                    help="padding-free evaluation: no unary chain nodes, edges read the child's own row")
    ap.add_argument("--f64", action="store_true",
                    help="also time the double-precision kernels on the same workload (extra object \"f64\")")
    ap.add_argument("--cpu-columns", type=int, default=0, help="oracle sample size in batch columns (0: auto)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="first run 5 plain device-to-device copies of this many MiB (calibrates the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters and gives the achievable copy rate)")
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
        copy_probe = {"mib": args.copy_probe_mib, "read_plus_write_GBs": round(2 * n * 4 / dt / 1e9, 1)}
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
    k = pkg.Circuit(*circ.arrays(), device=0, no_tail=args.no_tail, alias_chains=args.alias_chains)
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
            c = classes.setdefault(name, {"ms": 0.0, "launches": 0, "alg_bytes": 0.0})
            for f in c:
                c[f] += rec[f]
    k.set_profiling(False)
    # every class below except "split" is one kernel (one template instance) launched once per layer
    kernel_of = {"fwd_sum": "stream_kernel<OP_SUM>", "fwd_prod": "stream_kernel<OP_PROD>", "fwd_lse": "stream_kernel<OP_LSE>",
                 "fwd_max": "stream_kernel<OP_MAX>",
                 "bwd_sum": "stream_kernel<OP_SUM>", "bwd_softmax": "stream_kernel<OP_SOFTMAX_BWD>",
                 "split": "pass_kernel (segments and combine rows of split rows)", "tail_fwd": "tail_fwd_kernel",
                 "tail_bwd": "tail_bwd_kernel", "leaf": "leaf_fwd_kernel", "bwd_leaf": "leaf_bwd_kernel",
                 "root": "root_out_kernel", "seed": "seed_kernel", "prod_edges": "prod_edge_kernel"}
    dom = max(classes, key=lambda n: classes[n]["ms"])
    d = classes[dom]
    achieved = d["alg_bytes"] / (d["ms"] * 1e-3) / 1e9 if d["ms"] > 0 else 0.0
    kernel_ms_total = sum(c["ms"] for c in classes.values()) / prof_steps
    alg_bytes_step = sum(c["alg_bytes"] for c in classes.values()) / prof_steps
    # compulsory bytes: every row written once and read once per consuming sweep (forward: all rows but
    # the top layer's; backward: adjoint rows written and read once, value rows read once), plus indices
    n_top = k.layer_sizes()[0][-1]
    compulsory = 4.0 * B * (2 * N - n_top) + 4.0 * (E + N)
    if backward:
        compulsory += 4.0 * B * 3 * N + 4.0 * (E + N)
    step_traffic = MEASURED_TRAFFIC_PER_STEP.get((args.workload, B, backward, bool(args.alias_chains)))
    if semiring != pkg.KLAY_LOG or args.no_tail:
        step_traffic = None
    roofline = {
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": MEASURED_TRAFFIC_PER_LAUNCH.get((args.workload, B, dom)),
        "kernel": kernel_of.get(dom, dom) + " [" + dom + "]", "kernel_avg_launch_us": round(d["ms"] * 1e3 / max(1, d["launches"]), 2),
        "kernel_launches_per_step": d["launches"] // prof_steps,
        "kernel_alg_bytes_per_launch": round(d["alg_bytes"] / max(1, d["launches"])),
        "whole_step": {"alg_bytes": round(alg_bytes_step), "kernel_ms": round(kernel_ms_total, 3),
                       "achieved_GBs": round(alg_bytes_step / (ms_per_step * 1e-3) / 1e9, 1),
                       "frac": round(alg_bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "compulsory_bytes": round(compulsory),
                       "compulsory_frac": round(compulsory / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "measured_traffic_bytes": step_traffic,
                       "measured_traffic_frac": None if step_traffic is None else
                       round(step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "per_class_ms": {n: round(c["ms"] / prof_steps, 3) for n, c in classes.items() if c["launches"]},
        # no-reuse GB/s of every class (its algorithmic bytes over its summed launch durations)
        "per_class_GBs": {n: round(c["alg_bytes"] / (c["ms"] * 1e-3) / 1e9) for n, c in classes.items()
                          if c["launches"] and c["ms"] > 0},
    }

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import oracle
        threads = min(oracle.max_threads(), 16)
        # a bounded sample: about 1.3e9 edge evaluations, 10-20 s for the oracle on 16 threads
        cols = args.cpu_columns or max(threads, int(1.3e9 / max(1, E)) // threads * threads)
        cols = min(cols, B)
        sample = np.ascontiguousarray(w32[:cols]).astype(np.float64)
        oracle_semiring = {pkg.KLAY_LOG: oracle.LOG, pkg.KLAY_REAL: oracle.REAL, pkg.KLAY_MAXLOG: oracle.MAXLOG}[semiring]
        t0 = time.perf_counter()
        ref = oracle.forward(*circ.arrays(), sample, oracle_semiring,
                             nthreads=threads)
        if backward:
            rgrad = oracle.backward(*circ.arrays(), sample, oracle_semiring,
                                    np.ones_like(ref), nthreads=threads)
        t_cpu = time.perf_counter() - t0
        got = out[:cols].cpu().numpy()
        err = float(np.abs(got - ref).max())
        cpu_baseline = {
            "value": cols * E / t_cpu, "unit": "edge-evals/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d batch columns of the same workload, %s, fp64 post-order over the unlayered DAG "
                      "(%d nodes, %d edges); counted in layered edges like the GPU figure; %.1f s" % (
                          cols, B, "forward+backward" if backward else "forward", info["dag_nodes"],
                          info["dag_edges"], t_cpu),
            "max_abs_err_vs_gpu": err,
        }
        if backward:
            gerr = np.abs(dleaf[:cols].cpu().numpy() - rgrad) / np.maximum(1.0, np.abs(rgrad))
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
                   "layerization": "alias_chains (no unary chain nodes)" if args.alias_chains else
                                   "unary chain nodes per (node, layer)",
                   "layers": info["num_layers"], "layered_nodes": N, "layered_edges": E,
                   "dag_nodes": info["dag_nodes"], "dag_edges": info["dag_edges"],
                   "pad_nodes": info["num_pad_nodes"], "num_vars": info["num_vars"], "num_roots": info["num_roots"],
                   "max_fan_in": info["max_fan_in"], "max_fan_out": info["max_fan_out"],
                   "build_seconds": round(t_build, 2), "generate_seconds": round(t_gen, 2)},
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
