"""The five benchmark / parity workloads, as concrete seeded generator calls.

Each entry fixes everything about the input: circuit generator and its parameters, leaf
weight distribution, batch size, semiring(s) and whether the backward pass is part of it.
`scale` < 1 shrinks node counts (and nothing else) so that the CPU oracle finishes in
seconds for element-by-element parity; scale = 1 is the full-size workload.
"""
from __future__ import annotations

from .circuits import layered_random, tiny_ddnnf
from .weights import leaf_probs

CONFIGS = {
    # tiny d-DNNF from a random 3-CNF, checked against brute-force model counting
    "tiny_ddnnf": dict(kind="tiny", num_vars=12, num_clauses=30, batch=4, semirings=("log",),
                       backward=False, weights=("uniform", 0.05, 0.95)),
    # 1e5 nodes, depth 20
    "layered_100k": dict(kind="layered", num_vars=256, depth=20, num_nodes=100_000,
                         fanin=("geom", 2.0), groups=2, batch=128, semirings=("log",),
                         backward=False, weights=("uniform", 0.0, 1.0)),
    # 1e6 nodes, depth 40, B=1 (latency) and B=256, both semirings
    "layered_1m": dict(kind="layered", num_vars=1024, depth=40, num_nodes=1_000_000,
                       fanin=("geom", 2.0), groups=4, batch=256, semirings=("real", "log"),
                       backward=False, weights=("uniform", 0.0, 1.0)),
    # power-law fan-in: edges bind (1e7 edges), node count follows from the Zipf mean
    "powerlaw_10m": dict(kind="layered", num_vars=4096, depth=30, num_nodes=290_000,
                         fanin=("zipf", 1.5, 10_000), groups=2, batch=64, semirings=("log",),
                         backward=False, weights=("beta", 0.5, 0.5)),
    # the same configuration read the other way: 1e6 nodes AND ~1e7 edges, which a Zipf exponent of 1.77
    # (mean fan-in ~10 under the cap of 1e4) gives; the stated exponent 1.5 cannot (its mean is ~77)
    "powerlaw_1m_nodes": dict(kind="layered", num_vars=4096, depth=30, num_nodes=1_000_000,
                              fanin=("zipf", 1.77, 10_000), groups=2, batch=64, semirings=("log",),
                              backward=False, weights=("beta", 0.5, 0.5)),
    # headline: 3e6 nodes, 1e7 edges, depth 60, forward + backward
    "layered_3m_fwd_bwd": dict(kind="layered", num_vars=8192, depth=60, num_nodes=3_000_000,
                               fanin=("geom", 2.3), groups=4, batch=256, semirings=("log",),
                               backward=True, weights=("uniform", 0.0, 1.0)),
}


def make_config(name: str, seed: int = 0, scale: float = 1.0, batch: int | None = None):
    """Returns (circuit, p[B,V] fp64 probabilities, spec dict)."""
    spec = dict(CONFIGS[name])
    B = int(batch if batch is not None else spec["batch"])
    if spec["kind"] == "tiny":
        circ, cv, cp = tiny_ddnnf(seed, spec["num_vars"], spec["num_clauses"])
        spec["cnf"] = (cv, cp)
    else:
        n_gates = max(int(spec["num_nodes"] * scale) - 2 * spec["num_vars"], 40 * spec["depth"])
        circ = layered_random(seed, spec["num_vars"], spec["depth"], n_gates, fanin=spec["fanin"],
                              groups=spec["groups"])
    p = leaf_probs(seed + 7919, B, circ.num_vars, spec["weights"])
    spec["batch"] = B
    spec["seed"] = seed
    spec["scale"] = scale
    return circ, p, spec
