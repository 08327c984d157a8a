"""Seeded synthetic circuit DAGs (inputs only: no circuit arithmetic lives here).

Everything returns a :class:`Circuit`: a negation-normal-form DAG in CSR form
(paper Section 2: leaves are literals, inner nodes are AND / OR gates), which is
what both the GPU library's ``klay_build`` and the CPU oracle take.  The
generators stand in for the compiled circuits of the paper's experiments
(Section 6.1 / Appendix B: random 3-CNF compiled to d-DNNF; Table 1: 24-84
layers, 1e3-1e6 nodes, widths tapering to the roots), which are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

LIT, AND, OR, TRUE, FALSE = 0, 1, 2, 3, 4


@dataclass
class Circuit:
    num_vars: int
    node_type: np.ndarray  # uint8 [n]
    node_lit: np.ndarray   # int32 [n]  +(v+1) / -(v+1) for literals, else 0
    child_ptr: np.ndarray  # int64 [n+1]
    child_idx: np.ndarray  # int32 [child_ptr[-1]]
    roots: np.ndarray      # int32 [R]
    meta: dict = field(default_factory=dict)

    @property
    def num_nodes(self) -> int:
        return int(self.node_type.shape[0])

    @property
    def num_edges(self) -> int:
        return int(self.child_idx.shape[0])

    def arrays(self):
        return (self.num_vars, self.node_type, self.node_lit, self.child_ptr, self.child_idx, self.roots)

    def children(self, n: int):
        return self.child_idx[self.child_ptr[n]:self.child_ptr[n + 1]]


class CircuitBuilder:
    """Append-only builder for small hand-made circuits (tests, worked examples)."""

    def __init__(self, num_vars: int):
        self.num_vars = num_vars
        self.types: list[int] = []
        self.lits: list[int] = []
        self.kids: list[list[int]] = []
        self._lit_ids: dict[int, int] = {}

    def _add(self, t, lit, kids):
        self.types.append(t)
        self.lits.append(lit)
        self.kids.append(list(kids))
        return len(self.types) - 1

    def lit(self, var: int, positive: bool = True) -> int:
        code = (var + 1) if positive else -(var + 1)
        if code not in self._lit_ids:
            self._lit_ids[code] = self._add(LIT, code, [])
        return self._lit_ids[code]

    def true(self) -> int:
        return self._add(TRUE, 0, [])

    def false(self) -> int:
        return self._add(FALSE, 0, [])

    def and_(self, *kids: int) -> int:
        return self._add(AND, 0, kids)

    def or_(self, *kids: int) -> int:
        return self._add(OR, 0, kids)

    def finish(self, roots, meta=None) -> Circuit:
        ptr = np.zeros(len(self.types) + 1, dtype=np.int64)
        for i, k in enumerate(self.kids):
            ptr[i + 1] = ptr[i] + len(k)
        idx = np.array([c for k in self.kids for c in k], dtype=np.int32)
        return Circuit(self.num_vars, np.array(self.types, dtype=np.uint8),
                       np.array(self.lits, dtype=np.int32), ptr, idx,
                       np.array(list(roots), dtype=np.int32), dict(meta or {}))


def parse_text_circuit(text: str) -> Circuit:
    """Parse the small fixture format used under tests/golden/.

    Lines: ``vars a b c``; ``node NAME AND|OR child child ...`` where a child is a
    previously defined node name, a variable name (positive literal) or ``-name``
    (negative literal); ``roots NAME ...``; ``key value`` pairs go to ``meta``;
    ``#`` starts a comment.
    """
    names: dict[str, int] = {}
    var_ids: dict[str, int] = {}
    b = None
    roots: list[int] = []
    meta: dict = {}
    for raw in text.splitlines():
        line = raw.split("#", 1)[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "vars":
            var_ids = {v: i for i, v in enumerate(tok[1:])}
            b = CircuitBuilder(len(var_ids))
        elif tok[0] == "node":
            kids = []
            for c in tok[3:]:
                if c in names:
                    kids.append(names[c])
                elif c.startswith("-"):
                    kids.append(b.lit(var_ids[c[1:]], False))
                else:
                    kids.append(b.lit(var_ids[c], True))
            names[tok[1]] = b.and_(*kids) if tok[2] == "AND" else b.or_(*kids)
        elif tok[0] == "roots":
            for r in tok[1:]:
                if r in names:
                    roots.append(names[r])
                elif r.startswith("-"):
                    roots.append(b.lit(var_ids[r[1:]], False))
                else:
                    roots.append(b.lit(var_ids[r], True))
        else:
            meta[tok[0]] = tok[1:] if len(tok) > 2 else tok[1]
    meta["var_names"] = list(var_ids)
    meta["node_names"] = names
    return b.finish(roots, meta)


# --------------------------------------------------------------------------------------
# config 1: random 3-CNF compiled to an ordered decision diagram by Shannon expansion
# --------------------------------------------------------------------------------------

def random_3cnf(seed: int, num_vars: int, num_clauses: int):
    """k clauses of 3 distinct uniformly drawn variables with uniform signs (Appendix B recipe;
    the paper does not state the sign distribution).  Returns (vars[k,3], positive[k,3])."""
    rng = np.random.default_rng(seed)
    vs = np.stack([rng.choice(num_vars, size=3, replace=False) for _ in range(num_clauses)])
    pos = rng.integers(0, 2, size=(num_clauses, 3)).astype(bool)
    return vs.astype(np.int64), pos


def obdd_from_cnf(num_vars: int, clause_vars, clause_pos) -> Circuit:
    """Shannon-expand a CNF in the fixed order x0, x1, ... into a deterministic, decomposable
    NNF: every decision is OR(AND(x, hi), AND(-x, lo)); constant branches are simplified away
    and residual formulas are shared through a memo on the residual clause set.  Variables a
    sub-formula does not mention are skipped (the circuit is not smooth)."""
    clauses = frozenset(
        frozenset((int(v), bool(s)) for v, s in zip(cv, cp)) for cv, cp in zip(clause_vars, clause_pos)
    )
    b = CircuitBuilder(num_vars)
    memo: dict = {}

    def condition(cls, var, value):
        out = set()
        for c in cls:
            if (var, value) in c:
                continue                      # clause satisfied
            if (var, not value) in c:
                c = c - {(var, not value)}
                if not c:
                    return None               # empty clause: unsatisfiable
            out.add(c)
        return frozenset(out)

    def expand(cls):
        """returns node id, or True / False for constants"""
        if cls is None:
            return False
        if not cls:
            return True
        if cls in memo:
            return memo[cls]
        var = min(v for c in cls for v, _ in c)
        hi = expand(condition(cls, var, True))
        lo = expand(condition(cls, var, False))
        if hi is lo and isinstance(hi, bool):
            res = hi
        elif (not isinstance(hi, bool)) and (not isinstance(lo, bool)) and hi == lo:
            res = hi
        else:
            branches = []
            for child, positive in ((hi, True), (lo, False)):
                if child is False:
                    continue
                l = b.lit(var, positive)
                branches.append(l if child is True else b.and_(l, child))
            res = branches[0] if len(branches) == 1 else b.or_(*branches)
        memo[cls] = res
        return res

    import sys
    old = sys.getrecursionlimit()
    sys.setrecursionlimit(max(old, 10 * num_vars + 1000))
    try:
        root = expand(clauses)
    finally:
        sys.setrecursionlimit(old)
    if root is True:
        root = b.true()
    elif root is False:
        root = b.false()
    return b.finish([root], {"kind": "obdd_from_3cnf"})


def tiny_ddnnf(seed: int, num_vars: int = 12, num_clauses: int = 30):
    """Config 1.  Returns (circuit, clause_vars, clause_pos); redraws the CNF (seed, seed+1000,
    ...) until it is satisfiable and not a tautology so that the circuit is not a constant."""
    s = seed
    while True:
        cv, cp = random_3cnf(s, num_vars, num_clauses)
        c = obdd_from_cnf(num_vars, cv, cp)
        if c.node_type[c.roots[0]] not in (TRUE, FALSE):
            c.meta.update(seed=s, num_clauses=num_clauses)
            return c, cv, cp
        s += 1000


# --------------------------------------------------------------------------------------
# tautology: a smooth, deterministic decision circuit whose value is 1 for any weights
# --------------------------------------------------------------------------------------

def tautology(seed: int, num_vars: int, width: int = 3) -> Circuit:
    """Level i holds `width` decision nodes on variable i, each OR(AND(x_i, A), AND(-x_i, B))
    with A, B drawn from level i+1; the last level is OR(x, -x).  Every decision node is the
    constant TRUE function over variables i.., so its weighted count is 1 when w(x)+w(-x)=1."""
    rng = np.random.default_rng(seed)
    b = CircuitBuilder(num_vars)
    v = num_vars - 1
    level = [b.or_(b.lit(v, True), b.lit(v, False))]
    for v in range(num_vars - 2, -1, -1):
        new = []
        for _ in range(width):
            hi = level[int(rng.integers(len(level)))]
            lo = level[int(rng.integers(len(level)))]
            new.append(b.or_(b.and_(b.lit(v, True), hi), b.and_(b.lit(v, False), lo)))
        level = new
    return b.finish(level, {"kind": "tautology"})


# --------------------------------------------------------------------------------------
# configs 2-5: random layered circuits
# --------------------------------------------------------------------------------------

def _fanin_sampler(fanin):
    kind = fanin[0]
    if kind == "geom":
        mean_extra = float(fanin[1])            # fan-in = 1 + Geometric on {0,1,..} with this mean

        def draw(rng, n):
            if mean_extra <= 0:
                return np.ones(n, dtype=np.int64)
            p = 1.0 / (1.0 + mean_extra)
            return rng.geometric(p, size=n).astype(np.int64)   # support {1,2,..}, mean 1+mean_extra
        return draw
    if kind == "zipf":
        s, cap = float(fanin[1]), int(fanin[2])
        ks = np.arange(1, cap + 1, dtype=np.float64)
        cdf = np.cumsum(ks ** (-s))
        cdf /= cdf[-1]

        def draw(rng, n):
            return (np.searchsorted(cdf, rng.random(n), side="left") + 1).astype(np.int64)
        return draw
    raise ValueError(fanin)


def _layer_widths(depth, num_gates, num_roots, alpha):
    """Widths w[1..depth] tapering geometrically to num_roots at the top.  Going down from an OR
    layer the AND layer below is rho times wider; going down from an AND layer the OR layer
    below is alpha times narrower (every OR needs a parent AND of its own).  rho is solved so
    that the widths sum to num_gates."""
    def widths(rho):
        w = np.zeros(depth + 1)
        w[depth] = num_roots
        for l in range(depth, 1, -1):
            w[l - 1] = w[l] * rho if l % 2 == 0 else w[l] / alpha
        return w
    lo, hi = alpha, 64.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if widths(mid)[1:].sum() < num_gates:
            lo = mid
        else:
            hi = mid
    w = np.maximum(np.round(widths(hi)), 1).astype(np.int64)
    w[depth] = num_roots
    for l in range(depth, 1, -1):              # rounding must not break the covering constraints
        if l % 2 == 1:
            w[l] = max(w[l], w[l - 1])
    return w


def layered_random(seed: int, num_vars: int, depth: int, num_gates: int, fanin=("geom", 2.0),
                   groups: int = 4, num_roots: int = 64, alpha: float = 1.25,
                   window_back_prob: float = 0.3, shuffle_ids: bool = True) -> Circuit:
    """Random layered circuit: odd generator layers hold AND gates, even layers OR gates.

    * AND gate: one gate child from the layer below (none in layer 1) plus fan-in-1 distinct
      literals, drawn from a block of variables reserved for (its group, its AND level), so AND
      gates are decomposable and |log value| grows only linearly with depth.
    * OR gate: children are AND gates of its own variable group from the previous three layers
      (layers l-1 and l-3 hold the AND gates); every gate of layer l-1 gets at least one parent
      in layer l, the remaining fan-in is drawn uniformly from the group's gates in l-1 (prob.
      1-window_back_prob) or l-3.  Repeated draws are dropped, so realised fan-in can be lower.
    * Widths taper geometrically to `num_roots` roots in the top layer.
    * Node ids are shuffled at the end so that id order carries no locality.

    Fan-in: ("geom", m) = 1 + Geometric with mean m; ("zipf", s, cap) = Zipf(s) truncated at cap.
    """
    if depth < 2:
        raise ValueError("depth must be >= 2")
    rng = np.random.default_rng(seed)
    draw = _fanin_sampler(fanin)
    widths = _layer_widths(depth, num_gates, num_roots, alpha)
    n_and_levels = (depth + 1) // 2
    block = num_vars // (groups * n_and_levels)
    if block < 1:
        raise ValueError("too few variables for groups x AND levels")
    lit_id = lambda var, positive: 2 * var + (0 if positive else 1)   # node ids of the 2V literals
    next_id = 2 * num_vars

    par_list, chi_list = [], []          # edge lists (parent id, child id), concatenated later
    layer_ids: list = [None] * (depth + 1)   # node ids per generator layer
    layer_grp: list = [None] * (depth + 1)   # variable group per node
    types = [np.full(2 * num_vars, LIT, dtype=np.uint8)]

    for l in range(1, depth + 1):
        w = int(widths[l])
        if l % 2 == 1:                                   # ---- AND layer
            level = (l - 1) // 2
            if l > 1:
                w = max(w, layer_ids[l - 1].shape[0])
            ids = np.arange(next_id, next_id + w, dtype=np.int64)
            k = draw(rng, w)
            if l == 1:
                grp = rng.integers(0, groups, size=w)
                n_lit = np.clip(k, 1, block)
            else:
                below = layer_ids[l - 1]
                wb = below.shape[0]
                pick = np.concatenate([rng.permutation(wb), rng.integers(0, wb, size=w - wb)])
                pick = pick[rng.permutation(w)]
                grp = layer_grp[l - 1][pick]
                par_list.append(ids)
                chi_list.append(below[pick])
                n_lit = np.clip(k - 1, 0, block)
            base = (grp * n_and_levels + level) * block
            start = rng.integers(0, block, size=w)
            tot = int(n_lit.sum())
            owner = np.repeat(np.arange(w), n_lit)
            within = np.arange(tot) - np.repeat(np.cumsum(n_lit) - n_lit, n_lit)
            var = base[owner] + (start[owner] + within) % block
            sign = rng.integers(0, 2, size=tot).astype(bool)
            par_list.append(ids[owner])
            chi_list.append(2 * var + np.where(sign, 0, 1))
            types.append(np.full(w, AND, dtype=np.uint8))
        else:                                            # ---- OR layer
            below, gb = layer_ids[l - 1], layer_grp[l - 1]
            order = np.argsort(gb, kind="stable")
            cnt = np.bincount(gb, minlength=groups)
            # parents per group proportional to the group's share of the layer below, >= 1 each
            share = np.maximum(1, np.floor(cnt * w / max(1, below.shape[0]))).astype(np.int64)
            share[cnt == 0] = 0
            while share.sum() < w:
                share[np.argmax(cnt / np.maximum(share, 1))] += 1
            while share.sum() > w and share.max() > 1:
                share[np.argmax(share)] -= 1
            w = int(share.sum())
            ids = np.arange(next_id, next_id + w, dtype=np.int64)
            k = draw(rng, w)
            grp = np.repeat(np.arange(groups), share)
            gstart = np.cumsum(share) - share            # first parent slot of each group
            cstart = np.cumsum(cnt) - cnt                # first child slot of each group in `order`
            # primary children: deal each group's gates round-robin over the group's parents
            child_sorted = below[order]
            g_of_child = gb[order]
            rank = np.arange(below.shape[0]) - cstart[g_of_child]
            prim_parent = gstart[g_of_child] + rank % share[g_of_child]
            par_list.append(ids[prim_parent])
            chi_list.append(child_sorted)
            n_prim = np.bincount(prim_parent, minlength=w)
            extra = np.maximum(0, k - n_prim)
            tot = int(extra.sum())
            if tot:
                owner = np.repeat(np.arange(w), extra)
                og = grp[owner]
                use_back = np.zeros(tot, dtype=bool)
                if l >= 4:
                    back, gbk = layer_ids[l - 3], layer_grp[l - 3]
                    order_b = np.argsort(gbk, kind="stable")
                    cnt_b = np.bincount(gbk, minlength=groups)
                    cstart_b = np.cumsum(cnt_b) - cnt_b
                    use_back = (rng.random(tot) < window_back_prob) & (cnt_b[og] > 0)
                u = rng.random(tot)
                ch = np.empty(tot, dtype=np.int64)
                f = ~use_back
                ch[f] = child_sorted[cstart[og[f]] + np.minimum((u[f] * cnt[og[f]]).astype(np.int64), cnt[og[f]] - 1)]
                if use_back.any():
                    bsel = use_back
                    ch[bsel] = back[order_b][cstart_b[og[bsel]] + np.minimum(
                        (u[bsel] * cnt_b[og[bsel]]).astype(np.int64), cnt_b[og[bsel]] - 1)]
                par_list.append(ids[owner])
                chi_list.append(ch)
            types.append(np.full(w, OR, dtype=np.uint8))
        next_id += w
        layer_ids[l] = ids
        layer_grp[l] = grp

    n = next_id
    par = np.concatenate(par_list)
    chi = np.concatenate(chi_list)
    key = np.unique(par * n + chi)                        # drop repeated children, sort by parent
    par, chi = key // n, key % n
    node_type = np.concatenate(types)[:n]
    node_lit = np.zeros(n, dtype=np.int32)
    v = np.arange(num_vars)
    node_lit[2 * v] = v + 1
    node_lit[2 * v + 1] = -(v + 1)
    roots = layer_ids[depth].copy()

    if shuffle_ids:
        perm = rng.permutation(n)                         # old id -> new id
        inv = np.empty(n, dtype=np.int64)
        inv[perm] = np.arange(n)
        par, chi = perm[par], perm[chi]
        o = np.lexsort((rng.random(par.shape[0]), par))   # children of a gate in random order
        par, chi = par[o], chi[o]
        node_type, node_lit = node_type[inv], node_lit[inv]
        roots = perm[roots]
        roots = roots[rng.permutation(roots.shape[0])]
    child_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(par, minlength=n), out=child_ptr[1:])
    meta = {"kind": "layered_random", "seed": seed, "depth": depth, "fanin": fanin,
            "groups": groups, "widths": [int(x.shape[0]) for x in layer_ids[1:]]}
    return Circuit(num_vars, node_type, node_lit, child_ptr, chi.astype(np.int32),
                   roots.astype(np.int32), meta)
