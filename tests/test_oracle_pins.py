"""Pins for the fp64 CPU oracle: everything here checks the oracle against something other
than itself -- values the paper fixes for its worked circuits, closed forms derived from its
figures, brute-force weighted model counting, the tautology invariant, finite differences,
cross-semiring identities and scipy's logsumexp.  No GPU needed."""
import itertools

import numpy as np
import pytest
from scipy.special import logsumexp

from klay_synth import (AND, FALSE, LIT, OR, TRUE, CircuitBuilder, as_inputs, layered_random,
                        leaf_probs, make_config, tautology, tiny_ddnnf)
from oracle import oracle

REAL, LOG = oracle.REAL, oracle.LOG


# ----------------------------------------------------------------------------- helpers
def bool_eval(c, assignment):
    """Boolean value of every root under one assignment (Section 2, Eq. 1), plain recursion."""
    memo = {}

    def val(n):
        if n in memo:
            return memo[n]
        t = c.node_type[n]
        if t == LIT:
            l = int(c.node_lit[n])
            r = assignment[abs(l) - 1] if l > 0 else not assignment[abs(l) - 1]
        elif t == TRUE:
            r = True
        elif t == FALSE:
            r = False
        elif t == AND:
            r = all(val(int(k)) for k in c.children(n))
        else:
            r = any(val(int(k)) for k in c.children(n))
        memo[n] = r
        return r
    return [val(int(r)) for r in c.roots]


def brute_force_wmc(c, p):
    """sum over all 2^V assignments that satisfy the circuit of prod of literal weights (fp64);
    equals the circuit value when the circuit is deterministic and decomposable."""
    V = c.num_vars
    out = np.zeros((p.shape[0], c.roots.shape[0]))
    for bits in itertools.product([False, True], repeat=V):
        sat = bool_eval(c, bits)
        if not any(sat):
            continue
        a = np.array(bits)
        wt = np.prod(np.where(a[None, :], p, 1.0 - p), axis=1)
        for r, s in enumerate(sat):
            if s:
                out[:, r] += wt
    return out


def fwd(c, w, semiring, **kw):
    return oracle.forward(*c.arrays(), w, semiring, **kw)


def bwd(c, w, semiring, dout, **kw):
    return oracle.backward(*c.arrays(), w, semiring, dout, **kw)


def fig1b_closed_form(p):
    a, b, c, d = p[:, 0], p[:, 1], p[:, 2], p[:, 3]
    return (1 - a) * (1 - b * c * (1 - d)) + a * (1 - (1 - c) * d)


# ----------------------------------------------------------------------------- worked examples
def test_fig1b_value_printed_by_the_figure(golden):
    c = golden("fig1b_ddnnf.txt")
    assert c.num_nodes == 15 and c.num_edges == 16
    half = np.full((1, 4), 0.5)
    assert fwd(c, half, REAL)[0, 0] == pytest.approx(float(c.meta["value_all_half"]), abs=1e-15)
    assert fwd(c, np.log(half), LOG)[0, 0] == pytest.approx(np.log(0.8125), abs=1e-14)
    models = sum(bool_eval(c, bits)[0] for bits in itertools.product([False, True], repeat=4))
    assert models == int(c.meta["models"])


def test_fig1b_closed_form_and_brute_force(golden):
    c = golden("fig1b_ddnnf.txt")
    p = leaf_probs(1, 16, 4, ("uniform", 0.01, 0.99))
    ref = fig1b_closed_form(p)
    np.testing.assert_allclose(fwd(c, p, REAL)[:, 0], ref, rtol=1e-13)
    np.testing.assert_allclose(fwd(c, np.log(p), LOG)[:, 0], np.log(ref), atol=1e-13)
    np.testing.assert_allclose(brute_force_wmc(c, p)[:, 0], ref, rtol=1e-13)


def test_fig1b_closed_form_gradient(golden):
    c = golden("fig1b_ddnnf.txt")
    p = leaf_probs(2, 8, 4, ("uniform", 0.05, 0.95))
    a, b, cc, d = (p[:, i] for i in range(4))
    grad = np.stack([
        -(1 - b * cc * (1 - d)) + (1 - (1 - cc) * d),      # dP/da
        -(1 - a) * cc * (1 - d),                           # dP/db
        -(1 - a) * b * (1 - d) + a * d,                    # dP/dc
        (1 - a) * b * cc - a * (1 - cc),                   # dP/dd
    ], axis=1)
    np.testing.assert_allclose(bwd(c, p, REAL, np.ones((8, 1))), grad, rtol=1e-12, atol=1e-14)
    # log domain: d log P / d log p_v = p_v / P * dP/dp_v
    P = fig1b_closed_form(p)[:, None]
    np.testing.assert_allclose(bwd(c, np.log(p), LOG, np.ones((8, 1))), p / P * grad, rtol=1e-11, atol=1e-13)


def test_fig3_two_roots_share_a_subcircuit(golden):
    c = golden("fig3_multiroot.txt")
    p = leaf_probs(3, 8, 5, ("uniform", 0.01, 0.99))
    a, b, cc, d, e = (p[:, i] for i in range(5))
    root0 = fig1b_closed_form(p[:, :4])
    root1 = a * (1 - (1 - cc) * d) + (1 - a) * e
    out = fwd(c, p, REAL)
    np.testing.assert_allclose(out[:, 0], root0, rtol=1e-13)
    np.testing.assert_allclose(out[:, 1], root1, rtol=1e-13)
    np.testing.assert_allclose(fwd(c, np.log(p), LOG), np.log(np.stack([root0, root1], 1)), atol=1e-13)
    # the adjoint of the shared sub-circuit receives both roots' contributions
    dout = np.array([[0.3, -1.7]] * 8)
    g = bwd(c, p, REAL, dout)
    d_root1_dc = a * d
    d_root0_dc = -(1 - a) * b * (1 - d) + a * d
    np.testing.assert_allclose(g[:, 2], 0.3 * d_root0_dc - 1.7 * d_root1_dc, rtol=1e-12)


def test_fig3a_single(golden):
    c = golden("fig3a_single.txt")
    p = leaf_probs(4, 4, 4, ("uniform", 0.01, 0.99))
    a, cc, d, e = (p[:, i] for i in range(4))
    np.testing.assert_allclose(fwd(c, p, REAL)[:, 0], a * (1 - (1 - cc) * d) + (1 - a) * e, rtol=1e-13)


def test_appendix_d_digit_sum(golden):
    c = golden("appD_mnist_add.txt")
    p = leaf_probs(5, 8, 2, ("uniform", 0.0, 1.0))
    q, r = p[:, 0], p[:, 1]
    ref = np.stack([(1 - q) * (1 - r), (1 - q) * r + q * (1 - r), q * r], axis=1)
    out = fwd(c, p, REAL)
    np.testing.assert_allclose(out, ref, rtol=1e-13)
    np.testing.assert_allclose(out.sum(1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(np.exp(fwd(c, np.log(p), LOG)), ref, rtol=1e-12)


# ----------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tiny_ddnnf_matches_brute_force_over_the_cnf(seed):
    """config 1: the count is taken over the CNF itself (4096 assignments), so the Shannon
    compiler and the oracle are checked independently of each other."""
    c, cv, cp = tiny_ddnnf(seed, 12, 30)
    p = leaf_probs(seed, 4, 12, ("uniform", 0.05, 0.95))
    bits = ((np.arange(4096)[:, None] >> np.arange(12)[None, :]) & 1).astype(bool)   # [4096,12]
    sat = np.ones(4096, dtype=bool)
    for vs, pos in zip(cv, cp):
        sat &= (bits[:, vs] == pos[None, :]).any(axis=1)
    assert 0 < sat.sum() < 4096
    wt = np.prod(np.where(bits[None, sat, :], p[:, None, :], 1 - p[:, None, :]), axis=2)  # [B,nsat]
    ref = wt.sum(axis=1)
    np.testing.assert_allclose(fwd(c, p, REAL)[:, 0], ref, rtol=1e-12)
    w32 = as_inputs(p, True)
    p32 = np.exp(w32.astype(np.float64))
    wt32 = np.prod(np.where(bits[None, sat, :], p32[:, None, :], -np.expm1(w32.astype(np.float64))[:, None, :]), axis=2)
    np.testing.assert_allclose(fwd(c, w32, LOG)[:, 0], np.log(wt32.sum(1)), atol=1e-12)


def test_brute_force_over_the_circuit_function():
    c, _, _ = tiny_ddnnf(7, 8, 14)
    p = leaf_probs(7, 3, 8, ("uniform", 0.05, 0.95))
    np.testing.assert_allclose(fwd(c, p, REAL), brute_force_wmc(c, p), rtol=1e-12)


# ----------------------------------------------------------------------------- invariants
@pytest.mark.parametrize("seed", [0, 1])
def test_tautology_sums_to_one(seed):
    c = tautology(seed, 24, width=4)
    p = leaf_probs(seed, 6, 24, ("beta", 0.5, 0.5))
    out, vals = fwd(c, np.log(p), LOG, return_node_values=True)
    np.testing.assert_allclose(out, 0.0, atol=1e-13)
    ors = np.where(c.node_type == OR)[0]
    reach = ~np.isnan(vals[0, ors])                                  # unreachable nodes are not evaluated
    assert reach.sum() > 24
    np.testing.assert_allclose(vals[:, ors[reach]], 0.0, atol=1e-13)  # every decision node is 1
    np.testing.assert_allclose(fwd(c, p, REAL), 1.0, rtol=1e-13)
    # the value does not depend on the weights, so the gradient vanishes
    np.testing.assert_allclose(bwd(c, p, REAL, np.ones_like(out)), 0.0, atol=1e-12)


@pytest.mark.parametrize("name,scale", [("tiny_ddnnf", 1.0), ("layered_100k", 0.05)])
def test_log_and_real_semirings_agree(name, scale):
    c, p, _ = make_config(name, seed=3, scale=scale, batch=4)
    real = fwd(c, p, REAL)
    assert np.all(real > 1e-250) and np.all(real < 1e250)
    np.testing.assert_allclose(fwd(c, np.log(p), LOG), np.log(real), atol=1e-9)


# ----------------------------------------------------------------------------- library special cases
@pytest.mark.parametrize("k", [1, 2, 7, 300])
def test_single_gate_reduces_to_library_routines(k):
    b = CircuitBuilder(k)
    leaves = [b.lit(v) for v in range(k)]
    c = b.finish([b.or_(*leaves), b.and_(*leaves)])
    x = np.log(leaf_probs(k, 5, k, ("uniform", 0.0, 1.0))) * 30.0       # wide dynamic range
    out = fwd(c, x, LOG)
    np.testing.assert_allclose(out[:, 0], logsumexp(x, axis=1), rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(out[:, 1], x.sum(axis=1), rtol=1e-14)
    # softmax is the gradient of logsumexp
    g = bwd(c, x, LOG, np.array([[1.0, 0.0]] * 5))
    np.testing.assert_allclose(g, np.exp(x - logsumexp(x, axis=1, keepdims=True)), rtol=1e-12)


# ----------------------------------------------------------------------------- gradients
def _finite_difference(c, w, semiring, dout, h):
    g = np.zeros_like(w)
    for v in range(w.shape[1]):
        wp, wm = w.copy(), w.copy()
        wp[:, v] += h
        wm[:, v] -= h
        g[:, v] = ((fwd(c, wp, semiring) - fwd(c, wm, semiring)) * dout).sum(1) / (2 * h)
    return g


@pytest.mark.parametrize("semiring", [REAL, LOG])
def test_gradients_match_finite_differences_tiny(semiring):
    c, _, _ = tiny_ddnnf(1, 12, 30)
    p = leaf_probs(11, 3, 12, ("uniform", 0.1, 0.9))
    w = np.log(p) if semiring == LOG else p
    rng = np.random.default_rng(0)
    dout = rng.normal(size=(3, 1))
    g = bwd(c, w, semiring, dout)
    fd = _finite_difference(c, w, semiring, dout, 1e-6)
    np.testing.assert_allclose(g, fd, rtol=2e-6, atol=1e-8)


@pytest.mark.parametrize("semiring", [REAL, LOG])
def test_gradients_match_finite_differences_layered(semiring):
    c = layered_random(5, num_vars=24, depth=6, num_gates=300, fanin=("geom", 2.0), groups=2, num_roots=5)
    p = leaf_probs(12, 2, 24, ("uniform", 0.1, 0.9))
    w = np.log(p) if semiring == LOG else p
    dout = np.random.default_rng(1).normal(size=(2, c.roots.shape[0]))
    g = bwd(c, w, semiring, dout)
    fd = _finite_difference(c, w, semiring, dout, 1e-6)
    scale = np.abs(fd).max()
    np.testing.assert_allclose(g, fd, rtol=1e-5, atol=1e-7 * scale)


def test_log_gradient_equals_rescaled_real_gradient():
    c, p, _ = make_config("layered_100k", seed=2, scale=0.03, batch=3)
    R = c.roots.shape[0]
    P = fwd(c, p, REAL)
    dout = np.random.default_rng(2).normal(size=(3, R))
    g_log = bwd(c, np.log(p), LOG, dout)
    g_real = bwd(c, p, REAL, dout / P)          # d(sum dout*log P) = sum dout/P dP
    np.testing.assert_allclose(g_log, p * g_real, rtol=1e-8, atol=1e-10 * np.abs(g_log).max())


# ----------------------------------------------------------------------------- degenerate inputs
def test_zero_and_one_probabilities_give_no_nan():
    b = CircuitBuilder(3)
    x, nx, y, ny, z = b.lit(0), b.lit(0, False), b.lit(1), b.lit(1, False), b.lit(2)
    root = b.or_(b.and_(x, y), b.and_(nx, ny, z))
    dead = b.or_(b.and_(x, ny), b.and_(nx, y))
    c = b.finish([root, dead, b.true(), b.false(), b.and_(), b.or_()])
    p = np.array([[1.0, 1.0, 0.3], [0.0, 0.0, 0.0], [0.0, 1.0, 0.5]])
    real = fwd(c, p, REAL)
    np.testing.assert_array_equal(real, [[1, 0, 1, 0, 1, 0], [0, 0, 1, 0, 1, 0], [0, 1, 1, 0, 1, 0]])
    with np.errstate(divide="ignore"):
        lg = fwd(c, np.log(p), LOG)
    assert not np.isnan(lg).any()
    with np.errstate(divide="ignore"):
        np.testing.assert_array_equal(lg, np.log(real))
    with np.errstate(divide="ignore"):
        g = bwd(c, np.log(p), LOG, np.array([[1.0, 0, 0, 0, 0, 0]] * 3))
    assert not np.isnan(g[1]).any() and not np.isnan(g[2]).any()
    np.testing.assert_array_equal(g[1], 0.0)    # root is -inf on that column: no gradient flows


def test_cycle_is_reported():
    node_type = np.array([AND, OR, LIT], dtype=np.uint8)
    node_lit = np.array([0, 0, 1], dtype=np.int32)
    child_ptr = np.array([0, 2, 3, 3], dtype=np.int64)
    child_idx = np.array([1, 2, 0], dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.forward(1, node_type, node_lit, child_ptr, child_idx, np.array([0], np.int32),
                       np.zeros((1, 1)), REAL)


def test_threads_do_not_change_results():
    c, p, _ = make_config("layered_100k", seed=0, scale=0.05, batch=9)
    w = np.log(p)
    np.testing.assert_array_equal(fwd(c, w, LOG, nthreads=1), fwd(c, w, LOG, nthreads=4))
    d = np.ones((9, c.roots.shape[0]))
    np.testing.assert_array_equal(bwd(c, w, LOG, d, nthreads=1), bwd(c, w, LOG, d, nthreads=4))


def test_path_mass_bounds_the_gradient_and_equals_it_without_cancellation():
    c, p, _ = make_config("layered_100k", seed=4, scale=0.03, batch=3)
    R = c.roots.shape[0]
    w = np.log(p)
    dout = np.random.default_rng(4).normal(size=(3, R))
    g = bwd(c, w, LOG, dout)
    mass = oracle.backward(*c.arrays(), w, LOG, dout, path_mass=True)
    assert np.all(mass >= np.abs(g) * (1 - 1e-12))
    # a circuit without negated literals and a positive seed has no cancellation at all
    b = CircuitBuilder(4)
    x = [b.lit(v) for v in range(4)]
    root = b.or_(b.and_(x[0], x[1]), b.and_(x[1], x[2], x[3]), b.and_(x[0], x[3]))
    cc = b.finish([root])
    w = np.log(leaf_probs(0, 5, 4, ("uniform", 0.1, 0.9)))
    ones = np.ones((5, 1))
    np.testing.assert_allclose(oracle.backward(*cc.arrays(), w, LOG, ones, path_mass=True), bwd(cc, w, LOG, ones), rtol=1e-14)
    # and with a negated literal the mass is the sum of the two branches' magnitudes
    b = CircuitBuilder(1)
    cc = b.finish([b.or_(b.lit(0), b.lit(0, False))])      # p + (1-p) = 1: gradient 0, mass 2p
    pp = np.array([[0.3]])
    np.testing.assert_allclose(bwd(cc, pp, REAL, np.ones((1, 1))), 0.0, atol=1e-15)
    np.testing.assert_allclose(oracle.backward(*cc.arrays(), pp, REAL, np.ones((1, 1)), path_mass=True), 2.0, rtol=1e-14)


# ----------------------------------------------------------------------------- (max, +) semiring
MAXLOG = oracle.MAXLOG


def proof_tree_values(c, w):
    """log weights [n_trees, B] of all proof trees below each root, straight from the semiring
    reading of Section 4: an OR offers its children as alternatives, an AND joins one tree of
    every child, a tree's weight is the sum of its leaves' log weights."""
    memo = {}

    def trees(n):
        if n in memo:
            return memo[n]
        t = c.node_type[n]
        if t == LIT:
            l = int(c.node_lit[n])
            x = w[:, abs(l) - 1]
            r = (x if l > 0 else np.log(-np.expm1(x)))[None, :]
        elif t == TRUE:
            r = np.zeros((1, w.shape[0]))
        elif t == FALSE:
            r = np.zeros((0, w.shape[0]))
        elif t == AND:
            r = np.zeros((1, w.shape[0]))
            for k in c.children(n):
                tk = trees(int(k))
                r = (r[:, None, :] + tk[None, :, :]).reshape(-1, w.shape[0])
        else:
            r = np.concatenate([trees(int(k)) for k in c.children(n)], axis=0)
        memo[n] = r
        return r
    return [trees(int(r)) for r in c.roots]


@pytest.mark.parametrize("name", ["fig1b_ddnnf.txt", "fig3_multiroot.txt", "fig3a_single.txt", "appD_mnist_add.txt"])
def test_maxlog_is_the_heaviest_proof_tree_worked_examples(golden, name):
    c = golden(name)
    w = np.log(leaf_probs(3, 6, c.num_vars, ("uniform", 0.05, 0.95)))
    out = fwd(c, w, MAXLOG)
    for r, t in enumerate(proof_tree_values(c, w)):
        np.testing.assert_allclose(out[:, r], t.max(axis=0), rtol=0, atol=1e-13)
    # and the log semiring sums the same trees
    lg = fwd(c, w, LOG)
    for r, t in enumerate(proof_tree_values(c, w)):
        np.testing.assert_allclose(lg[:, r], logsumexp(t, axis=0), atol=1e-12)
        assert np.all(out[:, r] <= lg[:, r] + 1e-12) and np.all(lg[:, r] <= out[:, r] + np.log(t.shape[0]) + 1e-12)


@pytest.mark.parametrize("seed", [0, 1])
def test_maxlog_is_the_heaviest_proof_tree_random(seed):
    c = layered_random(seed, num_vars=10, depth=4, num_gates=24, fanin=("geom", 1.0), groups=1, num_roots=2)
    w = np.log(leaf_probs(seed, 5, 10, ("uniform", 0.05, 0.95)))
    out = fwd(c, w, MAXLOG)
    for r, t in enumerate(proof_tree_values(c, w)):
        assert t.shape[0] >= 2
        np.testing.assert_allclose(out[:, r], t.max(axis=0), rtol=0, atol=1e-13)


def _smooth_obdd(nv, clauses):
    """full Shannon expansion in variable order, branching on every variable (so every model sets
    every variable: smooth, deterministic, decomposable); clauses: list of [(var, positive)]"""
    b = CircuitBuilder(nv)
    memo = {}

    def go(i, rest):
        if any(len(cl) == 0 for cl in rest):
            return None
        if i == nv:
            return "true"
        key = (i, rest)
        if key in memo:
            return memo[key]
        branches = []
        for val in (True, False):
            nxt = []
            for cl in rest:
                if (i, val) in cl:
                    continue
                nxt.append(tuple(l for l in cl if l[0] != i))
            sub = go(i + 1, tuple(sorted(set(nxt))))
            if sub is None:
                continue
            lit = b.lit(i, val)
            branches.append(lit if sub == "true" else b.and_(lit, sub))
        node = None if not branches else (branches[0] if len(branches) == 1 else b.or_(*branches))
        memo[key] = node
        return node
    root = go(0, tuple(sorted(set(tuple(sorted(cl)) for cl in clauses))))
    assert root is not None and root != "true"
    return b.finish([root])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_maxlog_on_a_smooth_ddnnf_is_the_most_probable_model(seed):
    rng = np.random.default_rng(100 + seed)
    nv, ncl = 9, 14
    clauses = [[(int(v), bool(rng.integers(2))) for v in rng.choice(nv, 3, replace=False)] for _ in range(ncl)]
    c = _smooth_obdd(nv, clauses)
    p = leaf_probs(seed, 7, nv, ("uniform", 0.05, 0.95))
    bits = ((np.arange(2 ** nv)[:, None] >> np.arange(nv)[None, :]) & 1).astype(bool)
    sat = np.ones(2 ** nv, dtype=bool)
    for cl in clauses:
        sat &= np.any([bits[:, v] == pos for v, pos in cl], axis=0)
    assert 0 < sat.sum() < 2 ** nv
    logw = np.where(bits[None, sat, :], np.log(p)[:, None, :], np.log1p(-p)[:, None, :]).sum(axis=2)   # [B, nsat]
    np.testing.assert_allclose(fwd(c, np.log(p), MAXLOG)[:, 0], logw.max(axis=1), atol=1e-12)
    np.testing.assert_allclose(fwd(c, np.log(p), LOG)[:, 0], logsumexp(logw, axis=1), atol=1e-12)


def test_maxlog_single_gates_and_impossible_branches():
    b = CircuitBuilder(6)
    c = b.finish([b.or_(*[b.lit(v) for v in range(6)]), b.and_(*[b.lit(v, v % 2 == 0) for v in range(6)])])
    p = leaf_probs(4, 5, 6, ("uniform", 0.05, 0.95))
    out = fwd(c, np.log(p), MAXLOG)
    np.testing.assert_allclose(out[:, 0], np.log(p).max(axis=1), atol=0)
    np.testing.assert_allclose(out[:, 1], np.where(np.arange(6) % 2 == 0, np.log(p), np.log1p(-p)).sum(axis=1), atol=1e-13)
    p[:, :] = 0.0
    with np.errstate(divide="ignore"):
        out = fwd(c, np.log(p), MAXLOG)
    assert np.all(out == -np.inf)
    with pytest.raises(ValueError):
        bwd(c, np.log(np.full((1, 6), 0.5)), MAXLOG, np.ones((1, 2)))


# ----------------------------------------------------------------------------- literal weights of their own
def test_negative_literal_weights_fig1b_polynomial(golden):
    """Figure 1(b) read as a polynomial in the eight literal weights:
    -b -a  +  -a b (c d + -c)  +  (c d + -d) a"""
    c = golden("fig1b_ddnnf.txt")
    rng = np.random.default_rng(3)
    wp, wn = rng.uniform(0.1, 2.0, size=(5, 4)), rng.uniform(0.1, 2.0, size=(5, 4))
    a, b, cc, d = (wp[:, i] for i in range(4))
    na, nb, nc, nd = (wn[:, i] for i in range(4))
    ref = nb * na + na * b * (cc * d + nc) + (cc * d + nd) * a
    np.testing.assert_allclose(fwd(c, wp, REAL, neg_weights=wn)[:, 0], ref, rtol=1e-13)
    np.testing.assert_allclose(fwd(c, np.log(wp), LOG, neg_weights=np.log(wn))[:, 0], np.log(ref), atol=1e-12)
    # gradients of the polynomial, by hand
    dout = rng.normal(size=(5, 1))
    dp, dn = bwd(c, wp, REAL, dout, neg_weights=wn)
    np.testing.assert_allclose(dp[:, 0], dout[:, 0] * (cc * d + nd), rtol=1e-12)                 # d/da
    np.testing.assert_allclose(dn[:, 0], dout[:, 0] * (nb + b * (cc * d + nc)), rtol=1e-12)      # d/d(-a)
    np.testing.assert_allclose(dp[:, 3], dout[:, 0] * (na * b * cc + cc * a), rtol=1e-12)        # d/dd
    np.testing.assert_allclose(dn[:, 3], dout[:, 0] * a, rtol=1e-12)                             # d/d(-d)
    # log domain: d log f / d log w = w df/dw / f
    lp, ln = bwd(c, np.log(wp), LOG, dout, neg_weights=np.log(wn))
    np.testing.assert_allclose(lp, dp * wp / ref[:, None], rtol=1e-11)
    np.testing.assert_allclose(ln, dn * wn / ref[:, None], rtol=1e-11)


@pytest.mark.parametrize("seed", [0, 1])
def test_negative_literal_weights_weighted_model_count(seed):
    """smooth d-DNNF: the value is the sum over models of the product of arbitrary literal weights"""
    rng = np.random.default_rng(200 + seed)
    nv = 9
    clauses = [[(int(v), bool(rng.integers(2))) for v in rng.choice(nv, 3, replace=False)] for _ in range(14)]
    c = _smooth_obdd(nv, clauses)
    wp, wn = rng.uniform(0.2, 3.0, size=(4, nv)), rng.uniform(0.2, 3.0, size=(4, nv))
    bits = ((np.arange(2 ** nv)[:, None] >> np.arange(nv)[None, :]) & 1).astype(bool)
    sat = np.ones(2 ** nv, dtype=bool)
    for cl in clauses:
        sat &= np.any([bits[:, v] == pos for v, pos in cl], axis=0)
    ref = np.prod(np.where(bits[None, sat, :], wp[:, None, :], wn[:, None, :]), axis=2).sum(axis=1)
    np.testing.assert_allclose(fwd(c, wp, REAL, neg_weights=wn)[:, 0], ref, rtol=1e-12)
    np.testing.assert_allclose(fwd(c, np.log(wp), LOG, neg_weights=np.log(wn))[:, 0], np.log(ref), atol=1e-11)
    heaviest = np.log(np.where(bits[None, sat, :], wp[:, None, :], wn[:, None, :])).sum(axis=2).max(axis=1)
    np.testing.assert_allclose(fwd(c, np.log(wp), MAXLOG, neg_weights=np.log(wn))[:, 0], heaviest, atol=1e-11)


def test_negative_literal_weights_default_and_finite_differences():
    c = layered_random(5, num_vars=12, depth=6, num_gates=200, fanin=("geom", 2.0), groups=1, num_roots=3)
    p = leaf_probs(5, 3, 12, ("uniform", 0.1, 0.9))
    # 1 - p given explicitly is the default
    np.testing.assert_allclose(fwd(c, p, REAL, neg_weights=1 - p), fwd(c, p, REAL), rtol=1e-14)
    np.testing.assert_allclose(fwd(c, np.log(p), LOG, neg_weights=np.log1p(-p)), fwd(c, np.log(p), LOG), atol=1e-13)
    rng = np.random.default_rng(6)
    dout = rng.normal(size=(3, 3))
    for sem, a, b in ((REAL, p, rng.uniform(0.1, 0.9, size=p.shape)), (LOG, np.log(p), np.log(rng.uniform(0.1, 0.9, size=p.shape)))):
        dp, dn = bwd(c, a, sem, dout, neg_weights=b)
        h = 1e-6
        for v in (0, 5, 11):
            e = np.zeros_like(a); e[:, v] = h
            fd_p = ((fwd(c, a + e, sem, neg_weights=b) - fwd(c, a - e, sem, neg_weights=b)) * dout).sum(1) / (2 * h)
            fd_n = ((fwd(c, a, sem, neg_weights=b + e) - fwd(c, a, sem, neg_weights=b - e)) * dout).sum(1) / (2 * h)
            np.testing.assert_allclose(dp[:, v], fd_p, rtol=1e-5, atol=1e-8)
            np.testing.assert_allclose(dn[:, v], fd_n, rtol=1e-5, atol=1e-8)
    # the default's gradient is the chain rule over the two: dpos - dneg (REAL, neg = 1 - p)
    dp, dn = bwd(c, p, REAL, dout, neg_weights=1 - p)
    np.testing.assert_allclose(bwd(c, p, REAL, dout), dp - dn, rtol=1e-10, atol=1e-12)


def test_unary_gates_are_identities_for_values_and_gradients():
    """Section 3.1 pads with single-child gates, so a single-child gate in the input must be transparent:
    wrapping any node in OR(.) / AND(.) changes neither values nor gradients, also where the value is
    log 0 = -inf (a softmax over one element has weight 1, not 0/0)."""
    def circuit(wrap):
        b = CircuitBuilder(3)
        x, y, z, nz = b.lit(0), b.lit(1), b.lit(2), b.lit(2, False)
        u = b.and_(x, y)
        if wrap:
            u = b.or_(b.and_(b.or_(u)))
        dead = b.and_(z, nz, x)                       # impossible once p(z) is 0 or 1
        if wrap:
            dead = b.or_(dead)
        return b.finish([b.or_(u, b.and_(z, y)), dead, b.or_(dead, b.and_(dead, y))])
    p = np.array([[0.3, 0.6, 0.2], [0.5, 0.1, 1.0], [0.9, 0.4, 0.0]])
    dout = np.array([[1.0, -2.0, 0.5]] * 3)
    with np.errstate(divide="ignore"):
        w = np.log(p)
    plain, wrapped = circuit(False), circuit(True)
    np.testing.assert_array_equal(fwd(plain, w, LOG), fwd(wrapped, w, LOG))
    g0, g1 = bwd(plain, w, LOG, dout), bwd(wrapped, w, LOG, dout)
    assert not np.isnan(g0[0]).any() and np.all(np.isfinite(g0[0]))
    np.testing.assert_allclose(g1[0], g0[0], rtol=1e-14)
    # rows 1 and 2: root 1 is -inf; its adjoint still reaches the leaves through the unary gate exactly as
    # it does without it (the AND below passes it on), while the two-child OR at -inf (root 2) passes nothing
    for r in (1, 2):
        fin = np.isfinite(g0[r])
        np.testing.assert_array_equal(np.isfinite(g1[r]), fin)
        np.testing.assert_allclose(g1[r][fin], g0[r][fin], rtol=1e-14)
    only_root2 = bwd(plain, w, LOG, np.array([[0.0, 0.0, 1.0]] * 3))
    assert np.all(only_root2[1:][np.isfinite(only_root2[1:])] == 0.0)
    np.testing.assert_allclose(bwd(plain, p, REAL, dout), bwd(wrapped, p, REAL, dout), rtol=1e-14)
