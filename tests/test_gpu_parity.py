"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Tolerances: |delta log| <= 1e-4 (fp32 log semiring), relative 1e-5
(fp32 real semiring).  Gradients: with the adjoint seed dout = 1 the plain bound
|delta| <= 1e-4 max(1, |ref|) (assert_grad_plain); with a random dout of mixed signs the same bound plus
a cancellation term proportional to the path mass (assert_grad_close, derivation in tests/gpu_util.py);
the session summary prints how far above the plain bound the worst such case was."""
import numpy as np
import pytest

from klay_synth import (AND, CircuitBuilder, as_inputs, layered_random, leaf_probs, make_config,
                        parse_text_circuit, tautology)
from tests.gpu_util import (assert_grad_close, assert_grad_plain, assert_log_close, assert_real_close, gpu_eval,
                            oracle_eval)

pytestmark = pytest.mark.gpu

REAL, LOG = 0, 1


@pytest.fixture(scope="module")
def klay():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2410_11415_amd as pkg
    pkg.load()                         # fails loudly if the HIP library is missing
    return pkg


def build(klay, c, **kw):
    return klay.Circuit(*c.arrays(), device=0, **kw)


def layer_modes(klay, c):
    """Builds of one circuit that differ in where the padding-free lower part of the layerization ends:
    nowhere (the paper's layerization throughout), at the top layer (no persistent kernels), and at layers
    in between (layers wider than a cap are no candidates for the persistent kernels)."""
    kh = klay.Circuit(*c.arrays(), device=-1, unary_chains=True)
    nodes, _ = kh.layer_sizes()
    kh.close()
    caps = sorted({max(int(x), 1) for x in np.quantile(np.asarray(nodes[1:]), [0.3, 0.7])}) if len(nodes) > 2 else []
    return [dict(unary_chains=True), dict(no_tail=True)] + [dict(tail_rows_cap=cap) for cap in caps]


def check_both(klay, c, p, backward=True, semirings=(REAL, LOG), what="", plain=False, **kw):
    k = build(klay, c, **kw)
    rng = np.random.default_rng(123)
    stats = {}
    levels = k.num_layers // 2
    for s in semirings:
        w32 = as_inputs(p, s == LOG)
        can_bwd = backward
        dout = rng.normal(size=(p.shape[0], c.roots.shape[0])).astype(np.float32) if can_bwd else None
        got, gd = gpu_eval(k, w32, s, dout)
        ref, rd = oracle_eval(c, w32, s, dout, or_levels=levels)
        if s == LOG:
            stats["log"] = assert_log_close(got, ref, what + " log")
            if dout is not None:
                stats["grad"] = assert_grad_close(gd, rd, what + " grad")
                if plain:
                    # adjoint seed 1: the plain bound, no cancellation term
                    ones = np.ones_like(dout)
                    _, g1 = gpu_eval(k, w32, s, ones)
                    from oracle import oracle
                    with np.errstate(all="ignore"):
                        r1 = oracle.backward(*c.arrays(), w32.astype(np.float64), oracle.LOG, ones.astype(np.float64), nthreads=8)
                    stats["grad_plain"] = assert_grad_plain(g1, r1, what + " grad, dout = 1")
        else:
            stats["real"] = assert_real_close(got, ref, what + " real")
            if dout is not None:
                stats["real_grad"] = assert_grad_close(gd, rd, what + " real grad", real=True)
    k.close()
    return stats


# ------------------------------------------------------------------ the paper's worked circuits
@pytest.mark.parametrize("name,nv", [("fig1b_ddnnf.txt", 4), ("fig3_multiroot.txt", 5), ("fig3a_single.txt", 4),
                                      ("appD_mnist_add.txt", 2)])
def test_worked_examples(klay, golden, name, nv):
    c = golden(name)
    for B in (1, 3, 70):
        check_both(klay, c, leaf_probs(B, B, nv, ("uniform", 0.01, 0.99)), what=name)


# ------------------------------------------------------------------ circuits loaded from text files
def test_loaded_files_evaluate_on_the_gpu(klay):
    """the d-DNNF .nnf file of Fig. 1b, the hand-written .sdd and the d4 file, through Circuit.from_*,
    against the oracle on the arrays the readers return"""
    import os
    from oracle import oracle
    from paper_2410_11415_amd.d4 import load_d4
    from paper_2410_11415_amd.nnf import load_nnf
    from paper_2410_11415_amd.sdd import load_sdd
    from tests.conftest import GOLDEN
    cases = (("fig1b_ddnnf.nnf", klay.Circuit.from_nnf, load_nnf), ("a_and_b_or_c.sdd", klay.Circuit.from_sdd, load_sdd),
             ("a_and_b_or_c.d4", klay.Circuit.from_d4, load_d4))
    for fname, ctor, loader in cases:
        path = os.path.join(GOLDEN, fname)
        arr = loader(path)
        k = ctor(path, device=0)
        for B in (1, 5, 70):
            p = leaf_probs(B, B, arr[0], ("uniform", 0.02, 0.98))
            dout = np.ones((B, k.num_roots), dtype=np.float32)
            for s, osem in ((LOG, oracle.LOG), (REAL, oracle.REAL)):
                w32 = as_inputs(p, s == LOG)
                got, gd = gpu_eval(k, w32, s, dout)
                w64 = w32.astype(np.float64)
                ref = oracle.forward(*arr, w64, osem)
                rd = oracle.backward(*arr, w64, osem, dout.astype(np.float64))
                if s == LOG:
                    assert_log_close(got, ref, fname)
                    assert_grad_plain(gd, rd, fname + " grad")
                else:
                    assert_real_close(got, ref, fname)
                    np.testing.assert_allclose(gd, rd, rtol=2e-5, atol=1e-6, err_msg=fname + " real grad")
        if fname == "fig1b_ddnnf.nnf":      # 13 of 16 models at p = 1/2
            half = as_inputs(np.full((1, 4), 0.5), False)
            assert gpu_eval(k, half, REAL)[0][0, 0] == pytest.approx(13 / 16, rel=1e-6)
        k.close()


# ------------------------------------------------------------------ config 1
@pytest.mark.parametrize("seed", [0, 1])
def test_tiny_ddnnf_batch4(klay, seed):
    c, p, spec = make_config("tiny_ddnnf", seed=seed)
    assert p.shape[0] == 4
    check_both(klay, c, p, what="tiny_ddnnf", plain=True)
    # and against brute-force model counting over the CNF (4096 assignments)
    cv, cp = spec["cnf"]
    bits = ((np.arange(4096)[:, None] >> np.arange(12)[None, :]) & 1).astype(bool)
    sat = np.ones(4096, dtype=bool)
    for vs, pos in zip(cv, cp):
        sat &= (bits[:, vs] == pos[None, :]).any(axis=1)
    w32 = as_inputs(p, True)
    p32 = np.exp(w32.astype(np.float64))
    q32 = -np.expm1(w32.astype(np.float64))
    ref = np.log(np.prod(np.where(bits[None, sat, :], p32[:, None, :], q32[:, None, :]), axis=2).sum(1))
    k = build(klay, c)
    got, _ = gpu_eval(k, w32, LOG)
    assert_log_close(got[:, 0], ref, "tiny_ddnnf vs brute force")


# ------------------------------------------------------------------ config 2 (full size, element by element)
def test_layered_100k_full_size_log_forward(klay):
    c, p, spec = make_config("layered_100k", seed=0)
    assert p.shape[0] == 128
    stats = check_both(klay, c, p, backward=True, semirings=(LOG,), what="layered_100k", plain=True)
    print("layered_100k", stats)


# ------------------------------------------------------------------ configs 3-5 at reduced size, element by element
@pytest.mark.parametrize("name,scale,batches", [
    ("layered_1m", 0.05, (1, 256)),
    ("powerlaw_10m", 0.08, (64,)),
    ("powerlaw_1m_nodes", 0.03, (64,)),
    ("layered_3m_fwd_bwd", 0.02, (256,)),
])
def test_configs_reduced_size(klay, name, scale, batches):
    for B in batches:
        c, p, spec = make_config(name, seed=1, scale=scale, batch=B)
        sem = tuple(REAL if s == "real" else LOG for s in spec["semirings"])
        stats = check_both(klay, c, p, backward=True, semirings=sem, what="%s B=%d" % (name, B), plain=True)
        print(name, B, stats)


# ------------------------------------------------------------------ full sizes, every batch column
def _oracle_columns(c, w32, semiring, dout, chunk=64, nthreads=16):
    """oracle values (and gradients for the adjoint seed dout) of every batch column, a chunk of columns at
    a time so that the oracle's per-column node arrays stay small"""
    from oracle import oracle
    refs, grads = [], []
    for a in range(0, w32.shape[0], chunk):
        w64 = w32[a:a + chunk].astype(np.float64)
        with np.errstate(all="ignore"):
            refs.append(oracle.forward(*c.arrays(), w64, semiring, nthreads=nthreads))
            if dout is not None:
                grads.append(oracle.backward(*c.arrays(), w64, semiring, dout[a:a + chunk].astype(np.float64),
                                             nthreads=nthreads))
    return np.concatenate(refs), (np.concatenate(grads) if grads else None)


@pytest.mark.parametrize("name,semiring", [
    ("layered_1m", REAL), ("layered_1m", LOG), ("powerlaw_10m", LOG), ("powerlaw_1m_nodes", LOG),
    ("layered_3m_fwd_bwd", LOG),
])
def test_configs_full_size_every_column(klay, name, semiring):
    """The workloads at full size in the launch configuration the benchmark times (same batch, same build
    options): every output and, with dout = 1, every gradient entry of every batch column against the
    oracle.  Log-semiring gradients are held to the plain bound 1e-4 max(1, |ref|)."""
    c, p, spec = make_config(name, seed=0)
    B = p.shape[0]
    assert B == {"layered_1m": 256, "powerlaw_10m": 64, "powerlaw_1m_nodes": 64, "layered_3m_fwd_bwd": 256}[name]
    w32 = as_inputs(p, semiring == LOG)
    dout = np.ones((B, c.roots.shape[0]), dtype=np.float32)
    k = build(klay, c)
    # the default layerization: padding-free up to layer A, which lies strictly inside the layered circuits (their
    # narrow top runs in the persistent kernels) and is the top layer of the power-law ones (no narrow fan-ins)
    A, L = k.info()["alias_top_layer"], k.num_layers
    assert (A == L and k.info()["tail_first_layer"] == 0) if name.startswith("powerlaw") else (0 < A < L and k.info()["tail_first_layer"] == A + 1)
    got, gd = gpu_eval(k, w32, semiring, dout)
    if semiring == LOG:
        ref, rd = _oracle_columns(c, w32, LOG, dout)
        e = assert_log_close(got, ref, name)
        ratio = assert_grad_plain(gd, rd, name + " grad, dout = 1")
        print("%s B=%d, all columns: max|dlog| %.2e (max|log ref| %.1f); gradient error %.3g x the plain bound, max|grad ref| %.2e"
              % (name, B, e, np.abs(ref[np.isfinite(ref)]).max(), ratio, np.abs(rd).max()))
    else:
        ref, _ = _oracle_columns(c, w32, REAL, None)
        print("%s B=%d real, all columns: max rel %.2e" % (name, B, assert_real_close(got, ref, name)))
        # the real-semiring gradient is a difference of products: bound with the cancellation term, sampled columns
        cols = np.array([0, B // 3, B // 2 + 1, B - 1])
        _, rdc = oracle_eval(c, w32[cols], REAL, dout[cols], nthreads=4, or_levels=k.num_layers // 2)
        print("%s real grad: %.3g x the bound" % (name, assert_grad_close(gd[cols], rdc, name + " real grad", real=True)))
    if name == "layered_1m":      # B = 1 latency case on the same circuit, both semirings
        got1, gd1 = gpu_eval(k, w32[:1], semiring, dout[:1])
        if semiring == LOG:
            assert_log_close(got1, ref[:1], name + " B=1")
            assert_grad_plain(gd1, rd[:1], name + " B=1 grad")
        else:
            assert_real_close(got1, ref[:1], name + " real B=1")
    k.close()


def test_large_batch_crosses_32_bit_element_indices(klay):
    """Maximum sizes: B = 6000 on the 1e6-node circuit puts 4.9e9 floats (19 GB) into the activation buffer, so
    the rows of its upper layers start beyond 2^32 elements, and the column-major buffers of the persistent
    kernels are longer than that in bytes.  Sampled batch columns (both ends, the middle, random ones) against
    the oracle, values and gradients; and columns with identical inputs must give bitwise identical outputs
    wherever they sit in the batch."""
    B = 6000
    c, p, _ = make_config("layered_1m", seed=3, batch=B)
    w32 = as_inputs(p, True)
    w32[B - 1] = w32[0]
    w32[B // 2 + 7] = w32[3]
    dout = np.ones((B, c.roots.shape[0]), dtype=np.float32)
    k = build(klay, c)
    assert k.info()["num_nodes"] * B > 2 ** 32
    got, gd = gpu_eval(k, w32, LOG, dout)
    k.close()
    assert np.array_equal(got[B - 1], got[0]) and np.array_equal(gd[B - 1], gd[0])
    assert np.array_equal(got[B // 2 + 7], got[3]) and np.array_equal(gd[B // 2 + 7], gd[3])
    cols = np.unique(np.concatenate([[0, 1, B // 2, B - 2, B - 1], np.random.default_rng(3).integers(0, B, 11)]))
    ref, rd = _oracle_columns(c, w32[cols], LOG, dout[cols])
    e = assert_log_close(got[cols], ref, "B=6000")
    ratio = assert_grad_plain(gd[cols], rd, "B=6000 grad, dout = 1")
    print("layered_1m B=%d, %d sampled columns: max|dlog| %.2e, gradient error %.3g x the plain bound" % (B, len(cols), e, ratio))


# ------------------------------------------------------------------ batch shapes (lane mappings, ragged tails)
@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 8, 9, 17, 31, 32, 33, 63, 64, 65, 100, 101, 128, 129, 255, 257, 300, 513])
def test_batch_sizes(klay, B):
    c = layered_random(4, num_vars=48, depth=8, num_gates=1500, fanin=("geom", 2.0), groups=2, num_roots=7)
    check_both(klay, c, leaf_probs(B, B, 48), what="B=%d" % B)


@pytest.mark.parametrize("B", [1, 2, 3, 4, 5, 8, 9, 16, 17, 31, 32])
def test_small_batches_with_the_lanes_equal_edges_kernel(klay, B):
    """the alternative kernel for B <= 32 (a wave takes 64 / B index entries per step, rows are reduced
    across the lanes with a segmented scan): same results, with and without split rows, both sweeps,
    every layer a launch of its own so that no layer bypasses it"""
    c = layered_random(4, num_vars=48, depth=8, num_gates=1500, fanin=("geom", 2.0), groups=2, num_roots=7)
    check_both(klay, c, leaf_probs(B, B, 48), what="edges B=%d" % B, small_batch_edges=True, no_tail=True)
    z = layered_random(2, num_vars=64, depth=6, num_gates=1200, fanin=("zipf", 1.3, 400), groups=1, num_roots=5)
    pz = leaf_probs(5, B, 64, ("beta", 0.5, 0.5))
    for heavy, seg in ((2, 1), (8, 4), (0, 0)):
        check_both(klay, z, pz, what="edges split B=%d" % B, small_batch_edges=True, no_tail=True, heavy_fan=heavy,
                   min_segment=seg)
    check_max(klay, z, pz, what="edges maxlog", small_batch_edges=True, no_tail=True, heavy_fan=3, min_segment=2)


# ------------------------------------------------------------------ split rows (high fan-in / fan-out)
@pytest.mark.parametrize("heavy,seg", [(2, 1), (3, 2), (8, 4), (64, 16)])
@pytest.mark.parametrize("B", [3, 64, 256])
def test_split_rows(klay, heavy, seg, B):
    c = layered_random(2, num_vars=64, depth=6, num_gates=1200, fanin=("zipf", 1.3, 400), groups=1, num_roots=5)
    k = build(klay, c, heavy_fan=heavy, min_segment=seg)
    assert k.info()["num_split_rows"] > 0
    k.close()
    check_both(klay, c, leaf_probs(5, B, 64, ("beta", 0.5, 0.5)), what="split", heavy_fan=heavy, min_segment=seg)


@pytest.mark.parametrize("B", [40, 64])
def test_main_rows_and_combine_rows_in_one_launch(klay, B):
    """32 < B <= 64 and layers too large for one generic launch: the segments of split rows run first, then
    one launch takes the main rows and the combine rows together; all three semirings, both sweeps, both
    layerizations"""
    c, p, _ = make_config("powerlaw_10m", seed=2, scale=0.08, batch=B)
    k = build(klay, c)
    k.set_profiling(True)
    gpu_eval(k, as_inputs(p, True), LOG, np.ones((B, c.roots.shape[0]), np.float32))
    prof = k.get_profile()
    assert prof["main_combine"]["launches"] >= 1 and prof["main_combine"]["ms"] > 0
    k.close()
    check_both(klay, c, p, semirings=(LOG,), what="main+combine B=%d" % B)
    check_both(klay, c, p, semirings=(LOG,), what="main+combine, chains B=%d" % B, unary_chains=True)
    check_max(klay, c, p, what="main+combine maxlog B=%d" % B)
    # the real semiring (its values leave the fp32 range on the power-law circuit): a layered circuit whose rows
    # are split from 8 entries on
    c, p, _ = make_config("layered_1m", seed=2, scale=1.0, batch=B)
    k = build(klay, c, heavy_fan=8, min_segment=4)
    k.set_profiling(True)
    gpu_eval(k, as_inputs(p, False), REAL, np.ones((B, c.roots.shape[0]), np.float32))
    assert k.get_profile()["main_combine"]["launches"] >= 8
    k.close()
    check_both(klay, c, p, what="main+combine, layered B=%d" % B, heavy_fan=8, min_segment=4)


@pytest.mark.parametrize("B", [100, 256])
def test_fused_and_rows_forward_only_and_followed_by_backward(klay, B):
    """B > 64, log-domain semirings: a forward pass leaves out the AND rows that the OR rows above evaluate from
    their children (fused plans); klay_backward evaluates them first when it follows such a pass, and a handle
    that has seen a forward / backward pair writes every value in its next forward pass.  Every output of every
    call order against the oracle and against a handle built without fusion."""
    c, p, _ = make_config("layered_1m", seed=4, scale=0.3, batch=B)
    w32 = as_inputs(p, True)
    rng = np.random.default_rng(4)
    dout = rng.normal(size=(B, c.roots.shape[0])).astype(np.float32)
    k = build(klay, c, tail_rows_cap=1500)
    plain = build(klay, c, tail_rows_cap=1500, no_fusion=True)
    info = k.info()
    assert info["num_fused_rows"] > 1000 and 0 < info["alias_top_layer"] < k.num_layers
    assert plain.info()["num_fused_rows"] == 0
    ref, rd = oracle_eval(c, w32, LOG, dout, or_levels=k.num_layers // 2)
    want, wd = gpu_eval(plain, w32, LOG, dout)
    k.set_profiling(True)

    def fused_launches():
        return k.get_profile()["fwd_or_fused"]["launches"]

    a, _ = gpu_eval(k, w32, LOG)                    # forward only: fused
    assert fused_launches() > 0
    b, gb = gpu_eval(k, w32, LOG, dout)             # fused again, then the reverse sweep fills in the missing values
    assert fused_launches() > 0
    e, ge = gpu_eval(k, w32, LOG, dout)             # a backward pass followed the last forward pass: every value written
    assert fused_launches() == 0
    f, _ = gpu_eval(k, w32, LOG)                    # still in the training loop's mode
    assert fused_launches() == 0
    h, _ = gpu_eval(k, w32, LOG)                    # no backward pass followed: fused again
    assert fused_launches() > 0
    for got in (a, b, e, f, h):
        assert_log_close(got, ref, "fused forward B=%d" % B)
        np.testing.assert_allclose(got, want, rtol=0, atol=2e-5)
    for gd in (gb, ge):
        assert_grad_close(gd, rd, "gradient after a fused forward pass B=%d" % B)
        np.testing.assert_allclose(gd, wd, rtol=1e-4, atol=1e-5)
    m, _ = gpu_eval(k, w32, MAXLOG)
    assert fused_launches() > 0
    refm, _ = oracle_eval(c, w32, MAXLOG)
    assert_log_close(m, refm, "fused forward, (max, +) B=%d" % B)
    # the real semiring: products within the groups, and the reverse sweep after a fused pass
    doutr = np.ones((B, c.roots.shape[0]), dtype=np.float32)
    r, gr = gpu_eval(k, as_inputs(p, False), REAL, doutr)
    assert fused_launches() > 0
    refr, rdr = oracle_eval(c, as_inputs(p, False), REAL, doutr, or_levels=k.num_layers // 2)
    assert_real_close(r, refr, "fused forward, real B=%d" % B)
    assert_grad_close(gr, rdr, "real gradient after a fused forward pass B=%d" % B, real=True)
    r2, gr2 = gpu_eval(k, as_inputs(p, False), REAL, doutr)
    assert fused_launches() == 0
    np.testing.assert_allclose(r2, r, rtol=1e-6, atol=0)
    assert_grad_close(gr2, rdr, "real gradient in the loop's mode B=%d" % B, real=True)
    # batches of 64 columns or fewer run the ordinary plans
    s64, _ = gpu_eval(k, w32[:64], LOG)
    assert fused_launches() == 0
    assert_log_close(s64, ref[:64], "B=64 after fused")
    k.close(); plain.close()


def test_very_high_fan_in_and_gate_with_magnitude_aware_bound(klay):
    """one AND and one OR over 10^4 literals: exercises the split path at the fan-in cap; |log| of the
    AND reaches ~10^4, where fp32 cannot hold 1e-4 absolute, so the bound scales with sum |x_j| / 64"""
    V = 10_000
    b = CircuitBuilder(V)
    leaves = [b.lit(v, v % 3 != 0) for v in range(V)]
    c = b.finish([b.and_(*leaves), b.or_(*leaves)])
    p = leaf_probs(0, 64, V, ("uniform", 0.2, 1.0))
    w32 = as_inputs(p, True)
    k = build(klay, c)
    assert k.info()["max_fan_in"] == V and k.info()["num_split_rows"] >= 2
    got, _ = gpu_eval(k, w32, LOG)
    ref, _ = oracle_eval(c, w32, LOG)
    assert_log_close(got[:, 1], ref[:, 1], "OR over 1e4")
    bound = 1e-4 * np.maximum(1.0, np.abs(ref[:, 0]) / 64)
    assert np.all(np.abs(got[:, 0] - ref[:, 0]) <= bound)


# ------------------------------------------------------------------ degenerate inputs
def test_zero_one_probabilities_and_constants(klay):
    b = CircuitBuilder(3)
    x, nx, y, ny, z = b.lit(0), b.lit(0, False), b.lit(1), b.lit(1, False), b.lit(2)
    root = b.or_(b.and_(x, y), b.and_(nx, ny, z))
    dead = b.or_(b.and_(x, ny), b.and_(nx, y))
    t, f = b.true(), b.false()
    c = b.finish([root, dead, t, f, b.and_(t, z), b.or_(f, b.and_(z, x)), z, nx])
    p = np.array([[1.0, 1.0, 0.3], [0.0, 0.0, 0.0], [0.0, 1.0, 0.5], [0.4, 0.6, 0.2]])
    k = build(klay, c)
    with np.errstate(divide="ignore"):
        w32 = as_inputs(p, True)
    got, _ = gpu_eval(k, w32, LOG)
    ref, _ = oracle_eval(c, w32, LOG)
    assert_log_close(got, ref, "zero/one log")
    gotr, _ = gpu_eval(k, as_inputs(p, False), REAL)
    refr, _ = oracle_eval(c, as_inputs(p, False), REAL)
    assert_real_close(gotr, refr, "zero/one real")
    # gradients on the rows without infinite derivatives
    dout = np.zeros((4, 8), dtype=np.float32); dout[:, 0] = 1.0; dout[:, 4] = -2.0
    _, gd = gpu_eval(k, w32, LOG, dout)
    _, rd = oracle_eval(c, w32, LOG, dout)
    assert_grad_close(gd[3:], rd[3:], "grad")
    assert not np.isnan(gd).any()
    k.close()


def test_leaf_roots_and_repeated_roots(klay):
    b = CircuitBuilder(2)
    x, ny = b.lit(0), b.lit(1, False)
    c = b.finish([ny, x, ny])
    check_both(klay, c, leaf_probs(0, 5, 2, ("uniform", 0.1, 0.9)), what="leaf roots")
    b = CircuitBuilder(3)
    a = b.and_(b.lit(0), b.lit(1))
    o = b.or_(a, b.and_(b.lit(0, False), b.lit(2)))
    c = b.finish([o, a, b.lit(2), o, a])
    check_both(klay, c, leaf_probs(1, 6, 3, ("uniform", 0.1, 0.9)), what="mixed-height roots")


def test_tautology_is_one(klay):
    c = tautology(0, 40, width=5)
    p = leaf_probs(0, 16, 40, ("beta", 0.5, 0.5))
    k = build(klay, c)
    got, _ = gpu_eval(k, as_inputs(p, True), LOG)
    assert np.abs(got).max() <= 1e-4
    k.close()


def test_node_order_does_not_change_results(klay):
    c = layered_random(9, num_vars=32, depth=10, num_gates=3000, fanin=("geom", 2.0), groups=2, num_roots=9)
    p = leaf_probs(9, 40, 32)
    w32 = as_inputs(p, True)
    outs = []
    for kw in ({}, {"no_reorder": True}):
        k = build(klay, c, **kw)
        outs.append(gpu_eval(k, w32, LOG, np.ones((40, 9), np.float32)))
        k.close()
    ref, rd = oracle_eval(c, w32, LOG, np.ones((40, 9), np.float32))
    for got, gd in outs:
        assert_log_close(got, ref)
        assert_grad_close(gd, rd)


def test_runs_are_bitwise_reproducible_and_workspace_can_be_callers(klay):
    import torch
    c, p, _ = make_config("layered_100k", seed=3, scale=0.2, batch=96)
    w32 = as_inputs(p, True)
    d = np.ones((96, c.roots.shape[0]), np.float32)
    k = build(klay, c)
    a = gpu_eval(k, w32, LOG, d)
    b = gpu_eval(k, w32, LOG, d)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    ws = torch.empty(k.workspace_bytes(96, True) // 4, dtype=torch.float32, device="cuda")
    k.set_workspace(ws)
    e = gpu_eval(k, w32, LOG, d)
    np.testing.assert_array_equal(a[0], e[0])
    np.testing.assert_array_equal(a[1], e[1])
    small = torch.empty(1024, dtype=torch.float32, device="cuda")
    k.set_workspace(small)
    with pytest.raises(klay.KlayError) as err:
        gpu_eval(k, w32, LOG)
    assert err.value.status == 3
    k.set_workspace(None)
    k.close()


def test_call_order_errors(klay):
    import torch
    c, p, _ = make_config("tiny_ddnnf", seed=0)
    k = build(klay, c)
    d = torch.ones((4, 1), device="cuda")
    g = torch.empty((4, 12), device="cuda")
    with pytest.raises(klay.KlayError) as e:
        klay.klay_backward(k._h, d.data_ptr(), g.data_ptr(), 0)
    assert e.value.status == 5
    k.close()
    ka = build(klay, c, unary_chains=True)
    ka.forward_f64(torch.from_numpy(as_inputs(p, True).astype(np.float64)).cuda(), MAXLOG)
    with pytest.raises(klay.KlayError) as e:
        ka.backward_f64(d.double())
    assert e.value.status == 1          # (max, +) is not differentiated, in double precision either
    ka.close()


def test_profile_reports_kernel_classes(klay):
    c, p, _ = make_config("layered_100k", seed=0, scale=0.2, batch=64)
    k = build(klay, c, no_tail=True)
    k.set_profiling(True)
    gpu_eval(k, as_inputs(p, True), LOG, np.ones((64, c.roots.shape[0]), np.float32))
    prof = k.get_profile()
    assert prof["fwd_lse"]["launches"] >= 10 and prof["fwd_lse"]["ms"] > 0
    assert prof["bwd_softmax_one"]["launches"] >= 10 and prof["bwd_softmax_one"]["alg_bytes"] > 0
    assert prof["bwd_sum_enc"]["launches"] >= 9 and prof["bwd_softmax"]["launches"] == 0
    k.set_profiling(False)
    k.close()
    ka = build(klay, c, no_tail=True, unary_chains=True)
    ka.set_profiling(True)
    gpu_eval(ka, as_inputs(p, True), LOG, np.ones((64, c.roots.shape[0]), np.float32))
    prof = ka.get_profile()
    assert prof["bwd_softmax_one"]["launches"] >= 10 and prof["bwd_sum_enc"]["launches"] >= 9
    assert prof["bwd_softmax"]["launches"] == 0
    ka.close()


@pytest.mark.parametrize("B", [1, 3, 8, 37, 256, 300, 700, 1100, 2100])
def test_persistent_top_kernel_matches_per_layer_launches(klay, B):
    """the narrow top layers run in one LDS-resident kernel (1, 2, 4 or 8 batch columns per workgroup as
    the batch grows past 256, 512, 1024); with no_tail every layer is its own launch"""
    c, p, _ = make_config("layered_100k", seed=5, scale=0.3, batch=B)
    w32 = as_inputs(p, True)
    d = np.random.default_rng(5).normal(size=(B, c.roots.shape[0])).astype(np.float32)
    k_tail, k_flat = build(klay, c), build(klay, c, no_tail=True)
    assert k_tail.info()["tail_first_layer"] > 0 and k_flat.info()["tail_first_layer"] == 0
    k_tail.set_profiling(True)
    a = gpu_eval(k_tail, w32, LOG, d)
    prof = k_tail.get_profile()
    assert prof["tail_fwd"]["launches"] == 1 and prof["tail_bwd"]["launches"] == 1
    k_tail.set_profiling(False)
    b = gpu_eval(k_flat, w32, LOG, d)
    ref, rd = oracle_eval(c, w32, LOG, d, or_levels=k_tail.num_layers // 2)
    for got, gd in (a, b):
        assert_log_close(got, ref, "tail")
        assert_grad_close(gd, rd, "tail grad")
    np.testing.assert_allclose(a[0], b[0], rtol=0, atol=2e-5)
    ar, _ = gpu_eval(k_tail, as_inputs(p, False), REAL)
    refr, _ = oracle_eval(c, as_inputs(p, False), REAL)
    assert_real_close(ar, refr, "tail real")
    k_tail.close(); k_flat.close()


# ------------------------------------------------------------------ the paper's layerization throughout (unary_chains), and the boundary
# ------------------------------------------------------------------ between the padding-free lower part and the top at various layers
@pytest.mark.parametrize("name,scale,B", [("tiny_ddnnf", 1.0, 4), ("layered_100k", 0.3, 128), ("layered_1m", 0.05, 1),
                                          ("powerlaw_10m", 0.08, 64), ("layered_3m_fwd_bwd", 0.02, 256)])
def test_unary_chains_mode_matches_the_oracle(klay, name, scale, B):
    c, p, spec = make_config(name, seed=2, scale=scale, batch=B)
    sem = tuple(REAL if s == "real" else LOG for s in spec["semirings"])      # real underflows fp32 on powerlaw
    tops = set()
    for mode in layer_modes(klay, c):
        kh = klay.Circuit(*c.arrays(), device=-1, **mode)
        tops.add((kh.info()["alias_top_layer"], kh.num_layers))
        kh.close()
        print(name, mode, check_both(klay, c, p, semirings=sem, what="%s %s" % (name, mode), **mode))
    # the boundary was seen at layer 0, at the top and strictly in between
    assert any(a == 0 for a, L in tops) and any(a == L for a, L in tops), tops
    if name.startswith("layered"):            # (the power-law circuit has wide fan-ins at the top: no persistent kernels)
        assert any(0 < a < L for a, L in tops), tops


def test_unary_chains_mode_on_odd_shapes(klay, golden):
    for f, nv in (("fig1b_ddnnf.txt", 4), ("fig3_multiroot.txt", 5), ("appD_mnist_add.txt", 2)):
        for mode in layer_modes(klay, golden(f)) + [dict(tail_rows_cap=1), dict(tail_rows_cap=2)]:
            check_both(klay, golden(f), leaf_probs(1, 5, nv, ("uniform", 0.05, 0.95)), what="%s %s" % (f, mode), **mode)
    b = CircuitBuilder(3)
    x, y, z = b.lit(0), b.lit(1), b.lit(2)
    o = b.or_(x, y)                       # OR directly over leaves: lifted to layer 2, layer 1 stays empty
    a = b.and_(o, z)
    c = b.finish([a, o, x, a, b.lit(2, False)])
    for mode in layer_modes(klay, c) + [dict(tail_rows_cap=1), dict(tail_rows_cap=2), dict(tail_rows_cap=3)]:
        check_both(klay, c, leaf_probs(2, 9, 3, ("uniform", 0.05, 0.95)), what="lifted %s" % mode, **mode)
    c = layered_random(2, num_vars=64, depth=6, num_gates=1200, fanin=("zipf", 1.3, 400), groups=1, num_roots=5)
    for mode in layer_modes(klay, c):
        check_both(klay, c, leaf_probs(5, 70, 64, ("beta", 0.5, 0.5)), what="split %s" % mode, heavy_fan=4, min_segment=2,
                   **mode)


def test_unary_chains_full_size_every_column(klay):
    c, p, spec = make_config("layered_3m_fwd_bwd", seed=0)
    B = p.shape[0]
    w32 = as_inputs(p, True)
    dout = np.ones((B, c.roots.shape[0]), dtype=np.float32)
    k = build(klay, c, unary_chains=True)
    info = k.info()
    assert info["alias_top_layer"] == 0 and info["num_pad_nodes"] > 10 ** 6
    got, gd = gpu_eval(k, w32, LOG, dout)
    ref, rd = _oracle_columns(c, w32, LOG, dout)
    print("unary chains, full size, all columns: max|dlog| %.2e, gradient error %.3g x the plain bound" % (
        assert_log_close(got, ref), assert_grad_plain(gd, rd, "chains grad, dout = 1")))
    k.close()


def test_forward_backward_can_be_captured_in_a_hip_graph(klay):
    """klay_forward / klay_backward only enqueue kernels; a captured step must replay to the eager
    result several times, with eager work and synchronisation in between"""
    import torch
    c, p, _ = make_config("layered_100k", seed=6, scale=0.5, batch=96)
    k = build(klay, c)
    R, V = c.roots.shape[0], c.num_vars
    w = torch.from_numpy(as_inputs(p, True)).cuda()
    out = torch.empty((96, R), device="cuda")
    dout = torch.ones((96, R), device="cuda")
    dleaf = torch.empty((96, V), device="cuda")
    k.forward(w, LOG, out=out)
    k.backward(dout, dleaf=dleaf)
    torch.cuda.synchronize()
    ref_out, ref_grad = out.clone(), dleaf.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            k.forward(w, LOG, out=out, stream=side)
            k.backward(dout, dleaf=dleaf, stream=side)
    torch.cuda.synchronize()
    for i in range(4):
        out.fill_(float("nan")); dleaf.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(dleaf, ref_grad), "replay %d differs" % i
        # eager work between replays, on other inputs, must not disturb the next replay
        w2 = (w * 1.5).contiguous()
        k.forward(w2, LOG)
        torch.cuda.synchronize()
    k.close()


def test_real_semiring_gradient_with_zero_children(klay):
    """product layers with children that are exactly zero: the adjoint of the zero child is the
    product of the others, of everyone else zero (two zeros: all zero)"""
    b = CircuitBuilder(4)
    x = [b.lit(v) for v in range(4)]
    root = b.or_(b.and_(x[0], x[1], x[2]), b.and_(b.lit(0, False), x[3]), b.and_(x[1], x[3]))
    c = b.finish([root, b.and_(x[0], x[1], x[2], x[3])])
    p = np.array([[0.0, 0.5, 0.25, 0.8], [0.0, 0.0, 0.3, 0.6], [1.0, 0.2, 0.0, 0.0], [0.3, 0.6, 0.9, 0.1]])
    k = build(klay, c)
    dout = np.array([[1.0, 2.0]] * 4, dtype=np.float32)
    got, gd = gpu_eval(k, as_inputs(p, False), REAL, dout)
    ref, rd = oracle_eval(c, as_inputs(p, False), REAL, dout, or_levels=1)
    assert_real_close(got, ref)
    np.testing.assert_allclose(gd, np.asarray(rd), rtol=1e-5, atol=1e-7)
    k.close()


# ------------------------------------------------------------------ shapes at the edges of the launch logic
def test_deep_narrow_circuit_runs_mostly_in_the_persistent_kernel(klay):
    """300 layers of at most a few dozen nodes: almost every layer is a tail layer"""
    c = layered_random(11, num_vars=300, depth=300, num_gates=6000, fanin=("geom", 1.0), groups=1, num_roots=3)
    k = build(klay, c)
    assert k.num_layers == 300 and 0 < k.info()["tail_first_layer"] <= 2
    k.close()
    check_both(klay, c, leaf_probs(11, 33, 300, ("uniform", 0.2, 1.0)), semirings=(LOG,), what="deep")


def test_one_very_wide_layer(klay):
    """a single AND layer of 300k gates over two literals each, one OR root over all of them"""
    V = 2000
    rng = np.random.default_rng(0)
    n = 300_000
    a, b_ = rng.integers(0, V, size=n), rng.integers(0, V, size=n)
    b_ = np.where(a == b_, (b_ + 1) % V, b_)
    sa, sb = rng.integers(0, 2, size=n), rng.integers(0, 2, size=n)
    node_type = np.concatenate([np.zeros(2 * V, np.uint8), np.full(n, 1, np.uint8), np.array([2], np.uint8)])
    node_lit = np.zeros(2 * V + n + 1, np.int32)
    node_lit[0:2 * V:2] = np.arange(1, V + 1)
    node_lit[1:2 * V:2] = -np.arange(1, V + 1)
    child_ptr = np.concatenate([np.zeros(2 * V + 1, np.int64), 2 * np.arange(1, n + 1), [2 * n + n]]).astype(np.int64)
    child_idx = np.concatenate([np.stack([2 * a + sa, 2 * b_ + sb], 1).ravel(), 2 * V + np.arange(n)]).astype(np.int32)
    from klay_synth import Circuit as Dag
    c = Dag(V, node_type, node_lit, child_ptr, child_idx, np.array([2 * V + n], np.int32))
    p = leaf_probs(1, 48, V, ("uniform", 0.0, 1.0))
    w32 = as_inputs(p, True)
    k = build(klay, c)
    assert k.info()["max_layer_nodes"] > 100_000
    d = np.ones((48, 1), np.float32)
    got, gd = gpu_eval(k, w32, LOG, d)
    ref, rd = oracle_eval(c, w32, LOG, d, or_levels=1)
    assert_log_close(got, ref, "wide")
    assert_grad_close(gd, rd, "wide grad")
    k.close()


def test_constant_only_circuit_and_unused_variables(klay):
    b = CircuitBuilder(3)
    t, f = b.true(), b.false()
    c = b.finish([b.or_(t, f), b.and_(t, b.or_(f, t)), f])
    p = leaf_probs(0, 7, 3)
    k = build(klay, c)
    got, gd = gpu_eval(k, as_inputs(p, True), LOG, np.ones((7, 3), np.float32))
    ref, rd = oracle_eval(c, as_inputs(p, True), LOG, np.ones((7, 3), np.float32), or_levels=2)
    assert_log_close(got, ref, "constants")
    np.testing.assert_array_equal(gd, 0.0)           # no variable is used: every entry written as 0
    k.close()


def test_changing_batch_size_and_two_handles_on_one_stream(klay):
    c1 = layered_random(21, num_vars=40, depth=8, num_gates=2000, fanin=("geom", 2.0), groups=2, num_roots=6)
    c2 = layered_random(22, num_vars=40, depth=6, num_gates=900, fanin=("geom", 1.5), groups=1, num_roots=2)
    k1, k2 = build(klay, c1), build(klay, c2)
    for B in (300, 7, 64, 1, 129):
        p = leaf_probs(B, B, 40)
        w32 = as_inputs(p, True)
        d1 = np.ones((B, 6), np.float32); d2 = np.ones((B, 2), np.float32)
        # interleave the two handles: each keeps its own activations
        import torch
        w = torch.from_numpy(w32).cuda()
        o1 = k1.forward(w, LOG); o2 = k2.forward(w, LOG)
        g1 = k1.backward(torch.from_numpy(d1).cuda()); g2 = k2.backward(torch.from_numpy(d2).cuda())
        torch.cuda.synchronize()
        r1, rg1 = oracle_eval(c1, w32, LOG, d1, or_levels=4)
        r2, rg2 = oracle_eval(c2, w32, LOG, d2, or_levels=3)
        assert_log_close(o1.cpu().numpy(), r1); assert_log_close(o2.cpu().numpy(), r2)
        assert_grad_close(g1.cpu().numpy(), rg1); assert_grad_close(g2.cpu().numpy(), rg2)
    k1.close(); k2.close()


# ------------------------------------------------------------------ circuits added one at a time (Section 3.2)
def test_builder_circuits_share_nodes_and_keep_their_values(klay):
    """three circuits over the same variables, one of them added twice, built as one multi-rooted
    circuit: every root block equals the oracle on its own circuit, the gradient is the sum of the
    circuits' gradients, and the repeated circuit adds no rows"""
    from tests.gpu_util import GradRef
    V, B = 96, 70
    parts = [layered_random(seed=s, num_vars=V, depth=d, num_gates=g, fanin=("geom", 2.0), groups=1, num_roots=r)
             for s, d, g, r in ((11, 8, 3000, 3), (12, 14, 5000, 1), (13, 5, 800, 2))]
    bld = klay.Builder(V)
    first = [bld.add(*c.arrays()[1:]) for c in parts]
    assert first == [0, 3, 4]
    k3 = bld.finish(device=0)
    assert bld.add(*parts[0].arrays()[1:]) == 6
    k = bld.finish(device=0)
    assert k.info()["num_nodes"] == k3.info()["num_nodes"] and k.num_roots == 9
    p = leaf_probs(5, B, V, ("uniform", 0.0, 1.0))
    rng = np.random.default_rng(5)
    dout = rng.normal(size=(B, 9)).astype(np.float32)
    levels = k.num_layers // 2
    for s in (LOG, REAL):
        w32 = as_inputs(p, s == LOG)
        got, gd = gpu_eval(k, w32, s, dout)
        grad = np.zeros((B, V)); mass = np.zeros((B, V)); rel = 0.0
        for c, col in zip(parts + [parts[0]], first + [6]):
            r = c.roots.shape[0]
            ref, rd = oracle_eval(c, w32, s, dout[:, col:col + r], or_levels=levels)
            (assert_log_close if s == LOG else assert_real_close)(got[:, col:col + r], ref, "builder block %d" % col)
            grad += np.asarray(rd); mass += rd.mass; rel = max(rel, rd.rel)
        assert_grad_close(gd, GradRef(grad, mass, rel), "builder grad", real=(s == REAL))
    k.close(); k3.close()


# ------------------------------------------------------------------ (max, +) semiring, forward only
MAXLOG = 2


def check_max(klay, c, p, what="", **kw):
    k = build(klay, c, **kw)
    with np.errstate(divide="ignore"):
        w32 = as_inputs(p, True)
    got, _ = gpu_eval(k, w32, MAXLOG)
    ref, _ = oracle_eval(c, w32, MAXLOG)
    e = assert_log_close(got, ref, what + " maxlog")
    k.close()
    return e


def test_maxlog_worked_examples_and_small_batches(klay, golden):
    for name, nv in (("fig1b_ddnnf.txt", 4), ("fig3_multiroot.txt", 5), ("appD_mnist_add.txt", 2)):
        for B in (1, 5, 70):
            check_max(klay, golden(name), leaf_probs(B, B, nv, ("uniform", 0.01, 0.99)), what=name)
    c = layered_random(4, num_vars=48, depth=8, num_gates=1500, fanin=("geom", 2.0), groups=2, num_roots=7)
    for B in (1, 3, 17, 32, 33, 64, 65, 128, 129, 257, 513):
        check_max(klay, c, leaf_probs(B, B, 48), what="B=%d" % B)


@pytest.mark.parametrize("name,scale,B", [("layered_1m", 0.05, 256), ("powerlaw_10m", 0.08, 64),
                                           ("layered_3m_fwd_bwd", 0.02, 256), ("layered_100k", 1.0, 128)])
def test_maxlog_configs(klay, name, scale, B):
    c, p, spec = make_config(name, seed=1, scale=scale, batch=B)
    print(name, "maxlog max|dlog| %.2e" % check_max(klay, c, p, what=name))
    for mode in layer_modes(klay, c):
        check_max(klay, c, p, what="%s %s" % (name, mode), **mode)


@pytest.mark.parametrize("B", [3, 64, 256])
def test_maxlog_split_rows_and_impossible_branches(klay, B):
    c = layered_random(2, num_vars=64, depth=6, num_gates=1200, fanin=("zipf", 1.3, 400), groups=1, num_roots=5)
    p = leaf_probs(5, B, 64, ("beta", 0.5, 0.5))
    p[:, ::7] = 0.0
    p[:, 3::11] = 1.0
    for heavy, seg in ((2, 1), (8, 4), (64, 16)):
        check_max(klay, c, p, what="split", heavy_fan=heavy, min_segment=seg)


def test_maxlog_is_not_differentiated_and_leaves_the_handle_usable(klay):
    import torch
    c = layered_random(9, num_vars=32, depth=10, num_gates=3000, fanin=("geom", 2.0), groups=2, num_roots=9)
    p = leaf_probs(1, 40, 32)
    w32 = as_inputs(p, True)
    k = build(klay, c)
    got, _ = gpu_eval(k, w32, MAXLOG)
    with pytest.raises(klay.KlayError) as e:
        k.backward(torch.ones((40, 9), dtype=torch.float32, device="cuda"))
    assert e.value.status == 1
    dout = np.ones((40, 9), dtype=np.float32)
    got2, gd = gpu_eval(k, w32, LOG, dout)
    ref2, rd = oracle_eval(c, w32, LOG, dout, or_levels=k.num_layers // 2)
    assert_log_close(got2, ref2, "log after maxlog")
    assert_grad_close(gd, rd, "grad after maxlog")
    assert np.all(got <= got2 + 1e-4)
    k.close()


# ------------------------------------------------------------------ the circuit as a torch layer
def test_circuit_layer_backpropagates_into_a_network(klay):
    """autograd through the layer gives the oracle's gradient, chains into upstream parameters, and
    refuses to differentiate a forward pass whose activations have been overwritten"""
    import torch
    c = layered_random(9, num_vars=32, depth=10, num_gates=3000, fanin=("geom", 2.0), groups=2, num_roots=9)
    k = build(klay, c)
    layer = klay.CircuitLayer(k, klay.KLAY_LOG)
    B = 70
    torch.manual_seed(0)
    logits = torch.randn(B, 32, device="cuda", requires_grad=True)
    w = torch.nn.functional.logsigmoid(logits)                 # log p of every variable
    out = layer(w)
    coef = torch.linspace(-1.0, 1.0, 9, device="cuda")
    (out * coef).sum().backward()
    w32 = w.detach().cpu().numpy()
    dout = np.tile(coef.cpu().numpy(), (B, 1)).astype(np.float32)
    ref, rd = oracle_eval(c, w32, LOG, dout, or_levels=k.num_layers // 2)
    assert_log_close(out.detach().cpu().numpy(), ref, "layer")
    # chain rule through logsigmoid: d/dlogit = dleaf * (1 - p)
    p = np.exp(w32.astype(np.float64))
    from tests.gpu_util import GradRef
    want = GradRef(np.asarray(rd) * (1 - p), rd.mass * (1 - p), rd.rel)
    assert_grad_close(logits.grad.cpu().numpy(), want, "layer grad")
    # a few optimiser steps raise the log-probability of root 0
    net = torch.nn.Linear(4, 32).cuda()
    opt = torch.optim.SGD(net.parameters(), lr=0.05)
    x = torch.randn(B, 4, device="cuda")
    losses = []
    for _ in range(5):
        opt.zero_grad()
        loss = -layer(torch.nn.functional.logsigmoid(net(x)))[:, 0].mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < losses[0]
    # stale graph
    o1 = layer(torch.nn.functional.logsigmoid(logits))
    with torch.no_grad():
        layer(w.detach())
    with pytest.raises(RuntimeError):
        o1.sum().backward()
    with pytest.raises(RuntimeError):
        klay.CircuitLayer(k, klay.KLAY_MAXLOG)(torch.nn.functional.logsigmoid(logits))
    with torch.no_grad():
        m = klay.CircuitLayer(k, klay.KLAY_MAXLOG)(w.detach())
    assert torch.all(m <= out.detach() + 1e-4)
    k.close()


# ------------------------------------------------------------------ weights of their own for the negated literals
def _lits_case(klay, c, B, seed, semirings=(REAL, LOG), **kw):
    import torch
    from tests.gpu_util import GradRef, U32
    from oracle import oracle
    rng = np.random.default_rng(seed)
    V, R = c.num_vars, c.roots.shape[0]
    wp = rng.uniform(0.2, 1.0, size=(B, V)).astype(np.float32)
    wn = rng.uniform(0.2, 1.0, size=(B, V)).astype(np.float32)
    dout = rng.normal(size=(B, R)).astype(np.float32)
    k = build(klay, c, **kw)
    levels = k.num_layers // 2
    for s in semirings:
        a, b = (wp, wn) if s == REAL else (np.log(wp), np.log(wn))
        ta, tb, td = (torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in (a, b, dout))
        out = k.forward(ta, s, neg_weights=tb)
        can_bwd = True
        if can_bwd:
            dp, dn = (t.cpu().numpy() for t in k.backward(td))
        got = out.cpu().numpy()
        a64, b64, d64 = a.astype(np.float64), b.astype(np.float64), dout.astype(np.float64)
        with np.errstate(all="ignore"):
            ref, vals = oracle.forward(*c.arrays(), a64, s, nthreads=8, return_node_values=True, neg_weights=b64)
        (assert_log_close if s == LOG else assert_real_close)(got, ref, "lits")
        if not can_bwd:
            continue
        with np.errstate(all="ignore"):
            rp, rn = oracle.backward(*c.arrays(), a64, s, d64, nthreads=8, neg_weights=b64)
            mp, mn = oracle.backward(*c.arrays(), a64, s, d64, nthreads=8, neg_weights=b64, path_mass=True)
        fin = np.isfinite(vals)
        maxabs = float(np.abs(vals[fin]).max()) if fin.any() else 0.0
        rel = 64 * U32 + 4 * U32 * levels * maxabs if s == LOG else (64 + 16 * levels) * U32
        assert_grad_close(dp, GradRef(rp, mp, rel), "lits dpos", real=(s == REAL))
        assert_grad_close(dn, GradRef(rn, mn, rel), "lits dneg", real=(s == REAL))
    # (max, +) forward with the same weights
    ta, tb = (torch.from_numpy(np.ascontiguousarray(np.log(x))).cuda() for x in (wp, wn))
    got = k.forward(ta, MAXLOG, neg_weights=tb).cpu().numpy()
    ref = oracle.forward(*c.arrays(), np.log(wp).astype(np.float64), oracle.MAXLOG, nthreads=8,
                         neg_weights=np.log(wn).astype(np.float64))
    assert_log_close(got, ref, "lits maxlog")
    k.close()


def test_negative_literal_weights(klay, golden):
    for B in (1, 5, 70):
        _lits_case(klay, golden("fig1b_ddnnf.txt"), B, seed=B)
    c = layered_random(9, num_vars=32, depth=10, num_gates=3000, fanin=("geom", 2.0), groups=2, num_roots=9)
    for B in (3, 70, 300):
        _lits_case(klay, c, B, seed=10 + B)
    _lits_case(klay, c, 130, seed=1, no_tail=True)
    _lits_case(klay, c, 130, seed=2, unary_chains=True)
    _lits_case(klay, c, 130, seed=3, tail_rows_cap=250)
    _lits_case(klay, c, 70, seed=4, tail_rows_cap=100, no_merge=True)


def test_negative_literal_weights_default_and_call_pairing(klay):
    """1 - p passed explicitly gives the default's values; each forward flavour has its own backward"""
    import torch
    c = layered_random(9, num_vars=32, depth=10, num_gates=3000, fanin=("geom", 2.0), groups=2, num_roots=9)
    k = build(klay, c)
    p = torch.rand(40, 32, device="cuda") * 0.8 + 0.1
    a = k.forward(p, REAL)
    b = k.forward(p, REAL, neg_weights=(1 - p).contiguous())
    assert torch.equal(a, b)
    d = torch.ones(40, 9, device="cuda")
    with pytest.raises(klay.KlayError) as e:
        klay.klay_backward(k._h, d.data_ptr(), torch.empty(40, 32, device="cuda").data_ptr())
    assert e.value.status == 5
    dp, dn = k.backward(d)
    k.forward(p, REAL)
    g = k.backward(d)
    torch.testing.assert_close(g, dp - dn, rtol=1e-4, atol=1e-6)
    with pytest.raises(klay.KlayError) as e:
        klay.klay_backward_lits(k._h, d.data_ptr(), dp.data_ptr(), dn.data_ptr())
    assert e.value.status == 5
    # the torch layer differentiates both arrays
    layer = klay.CircuitLayer(k, klay.KLAY_LOG)
    lp = torch.log(p).requires_grad_(True)
    ln = torch.log(1 - p).requires_grad_(True)
    layer(lp, ln).sum().backward()
    k.forward(torch.log(p), LOG, neg_weights=torch.log(1 - p))
    rp, rn = k.backward(d)
    assert torch.equal(lp.grad, rp) and torch.equal(ln.grad, rn)
    k.close()


# ------------------------------------------------------------------ double-precision evaluation
def _f64_case(klay, c, p, what, backward=True, neg=False, **kw):
    import torch
    from oracle import oracle
    k = build(klay, c, **kw)
    rng = np.random.default_rng(17)
    B, R = p.shape[0], c.roots.shape[0]
    dout = rng.normal(size=(B, R))
    pn = rng.uniform(0.1, 0.9, size=p.shape) if neg else None
    for s, name in ((LOG, "log"), (REAL, "real"), (MAXLOG, "maxlog")):
        with np.errstate(divide="ignore"):
            w = p if s == REAL else np.log(p)
            wn = None if pn is None else (pn if s == REAL else np.log(pn))
        tw = torch.from_numpy(np.ascontiguousarray(w)).cuda()
        tn = None if wn is None else torch.from_numpy(np.ascontiguousarray(wn)).cuda()
        got = k.forward_f64(tw, s, neg_weights=tn).cpu().numpy()
        with np.errstate(all="ignore"):
            ref = oracle.forward(*c.arrays(), w, s, nthreads=8, neg_weights=wn)
        inf = np.isinf(ref)
        np.testing.assert_array_equal(got[inf], ref[inf])
        if s == REAL:
            np.testing.assert_allclose(got[~inf], ref[~inf], rtol=1e-12, atol=1e-300, err_msg=what + " f64 " + name)
        else:
            scale = max(1.0, np.abs(ref[~inf]).max()) if (~inf).any() else 1.0
            np.testing.assert_allclose(got[~inf], ref[~inf], rtol=0, atol=1e-11 * scale, err_msg=what + " f64 " + name)
        if backward and s in (LOG, REAL):
            g = k.backward_f64(torch.from_numpy(dout).cuda())
            with np.errstate(all="ignore"):
                r = oracle.backward(*c.arrays(), w, s, dout, nthreads=8, neg_weights=wn)
                m = oracle.backward(*c.arrays(), w, s, dout, nthreads=8, neg_weights=wn, path_mass=True)
            for gg, rr, mm in zip(g if neg else (g,), r if neg else (r,), m if neg else (m,)):
                gg = gg.cpu().numpy()
                fin = np.isfinite(rr)
                np.testing.assert_array_equal(gg[~fin], rr[~fin])
                assert np.all(np.abs(gg[fin] - rr[fin]) <= 1e-10 * np.maximum(1.0, mm[fin])), what + " f64 grad " + name
    k.close()


def test_f64_small_circuits_and_options(klay, golden):
    for name, nv in (("fig1b_ddnnf.txt", 4), ("fig3_multiroot.txt", 5), ("appD_mnist_add.txt", 2)):
        for B in (1, 70):
            _f64_case(klay, golden(name), leaf_probs(B, B, nv, ("uniform", 0.01, 0.99)), name)
    c = layered_random(4, num_vars=48, depth=8, num_gates=1500, fanin=("geom", 2.0), groups=2, num_roots=7)
    for B in (3, 64, 65, 300):
        _f64_case(klay, c, leaf_probs(B, B, 48), "B=%d" % B)
    _f64_case(klay, c, leaf_probs(9, 40, 48), "neg", neg=True)
    for mode in layer_modes(klay, c):
        _f64_case(klay, c, leaf_probs(9, 40, 48), str(mode), **mode)
        _f64_case(klay, c, leaf_probs(9, 40, 48), "neg %s" % mode, neg=True, **mode)
    z = layered_random(2, num_vars=64, depth=6, num_gates=1200, fanin=("zipf", 1.3, 400), groups=1, num_roots=5)
    pz = leaf_probs(5, 70, 64, ("beta", 0.5, 0.5)); pz[:, ::7] = 0.0; pz[:, 3::11] = 1.0
    _f64_case(klay, z, pz, "split", backward=False, heavy_fan=8, min_segment=4)
    _f64_case(klay, z, leaf_probs(5, 70, 64, ("beta", 0.5, 0.5)), "split grad", heavy_fan=8, min_segment=4)


@pytest.mark.parametrize("name,scale,B", [("powerlaw_10m", 0.08, 64), ("layered_3m_fwd_bwd", 0.02, 256)])
def test_f64_configs_reduced_size(klay, name, scale, B):
    c, p, spec = make_config(name, seed=1, scale=scale, batch=B)
    _f64_case(klay, c, p, name)


@pytest.mark.parametrize("name,semiring", [("layered_3m_fwd_bwd", LOG), ("layered_1m", LOG), ("layered_1m", REAL),
                                           ("powerlaw_10m", LOG)])
def test_fp32_against_f64_on_every_output_at_full_size(klay, name, semiring):
    """The workloads at full size and at the batch the benchmark times (headline: B = 256, the four-column
    tiles): the double-precision kernels agree with the oracle on sampled batch columns, and the fp32
    kernels with the double-precision kernels on every output and every gradient entry.  The
    double-precision path shares the host layerizer and the launch plans with the fp32 path, so only
    its oracle-checked columns are evidence of their own; the all-columns comparison is a relay."""
    import torch
    from oracle import oracle
    c, p, spec = make_config(name, seed=0)
    B = p.shape[0]
    w32 = as_inputs(p, semiring == LOG)
    k = build(klay, c)
    w64 = torch.from_numpy(w32.astype(np.float64)).cuda()
    out64 = k.forward_f64(w64, semiring)
    d64 = k.backward_f64(torch.ones_like(out64))
    cols = np.array([0, B // 3, B - 1])
    osem = oracle.LOG if semiring == LOG else oracle.REAL
    with np.errstate(all="ignore"):
        ref = oracle.forward(*c.arrays(), w32[cols].astype(np.float64), osem, nthreads=3)
        rgrad = oracle.backward(*c.arrays(), w32[cols].astype(np.float64), osem, np.ones_like(ref), nthreads=3)
    o64, g64 = out64.cpu().numpy(), d64.cpu().numpy()
    del out64, d64
    if semiring == LOG:
        np.testing.assert_allclose(o64[cols], ref, rtol=0, atol=1e-10)
        np.testing.assert_allclose(g64[cols], rgrad, rtol=1e-9, atol=1e-9)
    else:
        np.testing.assert_allclose(o64[cols], ref, rtol=1e-11, atol=1e-300)
        np.testing.assert_allclose(g64[cols], rgrad, rtol=1e-9, atol=1e-12 * np.abs(rgrad).max())
    got, gd = gpu_eval(k, w32, semiring, np.ones((B, c.roots.shape[0]), dtype=np.float32))
    if semiring == LOG:
        assert_log_close(got, o64, "fp32 vs f64, all outputs")
        ratio = assert_grad_plain(gd, g64, "fp32 vs f64, all gradient entries")
        print("%s B=%d fp32 vs f64: max|dlog| %.2e, gradient error %.3g x the plain bound" % (
            name, B, np.abs(got - o64).max(), ratio))
    else:
        print("%s B=%d real fp32 vs f64: max rel %.2e" % (name, B, assert_real_close(got, o64, "fp32 vs f64 real")))
    k.close()


def test_f64_real_semiring_reaches_below_the_fp32_range(klay):
    """deep products of small probabilities: the fp32 real semiring underflows to 0, the double-precision
    one still agrees with the oracle to rounding, values and gradients"""
    import torch
    from oracle import oracle
    b = CircuitBuilder(40)
    node = b.and_(b.lit(0), b.lit(1))
    for v in range(2, 40, 2):
        alt = b.and_(node, b.lit(v, False))                   # a second, even smaller alternative
        node = b.and_(b.or_(node, alt), b.lit(v), b.lit(v + 1))
    c = b.finish([node])
    p = np.full((3, 40), 1e-3); p[1] *= 2; p[2, ::3] = 0.5
    k = build(klay, c)
    out32, _ = gpu_eval(k, p.astype(np.float32), REAL)
    tw = torch.from_numpy(p).cuda()
    out64 = k.forward_f64(tw, REAL).cpu().numpy()
    ref = oracle.forward(*c.arrays(), p, oracle.REAL)
    assert np.all(ref > 0) and ref.min() < 1e-100 and np.all(out32[ref < 1e-60] == 0.0)
    np.testing.assert_allclose(out64, ref, rtol=1e-12)
    g = k.backward_f64(torch.ones(3, 1, dtype=torch.float64, device="cuda")).cpu().numpy()
    rg = oracle.backward(*c.arrays(), p, oracle.REAL, np.ones((3, 1)))
    np.testing.assert_allclose(g, rg, rtol=1e-10, atol=0)
    k.close()


# ------------------------------------------------------------------ random DAGs x random build options
def _random_dag(rng, V, n_gates, hub_share, max_fan):
    """arbitrary NNF DAG: gate types at random (no alternation), children anywhere below, a few hub
    nodes with many parents, constants included; children of a gate are distinct nodes"""
    b = CircuitBuilder(V)
    nodes = [b.lit(v, bool(s)) for v in range(V) for s in (1, 0)] + [b.true(), b.false()]
    lits_of = {n: i // 2 for i, n in enumerate(nodes[:2 * V])}
    for _ in range(n_gates):
        k = int(rng.integers(1, max_fan + 1))
        kids, seen_vars = [], set()
        for _ in range(k):
            c = int(nodes[int(rng.integers(0, min(len(nodes), 8)))] if rng.random() < hub_share else nodes[int(rng.integers(0, len(nodes)))])
            if c in kids:
                continue
            if c in lits_of:                      # one leaf node per literal here, so this never draws a literal twice
                if (lits_of[c], c) in seen_vars:
                    continue
                seen_vars.add((lits_of[c], c))
            kids.append(c)
        nodes.append(b.and_(*kids) if rng.random() < 0.5 else b.or_(*kids))
    roots = [int(nodes[int(rng.integers(2 * V, len(nodes)))]) for _ in range(int(rng.integers(1, 5)))]
    return b.finish(roots)


@pytest.mark.parametrize("seed", range(96))
def test_random_dags_with_random_options(klay, seed):
    rng = np.random.default_rng(1000 + seed)
    V = int(rng.integers(2, 14))
    c = _random_dag(rng, V, int(rng.integers(5, 400)), hub_share=0.25, max_fan=int(rng.choice([3, 6, 40])))
    opts = dict(unary_chains=bool(rng.integers(3) == 0), tail_rows_cap=int(rng.choice([0, 0, 3, 6, 12, 30])), no_merge=bool(rng.integers(2)), no_reorder=bool(rng.integers(2)),
                no_tail=bool(rng.integers(2)), heavy_fan=int(rng.choice([0, 2, 5, 17])), min_segment=int(rng.choice([0, 1, 3])),
                small_batch_edges=bool(seed % 3 == 0), no_fusion=bool(seed % 5 == 0))
    B = int(rng.choice([1, 2, 7, 33, 64, 100, 257]))
    # probabilities near 1/2 keep the real semiring inside fp32 whatever the random structure multiplies up
    p = rng.uniform(0.35, 0.65, size=(B, V))
    print("seed", seed, "V", V, "nodes", c.num_nodes, "B", B, opts, flush=True)
    try:
        k = build(klay, c, **opts)
    except klay.KlayError as e:
        assert e.status == 1, e                      # a structurally invalid draw is rejected, never mis-evaluated
        pytest.skip("rejected input: " + str(e))
    k.close()
    # an arbitrary DAG can push real-semiring values beyond the fp32 range (inf, then inf * 0): no claim there
    from oracle import oracle
    with np.errstate(all="ignore"):
        _, vals = oracle.forward(*c.arrays(), p, oracle.REAL, return_node_values=True)
    in_range = np.nanmax(np.abs(vals)) < 1e30
    # ... and so can a partial product (the split of a row into segments groups the children anew): a product node
    # with a zero child and large ones is 0 in exact arithmetic but inf * 0 in some grouping
    for i in np.flatnonzero(c.node_type == AND):
        ch = c.child_idx[c.child_ptr[i]:c.child_ptr[i + 1]]
        with np.errstate(all="ignore"):
            big = np.prod(np.maximum(np.abs(np.nan_to_num(vals[:, ch], nan=1.0)), 1.0), axis=1)
        in_range = in_range and bool(big.max() < 1e30)
    check_both(klay, c, p, what="random dag %d" % seed, semirings=(REAL, LOG) if in_range else (LOG,), **opts)
