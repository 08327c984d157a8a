"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle on
the same fp32 inputs widened to fp64, and compare to the stated tolerances."""
import numpy as np

LOG_ATOL = 1e-4      # |delta log| for the fp32 log semiring
REAL_RTOL = 1e-5     # relative error for the fp32 real semiring
REAL_FLOOR = 1.2e-38 # below fp32's normal range only absolute agreement is asked
# Gradients (log semiring), adjoint seed dout = 1: the plain bound |delta| <= GRAD_TOL * max(1, |ref|)
# (assert_grad_plain).  With a random dout of mixed signs the gradient is a difference of large path sums,
# and the bound gets a cancellation term (assert_grad_close):
# |delta| <= GRAD_TOL * max(1, |ref|) + rel * mass, where mass is the sum over all
# root-to-leaf paths of |contribution| (the oracle's path-mass sweep) and
#   rel = 64 u + 4 u * or_levels * max|node value|,   u = 2^-24:
# 64 unit roundoffs for the fp32 summations, and per OR level a softmax weight exp(N_c - N_r)
# whose argument carries the storage rounding u |N| of both values plus that of the difference.
# Real semiring: rel = (64 + 16 * or_levels) u, and the absolute part is REAL_RTOL * |ref| + fp32 floor.
GRAD_TOL = 1e-4
U32 = 2.0 ** -24


def gpu_eval(k, w32, semiring, dout=None):
    """k: paper_2410_11415_amd.Circuit on cuda:0.  Returns (out[B,R], dleaf[B,V] or None) as numpy."""
    import torch
    w = torch.from_numpy(np.ascontiguousarray(w32, dtype=np.float32)).cuda()
    out = k.forward(w, semiring)
    dleaf = None
    if dout is not None:
        d = torch.from_numpy(np.ascontiguousarray(dout, dtype=np.float32)).cuda()
        dleaf = k.backward(d).cpu().numpy()
    torch.cuda.synchronize()
    return out.cpu().numpy(), dleaf


def oracle_eval(c, w32, semiring, dout=None, nthreads=8, or_levels=None):
    """or_levels: number of OR layers of the layered circuit (for the gradient bound); default: from
    the input DAG's node count is not possible, so callers that check gradients pass it."""
    from oracle import oracle
    w64 = np.asarray(w32, dtype=np.float32).astype(np.float64)
    with np.errstate(all="ignore"):
        dleaf = None
        if dout is None:
            out = oracle.forward(*c.arrays(), w64, semiring, nthreads=nthreads)
        else:
            out, vals = oracle.forward(*c.arrays(), w64, semiring, nthreads=nthreads, return_node_values=True)
            finite = np.isfinite(vals)
            maxabs = float(np.abs(vals[finite]).max()) if finite.any() else 0.0
            del vals, finite
            d64 = np.asarray(dout, np.float32).astype(np.float64)
            dleaf = oracle.backward(*c.arrays(), w64, semiring, d64, nthreads=nthreads)
            mass = oracle.backward(*c.arrays(), w64, semiring, d64, nthreads=nthreads, path_mass=True)
            levels = 64 if or_levels is None else or_levels
            if semiring == 1:
                rel = 64 * U32 + 4 * U32 * levels * maxabs
            else:
                # real semiring: every level multiplies by a quotient of fp32 products (a few roundoffs each)
                rel = (64 + 16 * levels) * U32
            dleaf = GradRef(dleaf, mass, rel)
    return out, dleaf


class GradRef(np.ndarray):
    """oracle gradient that also carries the path mass sum |contribution| of each entry"""
    def __new__(cls, grad, mass, rel):
        obj = np.asarray(grad).view(cls)
        obj.mass = np.asarray(mass)
        obj.rel = rel
        return obj

    def __array_finalize__(self, obj):
        self.mass = getattr(obj, "mass", None)
        self.rel = getattr(obj, "rel", 64 * U32)

    def __getitem__(self, item):
        out = super().__getitem__(item)
        if isinstance(out, GradRef) and self.mass is not None:
            out.mass = self.mass[item]
        return out


def assert_log_close(got, ref, what=""):
    got = np.asarray(got, dtype=np.float64)
    inf = np.isinf(ref)
    assert not np.isnan(got).any(), what + ": NaN in GPU result"
    np.testing.assert_array_equal(got[inf], ref[inf], err_msg=what + ": infinities must match exactly")
    err = np.abs(got[~inf] - ref[~inf])
    assert err.size == 0 or err.max() <= LOG_ATOL, "%s: max |dlog| = %.3e (max |log ref| = %.1f)" % (
        what, err.max(), np.abs(ref[~inf]).max())
    return float(err.max()) if err.size else 0.0


def assert_real_close(got, ref, what=""):
    got = np.asarray(got, dtype=np.float64)
    assert not np.isnan(got).any(), what + ": NaN in GPU result"
    err = np.abs(got - ref)
    bound = REAL_RTOL * np.abs(ref) + REAL_FLOOR
    worst = (err / np.maximum(np.abs(ref), REAL_FLOOR)).max()
    assert np.all(err <= bound), "%s: max rel err = %.3e" % (what, worst)
    return float(worst)


def plain_grad_ratio(got, ref):
    """max over entries of |got - ref| / (GRAD_TOL * max(1, |ref|)): the plain gradient bound, <= 1 to pass"""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    fin = np.isfinite(ref)
    if not fin.any():
        return 0.0
    return float((np.abs(got[fin] - ref[fin]) / (GRAD_TOL * np.maximum(1.0, np.abs(ref[fin])))).max())


def assert_grad_plain(got, ref, what=""):
    """The plain bound |delta| <= 1e-4 max(1, |ref|), with no allowance for cancellation: asserted wherever
    the adjoint seed is dout = 1 (log semiring: every path contributes with a positive softmax weight, and
    the tied negated literal is the only source of opposite signs).  Returns the ratio error / bound."""
    got = np.asarray(got, dtype=np.float64)
    assert not np.isnan(got).any(), what + ": NaN in GPU gradient"
    ref = np.asarray(ref, dtype=np.float64)
    inf = np.isinf(ref)
    np.testing.assert_array_equal(got[inf], ref[inf])
    ratio = plain_grad_ratio(got, ref)
    assert ratio <= 1.0, "%s: gradient error is %.3g x the plain bound 1e-4 max(1, |ref|) (max |ref| %.3g)" % (
        what, ratio, np.abs(ref[~inf]).max())
    return ratio


def assert_grad_close(got, ref, what="", real=False):
    got = np.asarray(got, dtype=np.float64)
    assert not np.isnan(got).any(), what + ": NaN in GPU gradient"
    mass = getattr(ref, "mass", None)
    rel = getattr(ref, "rel", 64 * U32)
    ref = np.asarray(ref)
    mass = np.abs(ref) if mass is None else np.asarray(mass)
    inf = np.isinf(ref)
    np.testing.assert_array_equal(got[inf], ref[inf])
    bound = GRAD_TOL * np.maximum(1.0, np.abs(ref[~inf])) + rel * mass[~inf]
    if real:
        bound = REAL_RTOL * np.abs(ref[~inf]) + REAL_FLOOR + rel * mass[~inf]
    err = np.abs(got[~inf] - ref[~inf]) / bound
    assert err.size == 0 or err.max() <= 1.0, "%s: gradient error is %.3g x the bound (max |ref| %.3g, max mass %.3g)" % (
        what, err.max(), np.abs(ref[~inf]).max(), mass[~inf].max())
    if not real:
        # how the same errors stand against the plain bound (the mass term only matters under cancellation)
        WORST_PLAIN_RATIO[0] = max(WORST_PLAIN_RATIO[0], plain_grad_ratio(got, ref))
    return float(err.max()) if err.size else 0.0


# largest error / (1e-4 max(1, |ref|)) seen by assert_grad_close in this process (log semiring, random dout):
# printed by the test session's summary so that a reader sees how far above the plain bound any case was
WORST_PLAIN_RATIO = [0.0]
