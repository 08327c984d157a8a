"""ctypes front end of the fp64 CPU oracle (``klay_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the GPU library never does, and this
module imports nothing from the GPU package.

The oracle evaluates the original, unlayered circuit DAG node by node, children
before parents (paper Section 2, Eq. 1; log domain per Section 4 / Alg. 4 with
epsilon = 0), in fp64.  Parity unpinned: nothing (pins live in tests/test_oracle_pins.py).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

REAL = 0
LOG = 1
MAXLOG = 2     # (max, +) on log weights, forward only

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "klay_oracle.c")
_LIB = os.path.join(_HERE, "libklay_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math) and return the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i32, i64, dbl = ctypes.c_int32, ctypes.c_int64, ctypes.c_double
            p = ctypes.c_void_p
            lib.klay_oracle_postorder.restype = i64
            lib.klay_oracle_postorder.argtypes = [i64, p, p, i32, p, p]
            lib.klay_oracle_forward.restype = ctypes.c_int
            lib.klay_oracle_forward.argtypes = [i32, i64, p, p, p, p, i32, p, i32, p, p, ctypes.c_int, p, p, ctypes.c_int]
            lib.klay_oracle_backward.restype = ctypes.c_int
            lib.klay_oracle_backward.argtypes = [i32, i64, p, p, p, p, i32, p, i32, p, p, ctypes.c_int, p, p, p, ctypes.c_int, ctypes.c_int]
            lib.klay_oracle_max_threads.restype = ctypes.c_int
            _lib = lib
            del dbl
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _circuit_arrays(num_vars, node_type, node_lit, child_ptr, child_idx, roots):
    node_type = np.ascontiguousarray(node_type, dtype=np.uint8)
    node_lit = np.ascontiguousarray(node_lit, dtype=np.int32)
    child_ptr = np.ascontiguousarray(child_ptr, dtype=np.int64)
    child_idx = np.ascontiguousarray(child_idx, dtype=np.int32)
    roots = np.ascontiguousarray(roots, dtype=np.int32)
    n = node_type.shape[0]
    if node_lit.shape[0] != n or child_ptr.shape[0] != n + 1:
        raise ValueError("inconsistent circuit arrays")
    if child_ptr[0] != 0 or child_ptr[-1] != child_idx.shape[0] or np.any(np.diff(child_ptr) < 0):
        raise ValueError("bad child_ptr")
    if child_idx.size and (child_idx.min() < 0 or child_idx.max() >= n):
        raise ValueError("child index out of range")
    if roots.size == 0 or roots.min() < 0 or roots.max() >= n:
        raise ValueError("bad roots")
    lits = node_lit[node_type == 0]
    if lits.size and (np.abs(lits).min() < 1 or np.abs(lits).max() > num_vars):
        raise ValueError("literal out of range")
    if np.any(node_type > 4):
        raise ValueError("bad node type")
    return node_type, node_lit, child_ptr, child_idx, roots


def max_threads() -> int:
    return int(_load().klay_oracle_max_threads())


def postorder(node_type, node_lit, child_ptr, child_idx, roots):
    """The oracle's evaluation order: every node reachable from the roots, children before parents."""
    lib = _load()
    child_ptr = np.ascontiguousarray(child_ptr, dtype=np.int64)
    child_idx = np.ascontiguousarray(child_idx, dtype=np.int32)
    roots = np.ascontiguousarray(roots, dtype=np.int32)
    n = child_ptr.shape[0] - 1
    order = np.empty(n + 1, dtype=np.int32)
    count = lib.klay_oracle_postorder(n, _ptr(child_ptr), _ptr(child_idx), roots.shape[0], _ptr(roots), _ptr(order))
    if count == -1:
        raise ValueError("circuit has a cycle")
    if count < 0:
        raise MemoryError("oracle postorder failed (%d)" % count)
    return order[:count]


def forward(num_vars, node_type, node_lit, child_ptr, child_idx, roots, weights, semiring,
            nthreads: int = 1, return_node_values: bool = False, neg_weights=None):
    """Root values ``out[B,R]`` (fp64) for leaf weights ``weights[B,V]``.

    ``weights`` holds p (REAL) or log p (LOG, MAXLOG); it is widened to fp64 as given.
    With ``return_node_values`` also returns ``vals[B,num_nodes]`` (NaN where unreachable).
    ``neg_weights[B,V]`` gives the negated literals weights of their own instead of 1-p / log(1-e^x).
    """
    lib = _load()
    if int(semiring) not in (REAL, LOG, MAXLOG):
        raise ValueError("unknown semiring")
    node_type, node_lit, child_ptr, child_idx, roots = _circuit_arrays(
        num_vars, node_type, node_lit, child_ptr, child_idx, roots)
    w = np.ascontiguousarray(weights, dtype=np.float64)
    if w.ndim != 2 or w.shape[1] != num_vars:
        raise ValueError("weights must be [B,V]")
    B, R, n = w.shape[0], roots.shape[0], node_type.shape[0]
    out = np.empty((B, R), dtype=np.float64)
    vals = np.empty((B, n), dtype=np.float64) if return_node_values else None
    wn = None
    if neg_weights is not None:
        wn = np.ascontiguousarray(neg_weights, dtype=np.float64)
        if wn.shape != w.shape:
            raise ValueError("neg_weights must have the shape of weights")
    rc = lib.klay_oracle_forward(num_vars, n, _ptr(node_type), _ptr(node_lit), _ptr(child_ptr),
                                 _ptr(child_idx), R, _ptr(roots), B, _ptr(w), _ptr(wn) if wn is not None else None,
                                 int(semiring),
                                 _ptr(out), _ptr(vals) if vals is not None else None, int(nthreads))
    if rc == -1:
        raise ValueError("circuit has a cycle")
    if rc != 0:
        raise MemoryError("oracle forward failed (%d)" % rc)
    return (out, vals) if return_node_values else out


def backward(num_vars, node_type, node_lit, child_ptr, child_idx, roots, weights, semiring,
             dout, nthreads: int = 1, path_mass: bool = False, neg_weights=None):
    """``dleaf[B,V] = sum_r dout[b,r] * d out[b,r] / d weights[b,v]`` (fp64, reverse mode).

    With ``path_mass`` the sweep runs on absolute values and returns the sum over all root-to-leaf
    paths of |contribution| (>= |dleaf|): the scale of the cancellation in the gradient.
    With ``neg_weights`` the two weight arrays are independent inputs and the result is the pair
    ``(dpos[B,V], dneg[B,V])``."""
    lib = _load()
    if int(semiring) not in (REAL, LOG):
        raise ValueError("only the real and the log semiring are differentiated")
    node_type, node_lit, child_ptr, child_idx, roots = _circuit_arrays(
        num_vars, node_type, node_lit, child_ptr, child_idx, roots)
    w = np.ascontiguousarray(weights, dtype=np.float64)
    g = np.ascontiguousarray(dout, dtype=np.float64)
    B, R, n = w.shape[0], roots.shape[0], node_type.shape[0]
    if w.ndim != 2 or w.shape[1] != num_vars or g.shape != (B, R):
        raise ValueError("weights must be [B,V] and dout [B,R]")
    dleaf = np.empty((B, num_vars), dtype=np.float64)
    wn = dneg = None
    if neg_weights is not None:
        wn = np.ascontiguousarray(neg_weights, dtype=np.float64)
        if wn.shape != w.shape:
            raise ValueError("neg_weights must have the shape of weights")
        dneg = np.empty((B, num_vars), dtype=np.float64)
    rc = lib.klay_oracle_backward(num_vars, n, _ptr(node_type), _ptr(node_lit), _ptr(child_ptr),
                                  _ptr(child_idx), R, _ptr(roots), B, _ptr(w), _ptr(wn) if wn is not None else None,
                                  int(semiring), _ptr(g), _ptr(dleaf), _ptr(dneg) if dneg is not None else None,
                                  int(nthreads), int(bool(path_mass)))
    if rc == -1:
        raise ValueError("circuit has a cycle")
    if rc != 0:
        raise MemoryError("oracle backward failed (%d)" % rc)
    return dleaf if dneg is None else (dleaf, dneg)
