"""Thin ctypes binding of libklay.so: argument marshalling only.

The module-level ``klay_*`` functions mirror the C ABI in ``include/klay.h`` one to one (same
names, pointers passed as integers).  :class:`Circuit` is a small convenience wrapper that takes
numpy arrays for the circuit and torch CUDA tensors for the batch data; torch is used only for
device memory and streams.  There is no CPU fallback: if the HIP library cannot be loaded or
built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

KLAY_OK, KLAY_EINVAL, KLAY_ECYCLE, KLAY_ENOMEM, KLAY_EHIP, KLAY_ESTATE = range(6)
KLAY_REAL, KLAY_LOG, KLAY_MAXLOG = 0, 1, 2
KLAY_LIT, KLAY_AND, KLAY_OR, KLAY_TRUE, KLAY_FALSE = range(5)
KLAY_STATIC_WORKSPACE_BYTES = 64 << 20
KERNEL_CLASSES = ("leaf", "fwd_sum", "fwd_prod", "fwd_lse", "root", "seed", "bwd_sum", "bwd_softmax", "bwd_leaf",
                  "tail_fwd", "tail_bwd", "split", "prod_edges", "fwd_max", "bwd_sum_enc", "bwd_softmax_one",
                  "bwd_prod", "bwd_sum_mul", "bwd_prod_mul", "combine", "main_combine", "fwd_or_fused")

EXPORTS = ("klay_build", "klay_build_ex", "klay_forward", "klay_backward", "klay_info", "klay_layer_sizes",
           "klay_layer_csr", "klay_layer_nodes", "klay_workspace_bytes", "klay_set_workspace",
           "klay_set_profiling", "klay_get_profile", "klay_destroy", "klay_last_error", "klay_builder_create",
           "klay_builder_add", "klay_builder_finish", "klay_builder_destroy", "klay_forward_lits", "klay_backward_lits", "klay_root_positions", "klay_forward_f64",
           "klay_backward_f64", "klay_forward_static")


class KlayError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("klay status %d: %s" % (status, message))
        self.status = status


class klay_options(ctypes.Structure):
    _fields_ = [("no_reorder", ctypes.c_int32), ("heavy_fan", ctypes.c_int32), ("min_segment", ctypes.c_int32),
                ("no_tail", ctypes.c_int32), ("unary_chains", ctypes.c_int32), ("no_merge", ctypes.c_int32),
                ("small_batch_edges", ctypes.c_int32), ("tail_rows_cap", ctypes.c_int32), ("no_fusion", ctypes.c_int32)]


class klay_info_t(ctypes.Structure):
    _fields_ = [("num_vars", ctypes.c_int32), ("num_roots", ctypes.c_int32), ("num_layers", ctypes.c_int32),
                ("device", ctypes.c_int32), ("num_nodes", ctypes.c_int64), ("num_edges", ctypes.c_int64),
                ("dag_nodes", ctypes.c_int64), ("dag_edges", ctypes.c_int64), ("num_pad_nodes", ctypes.c_int64),
                ("max_layer_nodes", ctypes.c_int64), ("max_fan_in", ctypes.c_int64), ("max_fan_out", ctypes.c_int64),
                ("num_split_rows", ctypes.c_int64), ("index_bytes", ctypes.c_int64),
                ("tail_first_layer", ctypes.c_int64), ("num_merged_nodes", ctypes.c_int64),
                ("alias_top_layer", ctypes.c_int64), ("num_fused_rows", ctypes.c_int64)]


class klay_profile_t(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_float * len(KERNEL_CLASSES)), ("launches", ctypes.c_int32 * len(KERNEL_CLASSES)),
                ("alg_bytes", ctypes.c_double * len(KERNEL_CLASSES)), ("min_bytes", ctypes.c_double * len(KERNEL_CLASSES))]


_lib = None


def library_path() -> str:
    return _build.LIB_PATH


def load():
    """Load libklay.so, building it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    # PyTorch ships a HIP runtime of its own.  If libklay.so is loaded first it binds to the system
    # runtime, torch later brings its copy, and whichever of the two initialises the device second
    # finds none.  With torch imported first the library resolves to the runtime torch has loaded.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.klay_build.restype = ctypes.c_int
    lib.klay_build.argtypes = [i32, i64, vp, vp, vp, vp, i32, vp, i32, ctypes.POINTER(vp)]
    lib.klay_build_ex.restype = ctypes.c_int
    lib.klay_build_ex.argtypes = [i32, i64, vp, vp, vp, vp, i32, vp, i32, ctypes.POINTER(klay_options),
                                  ctypes.POINTER(vp)]
    lib.klay_forward.restype = ctypes.c_int
    lib.klay_forward.argtypes = [vp, vp, i32, vp, ctypes.c_int, vp]
    lib.klay_backward.restype = ctypes.c_int
    lib.klay_backward.argtypes = [vp, vp, vp, vp]
    lib.klay_forward_static.restype = ctypes.c_int
    lib.klay_forward_static.argtypes = [vp, vp, i32, vp, ctypes.c_int, vp]
    lib.klay_forward_lits.restype = ctypes.c_int
    lib.klay_forward_lits.argtypes = [vp, vp, vp, i32, vp, ctypes.c_int, vp]
    lib.klay_backward_lits.restype = ctypes.c_int
    lib.klay_backward_lits.argtypes = [vp, vp, vp, vp, vp]
    lib.klay_info.restype = ctypes.c_int
    lib.klay_info.argtypes = [vp, ctypes.POINTER(klay_info_t)]
    lib.klay_layer_sizes.restype = ctypes.c_int
    lib.klay_layer_sizes.argtypes = [vp, vp, vp]
    lib.klay_layer_csr.restype = ctypes.c_int
    lib.klay_layer_csr.argtypes = [vp, i32, vp, vp]
    lib.klay_layer_nodes.restype = ctypes.c_int
    lib.klay_layer_nodes.argtypes = [vp, i32, vp, vp]
    lib.klay_forward_f64.restype = ctypes.c_int
    lib.klay_forward_f64.argtypes = [vp, vp, vp, i32, vp, ctypes.c_int, vp]
    lib.klay_backward_f64.restype = ctypes.c_int
    lib.klay_backward_f64.argtypes = [vp, vp, vp, vp, vp]
    lib.klay_root_positions.restype = ctypes.c_int
    lib.klay_root_positions.argtypes = [vp, vp]
    lib.klay_workspace_bytes.restype = ctypes.c_size_t
    lib.klay_workspace_bytes.argtypes = [vp, i32, ctypes.c_int]
    lib.klay_set_workspace.restype = ctypes.c_int
    lib.klay_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.klay_set_profiling.restype = ctypes.c_int
    lib.klay_set_profiling.argtypes = [vp, i32]
    lib.klay_get_profile.restype = ctypes.c_int
    lib.klay_get_profile.argtypes = [vp, ctypes.POINTER(klay_profile_t)]
    lib.klay_builder_create.restype = ctypes.c_int
    lib.klay_builder_create.argtypes = [i32, ctypes.POINTER(vp)]
    lib.klay_builder_add.restype = ctypes.c_int
    lib.klay_builder_add.argtypes = [vp, i64, vp, vp, vp, vp, i32, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.klay_builder_finish.restype = ctypes.c_int
    lib.klay_builder_finish.argtypes = [vp, i32, ctypes.POINTER(klay_options), ctypes.POINTER(vp)]
    lib.klay_builder_destroy.restype = None
    lib.klay_builder_destroy.argtypes = [vp]
    lib.klay_destroy.restype = None
    lib.klay_destroy.argtypes = [vp]
    lib.klay_last_error.restype = ctypes.c_char_p
    lib.klay_last_error.argtypes = []
    _lib = lib
    return lib


def klay_last_error() -> str:
    return load().klay_last_error().decode()


def _check(status):
    if status != KLAY_OK:
        raise KlayError(status, klay_last_error())


def _np_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


# ---- one-to-one wrappers (pointers are ints / ctypes void pointers) -------------------------
def klay_build(num_vars, num_nodes, node_type_ptr, node_lit_ptr, child_ptr_ptr, child_idx_ptr, num_roots,
               roots_ptr, device, options: klay_options | None = None):
    h = ctypes.c_void_p()
    lib = load()
    if options is None:
        st = lib.klay_build(num_vars, num_nodes, node_type_ptr, node_lit_ptr, child_ptr_ptr, child_idx_ptr,
                            num_roots, roots_ptr, device, ctypes.byref(h))
    else:
        st = lib.klay_build_ex(num_vars, num_nodes, node_type_ptr, node_lit_ptr, child_ptr_ptr, child_idx_ptr,
                               num_roots, roots_ptr, device, ctypes.byref(options), ctypes.byref(h))
    _check(st)
    return h


def klay_forward(handle, leaf_weights_ptr, B, out_ptr, semiring, stream=0):
    _check(load().klay_forward(handle, leaf_weights_ptr, B, out_ptr, semiring, stream))


def klay_forward_static(handle, leaf_weights_ptr, B, out_ptr, semiring, stream=0):
    _check(load().klay_forward_static(handle, leaf_weights_ptr, B, out_ptr, semiring, stream))


def klay_backward(handle, dout_ptr, dleaf_ptr, stream=0):
    _check(load().klay_backward(handle, dout_ptr, dleaf_ptr, stream))


def klay_forward_lits(handle, pos_weights_ptr, neg_weights_ptr, B, out_ptr, semiring, stream=0):
    _check(load().klay_forward_lits(handle, pos_weights_ptr, neg_weights_ptr, B, out_ptr, semiring, stream))


def klay_backward_lits(handle, dout_ptr, dpos_ptr, dneg_ptr, stream=0):
    _check(load().klay_backward_lits(handle, dout_ptr, dpos_ptr, dneg_ptr, stream))


def klay_forward_f64(handle, pos_weights_ptr, neg_weights_ptr, B, out_ptr, semiring, stream=0):
    _check(load().klay_forward_f64(handle, pos_weights_ptr, neg_weights_ptr, B, out_ptr, semiring, stream))


def klay_backward_f64(handle, dout_ptr, dpos_ptr, dneg_ptr, stream=0):
    _check(load().klay_backward_f64(handle, dout_ptr, dpos_ptr, dneg_ptr, stream))


def klay_destroy(handle):
    load().klay_destroy(handle)


def klay_builder_create(num_vars):
    b = ctypes.c_void_p()
    _check(load().klay_builder_create(num_vars, ctypes.byref(b)))
    return b


def klay_builder_add(builder, num_nodes, node_type_ptr, node_lit_ptr, child_ptr_ptr, child_idx_ptr, num_roots,
                     roots_ptr) -> int:
    first = ctypes.c_int32(-1)
    _check(load().klay_builder_add(builder, num_nodes, node_type_ptr, node_lit_ptr, child_ptr_ptr, child_idx_ptr,
                                   num_roots, roots_ptr, ctypes.byref(first)))
    return first.value


def klay_builder_finish(builder, device, options: klay_options | None = None):
    h = ctypes.c_void_p()
    _check(load().klay_builder_finish(builder, device, ctypes.byref(options) if options is not None else None,
                                      ctypes.byref(h)))
    return h


def klay_builder_destroy(builder):
    load().klay_builder_destroy(builder)


# ---- convenience wrapper --------------------------------------------------------------------
class Circuit:
    """A built circuit.  ``device=-1`` gives a host-only handle (layerization inspection only)."""

    def __init__(self, num_vars, node_type, node_lit, child_ptr, child_idx, roots, device=0,
                 no_reorder=False, heavy_fan=0, min_segment=0, no_tail=False,
                 unary_chains=False, no_merge=False, small_batch_edges=False, tail_rows_cap=0, no_fusion=False):
        node_type = np.ascontiguousarray(node_type, dtype=np.uint8)
        node_lit = np.ascontiguousarray(node_lit, dtype=np.int32)
        child_ptr = np.ascontiguousarray(child_ptr, dtype=np.int64)
        child_idx = np.ascontiguousarray(child_idx, dtype=np.int32)
        roots = np.ascontiguousarray(roots, dtype=np.int32)
        if node_lit.shape[0] != node_type.shape[0] or child_ptr.shape[0] != node_type.shape[0] + 1:
            raise ValueError("node_type, node_lit and child_ptr sizes disagree")
        if child_ptr.shape[0] and child_idx.shape[0] != child_ptr[-1]:
            raise ValueError("child_idx must have child_ptr[-1] entries")
        opts = klay_options(int(no_reorder), int(heavy_fan), int(min_segment), int(no_tail), int(unary_chains),
                            int(no_merge), int(small_batch_edges), int(tail_rows_cap), int(no_fusion))
        self._h = None
        self._h = klay_build(int(num_vars), node_type.shape[0], _np_ptr(node_type), _np_ptr(node_lit),
                             _np_ptr(child_ptr), _np_ptr(child_idx) if child_idx.size else None,
                             roots.shape[0], _np_ptr(roots), int(device), opts)
        self._adopt(int(device))

    def _adopt(self, device):
        self.device = device
        self._workspace = None
        i = self.info()
        self.num_vars, self.num_roots, self.num_layers = i["num_vars"], i["num_roots"], i["num_layers"]

    @classmethod
    def _from_handle(cls, handle, device):
        c = cls.__new__(cls)
        c._h = handle
        c._adopt(int(device))
        return c

    @classmethod
    def from_nnf(cls, path: str, **kw):
        """Build from a d-DNNF compiler's ``.nnf`` text file (see :mod:`.nnf`)."""
        from .nnf import load_nnf
        return cls(*load_nnf(path), **kw)

    @classmethod
    def from_sdd(cls, path: str, num_vars=None, **kw):
        """Build from an SDD text file (see :mod:`.sdd`)."""
        from .sdd import load_sdd
        return cls(*load_sdd(path, num_vars), **kw)

    @classmethod
    def from_d4(cls, path: str, num_vars=None, **kw):
        """Build from a d4 decision-DNNF text file (see :mod:`.d4`)."""
        from .d4 import load_d4
        return cls(*load_d4(path, num_vars), **kw)

    # -- inspection
    def info(self) -> dict:
        s = klay_info_t()
        _check(load().klay_info(self._h, ctypes.byref(s)))
        return {k: int(getattr(s, k)) for k, _ in klay_info_t._fields_}

    def layer_sizes(self):
        L = self.num_layers if hasattr(self, "num_layers") else self.info()["num_layers"]
        nodes = np.zeros(L + 1, dtype=np.int64)
        edges = np.zeros(L + 1, dtype=np.int64)
        _check(load().klay_layer_sizes(self._h, _np_ptr(nodes), _np_ptr(edges)))
        return nodes, edges

    def layer_csr(self, layer: int):
        nodes, edges = self.layer_sizes()
        if not 1 <= layer <= self.num_layers:
            raise ValueError("layer out of range")
        row_ptr = np.zeros(nodes[layer] + 1, dtype=np.int64)
        child = np.zeros(max(int(edges[layer]), 1), dtype=np.int32)
        _check(load().klay_layer_csr(self._h, layer, _np_ptr(row_ptr), _np_ptr(child)))
        return row_ptr, child[: int(edges[layer])]

    def layer_nodes(self, layer: int):
        nodes, _ = self.layer_sizes()
        origin = np.zeros(max(int(nodes[layer]), 1), dtype=np.int32)
        is_pad = np.zeros(max(int(nodes[layer]), 1), dtype=np.uint8)
        _check(load().klay_layer_nodes(self._h, layer, _np_ptr(origin), _np_ptr(is_pad)))
        return origin[: int(nodes[layer])], is_pad[: int(nodes[layer])].astype(bool)

    def root_positions(self):
        pos = np.zeros(self.num_roots, dtype=np.int32)
        _check(load().klay_root_positions(self._h, _np_ptr(pos)))
        return pos

    def workspace_bytes(self, B: int, need_backward: bool = True) -> int:
        return int(load().klay_workspace_bytes(self._h, int(B), int(need_backward)))

    def set_workspace(self, tensor):
        """Use a caller-owned torch CUDA tensor as workspace (None: back to library-owned memory)."""
        if tensor is None:
            _check(load().klay_set_workspace(self._h, None, 0))
        else:
            _check(load().klay_set_workspace(self._h, tensor.data_ptr(), tensor.numel() * tensor.element_size()))
        self._workspace = tensor

    def set_profiling(self, enable: bool):
        _check(load().klay_set_profiling(self._h, int(enable)))

    def get_profile(self) -> dict:
        p = klay_profile_t()
        _check(load().klay_get_profile(self._h, ctypes.byref(p)))
        return {name: {"ms": float(p.ms[i]), "launches": int(p.launches[i]), "alg_bytes": float(p.alg_bytes[i]),
                       "min_bytes": float(p.min_bytes[i])}
                for i, name in enumerate(KERNEL_CLASSES)}

    # -- evaluation
    @staticmethod
    def _stream(stream):
        import torch
        s = torch.cuda.current_stream() if stream is None else stream
        return s.cuda_stream

    def forward(self, leaf_weights, semiring=KLAY_LOG, out=None, stream=None, neg_weights=None):
        """leaf_weights: torch float32 CUDA tensor [B, V], contiguous.  Returns out [B, R].
        neg_weights (same shape) gives the negated literals weights of their own."""
        import torch
        for t, name in ((leaf_weights, "leaf_weights"), (neg_weights, "neg_weights")):
            if t is None:
                continue
            if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
                raise ValueError(name + " must be a contiguous float32 CUDA tensor")
            if t.dim() != 2 or t.shape[1] != self.num_vars:
                raise ValueError(name + " must be [B, %d]" % self.num_vars)
        if neg_weights is not None and neg_weights.shape != leaf_weights.shape:
            raise ValueError("neg_weights must have the shape of leaf_weights")
        B = leaf_weights.shape[0]
        if out is None:
            out = torch.empty((B, self.num_roots), dtype=torch.float32, device=leaf_weights.device)
        elif out.shape != (B, self.num_roots) or out.dtype != torch.float32 or not out.is_contiguous():
            raise ValueError("out must be a contiguous float32 tensor [B, R]")
        if neg_weights is None:
            klay_forward(self._h, leaf_weights.data_ptr(), B, out.data_ptr(), int(semiring), self._stream(stream))
        else:
            klay_forward_lits(self._h, leaf_weights.data_ptr(), neg_weights.data_ptr(), B, out.data_ptr(),
                              int(semiring), self._stream(stream))
        self._last_B = B
        self._last_lits = neg_weights is not None
        return out

    def forward_static(self, leaf_weights, semiring=KLAY_LOG, out=None, stream=None):
        """klay_forward_static: the forward pass in the library's fixed device array (no allocation by the
        library; ``out`` should be passed in by a caller that must not allocate either)."""
        import torch
        if (leaf_weights.dtype != torch.float32 or not leaf_weights.is_cuda or not leaf_weights.is_contiguous()
                or leaf_weights.dim() != 2 or leaf_weights.shape[1] != self.num_vars):
            raise ValueError("leaf_weights must be a contiguous float32 CUDA tensor [B, %d]" % self.num_vars)
        B = leaf_weights.shape[0]
        if out is None:
            out = torch.empty((B, self.num_roots), dtype=torch.float32, device=leaf_weights.device)
        elif out.shape != (B, self.num_roots) or out.dtype != torch.float32 or not out.is_contiguous():
            raise ValueError("out must be a contiguous float32 tensor [B, R]")
        klay_forward_static(self._h, leaf_weights.data_ptr(), B, out.data_ptr(), int(semiring), self._stream(stream))
        return out

    def backward(self, dout, dleaf=None, stream=None, dneg=None):
        """dout: [B, R] float32 CUDA.  Returns dleaf [B, V]; after a forward pass with neg_weights
        the pair (dpos, dneg)."""
        import torch
        B = getattr(self, "_last_B", None)
        if B is None:
            raise KlayError(KLAY_ESTATE, "backward before forward")
        if dout.dtype != torch.float32 or not dout.is_cuda or not dout.is_contiguous() or dout.shape != (B, self.num_roots):
            raise ValueError("dout must be a contiguous float32 CUDA tensor [B, R]")
        lits = getattr(self, "_last_lits", False)
        outs = []
        for t, name in ((dleaf, "dleaf"), (dneg, "dneg")):
            if t is None:
                t = torch.empty((B, self.num_vars), dtype=torch.float32, device=dout.device)
            elif t.shape != (B, self.num_vars) or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
                raise ValueError(name + " must be a contiguous float32 CUDA tensor [B, V]")
            outs.append(t)
            if not lits:
                break
        if not lits:
            klay_backward(self._h, dout.data_ptr(), outs[0].data_ptr(), self._stream(stream))
            return outs[0]
        klay_backward_lits(self._h, dout.data_ptr(), outs[0].data_ptr(), outs[1].data_ptr(), self._stream(stream))
        return outs[0], outs[1]

    def forward_f64(self, leaf_weights, semiring=KLAY_LOG, stream=None, neg_weights=None):
        """Double-precision evaluation: leaf_weights (and neg_weights) torch float64 CUDA [B, V]."""
        import torch
        for t in (leaf_weights, neg_weights):
            if t is not None and (t.dtype != torch.float64 or not t.is_cuda or not t.is_contiguous()
                                  or t.dim() != 2 or t.shape[1] != self.num_vars):
                raise ValueError("weights must be contiguous float64 CUDA tensors [B, %d]" % self.num_vars)
        if neg_weights is not None and neg_weights.shape != leaf_weights.shape:
            raise ValueError("neg_weights must have the shape of leaf_weights")
        B = leaf_weights.shape[0]
        out = torch.empty((B, self.num_roots), dtype=torch.float64, device=leaf_weights.device)
        klay_forward_f64(self._h, leaf_weights.data_ptr(), None if neg_weights is None else neg_weights.data_ptr(), B,
                         out.data_ptr(), int(semiring), self._stream(stream))
        self._last64 = (B, neg_weights is not None)
        return out

    def backward_f64(self, dout, stream=None):
        """dout float64 CUDA [B, R]; returns dleaf, or (dpos, dneg) after a forward pass with neg_weights."""
        import torch
        B, lits = getattr(self, "_last64", (None, False))
        if B is None:
            raise KlayError(KLAY_ESTATE, "backward_f64 before forward_f64")
        if dout.dtype != torch.float64 or not dout.is_cuda or not dout.is_contiguous() or dout.shape != (B, self.num_roots):
            raise ValueError("dout must be a contiguous float64 CUDA tensor [B, R]")
        dpos = torch.empty((B, self.num_vars), dtype=torch.float64, device=dout.device)
        dneg = torch.empty_like(dpos) if lits else None
        klay_backward_f64(self._h, dout.data_ptr(), dpos.data_ptr(), None if dneg is None else dneg.data_ptr(),
                          self._stream(stream))
        return (dpos, dneg) if lits else dpos

    def close(self):
        if self._h is not None:
            klay_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Builder:
    """Collects circuits over the same variables and builds them as one multi-rooted circuit."""

    def __init__(self, num_vars):
        self._b = None
        self._b = klay_builder_create(int(num_vars))

    def add(self, node_type, node_lit, child_ptr, child_idx, roots) -> int:
        """Adds one circuit; returns the column of ``out`` its first root will occupy."""
        node_type = np.ascontiguousarray(node_type, dtype=np.uint8)
        node_lit = np.ascontiguousarray(node_lit, dtype=np.int32)
        child_ptr = np.ascontiguousarray(child_ptr, dtype=np.int64)
        child_idx = np.ascontiguousarray(child_idx, dtype=np.int32)
        roots = np.ascontiguousarray(roots, dtype=np.int32)
        if node_lit.shape[0] != node_type.shape[0] or child_ptr.shape[0] != node_type.shape[0] + 1:
            raise ValueError("node_type, node_lit and child_ptr sizes disagree")
        if child_idx.shape[0] != child_ptr[-1]:
            raise ValueError("child_idx must have child_ptr[-1] entries")
        return klay_builder_add(self._b, node_type.shape[0], _np_ptr(node_type), _np_ptr(node_lit),
                                _np_ptr(child_ptr), _np_ptr(child_idx) if child_idx.size else None,
                                roots.shape[0], _np_ptr(roots))

    def finish(self, device=0, no_reorder=False, heavy_fan=0, min_segment=0, no_tail=False,
               unary_chains=False, no_merge=False, small_batch_edges=False, tail_rows_cap=0, no_fusion=False) -> Circuit:
        opts = klay_options(int(no_reorder), int(heavy_fan), int(min_segment), int(no_tail), int(unary_chains),
                            int(no_merge), int(small_batch_edges), int(tail_rows_cap), int(no_fusion))
        return Circuit._from_handle(klay_builder_finish(self._b, int(device), opts), device)

    def close(self):
        if self._b is not None:
            klay_builder_destroy(self._b)
            self._b = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
