"""MI355X-native layered arithmetic-circuit evaluator (KLay hot path): HIP kernels behind a C ABI.

``binding`` holds the ctypes layer over ``lib/libklay.so``; ``build`` compiles it with hipcc.
"""
from .binding import (KLAY_AND, KLAY_FALSE, KLAY_LIT, KLAY_LOG, KLAY_MAXLOG, KLAY_OR, KLAY_REAL, KLAY_STATIC_WORKSPACE_BYTES, KLAY_TRUE,
                      Builder, Circuit,
                      KlayError, klay_backward, klay_backward_f64, klay_backward_lits, klay_build, klay_destroy, klay_forward,
                      klay_forward_f64, klay_forward_lits, klay_forward_static, klay_last_error,
                      library_path, load)

__all__ = ["KLAY_AND", "KLAY_FALSE", "KLAY_LIT", "KLAY_LOG", "KLAY_MAXLOG", "KLAY_OR", "KLAY_REAL", "KLAY_STATIC_WORKSPACE_BYTES",
           "KLAY_TRUE", "Builder", "Circuit",
           "KlayError", "klay_backward", "klay_backward_f64", "klay_backward_lits", "klay_build", "klay_destroy", "klay_forward",
           "klay_forward_f64", "klay_forward_lits", "klay_forward_static", "klay_last_error",
           "library_path", "load"]


def __getattr__(name):
    # the torch layer is imported on first use, so that the binding alone does not need torch
    if name == "CircuitLayer":
        from .autograd import CircuitLayer
        return CircuitLayer
    raise AttributeError(name)
