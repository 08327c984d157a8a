"""The circuit as a differentiable PyTorch layer (the paper's use: a network predicts the leaf
weights, the circuit turns them into query probabilities, the loss is back-propagated through
both; Sections 1 and 6).  Marshalling only: the forward call is ``klay_forward``, the backward call
``klay_backward`` on the same handle, on torch's current stream.

The handle keeps the activations of its most recent forward pass only, so each backward must
belong to that pass: evaluating the layer again before calling ``backward()`` on an earlier result
raises instead of returning the wrong gradient.
"""
from __future__ import annotations

import torch

from .binding import KLAY_LOG, KLAY_MAXLOG, Circuit


class _Evaluate(torch.autograd.Function):
    @staticmethod
    def forward(ctx, weights, neg_weights, layer):
        w = weights.contiguous()
        wn = None if neg_weights is None else neg_weights.contiguous()
        out = layer.circuit.forward(w, layer.semiring, neg_weights=wn)
        layer._ticket += 1
        ctx.layer, ctx.ticket, ctx.lits = layer, layer._ticket, wn is not None
        return out

    @staticmethod
    def backward(ctx, dout):
        layer = ctx.layer
        if ctx.ticket != layer._ticket:
            raise RuntimeError("this circuit was evaluated again after the forward pass being differentiated; "
                               "its activations are gone (use one CircuitLayer per concurrent graph)")
        if ctx.lits:
            dpos, dneg = layer.circuit.backward(dout.contiguous())
            return dpos, dneg, None
        return layer.circuit.backward(dout.contiguous()), None, None


class CircuitLayer(torch.nn.Module):
    """``out[B, R] = circuit(weights[B, V])`` with gradients to ``weights`` (float32, CUDA).

    ``semiring``: ``KLAY_LOG`` (weights are log-probabilities) or ``KLAY_REAL`` (probabilities);
    ``KLAY_MAXLOG`` can be evaluated under ``torch.no_grad()`` only.  ``neg_weights`` gives the negated
    literals weights of their own (default: ``1 - p``, in the log domain ``log(1 - exp(x))``); both
    arrays then receive gradients.
    """

    def __init__(self, circuit: Circuit, semiring: int = KLAY_LOG):
        super().__init__()
        self.circuit = circuit
        self.semiring = int(semiring)
        self._ticket = 0

    def forward(self, weights, neg_weights=None):
        needs_grad = torch.is_grad_enabled() and (
            weights.requires_grad or (neg_weights is not None and neg_weights.requires_grad))
        if self.semiring == KLAY_MAXLOG and needs_grad:
            raise RuntimeError("the (max, +) semiring is not differentiated; evaluate it under torch.no_grad()")
        if not needs_grad:
            self._ticket += 1
            return self.circuit.forward(weights.contiguous(), self.semiring,
                                        neg_weights=None if neg_weights is None else neg_weights.contiguous())
        return _Evaluate.apply(weights, neg_weights, self)
