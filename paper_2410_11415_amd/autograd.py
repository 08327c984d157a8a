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
    def forward(ctx, weights, layer):
        w = weights.contiguous()
        out = layer.circuit.forward(w, layer.semiring)
        layer._ticket += 1
        ctx.layer, ctx.ticket = layer, layer._ticket
        return out

    @staticmethod
    def backward(ctx, dout):
        layer = ctx.layer
        if ctx.ticket != layer._ticket:
            raise RuntimeError("this circuit was evaluated again after the forward pass being differentiated; "
                               "its activations are gone (use one CircuitLayer per concurrent graph)")
        return layer.circuit.backward(dout.contiguous()), None


class CircuitLayer(torch.nn.Module):
    """``out[B, R] = circuit(weights[B, V])`` with gradients to ``weights`` (float32, CUDA).

    ``semiring``: ``KLAY_LOG`` (weights are log-probabilities) or ``KLAY_REAL`` (probabilities);
    ``KLAY_MAXLOG`` can be evaluated under ``torch.no_grad()`` only.
    """

    def __init__(self, circuit: Circuit, semiring: int = KLAY_LOG):
        super().__init__()
        self.circuit = circuit
        self.semiring = int(semiring)
        self._ticket = 0

    def forward(self, weights):
        if self.semiring == KLAY_MAXLOG and torch.is_grad_enabled() and weights.requires_grad:
            raise RuntimeError("the (max, +) semiring is not differentiated; evaluate it under torch.no_grad()")
        if not (torch.is_grad_enabled() and weights.requires_grad):
            self._ticket += 1
            return self.circuit.forward(weights.contiguous(), self.semiring)
        return _Evaluate.apply(weights, self)
