"""LF-MMI objective as a torch.autograd.Function on top of the C ABI (Eq. 2, Eq. 3).

Argument marshalling only: both forward-backward passes, the objective and its
gradient with respect to the logits all come out of lfmmi_loss; this
file stores that gradient for backward() and scales it by the incoming gradient.
"""
from __future__ import annotations

import numpy as np

from . import binding


def _function_class():
    import torch

    class _ChainObjective(torch.autograd.Function):
        @staticmethod
        def forward(ctx, logits, lengths, num_graphs, den_graph, leak):
            x = logits.detach()
            if x.dtype != torch.float32 or not x.is_contiguous():
                x = x.float().contiguous()
            # numerator minus denominator (Eq. 2 / Eq. 3), one call
            objf, grad, status = binding.lfmmi_loss(num_graphs, den_graph, x, lengths, leak)
            ctx.save_for_backward(grad)
            ctx.logits_dtype = logits.dtype
            ctx.mark_non_differentiable(status)
            return objf, status

        @staticmethod
        def backward(ctx, grad_objf, _grad_status):
            (grad,) = ctx.saved_tensors
            g = grad * grad_objf.reshape(-1, 1, 1).to(grad.dtype)
            return g.to(ctx.logits_dtype), None, None, None, None

    return _ChainObjective


_cls = None


def chain_objective(logits, lengths, num_graphs, den_graph, leak=1e-5):
    """Per-sequence objective log p(num) - log p(den) of Eq. 2, differentiable in `logits`.

    logits: CUDA float tensor [B, T, P]; lengths: host ints [B]; num_graphs: a batch
    handle with one numerator graph per sequence; den_graph: the shared denominator
    handle. Returns (objf [B], status [B]); the gradient is Eq. 3, the difference
    of the numerator and denominator pdf occupancies."""
    global _cls
    if _cls is None:
        _cls = _function_class()
    return _cls.apply(logits, np.asarray(lengths, dtype=np.int32), num_graphs, den_graph, float(leak))


def chain_loss(logits, lengths, num_graphs, den_graph, leak=1e-5):
    """Negative objective summed over the batch and divided by the number of frames
    (a scalar to minimise). Sequences flagged in `status` make it non-finite."""
    objf, _status = chain_objective(logits, lengths, num_graphs, den_graph, leak)
    frames = float(np.asarray(lengths, dtype=np.int64).sum())
    return -objf.sum() / max(frames, 1.0)
