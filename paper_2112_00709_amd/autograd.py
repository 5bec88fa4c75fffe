"""LF-MMI objective as a differentiable PyTorch function on the GPU.

The network's output (pseudo-log-likelihoods, Sec. 3 of the paper) goes in, the
objective of Eq. 16 comes out; its derivative with respect to every network
output (Eq. 17: numerator minus denominator pdf posteriors) was already
computed by ``lfmmi_loss_grad`` in the forward call and is only scaled by the
incoming gradient in the backward call.  Splitting a batch into sub-batches and
calling ``backward`` once per sub-batch accumulates the parameter gradients of
the whole batch (the B/F scheme of the paper's training recipe), since the
objective is a sum over utterances.
"""
from __future__ import annotations

from typing import Optional

from . import Graph, fb_lfmmi_workspace_bytes, lfmmi_loss_grad


def _torch():
    import torch
    return torch


def _make_function():
    torch = _torch()

    class _LFMMI(torch.autograd.Function):
        @staticmethod
        def forward(ctx, emis, lengths, den, num, ws, lengths_host):
            if emis.dtype != torch.float32 or not emis.is_cuda:
                raise TypeError("emis must be a float32 tensor on the GPU")
            loss, zn, zd, grad = lfmmi_loss_grad(den, num, emis.contiguous(), lengths, ws=ws, lengths_host=lengths_host)
            ctx.save_for_backward(grad)
            ctx.mark_non_differentiable(zn, zd)
            return loss, zn, zd

        @staticmethod
        def backward(ctx, g_loss, _g_zn, _g_zd):
            (grad,) = ctx.saved_tensors
            return grad * g_loss.to(grad.dtype), None, None, None, None, None

    return _LFMMI


_fn = None


def lfmmi_loss(emis, lengths, den: Graph, num: Graph, ws: Optional[object] = None, lengths_host=None):
    """-> (loss [1] float64 (sum over utterances of log Z_num - log Z_den), logz_num [B], logz_den [B]).

    ``emis``: float32 CUDA tensor [B, N, D] that may require grad; ``lengths``: int32 CUDA tensor [B];
    ``den``: shared denominator graph; ``num``: packed numerator graphs of the same B utterances;
    ``ws``: optional reusable workspace (uint8 CUDA tensor of ``fb_lfmmi_workspace_bytes`` bytes);
    ``lengths_host``: optional host copy of ``lengths`` (the launches of the call are then scheduled by them).
    """
    global _fn
    if _fn is None:
        _fn = _make_function()
    return _fn.apply(emis, lengths, den, num, ws, lengths_host)


def workspace(den: Graph, num: Graph, B: int, N: int, D: int, device="cuda"):
    torch = _torch()
    return torch.empty((fb_lfmmi_workspace_bytes(den, num, B, N, D),), dtype=torch.uint8, device=device)
