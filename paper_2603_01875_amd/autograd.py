"""torch.autograd front end of the library: the distillation loss as a differentiable scalar.

The forward call runs the whole fused path (loss AND both gradients come out of one
kd_loss_fwd_bwd); backward only scales the stored gradients by the incoming scalar (the one
PyTorch op here: the chain rule through whatever the caller does with the loss).  No step of the
method runs in PyTorch: this module is argument marshalling, like kdloss.py.
"""
from __future__ import annotations

import torch

from . import kdloss as K


class _KDLossFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, h_s, W_s, h_t, W_t, mask, tau, kind, beta, w_layout, flags, teacher_scale, workspace,
                loss_scale):
        out = K.kd_loss_fwd_bwd(h_t, W_t, h_s, W_s, mask, tau=tau, kind=kind, beta=beta, w_layout=w_layout,
                                workspace=workspace, want_per_token=False, flags=flags,
                                teacher_scale=teacher_scale, loss_scale=loss_scale)
        ctx.save_for_backward(out["grad_h_s"], out["grad_W_s"])
        return out["loss"].reshape(())

    @staticmethod
    def backward(ctx, g):
        grad_h, grad_W = ctx.saved_tensors
        return (grad_h * g.to(grad_h.dtype), grad_W * g.to(grad_W.dtype)) + (None,) * 11


def kd_loss(h_s, W_s, h_t, W_t, mask=None, tau=1.0, kind=K.FKL, beta=0.5, w_layout=K.W_VH, flags=0,
            teacher_scale=0.0, workspace=None, loss_scale=1.0):
    """Masked-mean divergence between softmax(h_t W_t / tau) and softmax(h_s W_s / tau) as a scalar
    tensor; gradients flow to h_s and W_s (the teacher side is frozen).  Arguments as in
    kdloss.kd_loss_fwd_bwd.  A factor that is known before the call (1 / micro-batches, a loss weight)
    belongs in `loss_scale`: the library folds it into the loss and both gradients at no cost, whereas
    whatever multiplies the returned scalar afterwards costs backward() one more pass over the
    gradients (they are formed in forward, before that factor exists)."""
    return _KDLossFn.apply(h_s, W_s, h_t, W_t, mask, float(tau), int(kind), float(beta), int(w_layout),
                           int(flags), float(teacher_scale), workspace, float(loss_scale))
