"""torch.autograd front end of the C-ABI library (argument marshalling only: every number comes out of
rnnt_joint_loss_fwd_bwd_weighted).

    loss = rnnt_joint_loss(enc, pred, W_out, b_out, labels, T_len, U_len, blank=0)     # [B], -ln P(y_b|x_b)
    loss.sum().backward()        # or loss.mean(), (loss * mask).sum(), ...

The library computes the loss and all gradients in one call (Algorithm 1 of the paper: the gradients of the
output layer are accumulated while the samples are walked, nothing is kept for a later backward pass), so the
forward of the autograd function already holds the gradients of sum_b w_b loss_b for the weights w it was
given (default: ones).  backward() hands them out if the incoming gradient of the loss vector equals those
weights, and otherwise calls the library once more with the incoming gradient as the weights.  Pass
`sample_weight` (e.g. 1/B for a mean) to make the first call the only one.  The weights of the library are
non-negative, so the gradient that reaches the loss vector must be >= 0 for every sample (backward raises
otherwise).  The forward call's outputs and workspace stay alive until backward has run.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as Bd


class _RnntJointLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, enc, pred, W_out, b_out, labels, T_len, U_len, blank, sample_weight, workspace, keep_scores):
        if not (enc.is_cuda and enc.is_contiguous() and pred.is_contiguous() and W_out.is_contiguous()):
            raise ValueError("enc, pred, W_out must be contiguous CUDA tensors")
        B, T_max, H = enc.shape
        U_max = pred.shape[1] - 1
        V = W_out.shape[1]
        dtype = Bd.RNNT_BF16 if enc.dtype == torch.bfloat16 else Bd.RNNT_F32
        T_host = np.ascontiguousarray(T_len, dtype=np.int32)
        U_host = np.ascontiguousarray(U_len, dtype=np.int32)
        w_host = np.ones(B, dtype=np.float32) if sample_weight is None else \
            np.ascontiguousarray(sample_weight, dtype=np.float32)
        dev = dict(enc=enc, pred=pred, W_out=W_out, b_out=b_out, labels=labels, T_len=T_host, U_len=U_host)
        shape = (B, T_max, U_max, H, V, int(blank), dtype)
        # bf16 leaves get bf16 gradients: the library rounds them itself instead of a conversion pass here
        opts = dict(keep_scores=int(keep_scores), input_grads_bf16=int(dtype == Bd.RNNT_BF16))
        out = Bd.run_fwd_bwd(dev, *shape, workspace=workspace, sample_weight=w_host, **opts)
        ctx.dev, ctx.shape, ctx.w_host, ctx.out, ctx.opts = dev, shape, w_host, out, opts
        ctx.mark_non_differentiable(labels)
        return out["loss"]

    @staticmethod
    def backward(ctx, grad_loss):
        g = grad_loss.detach().float().cpu().numpy()          # B numbers; also orders this after the forward
        if not (np.all(np.isfinite(g)) and np.all(g >= 0.0)):
            # the library takes one weight >= 0 per sample (they scale posterior probabilities in log space)
            raise ValueError("rnnt_joint_loss: the gradient reaching the loss vector must be finite and >= 0 for "
                             "every sample (sum, mean, masks and positive scalings are; a negated loss is not)")
        out = ctx.out
        if not np.array_equal(g, ctx.w_host):
            out = Bd.run_fwd_bwd(ctx.dev, *ctx.shape, workspace=ctx.out["workspace"], sample_weight=g, **ctx.opts)
        enc, W_out, b_out = ctx.dev["enc"], ctx.dev["W_out"], ctx.dev["b_out"]
        return (out["d_enc"].to(enc.dtype), out["d_pred"].to(enc.dtype), out["dW_out"].to(W_out.dtype),
                out["db_out"].to(b_out.dtype), None, None, None, None, None, None, None)


def rnnt_joint_loss(enc, pred, W_out, b_out, labels, T_len, U_len, blank: int = 0, sample_weight=None,
                    workspace=None, keep_scores: bool = False):
    """Per-sample transducer loss [B] with gradients for enc, pred, W_out, b_out.

    enc [B,T_max,H], pred [B,U_max+1,H], W_out [H,V] (float32 or bfloat16, CUDA, contiguous), b_out [V] float32,
    labels [B,U_max] int32 on the device, T_len / U_len host arrays of B int32.  sample_weight: host array of B
    non-negative floats, the weights the loss vector is going to be summed with (None: ones).  keep_scores
    (bfloat16 only): the descriptor field of that name, scores kept in a larger workspace instead of computed twice."""
    return _RnntJointLoss.apply(enc, pred, W_out, b_out, labels, T_len, U_len, blank, sample_weight, workspace,
                                keep_scores)
