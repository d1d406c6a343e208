"""The fused call as a differentiable PyTorch loss, for trainers whose model body lives in PyTorch.

    loss = iw_pg_loss(hidden, W, tokens, mask, logp_behav, rewards, group_ids, K)
    loss.backward()          # hidden.grad / W.grad (and the body's parameters through hidden)

rapid_iw_pg_loss_fwd_bwd computes the loss of one IW-GRPG mini-batch (Alg. 1; Eq. (3) with the
advantages of Eq. (5)) together with its gradients with respect to the hidden states and the LM
head, so the autograd node only hands those over, scaled by the incoming gradient.  Every number is
produced by the library; this module marshals tensors.  The advantages are constants of the
gradient (Eq. (3) differentiates log pi only), exactly as in the library call.
"""
from __future__ import annotations

import torch

from . import binding as rb


class _IwPgLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, hidden, W, tokens, mask, logp_behav, rewards, group_ids, K, opts):
        out = rb.rapid_iw_pg_loss_fwd_bwd(hidden.detach().contiguous(), W.detach().contiguous(), tokens, mask,
                                          logp_behav, rewards, group_ids, K, **opts)
        ctx.save_for_backward(out.dhidden, out.dW)
        ctx.w_dtype = W.dtype
        ctx.outputs = out                       # diagnostics for the caller: loss.rapid_outputs
        return out.loss.reshape(())

    @staticmethod
    def backward(ctx, grad_loss):
        dh, dW = ctx.saved_tensors
        g = grad_loss.to(torch.float32)
        return ((dh.float() * g).to(dh.dtype), (dW.float() * g).to(ctx.w_dtype), None, None, None, None, None, None,
                None)


def iw_pg_loss(hidden, W, tokens, mask, logp_behav, rewards, group_ids, K, **opts):
    """Scalar loss tensor of rapid_iw_pg_loss_fwd_bwd, differentiable with respect to `hidden` and `W`
    (layout given by opts["w_layout"], default [d, V]).  `opts` are the keyword options of
    binding.rapid_iw_pg_loss_fwd_bwd (eta, coef_mode, baseline_mode, loss_scale, temperature,
    logits_cache, ratio_level, max_tokens, ...), except rms_weight: the final norm belongs to the
    caller's PyTorch graph here.  The per-call outputs (log-probs, ratios, advantages, diagnostics)
    are reachable as `loss.grad_fn.outputs` until the graph is freed."""
    if "rms_weight" in opts or "buffers" in opts:
        raise ValueError("rms_weight / buffers are not supported through the autograd wrapper")
    return _IwPgLoss.apply(hidden, W, tokens, mask, logp_behav, rewards, group_ids, K, opts)
