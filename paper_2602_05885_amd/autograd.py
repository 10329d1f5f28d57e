"""torch.autograd glue for trainers: the fused head as a loss whose backward is already done.

The library computes the loss and both gradients in one call (the backward needs the forward's
logsumexp and nothing else from it), so these Functions run that call in `forward`, keep dH and dW,
and hand them out in `backward`.  They only marshal arguments and hold tensors; every step of the
computation runs in the library's kernels.  The loss tensor they return is meant to be the last
node of the graph (`loss.backward()`, upstream gradient 1; scale the loss through
params.norm_override instead of multiplying it afterwards).  With scale_by_upstream=True the
upstream gradient is applied to dH and dW with one in-place multiply each (an extra pass over both).

    loss, aux = pg_head_loss(H, W, y, loss_mask, cu_seqlens, adv, seg_sample, old_logp, rollout_logp, params)
    loss.backward()            # H.grad is dH, W.grad is dW

`aux` holds the per-token log-probs, entropies and the counters (no gradient flows through them).
autograd hands W.grad over in the dtype of W (it casts the fp32 dW the C ABI writes); a trainer that
keeps fp32 gradients, or accumulates over microbatches, passes its own accumulator as `dW_accum`
(with params.accumulate_dW = 1 to add into it) and then receives no W.grad from here.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class _HeadLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, H, W, sft, y, loss_mask, cu_seqlens, adv, seg_sample, sample_keep, old_logp, rollout_logp,
                params, workspace, dW_accum, aux, scale_by_upstream):
        T, d = H.shape
        V = W.shape[0]
        if workspace is None:
            S = 0 if sft else cu_seqlens.numel() - 1
            workspace = B.alloc_workspace(T, d, V, S, params, B.CALL_LOSS_FWD_BWD, H.device)
        Hd, Wd = H.detach(), W.detach()
        if sft:
            out = B.pg_sft_fwd_bwd(Hd, Wd, y, loss_mask, params, workspace, dW=dW_accum)
        else:
            out = B.pg_loss_fwd_bwd(Hd, Wd, y, loss_mask, cu_seqlens, adv, seg_sample, old_logp, rollout_logp, params,
                                    workspace, dW=dW_accum, sample_keep=sample_keep)
        ctx.save_for_backward(out["dH"], out["dW"])
        ctx.external_dW = dW_accum is not None
        ctx.scale_by_upstream = scale_by_upstream
        aux.update(logp=out["logp"], entropy=out["entropy"], counters=out["counters"])
        return out["loss"].reshape(())

    @staticmethod
    def backward(ctx, grad_loss):
        dH, dW = ctx.saved_tensors
        if ctx.scale_by_upstream:          # no host sync: the scalar stays on the device
            dH = dH.mul_(grad_loss.to(dH.dtype))
            if not ctx.external_dW:
                dW = dW.mul_(grad_loss.to(dW.dtype))
        return (dH, None if ctx.external_dW else dW) + (None,) * 14


def pg_head_loss(H, W, y, loss_mask, cu_seqlens, adv, seg_sample, old_logp, rollout_logp, params: B.Params,
                 workspace: Optional[torch.Tensor] = None, sample_keep: Optional[torch.Tensor] = None,
                 dW_accum: Optional[torch.Tensor] = None, scale_by_upstream: bool = False):
    """Mismatch-corrected clipped policy-gradient loss of the LM head (see pg_loss_fwd_bwd in pg_head.h).

    Returns (loss, aux); loss is a 0-d tensor attached to H and W."""
    aux = {}
    loss = _HeadLoss.apply(H, W, False, y, loss_mask, cu_seqlens, adv, seg_sample, sample_keep, old_logp, rollout_logp,
                           params, workspace, dW_accum, aux, scale_by_upstream)
    return loss, aux


def sft_head_loss(H, W, y, loss_mask, params: B.Params, workspace: Optional[torch.Tensor] = None,
                  dW_accum: Optional[torch.Tensor] = None, scale_by_upstream: bool = False):
    """Token-mean cross-entropy of the LM head (see pg_sft_fwd_bwd in pg_head.h).  Returns (loss, aux)."""
    aux = {}
    loss = _HeadLoss.apply(H, W, True, y, loss_mask, None, None, None, None, None, None, params, workspace, dW_accum,
                           aux, scale_by_upstream)
    return loss, aux
