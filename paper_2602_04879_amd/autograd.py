"""The loss as a torch.autograd.Function, for a trainer that wants `loss.backward()`.

Argument marshalling only.  The library computes the loss and its gradient with respect to the
logits in ONE pass (dppo_loss_fwd_bwd of include/dppo.h: Eq. dppo_obj for the loss, Eq.
unified_grad for the gradient, the mask a constant), so `forward` already holds the gradient and
`backward` only hands it over, scaled by the incoming gradient of the scalar loss.  There is no
CPU fallback: without the HIP library the call raises.

    loss, aux = dppo_loss(logits, sampled_ids, mu_logp, advantages, delta=0.2, variant=BINARY_TV,
                          loss_scale=1.0 / T)
    loss.backward()            # logits.grad (bf16) is the fused kernel's gradient

`aux` holds the per-token divergence, mask and loss terms (no gradient flows through them).
With `in_place=True` the gradient is written over the logits' own storage (allowed by the
boundary): the logits are then consumed by the call, as a fused cross-entropy would consume them.
"""
from __future__ import annotations

import torch

from . import binding as B


class _DppoLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, logits, sampled_ids, mu_logp, advantages, mu_topk_ids, mu_topk_logp, mu_logits, opts):
        if logits.dtype != torch.bfloat16 or logits.dim() != 2 or not logits.is_cuda:
            raise ValueError("logits: a bf16 [T, V] tensor on the GPU")
        if logits.stride(1) != 1:
            raise ValueError("logits: rows must be contiguous")
        T = logits.shape[0]
        out = B.alloc_outputs(T, logits.device, want_diagnostics=opts.get("diagnostics", False))
        need_grad = ctx.needs_input_grad[0]
        grad = None
        if need_grad:
            grad = logits.detach() if opts.get("in_place", False) else torch.empty_like(logits)
        args = B.make_args(logits.detach(), sampled_ids, mu_logp, advantages, opts["delta"], opts["variant"], opts["loss_scale"], out,
                           mu_topk_ids, mu_topk_logp, grad_logits=grad, mu_logits=mu_logits,
                           mask_rule=opts.get("mask_rule", B.MASK_DIVERGENCE), eps_low=opts.get("eps_low", 0.2),
                           eps_high=opts.get("eps_high", 0.2), ratio_cap=opts.get("ratio_cap", 0.0), flags=opts.get("flags", 0))
        (B.dppo_loss_fwd_bwd if need_grad else B.dppo_loss_fwd)(args)
        ctx.grad_logits = grad
        side = [out[k] for k in ("divergence", "mask", "loss_tok")] + ([out["diagnostics"]] if out["diagnostics"] is not None else [])
        ctx.mark_non_differentiable(*side)
        return (out["loss"].reshape(()), *side)

    @staticmethod
    def backward(ctx, grad_loss, *unused):
        g = ctx.grad_logits
        ctx.grad_logits = None
        if g is None:
            return (None,) * 8
        # d(out)/d(logits) = grad_loss * d(loss)/d(logits); the scale is applied in fp32 and rounded once
        g = (g.float() * grad_loss.float()).to(torch.bfloat16) if not _is_one(grad_loss) else g
        return (g, None, None, None, None, None, None, None)


def _is_one(t: torch.Tensor) -> bool:
    # the usual case, loss.backward(): a scalar one, known on the host only at the cost of a
    # synchronisation, which one scalar read is
    return t.numel() == 1 and float(t) == 1.0


def dppo_loss(logits, sampled_ids, mu_logp, advantages, *, delta, variant=B.BINARY_TV, loss_scale=1.0,
              mu_topk_ids=None, mu_topk_logp=None, mu_logits=None, **opts):
    """loss (a 0-d fp32 tensor with a gradient path to `logits`) and a dict of the per-token
    outputs.  Keyword options: mask_rule, eps_low, eps_high, ratio_cap (the baselines of the
    unified gradient form), diagnostics, in_place, flags."""
    opts = dict(opts, delta=float(delta), variant=int(variant), loss_scale=float(loss_scale))
    res = _DppoLoss.apply(logits, sampled_ids, mu_logp, advantages, mu_topk_ids, mu_topk_logp, mu_logits, opts)
    aux = {"divergence": res[1], "mask": res[2], "loss_tok": res[3]}
    if len(res) > 4:
        aux["diagnostics"] = res[4]
    return res[0], aux
