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
                           eps_high=opts.get("eps_high", 0.2), ratio_cap=opts.get("ratio_cap", 0.0), flags=opts.get("flags", 0),
                           anchor_logp=opts.get("anchor_logp"), relax_alpha=opts.get("relax_alpha", 0.0),
                           relax_sides=opts.get("relax_sides", 0))
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
    unified gradient form), anchor_logp (the mask anchored to a recomputed policy: MiniRL, the
    decoupled objective), relax_alpha / relax_sides (the clip relaxed for low-probability tokens),
    diagnostics, in_place, flags."""
    opts = dict(opts, delta=float(delta), variant=int(variant), loss_scale=float(loss_scale))
    res = _DppoLoss.apply(logits, sampled_ids, mu_logp, advantages, mu_topk_ids, mu_topk_logp, mu_logits, opts)
    aux = {"divergence": res[1], "mask": res[2], "loss_tok": res[3]}
    if len(res) > 4:
        aux["diagnostics"] = res[4]
    return res[0], aux


class _DppoLmheadLoss(torch.autograd.Function):
    @staticmethod
    def forward(ctx, hidden, weight, sampled_ids, mu_logp, advantages, mu_topk_ids, mu_topk_logp, opts):
        if hidden.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16 or hidden.dim() != 2 or weight.dim() != 2:
            raise ValueError("hidden [T, d] and weight [V, d]: bf16 matrices on the GPU")
        if hidden.stride(1) != 1 or weight.stride(1) != 1 or hidden.shape[1] != weight.shape[1]:
            raise ValueError("hidden and weight: contiguous rows of the same length d")
        T, d = hidden.shape
        V = weight.shape[0]
        need_h, need_w = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        backward = need_h or need_w
        batch = {"hidden": hidden.detach(), "weight": weight.detach(), "d": d, "V": V, "sampled_ids": sampled_ids, "mu_logp": mu_logp,
                 "advantages": advantages, "delta": opts["delta"], "variant": opts["variant"], "loss_scale": opts["loss_scale"],
                 "mu_topk_ids": mu_topk_ids, "mu_topk_logp": mu_topk_logp, "anchor_logp": opts.get("anchor_logp")}
        gw = torch.empty((V, d), dtype=torch.float32, device=hidden.device) if need_w else None
        rule = {k: opts[k] for k in ("mask_rule", "eps_low", "eps_high", "ratio_cap", "relax_alpha", "relax_sides") if k in opts}
        res = B.run_lmhead(batch, backward=backward, chunk_rows=opts.get("chunk_rows", 0), diagnostics=opts.get("diagnostics", False),
                           grad_weight=gw, flags=opts.get("flags", 0), **rule)
        ctx.grads = (res["grad_hidden"] if need_h else None, gw)
        side = [res[k] for k in ("divergence", "mask", "loss_tok")] + ([res["diagnostics"]] if res["diagnostics"] is not None else [])
        ctx.mark_non_differentiable(*side)
        return (res["loss"].reshape(()), *side)

    @staticmethod
    def backward(ctx, grad_loss, *unused):
        gh, gw = ctx.grads
        ctx.grads = None
        one = _is_one(grad_loss)
        if gh is not None and not one:
            gh = (gh.float() * grad_loss.float()).to(torch.bfloat16)
        if gw is not None:
            # the library accumulates the weight's gradient in fp32; autograd wants the weight's own type
            gw = (gw if one else gw * grad_loss.float()).to(torch.bfloat16)
        return (gh, gw, None, None, None, None, None, None)


def dppo_lmhead_loss(hidden, weight, sampled_ids, mu_logp, advantages, *, delta, variant=B.BINARY_TV, loss_scale=1.0,
                     mu_topk_ids=None, mu_topk_logp=None, **opts):
    """The same loss one step earlier (dppo_lmhead_loss_fwd[_bwd] of include/dppo.h): from the final
    hidden states [T, d] and the lm_head weight [V, d], both bf16; the logits exist a chunk of
    tokens at a time inside the call (forward only: never).  Returns the loss, with gradient paths
    to `hidden` and `weight`, and the per-token outputs.  Options as for dppo_loss, plus chunk_rows."""
    opts = dict(opts, delta=float(delta), variant=int(variant), loss_scale=float(loss_scale))
    res = _DppoLmheadLoss.apply(hidden, weight, sampled_ids, mu_logp, advantages, mu_topk_ids, mu_topk_logp, opts)
    aux = {"divergence": res[1], "mask": res[2], "loss_tok": res[3]}
    if len(res) > 4:
        aux["diagnostics"] = res[4]
    return res[0], aux
