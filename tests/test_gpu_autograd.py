"""The torch.autograd wrapper of the loss: loss.backward() must deliver the fused kernel's gradient
(argument marshalling only: compared with the oracle like every other GPU result)."""
import numpy as np
import pytest
import torch

from paper_2602_04879_amd import autograd as A
from paper_2602_04879_amd import binding as B
from paper_2602_04879_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _call(b, logits, **kw):
    K = b["K"]
    return A.dppo_loss(logits, b["sampled_ids"], b["mu_logp"], b["advantages"], delta=b["delta"], variant=b["variant"],
                       loss_scale=b["loss_scale"], mu_topk_ids=b["mu_topk_ids"] if K else None,
                       mu_topk_logp=b["mu_topk_logp"] if K else None, **kw)


@pytest.mark.parametrize("variant,K,V", [(W.BINARY_TV, 0, 4096), (W.TOPK_KL, 20, 16384), (W.BINARY_KL, 0, 3001)])
def test_backward_delivers_the_fused_gradient(variant, K, V):
    w = W.Workload("autograd", 3, 40, V, variant, 0.05 if variant in (W.BINARY_KL, W.TOPK_KL) else 0.2, K=K,
                   logit_std=3.0, noise_std=1.0, adv="normal", seed=91)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    print(f"[case] autograd variant={variant} K={K} V={V} T={b['T']}", flush=True)
    rows = np.arange(b["T"])
    ref = P.oracle_rows(b, rows)
    logits = b["logits"].clone().requires_grad_(True)
    loss, aux = _call(b, logits, diagnostics=True)
    assert loss.requires_grad and not aux["divergence"].requires_grad
    loss.backward()
    torch.cuda.synchronize()
    res = dict(aux, loss=loss.detach().reshape(1), grad_logits=logits.grad)
    st = P.compare_rows(b, res, rows, ref=ref)
    P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    assert 0 < st["masked"] < b["T"]
    # the gradient of 3 * loss is 3 * the gradient, rounded once more to bf16
    logits3 = b["logits"].clone().requires_grad_(True)
    loss3, _ = _call(b, logits3)
    (3.0 * loss3).backward()
    torch.cuda.synchronize()
    want = (logits.grad.float() * 3.0).to(torch.bfloat16)
    assert torch.equal(logits3.grad, want)
    # without a gradient path the forward-only entry point runs and nothing is allocated for a gradient
    with torch.no_grad():
        loss0, aux0 = _call(b, b["logits"])
    torch.cuda.synchronize()
    assert not loss0.requires_grad
    assert torch.equal(aux0["divergence"], aux["divergence"]) and torch.equal(aux0["mask"], aux["mask"])
    assert abs(loss0.item() - loss.item()) <= 1e-6 * abs(loss.item()) + 1e-12


def test_in_place_gradient_over_the_logits():
    w = W.Workload("autograd_inplace", 2, 64, 16384, W.TOPK_TV, 0.1, K=8, logit_std=3.0, noise_std=1.0, adv="normal", seed=93)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    keep = b["logits"].clone().requires_grad_(True)
    loss_ref, _ = _call(b, keep)
    loss_ref.backward()
    leaf = b["logits"].clone().requires_grad_(True)
    storage = leaf.data_ptr()
    loss, _ = _call(b, leaf, in_place=True)
    loss.backward()
    torch.cuda.synchronize()
    assert torch.equal(leaf.grad, keep.grad) and torch.equal(loss.detach(), loss_ref.detach())
    assert leaf.grad.data_ptr() == storage          # the gradient lives in the logits' own storage


def test_hidden_state_form_backward_matches_the_direct_call():
    w = W.Workload("autograd_lm", 2, 150, 4160, W.TOPK_TV, 0.1, K=8, logit_std=3.0, noise_std=1.0, adv="normal", seed=95)
    b = W.make_lmhead_batch(w, 128, DEV, exact=True, shift_sampled=2.0)
    gw_ref = torch.empty((b["V"], b["d"]), dtype=torch.float32, device=DEV)
    ref = B.run_lmhead(b, chunk_rows=64, grad_weight=gw_ref)
    h = b["hidden"].clone().requires_grad_(True)
    wt = b["weight"].clone().requires_grad_(True)
    loss, aux = A.dppo_lmhead_loss(h, wt, b["sampled_ids"], b["mu_logp"], b["advantages"], delta=b["delta"], variant=b["variant"],
                                   loss_scale=b["loss_scale"], mu_topk_ids=b["mu_topk_ids"], mu_topk_logp=b["mu_topk_logp"], chunk_rows=64)
    loss.backward()
    torch.cuda.synchronize()
    assert torch.equal(loss.detach().reshape(1), ref["loss"]) and torch.equal(aux["mask"], ref["mask"])
    assert torch.equal(aux["divergence"], ref["divergence"])
    assert torch.equal(h.grad, ref["grad_hidden"])
    assert torch.equal(wt.grad, gw_ref.to(torch.bfloat16))
    assert 0 < (aux["mask"] == 0).sum().item() < b["T"]
    # forward only (no gradient path): no logit is written, same per-token results up to summation order
    with torch.no_grad():
        loss0, aux0 = A.dppo_lmhead_loss(b["hidden"], b["weight"], b["sampled_ids"], b["mu_logp"], b["advantages"], delta=b["delta"],
                                         variant=b["variant"], loss_scale=b["loss_scale"], mu_topk_ids=b["mu_topk_ids"],
                                         mu_topk_logp=b["mu_topk_logp"], chunk_rows=64)
    torch.cuda.synchronize()
    assert B.last_path() == "lmhead_fused"
    assert torch.equal(aux0["mask"], ref["mask"])
    assert torch.allclose(aux0["divergence"], ref["divergence"], rtol=1e-4, atol=1e-7)
