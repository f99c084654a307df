"""dppo_loss_fwd_bwd_static (the entry point for callers that cannot allocate: no workspace
argument, the partial sums live in the library's own static device array) against
dppo_loss_fwd_bwd, through the C ABI: two calls in a row on the same GPU, the second with a
smaller input, every output bit for bit (both run the same kernels; only the home of the
partial sums differs), plus the stated limit."""
import ctypes as C

import pytest
import torch

from paper_2602_04879_amd import binding as B
from paper_2602_04879_amd import workloads as W

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
KEYS = ("loss", "loss_tok", "divergence", "mask", "diagnostics")


def _both(w, shift=2.0):
    b = W.make_batch(w, DEV, shift_sampled=shift)
    ref = B.run_batch(b, diagnostics=True)                       # the existing entry point, caller's workspace
    path = B.last_path()
    out = B.alloc_outputs(b["T"], DEV, want_diagnostics=True)
    out["workspace"] = None                                      # nothing for the library to scribble on
    grad = torch.empty_like(b["logits"])
    a = B.make_args(b["logits"], b["sampled_ids"], b["mu_logp"], b["advantages"], b["delta"], b["variant"], b["loss_scale"],
                    out, b["mu_topk_ids"], b["mu_topk_logp"], V=b["V"], grad_logits=grad)
    a.ld = b["ld"]
    assert a.workspace is None and a.workspace_bytes == 0
    print(f"[case] static entry point {w.name} T={b['T']} V={b['V']} K={b['K']} variant={b['variant']}", flush=True)
    B.dppo_loss_fwd_bwd_static(a)
    torch.cuda.synchronize()
    assert B.last_path() == path
    for k in KEYS:
        assert torch.equal(ref[k], out[k]), k
    assert torch.equal(ref["grad_logits"], grad)
    assert 0 < (out["mask"] == 0).sum().item() < b["T"]
    return path


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    big = W.Workload("static_big", 3, 250, 16384, W.TOPK_TV, 0.1, K=20, logit_std=3.0, noise_std=1.0, adv="normal", seed=51)
    small = W.Workload("static_small", 2, 9, 3001, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=1.0, adv="normal", seed=52)
    tiny = W.Workload("static_tiny", 2, 9, 601, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=1.0, adv="normal", seed=52)
    assert B.lib().dppo_static_init() == 0
    assert _both(big) == "resident"          # 750 rows on every compute unit: all partial sums in use
    assert _both(small) == "resident"        # then a smaller call: 18 workgroups (ragged rows), stale sums beside them
    assert _both(tiny) == "streaming"        # and the two-pass kernel
    assert _both(big) == "resident"


def test_static_scratch_entry_point_limits():
    w = W.Workload("static_err", 1, 4, 64, W.BINARY_TV, 0.1, seed=1)
    b = W.make_batch(w, DEV)
    out = B.alloc_outputs(b["T"], DEV)
    out["workspace"] = None
    a = B.make_args(b["logits"], b["sampled_ids"], b["mu_logp"], b["advantages"], 0.1, W.BINARY_TV, 1.0, out,
                    grad_logits=torch.empty_like(b["logits"]))
    a.T = (1 << 22) + 1                      # beyond DPPO_STATIC_MAX_T: rejected on the host, nothing launched
    with pytest.raises(B.DppoError) as e:
        B.dppo_loss_fwd_bwd_static(a)
    assert e.value.status == 2
    a.T = b["T"]
    a.grad_logits = None
    with pytest.raises(B.DppoError) as e:
        B.dppo_loss_fwd_bwd_static(a)
    assert e.value.status == 1
    torch.cuda.synchronize()
