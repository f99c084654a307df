"""Element-by-element comparison of the HIP path with the float64 oracle.

Tolerances (relative 1e-4; the absolute term 1e-7 is on the probability scale and only matters
where pi ~ mu makes the divergence itself that small):
  divergence : |gpu - ref| <= 1e-4 |ref| + 1e-7     (the exact full-vocabulary variants, whose
               divergence is a sum over all V entries in fp32: 3e-7, see ATOL_D_FULL)
  loss_tok   : |gpu - ref| <= 1e-4 |ref| + 1e-7 |A|   (compared under the GPU's own mask for
               tokens inside the exemption band)
  loss       : |gpu - ref| <= 1e-4 |ref| + 1e-7 * loss_scale * sum|A|
  mask       : bit-exact, except tokens with |D_ref - delta| < 1e-6 or, where the divergence can
               exceed delta while r is at 1 (Top-K and full-vocabulary variants),
               |log pi(a) - log mu(a)| < 1e-6;
               under the ratio-clip rule, except tokens with log r within 1e-6 of a clip boundary
  diagnostics: ratio 1e-4 rel; log pi(a) 1e-6 rel + 1e-6; |pi - mu| 1e-7; covered masses 2e-7 (fp32
               outputs near 1 carry 6e-8 of rounding by themselves); entropy 1e-4 rel + 1e-5
  grad_logits: |gpu - ref| <= 1e-2 |ref| + 1e-30   (bf16 output, round to nearest even); the
               sampled token's entry also gets the oracle's own float64 cancellation error
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import dppo_oracle as O

RTOL_D, ATOL_D = 1e-4, 1e-7
# Exact full-vocabulary TV / KL: the divergence itself is accumulated over all V entries in fp32
# with one hardware exponential per entry (relative error about 1e-7 each, common-mode part from
# the fp32 fraction of log2 S about 3e-8), so its absolute error is bounded by about 2e-7 of the
# total mass 1; 3e-7 leaves a margin of 1.5.
ATOL_D_FULL = 3e-7
RTOL_G, ATOL_G = 1e-2, 1e-30
BAND = 1e-6


def oracle_rows(batch: dict, rows, want_grad=True) -> dict:
    """Run the oracle on the given rows of a (device or host) batch."""
    idx = torch.as_tensor(np.asarray(rows, dtype=np.int64))
    dev = batch["logits"].device
    sel = idx.to(dev)
    V = batch["V"]
    z = batch["logits"][sel][:, :V].float().cpu().numpy()
    tk_i = batch["mu_topk_ids"][sel].cpu().numpy() if batch["mu_topk_ids"] is not None else None
    tk_l = batch["mu_topk_logp"][sel].cpu().numpy() if batch["mu_topk_logp"] is not None else None
    return O.dppo_loss(z, batch["sampled_ids"][sel].cpu().numpy(), batch["mu_logp"][sel].cpu().numpy(),
                       batch["advantages"][sel].cpu().numpy(), batch["delta"], batch["variant"],
                       batch["loss_scale"], tk_i, tk_l, want_grad=want_grad,
                       mu_logits=(batch["mu_logits"][sel][:, :V].float().cpu().numpy() if batch.get("mu_logits") is not None else None),
                       anchor_logp=(batch["anchor_logp"][sel].cpu().numpy() if batch.get("anchor_logp") is not None else None),
                       **batch.get("rule", {}))


def compare_rows(batch: dict, res: dict, rows, check_grad=True, row_offset=0, ref=None) -> dict:
    """Compare GPU outputs `res` (tensors indexed by row - row_offset) with the oracle on `rows`.
    Returns summary statistics (max errors, mask counts)."""
    rows = np.asarray(rows, dtype=np.int64)
    if ref is None:
        ref = oracle_rows(batch, rows, want_grad=check_grad)
    loc = torch.as_tensor(rows - row_offset).to(res["divergence"].device)
    D = res["divergence"][loc].double().cpu().numpy()
    M = res["mask"][loc].cpu().numpy()
    A = batch["advantages"][torch.as_tensor(rows).to(batch["advantages"].device)].double().cpu().numpy()
    delta = float(np.float32(batch["delta"]))
    # the policy the mask compares pi(a_t) with: the rollout policy unless the batch names another anchor
    lsrc = batch["anchor_logp"] if batch.get("anchor_logp") is not None else batch["mu_logp"]
    lmu = lsrc[torch.as_tensor(rows).to(lsrc.device)].double().cpu().numpy()

    with np.errstate(invalid="ignore"):
        errD = np.where(D == ref["divergence"], 0.0, np.abs(D - ref["divergence"]))      # equal infinities agree
    finite_ref = np.where(np.isfinite(ref["divergence"]), np.abs(ref["divergence"]), 0.0)
    atol_d = ATOL_D_FULL if batch["variant"] in (O.FULL_TV, O.FULL_KL) else ATOL_D
    assert np.all(errD <= RTOL_D * finite_ref + atol_d), \
        f"divergence: max err {errD.max():.3e} at row {rows[errD.argmax()]}"
    rule = batch.get("rule", {})
    mask_rule = rule.get("mask_rule", O.MASK_DIVERGENCE)
    if mask_rule == O.MASK_DIVERGENCE:
        exempt = np.abs(ref["divergence"] - delta) < BAND
        if batch["variant"] in (O.TOPK_TV, O.TOPK_KL, O.FULL_TV, O.FULL_KL):
            exempt |= np.abs(ref["logp"] - lmu) < BAND
    elif mask_rule == O.MASK_RATIO_CLIP:      # log r within the band of either clip boundary
        dl = ref["logp"] - lmu
        exempt = (np.abs(dl - np.log1p(rule["eps_high"])) < BAND) | (np.abs(dl - np.log1p(-rule["eps_low"])) < BAND)
    else:
        exempt = np.zeros(len(rows), dtype=bool)
    bad = (M != ref["mask"]) & ~exempt
    assert not bad.any(), f"mask differs outside the band at rows {rows[bad][:8]}"
    assert np.all((M == 0) | (M == 1))

    if res.get("loss_tok") is not None:
        lt = res["loss_tok"][loc].double().cpu().numpy()
        lt_ref = np.where(M == ref["mask"], ref["loss_tok"], -M * ref["weight"] * A)
        errL = np.abs(lt - lt_ref)
        assert np.all(errL <= RTOL_D * np.abs(lt_ref) + ATOL_D * np.abs(A)), f"loss_tok: max err {errL.max():.3e}"
    stats = {"max_abs_err_D": float(errD.max()) if len(rows) else 0.0, "masked": int((M == 0).sum()),
             "exempt": int(exempt.sum()), "rows": int(len(rows))}

    if res.get("diagnostics") is not None:
        dg = res["diagnostics"][loc].double().cpu().numpy()
        live = (np.asarray(ref["logp"]) != 0) | (np.asarray(ref["ratio"]) != 0)      # ignored rows: all zeros
        assert np.all(dg[~live] == 0)
        checks = (("ratio", 0, 1e-4, 1e-7), ("logp", 1, 1e-6, 1e-6), ("abs_diff", 2, 0.0, 1e-7),
                  ("entropy", 3, 1e-4, 1e-5), ("mass_mu", 4, 0.0, 2e-7), ("mass_pi", 5, 0.0, 2e-7))
        for name, col, rtol, atol in checks:
            got, want = dg[live, col], np.asarray(ref[name], dtype=np.float64)[live]
            with np.errstate(invalid="ignore"):
                err = np.where(got == want, 0.0, np.abs(got - want))      # equal infinities (log 0) agree
                ok = err <= rtol * np.abs(want) + atol
            assert np.all(ok), f"diagnostics {name}: max err {err.max():.3e}"
        assert np.all(dg[:, 6:] == 0)
        stats["max_abs_err_entropy"] = float(np.abs(dg[live, 3] - ref["entropy"][live]).max()) if live.any() else 0.0

    if check_grad and res.get("grad_logits") is not None:
        V = batch["V"]
        g = res["grad_logits"][loc][:, :V].float().cpu().numpy().astype(np.float64)
        g_ref = ref["grad_logits"].copy()
        flip = M != ref["mask"]          # exempt tokens: compare under the GPU's mask
        for i in np.nonzero(flip)[0]:
            if M[i] == 0:
                g_ref[i] = 0.0
            else:
                row = oracle_single_grad_unmasked(batch, int(rows[i]))
                g_ref[i] = row
        err = np.abs(g - g_ref)
        tol = RTOL_G * np.abs(g_ref) + ATOL_G
        # The oracle forms the sampled token's entry as c*(pi_a - 1) in float64: when pi_a -> 1
        # that difference carries the oracle's own rounding, 2^-52 * |c|.  Allow for it there.
        a_ids = batch["sampled_ids"][torch.as_tensor(rows).to(batch["sampled_ids"].device)].cpu().numpy()
        c_ref = np.abs(batch["loss_scale"] * M * A * ref["weight"])
        for i, a in enumerate(a_ids):
            if 0 <= a < V:
                tol[i, a] += 4 * np.finfo(np.float64).eps * c_ref[i]
        if not np.all(err <= tol):
            i, j = np.unravel_index(np.argmax(err - tol), err.shape)
            raise AssertionError(f"grad_logits row {rows[i]} col {j}: gpu {g[i, j]:.6e} ref {g_ref[i, j]:.6e}")
        nz = g_ref != 0
        stats["max_rel_err_grad"] = float((err[nz] / np.abs(g_ref[nz])).max()) if nz.any() else 0.0
    return stats


def oracle_single_grad_unmasked(batch: dict, row: int) -> np.ndarray:
    """Oracle gradient of one row with M forced to 1."""
    b = dict(batch)
    b["rule"] = dict(batch.get("rule", {}), mask_rule=O.MASK_NONE)
    return oracle_rows(b, [row])["grad_logits"][0]


def check_loss_scalar(batch: dict, res: dict, ref_loss_tok_sum: float | None = None):
    """loss == loss_scale * sum(loss_tok) (GPU-internal consistency, any size) and, if the
    oracle's sum is given, agreement with it."""
    lt = res["loss_tok"].double().sum().item()
    A_abs = batch["advantages"].double().abs().sum().item() if res["loss_tok"].numel() == batch["advantages"].numel() else None
    got = float(res["loss"].item())
    want = batch["loss_scale"] * lt
    assert abs(got - want) <= 2e-6 * abs(want) + 1e-7 * batch["loss_scale"] * (A_abs or 1.0) + 1e-12, (got, want)
    if ref_loss_tok_sum is not None:
        ref = batch["loss_scale"] * ref_loss_tok_sum
        assert abs(got - ref) <= 1e-4 * abs(ref) + ATOL_D * batch["loss_scale"] * (A_abs or 1.0), (got, ref)
