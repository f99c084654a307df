"""Float64 CPU oracle for the DPPO per-token divergence trust-region loss.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
GPU library is checked against.  It is imported by the tests, by the smoke
check and by the benchmark's CPU-baseline leg; no product code path may call
it.  It shares no code with the HIP kernels and imports nothing from the
product package.

Everything is numpy float64, one row (one response token) at a time, in the
order and notation of the paper:

  * log-softmax of the trainer logits            (Sec. 3, token distribution pi(.|s_t))
  * ratio r_t = pi(a_t|s_t) / mu(a_t|s_t), mu the ROLLOUT policy
                                                  (Eq. ppo-clip; Sec. 5.2 Takeaway 2)
  * Binary-TV / Binary-KL                         (Eq. binary_tv, Eq. binary_kl)
  * Top-K reduced distributions, TV and KL        (Sec. 4.4 "Top-K Approximation",
                                                   Eq. topk_tv, Eq. topk_kl)
  * DPPO mask and masked surrogate                (Eq. dppo_obj)
  * gradient wrt the logits, mask held constant   (Eq. unified_grad with C = infinity)
  * exact full-vocabulary TV / KL (brute force)   (App. B, definitions of D_TV, D_KL); also as
    the divergence of the trust region itself when the rollout policy's full logits are given
  * the baselines' masks and the ratio cap         (App. C.1: unified gradient form,
                                                    Eq. unified_grad; PPO/GRPO clip mask;
                                                    M = 1 for PG-IS / CISPO; cap C)
  * the same path from the final hidden states and the lm_head weight (logits formed inside,
    gradient with respect to the hidden states), Sec. 4.4's memory concern
  * per-token health metrics the paper monitors   (App. F.1: |pi - mu| of the sampled token,
    (diagnostics)                                   policy entropy; App. B.1: mass covered by
                                                    the top-K set)

Readings taken where the paper is silent:
  - the library returns the quantity to MINIMISE: loss = -loss_scale * sum_t M_t r_t A_t;
    loss_scale is the caller's normalisation (the paper writes an expectation of a sum);
  - KL is D(mu || pi) in nats;
  - comparisons are strict, and "r > 1" is evaluated as log pi(a) > log mu(a);
  - x*log(x/y) = 0 when x = 0; a vanishing denominator y is floored at 1e-30 (the exact
    full-vocabulary KL used as a trust region has no floor: it is infinite where pi excludes a
    token that mu can sample);
  - mu probabilities > 1 from rounding are clamped to 1, and the "other" bucket of either
    policy is clamped to >= 0;
  - a top-K id equal to a_t is dropped (a_t's own mu log-prob is used), ids outside [0, V)
    are padding;
  - a row whose sampled id is outside [0, V) is ignored: D = 0, M = 0, loss term 0, zero
    gradient row;
  - with a finite ratio cap C the gradient is the one Eq. unified_grad states,
    M min(r, C) A grad log pi (the weight is a constant), and the reported loss term is
    -M min(r, C) A; "r > 1 + eps" of the clip mask is evaluated as
    log pi(a) - log mu(a) > log(1 + eps).

  - from hidden states: the logits are the exact product h W^T rounded ONCE to bfloat16 (what a
    bf16 lm_head with wide accumulation hands over), and that rounding passes gradients through.

All pins for these functions live in tests/test_oracle_*.py.  "parity unpinned": the loss
normalisation (the paper fixes no minibatch formula; it is the caller's loss_scale) and the
VALUE reported as loss under a finite ratio cap (the paper defines only the gradient there).
"""
from __future__ import annotations

import numpy as np

BINARY_TV, BINARY_KL, TOPK_TV, TOPK_KL, FULL_TV, FULL_KL = 0, 1, 2, 3, 4, 5
MASK_DIVERGENCE, MASK_RATIO_CLIP, MASK_NONE = 0, 1, 2
RELAX_HIGH, RELAX_LOW = 1, 2      # which clip threshold goes to infinity for low-probability tokens (Sec. 6)
VARIANT_NAMES = {BINARY_TV: "binary_tv", BINARY_KL: "binary_kl",
                 TOPK_TV: "topk_tv", TOPK_KL: "topk_kl",
                 FULL_TV: "full_tv", FULL_KL: "full_kl"}
_TINY = 1e-30


# --------------------------------------------------------------------------- softmax
def log_softmax(z):
    """log pi_j = z_j - (m + ln sum_j exp(z_j - m)) for one row z[V]  (Sec. 3)."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max()
    S = np.exp(z - m).sum()
    return z - (m + np.log(S))


# --------------------------------------------------------------------------- divergences
def _xlogx_over_y(x, y):
    """x * ln(x / y) with 0*ln 0 = 0 and y floored at 1e-30 (reading for saturated cases)."""
    if x <= 0.0:
        return 0.0
    return x * (np.log(x) - np.log(max(y, _TINY)))


def binary_tv(lmu_a, lpi_a):
    """|mu(a_t) - pi(a_t)|  (Eq. binary_tv)."""
    p = np.exp(min(lmu_a, 0.0))
    q = np.exp(lpi_a)
    return abs(p - q)


def binary_kl(lmu_a, lpi_a, one_minus_q=None):
    """mu ln(mu/pi) + (1-mu) ln((1-mu)/(1-pi))  (Eq. binary_kl).

    one_minus_q, when given, is sum_{j != a} pi_j computed from the full row (avoids
    1 - q cancellation); otherwise -expm1(lpi_a) is used.
    """
    lmu_a = min(lmu_a, 0.0)
    p = np.exp(lmu_a)
    q = np.exp(lpi_a)
    one_minus_p = -np.expm1(lmu_a)
    if one_minus_q is None:
        one_minus_q = -np.expm1(min(lpi_a, 0.0))
    return _xlogx_over_y(p, q) + _xlogx_over_y(one_minus_p, one_minus_q)


def reduced_distributions(logpi, a, lmu_a, topk_ids, topk_logp):
    """Reduced categorical distributions over A'' = TopK(mu, K) U {a_t} U {other}.

    Returns (p, q, p_other, q_other) with p, q arrays over A' (a_t first).  For tokens in
    A' the probabilities are the original ones; "other" is one minus their sum, clamped at
    0 (Sec. 4.4, Top-K Approximation).
    """
    ids = [int(a)]
    p = [np.exp(min(float(lmu_a), 0.0))]
    if topk_ids is not None:
        for i, lp in zip(np.asarray(topk_ids).tolist(), np.asarray(topk_logp, dtype=np.float64).tolist()):
            if i < 0 or i >= len(logpi) or i == int(a):
                continue  # padding (id outside the vocabulary), or a_t already present
            ids.append(int(i))
            p.append(np.exp(min(lp, 0.0)))
    p = np.asarray(p, dtype=np.float64)
    q = np.exp(logpi[np.asarray(ids, dtype=np.int64)])
    p_other = max(1.0 - p.sum(), 0.0)
    q_other = max(1.0 - q.sum(), 0.0)
    return p, q, p_other, q_other


def topk_tv(p, q, p_other, q_other):
    """1/2 sum_{A''} |p^mu - p^pi|  (Eq. topk_tv)."""
    return 0.5 * (np.abs(p - q).sum() + abs(p_other - q_other))


def topk_kl(p, q, p_other, q_other):
    """sum_{A''} p^mu ln(p^mu / p^pi)  (Eq. topk_kl)."""
    d = 0.0
    for x, y in zip(p.tolist(), q.tolist()):
        d += _xlogx_over_y(x, y)
    return d + _xlogx_over_y(p_other, q_other)


def full_tv(mu_probs, pi_probs):
    """Exact D_TV = 1/2 sum_a |mu(a) - pi(a)|  (App. B.1)."""
    mu_probs = np.asarray(mu_probs, dtype=np.float64)
    pi_probs = np.asarray(pi_probs, dtype=np.float64)
    return 0.5 * np.abs(mu_probs - pi_probs).sum()


def full_kl(mu_probs, pi_probs):
    """Exact D_KL(mu || pi) = sum_a mu(a) ln(mu(a)/pi(a))  (App. B.2)."""
    d = 0.0
    for x, y in zip(np.asarray(mu_probs, dtype=np.float64).tolist(),
                    np.asarray(pi_probs, dtype=np.float64).tolist()):
        d += _xlogx_over_y(x, y)
    return d


def full_kl_from_logs(lmu, lpi):
    """Exact D_KL(mu || pi) = sum_a mu(a) (ln mu(a) - ln pi(a)) from the two rows of log-probs
    (App. B.2), with 0 ln 0 = 0 and no floor: a token pi excludes (ln pi = -inf) that mu can
    still sample makes the divergence infinite, as the definition does."""
    lmu = np.asarray(lmu, dtype=np.float64)
    lpi = np.asarray(lpi, dtype=np.float64)
    d = 0.0
    for x, y in zip(lmu.tolist(), lpi.tolist()):
        if x == -np.inf:
            continue
        d += np.exp(x) * (x - y)
    return d


def entropy(logpi):
    """Token entropy -sum_j pi_j ln pi_j in nats, 0 ln 0 = 0  (the "policy entropy" of App. F.1)."""
    logpi = np.asarray(logpi, dtype=np.float64)
    pi = np.exp(logpi)
    nz = pi > 0.0
    return float(-(pi[nz] * logpi[nz]).sum())


# --------------------------------------------------------------------------- mask
def dppo_mask(D, delta, adv, lpi_a, lmu_a):
    """M_t of Eq. dppo_obj: 0 iff D > delta and the update moves r further from 1 in the
    direction the advantage favours; 1 otherwise.  r > 1 is tested as lpi_a > lmu_a."""
    if D > delta and ((adv > 0.0 and lpi_a > lmu_a) or (adv < 0.0 and lpi_a < lmu_a)):
        return 0
    return 1


def ratio_clip_mask(adv, lpi_a, lmu_a, eps_low, eps_high):
    """PPO / GRPO(-ClipHigher) mask of App. C.1 and App. E: 0 iff (A > 0 and r > 1 + eps_high) or
    (A < 0 and r < 1 - eps_low), 1 otherwise; r compared in the log domain."""
    d = lpi_a - lmu_a
    # an infinite eps_high never blocks; eps_low >= 1 puts the lower bound at or below 0, which no ratio undercuts
    hi = np.log1p(eps_high)
    lo = np.log1p(-eps_low) if eps_low < 1.0 else -np.inf
    if (adv > 0.0 and d > hi) or (adv < 0.0 and d < lo):
        return 0
    return 1


# --------------------------------------------------------------------------- whole path
def dppo_loss(logits, sampled_ids, mu_logp, advantages, delta, variant, loss_scale=1.0,
              mu_topk_ids=None, mu_topk_logp=None, want_grad=True,
              mask_rule=MASK_DIVERGENCE, eps_low=0.2, eps_high=0.2, ratio_cap=None,
              mu_logits=None, anchor_logp=None, relax_alpha=0.0, relax_sides=0):
    """The whole hot path for T rows.

    logits [T, V] (any float dtype; widened to float64), sampled_ids [T] int,
    mu_logp [T], advantages [T], optional mu_topk_ids / mu_topk_logp [T, K].
    mask_rule picks M_t: the DPPO divergence mask (default), the PPO/GRPO ratio-clip mask with
    eps_low / eps_high, or none (M = 1: PG-IS, CISPO).  ratio_cap is C of Eq. unified_grad
    (None or inf: no cap).  The FULL_TV / FULL_KL variants take the trust region on the exact
    divergence between the two next-token distributions (App. B) and need mu_logits [T, V], the
    rollout policy's logits (any shift of a row is immaterial); the ratio still uses mu_logp.
    anchor_logp [T] (optional): log-prob of a_t under the policy the MASK is anchored to when that
    is not the rollout policy, i.e. the trainer's recomputed pi_theta' (App. C.1: MiniRL and
    MiniRL-TIS clip on r' = pi / pi_theta'; Sec. 5.2: the decoupled DPPO, whose divergence and
    r' <> 1 test are taken against pi_theta').  It replaces mu_logp in the divergence and in the
    mask; the weight min(r, C) and the loss keep r = pi / mu (Eq. unified_grad).
    relax_alpha, relax_sides (ratio-clip mask only; Sec. 6): for tokens the ROLLOUT policy gave a
    probability below alpha, the upper clip threshold (RELAX_HIGH), the lower one (RELAX_LOW) or both
    are set to infinity.  mu(a_t) < alpha is evaluated as log mu(a_t) < log alpha.
    Returns a dict: loss (float), loss_tok [T], divergence [T], mask [T] uint8,
    ratio [T], logp [T] (log pi(a_t)), lse [T], grad_logits [T, V] float64 or None, and the
    diagnostics abs_diff [T] = |pi(a_t) - mu(a_t)|, entropy [T], mass_mu [T], mass_pi [T]
    (probability mu resp. pi puts on A' = TopK(mu, K) U {a_t}; A' = {a_t} for the Binary variants).
    """
    logits = np.asarray(logits, dtype=np.float64)
    T, V = logits.shape
    sampled_ids = np.asarray(sampled_ids, dtype=np.int64)
    mu_logp = np.asarray(mu_logp, dtype=np.float64)
    advantages = np.asarray(advantages, dtype=np.float64)
    topk = variant in (TOPK_TV, TOPK_KL)
    if variant not in VARIANT_NAMES:
        raise ValueError("unknown variant")
    if variant in (FULL_TV, FULL_KL) and mu_logits is None:
        raise ValueError("the full-vocabulary variants need mu_logits")

    out = {
        "loss_tok": np.zeros(T), "divergence": np.zeros(T), "mask": np.zeros(T, dtype=np.uint8),
        "ratio": np.zeros(T), "logp": np.zeros(T), "lse": np.zeros(T),
        "abs_diff": np.zeros(T), "entropy": np.zeros(T), "mass_mu": np.zeros(T), "mass_pi": np.zeros(T),
        "weight": np.zeros(T),
        "grad_logits": np.zeros((T, V)) if want_grad else None,
    }
    for t in range(T):
        a = int(sampled_ids[t])
        if a < 0 or a >= V:
            continue  # ignored row (id outside the vocabulary): everything stays 0
        z = logits[t]
        logpi = log_softmax(z)                       # step 1
        lpi = logpi[a]
        lmu = float(mu_logp[t])
        r = np.exp(lpi - lmu)                        # step 2
        lanc = lmu if anchor_logp is None else float(anchor_logp[t])     # the mask's anchor policy at a_t
        mass_mu, mass_pi = np.exp(min(lanc, 0.0)), np.exp(lpi)
        if variant == BINARY_TV:                     # step 3
            D = binary_tv(lanc, lpi)
        elif variant == BINARY_KL:
            pi_row = np.exp(logpi)
            one_minus_q = pi_row[:a].sum() + pi_row[a + 1:].sum()
            D = binary_kl(lanc, lpi, one_minus_q)
        elif variant in (FULL_TV, FULL_KL):
            logmu = log_softmax(np.asarray(mu_logits[t], dtype=np.float64))
            D = full_tv(np.exp(logmu), np.exp(logpi)) if variant == FULL_TV else full_kl_from_logs(logmu, logpi)
            mass_mu, mass_pi = 1.0, 1.0              # A' is the whole vocabulary
        else:
            ids = mu_topk_ids[t] if (mu_topk_ids is not None) else None
            lps = mu_topk_logp[t] if (mu_topk_logp is not None) else None
            p, q, po, qo = reduced_distributions(logpi, a, lanc, ids, lps)
            D = topk_tv(p, q, po, qo) if variant == TOPK_TV else topk_kl(p, q, po, qo)
            mass_mu, mass_pi = p.sum(), q.sum()
        A = float(advantages[t])
        if mask_rule == MASK_DIVERGENCE:             # step 4
            M = dppo_mask(D, delta, A, lpi, lanc)
        elif mask_rule == MASK_RATIO_CLIP:
            lo_eps, hi_eps = eps_low, eps_high
            if relax_alpha > 0.0 and lmu < np.log(float(relax_alpha)):      # a low-probability token (Sec. 6)
                if relax_sides & RELAX_HIGH:
                    hi_eps = np.inf
                if relax_sides & RELAX_LOW:
                    lo_eps = np.inf
            M = ratio_clip_mask(A, lpi, lanc, lo_eps, hi_eps)
        elif mask_rule == MASK_NONE:
            M = 1
        else:
            raise ValueError("unknown mask rule")
        w = r if (ratio_cap is None or not np.isfinite(ratio_cap)) else min(r, float(ratio_cap))
        out["divergence"][t] = D
        out["mask"][t] = M
        out["ratio"][t] = r
        out["weight"][t] = w
        out["logp"][t] = lpi
        out["lse"][t] = z[a] - lpi
        out["abs_diff"][t] = binary_tv(lanc, lpi)
        out["entropy"][t] = entropy(logpi)
        out["mass_mu"][t] = mass_mu
        out["mass_pi"][t] = mass_pi
        out["loss_tok"][t] = -M * w * A              # step 5
        if want_grad:                                # step 6
            g = np.exp(logpi)
            g[a] -= 1.0
            out["grad_logits"][t] = (loss_scale * M * A * w) * g
    out["loss"] = float(loss_scale * out["loss_tok"].sum())
    return out


# --------------------------------------------------------------------------- from the hidden states
def bf16_round(x):
    """Round float64 values to the nearest bfloat16 (8 significant bits, ties to even), returned
    as float64.  Normal range only (no subnormals, no overflow): what logits need."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def lmhead_logits(hidden, weight):
    """The trainer's bf16 logits z = h W^T: the exact product, rounded once to bfloat16."""
    hidden = np.asarray(hidden, dtype=np.float64)
    weight = np.asarray(weight, dtype=np.float64)
    return bf16_round(hidden @ weight.T)


def lmhead_dppo_loss(hidden, weight, sampled_ids, mu_logp, advantages, delta, variant, loss_scale=1.0,
                     mu_topk_ids=None, mu_topk_logp=None, want_grad=True, **rule):
    """The whole path from the final hidden states h [T, d] and the lm_head weight W [V, d]
    (the memory-saving form of Sec. 4.4's concern: no [T, V] array is needed outside this oracle):
    logits as the trainer's lm_head produces them, dppo_loss on them, and the gradient with respect
    to the hidden states by the chain rule, d loss / d h = (d loss / d z) W, the rounding of the
    logits passing gradients through unchanged; likewise d loss / d W = (d loss / d z)^T h for the
    lm_head weight.  Returns dppo_loss's dict plus logits, grad_hidden [T, d] and grad_weight [V, d]
    (None without want_grad)."""
    z = lmhead_logits(hidden, weight)
    out = dppo_loss(z, sampled_ids, mu_logp, advantages, delta, variant, loss_scale, mu_topk_ids, mu_topk_logp,
                    want_grad=want_grad, **rule)
    out["logits"] = z
    out["grad_hidden"] = out["grad_logits"] @ np.asarray(weight, dtype=np.float64) if want_grad else None
    out["grad_weight"] = out["grad_logits"].T @ np.asarray(hidden, dtype=np.float64) if want_grad else None
    return out
