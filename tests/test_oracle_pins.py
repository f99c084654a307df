"""Pins for the float64 oracle: each test ties one part of oracle/dppo_oracle.py to
something other than itself -- values the paper prints, a library routine, a closed form,
a theorem of App. B, brute force on tiny vocabularies, finite differences, autograd."""
import math
import os

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

from oracle import dppo_oracle as O
from paper_2602_04879_amd import workloads as W

RNG = np.random.default_rng(20260204)


def _rand_dist(V, peaked=False):
    z = RNG.normal(0, 3.0 if peaked else 1.0, size=V)
    p = np.exp(z - z.max())
    return p / p.sum()


def _logits_for(probs):
    """Logits whose softmax is exactly `probs` (up to float64 rounding)."""
    return np.log(np.asarray(probs, dtype=np.float64))


# ------------------------------------------------------------------ log-softmax (Sec. 3)
@pytest.mark.parametrize("V", [1, 2, 7, 1000])
def test_log_softmax_matches_library(V):
    z = RNG.normal(0, 5, size=V) + 30.0
    got = O.log_softmax(z)
    np.testing.assert_allclose(got, scipy.special.log_softmax(z), rtol=0, atol=1e-12)
    assert abs(np.exp(got).sum() - 1.0) < 1e-12
    # shift invariance and no overflow at large offsets
    np.testing.assert_allclose(O.log_softmax(z + 1e4), got, atol=1e-9)


# ------------------------------------------------------------------ paper's worked example
def _worked_rows(golden_dir):
    rows = {}
    with open(os.path.join(golden_dir, "worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, mu, pi, r, d = line.split()
            rows[name] = tuple(map(float, (mu, pi, r, d)))
    return rows


def _row_with(pi_a, V=50, a=3):
    """A logits row whose softmax gives exactly pi_a to token a, the rest spread randomly."""
    rest = _rand_dist(V - 1) * (1.0 - pi_a)
    probs = np.insert(rest, a, pi_a)
    return _logits_for(probs)


def test_worked_example_ratio_divergence_mask(golden_dir):
    rows = _worked_rows(golden_dir)
    a = 3
    for name, (mu, pi, r_printed, d_printed) in rows.items():
        z = _row_with(pi, a=a)
        for adv in (+1.0, -1.0):
            out = O.dppo_loss(z[None, :], [a], [math.log(mu)], [adv], delta=0.2, variant=O.BINARY_TV)
            assert out["ratio"][0] == pytest.approx(r_printed, rel=1e-3)   # 0.808 is printed to 3 digits
            assert out["divergence"][0] == pytest.approx(d_printed, rel=1e-9)
    mu, pi, _, _ = rows["low"]
    z = _row_with(pi, a=a)
    # r = 100 with a positive advantage: PPO would clip it, DPPO keeps it (D = 0.0099 << delta)
    out = O.dppo_loss(z[None, :], [a], [math.log(mu)], [1.0], delta=0.15, variant=O.BINARY_TV)
    assert out["ratio"][0] == pytest.approx(100.0, rel=1e-12) and out["mask"][0] == 1
    mu, pi, _, _ = rows["high"]
    z = _row_with(pi, a=a)
    # r = 0.808 stays inside a 0.2 ratio clip, but removes 0.19 mass: blocked at delta_TV = 0.15
    # (App. C.1 threshold) for a negative advantage, allowed at delta_TV = 0.2 (App. E).
    for delta, adv, m in ((0.15, -1.0, 0), (0.2, -1.0, 1), (0.15, +1.0, 1)):
        out = O.dppo_loss(z[None, :], [a], [math.log(mu)], [adv], delta=delta, variant=O.BINARY_TV)
        assert out["mask"][0] == m, (delta, adv)


# ------------------------------------------------------------------ Binary-KL (Eq. binary_kl)
def test_binary_kl_is_bernoulli_kl_from_library():
    for _ in range(200):
        p, q = RNG.uniform(1e-6, 1 - 1e-6, size=2)
        ref = scipy.special.rel_entr([p, 1 - p], [q, 1 - q]).sum()
        assert O.binary_kl(math.log(p), math.log(q)) == pytest.approx(ref, rel=1e-9, abs=1e-15)
        assert O.binary_kl(math.log(p), math.log(q), one_minus_q=1 - q) == pytest.approx(ref, rel=1e-9, abs=1e-15)
        # Pinsker on the Bernoulli pair (Sec. 2): TV^2 <= KL / 2
        assert O.binary_tv(math.log(p), math.log(q)) ** 2 <= 0.5 * ref + 1e-15
    assert O.binary_kl(math.log(0.3), math.log(0.3)) == pytest.approx(0.0, abs=1e-16)
    # direction: D(mu || pi), not D(pi || mu)
    p, q = 0.9, 0.1
    assert O.binary_kl(math.log(p), math.log(q)) == pytest.approx(
        p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q)), rel=1e-12)
    p, q = 0.5, 0.01
    assert O.binary_kl(math.log(p), math.log(q)) != pytest.approx(O.binary_kl(math.log(q), math.log(p)))


def test_binary_saturation_readings():
    # mu log-prob slightly above 0 from fp32 noise: p clamps to 1, (1-p) term vanishes
    d = O.binary_kl(1e-7, math.log(0.9))
    assert d == pytest.approx(-math.log(0.9), rel=1e-12)
    assert O.binary_tv(1e-7, math.log(0.9)) == pytest.approx(0.1, rel=1e-12)
    # pi(a) == 1 exactly while mu(a) < 1: denominator floored -> finite and large
    d = O.binary_kl(math.log(0.5), 0.0, one_minus_q=0.0)
    assert np.isfinite(d) and d > 10.0


# ------------------------------------------------------------------ exact divergences (App. B)
def test_full_tv_and_kl_match_definitions_and_identities():
    for V in (2, 5, 64):
        mu, pi = _rand_dist(V, True), _rand_dist(V, True)
        tv = O.full_tv(mu, pi)
        # Eq. tv_as_expectation: D_TV = 1/2 E_{a~mu} |r(a) - 1|
        assert tv == pytest.approx(0.5 * (mu * np.abs(pi / mu - 1.0)).sum(), rel=1e-12)
        assert 0.0 <= tv <= 1.0
        assert O.full_kl(mu, pi) == pytest.approx(scipy.stats.entropy(mu, pi), rel=1e-10)
        assert tv ** 2 <= 0.5 * O.full_kl(mu, pi) + 1e-15      # Pinsker
    assert O.full_tv([1, 0], [0, 1]) == 1.0
    assert O.full_kl([0.5, 0.5, 0.0], [0.25, 0.25, 0.5]) == pytest.approx(math.log(2))  # 0 ln 0 = 0


# ------------------------------------------------------------------ Top-K (Sec. 4.4)
def _topk_inputs(mu, K, a):
    ids = np.argsort(-mu, kind="stable")[:K].astype(np.int64)
    return ids, np.log(mu[ids])


@pytest.mark.parametrize("variant_pair", [(O.BINARY_TV, O.TOPK_TV), (O.BINARY_KL, O.TOPK_KL)])
def test_topk_with_k0_is_binary(variant_pair):
    vb, vt = variant_pair
    V = 40
    for _ in range(20):
        mu, pi = _rand_dist(V, True), _rand_dist(V, True)
        a = int(RNG.integers(V))
        z = _logits_for(pi)[None, :]
        ob = O.dppo_loss(z, [a], [math.log(mu[a])], [1.0], 0.1, vb)
        ot = O.dppo_loss(z, [a], [math.log(mu[a])], [1.0], 0.1, vt)          # no top-K given
        ot2 = O.dppo_loss(z, [a], [math.log(mu[a])], [1.0], 0.1, vt,
                          mu_topk_ids=np.full((1, 3), -1), mu_topk_logp=np.zeros((1, 3)))  # all padding
        assert ot["divergence"][0] == pytest.approx(ob["divergence"][0], rel=1e-9, abs=1e-15)
        assert ot2["divergence"][0] == pytest.approx(ob["divergence"][0], rel=1e-9, abs=1e-15)


def test_topk_with_whole_vocabulary_is_exact_divergence():
    V = 24
    for _ in range(20):
        mu, pi = _rand_dist(V, True), _rand_dist(V, True)
        a = int(RNG.integers(V))
        z = _logits_for(pi)
        ids, lps = _topk_inputs(mu, V, a)          # K = V: "other" is empty
        p, q, po, qo = O.reduced_distributions(O.log_softmax(z), a, math.log(mu[a]), ids, lps)
        assert len(p) == V and po == pytest.approx(0, abs=1e-12) and qo == pytest.approx(0, abs=1e-12)
        assert O.topk_tv(p, q, po, qo) == pytest.approx(O.full_tv(mu, pi), rel=1e-9)
        assert O.topk_kl(p, q, po, qo) == pytest.approx(scipy.stats.entropy(mu, pi), rel=1e-9)
        ids, lps = _topk_inputs(mu, V - 1, a)      # K = V-1: "other" is a single token -> still exact
        p, q, po, qo = O.reduced_distributions(O.log_softmax(z), a, math.log(mu[a]), ids, lps)
        assert O.topk_tv(p, q, po, qo) == pytest.approx(O.full_tv(mu, pi), rel=1e-9)
        assert O.topk_kl(p, q, po, qo) == pytest.approx(scipy.stats.entropy(mu, pi), rel=1e-8)


def test_lower_bound_chain_binary_topk_full():
    """Coarsening cannot raise TV (triangle inequality) or KL (log-sum inequality): App. B.
    The Top-K partition refines the Binary one, so D_bin <= D_topK <= D_full; and the TV gap
    is at most half the mass both policies put on "other"."""
    V = 64
    for trial in range(100):
        mu, pi = _rand_dist(V, True), _rand_dist(V, True)
        a = int(RNG.choice(V, p=mu))
        K = int(RNG.integers(1, 12))
        ids, lps = _topk_inputs(mu, K, a)
        lpi = O.log_softmax(_logits_for(pi))
        p, q, po, qo = O.reduced_distributions(lpi, a, math.log(mu[a]), ids, lps)
        tv_b, tv_k, tv_f = O.binary_tv(math.log(mu[a]), lpi[a]), O.topk_tv(p, q, po, qo), O.full_tv(mu, pi)
        kl_b, kl_k, kl_f = O.binary_kl(math.log(mu[a]), lpi[a]), O.topk_kl(p, q, po, qo), O.full_kl(mu, pi)
        assert tv_b <= tv_k + 1e-14 <= tv_f + 2e-14
        assert -1e-15 <= kl_b <= kl_k + 1e-14 <= kl_f + 2e-14
        assert tv_f - tv_k <= 0.5 * (po + qo) + 1e-14
        assert tv_k ** 2 <= 0.5 * kl_k + 1e-15


def test_equality_conditions():
    V, K, a = 32, 5, 7
    mu = _rand_dist(V, True)
    ids, lps = _topk_inputs(mu, K, a)
    inside = set(ids.tolist()) | {a}
    tail = np.array([j for j in range(V) if j not in inside])
    # TV equality: mu - pi has one sign inside every cell.  Move mass from the tail
    # (every tail token loses) onto tokens of A'.
    pi = mu.copy()
    take = 0.5 * mu[tail]
    pi[tail] -= take
    pi[ids[0]] += take.sum()
    lpi = O.log_softmax(_logits_for(pi))
    p, q, po, qo = O.reduced_distributions(lpi, a, math.log(mu[a]), ids, lps)
    assert O.topk_tv(p, q, po, qo) == pytest.approx(O.full_tv(mu, pi), rel=1e-10)
    # ... and a tail perturbation of mixed sign leaves a strict gap
    pi2 = mu.copy()
    pi2[tail[0]] += 0.5 * mu[tail[1]]
    pi2[tail[1]] -= 0.5 * mu[tail[1]]
    lpi2 = O.log_softmax(_logits_for(pi2))
    p, q, po, qo = O.reduced_distributions(lpi2, a, math.log(mu[a]), ids, lps)
    assert O.topk_tv(p, q, po, qo) < O.full_tv(mu, pi2) - 1e-6
    # KL equality: mu/pi constant on "other" -> scale the whole tail by one factor
    pi3 = mu.copy()
    pi3[tail] *= 0.25
    pi3[ids[1]] += 0.75 * mu[tail].sum()
    lpi3 = O.log_softmax(_logits_for(pi3))
    p, q, po, qo = O.reduced_distributions(lpi3, a, math.log(mu[a]), ids, lps)
    assert O.topk_kl(p, q, po, qo) == pytest.approx(O.full_kl(mu, pi3), rel=1e-9)
    # Binary-KL equality: all tokens other than a_t scaled by one factor
    pi4 = mu.copy()
    pi4[a] = 0.5 * mu[a]
    others = np.arange(V) != a
    pi4[others] *= (1 - pi4[a]) / (1 - mu[a])
    lpi4 = O.log_softmax(_logits_for(pi4))
    assert O.binary_kl(math.log(mu[a]), lpi4[a]) == pytest.approx(O.full_kl(mu, pi4), rel=1e-9)
    assert O.binary_tv(math.log(mu[a]), lpi4[a]) == pytest.approx(O.full_tv(mu, pi4), rel=1e-9)


def test_topk_dedupes_sampled_token_and_skips_padding():
    V, a = 16, 2
    mu, pi = _rand_dist(V, True), _rand_dist(V, True)
    lpi = O.log_softmax(_logits_for(pi))
    ids = np.array([5, a, 9, -1])
    lps = np.log(mu[[5, a, 9, 0]])
    lps[1] = math.log(0.999)          # the top-K copy of a_t's log-prob must NOT be used
    p, q, po, qo = O.reduced_distributions(lpi, a, math.log(mu[a]), ids, lps)
    np.testing.assert_allclose(p, mu[[a, 5, 9]], rtol=1e-12)
    np.testing.assert_allclose(q, pi[[a, 5, 9]], rtol=1e-12)
    assert po == pytest.approx(1 - mu[[a, 5, 9]].sum(), rel=1e-12)
    assert qo == pytest.approx(1 - pi[[a, 5, 9]].sum(), rel=1e-12)
    # mu log-probs summing past 1 (fp32 noise): "other" clamps to 0, never negative
    p, q, po, qo = O.reduced_distributions(lpi, a, math.log(0.6), np.array([5]), np.array([math.log(0.5)]))
    assert po == 0.0


def test_topk_tv_hand_computed():
    # 4 tokens, A' = {0 (sampled), 1}, other = {2, 3}
    mu = np.array([0.5, 0.3, 0.15, 0.05])
    pi = np.array([0.4, 0.35, 0.05, 0.20])
    lpi = O.log_softmax(_logits_for(pi))
    p, q, po, qo = O.reduced_distributions(lpi, 0, math.log(0.5), np.array([1]), np.array([math.log(0.3)]))
    assert po == pytest.approx(0.2) and qo == pytest.approx(0.25)
    assert O.topk_tv(p, q, po, qo) == pytest.approx(0.5 * (0.1 + 0.05 + 0.05))
    assert O.full_tv(mu, pi) == pytest.approx(0.5 * (0.1 + 0.05 + 0.10 + 0.15))
    kl = 0.5 * math.log(0.5 / 0.4) + 0.3 * math.log(0.3 / 0.35) + 0.2 * math.log(0.2 / 0.25)
    assert O.topk_kl(p, q, po, qo) == pytest.approx(kl, rel=1e-12)


# ------------------------------------------------------------------ mask (Eq. dppo_obj)
def test_mask_truth_table(golden_dir):
    delta = 0.1
    val = {"gt": 1, "eq": 0, "lt": -1}
    n = 0
    with open(os.path.join(golden_dir, "mask_truth_table.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            s, rr, dd, m = line.split()
            adv = {"+": 0.7, "0": 0.0, "-": -0.7}[s]
            lmu = -1.25
            lpi = lmu + 0.5 * val[rr]
            D = delta + 0.03 * val[dd]
            assert O.dppo_mask(D, delta, adv, lpi, lmu) == int(m), line
            n += 1
    assert n == 27


def test_mask_with_ratio_distance_recovers_ppo_clip():
    """Replacing D by |r - 1| gives the PPO/GRPO clip mask with a symmetric epsilon (Sec. 4.3);
    the GRPO mask is written out from App. C.1."""
    eps = 0.2
    for _ in range(2000):
        lmu = -RNG.uniform(0.01, 5)
        lpi = lmu + RNG.normal(0, 0.3)
        adv = RNG.choice([-1.0, 0.0, 1.0]) * RNG.uniform(0.1, 2)
        r = math.exp(lpi - lmu)
        grpo = 0 if ((adv > 0 and r > 1 + eps) or (adv < 0 and r < 1 - eps)) else 1
        assert O.dppo_mask(abs(r - 1.0), eps, adv, lpi, lmu) == grpo


# ------------------------------------------------------------------ whole path on generated batches
def _small_batch(variant, K=0, V=257, n_seq=4, seq_len=6, noise=0.3, shift=0.0, seed=7):
    w = W.Workload("t", n_seq, seq_len, V, variant, 0.05, K=K, logit_std=2.0, noise_std=noise,
                   adv="normal", seed=seed)
    b = W.make_batch(w, "cpu", keep_mu_full=True, shift_sampled=shift)
    return W.to_host(b)


def _run(h, **kw):
    args = dict(logits=h["logits"], sampled_ids=h["sampled_ids"], mu_logp=h["mu_logp"],
                advantages=h["advantages"], delta=h["delta"], variant=h["variant"],
                loss_scale=h["loss_scale"], mu_topk_ids=h["mu_topk_ids"], mu_topk_logp=h["mu_topk_logp"])
    args.update(kw)
    return O.dppo_loss(**args)


@pytest.mark.parametrize("variant,K", [(O.BINARY_TV, 0), (O.BINARY_KL, 0), (O.TOPK_TV, 8), (O.TOPK_KL, 8)])
def test_generated_batch_against_brute_force(variant, K):
    h = _small_batch(variant, K, shift=3.0)
    out = _run(h)
    mu_full = np.exp(h["mu_logp_full"].astype(np.float64))
    pi_full = np.exp(np.stack([O.log_softmax(r) for r in h["logits"]]))
    masked = 0
    for t in range(h["T"]):
        exact = O.full_tv(mu_full[t], pi_full[t]) if variant in (O.BINARY_TV, O.TOPK_TV) \
            else O.full_kl(mu_full[t], pi_full[t])
        # mu comes in fp32, so allow its rounding in the bound
        assert -1e-12 <= out["divergence"][t] <= exact + 1e-6
        a = int(h["sampled_ids"][t])
        assert out["ratio"][t] == pytest.approx(pi_full[t, a] / math.exp(h["mu_logp"][t]), rel=1e-9)
        masked += int(out["mask"][t] == 0)
    assert 0 < masked < h["T"]          # the stress recipe exercises both mask values


def test_topk_tv_gap_shrinks_with_k():
    h = _small_batch(O.TOPK_TV, 16, V=300, shift=1.0)
    d_prev = _run(h, variant=O.BINARY_TV)["divergence"]
    for k in (1, 4, 16):
        d = _run(h, mu_topk_ids=h["mu_topk_ids"][:, :k], mu_topk_logp=h["mu_topk_logp"][:, :k])["divergence"]
        assert np.all(d >= d_prev - 1e-12)
        d_prev = d


@pytest.mark.parametrize("variant,K", [(O.BINARY_TV, 0), (O.BINARY_KL, 0), (O.TOPK_TV, 5), (O.TOPK_KL, 5)])
def test_identical_policies_give_zero_divergence_full_mask_closed_form_loss(variant, K):
    h = _small_batch(variant, K, V=129, noise=0.0)
    # with zero rollout noise mu is the fp32 log-softmax of the same logits: pi == mu to ~1e-7
    out = _run(h, delta=1e-5)
    assert np.all(out["divergence"] < 5e-6) and np.all(out["divergence"] >= -1e-14)
    assert np.all(out["mask"] == 1)
    np.testing.assert_allclose(out["ratio"], 1.0, atol=1e-5)
    assert out["loss"] == pytest.approx(-h["loss_scale"] * h["advantages"].astype(np.float64).sum(), rel=1e-5, abs=1e-7)
    # exactly identical: feed float64 log-probs of pi itself
    lp = np.stack([O.log_softmax(r) for r in h["logits"]])
    a = h["sampled_ids"].astype(np.int64)
    lmu = lp[np.arange(h["T"]), a]
    tk = np.take_along_axis(lp, h["mu_topk_ids"].astype(np.int64), 1) if K else None
    out = _run(h, mu_logp=lmu, mu_topk_logp=tk, delta=0.0)
    assert np.all(np.abs(out["divergence"]) <= 1e-14) and np.all(out["mask"] == 1)
    assert out["loss"] == pytest.approx(-h["loss_scale"] * h["advantages"].astype(np.float64).sum(), rel=1e-12)


@pytest.mark.parametrize("variant,K", [(O.BINARY_TV, 0), (O.TOPK_KL, 4)])
def test_gradient_finite_differences_and_structure(variant, K):
    h = _small_batch(variant, K, V=33, n_seq=2, seq_len=3, shift=1.0)
    out = _run(h)
    g = out["grad_logits"]
    z = h["logits"].astype(np.float64)
    eps = 1e-6

    def frozen_loss(zz):
        """Step 5 with the mask of the unperturbed point held constant (Eq. unified_grad treats
        M as a factor, not a function of theta)."""
        tot = 0.0
        for t in range(h["T"]):
            lpi = O.log_softmax(zz[t])[int(h["sampled_ids"][t])]
            tot += -float(out["mask"][t]) * math.exp(lpi - float(h["mu_logp"][t])) * float(h["advantages"][t])
        return h["loss_scale"] * tot

    for t in range(h["T"]):
        for j in list(RNG.choice(33, 6, replace=False)) + [int(h["sampled_ids"][t])]:
            zp, zm = z.copy(), z.copy()
            zp[t, j] += eps
            zm[t, j] -= eps
            fd = (frozen_loss(zp) - frozen_loss(zm)) / (2 * eps)
            assert g[t, j] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    for t in range(h["T"]):
        a, A, M = int(h["sampled_ids"][t]), float(h["advantages"][t]), int(out["mask"][t])
        assert abs(g[t].sum()) < 1e-12                         # softmax-minus-onehot sums to 0
        if M == 0 or A == 0:
            assert np.all(g[t] == 0)
        else:
            assert np.sign(g[t, a]) == -np.sign(A)
            others = np.delete(g[t], a)
            assert np.all(np.sign(others) == np.sign(A))


@pytest.mark.parametrize("variant,K", [(O.BINARY_KL, 0), (O.TOPK_TV, 6)])
def test_gradient_matches_autograd_of_masked_surrogate(variant, K):
    h = _small_batch(variant, K, V=65, shift=1.0)
    out = _run(h)
    z = torch.tensor(h["logits"], dtype=torch.float64, requires_grad=True)
    lp = torch.log_softmax(z, -1).gather(1, torch.tensor(h["sampled_ids"], dtype=torch.int64)[:, None]).squeeze(1)
    r = torch.exp(lp - torch.tensor(h["mu_logp"], dtype=torch.float64))
    M = torch.tensor(out["mask"], dtype=torch.float64)        # constant
    loss = -(M * r * torch.tensor(h["advantages"], dtype=torch.float64)).sum() * h["loss_scale"]
    loss.backward()
    assert out["loss"] == pytest.approx(float(loss.detach()), rel=1e-12)
    np.testing.assert_allclose(out["grad_logits"], z.grad.numpy(), rtol=1e-9, atol=1e-15)


def test_ignored_rows_and_loss_scale():
    h = _small_batch(O.BINARY_TV, 0, V=40)
    ids = h["sampled_ids"].copy()
    ids[::3] = -1
    out = _run(h, sampled_ids=ids)
    for t in range(h["T"]):
        if ids[t] < 0:
            assert out["divergence"][t] == 0 and out["mask"][t] == 0 and out["loss_tok"][t] == 0
            assert np.all(out["grad_logits"][t] == 0)
    ref = _run(h)
    keep = ids >= 0
    np.testing.assert_array_equal(out["divergence"][keep], ref["divergence"][keep])
    assert out["loss"] == pytest.approx(h["loss_scale"] * ref["loss_tok"][keep].sum(), rel=1e-12)
    out2 = _run(h, loss_scale=3.0 * h["loss_scale"])
    assert out2["loss"] == pytest.approx(3.0 * ref["loss"], rel=1e-12)
    np.testing.assert_allclose(out2["grad_logits"], 3.0 * ref["grad_logits"], rtol=1e-12)


# ------------------------------------------------------------------ diagnostics (App. F.1, App. B.1)
def test_diagnostics_entropy_abs_diff_and_covered_mass():
    for V in (2, 9, 300):
        pi = _rand_dist(V, True)
        assert O.entropy(np.log(pi)) == pytest.approx(scipy.stats.entropy(pi), rel=1e-10)
    assert O.entropy(np.log(np.full(8, 1 / 8))) == pytest.approx(math.log(8))
    assert O.entropy(np.array([0.0, -np.inf, -np.inf])) == 0.0                  # 0 ln 0 = 0
    h = _small_batch(O.TOPK_TV, 6, V=200, shift=1.0)
    out = _run(h)
    mu_full = np.exp(h["mu_logp_full"].astype(np.float64))
    for t in range(h["T"]):
        a = int(h["sampled_ids"][t])
        pi = np.exp(O.log_softmax(h["logits"][t]))
        assert out["entropy"][t] == pytest.approx(scipy.stats.entropy(pi), rel=1e-9)
        assert out["abs_diff"][t] == pytest.approx(abs(mu_full[t, a] - pi[a]), abs=1e-7)   # mu arrives in fp32
        ids = sorted(set(h["mu_topk_ids"][t].tolist()) | {a})
        assert out["mass_mu"][t] == pytest.approx(mu_full[t, ids].sum(), abs=1e-6)
        assert out["mass_pi"][t] == pytest.approx(pi[ids].sum(), rel=1e-9)
    hb = dict(h)
    outb = _run(hb, variant=O.BINARY_TV)
    np.testing.assert_allclose(outb["mass_pi"], np.exp(outb["logp"]), rtol=1e-12)
    np.testing.assert_allclose(outb["abs_diff"], outb["divergence"], rtol=1e-12)


# ------------------------------------------------------------------ baselines of App. C.1 / App. E
def test_ratio_clip_mask_truth_table_and_hyperparameters():
    """GRPO-ClipHigher: M = 0 iff (A > 0 and r > 1 + eps_high) or (A < 0 and r < 1 - eps_low)."""
    for eps_low, eps_high in ((0.2, 0.28), (0.2, 0.27), (0.2, 0.2)):
        for adv in (-1.0, 0.0, 1.0):
            for r in (0.5, 1 - eps_low - 1e-9, 1 - eps_low + 1e-9, 1.0, 1 + eps_high - 1e-9, 1 + eps_high + 1e-9, 3.0):
                want = 0 if ((adv > 0 and r > 1 + eps_high) or (adv < 0 and r < 1 - eps_low)) else 1
                lmu = -2.0
                assert O.ratio_clip_mask(adv, lmu + math.log(r), lmu, eps_low, eps_high) == want, (adv, r)
    # the tokens of App. D: "r > 1.28" on positive samples and "r < 0.8" on negative ones are clipped
    assert O.ratio_clip_mask(1.0, math.log(1.29), 0.0, 0.2, 0.28) == 0
    assert O.ratio_clip_mask(-1.0, math.log(0.79), 0.0, 0.2, 0.28) == 0
    assert O.ratio_clip_mask(1.0, math.log(0.5), 0.0, 0.2, 0.28) == 1      # moving back toward r = 1 is never blocked
    assert O.ratio_clip_mask(-1.0, math.log(2.0), 0.0, 0.2, 0.28) == 1


def test_unified_gradient_form_masks_and_cap():
    h = _small_batch(O.BINARY_TV, 0, V=65, shift=3.0, noise=0.5)
    base = _run(h)
    # C = infinity and the divergence mask: nothing changes
    same = _run(h, ratio_cap=float("inf"), mask_rule=O.MASK_DIVERGENCE)
    np.testing.assert_array_equal(same["grad_logits"], base["grad_logits"])
    # PG-IS: M = 1, C = infinity
    pgis = _run(h, mask_rule=O.MASK_NONE)
    assert np.all(pgis["mask"] == 1)
    assert pgis["loss"] == pytest.approx(-h["loss_scale"] * (pgis["ratio"] * h["advantages"]).sum(), rel=1e-12)
    # CISPO / PG-TIS: M = 1, C = 3; GRPO: clip mask, C = infinity; a capped DPPO
    for kw in (dict(mask_rule=O.MASK_NONE, ratio_cap=3.0), dict(mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28),
               dict(mask_rule=O.MASK_DIVERGENCE, ratio_cap=5.0), dict(mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.27, ratio_cap=5.0)):
        out = _run(h, **kw)
        C = kw.get("ratio_cap", float("inf"))
        np.testing.assert_allclose(out["weight"], np.minimum(out["ratio"], C), rtol=1e-12)
        if C < float("inf"):
            assert (out["ratio"] > C).any() and (out["ratio"] < C).any()       # the cap bites on some tokens only
        # Eq. unified_grad: gradient = M * min(r, C) * A * grad log pi(a), weight held constant
        z = torch.tensor(h["logits"], dtype=torch.float64, requires_grad=True)
        lp = torch.log_softmax(z, -1).gather(1, torch.tensor(h["sampled_ids"], dtype=torch.int64)[:, None]).squeeze(1)
        coef = torch.tensor(out["mask"] * out["weight"] * h["advantages"], dtype=torch.float64)
        (-(coef * lp).sum() * h["loss_scale"]).backward()
        np.testing.assert_allclose(out["grad_logits"], z.grad.numpy(), rtol=1e-9, atol=1e-15)
        if kw["mask_rule"] == O.MASK_RATIO_CLIP:
            want = [O.ratio_clip_mask(float(a), float(lp_), float(lm), kw["eps_low"], kw["eps_high"])
                    for a, lp_, lm in zip(h["advantages"], out["logp"], h["mu_logp"])]
            np.testing.assert_array_equal(out["mask"], want)
            assert 0 < int((out["mask"] == 0).sum()) < h["T"]


def test_mask_anchored_to_a_recomputed_policy_minirl_and_decoupled_dppo():
    """App. C.1: MiniRL's clip mask is GRPO's with r' = pi / pi_theta' (the trainer's recomputed
    policy) in place of r = pi / mu, while the weight min(r, C) keeps the rollout ratio; Sec. 5.2:
    the decoupled DPPO takes divergence and direction test against pi_theta' too.  The anchor's
    log-prob comes in as one more per-token input."""
    h = _small_batch(O.BINARY_TV, 0, V=65, shift=3.0, noise=0.5)
    rng = np.random.default_rng(5)
    anchor = (h["mu_logp"].astype(np.float64) + rng.normal(0.0, 0.6, h["T"])).astype(np.float32)
    anchor = np.minimum(anchor, 0.0)
    base = _run(h)
    # an anchor equal to the rollout policy changes nothing, under every rule
    for kw in (dict(), dict(mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28), dict(mask_rule=O.MASK_NONE, ratio_cap=3.0)):
        a, b = _run(h, **kw), _run(h, anchor_logp=h["mu_logp"], **kw)
        for k in ("loss_tok", "divergence", "mask", "grad_logits", "ratio", "weight"):
            np.testing.assert_array_equal(a[k], b[k])
    # MiniRL / MiniRL-TIS: the GRPO mask evaluated on r', weight and loss on r
    for C in (None, 3.0):
        out = _run(h, anchor_logp=anchor, mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28, ratio_cap=C)
        want = [O.ratio_clip_mask(float(a), float(lp), float(la), 0.2, 0.28) for a, lp, la in zip(h["advantages"], out["logp"], anchor)]
        np.testing.assert_array_equal(out["mask"], want)
        grpo = _run(h, mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28, ratio_cap=C)
        assert (out["mask"] != grpo["mask"]).any()                           # the anchor matters on this batch
        np.testing.assert_array_equal(out["ratio"], base["ratio"])           # r stays pi / mu
        w = out["ratio"] if C is None else np.minimum(out["ratio"], C)
        np.testing.assert_allclose(out["loss_tok"], -out["mask"].astype(np.float64) * w * h["advantages"], rtol=1e-12)
        z = torch.tensor(h["logits"], dtype=torch.float64, requires_grad=True)
        lp = torch.log_softmax(z, -1).gather(1, torch.tensor(h["sampled_ids"], dtype=torch.int64)[:, None]).squeeze(1)
        coef = torch.tensor(out["mask"] * w * h["advantages"], dtype=torch.float64)
        (-(coef * lp).sum() * h["loss_scale"]).backward()
        np.testing.assert_allclose(out["grad_logits"], z.grad.numpy(), rtol=1e-9, atol=1e-15)
    # r' on either side of the clip range while r sits inside it, and the other way round
    one = dict(logits=np.log(np.array([[0.5, 0.3, 0.2]])), sampled_ids=np.array([0]), advantages=np.array([1.0]),
               delta=0.1, variant=O.BINARY_TV, mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28)
    assert O.dppo_loss(mu_logp=np.log([0.45]), anchor_logp=np.log([0.30]), **one)["mask"][0] == 0    # r = 1.11, r' = 1.67
    assert O.dppo_loss(mu_logp=np.log([0.30]), anchor_logp=np.log([0.45]), **one)["mask"][0] == 1    # r = 1.67, r' = 1.11
    assert O.dppo_loss(mu_logp=np.log([0.30]), **one)["mask"][0] == 0                                # GRPO on r
    # decoupled DPPO: divergence and direction test against the anchor, in closed form (Eq. binary_tv)
    dec = _run(h, anchor_logp=anchor)
    lpi = dec["logp"]
    np.testing.assert_allclose(dec["divergence"], np.abs(np.exp(anchor.astype(np.float64)) - np.exp(lpi)), rtol=1e-12, atol=1e-15)
    A = h["advantages"].astype(np.float64)
    blocked = (dec["divergence"] > h["delta"]) & (((A > 0) & (lpi > anchor)) | ((A < 0) & (lpi < anchor)))
    np.testing.assert_array_equal(dec["mask"], 1 - blocked.astype(np.uint8))
    np.testing.assert_array_equal(dec["ratio"], base["ratio"])
    assert (dec["divergence"] != base["divergence"]).any()
    one_d = dict(one, mask_rule=O.MASK_DIVERGENCE)
    # pi(a) = 0.5, mu(a) = 0.45: D = 0.05 < delta = 0.1 keeps the token; against pi_theta'(a) = 0.30, D = 0.20 blocks it
    assert O.dppo_loss(mu_logp=np.log([0.45]), **one_d)["mask"][0] == 1
    blocked_row = O.dppo_loss(mu_logp=np.log([0.45]), anchor_logp=np.log([0.30]), **one_d)
    assert blocked_row["mask"][0] == 0 and blocked_row["divergence"][0] == pytest.approx(0.2, rel=1e-12)
    # the direction test looks at the anchor too: pi(a) = 0.5 is below mu(a) = 0.6 but above pi_theta'(a) = 0.3
    assert O.dppo_loss(mu_logp=np.log([0.6]), anchor_logp=np.log([0.30]), **one_d)["mask"][0] == 0
    assert O.dppo_loss(mu_logp=np.log([0.3]), anchor_logp=np.log([0.60]), **one_d)["mask"][0] == 1
    # Top-K: the anchor takes the sampled token's place in the reduced distributions
    hk = _small_batch(O.TOPK_KL, 8, V=65, shift=3.0, noise=0.5)
    anchor_k = np.minimum(hk["mu_logp"] - 0.3, 0.0).astype(np.float32)
    outk = _run(hk, anchor_logp=anchor_k)
    for t in range(hk["T"]):
        p, q, po, qo = O.reduced_distributions(O.log_softmax(hk["logits"][t].astype(np.float64)), int(hk["sampled_ids"][t]),
                                               float(anchor_k[t]), hk["mu_topk_ids"][t], hk["mu_topk_logp"][t])
        assert outk["divergence"][t] == pytest.approx(O.topk_kl(p, q, po, qo), rel=1e-12, abs=1e-15)


def test_clip_relaxed_for_low_probability_tokens():
    """Sec. 6: the clip threshold goes to infinity, on the upper side (Relax-high), the lower side
    (Relax-low) or both, for tokens whose ROLLOUT probability is below alpha; all others keep
    GRPO's range.  Truth table over sign(A) x r outside / inside the range x mu(a) below / above alpha."""
    eps_low, eps_high, alpha = 0.2, 0.28, 0.1
    for sides in (0, O.RELAX_HIGH, O.RELAX_LOW, O.RELAX_HIGH | O.RELAX_LOW):
        for mu_a in (0.02, 0.0999, 0.1001, 0.5):
            for r in (0.5, 0.79, 1.0, 1.29, 4.0):
                pi_a = mu_a * r
                if pi_a >= 1.0:
                    continue
                for adv in (-1.0, 0.0, 1.0):
                    z = np.log(np.array([[pi_a, (1 - pi_a) * 0.6, (1 - pi_a) * 0.4]]))
                    out = O.dppo_loss(z, np.array([0]), np.log([mu_a]), np.array([adv]), 0.1, O.BINARY_TV, mask_rule=O.MASK_RATIO_CLIP,
                                      eps_low=eps_low, eps_high=eps_high, relax_alpha=alpha, relax_sides=sides)
                    low = mu_a < alpha
                    hi_blocks = adv > 0 and r > 1 + eps_high and not (low and sides & O.RELAX_HIGH)
                    lo_blocks = adv < 0 and r < 1 - eps_low and not (low and sides & O.RELAX_LOW)
                    assert out["mask"][0] == (0 if (hi_blocks or lo_blocks) else 1), (sides, mu_a, r, adv)
                    assert out["ratio"][0] == pytest.approx(r, rel=1e-12)
    # alpha = 0 (GRPO) and "no side" are the plain clip mask; both sides with alpha = 1 is no mask at all
    h = _small_batch(O.BINARY_TV, 0, V=65, shift=3.0, noise=0.5)
    clip = dict(mask_rule=O.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28)
    grpo = _run(h, **clip)
    np.testing.assert_array_equal(_run(h, relax_alpha=0.0, relax_sides=3, **clip)["mask"], grpo["mask"])
    np.testing.assert_array_equal(_run(h, relax_alpha=0.5, relax_sides=0, **clip)["mask"], grpo["mask"])
    assert np.all(_run(h, relax_alpha=1.0, relax_sides=3, **clip)["mask"][np.exp(h["mu_logp"]) < 1.0] == 1)
    both = _run(h, relax_alpha=0.3, relax_sides=3, **clip)
    assert (both["mask"] != grpo["mask"]).any() and np.all(both["mask"] >= grpo["mask"])      # relaxing only ever unmasks
    # the DPPO mask ignores the relaxation
    np.testing.assert_array_equal(_run(h, relax_alpha=0.5, relax_sides=3)["mask"], _run(h)["mask"])


# ------------------------------------------------------------------ exact divergence as the trust region (App. B)
def test_full_kl_from_logs_is_the_library_relative_entropy():
    for V in (2, 9, 300):
        mu, pi = _rand_dist(V, True), _rand_dist(V, True)
        d = O.full_kl_from_logs(np.log(mu), np.log(pi))
        assert d == pytest.approx(float(scipy.special.rel_entr(mu, pi).sum()), rel=1e-10)
        assert d == pytest.approx(O.full_kl(mu, pi), rel=1e-10)
        assert d != pytest.approx(float(scipy.special.rel_entr(pi, mu).sum()), rel=1e-3)     # the direction is mu || pi
    # 0 ln 0 = 0: a token mu never samples adds nothing, whatever pi gives it
    assert O.full_kl_from_logs([math.log(0.5), math.log(0.5), -np.inf], np.log([0.25, 0.25, 0.5])) == pytest.approx(math.log(2))
    # pi excludes a token mu can sample: infinite, as the definition is
    assert O.full_kl_from_logs(np.log([0.5, 0.5]), [0.0, -np.inf]) == np.inf


@pytest.mark.parametrize("variant", [O.FULL_TV, O.FULL_KL])
def test_full_variants_use_the_exact_divergence_of_the_two_rows(variant):
    V, T = 50, 40
    rng = np.random.default_rng(77)
    z = rng.normal(0, 2.0, size=(T, V))
    y = z + rng.normal(0, 0.7, size=(T, V)) + rng.normal(0, 5.0, size=(T, 1))     # a row shift of the logits is immaterial
    mu = scipy.special.softmax(y, axis=1)
    pi = scipy.special.softmax(z, axis=1)
    a = np.array([rng.choice(V, p=mu[t]) for t in range(T)])
    lmu_a = np.log(mu[np.arange(T), a])
    adv = rng.choice([-1.0, 1.0], size=T)
    delta = 0.25 if variant == O.FULL_TV else 0.2
    out = O.dppo_loss(z, a, lmu_a, adv, delta, variant, mu_logits=y)
    want = 0.5 * np.abs(mu - pi).sum(1) if variant == O.FULL_TV else scipy.special.rel_entr(mu, pi).sum(1)
    np.testing.assert_allclose(out["divergence"], want, rtol=1e-10)
    # the mask is Eq. dppo_obj on that divergence
    r = pi[np.arange(T), a] / mu[np.arange(T), a]
    blocked = (want > delta) & (((adv > 0) & (r > 1)) | ((adv < 0) & (r < 1)))
    np.testing.assert_array_equal(out["mask"], 1 - blocked.astype(np.uint8))
    assert 0 < blocked.sum() < T
    np.testing.assert_array_equal(out["mass_mu"], 1.0)
    np.testing.assert_array_equal(out["mass_pi"], 1.0)
    # every approximation of Sec. 4.4 lower-bounds it (App. B), token by token
    ids = np.argsort(-mu, axis=1, kind="stable")[:, :6]
    lps = np.log(np.take_along_axis(mu, ids, 1))
    vb, vk = (O.BINARY_TV, O.TOPK_TV) if variant == O.FULL_TV else (O.BINARY_KL, O.TOPK_KL)
    Db = O.dppo_loss(z, a, lmu_a, adv, delta, vb)["divergence"]
    Dk = O.dppo_loss(z, a, lmu_a, adv, delta, vk, mu_topk_ids=ids, mu_topk_logp=lps)["divergence"]
    assert np.all(Db <= Dk + 1e-13) and np.all(Dk <= out["divergence"] + 1e-13)
    # identical policies: zero divergence, nothing masked
    same = O.dppo_loss(z, a, np.log(pi[np.arange(T), a]), adv, delta, variant, mu_logits=z + 3.0)
    np.testing.assert_allclose(same["divergence"], 0.0, atol=1e-14)
    assert np.all(same["mask"] == 1)
    with pytest.raises(ValueError):
        O.dppo_loss(z, a, lmu_a, adv, delta, variant)


# ------------------------------------------------------------------ from the hidden states
def test_bf16_round_matches_the_library_cast_and_ties_go_to_even():
    x = np.concatenate([RNG.normal(0, 30.0, 5000), RNG.normal(0, 1e-3, 1000), [0.0, 1.0, -1.0, 255.0, 256.0, 3.0e4]]).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).double().numpy()          # float32 -> bf16, nearest even
    np.testing.assert_array_equal(O.bf16_round(x.astype(np.float64)), want)
    assert O.bf16_round(1.0 + 2.0 ** -8) == 1.0                          # halfway: to the even neighbour
    assert O.bf16_round(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert O.bf16_round(-(1.0 + 2.0 ** -8 + 2.0 ** -30)) == -(1.0 + 2.0 ** -7)
    assert O.bf16_round(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7  # no double rounding through float32


def test_lmhead_path_is_the_chain_rule_through_the_logits():
    rng = np.random.default_rng(9)
    T, d, V = 40, 16, 40
    # small integers: every logit is an integer below 256, so the bf16 rounding is the identity and
    # the whole path must equal float64 autograd of the masked surrogate through h W^T
    h = rng.integers(-2, 3, size=(T, d)).astype(np.float64)
    W = rng.integers(-2, 3, size=(V, d)).astype(np.float64)
    z = h @ W.T
    assert np.abs(z).max() < 256
    np.testing.assert_array_equal(O.lmhead_logits(h, W), z)
    y = z / 8 + rng.normal(0, 1.5, size=z.shape)
    mu = scipy.special.softmax(y, axis=1)
    a = np.array([rng.choice(V, p=mu[t]) for t in range(T)])
    lmu = np.log(mu[np.arange(T), a])
    adv = rng.normal(size=T)
    ids = np.argsort(-mu, axis=1, kind="stable")[:, :5]
    lps = np.log(np.take_along_axis(mu, ids, 1))
    hs, Ws = h / 8, W                    # logits z / 8: exact in bf16 as well
    for variant, kw in ((O.BINARY_TV, {}), (O.TOPK_KL, dict(mu_topk_ids=ids, mu_topk_logp=lps))):
        out = O.lmhead_dppo_loss(hs, Ws, a, lmu, adv, 0.05, variant, loss_scale=0.25, **kw)
        ref = O.dppo_loss(z / 8, a, lmu, adv, 0.05, variant, loss_scale=0.25, **kw)
        for k in ("loss_tok", "divergence", "mask", "grad_logits"):
            np.testing.assert_array_equal(out[k], ref[k])
        assert 0 < (out["mask"] == 0).sum() < T
        ht = torch.tensor(hs, dtype=torch.float64, requires_grad=True)
        wt = torch.tensor(Ws, dtype=torch.float64, requires_grad=True)
        lp = torch.log_softmax(ht @ wt.T, -1).gather(1, torch.tensor(a)[:, None]).squeeze(1)
        coef = torch.tensor(out["mask"] * out["ratio"] * adv, dtype=torch.float64)
        (-(coef * lp).sum() * 0.25).backward()
        np.testing.assert_allclose(out["grad_hidden"], ht.grad.numpy(), rtol=1e-9, atol=1e-14)
        np.testing.assert_allclose(out["grad_weight"], wt.grad.numpy(), rtol=1e-9, atol=1e-14)
        assert out["grad_weight"].shape == (V, d) and np.abs(out["grad_weight"].sum(0)).max() < 1e-12    # rows of g sum to 0
    # logits that do need rounding: rounded once, to 8 significant bits
    h2, W2 = rng.normal(size=(3, 8)), rng.normal(size=(5, 8))
    z2 = O.lmhead_logits(h2, W2)
    exact = h2 @ W2.T
    assert np.all(np.abs(z2 - exact) <= np.abs(exact) * 2.0 ** -8) and np.any(z2 != exact)
    np.testing.assert_array_equal(z2, torch.tensor(z2).to(torch.bfloat16).double().numpy())
