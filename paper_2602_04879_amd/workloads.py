"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and calls torch library routines to stand in for the
two engines that surround the loss in RL fine-tuning of an LLM: the trainer's forward pass
(which hands over bf16 logits) and the rollout engine (which hands over the sampled token,
its log-prob under mu, and mu's top-K log-probs -- Sec. 1 and Sec. 4.4 of the paper, K=20
in its experiments, App. F).  None of the DPPO arithmetic lives here; the GPU library and
the CPU oracle are both fed from it and neither imports the other.

No model, dataset or benchmark item is involved: every value is drawn from the seeded
distributions written out below, which stand in for a Qwen3-vocabulary (V = 151936) policy
under train/inference mismatch.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch

BINARY_TV, BINARY_KL, TOPK_TV, TOPK_KL, FULL_TV, FULL_KL = 0, 1, 2, 3, 4, 5


@dataclass
class Workload:
    name: str
    n_seq: int
    seq_len: int
    V: int
    variant: int
    delta: float
    K: int = 0
    logit_std: float = 3.0
    noise_std: float = 0.05
    zipf_s: float = 0.0           # log-prior -s*ln(id+1) added to the logits
    boost_frac: float = 0.0       # fraction of vocabulary ids whose logit gets +boost
    boost: float = 0.0
    temperature: tuple | None = None   # per-token temperature ~ U(lo, hi) applied before the bf16 cast
    drift_frac: float = 0.0       # fraction of tokens whose sampled-token logit has moved since the
    drift_std: float = 0.0        # rollout (policy updates in between), by N(0, drift_std)
    mu_full: bool = False         # also hand over the rollout policy's full logits, rounded to bf16
    d_model: int = 0              # > 0: the batch starts from hidden states [T, d_model] and an lm_head weight
    adv: str = "pm1"              # "pm1" | "normal" | "group_norm"
    group: int = 8
    chunk_rows: int = 0           # caller-side T-chunking (0 = one call)
    seed: int = 1000
    extra: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return self.n_seq * self.seq_len


# The configurations this repository is measured and tested on.
WORKLOADS = {
    "c1_tiny_binary_tv": Workload("c1_tiny_binary_tv", 4, 64, 4096, BINARY_TV, 0.2,
                                  logit_std=2.0, noise_std=0.05, adv="pm1", seed=1000),
    "c2_binary_tv": Workload("c2_binary_tv", 16, 512, 32768, BINARY_TV, 0.1, logit_std=3.0,
                             noise_std=0.1, boost_frac=0.01, boost=8.0, adv="normal", seed=1001),
    "c2_binary_kl": Workload("c2_binary_kl", 16, 512, 32768, BINARY_KL, 0.1, logit_std=3.0,
                             noise_std=0.1, boost_frac=0.01, boost=8.0, adv="normal", seed=1001),
    "c3_qwen3_binary_tv": Workload("c3_qwen3_binary_tv", 16, 2048, 151936, BINARY_TV, 0.2,
                                   logit_std=3.0, noise_std=0.05, zipf_s=1.1, drift_frac=0.05, drift_std=1.5,
                                   adv="group_norm", group=8, seed=1002),
    "c4_qwen3_topk_tv": Workload("c4_qwen3_topk_tv", 16, 2048, 151936, TOPK_TV, 0.2, K=20,
                                 logit_std=3.0, noise_std=0.05, zipf_s=1.1, drift_frac=0.05, drift_std=1.5,
                                 adv="group_norm", group=8, seed=1002),
    "c5_long_topk_kl": Workload("c5_long_topk_kl", 32, 4096, 151936, TOPK_KL, 0.05, K=64,
                                logit_std=3.0, noise_std=0.1, zipf_s=1.1, temperature=(0.6, 1.2),
                                drift_frac=0.05, drift_std=1.5, adv="pm1", chunk_rows=16384, seed=1004),
    # The headline shape with the trust region on the exact divergence between the two rows
    # (the rollout policy's full logits are given as a second bf16 matrix).
    "c6_qwen3_full_tv": Workload("c6_qwen3_full_tv", 16, 2048, 151936, FULL_TV, 0.2, mu_full=True,
                                 logit_std=3.0, noise_std=0.05, zipf_s=1.1, drift_frac=0.05, drift_std=1.5,
                                 adv="group_norm", group=8, seed=1002),
    "c6_qwen3_full_kl": Workload("c6_qwen3_full_kl", 16, 2048, 151936, FULL_KL, 0.05, mu_full=True,
                                 logit_std=3.0, noise_std=0.05, zipf_s=1.1, drift_frac=0.05, drift_std=1.5,
                                 adv="group_norm", group=8, seed=1002),
    # The headline recipe at the vocabulary of the paper's other model family (Sec. 7, alignment
    # runs on Gemma-2: 256000 entries, rows of 500 KiB), half the rows: the long-row kernel.
    "c8_vocab256k_binary_tv": Workload("c8_vocab256k_binary_tv", 16, 1024, 256000, BINARY_TV, 0.2,
                                       logit_std=3.0, noise_std=0.05, zipf_s=1.1, drift_frac=0.05, drift_std=1.5,
                                       adv="group_norm", group=8, seed=1008),
    # Rows of middle length, many of them: C2's vocabulary and recipe at eight times its token
    # count (the headline's, twice over): the kernel that takes several rows per workgroup.
    "c9_vocab32k_binary_tv": Workload("c9_vocab32k_binary_tv", 64, 1024, 32768, BINARY_TV, 0.1, logit_std=3.0,
                                      noise_std=0.1, boost_frac=0.01, boost=8.0, adv="normal", seed=1009),
    # The headline recipe with the vocabulary cut to an odd length (a trainer that slices the padding
    # of the embedding matrix off the logits), half the rows: no row starts on a 16-byte boundary but
    # every eighth: the ragged form of the register-resident kernel.
    "c10_vocab151643_binary_tv": Workload("c10_vocab151643_binary_tv", 16, 1024, 151643, BINARY_TV, 0.2,
                                          logit_std=3.0, noise_std=0.05, zipf_s=1.1, drift_frac=0.05, drift_std=1.5,
                                          adv="group_norm", group=8, seed=1010),
    # The headline shape entered one step earlier: final hidden states of a d = 4096 model (the
    # Qwen3-8B size) and its lm_head weight; the logits exist one chunk of tokens at a time.
    "c7_qwen3_lmhead_binary_tv": Workload("c7_qwen3_lmhead_binary_tv", 16, 2048, 151936, BINARY_TV, 0.2, d_model=4096,
                                          logit_std=3.0, noise_std=0.05, drift_frac=0.05, drift_std=1.5,
                                          adv="group_norm", group=8, seed=1007),
}


def scaled(w: Workload, n_seq: int | None = None, seq_len: int | None = None, V: int | None = None,
           **kw) -> Workload:
    """A copy of a workload at another size (same distributions, same seed)."""
    d = dict(w.__dict__)
    if n_seq is not None:
        d["n_seq"] = n_seq
    if seq_len is not None:
        d["seq_len"] = seq_len
    if V is not None:
        d["V"] = V
    d.update(kw)
    d["extra"] = dict(w.extra)
    return Workload(**d)


def _advantages(w: Workload, g: torch.Generator, device) -> torch.Tensor:
    """One value per sequence, broadcast to its tokens (sequence-level advantage, Sec. 3)."""
    n = w.n_seq
    if w.adv == "pm1":
        a = torch.ones(n, device=device)
        a[torch.randperm(n, generator=g, device=device)[: n // 2]] = -1.0   # both signs present
    elif w.adv == "normal":
        a = torch.randn(n, generator=g, device=device)
    elif w.adv == "group_norm":
        # rewards in {0,1}; A = (R - mean_G) / (std_G + 1e-6) inside groups of w.group rollouts
        r = (torch.rand(n, generator=g, device=device) < 0.5).float()
        grp = r.view(-1, min(w.group, n))
        a = ((grp - grp.mean(1, keepdim=True)) / (grp.std(1, unbiased=False, keepdim=True) + 1e-6)).reshape(n)
    else:
        raise ValueError(w.adv)
    return a.repeat_interleave(w.seq_len).contiguous()


@torch.no_grad()
def make_batch(w: Workload, device="cpu", ld: int | None = None, keep_mu_full: bool = False,
               rows_per_step: int = 1024, shift_sampled: float = 0.0) -> dict:
    """Draw one batch.

    Returns a dict of tensors on `device`:
      logits [T, ld] bf16 (columns V..ld-1, if any, hold a poison value the path must ignore),
      sampled_ids [T] int32, mu_logp [T] f32, mu_topk_ids / mu_topk_logp [T, K] (or None),
      advantages [T] f32, mu_logits [T, ld] bf16 (workloads with mu_full, else None), plus python scalars delta, variant, K, loss_scale, T, V, ld.
    With keep_mu_full the rollout policy's full log-probs [T, V] (f32) are kept as
    "mu_logp_full" so exact divergences can be brute-forced on small V.
    shift_sampled != 0 adds +/-shift to the trainer's logit of the sampled token on
    alternating rows AFTER the rollout was drawn: a stress recipe that pushes tokens across
    the trust-region boundary (parity tests only).
    """
    dev = torch.device(device)
    T, V, K = w.T, w.V, w.K
    ld = V if ld is None else ld
    assert ld >= V
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)

    logits = torch.empty((T, ld), dtype=torch.bfloat16, device=dev)
    if ld > V:
        logits[:, V:] = 1.0e4   # poison: must never be read as vocabulary
    sampled = torch.empty(T, dtype=torch.int32, device=dev)
    mu_logp = torch.empty(T, dtype=torch.float32, device=dev)
    tk_ids = torch.empty((T, K), dtype=torch.int32, device=dev) if K > 0 else None
    tk_lp = torch.empty((T, K), dtype=torch.float32, device=dev) if K > 0 else None
    mu_full = torch.empty((T, V), dtype=torch.float32, device=dev) if keep_mu_full else None
    mu_logits = None
    if w.mu_full:
        mu_logits = torch.empty((T, ld), dtype=torch.bfloat16, device=dev)
        if ld > V:
            mu_logits[:, V:] = 1.0e4

    prior = None
    if w.zipf_s > 0:
        prior = -w.zipf_s * torch.log(torch.arange(1, V + 1, device=dev, dtype=torch.float32))
    boost = None
    if w.boost_frac > 0:
        nb = int(round(w.boost_frac * V))
        boost = torch.zeros(V, device=dev)
        boost[torch.randperm(V, generator=g, device=dev)[:nb]] = w.boost

    for r0 in range(0, T, rows_per_step):
        r1 = min(T, r0 + rows_per_step)
        n = r1 - r0
        x = torch.randn((n, V), generator=g, device=dev) * w.logit_std
        if prior is not None:
            x += prior
        if boost is not None:
            x += boost
        if w.temperature is not None:
            lo, hi = w.temperature
            tau = lo + (hi - lo) * torch.rand((n, 1), generator=g, device=dev)
            x /= tau
        zb = x.to(torch.bfloat16)                      # what the trainer hands over
        # rollout engine: same logits seen through inference-side numerical mismatch
        y = zb.float() + w.noise_std * torch.randn((n, V), generator=g, device=dev)
        if w.mu_full:                                  # the rollout logits as handed over: bf16
            mu_logits[r0:r1, :V] = y.to(torch.bfloat16)
            y = mu_logits[r0:r1, :V].float()
        lmu = torch.log_softmax(y, dim=-1)
        a = torch.multinomial(lmu.exp(), 1, generator=g).squeeze(1)
        sampled[r0:r1] = a.to(torch.int32)
        mu_logp[r0:r1] = lmu.gather(1, a[:, None]).squeeze(1)
        if K > 0:
            v, i = torch.topk(lmu, K, dim=-1)
            tk_ids[r0:r1] = i.to(torch.int32)
            tk_lp[r0:r1] = v
        if keep_mu_full:
            mu_full[r0:r1] = lmu
        if shift_sampled != 0.0:
            rows = torch.arange(n, device=dev)
            sgn = torch.where((rows + r0) % 2 == 0, 1.0, -1.0)
            zf = zb.float()
            zf[rows, a] += sgn * shift_sampled
            zb = zf.to(torch.bfloat16)
        if w.drift_frac > 0:
            moved = torch.rand(n, generator=g, device=dev) < w.drift_frac
            step = w.drift_std * torch.randn(n, generator=g, device=dev)
            zf = zb.float()
            rows = torch.arange(n, device=dev)
            zf[rows, a] += torch.where(moved, step, torch.zeros_like(step))
            zb = zf.to(torch.bfloat16)
        logits[r0:r1, :V] = zb

    return {
        "logits": logits, "sampled_ids": sampled, "mu_logp": mu_logp,
        "mu_topk_ids": tk_ids, "mu_topk_logp": tk_lp, "advantages": _advantages(w, g, dev),
        "mu_logp_full": mu_full, "mu_logits": mu_logits, "delta": float(w.delta), "variant": int(w.variant), "K": int(K),
        "loss_scale": 1.0 / float(T), "T": T, "V": V, "ld": ld, "name": w.name,
    }


@torch.no_grad()
def make_lmhead_batch(w: Workload, d: int, device="cpu", exact: bool = False, rows_per_step: int = 1024,
                      shift_sampled: float = 0.0) -> dict:
    """One batch for the path that starts from the final hidden states: hidden [T, d] and lm_head
    weight [V, d] in bf16 whose product has logits of standard deviation about w.logit_std, and a
    rollout drawn from those logits (rounded to bf16, plus the mismatch noise) as in make_batch.

    exact=True draws both matrices from small integers over a power of two, so that every product
    and every partial sum of a logit is exact in fp32: the bf16 logits are then the same
    whatever the order of accumulation.  shift_sampled moves the ROLLOUT's logit of the sampled
    token on alternating rows after sampling (so mu_logp changes, not the hidden states)."""
    dev = torch.device(device)
    T, V, K = w.T, w.V, w.K
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    if exact:
        # integers -8..8 have variance 24: a logit is a sum of d products of variance (24/64 / s)^2
        s = 2.0 ** round(0.5 * torch.log2(torch.tensor(d / 64.0)).item() + torch.log2(torch.tensor(3.0 / w.logit_std)).item())
        hidden = (torch.randint(-8, 9, (T, d), generator=g, device=dev).float() / (8.0 * s)).to(torch.bfloat16)
        weight = (torch.randint(-8, 9, (V, d), generator=g, device=dev).float() / 8.0).to(torch.bfloat16)
    else:
        hidden = torch.randn((T, d), generator=g, device=dev).to(torch.bfloat16)
        weight = (torch.randn((V, d), generator=g, device=dev) * (w.logit_std / d ** 0.5)).to(torch.bfloat16)
    sampled = torch.empty(T, dtype=torch.int32, device=dev)
    mu_logp = torch.empty(T, dtype=torch.float32, device=dev)
    tk_ids = torch.empty((T, K), dtype=torch.int32, device=dev) if K > 0 else None
    tk_lp = torch.empty((T, K), dtype=torch.float32, device=dev) if K > 0 else None
    wf = weight.float()
    for r0 in range(0, T, rows_per_step):
        r1 = min(T, r0 + rows_per_step)
        n = r1 - r0
        zb = (hidden[r0:r1].float() @ wf.T).to(torch.bfloat16)      # the rollout engine's own forward
        y = zb.float() + w.noise_std * torch.randn((n, V), generator=g, device=dev)
        a = torch.multinomial(torch.softmax(y, -1), 1, generator=g).squeeze(1)
        if shift_sampled != 0.0:
            rows = torch.arange(n, device=dev)
            y[rows, a] += torch.where((rows + r0) % 2 == 0, 1.0, -1.0) * shift_sampled
        if w.drift_frac > 0:     # the trainer has moved since the rollout: seen from the trainer, mu is what is off
            moved = torch.rand(n, generator=g, device=dev) < w.drift_frac
            stepv = w.drift_std * torch.randn(n, generator=g, device=dev)
            y[torch.arange(n, device=dev), a] -= torch.where(moved, stepv, torch.zeros_like(stepv))
        lmu = torch.log_softmax(y, dim=-1)
        sampled[r0:r1] = a.to(torch.int32)
        mu_logp[r0:r1] = lmu.gather(1, a[:, None]).squeeze(1)
        if K > 0:
            v, i = torch.topk(lmu, K, dim=-1)
            tk_ids[r0:r1] = i.to(torch.int32)
            tk_lp[r0:r1] = v
    return {
        "hidden": hidden, "weight": weight, "d": int(d), "sampled_ids": sampled, "mu_logp": mu_logp,
        "mu_topk_ids": tk_ids, "mu_topk_logp": tk_lp, "advantages": _advantages(w, g, dev),
        "delta": float(w.delta), "variant": int(w.variant), "K": int(K), "loss_scale": 1.0 / float(T),
        "T": T, "V": V, "name": w.name,
    }


def to_host(batch: dict) -> dict:
    """Host copies for the oracle: bf16 logits widened exactly to float32 numpy, rest as numpy."""
    out = {}
    for k, v in batch.items():
        if isinstance(v, torch.Tensor):
            v = v.detach().cpu()
            out[k] = (v.float() if v.dtype == torch.bfloat16 else v).numpy()
        else:
            out[k] = v
    if out.get("logits") is not None:
        out["logits"] = out["logits"][:, : batch["V"]]
    return out
