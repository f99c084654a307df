"""The pins must notice a plausible mistake anywhere in the oracle.  Each case plants ONE mistake
in a copy of oracle/dppo_oracle.py (on the CPU; the GPU path is not involved) and checks that
at least one pin of tests/test_oracle_pins.py then fails."""
import importlib.util
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "dppo_oracle.py")).read()

MUTATIONS = [
    ("softmax: max not subtracted inside exp", "S = np.exp(z - m).sum()", "S = np.exp(z).sum()"),
    ("ratio inverted", "r = np.exp(lpi - lmu)", "r = np.exp(lmu - lpi)"),
    ("binary TV signed", "return abs(p - q)", "return p - q"),
    ("binary KL: second term dropped", "return _xlogx_over_y(p, q) + _xlogx_over_y(one_minus_p, one_minus_q)",
     "return _xlogx_over_y(p, q)"),
    ("binary KL: direction swapped", "return _xlogx_over_y(p, q) + _xlogx_over_y(one_minus_p, one_minus_q)",
     "return _xlogx_over_y(q, p) + _xlogx_over_y(one_minus_q, one_minus_p)"),
    ("top-K TV: half missing", "return 0.5 * (np.abs(p - q).sum() + abs(p_other - q_other))",
     "return np.abs(p - q).sum() + abs(p_other - q_other)"),
    ("top-K TV: other bucket dropped", "return 0.5 * (np.abs(p - q).sum() + abs(p_other - q_other))",
     "return 0.5 * np.abs(p - q).sum()"),
    ("top-K KL: other bucket dropped", "return d + _xlogx_over_y(p_other, q_other)", "return d"),
    ("top-K: sampled token not de-duplicated", "if i < 0 or i >= len(logpi) or i == int(a):", "if i < 0 or i >= len(logpi):"),
    ("top-K: pi gathered at wrong ids", "q = np.exp(logpi[np.asarray(ids, dtype=np.int64)])",
     "q = np.exp(logpi[np.asarray(ids, dtype=np.int64)[::-1]])"),
    ("mask: non-strict threshold", "if D > delta and", "if D >= delta and"),
    ("mask: wrong side for negative advantage", "(adv < 0.0 and lpi_a < lmu_a)", "(adv < 0.0 and lpi_a > lmu_a)"),
    ("mask: symmetric (blocks moves toward r = 1 too)", "if D > delta and ((adv > 0.0 and lpi_a > lmu_a) or (adv < 0.0 and lpi_a < lmu_a)):",
     "if D > delta and adv != 0.0:"),
    ("loss sign", 'out["loss_tok"][t] = -M * w * A', 'out["loss_tok"][t] = M * w * A'),
    ("loss ignores mask", 'out["loss_tok"][t] = -M * w * A', 'out["loss_tok"][t] = -w * A'),
    ("grad: one-hot not subtracted", "g[a] -= 1.0", "g[a] -= 0.0"),
    ("grad: ratio missing", "(loss_scale * M * A * w) * g", "(loss_scale * M * A) * g"),
    ("grad: sign", "(loss_scale * M * A * w) * g", "(-loss_scale * M * A * w) * g"),
    ("cap: max instead of min", "min(r, float(ratio_cap))", "max(r, float(ratio_cap))"),
    ("cap ignored in the gradient", "(loss_scale * M * A * w) * g", "(loss_scale * M * A * r) * g"),
    ("clip mask: eps_low and eps_high swapped", "    hi = np.log1p(eps_high)\n    lo = np.log1p(-eps_low) if eps_low < 1.0 else -np.inf",
     "    hi = np.log1p(eps_low)\n    lo = np.log1p(-eps_high) if eps_high < 1.0 else -np.inf"),
    ("clip mask: symmetric in the advantage", "if (adv > 0.0 and d > hi) or (adv < 0.0 and d < lo):", "if d > hi or d < lo:"),
    ("relaxation: sides swapped", "                if relax_sides & RELAX_HIGH:\n                    hi_eps = np.inf\n                if relax_sides & RELAX_LOW:\n                    lo_eps = np.inf",
     "                if relax_sides & RELAX_LOW:\n                    hi_eps = np.inf\n                if relax_sides & RELAX_HIGH:\n                    lo_eps = np.inf"),
    ("relaxation: applied to the likely tokens", "if relax_alpha > 0.0 and lmu < np.log(float(relax_alpha)):", "if relax_alpha > 0.0 and lmu > np.log(float(relax_alpha)):"),
    ("relaxation: keyed on the trainer's probability", "if relax_alpha > 0.0 and lmu < np.log(float(relax_alpha)):", "if relax_alpha > 0.0 and lpi < np.log(float(relax_alpha)):"),
    ("relaxation: applied to every token", "if relax_alpha > 0.0 and lmu < np.log(float(relax_alpha)):", "if relax_alpha > 0.0:"),
    ("mask rule none still masks", "            M = 1\n", "            M = dppo_mask(D, delta, A, lpi, lmu)\n"),
    ("entropy sign", "return float(-(pi[nz] * logpi[nz]).sum())", "return float((pi[nz] * logpi[nz]).sum())"),
    ("covered mass of pi uses mu", "mass_mu, mass_pi = p.sum(), q.sum()", "mass_mu, mass_pi = p.sum(), p.sum()"),
    ("full TV: half missing", "return 0.5 * np.abs(mu_probs - pi_probs).sum()", "return np.abs(mu_probs - pi_probs).sum()"),
    ("full KL as trust region: direction swapped", "d += np.exp(x) * (x - y)", "d += np.exp(y) * (y - x)"),
    ("full KL as trust region: weight missing", "d += np.exp(x) * (x - y)", "d += (x - y)"),
    ("full variants: rollout logits not normalised", "logmu = log_softmax(np.asarray(mu_logits[t], dtype=np.float64))",
     "logmu = np.asarray(mu_logits[t], dtype=np.float64)"),
    ("full variants: TV and KL swapped", "if variant == FULL_TV else full_kl_from_logs(logmu, logpi)",
     "if variant == FULL_KL else full_kl_from_logs(logmu, logpi)"),
    ("bf16 rounding truncates", "return np.ldexp(np.rint(m * 256.0) / 256.0, e)", "return np.ldexp(np.trunc(m * 256.0) / 256.0, e)"),
    ("bf16 rounding keeps 9 bits", "return np.ldexp(np.rint(m * 256.0) / 256.0, e)", "return np.ldexp(np.rint(m * 512.0) / 512.0, e)"),
    ("lm_head: weight not transposed in the gradient", 'out["grad_logits"] @ np.asarray(weight, dtype=np.float64) if want_grad',
     'out["grad_logits"] @ np.asarray(weight, dtype=np.float64)[::-1] if want_grad'),
    ("lm_head: weight gradient contracts the wrong index", 'out["grad_logits"].T @ np.asarray(hidden, dtype=np.float64) if want_grad',
     'out["grad_logits"].T[:, ::-1] @ np.asarray(hidden, dtype=np.float64) if want_grad'),
    ("lm_head: logits not rounded", "return bf16_round(hidden @ weight.T)", "return hidden @ weight.T"),
    ("anchor ignored by the divergence mask", "M = dppo_mask(D, delta, A, lpi, lanc)", "M = dppo_mask(D, delta, A, lpi, lmu)"),
    ("anchor ignored by the clip mask", "M = ratio_clip_mask(A, lpi, lanc, lo_eps, hi_eps)", "M = ratio_clip_mask(A, lpi, lmu, lo_eps, hi_eps)"),
    ("anchor ignored by the divergence", "D = binary_tv(lanc, lpi)", "D = binary_tv(lmu, lpi)"),
    ("anchor ignored by the reduced distributions", "reduced_distributions(logpi, a, lanc, ids, lps)", "reduced_distributions(logpi, a, lmu, ids, lps)"),
    ("anchor leaks into the importance weight", "        lanc = lmu if anchor_logp is None else float(anchor_logp[t])",
     "        lanc = lmu if anchor_logp is None else float(anchor_logp[t])\n        r = np.exp(lpi - lanc)\n        dummy = 0"),
    ("binary KL uses clamped-away 1-q", "one_minus_q = pi_row[:a].sum() + pi_row[a + 1:].sum()", "one_minus_q = pi_row[:a].sum()"),
]


def _count_failing_pins(source, tmp_path, monkeypatch):
    mutated = tmp_path / "dppo_oracle_mutated.py"
    mutated.write_text(source)
    spec = importlib.util.spec_from_file_location("dppo_oracle_mutated", str(mutated))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)

    from tests import test_oracle_pins as pins
    monkeypatch.setattr(pins, "O", mod)
    golden = os.path.join(ROOT, "tests", "golden")
    failures = 0
    for attr in dir(pins):
        fn = getattr(pins, attr)
        if not (attr.startswith("test_") and callable(fn)):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        argsets = [()]
        if marks:
            names = [n.strip() for n in marks[0].args[0].split(",")]
            argsets = [a if isinstance(a, tuple) and len(names) > 1 else (a,) for a in marks[0].args[1]]
        for args in argsets:
            kwargs = {}
            code = fn.__code__
            if "golden_dir" in code.co_varnames[:code.co_argcount]:
                kwargs["golden_dir"] = golden
            try:
                fn(*args, **kwargs)
            except Exception:      # any failing pin (assertion or crash) notices the mistake
                failures += 1
    return failures


def test_the_unmodified_oracle_passes_every_pin_under_this_harness(tmp_path, monkeypatch):
    assert _count_failing_pins(SRC, tmp_path, monkeypatch) == 0


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_some_pin(name, old, new, tmp_path, monkeypatch):
    assert SRC.count(old) == 1, f"mutation target not unique/present: {old!r}"
    assert _count_failing_pins(SRC.replace(old, new), tmp_path, monkeypatch) > 0, f"no pin noticed: {name}"
