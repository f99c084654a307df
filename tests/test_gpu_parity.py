"""GPU parity: the HIP path (through the C ABI) against the float64 oracle, element by element.

Small and medium cases compare every row; the full-size cases run the launch configuration
bench.py times and compare a sample of rows the oracle can do one by one, plus properties
that hold at any size."""
import numpy as np
import pytest
import torch

from paper_2602_04879_amd import binding as B
from paper_2602_04879_amd import workloads as W
from tests import parity as P

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def _run_and_compare(w, *, backward=True, in_place=False, flags=0, ld=None, shift=0.0, rows=None,
                     check_grad=True, rule=None, **mk):
    _say(f"[case] {w.name} T={w.T} V={w.V} K={w.K} variant={w.variant} ld={ld} in_place={in_place} flags={flags} shift={shift} rule={rule}")
    b = W.make_batch(w, DEV, ld=ld, shift_sampled=shift, **mk)
    rule = rule or {}
    b["rule"] = rule
    rows = np.arange(b["T"]) if rows is None else rows
    ref = P.oracle_rows(b, rows, want_grad=backward and check_grad)   # before an in-place run overwrites the logits
    res = B.run_batch(b, backward=backward, in_place=in_place, flags=flags, diagnostics=True, **rule)
    torch.cuda.synchronize()
    st = P.compare_rows(b, res, rows, check_grad=backward and check_grad, ref=ref)
    if len(rows) == b["T"]:
        P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    _say(f"       path={B.last_path()} {st}")
    return b, res, st


# --------------------------------------------------------------------------- small: every row
# V = 4096: one wave per row with the row in registers, or (forced) the general two-pass kernel
PATHS_SMALL_V = [(0, "resident"), (B.FLAG_FORCE_STREAMING, "streaming")]


@pytest.mark.parametrize("name", ["c1_tiny_binary_tv"])
@pytest.mark.parametrize("flags,path", PATHS_SMALL_V)
def test_c1_tiny_all_rows(name, flags, path):
    _run_and_compare(W.WORKLOADS[name], flags=flags)
    assert B.last_path() == path


@pytest.mark.parametrize("variant,K", [(W.BINARY_TV, 0), (W.BINARY_KL, 0), (W.TOPK_TV, 20), (W.TOPK_KL, 64)])
@pytest.mark.parametrize("shift", [0.0, 2.0])
@pytest.mark.parametrize("flags,path", PATHS_SMALL_V)
def test_c1_shape_all_variants_with_mask_stress(variant, K, shift, flags, path):
    w = W.scaled(W.WORKLOADS["c1_tiny_binary_tv"], variant=variant, K=K,
                 noise_std=1.0 if shift else 0.05, delta=0.05 if variant in (W.BINARY_KL, W.TOPK_KL) else 0.2)
    b, res, st = _run_and_compare(w, shift=shift, flags=flags)
    assert B.last_path() == path
    if shift:
        assert 0 < st["masked"] < b["T"]     # the stress recipe exercises both mask values


@pytest.mark.parametrize("name", ["c2_binary_tv", "c2_binary_kl"])
def test_c2_shape_subset_of_sequences(name):
    # full vocabulary and distribution of C2, 2 of its 16 sequences (the oracle does 1024 rows in seconds)
    w = W.scaled(W.WORKLOADS[name], n_seq=2)
    _run_and_compare(w)
    _run_and_compare(w, shift=2.0, in_place=True)


@pytest.mark.parametrize("name", ["c3_qwen3_binary_tv", "c4_qwen3_topk_tv", "c5_long_topk_kl"])
def test_qwen3_vocab_small_t(name):
    # V = 151936 (several tiles per row and a ragged tail: 151936 = 8 * 18992), 2 x 48 rows
    w = W.scaled(W.WORKLOADS[name], n_seq=2, seq_len=48, adv="normal")       # per-sequence N(0,1): never all zero
    _run_and_compare(w)
    _run_and_compare(w, shift=2.0, flags=B.FLAG_FORCE_STREAMING)


# --------------------------------------------------------------------------- resident-kernel shapes
@pytest.mark.parametrize("V,ld,expect", [
    (1016, 1016, "streaming"),         # below the smallest resident row
    (1024, 1024, "resident"),          # smallest resident row: one wave x 4 chunks, two of them used
    (2048, 2056, "resident"),          # one wave x 4 chunks exactly full, pitch > V
    (4104, 4104, "resident"),          # one vector into one wave x 16 chunks
    (8192, 8192, "resident"),          # longest row of one wave: 64 threads x 16 chunks, exactly full
    (8200, 8200, "resident"),          # one vector more: 256 threads x 4 chunks
    (16384, 16384, "resident"),        # 256 x 8 exactly full
    (12296, 12304, "resident"),        # pitch > V (still a multiple of 8)
    (40960, 40960, "resident"),        # 256 x 20 exactly full
    (40968, 40968, "resident"),        # first 512-thread shape (512 x 12)
    (100000, 100000, "resident"),      # 512 x 28, ragged last chunk
    (128256, 128256, "resident"),      # a Llama-3 sized vocabulary: 512 x 32
    (155648, 155648, "resident"),      # largest resident row: 512 x 38 exactly full
    (155656, 155656, "resident_long"), # one vector more: 39 chunks, 30 in registers and 9 in LDS
    (196608, 196608, "resident_long"), # 48 chunks exactly full: registers and LDS, nothing read twice
    (196616, 196624, "resident_long"), # one vector into the first chunk that passes through twice; pitch > V
    (229376, 229376, "resident_long"), # 56 chunks: one full window of them
    (229384, 229384, "resident_long"), # one vector into the second window
    (256000, 256000, "resident_long"), # a Gemma-2 sized vocabulary: 62.5 chunks
    (262144, 262144, "resident_long"), # longest row of this form: 64 chunks exactly full
    (262152, 262152, "streaming"),     # one vector more: the two-pass kernel
    (40004, 40004, "resident"),        # V not a multiple of 8: the ragged form (rows start 0, 8, 0, 8 bytes into a 16-byte block)
    (16384, 16388, "resident"),        # pitch not a multiple of 8: rows not 16-byte aligned, the ragged form
    (50257, 50257, "resident"),        # a GPT-2 sized vocabulary: odd, so every row starts 2 bytes further into its block
    (50257, 50264, "resident"),        # ... in a pitch that is a multiple of 8: aligned rows, ragged end
    (151643, 151643, "resident"),      # 512 x 38, odd
    (155585, 155591, "resident"),      # the longest ragged row: a frame of 19456 blocks at most
    (155586, 155586, "streaming"),     # one entry more: a frame of 19457 blocks for some rows
    (8190, 8190, "resident"),          # frames of 1024 to 1032 blocks: 256 threads x 8 chunks, the shortest frame ending with chunk 3
    (8181, 8181, "streaming"),         # frames of 1023 to 1031 blocks: no shape takes all of them within its slack
    (100008, 100008, "resident"),      # 16-byte aligned rows that do not start on 128-byte lines: the ragged form, on whole lines
    (1030, 1031, "resident"),          # smallest ragged shapes
])
@pytest.mark.parametrize("variant,K", [(W.BINARY_KL, 0), (W.TOPK_KL, 20)])
def test_resident_shapes_and_fallback(V, ld, expect, variant, K):
    w = W.Workload("shape", 3, 4, V, variant, 0.05, K=K, logit_std=3.0, noise_std=1.0, zipf_s=1.1, adv="normal", seed=31)
    b, res, st = _run_and_compare(w, ld=ld, shift=2.0)
    assert B.last_path() == expect


def test_resident_more_rows_than_workgroups_in_place_with_special_rows():
    """Several rows per persistent workgroup (T > 256 compute units), gradient in place, with ignored
    rows, zero-advantage rows and masked rows scattered among them."""
    w = W.Workload("persist", 3, 250, 16384, W.TOPK_TV, 0.1, K=20, logit_std=3.0, noise_std=1.0, adv="normal", seed=37)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    b["sampled_ids"][::11] = -1
    b["advantages"][5::13] = 0.0
    rows = np.arange(b["T"])
    ref = P.oracle_rows(b, rows)
    res = B.run_batch(b, in_place=True, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    st = P.compare_rows(b, res, rows, ref=ref)
    assert st["masked"] > 50
    P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    _say(f"       {st}")


def test_one_wave_per_row_many_rows_per_wave_in_place_with_special_rows():
    """V = 4096: one wave per row, more rows than resident waves (several rows per wave), gradient in
    place, ignored / zero-advantage / masked rows among them, Top-K with K beyond the wave's width."""
    w = W.Workload("waves", 8, 1200, 4096, W.TOPK_KL, 0.05, K=70, logit_std=3.0, noise_std=1.0, adv="normal", seed=41)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    b["sampled_ids"][::17] = -1
    b["advantages"][3::19] = 0.0
    rows = np.arange(b["T"])
    ref = P.oracle_rows(b, rows)
    res = B.run_batch(b, in_place=True, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    st = P.compare_rows(b, res, rows, ref=ref)
    assert st["masked"] > 50
    P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    _say(f"       {st}")


def test_rows_handed_out_at_run_time_match_rows_fixed_by_index():
    """Long rows with the gradient and many rows per workgroup: the kernel hands its rows out at run
    time (one counter, one loss term per row).  Every per-row output must be bit for bit what
    the form with rows fixed by the workgroup index writes, run after run, ignored / zero-advantage
    / masked rows included; the scalar loss is summed per row in a fixed order, so it too repeats
    bit for bit; and a workspace of the minimum size falls back to the fixed rows."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    T = 12 * cus + 37
    w = W.Workload("dynrows", 1, T, 100000, W.TOPK_KL, 0.05, K=20, logit_std=3.0, noise_std=1.0, zipf_s=1.1, adv="normal", seed=61)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    b["advantages"] = torch.randn(T, device=DEV)             # per token, so that both signs and sizes occur
    b["sampled_ids"][::17] = -1
    b["advantages"][5::19] = 0.0
    fixed = B.run_batch(b, diagnostics=True, flags=B.FLAG_STATIC_ROWS)
    runs = [B.run_batch(b, diagnostics=True) for _ in range(3)]
    small = B.alloc_outputs(T, DEV, want_diagnostics=True)
    small["workspace"] = torch.empty(B.WORKSPACE_BYTES, dtype=torch.uint8, device=DEV)
    rmin = B.run_batch(b, out=small)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    for r in runs + [rmin]:
        for k in ("loss_tok", "divergence", "mask", "diagnostics", "grad_logits"):
            assert torch.equal(fixed[k], r[k]), k
    for r in runs[1:]:
        assert torch.equal(runs[0]["loss"], r["loss"])
    assert torch.equal(fixed["loss"], rmin["loss"])
    assert abs(runs[0]["loss"].item() - fixed["loss"].item()) <= 1e-6 * abs(fixed["loss"].item())
    rows = np.arange(T)[::3]
    ref = P.oracle_rows(b, rows, want_grad=False)
    st = P.compare_rows(b, runs[0], rows, check_grad=False, ref=ref)
    P.check_loss_scalar(b, runs[0])
    P.compare_rows(b, runs[0], rows[::16])
    assert st["masked"] > 50
    _say(f"       {st}")


@pytest.mark.parametrize("V", [256000, 180000])
def test_long_rows_handed_out_at_run_time_and_fixed_with_special_rows(V):
    """Rows beyond the register file (registers + LDS + a tail read twice; V = 180000: registers +
    LDS only), several rows per workgroup, in place: rows handed out at run time must equal rows
    fixed by the workgroup index bit for bit, run after run, ignored / zero-advantage / masked rows
    and sampled tokens in every part of the row included; per-token outputs against the oracle on
    every row, gradients on a sample."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    T = 12 * cus + 37
    w = W.Workload("longrows", 1, T, V, W.TOPK_KL, 0.05, K=20, logit_std=3.0, noise_std=1.0, zipf_s=1.1, adv="normal", seed=67)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    b["advantages"] = torch.randn(T, device=DEV)
    b["sampled_ids"][::17] = -1
    b["advantages"][5::19] = 0.0
    # sampled tokens in the register part, the LDS part, both windows of the tail, and the last entry
    for t, a in zip(range(2, 62, 6), [0, 4095, 30 * 4096 - 1, 30 * 4096, 40 * 4096 + 77, 48 * 4096 - 1, 48 * 4096, 52 * 4096 + 5, 56 * 4096, V - 1]):
        b["sampled_ids"][t] = min(a, V - 1)
    fixed = B.run_batch(b, diagnostics=True, flags=B.FLAG_STATIC_ROWS)
    assert B.last_path() == "resident_long"
    runs = [B.run_batch(b, diagnostics=True) for _ in range(2)]
    torch.cuda.synchronize()
    assert B.last_path() == "resident_long"
    for r in runs:
        for k in ("loss_tok", "divergence", "mask", "diagnostics", "grad_logits"):
            assert torch.equal(fixed[k], r[k]), k
    assert torch.equal(runs[0]["loss"], runs[1]["loss"])
    assert abs(runs[0]["loss"].item() - fixed["loss"].item()) <= 1e-6 * abs(fixed["loss"].item())
    two_pass = B.run_batch(b, diagnostics=True, flags=B.FLAG_FORCE_STREAMING)
    torch.cuda.synchronize()
    assert B.last_path() == "streaming"
    assert torch.equal(two_pass["mask"], fixed["mask"])
    rows = np.arange(T)
    some = np.unique(np.concatenate([rows[:64], rows[::5], rows[-8:]]))
    ref = P.oracle_rows(b, some, want_grad=False)
    st = P.compare_rows(b, runs[0], some, check_grad=False, ref=ref)
    P.check_loss_scalar(b, runs[0])
    P.compare_rows(b, runs[0], np.unique(np.concatenate([np.arange(0, 62), rows[::97], rows[-3:]])))
    assert st["masked"] > 20
    # in place: the gradient over the logits
    inp = B.run_batch(b, in_place=True, diagnostics=True)
    torch.cuda.synchronize()
    assert torch.equal(inp["grad_logits"], fixed["grad_logits"]) and torch.equal(inp["loss_tok"], fixed["loss_tok"])
    _say(f"       {st}")


@pytest.mark.parametrize("V,rows_per_group,groups_per_cu", [(24576, 6, 24), (20488, 6, 24), (30000, 4, 24), (32768, 4, 24), (40960, 3, 16), (41000, 3, 16), (49152, 3, 16), (50304, 2, 32),
                                                             (57352, 2, 32), (65536, 2, 32),
                                                             # the ragged form: odd vocabularies, and rows that are 16-byte aligned but not on 128-byte lines
                                                             (24499, 6, 24), (32003, 4, 24), (40001, 3, 16), (50257, 2, 32), (32008, 4, 24)])
def test_groups_of_rows_per_workgroup_with_special_rows(V, rows_per_group, groups_per_cu):
    """Rows of middle length, forward + backward, many rows per compute unit: groups of 6 / 4 / 3 / 2
    consecutive rows per workgroup, handed out at run time, the last group incomplete.  Ignored, zero-advantage and
    masked rows, sampled tokens at both ends of the row and on chunk borders; per-token outputs
    against the oracle on 3000 rows (the first and last groups among them), gradients on a sample
    of those; run after run bit for bit the same; in place; and the one-row form (other shapes,
    so other summation orders) writes the same masks."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    T = groups_per_cu * cus * rows_per_group + 37
    K = 100 if V == 49152 else 20                                  # (beyond one wave's 64 lanes once)
    w = W.Workload("groups", 1, T, V, W.TOPK_KL, 0.05, K=K, logit_std=3.0, noise_std=1.0, zipf_s=1.1, adv="normal", seed=71)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    b["advantages"] = torch.randn(T, device=DEV)
    b["sampled_ids"][::17] = -1
    b["advantages"][5::19] = 0.0
    special = [0, 7, 8, 4095, 4096, 4097, V // 2, V - 4097, V - 9, V - 8, V - 1]
    for t, a in zip(range(2, 2 + 3 * len(special), 3), special):
        b["sampled_ids"][t] = max(0, min(a, V - 1))
        b["sampled_ids"][T - 1 - t] = max(0, min(a, V - 1))      # and in the last groups
    pad = 64
    gbuf = torch.full((T * V + 2 * pad,), 7.0, dtype=torch.bfloat16, device=DEV)     # canaries around the gradient
    runs = [B.run_batch(b, diagnostics=True, grad=gbuf[pad:pad + T * V].view(T, V)), B.run_batch(b, diagnostics=True)]
    torch.cuda.synchronize()
    assert B.last_path() == "resident_multi"
    assert torch.all(gbuf[:pad] == 7.0) and torch.all(gbuf[pad + T * V:] == 7.0)
    for k in ("loss", "loss_tok", "divergence", "mask", "diagnostics", "grad_logits"):
        assert torch.equal(runs[0][k], runs[1][k]), k
    fixed = B.run_batch(b, diagnostics=True, flags=B.FLAG_STATIC_ROWS)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    assert torch.equal(fixed["mask"], runs[0]["mask"])
    assert abs(runs[0]["loss"].item() - fixed["loss"].item()) <= 1e-5 * abs(fixed["loss"].item())
    rows = np.arange(T)
    some = np.unique(np.concatenate([rows[:1000], rows[-1000:], rows[1000:-1000:max(1, (T - 2000) // 1000)]]))
    masked = 0
    for r0 in range(0, len(some), 1024):
        rr = some[r0:r0 + 1024]
        ref = P.oracle_rows(b, rr, want_grad=False)
        st = P.compare_rows(b, runs[0], rr, check_grad=False, ref=ref)
        masked += st["masked"]
    _full_size_properties(b, runs[0])
    assert masked > 50
    st = P.compare_rows(b, runs[0], np.unique(np.concatenate([np.arange(0, 40), some[::53], rows[-40:]])))
    inp = B.run_batch(b, in_place=True, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident_multi"
    assert torch.equal(inp["grad_logits"], runs[0]["grad_logits"]) and torch.equal(inp["loss_tok"], runs[0]["loss_tok"])
    _say(f"       masked={masked} {st}")


def test_groups_of_rows_saturated_and_minus_inf():
    """pi(a_t) -> 1, blocks of -inf, every logit hugely negative or hugely positive: in groups of rows."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    T = 24 * cus * 4
    w = W.Workload("sat_groups", 1, T, 32768, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=0.2, adv="pm1", seed=73)
    b = W.make_batch(w, DEV)
    a = b["sampled_ids"].long()
    rows = torch.arange(b["T"], device=DEV)
    b["logits"][rows[:6], a[:6]] = torch.tensor([20.0, 30.0, 40.0, 50.0, 60.0, 80.0], device=DEV).bfloat16()
    b["logits"][6:8, 1000:30000] = float("-inf")
    b["logits"][8:10, 5:32768 - 5] = float("-inf")
    b["logits"][10, :] = -1.0e4
    b["logits"][11, :] = -50.0
    b["logits"][12, :] = 3.0e4
    for r in range(6, 10):                                   # keep the sampled token finite in those rows
        b["logits"][r, a[r]] = 1.0
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident_multi"
    assert torch.isfinite(res["divergence"]).all() and torch.isfinite(res["grad_logits"].float()).all()
    st = P.compare_rows(b, res, np.arange(64))
    _say(f"       {st}")


@pytest.mark.parametrize("V", [180224, 237568])
def test_long_rows_saturated_and_minus_inf(V):
    """pi(a_t) -> 1, blocks of -inf across the parts of the row (registers, LDS, the tail that is
    read twice), every logit hugely negative or hugely positive: on the long-row path."""
    w = W.Workload("sat_long", 2, 8, V, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=0.2, adv="pm1", seed=43)
    b = W.make_batch(w, DEV)
    a = b["sampled_ids"].long()
    rows = torch.arange(b["T"], device=DEV)
    b["logits"][rows[:6], a[:6]] = torch.tensor([20.0, 30.0, 40.0, 50.0, 60.0, 80.0], device=DEV).bfloat16()
    b["logits"][6:8, 1000:150000] = float("-inf")            # most of the register part
    b["logits"][8:10, 120000:V - 5] = float("-inf")          # the LDS part and the tail
    b["logits"][10, :] = -1.0e4
    b["logits"][11, :] = -50.0
    b["logits"][12, :] = 3.0e4
    for r in range(6, 10):                                   # keep the sampled token finite in those rows
        b["logits"][r, a[r]] = 1.0
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident_long"
    assert torch.isfinite(res["divergence"]).all() and torch.isfinite(res["grad_logits"].float()).all()
    st = P.compare_rows(b, res, np.arange(b["T"]))
    _say(f"       {st}")


def test_resident_saturated_rows():
    """pi(a_t) -> 1 on the register-resident path: 1 - pi(a_t) must keep its relative accuracy."""
    w = W.Workload("sat_res", 2, 8, 16384, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=0.2, adv="pm1", seed=41)
    b = W.make_batch(w, DEV)
    a = b["sampled_ids"].long()
    rows = torch.arange(b["T"], device=DEV)
    b["logits"][rows[:6], a[:6]] = torch.tensor([20.0, 30.0, 40.0, 50.0, 60.0, 80.0], device=DEV).bfloat16()
    b["logits"][6:10, 1000:9000] = float("-inf")
    b["logits"][10, :] = -1.0e4                    # every logit negative and far from 0
    b["logits"][11, :] = -50.0
    b["logits"][12, :] = 3.0e4
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    assert torch.isfinite(res["divergence"]).all() and torch.isfinite(res["grad_logits"].float()).all()
    st = P.compare_rows(b, res, np.arange(b["T"]))
    _say(f"       {st}")


# --------------------------------------------------------------------------- baselines' masks, ratio cap
@pytest.mark.parametrize("rule", [
    dict(mask_rule=B.MASK_NONE),                                              # PG-IS
    dict(mask_rule=B.MASK_NONE, ratio_cap=3.0),                               # PG-TIS / CISPO
    dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28),            # GRPO with Clip-Higher
    dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.27, ratio_cap=5.0),
    dict(mask_rule=B.MASK_DIVERGENCE, ratio_cap=5.0),                         # DPPO with the default cap of App. E
    dict(mask_rule=B.MASK_DIVERGENCE, ratio_cap=float("inf")),
])
@pytest.mark.parametrize("V,flags", [(16384, 0), (3001, 0), (16384, B.FLAG_FORCE_STREAMING)])
def test_mask_rules_and_ratio_cap(rule, V, flags):
    w = W.Workload("rules", 4, 24, V, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=1.0, adv="normal", seed=43)
    b, res, st = _run_and_compare(w, shift=2.0, rule=rule, flags=flags)
    if rule["mask_rule"] == B.MASK_NONE:
        assert st["masked"] == 0
    else:
        assert 0 < st["masked"] < b["T"]
    if rule.get("ratio_cap", 0) and rule["ratio_cap"] < float("inf"):
        r = res["diagnostics"][:, B.DIAG_RATIO]
        assert (r > rule["ratio_cap"]).any()           # the cap bites on some tokens


@pytest.mark.parametrize("V,path", [(4096, "resident"), (1000, "streaming"), (4091, "resident"), (16384, "resident"), (151936, "resident"), (200000, "resident_long")])
@pytest.mark.parametrize("variant,K,rule", [
    (W.BINARY_TV, 0, dict()),                                                           # decoupled DPPO (Sec. 5.2)
    (W.TOPK_KL, 20, dict()),
    (W.BINARY_KL, 0, dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28)),      # MiniRL (App. C.1)
    (W.BINARY_TV, 0, dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28, ratio_cap=3.0)),   # MiniRL-TIS
])
def test_mask_anchored_to_a_recomputed_policy(V, path, variant, K, rule):
    """anchor_logp: the mask (and the divergence it gates on) compares pi with the trainer's
    recomputed policy instead of the rollout policy; weight and loss keep r = pi / mu."""
    w = W.Workload("anchor", 3, 30, V, variant, 0.05 if variant in (W.BINARY_KL, W.TOPK_KL) else 0.2, K=K,
                   logit_std=3.0, noise_std=1.0, adv="normal", seed=97)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    g = torch.Generator(device="cpu").manual_seed(5)
    noise = torch.randn(b["T"], generator=g).to(DEV) * 0.5
    b["anchor_logp"] = torch.minimum(b["mu_logp"] + noise, torch.zeros_like(b["mu_logp"]))
    b["rule"] = rule
    rows = np.arange(b["T"])
    ref = P.oracle_rows(b, rows)
    res = B.run_batch(b, diagnostics=True, **rule)
    torch.cuda.synchronize()
    assert B.last_path() == path
    st = P.compare_rows(b, res, rows, ref=ref)
    P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    # the anchor matters on this batch: without it masks or divergences differ
    plain = dict(b)
    plain["anchor_logp"] = None
    res0 = B.run_batch(plain, **rule)
    torch.cuda.synchronize()
    assert (res0["mask"] != res["mask"]).any() or (res0["divergence"] != res["divergence"]).any()
    # ... and an anchor equal to the rollout policy is the same as none, bit for bit
    same = dict(b)
    same["anchor_logp"] = b["mu_logp"].clone()
    res1 = B.run_batch(same, **rule)
    torch.cuda.synchronize()
    for k in ("loss", "loss_tok", "divergence", "mask", "grad_logits"):
        assert torch.equal(res0[k], res1[k]), k
    assert 0 < st["masked"] < b["T"]
    _say(f"       {st}")


@pytest.mark.parametrize("V,path", [(4096, "resident"), (1000, "streaming"), (4091, "resident"), (32768, "resident"), (151936, "resident"), (200000, "resident_long")])
@pytest.mark.parametrize("sides", [B.RELAX_HIGH, B.RELAX_LOW, B.RELAX_HIGH | B.RELAX_LOW])
def test_clip_relaxed_for_low_probability_tokens(V, path, sides):
    """Sec. 6: the ratio-clip mask with its upper, lower or both thresholds infinite for tokens whose
    rollout probability is below alpha (Relax-high / Relax-low / Relax-both)."""
    w = W.Workload("relax", 3, 40, V, W.BINARY_TV, 0.2, logit_std=3.0, noise_std=1.0, adv="normal", seed=103)
    b = W.make_batch(w, DEV, shift_sampled=2.0)
    rule = dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28, relax_alpha=0.1, relax_sides=sides)
    b["rule"] = rule
    rows = np.arange(b["T"])
    ref = P.oracle_rows(b, rows)
    res = B.run_batch(b, diagnostics=True, **rule)
    torch.cuda.synchronize()
    assert B.last_path() == path
    st = P.compare_rows(b, res, rows, ref=ref)
    P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    grpo = B.run_batch(b, mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28)
    torch.cuda.synchronize()
    assert torch.all(res["mask"] >= grpo["mask"])                                  # relaxing only ever unmasks
    if sides == (B.RELAX_HIGH | B.RELAX_LOW):
        assert (res["mask"] != grpo["mask"]).any()
    _say(f"       {st}")


# --------------------------------------------------------------------------- edge cases
@pytest.mark.parametrize("V,ld", [(1, 1), (1, 8), (2, 2), (7, 7), (8, 8), (9, 11), (63, 63), (1001, 1001),
                                  (1000, 1003), (4097, 4100), (32768 + 5, 32768 + 8)])
@pytest.mark.parametrize("variant,K", [(W.BINARY_KL, 0), (W.TOPK_TV, 5)])
def test_ragged_vocab_and_pitch(V, ld, variant, K):
    K = min(K, V)
    w = W.Workload("ragged", 3, 5, V, variant, 0.05, K=K, logit_std=2.0, noise_std=0.5, adv="normal", seed=11)
    _run_and_compare(w, ld=ld)      # with ld > V the pad columns hold a poison value that must not be read


@pytest.mark.parametrize("V,ld,path", [(1000, 1016, "streaming"), (5003, 5011, "resident"), (5003, 5003, "resident"), (50257, 50264, "resident")])
def test_pitch_columns_untouched_and_canaries(V, ld, path):
    """Writes stay inside [T, V) of grad_logits and inside [T) of the per-token outputs: in the
    two-pass kernel, and in the ragged form of the register-resident one, which works on the aligned
    16-byte blocks around a row and must write the row's own entries only."""
    w = W.Workload("canary", 4, 9, V, W.TOPK_KL, 0.05, K=7, logit_std=2.0, noise_std=0.5, adv="normal", seed=5)
    b = W.make_batch(w, DEV, ld=ld)
    T, V = b["T"], b["V"]
    pad = 64
    gbuf = torch.full((T * ld + 2 * pad,), 7.0, dtype=torch.bfloat16, device=DEV)
    grad = gbuf[pad:pad + T * ld].view(T, ld)
    dbuf = torch.full((T + 2 * pad,), -3.0, dtype=torch.float32, device=DEV)
    lbuf = torch.full((T + 2 * pad,), -3.0, dtype=torch.float32, device=DEV)
    mbuf = torch.full((T + 2 * pad,), 9, dtype=torch.uint8, device=DEV)
    out = B.alloc_outputs(T, DEV)
    out["divergence"], out["loss_tok"], out["mask"] = dbuf[pad:pad + T], lbuf[pad:pad + T], mbuf[pad:pad + T]
    res = B.run_batch(b, out=out, grad=grad)
    torch.cuda.synchronize()
    assert B.last_path() == path
    assert torch.all(gbuf[:pad] == 7.0) and torch.all(gbuf[pad + T * ld:] == 7.0)
    assert torch.all(grad[:, V:] == 7.0)
    for buf, v in ((dbuf, -3.0), (lbuf, -3.0), (mbuf, 9)):
        assert torch.all(buf[:pad] == v) and torch.all(buf[pad + T:] == v)
    P.compare_rows(b, res, np.arange(T))


@pytest.mark.parametrize("V,ld", [(100003, 100003), (50257, 50257), (151643, 151646), (12345, 12345)])
def test_ragged_rows_in_registers_with_special_rows(V, ld):
    """Odd vocabularies (every row starts another 2 bytes into its 16-byte block) on the register-resident
    kernel, many rows per workgroup (rows handed out at run time where the shape has one workgroup per
    compute unit): sampled tokens in the first and last block of the row, ignored / zero-advantage /
    masked rows; every per-token output against the oracle, gradients on a sample; rows fixed by the
    workgroup index, forward only and in place write the same; nothing outside [T, V) is written."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    T = 12 * cus + 37
    w = W.Workload("ragged_rows", 1, T, V, W.TOPK_KL, 0.05, K=20, logit_std=3.0, noise_std=1.0, zipf_s=1.1, adv="normal", seed=81)
    b = W.make_batch(w, DEV, ld=ld, shift_sampled=2.0)
    b["advantages"] = torch.randn(T, device=DEV)
    b["sampled_ids"][::17] = -1
    b["advantages"][5::19] = 0.0
    special = [0, 1, 6, 7, 8, 9, V - 10, V - 9, V - 8, V - 7, V - 2, V - 1]
    for i, a in enumerate(special * 4):                      # rows 2 .. 49: every head offset meets every special id
        b["sampled_ids"][2 + i] = a
    pad = 64
    gbuf = torch.full((T * ld + 2 * pad,), 7.0, dtype=torch.bfloat16, device=DEV)
    grad = gbuf[pad:pad + T * ld].view(T, ld)
    res = B.run_batch(b, diagnostics=True, grad=grad)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    assert torch.all(gbuf[:pad] == 7.0) and torch.all(gbuf[pad + T * ld:] == 7.0) and torch.all(grad[:, V:] == 7.0)
    rows = np.arange(T)
    some = np.unique(np.concatenate([rows[:64], rows[::4], rows[-16:]]))
    ref = P.oracle_rows(b, some, want_grad=False)
    st = P.compare_rows(b, res, some, check_grad=False, ref=ref)
    P.check_loss_scalar(b, res)
    P.compare_rows(b, res, np.unique(np.concatenate([np.arange(0, 52), rows[::97], rows[-9:]])))
    assert st["masked"] > 20
    fixed = B.run_batch(b, diagnostics=True, flags=B.FLAG_STATIC_ROWS)
    fwd = B.run_batch(b, diagnostics=True, backward=False)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    for k in ("loss_tok", "divergence", "mask", "diagnostics"):
        assert torch.equal(fixed[k], res[k]), k
        assert torch.equal(fwd[k], res[k]), k
    assert torch.equal(fixed["grad_logits"][:, :V], grad[:, :V])
    inp = B.run_batch(b, in_place=True, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    assert torch.equal(inp["grad_logits"][:, :V], grad[:, :V]) and torch.equal(inp["loss_tok"], res["loss_tok"])
    _say(f"       {st}")


@pytest.mark.parametrize("V,ld,T,variant,K,off,path", [
    (37372, 37372, 17416, W.TOPK_KL, 70, 8, "resident_multi"),
    (58002, 58013, 17237, W.TOPK_TV, 20, 1, "resident_multi"),
    (21787, 21790, 45892, W.TOPK_TV, 20, 1, "resident_multi"),
    (50450, 50461, 19817, W.BINARY_TV, 0, 5, "resident_multi"),
    (49872, 49872, 20051, W.BINARY_TV, 0, 24, "resident_multi"),
    (6682, 6720, 26116, W.BINARY_TV, 0, 24, "resident"),
    (2363, 2363, 52226, W.BINARY_TV, 0, 1, "resident"),
    (122024, 122025, 8195, W.TOPK_KL, 70, 0, "resident"),
    (154736, 154737, 6462, W.BINARY_KL, 0, 0, "resident"),
    (174024, 174080, 5744, W.TOPK_KL, 70, 0, "resident_long"),
])
def test_fast_paths_agree_with_the_two_pass_kernel_on_odd_layouts(V, ld, T, variant, K, off, path):
    """Vocabulary sizes, pitches and buffer offsets (in elements, the same for logits and gradient)
    off every boundary the fast kernels like, at sizes the oracle would take minutes for: the
    register-resident kernels (plain and ragged, one row and groups of rows) against the general
    two-pass kernel on the same call: masks equal outside the 1e-5 band around delta, divergences,
    loss terms and gradients within the parity tolerances, and no byte outside [T, V) written."""
    delta = 0.05 if variant in (W.BINARY_KL, W.TOPK_KL) else 0.15
    w = W.Workload("layouts", 1, T, V, variant, delta, K=K, logit_std=3.0, noise_std=1.0, zipf_s=1.1, adv="normal", seed=V + T)
    b = W.make_batch(w, DEV, ld=ld, shift_sampled=2.0)
    b["advantages"] = torch.randn(T, device=DEV)
    b["sampled_ids"][::23] = -1
    for i, a in enumerate([0, 1, 7, 8, V - 1, V - 2, V - 8, V - 9, V // 2] * 6):
        b["sampled_ids"][3 + 5 * i] = a
    big = torch.zeros(T * ld + 64, dtype=torch.bfloat16, device=DEV)
    big[off:off + T * ld] = b["logits"].reshape(-1)
    b["logits"] = big[off:off + T * ld].view(T, ld)
    gbuf = torch.full((T * ld + 64,), 7.0, dtype=torch.bfloat16, device=DEV)
    grad = gbuf[off:off + T * ld].view(T, ld)
    r = B.run_batch(b, diagnostics=True, grad=grad)
    assert B.last_path() == path
    s = B.run_batch(b, diagnostics=True, flags=B.FLAG_FORCE_STREAMING)
    torch.cuda.synchronize()
    assert torch.all(gbuf[:off] == 7.0) and torch.all(gbuf[off + T * ld:] == 7.0) and torch.all(grad[:, V:] == 7.0)
    D1, D2 = r["divergence"].double(), s["divergence"].double()
    same = r["mask"] == s["mask"]
    assert torch.all(same | ((D1 - delta).abs() < 1e-5))
    assert torch.all((D1 - D2).abs() <= 1e-6 + 1e-4 * D2.abs())
    lt1, lt2 = r["loss_tok"].double()[same], s["loss_tok"].double()[same]
    assert torch.all((lt1 - lt2).abs() <= 1e-5 * (1 + lt2.abs()))
    g1, g2 = grad[:, :V].float()[same], s["grad_logits"][:, :V].float()[same]
    assert torch.all((g1 - g2).abs() <= 2e-2 * g2.abs() + 1e-30)
    assert 0 < (r["mask"] == 0).sum().item() < T


def test_misaligned_gradient_buffer_takes_elementwise_path():
    w = W.Workload("misaligned", 2, 7, 2051, W.BINARY_TV, 0.1, logit_std=2.0, noise_std=0.5, adv="pm1", seed=3)
    b = W.make_batch(w, DEV)
    T, V = b["T"], b["V"]
    gbuf = torch.zeros(T * V + 8, dtype=torch.bfloat16, device=DEV)
    grad = gbuf[3:3 + T * V].view(T, V)      # 6 bytes off the logits' alignment
    res = B.run_batch(b, grad=grad)
    torch.cuda.synchronize()
    assert B.last_path() == "streaming"
    P.compare_rows(b, res, np.arange(T))
    # logits themselves at an odd element offset
    lbuf = torch.zeros(T * V + 8, dtype=torch.bfloat16, device=DEV)
    lbuf[5:5 + T * V] = b["logits"].reshape(-1)
    b2 = dict(b)
    b2["logits"] = lbuf[5:5 + T * V].view(T, V)
    res = B.run_batch(b2)
    torch.cuda.synchronize()
    P.compare_rows(b2, res, np.arange(T))
    # in place both share the misalignment: the ragged form of the register-resident kernel, whose
    # first frame begins 10 bytes in front of the first row
    res = B.run_batch(b2, in_place=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    P.compare_rows(b, res, np.arange(T))
    assert torch.all(lbuf[:5] == 0) and torch.all(lbuf[5 + T * V:] == 0)


def test_ignored_rows_padding_ids_and_zero_advantage():
    w = W.Workload("ignored", 4, 8, 3000, W.TOPK_TV, 0.05, K=12, logit_std=2.0, noise_std=0.5, adv="normal", seed=9)
    b = W.make_batch(w, DEV)
    b["sampled_ids"][::5] = -1
    b["sampled_ids"][3::7] = b["V"] + 10          # outside the vocabulary: also ignored
    b["mu_topk_ids"][:, 4] = -1                   # padding entries
    b["mu_topk_ids"][1::2, 9] = b["V"]
    b["advantages"][2::6] = 0.0
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    P.compare_rows(b, res, np.arange(b["T"]))
    ign = (b["sampled_ids"] < 0) | (b["sampled_ids"] >= b["V"])
    assert torch.all(res["grad_logits"][ign] == 0) and torch.all(res["mask"][ign] == 0)
    assert torch.all(res["divergence"][ign] == 0) and torch.all(res["loss_tok"][ign] == 0)
    assert torch.all(res["grad_logits"][b["advantages"] == 0] == 0)


def test_topk_contains_sampled_token_and_k_beyond_one_wave():
    w = W.Workload("bigk", 2, 6, 5000, W.TOPK_KL, 0.05, K=150, logit_std=3.0, noise_std=0.3, adv="pm1", seed=13)
    b, res, _ = _run_and_compare(w)
    hit = (b["mu_topk_ids"] == b["sampled_ids"][:, None]).any(1)
    assert hit.any()       # a_t inside mu's top-K: the de-duplication path ran


def test_topk_with_k0_equals_binary():
    w = W.Workload("k0", 2, 8, 777, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=0.5, adv="pm1", seed=17)
    b = W.make_batch(w, DEV)
    r_bin = B.run_batch(b)
    b2 = dict(b)
    b2["variant"] = W.TOPK_KL
    r_top = B.run_batch(b2)
    torch.cuda.synchronize()
    assert torch.equal(r_bin["divergence"], r_top["divergence"]) and torch.equal(r_bin["mask"], r_top["mask"])
    assert torch.equal(r_bin["grad_logits"], r_top["grad_logits"])


def test_saturated_and_minus_inf_logits():
    w = W.Workload("sat", 2, 6, 4096, W.BINARY_KL, 0.05, logit_std=2.0, noise_std=0.2, adv="pm1", seed=21)
    b = W.make_batch(w, DEV)
    a = b["sampled_ids"].long()
    rows = torch.arange(b["T"], device=DEV)
    b["logits"][rows[:4], a[:4]] = 60.0            # pi(a) == 1 to fp32: 1 - pi(a) underflows
    b["logits"][4:8, 100:2000] = float("-inf")     # masked vocabulary entries
    b["logits"][8, :] = -1.0e4                     # flat, far from 0
    b["logits"][9, :] = 3.0e4
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    assert torch.isfinite(res["divergence"]).all() and torch.isfinite(res["loss"]).all()
    assert torch.isfinite(res["grad_logits"].float()).all()
    P.compare_rows(b, res, np.arange(b["T"]))
    assert torch.all(res["grad_logits"][4:8, 100:2000] == 0)


def test_empty_and_single_row():
    # one row on every kernel path: two-pass, one wave per row, 256 and 512 threads, long rows
    for V, path in ((513, "streaming"), (4096, "resident"), (32768, "resident"), (151936, "resident"), (256000, "resident_long")):
        w1 = W.Workload("one", 1, 1, V, W.BINARY_TV, 0.1, logit_std=2.0, noise_std=0.5, adv="pm1", seed=2)
        _run_and_compare(w1)
        assert B.last_path() == path
    w = W.Workload("one", 1, 1, 513, W.BINARY_TV, 0.1, logit_std=2.0, noise_std=0.5, adv="pm1", seed=2)
    b = W.make_batch(w, DEV)
    out = B.alloc_outputs(0, DEV)
    out["loss"].fill_(5.0)
    args = B.make_args(b["logits"][:0], b["sampled_ids"][:0], b["mu_logp"][:0], b["advantages"][:0], 0.1,
                       W.BINARY_TV, 1.0, out, V=513, grad_logits=b["logits"][:0])
    args.ld = 513
    B.dppo_loss_fwd_bwd(args)
    B.dppo_loss_fwd(args)
    torch.cuda.synchronize()
    assert out["loss"].item() == 0.0


def test_forward_only_matches_forward_backward_and_runs_are_bitwise_reproducible():
    w = W.scaled(W.WORKLOADS["c4_qwen3_topk_tv"], n_seq=2, seq_len=40, adv="normal")
    b = W.make_batch(w, DEV, shift_sampled=1.0)
    r1 = B.run_batch(b)
    path1 = B.last_path()
    r2 = B.run_batch(b)
    rf = B.run_batch(b, backward=False)
    pathf = B.last_path()
    rs = B.run_batch(b, flags=B.FLAG_FORCE_STREAMING)
    rsf = B.run_batch(b, backward=False, flags=B.FLAG_FORCE_STREAMING)
    torch.cuda.synchronize()
    assert path1 == "resident" and pathf == "resident" and B.last_path() == "streaming"
    for k in ("loss", "loss_tok", "divergence", "mask"):
        assert torch.equal(r1[k], r2[k]), k                 # same path twice: bit for bit
        assert torch.equal(r1[k], rf[k]), k                 # forward-only == forward of fwd+bwd (same statistics code)
    # the two-pass kernel runs forward-only calls with smaller workgroups (no second pass to keep
    # the row in cache for): the same sums in another order
    assert torch.equal(rs["mask"], rsf["mask"])
    torch.testing.assert_close(rs["divergence"], rsf["divergence"], rtol=1e-4, atol=2e-7)
    torch.testing.assert_close(rs["loss_tok"], rsf["loss_tok"], rtol=1e-4, atol=2e-7 * b["advantages"].abs().max().item())
    torch.testing.assert_close(rs["loss"], rsf["loss"], rtol=1e-4, atol=1e-9)
    assert torch.equal(r1["grad_logits"], r2["grad_logits"])
    assert r1["grad_logits"].float().abs().max().item() > 0 and 0 < (r1["mask"] == 0).sum().item() < b["T"]
    # the two kernel paths differ only by summation order
    assert torch.equal(r1["mask"], rs["mask"])
    torch.testing.assert_close(r1["divergence"], rs["divergence"], rtol=1e-4, atol=2e-7)
    torch.testing.assert_close(r1["loss_tok"], rs["loss_tok"], rtol=1e-4, atol=2e-7 * b["advantages"].abs().max().item())
    torch.testing.assert_close(r1["grad_logits"].float(), rs["grad_logits"].float(), rtol=2 ** -7, atol=1e-30)


@pytest.mark.parametrize("name", ["c2_binary_kl", "c5_long_topk_kl"])
def test_forward_only_against_oracle(name):
    w = W.scaled(W.WORKLOADS[name], n_seq=2, seq_len=40, group=2)
    _run_and_compare(w, backward=False, shift=2.0)
    _run_and_compare(w, backward=False, shift=2.0, flags=B.FLAG_FORCE_STREAMING)


def test_other_stream_and_loss_tok_optional():
    w = W.Workload("stream", 2, 16, 2048, W.TOPK_TV, 0.1, K=8, logit_std=2.0, noise_std=0.5, adv="pm1", seed=4)
    b = W.make_batch(w, DEV)
    ref = B.run_batch(b)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    out = B.alloc_outputs(b["T"], DEV, want_loss_tok=False)
    res = B.run_batch(b, out=out, stream=s)
    s.synchronize()
    assert torch.equal(ref["divergence"], res["divergence"]) and torch.equal(ref["grad_logits"], res["grad_logits"])
    assert torch.equal(ref["loss"], res["loss"])


def test_error_codes_on_device():
    w = W.Workload("err", 1, 4, 64, W.BINARY_TV, 0.1, seed=1)
    b = W.make_batch(w, DEV)
    out = B.alloc_outputs(b["T"], DEV)
    args = B.make_args(b["logits"], b["sampled_ids"], b["mu_logp"], b["advantages"], 0.1, 7, 1.0, out,
                       grad_logits=torch.empty_like(b["logits"]))
    with pytest.raises(B.DppoError) as e:
        B.dppo_loss_fwd_bwd(args)
    assert e.value.status == 4


# --------------------------------------------------------------------------- full size
def _sample_rows(b, res, n=64, seed=0):
    """First, last, masked rows, zero-advantage rows, the largest |coefficient| row, random rows."""
    T = b["T"]
    rng = np.random.default_rng(seed)
    rows = {0, T - 1}
    M = res["mask"].cpu().numpy()
    A = b["advantages"].cpu().numpy()
    lt = res["loss_tok"].abs().cpu().numpy()
    rows |= set(np.nonzero(M == 0)[0][:6].tolist())
    rows |= set(np.nonzero(A == 0)[0][:3].tolist())
    rows.add(int(lt.argmax()))
    rows |= set(rng.choice(T, n, replace=False).tolist())
    return np.array(sorted(rows))


def _full_size_properties(b, res):
    T = b["T"]
    M, D = res["mask"], res["divergence"]
    assert torch.all((M == 0) | (M == 1)) and torch.all(D >= -1e-7) and torch.isfinite(D).all()
    P.check_loss_scalar(b, res)
    # softmax-minus-onehot rows sum to ~0 (bf16 rounding of ~V entries) -- checked on a slice
    g = res["grad_logits"][: min(T, 2048), : b["V"]].float()
    s = g.sum(1).abs()
    scale = g.abs().sum(1)
    assert torch.all(s <= 4e-3 * scale + 1e-30)
    zero = torch.nonzero((b["advantages"] == 0) | (M == 0)).flatten()[:64]
    assert torch.all(res["grad_logits"][zero] == 0)


@pytest.mark.parametrize("name,path", [("c3_qwen3_binary_tv", "resident"), ("c4_qwen3_topk_tv", "resident"), ("c8_vocab256k_binary_tv", "resident_long"),
                                       ("c9_vocab32k_binary_tv", "resident_multi"), ("c10_vocab151643_binary_tv", "resident")])
def test_full_size_headline_configs(name, path):
    w = W.WORKLOADS[name]
    _say(f"[case] full size {name} T={w.T} V={w.V}")
    b = W.make_batch(w, DEV, rows_per_step=2048)
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    _say(f"       path={B.last_path()} loss={res['loss'].item():.6e} masked={(res['mask'] == 0).sum().item()}")
    assert B.last_path() == path
    _full_size_properties(b, res)
    rows = _sample_rows(b, res)
    st = P.compare_rows(b, res, rows)
    _say(f"       {st}")
    # every row's per-token scalars on a larger sample (no gradient): 2048 rows
    rows2 = np.random.default_rng(1).choice(b["T"], 2048, replace=False)
    st2 = P.compare_rows(b, res, np.sort(rows2), check_grad=False)
    _say(f"       {st2}")


def _run_chunked(b, w, out, backward, in_place):
    """The caller-side chunking of the long-response configuration: one call per chunk_rows rows on
    one stream, one scalar loss per call."""
    T = b["T"]
    losses = []
    for c0 in range(0, T, w.chunk_rows):
        c1 = min(T, c0 + w.chunk_rows)
        o = dict(out)
        o["loss"] = torch.empty(1, dtype=torch.float32, device=DEV)
        for k in ("loss_tok", "divergence", "mask"):
            o[k] = out[k][c0:c1]
        B.run_batch(b, backward=backward, in_place=in_place, out=o, rows=(c0, c1))
        losses.append(o["loss"])
    torch.cuda.synchronize()
    res = dict(out)
    res["grad_logits"] = b["logits"] if backward else None
    res["loss"] = torch.stack(losses).double().sum().float()
    return res


def test_full_size_long_response_chunked_in_place():
    """C5: T = 131072 rows processed as 8 calls of 16384 rows on one stream, gradient written in
    place over the logits; the 8 scalar losses add up.  A forward-only pass (which leaves the logits
    alone) picks the sample: gradient rows = first, last, the rows either side of a chunk boundary,
    masked rows, the largest |coefficient| row and 64 random rows; per-token scalars on 2048 rows."""
    w = W.WORKLOADS["c5_long_topk_kl"]
    _say(f"[case] full size {w.name} T={w.T} V={w.V} chunks of {w.chunk_rows}")
    b = W.make_batch(w, DEV, rows_per_step=2048)
    T = b["T"]
    fwd = _run_chunked(b, w, B.alloc_outputs(T, DEV), backward=False, in_place=False)
    assert (fwd["mask"] == 0).sum().item() > 0        # the recipe leaves some tokens masked
    rows = np.unique(np.concatenate([_sample_rows(b, fwd, n=64, seed=5), [w.chunk_rows - 1, w.chunk_rows, T - w.chunk_rows]]))
    assert (fwd["mask"][torch.as_tensor(rows).to(DEV)] == 0).any() and len(rows) >= 64
    rows2 = np.sort(np.random.default_rng(6).choice(T, 2048, replace=False))
    ref = P.oracle_rows(b, rows)                       # before the logits are overwritten
    ref2 = [P.oracle_rows(b, rows2[i:i + 512], want_grad=False) for i in range(0, len(rows2), 512)]
    fwd = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in fwd.items() if k in ("loss", "loss_tok", "divergence", "mask")}
    res = _run_chunked(b, w, B.alloc_outputs(T, DEV), backward=True, in_place=True)
    _say(f"       path={B.last_path()} loss={res['loss'].item():.6e} masked={(res['mask'] == 0).sum().item()}")
    for k in ("loss", "loss_tok", "divergence", "mask"):
        assert torch.equal(fwd[k], res[k]), k          # forward-only == forward of forward+backward
    st = P.compare_rows(b, res, rows, ref=ref)
    _say(f"       {st}")
    for i, r2 in zip(range(0, len(rows2), 512), ref2):
        st2 = P.compare_rows(b, res, rows2[i:i + 512], check_grad=False, ref=r2)
    _say(f"       {st2}")
    P.check_loss_scalar(b, res)


@pytest.mark.parametrize("name", ["c2_binary_tv", "c2_binary_kl"])
def test_c2_at_its_full_size(name):
    """C2 as stated: T = 8192 rows of V = 32768 (32 rows per persistent workgroup slot); per-token
    scalars and the scalar loss on every row, the gradient on 64 rows (first, last, masked,
    zero-advantage and largest-coefficient rows among them)."""
    w = W.WORKLOADS[name]
    _say(f"[case] full size {name} T={w.T} V={w.V}")
    b = W.make_batch(w, DEV)
    res = B.run_batch(b, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "resident"
    _full_size_properties(b, res)
    T = b["T"]
    tot = 0.0
    for r0 in range(0, T, 2048):
        rr = np.arange(r0, min(T, r0 + 2048))
        ref = P.oracle_rows(b, rr, want_grad=False)
        st = P.compare_rows(b, res, rr, check_grad=False, ref=ref)
        tot += float(ref["loss_tok"].sum())
    P.check_loss_scalar(b, res, tot)
    st = P.compare_rows(b, res, _sample_rows(b, res, n=56, seed=2))
    _say(f"       path={B.last_path()} loss={res['loss'].item():.6e} masked={(res['mask'] == 0).sum().item()} {st}")


# --------------------------------------------------------------------------- HIP graph capture
def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """The library allocates nothing, never synchronises and clears nothing with memset: a call is
    capturable.  Capture forward+backward of two shapes (both kernel paths) in one graph, replay it
    several times with eager work and synchronisations in between, and compare every replay bit for
    bit with the eager result."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    shapes = [W.scaled(W.WORKLOADS["c2_binary_kl"], n_seq=2, seq_len=96), W.scaled(W.WORKLOADS["c1_tiny_binary_tv"], K=8, variant=W.TOPK_TV, V=1000),
              W.scaled(W.WORKLOADS["c1_tiny_binary_tv"], K=8, variant=W.TOPK_TV, V=4091),     # the ragged form of the register-resident kernel
              # rows handed out at run time (a counter-clearing kernel in front, no memset), and the long-row kernel
              W.Workload("graph_dyn", 1, 12 * cus + 5, 100000, W.TOPK_KL, 0.05, K=20, logit_std=3.0, noise_std=1.0, adv="normal", seed=63),
              W.Workload("graph_long", 1, 40, 200000, W.BINARY_TV, 0.2, logit_std=3.0, noise_std=1.0, adv="normal", seed=64),
              # groups of rows per workgroup, handed out at run time
              W.Workload("graph_groups_dyn", 1, 16 * cus * 3 + 1, 49152, W.TOPK_TV, 0.2, K=20, logit_std=3.0, noise_std=1.0, adv="normal", seed=66)]
    batches = [W.make_batch(w, DEV, shift_sampled=1.0) for w in shapes]
    eager = []
    for b in batches:
        r = B.run_batch(b, diagnostics=True)
        torch.cuda.synchronize()
        eager.append({k: r[k].clone() for k in ("loss", "loss_tok", "divergence", "mask", "grad_logits", "diagnostics")})
    paths = set()
    outs = [B.alloc_outputs(b["T"], DEV, want_diagnostics=True) for b in batches]
    grads = [torch.empty_like(b["logits"]) for b in batches]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for b, o, gr in zip(batches, outs, grads):
                B.run_batch(b, out=o, grad=gr)          # enqueued on the capturing (current) stream
                paths.add(B.last_path())
    assert paths == {"resident", "streaming", "resident_long", "resident_multi"}
    scratch = torch.zeros(1 << 20, device=DEV)
    for rep in range(3):
        for o, gr in zip(outs, grads):                   # poison the outputs between replays
            for k in ("loss", "loss_tok", "divergence", "diagnostics"):
                o[k].fill_(float("nan"))
            o["mask"].fill_(7)
            gr.fill_(float("nan"))
        scratch.add_(1.0)                                # eager work of the program itself
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for e, o, gr in zip(eager, outs, grads):
            for k in ("loss", "loss_tok", "divergence", "mask", "diagnostics"):
                assert torch.equal(e[k], o[k]), (rep, k)
            assert torch.equal(e["grad_logits"], gr), rep
    _say(f"       graph with the kernel paths {sorted(paths)} replayed 3 times, bitwise equal to eager")


# --------------------------------------------------------------------------- measurement utilities
def test_probe_kernels_copy_fill_read():
    """The plain copy / fill / read kernels that the benchmark compares the loss kernels with do what
    they say, byte for byte, and leave everything else alone."""
    g = torch.Generator(device=DEV); g.manual_seed(7)
    n = (1 << 20) + 48
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, generator=g, device=DEV)
    dst = torch.zeros(n + 32, dtype=torch.uint8, device=DEV)
    B.probe_copy(dst[:n], src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and (dst[n:] == 0).all()
    B.probe_fill(dst[:n], 0x3c003c00)
    torch.cuda.synchronize()
    assert (dst[:n].view(torch.int32) == 0x3c003c00).all() and (dst[n:] == 0).all()
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    B.probe_read(src, sink)
    torch.cuda.synchronize()
    assert sink.item() == 0
    # row by row, with a pitch: columns past the row stay untouched; more rows than workgroups
    rows, cols, ld = 700, 4104, 4112
    a = torch.randn((rows, ld), generator=g, device=DEV).bfloat16()
    b = torch.full((rows, ld), -7.0, dtype=torch.bfloat16, device=DEV)
    B.probe_copy_rows(b[:, :cols], a[:, :cols])
    torch.cuda.synchronize()
    assert torch.equal(b[:, :cols], a[:, :cols]) and (b[:, cols:] == -7.0).all()
    # the register-resident copy (the loss kernel's memory pattern): a ragged row length, the longest
    # row it holds, more rows than workgroups and fewer
    for rows, cols, ld in ((700, 4104, 4112), (300, 155648, 155648), (5, 151936, 151936)):
        a = torch.randn((rows, ld), generator=g, device=DEV).bfloat16()
        b = torch.full((rows, ld), -7.0, dtype=torch.bfloat16, device=DEV)
        B.probe_copy_resident(b[:, :cols], a[:, :cols])
        torch.cuda.synchronize()
        assert torch.equal(b[:, :cols], a[:, :cols]) and (b[:, cols:] == -7.0).all()
    with pytest.raises(B.DppoError):
        B.probe_copy_resident(torch.empty((2, 155656), dtype=torch.bfloat16, device=DEV), torch.empty((2, 155656), dtype=torch.bfloat16, device=DEV))


def test_probe_matrix_core_loop():
    """The products-only loop that gives the matrix-core ceiling: runs for both instruction shapes,
    reports its operation count, is deterministic, and rejects what it cannot run."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.full((cus * 256 + 64,), -3.0, dtype=torch.float32, device=DEV)
    for shape in (16, 32):
        assert B.probe_mfma(shape, 0, out) == 0.0
        torch.cuda.synchronize()
        assert (out[:cus * 256] == 0).all() and (out[cus * 256:] == -3.0).all()
        fl = B.probe_mfma(shape, 3, out)
        torch.cuda.synchronize()
        assert fl == 2.0 * (524288 if shape == 16 else 262144) * 4 * cus * 3
        first = out.clone()
        assert torch.isfinite(first[:cus * 256]).all() and (first[:cus * 256] != 0).any()
        B.probe_mfma(shape, 3, out)
        torch.cuda.synchronize()
        assert torch.equal(out, first)
        out[:cus * 256] = -3.0
    with pytest.raises(B.DppoError):
        B.probe_mfma(8, 1, out)
    with pytest.raises(B.DppoError):
        B.probe_mfma(16, 1, out[:1024])
    torch.cuda.synchronize()
    assert (out == -3.0).all()
