"""GPU parity of the path that starts from the final hidden states (logits formed chunk by chunk on
the matrix cores, never [T, V] at once; gradient with respect to the hidden states) against the
float64 oracle, through the C ABI.

Strict cases use inputs whose logits are exact in fp32 whatever the order of accumulation, so the
bf16 logits of both sides are the same numbers and the per-token bar of the logits path applies
unchanged.  With ordinary inputs an fp32-accumulated logit can fall on the other side of a bf16
rounding boundary than the exact product does; those cases compare the rows where no token that
matters sits that close to a boundary (decided on the oracle side alone)."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import dppo_oracle as O
from paper_2602_04879_amd import binding as B
from paper_2602_04879_amd import workloads as W
from tests import parity as P
from tests.test_gpu_parity import DEV, _say

pytestmark = pytest.mark.gpu


# Relative standard deviation of a logit-gradient entry as the loss kernels leave it: one rounding to
# bf16 (8 significant bits) of a value with mantissa m in [1, 2) is uniform within 2^-8 / m relative,
# variance 2^-16 / (3 m^2), and with a log-uniform density of mantissas E[1/m^2] = (3/8) / ln 2.
SIGMA_BF16 = 2.0 ** -8 * np.sqrt((3.0 / 8.0) / np.log(2.0) / 3.0)


def _oracle(b, rows, **rule):
    sel = torch.as_tensor(np.asarray(rows, dtype=np.int64)).to(b["hidden"].device)
    tk_i = b["mu_topk_ids"][sel].cpu().numpy() if b["mu_topk_ids"] is not None else None
    tk_l = b["mu_topk_logp"][sel].cpu().numpy() if b["mu_topk_logp"] is not None else None
    return O.lmhead_dppo_loss(b["hidden"][sel].float().cpu().numpy(), b["weight"].float().cpu().numpy(),
                              b["sampled_ids"][sel].cpu().numpy(), b["mu_logp"][sel].cpu().numpy(),
                              b["advantages"][sel].cpu().numpy(), b["delta"], b["variant"], b["loss_scale"], tk_i, tk_l,
                              anchor_logp=(b["anchor_logp"][sel].cpu().numpy() if b.get("anchor_logp") is not None else None), **rule)


def _check_grad_hidden(b, res, rows, ref, skip=None):
    """|gpu - ref| <= 1e-2 |ref| + 6 sigma, sigma the standard deviation of what rounding each
    logit-gradient entry to bf16 leaves on the sum over the vocabulary (SIGMA_BF16 relative per
    entry, independent over the vocabulary); 6 sigma because a test looks at up to 10^6 entries."""
    g = res["grad_hidden"][torch.as_tensor(rows).to(DEV)].double().cpu().numpy()
    Wd = b["weight"].double().cpu().numpy()
    sigma = np.sqrt((ref["grad_logits"] ** 2) @ (Wd ** 2)) * SIGMA_BF16
    tol = 1e-2 * np.abs(ref["grad_hidden"]) + 6.0 * sigma + 1e-30
    err = np.abs(g - ref["grad_hidden"])
    if skip is not None:
        err[skip] = 0.0
    if not np.all(err <= tol):
        i, j = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"grad_hidden row {rows[i]} col {j}: gpu {g[i, j]:.6e} ref {ref['grad_hidden'][i, j]:.6e} tol {tol[i, j]:.3e}")
    nz = np.abs(ref["grad_hidden"]) > 0
    return float(np.median(err[nz] / np.abs(ref["grad_hidden"][nz]))) if nz.any() else 0.0


def _check_grad_weight(b, res, ref, M):
    """All T rows were run and compared: the summed weight gradient against the oracle's, within
    1e-3 |ref| + 6 sigma of the bf16 rounding of g (as for grad_hidden; the result itself is fp32)."""
    if not np.array_equal(M, ref["mask"]):
        return None                                 # a token inside the exemption band took the other mask value
    gw = res["grad_weight"].double().cpu().numpy()
    h = b["hidden"].double().cpu().numpy()
    sigma = np.sqrt((ref["grad_logits"] ** 2).T @ (h ** 2)) * SIGMA_BF16
    tol = 1e-3 * np.abs(ref["grad_weight"]) + 6.0 * sigma + 1e-30
    err = np.abs(gw - ref["grad_weight"])
    if not np.all(err <= tol):
        i, j = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"grad_weight [{i}, {j}]: gpu {gw[i, j]:.6e} ref {ref['grad_weight'][i, j]:.6e} tol {tol[i, j]:.3e}")
    return float(err.max())


def _run_and_compare(w, d, *, exact=True, backward=True, chunk_rows=0, shift=0.0, rows=None, rule=None):
    _say(f"[case] lmhead {w.name} T={w.T} V={w.V} d={d} K={w.K} variant={w.variant} exact={exact} chunk={chunk_rows} shift={shift} rule={rule}")
    b = W.make_lmhead_batch(w, d, DEV, exact=exact, shift_sampled=shift)
    rule = rule or {}
    b["rule"] = rule
    all_rows = rows is None
    rows = np.arange(b["T"]) if rows is None else rows
    gw = torch.full((b["V"], d + 4), 7.0, dtype=torch.float32, device=DEV)[:, :d] if (backward and all_rows) else None
    res = B.run_lmhead(b, backward=backward, chunk_rows=chunk_rows, diagnostics=True, grad_weight=gw, **rule)
    torch.cuda.synchronize()
    ref = _oracle(b, rows, want_grad=backward, **rule)
    cmp_batch = dict(b, logits=None)
    st = P.compare_rows(cmp_batch, res, rows, check_grad=False, ref=ref)
    if len(rows) == b["T"]:
        P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    if backward:
        st["median_rel_err_grad_hidden"] = _check_grad_hidden(b, res, rows, ref)
        if all_rows:
            st["max_abs_err_grad_weight"] = _check_grad_weight(b, res, ref, res["mask"].cpu().numpy())
    _say(f"       {st}")
    return b, res, st, ref


# --------------------------------------------------------------------------- the matrix product alone
@pytest.mark.parametrize("M,N,K,lda,ldb,ldc", [
    (256, 256, 64, 64, 64, 256), (1, 1, 64, 64, 64, 1), (300, 520, 128, 136, 128, 528), (1000, 777, 192, 192, 200, 777),
    (257, 4160, 4096, 4096, 4096, 4160), (513, 64, 8192, 8192, 8192, 64)])
def test_gemm_exact_inputs_bitwise(M, N, K, lda, ldb, ldc):
    _say(f"[case] gemm M={M} N={N} K={K}")
    g = torch.Generator(device=DEV); g.manual_seed(M * 7 + N)
    a = torch.zeros((M, lda), dtype=torch.bfloat16, device=DEV); b = torch.zeros((N, ldb), dtype=torch.bfloat16, device=DEV)
    a[:, :K] = (torch.randint(-8, 9, (M, K), generator=g, device=DEV).float() / 64).bfloat16()
    b[:, :K] = (torch.randint(-8, 9, (N, K), generator=g, device=DEV).float() / 8).bfloat16()
    a[:, K:] = 7.0; b[:, K:] = -5.0                                # pitch padding must never be read
    c = torch.full((M, ldc), 123.0, dtype=torch.bfloat16, device=DEV)
    B.gemm_nt(a[:, :K], b[:, :K], c[:, :N])
    torch.cuda.synchronize()
    ref = O.lmhead_logits(a[:, :K].float().cpu().numpy(), b[:, :K].float().cpu().numpy())
    np.testing.assert_array_equal(c[:, :N].double().cpu().numpy(), ref)
    assert (c[:, N:] == 123.0).all()


@pytest.mark.parametrize("M,N,K,lda,ldb,ldc", [
    (256, 256, 64, 64, 256, 256), (1, 1, 64, 64, 8, 1), (300, 520, 128, 136, 520, 528), (1000, 777, 192, 192, 784, 777),
    (257, 4160, 4096, 4096, 4160, 4160), (513, 64, 8192, 8192, 64, 64)])
def test_gemm_nn_exact_inputs_bitwise(M, N, K, lda, ldb, ldc):
    """C = A B with B stored with the contraction index as its row index (a weight [V, d] as it lies)."""
    _say(f"[case] gemm nn M={M} N={N} K={K}")
    g = torch.Generator(device=DEV); g.manual_seed(M * 5 + N)
    a = torch.full((M, lda), 7.0, dtype=torch.bfloat16, device=DEV); b = torch.full((K, ldb), -5.0, dtype=torch.bfloat16, device=DEV)
    a[:, :K] = (torch.randint(-8, 9, (M, K), generator=g, device=DEV).float() / 64).bfloat16()
    b[:, :N] = (torch.randint(-8, 9, (K, N), generator=g, device=DEV).float() / 8).bfloat16()
    c = torch.full((M, ldc), 123.0, dtype=torch.bfloat16, device=DEV)
    B.gemm_nn(a[:, :K], b[:, :N], c[:, :N])
    torch.cuda.synchronize()
    ref = O.bf16_round(a[:, :K].double().cpu().numpy() @ b[:, :N].double().cpu().numpy())
    np.testing.assert_array_equal(c[:, :N].double().cpu().numpy(), ref)
    assert (c[:, N:] == 123.0).all()


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (1000, 260, 192), (4160, 128, 320)])
def test_gemm_fp32_result_exact_inputs_bitwise_and_accumulation(M, N, K):
    _say(f"[case] gemm fp32 M={M} N={N} K={K}")
    g = torch.Generator(device=DEV); g.manual_seed(M + N)
    a = (torch.randint(-8, 9, (M, K), generator=g, device=DEV).float() / 64).bfloat16()
    b = (torch.randint(-8, 9, (N, K), generator=g, device=DEV).float() / 8).bfloat16()
    c = torch.full((M, N + 4), 3.0, dtype=torch.float32, device=DEV)
    B.gemm_nt_f32(a, b, c[:, :N])
    torch.cuda.synchronize()
    ref = a.double().cpu().numpy() @ b.double().cpu().numpy().T          # exact, and exactly representable in fp32
    np.testing.assert_array_equal(c[:, :N].double().cpu().numpy(), ref)
    B.gemm_nt_f32(a, b, c[:, :N], accumulate=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(c[:, :N].double().cpu().numpy(), 2 * ref)
    assert (c[:, N:] == 3.0).all()


@pytest.mark.parametrize("M,N,K,lda,ldb,ldc", [
    (256, 256, 64, 256, 256, 256), (8, 8, 1, 8, 8, 8), (300, 520, 100, 304, 520, 520), (1000, 776, 193, 1008, 784, 780),
    (4160, 128, 321, 4160, 128, 128), (130, 4100, 4096, 136, 4104, 4100), (151936, 64, 130, 151936, 64, 64),
    (777, 261, 129, 784, 264, 264)])
def test_gemm_tn_exact_inputs_bitwise_and_accumulation(M, N, K, lda, ldb, ldc):
    """C = A^T B with both operands stored with the contraction index as the row index (the form of
    the weight gradient), any K, ragged M and N, pitches of their own, then once more accumulating."""
    _say(f"[case] gemm tn M={M} N={N} K={K}")
    g = torch.Generator(device=DEV); g.manual_seed(M * 3 + N + K)
    a = torch.full((K, lda), 7.0, dtype=torch.bfloat16, device=DEV); b = torch.full((K, ldb), -5.0, dtype=torch.bfloat16, device=DEV)
    a[:, :M] = (torch.randint(-8, 9, (K, M), generator=g, device=DEV).float() / 64).bfloat16()
    b[:, :N] = (torch.randint(-8, 9, (K, N), generator=g, device=DEV).float() / 8).bfloat16()
    c = torch.full((M, ldc), 3.0, dtype=torch.float32, device=DEV)
    B.gemm_tn_f32(a[:, :M], b[:, :N], c[:, :N])
    torch.cuda.synchronize()
    ref = (a[:, :M].double().T @ b[:, :N].double()).cpu().numpy()       # exact, and exactly representable in fp32
    np.testing.assert_array_equal(c[:, :N].double().cpu().numpy(), ref)
    B.gemm_tn_f32(a[:, :M], b[:, :N], c[:, :N], accumulate=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(c[:, :N].double().cpu().numpy(), 2 * ref)
    assert (c[:, N:] == 3.0).all()


def test_gemm_tn_poisoned_neighbourhood_and_error_codes():
    """What lies next to the operands (pitch padding, rows past K in a larger buffer) holds NaN and
    infinities and must not reach any result; bad arguments are refused."""
    g = torch.Generator(device=DEV); g.manual_seed(11)
    K, M, N = 70, 264, 72
    big_a = torch.full((K + 64, M + 8), float("nan"), dtype=torch.bfloat16, device=DEV)
    big_b = torch.full((K + 64, N + 8), float("inf"), dtype=torch.bfloat16, device=DEV)
    big_a[:K, :M] = (torch.randint(-8, 9, (K, M), generator=g, device=DEV).float() / 8).bfloat16()
    big_b[:K, :N] = (torch.randint(-8, 9, (K, N), generator=g, device=DEV).float() / 8).bfloat16()
    c = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    B.gemm_tn_f32(big_a[:K, :M], big_b[:K, :N], c)
    torch.cuda.synchronize()
    ref = (big_a[:K, :M].double().T @ big_b[:K, :N].double()).cpu().numpy()
    np.testing.assert_array_equal(c.double().cpu().numpy(), ref)
    a, b = big_a[:K, :M], big_b[:K, :N]
    for bad in (lambda: B.gemm_tn_f32(a[:, 1:], b, c[1:]),                      # misaligned A
                lambda: B.gemm_tn_f32(a[:0], b[:0], c),                          # K = 0
                lambda: B.gemm_tn_f32(a, b, c.view(-1)[: M * N - M].view(M, N - 1)[:, :N - 1])):   # ldc not a multiple of 4
        with pytest.raises(B.DppoError):
            bad()
    torch.cuda.synchronize()


def test_gemm_ordinary_inputs_within_one_rounding():
    M, N, K = 384, 1000, 1024
    g = torch.Generator(device=DEV); g.manual_seed(3)
    a = torch.randn((M, K), generator=g, device=DEV).bfloat16(); b = (torch.randn((N, K), generator=g, device=DEV) / 8).bfloat16()
    c = B.gemm_nt(a, b)
    torch.cuda.synchronize()
    exact = a.double().cpu().numpy() @ b.double().cpu().numpy().T
    got = c.double().cpu().numpy()
    # fp32 accumulation error (<= K eps32 sum|a||b|) plus one rounding to 8 significant bits
    bound = 2.0 ** -8 * np.abs(exact) + K * 2.0 ** -24 * (np.abs(a.double().cpu().numpy()) @ np.abs(b.double().cpu().numpy()).T)
    assert np.all(np.abs(got - exact) <= bound)
    assert np.mean(got == O.bf16_round(exact)) > 0.99          # and almost always THE nearest bf16


def test_gemm_error_codes():
    a = torch.zeros((64, 128), dtype=torch.bfloat16, device=DEV); b = torch.zeros((64, 128), dtype=torch.bfloat16, device=DEV)
    c = torch.zeros((64, 64), dtype=torch.bfloat16, device=DEV)
    f = B.lib().dppo_gemm_nt
    assert f(a.data_ptr(), 128, b.data_ptr(), 128, c.data_ptr(), 64, 64, 64, 128, None) == 0
    assert f(a.data_ptr(), 128, b.data_ptr(), 128, c.data_ptr(), 64, 64, 64, 96, None) == 2       # K not a multiple of 64
    assert f(a.data_ptr(), 100, b.data_ptr(), 128, c.data_ptr(), 64, 64, 64, 128, None) == 2      # lda < K
    assert f(a.data_ptr(), 128, b.data_ptr(), 128, c.data_ptr(), 32, 64, 64, 128, None) == 2      # ldc < N
    assert f(a.data_ptr() + 2, 128, b.data_ptr(), 128, c.data_ptr(), 64, 64, 64, 128, None) == 3
    assert f(None, 128, b.data_ptr(), 128, c.data_ptr(), 64, 64, 64, 128, None) == 1
    assert f(None, 128, None, 128, None, 64, 0, 64, 128, None) == 0                               # empty
    torch.cuda.synchronize()


# --------------------------------------------------------------------------- the whole path, every row
@pytest.mark.parametrize("variant,K,delta", [(W.BINARY_TV, 0, 0.2), (W.BINARY_KL, 0, 0.05), (W.TOPK_TV, 20, 0.2), (W.TOPK_KL, 64, 0.05)])
@pytest.mark.parametrize("shift", [0.0, 2.0])
def test_small_all_rows_several_chunks(variant, K, delta, shift):
    # T = 300 in chunks of 128 (two full chunks and a ragged one), V = 4160 = 16 tiles + a quarter tile
    w = W.Workload("lm_small", 3, 100, 4160, variant, delta, K=K, logit_std=3.0, noise_std=1.0 if shift else 0.05, adv="normal", seed=71)
    b, res, st, ref = _run_and_compare(w, 128, chunk_rows=128, shift=shift)
    if shift:
        assert 0 < st["masked"] < b["T"]


@pytest.mark.parametrize("V,d,chunk", [(8192, 64, 0), (16384, 256, 1000), (64, 64, 7)])
def test_shapes_resident_loss_kernel_inside_and_tiny(V, d, chunk):
    w = W.Workload("lm_shape", 2, 150, V, W.TOPK_TV, 0.1, K=8, logit_std=3.0, noise_std=1.0, adv="pm1", seed=73)
    _run_and_compare(w, d, chunk_rows=chunk, shift=2.0)
    _run_and_compare(w, d, chunk_rows=chunk, shift=2.0, backward=False)


def test_ignored_rows_and_baseline_rule_run_to_run():
    w = W.Workload("lm_rule", 2, 130, 4096, W.BINARY_TV, 0.1, logit_std=3.0, noise_std=1.0, adv="normal", seed=79)
    b = W.make_lmhead_batch(w, 128, DEV, exact=True, shift_sampled=2.0)
    b["sampled_ids"][::9] = -1
    b["advantages"][4::11] = 0.0
    rule = dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28, ratio_cap=3.0)
    b["rule"] = rule
    rows = np.arange(b["T"])
    ref = _oracle(b, rows, **rule)
    outs = []
    for _ in range(2):                          # twice: the path is bitwise reproducible run to run
        res = B.run_lmhead(b, chunk_rows=64, diagnostics=True, **rule)
        torch.cuda.synchronize()
        st = P.compare_rows(dict(b, logits=None), res, rows, check_grad=False, ref=ref)
        _check_grad_hidden(b, res, rows, ref)
        P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
        outs.append(res)
        _say(f"       {st}")
    assert torch.equal(outs[0]["grad_hidden"], outs[1]["grad_hidden"])
    assert (outs[0]["grad_hidden"][::9] == 0).all()
    assert st["masked"] > 0


def test_ordinary_inputs_rows_clear_of_rounding_boundaries():
    w = W.Workload("lm_real", 2, 128, 4096, W.TOPK_TV, 0.1, K=20, logit_std=3.0, noise_std=0.5, adv="pm1", seed=83)
    d = 512
    b = W.make_lmhead_batch(w, d, DEV, exact=False, shift_sampled=1.0)
    rows = np.arange(b["T"])
    res = B.run_lmhead(b, chunk_rows=100, diagnostics=True)
    torch.cuda.synchronize()
    ref = _oracle(b, rows)
    # oracle side only: which logits lie within fp32-accumulation reach of a bf16 rounding boundary
    h, Wm = b["hidden"].double().cpu().numpy(), b["weight"].double().cpu().numpy()
    exact = h @ Wm.T
    _, e = np.frexp(exact)
    half_ulp = np.ldexp(1.0, e - 9)
    margin = half_ulp - np.abs(exact - ref["logits"])
    # d/8 fp32 roundings along an accumulator, each of at most 2^-24 of a partial sum, whose size is that
    # of a random walk over the products: |final| + 4 standard deviations
    reach = (d / 8) * 2.0 ** -24 * (np.abs(exact) + 4.0 * np.sqrt((h ** 2) @ (Wm ** 2).T))
    near = margin <= reach
    pi = np.exp(ref["logits"] - ref["logits"].max(1, keepdims=True)); pi /= pi.sum(1, keepdims=True)
    matters = pi > 1e-3
    a = b["sampled_ids"].cpu().numpy()
    matters[np.arange(len(a)), a] = True
    np.put_along_axis(matters, b["mu_topk_ids"].cpu().numpy().astype(np.int64), True, axis=1)
    clear = ~(near & matters).any(1)
    assert clear.sum() > 0.4 * b["T"]
    # rows clear of boundaries: a flipped logit of a token below 1e-3 moves the log-normaliser by at most
    # pi_j * ulp(z_j) < 1e-3 * 0.03, and every probability with it: an absolute 2e-5 on D covers those (measured 6e-6)
    D = res["divergence"].double().cpu().numpy()
    M = res["mask"].cpu().numpy()
    errD = np.abs(D - ref["divergence"])[clear]
    assert np.all(errD <= 1e-4 * np.abs(ref["divergence"][clear]) + 2e-5), errD.max()
    exempt = (np.abs(ref["divergence"] - b["delta"]) < 2e-4) | (np.abs(ref["logp"] - b["mu_logp"].double().cpu().numpy()) < 2e-4)
    assert np.all((M == ref["mask"])[clear & ~exempt])
    same = clear & (M == ref["mask"])
    lt = res["loss_tok"].double().cpu().numpy()
    assert np.all(np.abs(lt - ref["loss_tok"])[same] <= 1e-3 * np.abs(ref["loss_tok"][same]) + 1e-4)
    _check_grad_hidden(b, res, rows, ref, skip=~same)
    _say(f"       clear rows {clear.sum()} of {b['T']}, max |dD| on them {errD.max():.2e}, masked {(M == 0).sum()}")


def test_weight_gradient_accumulates_onto_the_callers_buffer():
    w = W.Workload("lm_acc", 2, 100, 4096, W.BINARY_KL, 0.05, logit_std=3.0, noise_std=1.0, adv="normal", seed=101)
    b = W.make_lmhead_batch(w, 128, DEV, exact=True, shift_sampled=2.0)
    g1 = torch.empty((b["V"], 128), dtype=torch.float32, device=DEV)
    B.run_lmhead(b, chunk_rows=64, grad_weight=g1)
    g2 = torch.full((b["V"], 128), 0.5, dtype=torch.float32, device=DEV)
    B.run_lmhead(b, chunk_rows=64, grad_weight=g2, accumulate=True)
    torch.cuda.synchronize()
    assert (g2 - (g1 + 0.5)).abs().max().item() <= 5e-7          # four chunk sums, each rounded at the size of 0.5
    g3 = torch.empty((b["V"], 128), dtype=torch.float32, device=DEV)
    B.run_lmhead(b, chunk_rows=200, grad_weight=g3)                    # one chunk: same sum, another order
    torch.cuda.synchronize()
    assert (g3 - g1).abs().max().item() <= 1e-6 * g1.abs().max().item() + 1e-12


def test_hidden_state_path_can_be_captured_in_a_hip_graph_and_replayed():
    """The chunk loop (products, loss in place, accumulation) allocates nothing and never
    synchronises: with the workspace and every output preallocated one call is a capturable chain of
    kernels.  Replayed three times with eager work in between, every replay bit for bit the eager result."""
    w = W.Workload("lm_graph", 3, 100, 4096, W.BINARY_TV, 0.1, logit_std=3.0, noise_std=1.0, adv="normal", seed=103)
    b = W.make_lmhead_batch(w, 128, DEV, exact=True, shift_sampled=2.0)
    T, V, d = b["T"], b["V"], 128
    gw_e = torch.empty((V, d), dtype=torch.float32, device=DEV)
    e = B.run_lmhead(b, chunk_rows=128, diagnostics=True, grad_weight=gw_e)
    torch.cuda.synchronize()
    eager = {k: e[k].clone() for k in ("loss", "loss_tok", "divergence", "mask", "diagnostics", "grad_hidden")}
    out = B.alloc_outputs(T, DEV, want_diagnostics=True)
    gh = torch.empty((T, d), dtype=torch.bfloat16, device=DEV)
    gw = torch.empty((V, d), dtype=torch.float32, device=DEV)
    ws = torch.empty(B.lmhead_workspace_bytes(T, V, 128), dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            B.run_lmhead(b, chunk_rows=128, out=out, grad_hidden=gh, grad_weight=gw, workspace=ws)
    scratch = torch.zeros(1 << 20, device=DEV)
    for rep in range(3):
        for k in ("loss", "loss_tok", "divergence", "diagnostics"):
            out[k].fill_(float("nan"))
        out["mask"].fill_(7)
        gh.fill_(float("nan")); gw.fill_(float("nan")); ws.fill_(0xff)
        scratch.add_(1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ("loss", "loss_tok", "divergence", "mask", "diagnostics"):
            assert torch.equal(eager[k], out[k]), (rep, k)
        assert torch.equal(eager["grad_hidden"], gh) and torch.equal(gw_e, gw), rep
    _say("       hidden-state path captured and replayed 3 times, bitwise equal to eager")


def test_error_codes():
    w = W.Workload("lm_err", 1, 16, 256, W.BINARY_TV, 0.2, logit_std=3.0, adv="pm1", seed=89)
    b = W.make_lmhead_batch(w, 64, DEV, exact=True)
    res = B.run_lmhead(b)
    torch.cuda.synchronize()
    a = res["args"]

    def status(**kw):
        saved = {k: getattr(a, k) for k in kw}
        for k, v in kw.items():
            setattr(a, k, v)
        st = B.lib().dppo_lmhead_loss_fwd_bwd(C.byref(a), None)
        for k, v in saved.items():
            setattr(a, k, v)
        return st

    assert status() == 0
    assert status(d=96) == 2
    assert status(ld_hidden=32) == 2
    assert status(hidden=None) == 1
    assert status(grad_hidden=None) == 1
    assert status(workspace_bytes=1024) == 6
    assert status(workspace=a.workspace + 8) == 3
    assert status(hidden=a.hidden + 2) == 3
    a.loss.variant = W.FULL_TV
    assert status() == 4
    a.loss.variant = W.BINARY_TV
    a.loss.V = 200
    assert status() == 2                      # V not a multiple of 64
    a.loss.V = 256
    assert status() == 0
    torch.cuda.synchronize()


def test_headline_vocabulary_sampled_rows():
    """V = 151936, d = 4096, T = 4608 in chunks of 2048 (two full chunks and a ragged one): sampled
    rows against the oracle on inputs whose logits are exact in fp32."""
    w = W.Workload("lm_qwen3", 9, 512, 151936, W.TOPK_TV, 0.2, K=20, logit_std=3.0, noise_std=0.3, adv="pm1", seed=97)
    _say(f"[case] lmhead {w.name} T={w.T} V={w.V} d=4096 exact inputs, chunks of 2048")
    b = W.make_lmhead_batch(w, 4096, DEV, exact=True, shift_sampled=1.0)
    gw = torch.empty((w.V, 4096), dtype=torch.float32, device=DEV)
    res = B.run_lmhead(b, chunk_rows=2048, diagnostics=True, grad_weight=gw)
    torch.cuda.synchronize()
    # every row of d loss / d z sums to zero, so the columns of the weight gradient do (up to the bf16 rounding of g)
    col_sum, col_abs = gw.double().sum(0), gw.double().abs().sum(0)
    assert torch.isfinite(gw).all() and (col_sum.abs() <= 1e-2 * col_abs + 1e-30).all() and col_abs.min().item() > 0
    del gw
    mask = res["mask"].cpu().numpy()
    rng = np.random.default_rng(11)
    pick = {0, w.T - 1, 2047, 2048, 4095, 4096} | set(rng.integers(0, w.T, 8).tolist()) | set(np.nonzero(mask == 0)[0][:4].tolist())
    rows = np.array(sorted(pick))
    ref = _oracle(b, rows)
    st = P.compare_rows(dict(b, logits=None), res, rows, check_grad=False, ref=ref)
    st["median_rel_err_grad_hidden"] = _check_grad_hidden(b, res, rows, ref)
    P.check_loss_scalar(b, res)
    assert 0 < (mask == 0).sum() < w.T and st["masked"] > 0
    _say(f"       masked={(mask == 0).sum()} {st}")


# --------------------------------------------------------------------------- forward only: no logit is ever written
@pytest.mark.parametrize("variant,K,delta", [(W.BINARY_TV, 0, 0.2), (W.BINARY_KL, 0, 0.05), (W.TOPK_TV, 20, 0.2), (W.TOPK_KL, 150, 0.05)])
@pytest.mark.parametrize("shift", [0.0, 2.0])
def test_forward_only_from_tile_statistics(variant, K, delta, shift):
    """dppo_lmhead_loss_fwd: the product kernel leaves per-tile softmax statistics and the gathered
    logits instead of logits.  T = 300 in chunks of 128, V = 4160 = 16 tiles + a quarter tile, every
    row against the oracle at the bar of the logits path, and against the route through a chunk of
    logits (same bf16 logits, another summation order)."""
    w = W.Workload("lm_fused", 3, 100, 4160, variant, delta, K=K, logit_std=3.0, noise_std=1.0 if shift else 0.05, adv="normal", seed=107)
    b, res, st, ref = _run_and_compare(w, 128, chunk_rows=128, shift=shift, backward=False)
    assert B.last_path() == "lmhead_fused"
    if shift:
        assert 0 < st["masked"] < b["T"]
    ws = res["workspace_buf"].numel()
    assert ws == B.lmhead_fwd_workspace_bytes(b["T"], b["V"], K, 128) and ws < B.lmhead_workspace_bytes(b["T"], b["V"], 128)
    chunked = B.run_lmhead(b, backward=False, chunk_rows=128, diagnostics=True, flags=B.FLAG_FORCE_STREAMING)
    torch.cuda.synchronize()
    assert B.last_path() == "lmhead"
    assert torch.equal(res["mask"], chunked["mask"])
    torch.testing.assert_close(res["divergence"], chunked["divergence"], rtol=1e-4, atol=2e-7)
    torch.testing.assert_close(res["loss"], chunked["loss"], rtol=1e-5, atol=1e-9)
    again = B.run_lmhead(b, backward=False, chunk_rows=128, diagnostics=True)      # bitwise reproducible
    torch.cuda.synchronize()
    for k in ("loss", "loss_tok", "divergence", "mask", "diagnostics"):
        assert torch.equal(res[k], again[k]), k


def test_forward_only_ignored_rows_padding_ids_and_ids_in_the_ragged_last_tile():
    w = W.Workload("lm_fused_edge", 2, 140, 4160, W.TOPK_TV, 0.1, K=12, logit_std=3.0, noise_std=1.0, adv="normal", seed=109)
    b = W.make_lmhead_batch(w, 64, DEV, exact=True, shift_sampled=2.0)
    b["sampled_ids"][::9] = -1
    b["sampled_ids"][3::13] = b["V"] + 5
    b["sampled_ids"][5::17] = b["V"] - 1                       # last column, in the quarter tile
    b["mu_logp"][5::17] = -3.0
    b["mu_topk_ids"][:, 4] = -1                                # padding entries
    b["mu_topk_ids"][1::2, 7] = b["V"]
    b["mu_topk_ids"][::3, 2] = b["V"] - 2
    b["advantages"][2::6] = 0.0
    rows = np.arange(b["T"])
    ref = _oracle(b, rows, want_grad=False)
    res = B.run_lmhead(b, backward=False, chunk_rows=100, diagnostics=True)
    torch.cuda.synchronize()
    assert B.last_path() == "lmhead_fused"
    st = P.compare_rows(dict(b, logits=None), res, rows, check_grad=False, ref=ref)
    P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
    ign = (b["sampled_ids"] < 0) | (b["sampled_ids"] >= b["V"])
    assert torch.all(res["mask"][ign] == 0) and torch.all(res["divergence"][ign] == 0) and torch.all(res["loss_tok"][ign] == 0)
    _say(f"       {st}")


def test_forward_only_headline_vocabulary_sampled_rows():
    """V = 151936 (593 tiles and a half), d = 4096, T = 2560 in chunks of 1024: sampled rows against
    the oracle on inputs whose logits are exact in fp32, Top-K TV and Binary KL."""
    for variant, K, delta in ((W.TOPK_TV, 20, 0.2), (W.BINARY_KL, 0, 0.05)):
        w = W.Workload("lm_qwen3_fwd", 5, 512, 151936, variant, delta, K=K, logit_std=3.0, noise_std=0.3, adv="pm1", seed=113)
        _say(f"[case] lmhead forward only {w.name} T={w.T} V={w.V} d=4096 variant={variant}")
        b = W.make_lmhead_batch(w, 4096, DEV, exact=True, shift_sampled=1.0)
        res = B.run_lmhead(b, backward=False, chunk_rows=1024, diagnostics=True)
        torch.cuda.synchronize()
        assert B.last_path() == "lmhead_fused"
        mask = res["mask"].cpu().numpy()
        rng = np.random.default_rng(13)
        pick = {0, w.T - 1, 1023, 1024, 2047, 2048} | set(rng.integers(0, w.T, 6).tolist()) | set(np.nonzero(mask == 0)[0][:4].tolist())
        rows = np.array(sorted(pick))
        ref = _oracle(b, rows, want_grad=False)
        st = P.compare_rows(dict(b, logits=None), res, rows, check_grad=False, ref=ref)
        P.check_loss_scalar(b, res)
        assert 0 < (mask == 0).sum() < w.T and st["masked"] > 0
        _say(f"       masked={(mask == 0).sum()} {st}")


def test_empty_batch_and_single_token():
    w = W.Workload("lm_one", 1, 1, 256, W.TOPK_KL, 0.05, K=4, logit_std=3.0, noise_std=0.5, adv="pm1", seed=103)
    _run_and_compare(w, 64, shift=1.0)
    b = W.make_lmhead_batch(w, 64, DEV, exact=True)
    empty = dict(b, hidden=b["hidden"][:0], sampled_ids=b["sampled_ids"][:0], mu_logp=b["mu_logp"][:0],
                 advantages=b["advantages"][:0], mu_topk_ids=b["mu_topk_ids"][:0], mu_topk_logp=b["mu_topk_logp"][:0], T=0)
    gw = torch.full((b["V"], 64), 2.0, dtype=torch.float32, device=DEV)
    res = B.run_lmhead(empty, grad_weight=gw)
    torch.cuda.synchronize()
    assert res["loss"].item() == 0.0 and (gw == 2.0).all()          # nothing to add, nothing touched
    res = B.run_lmhead(empty, backward=False)
    torch.cuda.synchronize()
    assert res["loss"].item() == 0.0
    _run_and_compare(w, 64, shift=1.0, backward=False)


def test_mask_anchored_to_a_recomputed_policy_on_the_hidden_state_path():
    """anchor_logp on both forms of the hidden-state path (through a chunk of logits with the
    gradients, and forward only from tile statistics): MiniRL-TIS (App. C.1)."""
    w = W.Workload("lm_anchor", 2, 150, 4160, W.BINARY_KL, 0.05, logit_std=3.0, noise_std=1.0, adv="normal", seed=99)
    b = W.make_lmhead_batch(w, 128, DEV, exact=True, shift_sampled=2.0)
    g = torch.Generator(device="cpu").manual_seed(7)
    b["anchor_logp"] = torch.minimum(b["mu_logp"] + torch.randn(b["T"], generator=g).to(DEV) * 0.5, torch.zeros_like(b["mu_logp"]))
    rule = dict(mask_rule=B.MASK_RATIO_CLIP, eps_low=0.2, eps_high=0.28, ratio_cap=3.0)
    b["rule"] = rule
    rows = np.arange(b["T"])
    ref = _oracle(b, rows, **rule)
    for backward in (True, False):
        res = B.run_lmhead(b, backward=backward, chunk_rows=64, diagnostics=True, **rule)
        torch.cuda.synchronize()
        st = P.compare_rows(dict(b, logits=None), res, rows, check_grad=False, ref=ref)
        P.check_loss_scalar(b, res, float(ref["loss_tok"].sum()))
        if backward:
            _check_grad_hidden(b, res, rows, ref)
        assert 0 < st["masked"] < b["T"]
    plain = dict(b, anchor_logp=None)
    res0 = B.run_lmhead(plain, backward=False, chunk_rows=64, **rule)
    torch.cuda.synchronize()
    assert (res0["mask"] != res["mask"]).any()
