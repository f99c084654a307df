"""Thin ctypes binding of the C ABI in include/dppo.h (and the measurement utilities of
include/dppo_probe.h).

Argument marshalling only: every step of the loss runs in the HIP kernels of libdppo.so.
PyTorch is used for device memory and the stream handle.  There is no CPU fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

BINARY_TV, BINARY_KL, TOPK_TV, TOPK_KL, FULL_TV, FULL_KL = 0, 1, 2, 3, 4, 5
MASK_DIVERGENCE, MASK_RATIO_CLIP, MASK_NONE = 0, 1, 2
NDIAG = 8
DIAG_RATIO, DIAG_LOGP, DIAG_ABS_DIFF, DIAG_ENTROPY, DIAG_MASS_MU, DIAG_MASS_PI = 0, 1, 2, 3, 4, 5
FLAG_FORCE_STREAMING = 1
FLAG_STATIC_ROWS = 2
RELAX_HIGH, RELAX_LOW = 1, 2
WORKSPACE_BYTES = 65536       # the smallest workspace any call accepts; workspace_bytes(T, V, K) is what a call wants

# DPPO_LIB overrides the library path (e.g. a build with other compile-time settings).
_LIB_PATH = os.environ.get("DPPO_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdppo.so")
_lib = None


class DppoArgs(C.Structure):
    """Mirror of dppo_args_t."""
    _fields_ = [
        ("logits", C.c_void_p), ("T", C.c_int64), ("V", C.c_int64), ("ld", C.c_int64),
        ("sampled_ids", C.c_void_p), ("mu_logp", C.c_void_p),
        ("mu_topk_ids", C.c_void_p), ("mu_topk_logp", C.c_void_p),
        ("K", C.c_int32), ("variant", C.c_int32),
        ("advantages", C.c_void_p), ("delta", C.c_float), ("loss_scale", C.c_float),
        ("mask_rule", C.c_int32), ("eps_low", C.c_float), ("eps_high", C.c_float), ("ratio_cap", C.c_float),
        ("relax_alpha", C.c_float), ("relax_sides", C.c_uint32),
        ("mu_logits", C.c_void_p), ("mu_ld", C.c_int64), ("anchor_logp", C.c_void_p),
        ("loss", C.c_void_p), ("loss_tok", C.c_void_p), ("divergence", C.c_void_p),
        ("mask", C.c_void_p), ("grad_logits", C.c_void_p), ("diagnostics", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("flags", C.c_uint32),
    ]


class DppoLmheadArgs(C.Structure):
    """Mirror of dppo_lmhead_args_t."""
    _fields_ = [
        ("loss", DppoArgs),
        ("hidden", C.c_void_p), ("ld_hidden", C.c_int64), ("d", C.c_int64),
        ("weight", C.c_void_p), ("ld_weight", C.c_int64),
        ("chunk_rows", C.c_int64),
        ("grad_hidden", C.c_void_p), ("ld_grad_hidden", C.c_int64),
        ("grad_weight", C.c_void_p), ("ld_grad_weight", C.c_int64), ("grad_weight_accumulate", C.c_int32),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class DppoError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"dppo status {status}: {lib().dppo_status_str(status).decode()}")


def lib() -> C.CDLL:
    """Open libdppo.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2602_04879_amd.build` "
                              "(there is no fallback implementation)")
        l = C.CDLL(_LIB_PATH)
        l.dppo_workspace_bytes.restype = C.c_size_t
        l.dppo_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32]
        l.dppo_static_init.restype = C.c_int
        l.dppo_static_init.argtypes = []
        for f in (l.dppo_loss_fwd, l.dppo_loss_fwd_bwd, l.dppo_loss_fwd_bwd_static):
            f.restype = C.c_int
            f.argtypes = [C.POINTER(DppoArgs), C.c_void_p]
        l.dppo_status_str.restype = C.c_char_p
        l.dppo_status_str.argtypes = [C.c_int]
        l.dppo_version.restype = C.c_int
        l.dppo_last_path.restype = C.c_char_p
        l.dppo_args_size.restype = C.c_size_t
        l.dppo_probe_copy.restype = C.c_int
        l.dppo_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.dppo_probe_copy_rows.restype = C.c_int
        l.dppo_probe_copy_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_size_t, C.c_size_t, C.c_void_p]
        l.dppo_probe_copy_resident.restype = C.c_int
        l.dppo_probe_copy_resident.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_size_t, C.c_size_t, C.c_void_p]
        l.dppo_probe_fill.restype = C.c_int
        l.dppo_probe_fill.argtypes = [C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
        l.dppo_probe_read.restype = C.c_int
        l.dppo_probe_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        l.dppo_probe_mfma.restype = C.c_int
        l.dppo_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.c_void_p]
        for f in (l.dppo_gemm_nt, l.dppo_gemm_nn):
            f.restype = C.c_int
            f.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                          C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
        l.dppo_lmhead_workspace_bytes.restype = C.c_size_t
        l.dppo_lmhead_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int64]
        for f in (l.dppo_gemm_nt_f32, l.dppo_gemm_tn_f32):
            f.restype = C.c_int
            f.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                          C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_void_p]
        for f in (l.dppo_lmhead_loss_fwd, l.dppo_lmhead_loss_fwd_bwd):
            f.restype = C.c_int
            f.argtypes = [C.POINTER(DppoLmheadArgs), C.c_void_p]
        l.dppo_lmhead_fwd_workspace_bytes.restype = C.c_size_t
        l.dppo_lmhead_fwd_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int64]
        l.dppo_lmhead_args_size.restype = C.c_size_t
        if l.dppo_lmhead_args_size() != C.sizeof(DppoLmheadArgs):
            raise ImportError("dppo_lmhead_args_t layout differs between libdppo.so and this binding")
        if l.dppo_args_size() != C.sizeof(DppoArgs):
            raise ImportError("dppo_args_t layout differs between libdppo.so and this binding")
        _lib = l
    return _lib


def _ptr(t):
    return None if t is None else t.data_ptr()


def workspace_bytes(T: int, V: int, K: int) -> int:
    return lib().dppo_workspace_bytes(T, V, K)


def make_args(logits, sampled_ids, mu_logp, advantages, delta, variant, loss_scale, out,
              mu_topk_ids=None, mu_topk_logp=None, V=None, flags=0, grad_logits=None,
              mask_rule=MASK_DIVERGENCE, eps_low=0.2, eps_high=0.2, ratio_cap=0.0, mu_logits=None,
              anchor_logp=None, relax_alpha=0.0, relax_sides=0) -> DppoArgs:
    """Fill a dppo_args_t from torch tensors.  `out` is a dict with loss [1] f32, divergence [T]
    f32, mask [T] u8, workspace (u8), optional loss_tok [T] f32."""
    T, ld = logits.shape[0], (logits.stride(0) if logits.shape[0] > 1 else logits.shape[1])
    a = DppoArgs()
    a.logits, a.T, a.V, a.ld = _ptr(logits), T, (logits.shape[1] if V is None else V), ld
    a.sampled_ids, a.mu_logp = _ptr(sampled_ids), _ptr(mu_logp)
    a.mu_topk_ids, a.mu_topk_logp = _ptr(mu_topk_ids), _ptr(mu_topk_logp)
    a.K = 0 if mu_topk_ids is None else mu_topk_ids.shape[1]
    a.variant = variant
    a.advantages, a.delta, a.loss_scale = _ptr(advantages), delta, loss_scale
    a.mask_rule, a.eps_low, a.eps_high = mask_rule, eps_low, eps_high
    a.ratio_cap = 0.0 if ratio_cap is None else ratio_cap
    a.mu_logits = _ptr(mu_logits)
    a.anchor_logp = _ptr(anchor_logp)
    a.relax_alpha, a.relax_sides = relax_alpha, relax_sides
    a.mu_ld = 0 if mu_logits is None else (mu_logits.stride(0) if mu_logits.shape[0] > 1 else mu_logits.shape[1])
    a.loss, a.loss_tok = _ptr(out["loss"]), _ptr(out.get("loss_tok"))
    a.divergence, a.mask = _ptr(out["divergence"]), _ptr(out["mask"])
    a.grad_logits = _ptr(grad_logits)
    a.diagnostics = _ptr(out.get("diagnostics"))
    ws = out.get("workspace")
    a.workspace, a.workspace_bytes = _ptr(ws), (0 if ws is None else ws.numel())
    a.flags = flags
    return a


def alloc_outputs(T: int, device, want_loss_tok: bool = True, want_diagnostics: bool = False) -> dict:
    return {
        "diagnostics": torch.empty((T, NDIAG), dtype=torch.float32, device=device) if want_diagnostics else None,
        "loss": torch.empty(1, dtype=torch.float32, device=device),
        "loss_tok": torch.empty(T, dtype=torch.float32, device=device) if want_loss_tok else None,
        "divergence": torch.empty(T, dtype=torch.float32, device=device),
        "mask": torch.empty(T, dtype=torch.uint8, device=device),
        "workspace": torch.empty(WORKSPACE_BYTES + 8 * T, dtype=torch.uint8, device=device),
    }


def _stream_handle(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def dppo_loss_fwd(args: DppoArgs, stream=None) -> None:
    """dppo_loss_fwd of include/dppo.h on `stream` (default: torch's current stream)."""
    st = lib().dppo_loss_fwd(C.byref(args), C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def dppo_loss_fwd_bwd(args: DppoArgs, stream=None) -> None:
    """dppo_loss_fwd_bwd of include/dppo.h on `stream` (default: torch's current stream)."""
    st = lib().dppo_loss_fwd_bwd(C.byref(args), C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def dppo_loss_fwd_bwd_static(args: DppoArgs, stream=None) -> None:
    """dppo_loss_fwd_bwd_static of include/dppo.h: no workspace, nothing allocated."""
    st = lib().dppo_loss_fwd_bwd_static(C.byref(args), C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def probe_copy(dst, src, stream=None) -> None:
    """dppo_probe_copy: plain 16-byte-vector device copy of src into dst (same byte size)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    st = lib().dppo_probe_copy(dst.data_ptr(), src.data_ptr(), n, C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def probe_copy_rows(dst, src, stream=None) -> None:
    """dppo_probe_copy_rows: copy a 2-D tensor row by row, one workgroup per row."""
    assert dst.shape == src.shape and dst.stride() == src.stride() and src.stride(1) == 1
    es = src.element_size()
    st = lib().dppo_probe_copy_rows(dst.data_ptr(), src.data_ptr(), src.shape[0], src.shape[1] * es, src.stride(0) * es,
                                    C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def probe_copy_resident(dst, src, stream=None) -> None:
    """dppo_probe_copy_resident: copy a 2-D tensor row by row with the register-resident loss
    kernel's memory pattern (row held in registers, one run of stores, one run of loads)."""
    assert dst.shape == src.shape and dst.stride() == src.stride() and src.stride(1) == 1
    es = src.element_size()
    st = lib().dppo_probe_copy_resident(dst.data_ptr(), src.data_ptr(), src.shape[0], src.shape[1] * es, src.stride(0) * es,
                                        C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def probe_fill(dst, value: int = 0, stream=None) -> None:
    """dppo_probe_fill: write-only pass over dst."""
    st = lib().dppo_probe_fill(dst.data_ptr(), dst.numel() * dst.element_size(), value, C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def probe_mfma(shape: int, iters: int, out, stream=None) -> float:
    """dppo_probe_mfma: a loop of bf16 matrix-core products on every compute unit; returns the
    floating-point operations of the launch (out: device float tensor, 256 per compute unit)."""
    flop = C.c_double(0.0)
    st = lib().dppo_probe_mfma(shape, iters, out.data_ptr(), out.numel() * out.element_size(), C.byref(flop),
                               C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)
    return flop.value


def probe_read(src, sink, stream=None) -> None:
    """dppo_probe_read: read-only pass over src."""
    st = lib().dppo_probe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                               C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)


def gemm_nt(a, b, c=None, stream=None):
    """dppo_gemm_nt: c[M, N] = a[M, K] @ b[N, K]^T for bf16 tensors with unit inner stride."""
    M, K = a.shape
    N = b.shape[0]
    assert b.shape[1] == K and a.stride(1) == 1 and b.stride(1) == 1
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    st = lib().dppo_gemm_nt(a.data_ptr(), a.stride(0), b.data_ptr(), b.stride(0), c.data_ptr(), c.stride(0),
                            M, N, K, C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)
    return c


def gemm_nn(a, b, c=None, stream=None):
    """dppo_gemm_nn: c[M, N] = a[M, K] @ b[K, N] for bf16 tensors with unit inner stride."""
    M, K = a.shape
    N = b.shape[1]
    assert b.shape[0] == K and a.stride(1) == 1 and b.stride(1) == 1
    if c is None:
        c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    st = lib().dppo_gemm_nn(a.data_ptr(), a.stride(0), b.data_ptr(), b.stride(0), c.data_ptr(), c.stride(0),
                            M, N, K, C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)
    return c


def gemm_nt_f32(a, b, c, accumulate: bool = False, stream=None):
    """dppo_gemm_nt_f32: c[M, N] (+)= a[M, K] @ b[N, K]^T, c fp32."""
    M, K = a.shape
    N = b.shape[0]
    st = lib().dppo_gemm_nt_f32(a.data_ptr(), a.stride(0), b.data_ptr(), b.stride(0), c.data_ptr(), c.stride(0),
                                M, N, K, int(accumulate), C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)
    return c


def gemm_tn_f32(a, b, c, accumulate: bool = False, stream=None):
    """dppo_gemm_tn_f32: c[M, N] (+)= a[K, M]^T @ b[K, N], c fp32."""
    K, M = a.shape
    N = b.shape[1]
    st = lib().dppo_gemm_tn_f32(a.data_ptr(), a.stride(0), b.data_ptr(), b.stride(0), c.data_ptr(), c.stride(0),
                                M, N, K, int(accumulate), C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)
    return c


def last_path() -> str:
    return lib().dppo_last_path().decode()


def run_batch(batch: dict, backward: bool = True, in_place: bool = False, flags: int = 0, out=None,
              grad=None, stream=None, rows=None, diagnostics: bool = False, **rule) -> dict:
    """Convenience for tests and benchmarks: run one workload batch (see workloads.make_batch),
    optionally restricted to rows [r0, r1).  Returns the output tensors (device)."""
    r0, r1 = (0, batch["T"]) if rows is None else rows
    sl = slice(r0, r1)
    logits = batch["logits"][sl]
    T = r1 - r0
    if out is None:
        out = alloc_outputs(T, logits.device, want_diagnostics=diagnostics)
    if backward and grad is None:
        grad = logits if in_place else torch.empty_like(logits)
    tk_i = batch["mu_topk_ids"][sl] if batch["mu_topk_ids"] is not None else None
    tk_l = batch["mu_topk_logp"][sl] if batch["mu_topk_logp"] is not None else None
    args = make_args(logits, batch["sampled_ids"][sl], batch["mu_logp"][sl], batch["advantages"][sl],
                     batch["delta"], batch["variant"], batch["loss_scale"], out, tk_i, tk_l,
                     V=batch["V"], flags=flags, grad_logits=grad if backward else None,
                     mu_logits=batch["mu_logits"][sl] if batch.get("mu_logits") is not None else None,
                     anchor_logp=batch["anchor_logp"][sl] if batch.get("anchor_logp") is not None else None, **rule)
    args.ld = batch["ld"]
    if batch.get("mu_logits") is not None:
        args.mu_ld = batch["mu_logits"].stride(0)
    (dppo_loss_fwd_bwd if backward else dppo_loss_fwd)(args, stream)
    res = dict(out)
    res["grad_logits"] = grad if backward else None
    res["args"] = args
    return res


def lmhead_workspace_bytes(T: int, V: int, chunk_rows: int = 0) -> int:
    return lib().dppo_lmhead_workspace_bytes(T, V, chunk_rows)


def lmhead_fwd_workspace_bytes(T: int, V: int, K: int, chunk_rows: int = 0) -> int:
    return lib().dppo_lmhead_fwd_workspace_bytes(T, V, K, chunk_rows)


def run_lmhead(batch: dict, backward: bool = True, chunk_rows: int = 0, out=None, grad_hidden=None,
               workspace=None, stream=None, diagnostics: bool = False, grad_weight=None, accumulate: bool = False,
               flags: int = 0, **rule) -> dict:
    """Run one hidden-state batch (workloads.make_lmhead_batch) through dppo_lmhead_loss_fwd[_bwd].
    Returns the output tensors (device), grad_hidden among them."""
    h, w = batch["hidden"], batch["weight"]
    T, d, V = h.shape[0], batch["d"], batch["V"]
    dev = h.device
    if out is None:
        out = alloc_outputs(T, dev, want_diagnostics=diagnostics)
    if backward and grad_hidden is None:
        grad_hidden = torch.empty((T, d), dtype=torch.bfloat16, device=dev)
    if workspace is None:
        fused = not backward and not (flags & FLAG_FORCE_STREAMING)
        K = batch["mu_topk_ids"].shape[1] if batch["mu_topk_ids"] is not None else 0
        workspace = torch.empty(lmhead_fwd_workspace_bytes(T, V, K, chunk_rows) if fused else lmhead_workspace_bytes(T, V, chunk_rows),
                                dtype=torch.uint8, device=dev)
    a = DppoLmheadArgs()
    a.loss = make_args(torch.empty((0, V), dtype=torch.bfloat16, device=dev), batch["sampled_ids"], batch["mu_logp"],
                       batch["advantages"], batch["delta"], batch["variant"], batch["loss_scale"], out,
                       batch["mu_topk_ids"], batch["mu_topk_logp"], V=V, flags=flags, anchor_logp=batch.get("anchor_logp"), **rule)
    a.loss.T, a.loss.logits = T, None
    a.hidden, a.ld_hidden, a.d = h.data_ptr(), h.stride(0), d
    a.weight, a.ld_weight = w.data_ptr(), w.stride(0)
    a.chunk_rows = chunk_rows
    a.grad_hidden, a.ld_grad_hidden = _ptr(grad_hidden if backward else None), (grad_hidden.stride(0) if backward else 0)
    a.grad_weight, a.ld_grad_weight = _ptr(grad_weight), (0 if grad_weight is None else grad_weight.stride(0))
    a.grad_weight_accumulate = int(accumulate)
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    fn = lib().dppo_lmhead_loss_fwd_bwd if backward else lib().dppo_lmhead_loss_fwd
    st = fn(C.byref(a), C.c_void_p(_stream_handle(stream)))
    if st != 0:
        raise DppoError(st)
    res = dict(out)
    res["grad_hidden"] = grad_hidden if backward else None
    res["grad_weight"] = grad_weight if backward else None
    res["args"], res["workspace_buf"] = a, workspace
    return res
