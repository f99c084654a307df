"""CPU-only checks of the boundary: the library loads, exports every symbol the header
declares, the ctypes mirror matches the C struct, and host-side argument validation returns
the documented codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2602_04879_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if fn.endswith(".h"):
            src = open(os.path.join(ROOT, "include", fn)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names += re.findall(r"\b(dppo_[a-z_0-9]+)\s*\(", src)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_functions()
    assert {"dppo_loss_fwd", "dppo_loss_fwd_bwd", "dppo_workspace_bytes", "dppo_status_str"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_mirror_and_constants():
    lib = B.lib()
    assert lib.dppo_args_size() == C.sizeof(B.DppoArgs)
    assert lib.dppo_version() >= 100
    assert B.workspace_bytes(32768, 151936, 20) == B.WORKSPACE_BYTES + 8 * 32768
    assert B.workspace_bytes(0, 151936, 0) == B.WORKSPACE_BYTES
    for code in range(0, 9):
        assert len(lib.dppo_status_str(code)) > 0


def _valid_args():
    a = B.DppoArgs()
    # fake non-NULL device addresses: validation must reject before touching them
    a.logits, a.T, a.V, a.ld = 0x1000, 4, 16, 16
    a.sampled_ids = a.mu_logp = a.advantages = 0x2000
    a.loss = a.divergence = a.mask = a.grad_logits = 0x3000
    a.workspace, a.workspace_bytes = 0x4000, B.WORKSPACE_BYTES
    a.K, a.variant, a.delta, a.loss_scale = 0, B.BINARY_TV, 0.1, 1.0
    return a


@pytest.mark.parametrize("mutate,code", [
    (lambda a: setattr(a, "V", 0), 2),
    (lambda a: setattr(a, "ld", 8), 2),
    (lambda a: setattr(a, "T", -1), 2),
    (lambda a: setattr(a, "V", 1 << 31), 2),
    (lambda a: setattr(a, "variant", 6), 4),
    (lambda a: setattr(a, "variant", B.FULL_TV), 1),                                                    # no mu_logits
    (lambda a: (setattr(a, "variant", B.FULL_KL), setattr(a, "mu_logits", 0x6000), setattr(a, "mu_ld", 8)), 2),
    (lambda a: (setattr(a, "variant", B.FULL_KL), setattr(a, "mu_logits", 0x6001), setattr(a, "mu_ld", 16)), 3),
    (lambda a: setattr(a, "variant", -1), 4),
    (lambda a: setattr(a, "K", -1), 5),
    (lambda a: setattr(a, "K", 1025), 5),
    (lambda a: (setattr(a, "variant", B.TOPK_TV), setattr(a, "K", 4)), 5),      # K > 0, no top-K pointers
    (lambda a: setattr(a, "loss", None), 1),
    (lambda a: setattr(a, "logits", None), 1),
    (lambda a: setattr(a, "sampled_ids", None), 1),
    (lambda a: setattr(a, "divergence", None), 1),
    (lambda a: setattr(a, "grad_logits", None), 1),
    (lambda a: setattr(a, "logits", 0x1001), 3),
    (lambda a: setattr(a, "workspace", 0x4004), 3),
    (lambda a: setattr(a, "workspace", None), 6),
    (lambda a: setattr(a, "workspace_bytes", 16), 6),
    (lambda a: setattr(a, "delta", float("nan")), 8),
    (lambda a: setattr(a, "ratio_cap", float("nan")), 8),
    (lambda a: setattr(a, "mask_rule", 3), 8),
    (lambda a: setattr(a, "mask_rule", -1), 8),
    (lambda a: (setattr(a, "mask_rule", B.MASK_RATIO_CLIP), setattr(a, "eps_low", 1.0), setattr(a, "eps_high", 0.2)), 8),
    (lambda a: (setattr(a, "mask_rule", B.MASK_RATIO_CLIP), setattr(a, "eps_low", 0.2), setattr(a, "eps_high", -0.1)), 8),
    (lambda a: setattr(a, "relax_alpha", 1.5), 8),
    (lambda a: setattr(a, "relax_alpha", -0.1), 8),
    (lambda a: setattr(a, "relax_alpha", float("nan")), 8),
    (lambda a: setattr(a, "relax_sides", 4), 8),
    (lambda a: setattr(a, "diagnostics", 0x5008), 3),
])
def test_argument_validation_codes(mutate, code):
    a = _valid_args()
    mutate(a)
    assert B.lib().dppo_loss_fwd_bwd(C.byref(a), None) == code
    assert str(code) in str(B.DppoError(code))


def test_null_args_pointer():
    assert B.lib().dppo_loss_fwd(None, None) == 1


def test_forward_ignores_missing_grad_pointer():
    a = _valid_args()
    a.grad_logits = None
    a.V = 0     # still invalid for another reason, so nothing is launched
    assert B.lib().dppo_loss_fwd(C.byref(a), None) == 2


def test_product_package_never_reaches_the_oracle():
    """The product path must not import, call or link anything under oracle/."""
    pat = re.compile(r"^\s*(from|import)\s+oracle\b|oracle[/.]dppo_oracle|dppo_oracle", re.M)
    for top in ("paper_2602_04879_amd", "include"):
        for dirpath, _, files in os.walk(os.path.join(ROOT, top)):
            for f in files:
                if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                    assert not pat.search(open(os.path.join(dirpath, f)).read()), os.path.join(dirpath, f)


def test_header_is_plain_c(tmp_path):
    """include/dppo.h is the boundary for callers in any language: it must compile as C99 and as C++
    on its own, with nothing but the standard headers it names."""
    import shutil
    import subprocess
    src = tmp_path / "use_dppo.c"
    src.write_text('#include "dppo.h"\n#include "dppo_probe.h"\n'
                   'int probe(void) { dppo_args_t a; dppo_lmhead_args_t l; (void)a; (void)l;\n'
                   '  return (int)sizeof(a) + (int)sizeof(l) + DPPO_KMAX + DPPO_NDIAG + (int)DPPO_FULL_KL + (int)DPPO_MASK_NONE; }\n')
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not available")
        r = subprocess.run([cc, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x", "c" if cc == "gcc" else "c++",
                            "-I", inc, str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_static_scratch_entry_point_validates_on_the_host():
    """dppo_loss_fwd_bwd_static: the usual argument checks (workspace excepted: it takes none), then
    its own size limit, all before any device call."""
    lib = B.lib()
    assert lib.dppo_loss_fwd_bwd_static(None, None) == 1
    a = _valid_args()
    a.workspace, a.workspace_bytes = None, 0
    a.grad_logits = None
    assert lib.dppo_loss_fwd_bwd_static(C.byref(a), None) == 1          # a gradient buffer is required
    a = _valid_args()
    a.workspace, a.workspace_bytes = None, 0
    a.V = 0
    assert lib.dppo_loss_fwd_bwd_static(C.byref(a), None) == 2
    a = _valid_args()
    a.workspace, a.workspace_bytes = None, 0
    a.T = (1 << 22) + 1                                                  # beyond DPPO_STATIC_MAX_T
    assert lib.dppo_loss_fwd_bwd_static(C.byref(a), None) == 2


def test_workspace_sizes():
    """64 KiB + 8 bytes per row for the logits entry points; the hidden-state forward needs tile
    statistics and gathered logits only, far less than a chunk of logits."""
    assert B.workspace_bytes(1000, 4096, 0) == 65536 + 8000
    T, V, K, chunk = 32768, 151936, 20, 8192
    tiles = (V + 255) // 256
    fwd = B.lmhead_fwd_workspace_bytes(T, V, K, chunk)
    assert fwd == 65536 + 8 * T + chunk * tiles * 16 + chunk * (K + 1) * 4      # every part already a multiple of 256
    both = B.lmhead_workspace_bytes(T, V, chunk)
    assert both == 65536 + chunk * V * 2 and fwd < both // 20
    assert B.lmhead_fwd_workspace_bytes(10, 64, 0, 0) <= B.lmhead_workspace_bytes(10, 64, 0)
