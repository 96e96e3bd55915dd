"""CPU-only checks of the boundary: the library loads, exports every symbol the header declares,
and its host-side validation rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2510_04212_amd import binding as b
    return b


def _declared_functions(header):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(attn_[a-z_]+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported(binding):
    declared = _declared_functions(os.path.join(ROOT, "include", "attn.h"))
    assert set(declared) == set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert not any("probe" in n for n in declared)       # measurement aids are not part of the boundary


def test_the_probe_library_exports_what_its_header_declares():
    from paper_2510_04212_amd import probe
    declared = _declared_functions(os.path.join(ROOT, "paper_2510_04212_amd", "csrc", "probe.h"))
    assert declared == ["attn_probe_lds_clock", "attn_probe_matrix_clock"]
    lib = ctypes.CDLL(probe.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    # argument checks happen on the host, before any launch
    assert lib.attn_probe_matrix_clock(None, 8, 10, None) == 1
    assert lib.attn_probe_matrix_clock(ctypes.c_void_p(0x1000), 0, 10, None) == 2
    assert lib.attn_probe_lds_clock(ctypes.c_void_p(0x1000), 2, 8, 10, None) == 2


def test_status_strings(binding):
    for st in range(6):
        s = binding.status_string(st)
        assert s and "unknown" not in s
    assert "unknown" in binding.status_string(99)


def test_key_tile_and_workspace_queries(binding):
    assert binding.fwd_key_tile(64) == 64 and binding.fwd_key_tile(128) == 64
    assert binding.fwd_key_tile(96) == 64 and binding.fwd_key_tile(80) == 0
    assert binding.bwd_workspace_bytes(4, 32, 4096, 128) == 4 * 32 * 4096 * 4
    assert binding.bwd_workspace_bytes(1, 1, 128, 64) == 512          # rounded up to 256
    assert binding.bwd_workspace_bytes(1, 1, 100, 64) == 512          # any N >= 1 is accepted
    assert binding.bwd_workspace_bytes(1, 1, 128, 80) == 0            # unsupported head dim
    assert binding.bwd_workspace_bytes(0, 4, 128, 64) == 0


def test_argument_validation_happens_on_the_host(binding):
    """None of these calls reaches a kernel launch (no GPU is needed to run them)."""
    lib = binding.raw()
    OK, NULL, BAD, UNSUP, WS = 0, 1, 2, 3, 4
    p = ctypes.c_void_p(0x1000)          # a non-NULL, aligned fake pointer: never dereferenced
    mis = ctypes.c_void_p(0x1004)
    fwd = lambda Q, K, V, O, L, B, H, N, d, var=0, scale=0.125: lib.attn_fwd(Q, K, V, O, L, B, H, N, d, 1, scale, var, None)
    assert fwd(p, p, p, p, p, 1, 1, 128, 80) == UNSUP        # head dim
    assert fwd(p, p, p, p, p, 1, 1, 0, 64) == UNSUP
    assert fwd(p, p, p, p, p, -1, 1, 128, 64) == BAD
    assert fwd(p, p, p, p, p, 1, 1, 128, 64, var=3) == BAD and fwd(p, p, p, p, p, 1, 1, 128, 64, var=-1) == BAD
    assert fwd(p, p, p, p, p, 1, 1, 128, 64, scale=0.0) == BAD
    assert fwd(None, p, p, p, p, 1, 1, 128, 64) == NULL
    assert fwd(p, p, p, p, None, 1, 1, 128, 64) == NULL
    assert fwd(mis, p, p, p, p, 1, 1, 128, 64) == BAD
    q = ctypes.c_void_p(0x2000)
    assert fwd(q, p, p, q, p, 1, 1, 128, 64) == BAD          # O aliases Q
    assert fwd(None, None, None, None, None, 0, 5, 128, 64) == OK      # empty batch: no-op
    ex = lambda beta, eps: lib.attn_fwd_ex(q, p, p, p, p, 1, 1, 128, 64, 1, 0.125, 1, beta, eps, None)
    assert ex(1.0, 1e-3) == BAD and ex(2.0, -1.0) == BAD and ex(float("nan"), 1e-3) == BAD
    ptrs_for_strided = [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(9)]
    ws_for_strided = ctypes.c_void_p(0x100000)
    opt = lambda ohp, ones, fired, flags=0, O=q: lib.attn_fwd_opt(p, p, p, O, p, ohp, ones, fired, 1, 1, 128, 64, 1, 0.125, 0, 2.0, 1e-3, flags, None)
    assert opt(None, None, None, flags=8) == BAD                 # unknown flag bit
    assert opt(mis, None, None) == BAD                           # misaligned optional output
    assert opt(q, None, None) == BAD                             # O_hp aliases O
    r_ = ctypes.c_void_p(0x3000)
    assert opt(None, r_, r_) == BAD                              # the two count outputs alias
    assert lib.attn_fwd_opt(p, p, p, q, p, None, None, None, 1, 1, 128, 80, 1, 0.125, 0, 2.0, 1e-3, 0, None) == UNSUP
    assert lib.attn_delta_hp(None, p, q, 1, 1, 128, 64, None) == NULL
    assert lib.attn_delta_hp(p, p, p, 1, 1, 128, 64, None) == BAD  # delta aliases an input
    assert lib.attn_delta_hp(None, None, None, 0, 3, 128, 64, None) == OK
    fs = lambda sb, sh, sn, d=64: lib.attn_fwd_strided(p, p, p, q, p, sb, sh, sn, 1, 1, 128, d, 1, 0.125, 0, 2.0, 1e-3, None)
    assert fs(0, 64, 64) == BAD and fs(8192, 8192, 60) == BAD and fs(8192, 8192, 32) == BAD   # zero, not a multiple of 8, rows overlap
    assert fs(8192, 8192, 1 << 24) == BAD and fs(8192, 8192, 80, d=80) == UNSUP
    assert lib.attn_bwd_strided(*ptrs_for_strided, ws_for_strided, 4096, 8192, 8192, 4, 1, 1, 128, 64, 1, 0.125, 0, None) == BAD
    gq = lambda H, Hkv: lib.attn_fwd_gqa(p, p, p, q, p, 1, H, Hkv, 128, 64, 1, 0.125, 0, 2.0, 1e-3, None)
    assert gq(6, 4) == BAD and gq(4, 0) == BAD and gq(2, 4) == BAD and gq(0, 0) == OK
    assert lib.attn_bwd_gqa(*ptrs_for_strided, ws_for_strided, 4096, 1, 6, 4, 128, 64, 1, 0.125, 0, None) == BAD
    fr = lambda Nq, Nk, d=64, Q=p: lib.attn_fwd_rect(Q, p, p, q, p, 1, 1, Nq, Nk, d, 1, 0.125, 0, 2.0, 1e-3, None)
    assert fr(128, 0) == UNSUP and fr(0, 128) == UNSUP and fr(-1, 128) == BAD and fr(128, -1) == BAD
    assert fr(128, 256, d=80) == UNSUP and fr(128, 256, Q=None) == NULL
    assert lib.attn_fwd_rect(None, None, None, None, None, 0, 4, 128, 256, 64, 1, 0.125, 0, 2.0, 1e-3, None) == OK
    br = lambda Nq, Nk, wb: lib.attn_bwd_rect(*ptrs_for_strided, ws_for_strided, wb, 1, 1, Nq, Nk, 64, 1, 0.125, 0, None)
    assert br(128, 0, 4096) == UNSUP and br(200, 64, 512) == WS     # delta has Nq = 200 floats: 1024 bytes
    dqd = lambda *a: lib.attn_bwd_dq_delta(*a, 1, 1, 128, 64, 1, 0.125, None)
    pp = [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(8)]
    assert dqd(*pp[:7], None) == NULL and dqd(*pp[:6], pp[0], pp[7]) == BAD      # dQ aliases Q
    assert dqd(*pp[:6], pp[6], pp[6]) == BAD and dqd(*pp[:6], pp[6], pp[3]) == BAD   # delta aliases dQ / O
    assert lib.attn_bwd_dq_delta(*([None] * 8), 0, 2, 128, 64, 1, 0.125, None) == OK
    rc = lambda *a: lib.attn_delta_recompute(*a, 1, 1, 128, 64, 1, 0.125, None)
    assert rc(p, p, p, p, p, None) == NULL and rc(p, p, p, p, p, p) == BAD and rc(p, p, p, mis, p, q) == BAD
    assert lib.attn_delta_recompute(p, p, p, p, p, q, 1, 1, 128, 64, 1, -1.0, None) == BAD
    assert lib.attn_delta(None, p, p, 1, 1, 128, 64, None) == NULL
    assert lib.attn_delta(p, p, p, 1, 1, 130, 48, None) == UNSUP
    assert lib.attn_delta(None, None, None, 2, 0, 128, 64, None) == OK
    ptrs = [ctypes.c_void_p(0x1000 * (i + 1)) for i in range(9)]
    ws = ctypes.c_void_p(0x100000)
    bwd = lambda a, w, wb, N=128: lib.attn_bwd(*a, w, wb, 1, 1, N, 64, 1, 0.125, 0, None)
    assert bwd(ptrs, ws, 0) == WS                            # too small
    assert bwd(ptrs, ctypes.c_void_p(0x100010), 4096) == WS  # not 256-byte aligned
    assert bwd(ptrs, None, 4096) == NULL
    assert bwd(ptrs, ws, 4096, N=0) == UNSUP
    assert bwd(ptrs, ws, 256, N=100) == WS                   # ragged N is accepted; 100 floats need 512 bytes
    alias = list(ptrs); alias[6] = alias[0]
    assert bwd(alias, ws, 4096) == BAD                       # dQ aliases Q
    alias = list(ptrs); alias[7] = alias[8]
    assert bwd(alias, ws, 4096) == BAD                       # dK aliases dV
    nul = list(ptrs); nul[5] = None
    assert bwd(nul, ws, 4096) == NULL


def test_binding_refuses_to_import_without_the_built_library(tmp_path):
    """No fallback: a copy of the binding that has no libattn_gfx950.so beside it must not import."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "attn_binding_copy"
    pkg.mkdir()
    shutil.copy(os.path.join(ROOT, "paper_2510_04212_amd", "binding.py"), pkg / "binding.py")
    (pkg / "__init__.py").write_text("")
    r = subprocess.run([sys.executable, "-c", "import attn_binding_copy.binding"], cwd=tmp_path,
                       capture_output=True, text=True)
    assert r.returncode != 0
    assert "ImportError" in r.stderr and "libattn_gfx950.so" in r.stderr and "no CPU" in r.stderr


def test_product_package_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import it."""
    pkg = os.path.join(ROOT, "paper_2510_04212_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
