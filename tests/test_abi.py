"""The C-ABI library loads, exports every declared symbol, and rejects bad
arguments before touching the GPU (all of this runs without one)."""
import ctypes
import os
import re

import pytest

from paper_2106_09236_amd import binding as psa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "probsparse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith(("probsparse_", "dense_"))})


def test_exports_match_header():
    lib = psa.load()
    declared = _declared_symbols()
    assert declared == sorted(psa.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert psa.version() >= 100


def test_workspace_and_u_max_are_pure_host_arithmetic():
    s = psa.make_shape(16, 4, 512, 32, psa.PSA_F32)
    assert psa.u_max(s, 5.0) == 32
    assert psa.u_max(psa.make_shape(1, 4, 128, 25, psa.PSA_F32), 5.0) == 25
    assert psa.u_max(psa.make_shape(8, 8, 2048, 39, psa.PSA_BF16), 5.0) == 39
    assert psa.u_max(psa.make_shape(1, 8, 16384, 49, psa.PSA_BF16), 5.0) == 49
    assert psa.u_max(psa.make_shape(1, 1, 77, 3, psa.PSA_F32), 1e12) == 77
    n = psa.workspace_bytes(s, 5.0)
    assert n > 16 * 4 * 512 * 4 and n % 256 == 0
    # invalid -> 0
    assert psa.workspace_bytes(psa.make_shape(16, 4, 512, 32, psa.PSA_F32, D=128), 5.0) == 0
    assert psa.workspace_bytes(s, -1.0) == 0
    assert psa.workspace_bytes(s, float("nan")) == 0


def _call(shape, c=5.0, Q=0x1000, K=0x2000, V=0x3000, idx=0x4000, out=0x5000, ws=0x10000, ws_bytes=1 << 40,
          lengths=None, mask=None):
    lib = psa.load()
    args = [Q, K, V, lengths, idx, c, out, ctypes.byref(shape) if shape is not None else None, ws, ws_bytes, None]
    if mask is None:
        return lib.probsparse_attn_fwd(*args)
    return lib.probsparse_attn_fwd_stages(*args, mask)


def test_argument_errors_before_any_launch():
    good = psa.make_shape(2, 2, 64, 8, psa.PSA_F32)
    assert _call(good, Q=None) == -1
    assert _call(good, idx=None) == -1
    assert _call(good, out=None) == -1
    assert _call(good, ws=None) == -1
    assert _call(None) == -1
    assert _call(psa.make_shape(0, 2, 64, 8, psa.PSA_F32)) == -2
    assert _call(psa.make_shape(2, 2, 64, 0, psa.PSA_F32)) == -2
    assert _call(psa.make_shape(2, 2, 64, 8, psa.PSA_F32, D=32)) == -2
    assert _call(psa.make_shape(2, 2, 64, 8, psa.PSA_F32, L_Q=32)) == -2
    assert _call(psa.make_shape(70000, 1, 64, 8, psa.PSA_F32)) == -2
    assert _call(psa.make_shape(2, 2, 64, 8, 7)) == -3
    assert _call(good, c=0.0) == -4
    assert _call(good, c=float("inf")) == -4
    assert _call(good, c=float("nan")) == -4
    assert _call(good, mask=0) == -4
    assert _call(good, mask=8) == -4
    assert _call(good, ws_bytes=16) == -5
    assert _call(good, Q=0x1004) == -7
    assert _call(good, ws=0x10010) == -7
    for code in range(-7, 1):
        assert psa.strerror(code) and "unknown" not in psa.strerror(code)
    assert "unknown" in psa.strerror(-99)


def test_options_and_given_indices_entry_points_check_arguments():
    lib = psa.load()
    good = psa.make_shape(2, 2, 64, 8, psa.PSA_F32)
    sh = ctypes.byref(good)

    def opt(rule=psa.U_RATIO, fill=psa.FILL_VALUE, factor=0.5):
        return psa.PsaOptions(rule, fill, factor)

    # host arithmetic: u_max by rule (Sec. 3.2: L_sparse = r_sparse * L, rounded up)
    big = psa.make_shape(16, 4, 512, 32, psa.PSA_F32)
    assert lib.probsparse_u_max_opt(ctypes.byref(big), ctypes.byref(opt())) == 256
    assert lib.probsparse_u_max_opt(ctypes.byref(big), ctypes.byref(opt(factor=0.35))) == 180
    assert lib.probsparse_u_max_opt(ctypes.byref(big), ctypes.byref(opt(factor=3.0))) == 512
    assert lib.probsparse_u_max_opt(ctypes.byref(big), ctypes.byref(opt(rule=psa.U_LOG, factor=5.0))) == 32
    assert lib.probsparse_u_max_opt(ctypes.byref(big), ctypes.byref(opt(rule=5))) == 0
    assert lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(big), ctypes.byref(opt())) % 256 == 0
    assert lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(big), ctypes.byref(opt())) > 0
    assert lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(big), ctypes.byref(opt(fill=9))) == 0
    assert lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(big), ctypes.byref(opt(factor=-1.0))) == 0
    assert lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(big), None) == 0

    def fwd_opt(o, Q=0x1000, ws_bytes=1 << 40):
        return lib.probsparse_attn_fwd_opt(Q, 0x2000, 0x3000, None, 0x4000, ctypes.byref(o) if o is not None else None,
                                           0x5000, sh, 0x10000, ws_bytes, None, None, None, None)
    assert fwd_opt(None) == -1
    assert fwd_opt(opt(), Q=None) == -1
    assert fwd_opt(opt(rule=2)) == -4
    assert fwd_opt(opt(fill=-1)) == -4
    assert fwd_opt(opt(factor=0.0)) == -4
    assert fwd_opt(opt(factor=float("nan"))) == -4
    assert fwd_opt(opt(), ws_bytes=16) == -5
    assert fwd_opt(opt(), Q=0x1008) == -7

    def with_idx(sel=0x6000, u=0x7000, stride=8, fill=psa.FILL_MEAN, ws_bytes=1 << 40, Q=0x1000):
        return lib.probsparse_attn_fwd_with_indices(Q, 0x2000, 0x3000, None, sel, u, stride, fill, 0x5000, sh,
                                                    0x10000, ws_bytes, None)
    assert with_idx(sel=None) == -1
    assert with_idx(u=None) == -1
    assert with_idx(Q=None) == -1
    assert with_idx(stride=0) == -4
    assert with_idx(stride=65) == -4           # more columns than queries
    assert with_idx(fill=2) == -4
    assert with_idx(ws_bytes=16) == -5
    assert with_idx(sel=0x6002) == -7
    assert lib.probsparse_attn_with_indices_workspace_bytes(sh, 8) > 0
    assert lib.probsparse_attn_with_indices_workspace_bytes(sh, 0) == 0
    assert lib.probsparse_attn_with_indices_workspace_bytes(sh, 65) == 0


def test_exact_measure_checks_arguments():
    lib = psa.load()
    good = psa.make_shape(2, 2, 64, 8, psa.PSA_F32)
    sh = ctypes.byref(good)
    assert lib.probsparse_exact_measure(None, 0x2000, None, 0x3000, sh, None) == -1
    assert lib.probsparse_exact_measure(0x1000, 0x2000, None, None, sh, None) == -1
    assert lib.probsparse_exact_measure(0x1000, 0x2000, None, 0x3000, None, None) == -1
    assert lib.probsparse_exact_measure(0x1000, 0x2000, None, 0x3000,
                                        ctypes.byref(psa.make_shape(2, 2, 64, 8, 3)), None) == -3
    assert lib.probsparse_exact_measure(0x1000, 0x2000, None, 0x3000,
                                        ctypes.byref(psa.make_shape(2, 2, 64, 8, psa.PSA_F32, D=16)), None) == -2
    assert lib.probsparse_exact_measure(0x1008, 0x2000, None, 0x3000, sh, None) == -7
    assert lib.probsparse_exact_measure(0x1000, 0x2000, None, 0x3002, sh, None) == -7


def test_projection_entry_points_check_arguments():
    lib = psa.load()
    good = psa.make_shape(2, 2, 64, 8, psa.PSA_F32)
    sh = ctypes.byref(good)

    def wts(**kw):
        base = dict(Wq=0x100000, Wk=0x200000, Wv=0x300000, Wo=0x400000, bq=None, bk=None, bv=None, bo=0x500000)
        base.update(kw)
        return psa.PsaMhsaWeights(*[base[n] for n in ("Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo")])
    w = wts()
    assert lib.probsparse_qkv_project(None, ctypes.byref(w), 0x1000, 0x2000, 0x3000, sh, None) == -1
    assert lib.probsparse_qkv_project(0x9000, None, 0x1000, 0x2000, 0x3000, sh, None) == -1
    assert lib.probsparse_qkv_project(0x9000, ctypes.byref(wts(Wk=None)), 0x1000, 0x2000, 0x3000, sh, None) == -1
    assert lib.probsparse_qkv_project(0x9000, ctypes.byref(wts(Wq=0x100008)), 0x1000, 0x2000, 0x3000, sh, None) == -7
    assert lib.probsparse_qkv_project(0x9000, ctypes.byref(w), 0x1004, 0x2000, 0x3000, sh, None) == -7
    assert lib.probsparse_qkv_project(0x9000, ctypes.byref(w), 0x1000, 0x2000, 0x3000,
                                      ctypes.byref(psa.make_shape(2, 2, 64, 8, psa.PSA_F32, D=32)), None) == -2
    assert lib.probsparse_out_project(0x9000, ctypes.byref(wts(Wo=None)), 0x1000, sh, None) == -1
    assert lib.probsparse_out_project(0x9000, ctypes.byref(wts(bo=0x500002)), 0x1000, sh, None) == -7
    opt = psa.PsaOptions(psa.U_LOG, psa.FILL_MEAN, 5.0)
    need = lib.probsparse_mhsa_workspace_bytes(sh, ctypes.byref(opt))
    inner = lib.probsparse_attn_workspace_bytes_opt(sh, ctypes.byref(opt))
    assert need == inner + 4 * 2 * 2 * 64 * 64 * 4 and need % 256 == 0
    assert lib.probsparse_mhsa_workspace_bytes(sh, ctypes.byref(psa.PsaOptions(7, 0, 5.0))) == 0

    def mhsa(X=0x9000, wp=w, idx=0x4000, o=opt, ws=0x10000, ws_bytes=1 << 40):
        return lib.probsparse_mhsa_fwd(X, ctypes.byref(wp), None, idx, ctypes.byref(o), 0x8000, sh, ws, ws_bytes, None)
    assert mhsa(X=None) == -1
    assert mhsa(idx=None) == -1
    assert mhsa(wp=wts(Wv=None)) == -1
    assert mhsa(o=psa.PsaOptions(psa.U_LOG, 3, 5.0)) == -4
    assert mhsa(ws_bytes=need - 1) == -5
    assert mhsa(ws=0x10010) == -7


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(psa, "_lib", None)
    monkeypatch.setattr(psa, "LIB_PATH", "/nonexistent/libprobsparse.so")
    with pytest.raises(FileNotFoundError):
        psa.load()


def test_static_scratch_entry_point_checks_size_on_the_host():
    import ctypes
    lib = psa.load()
    assert lib.probsparse_static_workspace_bytes() == 16 << 20
    big = psa.make_shape(512, 8, 4096, 40, psa.PSA_BF16)
    assert psa.workspace_bytes(big, 5.0) > lib.probsparse_static_workspace_bytes()
    args = [0x1000, 0x2000, 0x3000, None, 0x4000, 5.0, 0x5000]
    assert lib.probsparse_attn_fwd_static(*args, ctypes.byref(big), None) == -5       # PSA_ERR_WORKSPACE, no GPU needed
    assert lib.probsparse_attn_fwd_static(*args, None, None) == -1
    bad = psa.make_shape(2, 2, 64, 8, psa.PSA_F32, D=32)
    assert lib.probsparse_attn_fwd_static(*args, ctypes.byref(bad), None) == -2
    good = psa.make_shape(2, 2, 64, 8, psa.PSA_F32)
    assert lib.probsparse_attn_fwd_static(*args[:5], -1.0, 0x5000, ctypes.byref(good), None) == -4
    assert lib.probsparse_attn_fwd_static(None, *args[1:], ctypes.byref(good), None) == -1


def test_backward_entry_point_checks_arguments_on_the_host():
    import ctypes
    lib = psa.load()
    good = psa.make_shape(2, 2, 64, 1, psa.PSA_F32)
    need = lib.probsparse_attn_bwd_workspace_bytes(ctypes.byref(good), 25)
    assert need > 0 and need % 256 == 0
    assert lib.probsparse_attn_bwd_workspace_bytes(ctypes.byref(good), 0) == 0
    assert lib.probsparse_attn_bwd_workspace_bytes(ctypes.byref(good), 65) == 0

    def call(shape=good, Q=0x1000, sel=0x4000, u=0x4100, u_stride=25, fill=0, G=0x5000, dQ=0x6000, ws=0x10000,
             ws_bytes=1 << 40):
        return lib.probsparse_attn_bwd(Q, 0x2000, 0x3000, None, sel, u, u_stride, fill, G, dQ, 0x7000, 0x8000,
                                       ctypes.byref(shape) if shape is not None else None, ws, ws_bytes, None)
    assert call(Q=None) == -1 and call(sel=None) == -1 and call(G=None) == -1 and call(dQ=None) == -1
    assert call(shape=None) == -1 and call(ws=None) == -1
    assert call(shape=psa.make_shape(2, 2, 64, 1, psa.PSA_F32, D=32)) == -2
    assert call(shape=psa.make_shape(2, 2, 64, 1, 7)) == -3
    assert call(u_stride=0) == -4 and call(u_stride=65) == -4 and call(fill=2) == -4
    assert call(ws_bytes=need - 1) == -5
    assert call(Q=0x1004) == -7 and call(ws=0x10010) == -7 and call(sel=0x4002) == -7
