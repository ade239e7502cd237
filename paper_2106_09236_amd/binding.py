"""Thin ctypes binding over libprobsparse.so (the C ABI in include/probsparse.h).

Argument marshalling only: every step of the forward runs in the library's HIP
kernels.  PyTorch is used for device memory and streams.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libprobsparse.so")

PSA_F32, PSA_BF16 = 0, 1
STAGE_MEASURE, STAGE_SELECT, STAGE_ATTEND, STAGE_ALL = 1, 2, 4, 7
U_LOG, U_RATIO = 0, 1
FILL_MEAN, FILL_VALUE = 0, 1

EXPORTS = [
    "probsparse_attn_workspace_bytes", "probsparse_attn_fwd", "probsparse_attn_fwd_debug",
    "probsparse_attn_fwd_stages", "probsparse_u_max", "dense_attn_workspace_bytes", "dense_attn_fwd",
    "probsparse_attn_workspace_bytes_opt", "probsparse_u_max_opt", "probsparse_attn_fwd_opt",
    "probsparse_attn_with_indices_workspace_bytes", "probsparse_attn_fwd_with_indices",
    "probsparse_exact_measure", "probsparse_qkv_project", "probsparse_out_project",
    "probsparse_mhsa_workspace_bytes", "probsparse_mhsa_fwd",
    "probsparse_describe_plan", "probsparse_init", "probsparse_strerror", "probsparse_version",
    "probsparse_static_workspace_bytes", "probsparse_attn_fwd_static",
    "probsparse_attn_bwd_workspace_bytes", "probsparse_attn_bwd",
]


class PsaShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L_Q", ctypes.c_int32), ("L_K", ctypes.c_int32),
                ("D", ctypes.c_int32), ("U", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class PsaOptions(ctypes.Structure):
    _fields_ = [("u_rule", ctypes.c_int32), ("fill", ctypes.c_int32), ("factor", ctypes.c_double)]


class PsaMhsaWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo")]


class ProbSparseError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libprobsparse: {msg} (status {code})")
        self.code = code


_lib = None


def load() -> ctypes.CDLL:
    """Load the library (once).  Raises FileNotFoundError if it was never built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2106_09236_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    shp = ctypes.POINTER(PsaShape)
    fwd_args = [vp, vp, vp, i32p, i32p, ctypes.c_double, vp, shp, vp, ctypes.c_size_t, vp]
    lib.probsparse_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.probsparse_attn_workspace_bytes.argtypes = [shp, ctypes.c_double]
    lib.probsparse_u_max.restype = ctypes.c_int32
    lib.probsparse_u_max.argtypes = [shp, ctypes.c_double]
    lib.probsparse_attn_fwd.restype = ctypes.c_int
    lib.probsparse_attn_fwd.argtypes = fwd_args
    lib.probsparse_static_workspace_bytes.restype = ctypes.c_size_t
    lib.probsparse_static_workspace_bytes.argtypes = []
    lib.probsparse_attn_fwd_static.restype = ctypes.c_int
    lib.probsparse_attn_fwd_static.argtypes = [vp, vp, vp, i32p, i32p, ctypes.c_double, vp, shp, vp]
    lib.probsparse_attn_fwd_debug.restype = ctypes.c_int
    lib.probsparse_attn_fwd_debug.argtypes = fwd_args + [f32p, i32p, i32p]
    lib.probsparse_attn_fwd_stages.restype = ctypes.c_int
    lib.probsparse_attn_fwd_stages.argtypes = fwd_args + [ctypes.c_int]
    optp = ctypes.POINTER(PsaOptions)
    lib.probsparse_attn_workspace_bytes_opt.restype = ctypes.c_size_t
    lib.probsparse_attn_workspace_bytes_opt.argtypes = [shp, optp]
    lib.probsparse_u_max_opt.restype = ctypes.c_int32
    lib.probsparse_u_max_opt.argtypes = [shp, optp]
    lib.probsparse_attn_fwd_opt.restype = ctypes.c_int
    lib.probsparse_attn_fwd_opt.argtypes = [vp, vp, vp, i32p, i32p, optp, vp, shp, vp, ctypes.c_size_t, vp,
                                            f32p, i32p, i32p]
    lib.probsparse_attn_with_indices_workspace_bytes.restype = ctypes.c_size_t
    lib.probsparse_attn_with_indices_workspace_bytes.argtypes = [shp, ctypes.c_int32]
    lib.probsparse_attn_fwd_with_indices.restype = ctypes.c_int
    lib.probsparse_attn_fwd_with_indices.argtypes = [vp, vp, vp, i32p, i32p, i32p, ctypes.c_int32, ctypes.c_int32,
                                                     vp, shp, vp, ctypes.c_size_t, vp]
    lib.probsparse_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.probsparse_attn_bwd_workspace_bytes.argtypes = [shp, ctypes.c_int32]
    lib.probsparse_attn_bwd.restype = ctypes.c_int
    lib.probsparse_attn_bwd.argtypes = [vp, vp, vp, i32p, i32p, i32p, ctypes.c_int32, ctypes.c_int32,
                                        vp, vp, vp, vp, shp, vp, ctypes.c_size_t, vp]
    lib.probsparse_exact_measure.restype = ctypes.c_int
    lib.probsparse_exact_measure.argtypes = [vp, vp, i32p, f32p, shp, vp]
    wp = ctypes.POINTER(PsaMhsaWeights)
    lib.probsparse_qkv_project.restype = ctypes.c_int
    lib.probsparse_qkv_project.argtypes = [vp, wp, vp, vp, vp, shp, vp]
    lib.probsparse_out_project.restype = ctypes.c_int
    lib.probsparse_out_project.argtypes = [vp, wp, vp, shp, vp]
    lib.probsparse_mhsa_workspace_bytes.restype = ctypes.c_size_t
    lib.probsparse_mhsa_workspace_bytes.argtypes = [shp, optp]
    lib.probsparse_mhsa_fwd.restype = ctypes.c_int
    lib.probsparse_mhsa_fwd.argtypes = [vp, wp, i32p, i32p, optp, vp, shp, vp, ctypes.c_size_t, vp]
    lib.dense_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.dense_attn_workspace_bytes.argtypes = [shp]
    lib.dense_attn_fwd.restype = ctypes.c_int
    lib.dense_attn_fwd.argtypes = [vp, vp, vp, i32p, vp, shp, vp, ctypes.c_size_t, vp]
    lib.probsparse_strerror.restype = ctypes.c_char_p
    lib.probsparse_strerror.argtypes = [ctypes.c_int]
    lib.probsparse_version.restype = ctypes.c_int
    lib.probsparse_version.argtypes = []
    lib.probsparse_init.restype = ctypes.c_int
    lib.probsparse_init.argtypes = []
    lib.probsparse_describe_plan.restype = ctypes.c_int
    lib.probsparse_describe_plan.argtypes = [shp, optp, ctypes.c_int32, ctypes.c_char_p, ctypes.c_size_t]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().probsparse_strerror(code).decode()


def _check(code: int):
    if code != 0:
        raise ProbSparseError(code, strerror(code))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PSA_F32
    if t.dtype == torch.bfloat16:
        return PSA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_shape(B: int, H: int, L: int, U: int, dtype: int, D: int = 64, L_Q: Optional[int] = None) -> PsaShape:
    return PsaShape(B, H, L if L_Q is None else L_Q, L, D, U, dtype)


def _shape_of(Q: torch.Tensor, sample_idx: Optional[torch.Tensor]) -> PsaShape:
    B, H, L, D = Q.shape
    U = 1 if sample_idx is None else sample_idx.shape[-1]
    return make_shape(B, H, L, U, _dtype_code(Q), D)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def _require_dev(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def workspace_bytes(shape: PsaShape, c: float) -> int:
    return load().probsparse_attn_workspace_bytes(ctypes.byref(shape), c)


def u_max(shape: PsaShape, c: float) -> int:
    return load().probsparse_u_max(ctypes.byref(shape), c)


def alloc_workspace(shape: PsaShape, c: float, device="cuda") -> torch.Tensor:
    n = workspace_bytes(shape, c)
    if n == 0:
        raise ProbSparseError(-2, "invalid shape or c for workspace sizing")
    return torch.empty(n, dtype=torch.uint8, device=device)


def probsparse_attn_fwd(Q, K, V, lengths, sample_idx, c: float, out=None, workspace=None):
    """out = prob-sparse self-attention of (Q, K, V); see include/probsparse.h."""
    _require_dev(Q, K, V, lengths, sample_idx, out, workspace)
    shape = _shape_of(Q, sample_idx)
    if out is None:
        out = torch.empty_like(Q)
    if workspace is None:
        workspace = alloc_workspace(shape, c, Q.device)
    _check(load().probsparse_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sample_idx), c, _ptr(out),
                                      ctypes.byref(shape), _ptr(workspace), workspace.numel(), _stream_ptr()))
    return out


def probsparse_attn_fwd_static(Q, K, V, lengths, sample_idx, c: float, out):
    """The forward on the library's own static scratch: no workspace argument, nothing allocated
    (`out` must be given)."""
    _require_dev(Q, K, V, lengths, sample_idx, out)
    shape = _shape_of(Q, sample_idx)
    _check(load().probsparse_attn_fwd_static(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sample_idx), c, _ptr(out),
                                             ctypes.byref(shape), _stream_ptr()))
    return out


def probsparse_attn_fwd_debug(Q, K, V, lengths, sample_idx, c: float, out=None, workspace=None):
    """Returns (out, M [B,H,L] f32, sel [B,H,u_max] i32, u [B] i32)."""
    _require_dev(Q, K, V, lengths, sample_idx, out, workspace)
    shape = _shape_of(Q, sample_idx)
    B, H, L, _ = Q.shape
    if out is None:
        out = torch.empty_like(Q)
    if workspace is None:
        workspace = alloc_workspace(shape, c, Q.device)
    um = u_max(shape, c)
    M = torch.empty((B, H, L), dtype=torch.float32, device=Q.device)
    sel = torch.empty((B, H, um), dtype=torch.int32, device=Q.device)
    u = torch.empty((B,), dtype=torch.int32, device=Q.device)
    _check(load().probsparse_attn_fwd_debug(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sample_idx), c, _ptr(out),
                                            ctypes.byref(shape), _ptr(workspace), workspace.numel(), _stream_ptr(),
                                            _ptr(M), _ptr(sel), _ptr(u)))
    return out, M, sel, u


def probsparse_attn_fwd_stages(Q, K, V, lengths, sample_idx, c: float, out, workspace, stage_mask: int):
    _require_dev(Q, K, V, lengths, sample_idx, out, workspace)
    shape = _shape_of(Q, sample_idx)
    _check(load().probsparse_attn_fwd_stages(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sample_idx), c, _ptr(out),
                                             ctypes.byref(shape), _ptr(workspace), workspace.numel(), _stream_ptr(),
                                             stage_mask))
    return out


def probsparse_attn_fwd_opt(Q, K, V, lengths, sample_idx, u_rule: int, factor: float, fill: int,
                            out=None, workspace=None, taps: bool = True):
    """The forward with the rule for u (U_LOG: ceil(factor ln n), U_RATIO: ceil(factor n))
    and the fill (FILL_MEAN, FILL_VALUE) selectable.  Returns (out, M, sel, u) with
    taps, else out."""
    _require_dev(Q, K, V, lengths, sample_idx, out, workspace)
    shape = _shape_of(Q, sample_idx)
    opt = PsaOptions(u_rule, fill, factor)
    B, H, L, _ = Q.shape
    lib = load()
    if out is None:
        out = torch.empty_like(Q)
    if workspace is None:
        n = lib.probsparse_attn_workspace_bytes_opt(ctypes.byref(shape), ctypes.byref(opt))
        if n == 0:
            raise ProbSparseError(-4, "invalid shape or options for workspace sizing")
        workspace = torch.empty(n, dtype=torch.uint8, device=Q.device)
    M = sel = u = None
    if taps:
        um = lib.probsparse_u_max_opt(ctypes.byref(shape), ctypes.byref(opt))
        M = torch.empty((B, H, L), dtype=torch.float32, device=Q.device)
        sel = torch.empty((B, H, um), dtype=torch.int32, device=Q.device)
        u = torch.empty((B,), dtype=torch.int32, device=Q.device)
    _check(lib.probsparse_attn_fwd_opt(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sample_idx), ctypes.byref(opt),
                                       _ptr(out), ctypes.byref(shape), _ptr(workspace), workspace.numel(),
                                       _stream_ptr(), _ptr(M), _ptr(sel), _ptr(u)))
    return (out, M, sel, u) if taps else out


def probsparse_attn_fwd_with_indices(Q, K, V, lengths, sel, u, fill: int = FILL_MEAN, out=None, workspace=None):
    """Steps a3 + a4 for given index sets: sel [B, H, u_stride] int32, u [B] int32."""
    _require_dev(Q, K, V, lengths, sel, u, out, workspace)
    shape = _shape_of(Q, None)
    u_stride = sel.shape[-1]
    lib = load()
    if out is None:
        out = torch.empty_like(Q)
    if workspace is None:
        n = lib.probsparse_attn_with_indices_workspace_bytes(ctypes.byref(shape), u_stride)
        if n == 0:
            raise ProbSparseError(-4, "invalid shape or u_stride for workspace sizing")
        workspace = torch.empty(n, dtype=torch.uint8, device=Q.device)
    _check(lib.probsparse_attn_fwd_with_indices(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sel), _ptr(u),
                                                u_stride, fill, _ptr(out), ctypes.byref(shape), _ptr(workspace),
                                                workspace.numel(), _stream_ptr()))
    return out


def probsparse_attn_bwd(Q, K, V, lengths, sel, u, dOut, fill: int = FILL_MEAN, workspace=None):
    """Gradients (dQ, dK, dV) of steps a3 + a4 for the index sets sel [B, H, u_stride], u [B]."""
    _require_dev(Q, K, V, lengths, sel, u, dOut, workspace)
    shape = _shape_of(Q, None)
    u_stride = sel.shape[-1]
    lib = load()
    if workspace is None:
        n = lib.probsparse_attn_bwd_workspace_bytes(ctypes.byref(shape), u_stride)
        if n == 0:
            raise ProbSparseError(-4, "invalid shape or u_stride for workspace sizing")
        workspace = torch.empty(n, dtype=torch.uint8, device=Q.device)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(Q)
    _check(lib.probsparse_attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(sel), _ptr(u), u_stride, fill,
                                   _ptr(dOut), _ptr(dQ), _ptr(dK), _ptr(dV), ctypes.byref(shape), _ptr(workspace),
                                   workspace.numel(), _stream_ptr()))
    return dQ, dK, dV


def probsparse_exact_measure(Q, K, lengths, M_out=None):
    """The exact sparsity measure of Eq. 10, [B, H, L] float32 (a diagnostic; dense in the keys)."""
    _require_dev(Q, K, lengths, M_out)
    shape = _shape_of(Q, None)
    B, H, L, _ = Q.shape
    if M_out is None:
        M_out = torch.empty((B, H, L), dtype=torch.float32, device=Q.device)
    _check(load().probsparse_exact_measure(_ptr(Q), _ptr(K), _ptr(lengths), _ptr(M_out), ctypes.byref(shape),
                                           _stream_ptr()))
    return M_out


def make_weights(Wq=None, Wk=None, Wv=None, Wo=None, bq=None, bk=None, bv=None, bo=None) -> PsaMhsaWeights:
    _require_dev(Wq, Wk, Wv, Wo, bq, bk, bv, bo)
    return PsaMhsaWeights(*[_ptr(t) for t in (Wq, Wk, Wv, Wo, bq, bk, bv, bo)])


def _mhsa_shape(X: torch.Tensor, U: int) -> PsaShape:
    B, L, dm = X.shape
    return make_shape(B, dm // 64, L, U, _dtype_code(X))


def probsparse_qkv_project(X, weights: PsaMhsaWeights):
    """X [B, L, H*64] -> Q, K, V [B, H, L, 64] (Sec. 3.1)."""
    _require_dev(X)
    shape = _mhsa_shape(X, 1)
    B, L, _ = X.shape
    Q, K, V = (torch.empty((B, shape.H, L, 64), dtype=X.dtype, device=X.device) for _ in range(3))
    _check(load().probsparse_qkv_project(_ptr(X), ctypes.byref(weights), _ptr(Q), _ptr(K), _ptr(V), ctypes.byref(shape),
                                         _stream_ptr()))
    return Q, K, V


def probsparse_out_project(A, weights: PsaMhsaWeights):
    """A [B, H, L, 64] -> Y [B, L, H*64]."""
    _require_dev(A)
    B, H, L, _ = A.shape
    shape = make_shape(B, H, L, 1, _dtype_code(A))
    Y = torch.empty((B, L, H * 64), dtype=A.dtype, device=A.device)
    _check(load().probsparse_out_project(_ptr(A), ctypes.byref(weights), _ptr(Y), ctypes.byref(shape), _stream_ptr()))
    return Y


def probsparse_mhsa_fwd(X, weights: PsaMhsaWeights, lengths, sample_idx, u_rule: int, factor: float, fill: int,
                        Y=None, workspace=None):
    """The whole module: projections, prob-sparse attention per head, output matrix."""
    _require_dev(X, lengths, sample_idx, Y, workspace)
    shape = _mhsa_shape(X, sample_idx.shape[-1])
    opt = PsaOptions(u_rule, fill, factor)
    lib = load()
    if Y is None:
        Y = torch.empty_like(X)
    if workspace is None:
        n = lib.probsparse_mhsa_workspace_bytes(ctypes.byref(shape), ctypes.byref(opt))
        if n == 0:
            raise ProbSparseError(-4, "invalid shape or options for workspace sizing")
        workspace = torch.empty(n, dtype=torch.uint8, device=X.device)
    _check(lib.probsparse_mhsa_fwd(_ptr(X), ctypes.byref(weights), _ptr(lengths), _ptr(sample_idx), ctypes.byref(opt),
                                   _ptr(Y), ctypes.byref(shape), _ptr(workspace), workspace.numel(), _stream_ptr()))
    return Y


def dense_workspace_bytes(shape: PsaShape) -> int:
    return load().dense_attn_workspace_bytes(ctypes.byref(shape))


def dense_attn_fwd(Q, K, V, lengths, out=None, workspace=None):
    """Baseline: dense softmax(QK^T/sqrt(d))V over the valid keys."""
    _require_dev(Q, K, V, lengths, out, workspace)
    shape = _shape_of(Q, None)
    if out is None:
        out = torch.empty_like(Q)
    if workspace is None:
        workspace = torch.empty(max(256, dense_workspace_bytes(shape)), dtype=torch.uint8, device=Q.device)
    _check(load().dense_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(lengths), _ptr(out), ctypes.byref(shape),
                                 _ptr(workspace), workspace.numel(), _stream_ptr()))
    return out


def version() -> int:
    return load().probsparse_version()


def probsparse_describe_plan(shape, opt=None, u_stride: int = 0) -> dict:
    """The kernels a call with this shape would launch (host only), as a dict of the words of
    probsparse_describe_plan(); `opt` is a PsaOptions (selection rule) or None with u_stride > 0."""
    buf = ctypes.create_string_buffer(512)
    _check(load().probsparse_describe_plan(ctypes.byref(shape), None if opt is None else ctypes.byref(opt),
                                           u_stride, buf, len(buf)))
    return dict(word.split("=", 1) for word in buf.value.decode().split())


def probsparse_init() -> None:
    """Optional per-device set-up (see include/probsparse.h); needed only before capturing the first call on a device."""
    _check(load().probsparse_init())
