"""Thin ctypes binding over the C ABI declared in include/attn.h.

Argument marshalling only: every step of the attention forward/backward runs in the HIP
kernels of libattn_gfx950.so.  torch is used for device memory and for the current stream.
There is no fallback: if the library has not been built, importing this module raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_gfx950.so")

STANDARD = 0
MITIGATED = 1
MITIGATED_ROW = 2
DEFAULT_BETA = 2.0
DEFAULT_EPS = 1e-3

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first with `python -m paper_2510_04212_amd.build` "
        "(there is no CPU or PyTorch fallback for the attention kernels)")

_lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
_lib.attn_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _vp]
_lib.attn_fwd.restype = _i
_lib.attn_fwd_ex.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _i, _f, _f, _vp]
_lib.attn_fwd_ex.restype = _i
_lib.attn_fwd_opt.argtypes = [_vp] * 8 + [_i, _i, _i, _i, _i, _f, _i, _f, _f, ctypes.c_uint, _vp]
_lib.attn_fwd_opt.restype = _i
_lib.attn_delta.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp]
_lib.attn_delta.restype = _i
_lib.attn_delta_hp.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp]
_lib.attn_delta_hp.restype = _i
_lib.attn_delta_recompute.argtypes = [_vp] * 6 + [_i, _i, _i, _i, _i, _f, _vp]
_lib.attn_delta_recompute.restype = _i
_ll = ctypes.c_longlong
_lib.attn_fwd_strided.argtypes = [_vp] * 5 + [_ll, _ll, _ll, _i, _i, _i, _i, _i, _f, _i, _f, _f, _vp]
_lib.attn_fwd_strided.restype = _i
_lib.attn_bwd_strided.argtypes = [_vp] * 9 + [_vp, _sz, _ll, _ll, _ll, _i, _i, _i, _i, _i, _f, _i, _vp]
_lib.attn_bwd_strided.restype = _i
_lib.attn_fwd_gqa.argtypes = [_vp] * 5 + [_i, _i, _i, _i, _i, _i, _f, _i, _f, _f, _vp]
_lib.attn_fwd_gqa.restype = _i
_lib.attn_bwd_gqa.argtypes = [_vp] * 9 + [_vp, _sz, _i, _i, _i, _i, _i, _i, _f, _i, _vp]
_lib.attn_bwd_gqa.restype = _i
_lib.attn_fwd_rect.argtypes = [_vp] * 5 + [_i, _i, _i, _i, _i, _i, _f, _i, _f, _f, _vp]
_lib.attn_fwd_rect.restype = _i
_lib.attn_bwd_rect.argtypes = [_vp] * 9 + [_vp, _sz, _i, _i, _i, _i, _i, _i, _f, _i, _vp]
_lib.attn_bwd_rect.restype = _i
_lib.attn_bwd.argtypes = [_vp] * 9 + [_vp, _sz, _i, _i, _i, _i, _i, _f, _i, _vp]
_lib.attn_bwd.restype = _i
_lib.attn_bwd_noalloc.argtypes = [_vp] * 9 + [_i, _i, _i, _i, _i, _f, _i, _vp]
_lib.attn_bwd_noalloc.restype = _i
_lib.attn_bwd_noalloc_max_rows.argtypes = []
_lib.attn_bwd_noalloc_max_rows.restype = _sz
_lib.attn_bwd_dkdv.argtypes = [_vp] * 8 + [_i, _i, _i, _i, _i, _f, _vp]
_lib.attn_bwd_dkdv.restype = _i
_lib.attn_bwd_dq.argtypes = [_vp] * 7 + [_i, _i, _i, _i, _i, _f, _vp]
_lib.attn_bwd_dq_delta.argtypes = [_vp] * 8 + [_i, _i, _i, _i, _i, _f, _vp]
_lib.attn_bwd_dq_delta.restype = _i
_lib.attn_bwd_dq.restype = _i
_lib.attn_bwd_workspace_bytes.argtypes = [_i, _i, _i, _i]
_lib.attn_bwd_workspace_bytes.restype = _sz
_lib.attn_status_string.argtypes = [_i]
_lib.attn_status_string.restype = ctypes.c_char_p
_lib.attn_fwd_key_tile.argtypes = [_i]
_lib.attn_fwd_key_tile.restype = _i

FWD_SINGLE_ROUNDING = 1
FWD_PV_E4M3 = 2
FWD_GUARD_UNDERFLOW = 4

EXPORTS = ["attn_fwd", "attn_fwd_ex", "attn_fwd_opt", "attn_delta", "attn_delta_hp",
           "attn_delta_recompute", "attn_bwd", "attn_bwd_noalloc", "attn_bwd_noalloc_max_rows",
           "attn_bwd_dkdv", "attn_bwd_dq", "attn_bwd_dq_delta", "attn_fwd_strided", "attn_bwd_strided",
           "attn_fwd_gqa", "attn_bwd_gqa", "attn_fwd_rect", "attn_bwd_rect",
           "attn_bwd_workspace_bytes",
           "attn_status_string", "attn_fwd_key_tile"]


class AttnError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        super().__init__(_lib.attn_status_string(int(status)).decode())


def raw():
    """The ctypes library object (for tests that call the C ABI with hand-made arguments)."""
    return _lib


def status_string(status):
    return _lib.attn_status_string(int(status)).decode()


def fwd_key_tile(d):
    return int(_lib.attn_fwd_key_tile(int(d)))


def bwd_workspace_bytes(B, H, N, d):
    return int(_lib.attn_bwd_workspace_bytes(B, H, N, d))


def _check(status):
    if status != 0:
        raise AttnError(status)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _bhnd(t, name):
    if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
        raise ValueError(f"{name} must be a contiguous CUDA bfloat16 tensor [B,H,N,d]")
    return t.shape


def attn_fwd(Q, K, V, causal, softmax_scale, variant=STANDARD, beta=None, eps=None,
             O=None, LSE=None, stream=None):
    """O, LSE = attention forward (attn_fwd / attn_fwd_ex of the C ABI)."""
    B, H, N, d = _bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V)):
        if _bhnd(t, n) != (B, H, N, d):
            raise ValueError(f"{n} shape differs from Q")
    if O is None:
        O = torch.empty_like(Q)
    if LSE is None:
        LSE = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    if beta is None and eps is None:
        st = _lib.attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), B, H, N, d, int(bool(causal)),
                           float(softmax_scale), int(variant), _stream(stream))
    else:
        st = _lib.attn_fwd_ex(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), B, H, N, d, int(bool(causal)),
                              float(softmax_scale), int(variant),
                              float(DEFAULT_BETA if beta is None else beta),
                              float(DEFAULT_EPS if eps is None else eps), _stream(stream))
    _check(st)
    return O, LSE


def attn_fwd_opt(Q, K, V, causal, softmax_scale, variant=STANDARD, beta=None, eps=None,
                 want_O_hp=False, want_counts=False, single_rounding=False, pv_e4m3=False,
                 guard_underflow=False, O=None, LSE=None, stream=None):
    """attn_fwd_opt of the C ABI: returns a dict with O, LSE and, when asked for, O_hp (float32
    [B,H,N,d]), ones and fired (int32 [B,H,N])."""
    B, H, N, d = _bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V)):
        if _bhnd(t, n) != (B, H, N, d):
            raise ValueError(f"{n} shape differs from Q")
    out = {"O": torch.empty_like(Q) if O is None else O,
           "LSE": torch.empty((B, H, N), dtype=torch.float32, device=Q.device) if LSE is None else LSE}
    if want_O_hp:
        out["O_hp"] = torch.empty((B, H, N, d), dtype=torch.float32, device=Q.device)
    if want_counts:
        out["ones"] = torch.empty((B, H, N), dtype=torch.int32, device=Q.device)
        out["fired"] = torch.empty((B, H, N), dtype=torch.int32, device=Q.device)
    opt = lambda k: _ptr(out[k]) if k in out else None
    st = _lib.attn_fwd_opt(_ptr(Q), _ptr(K), _ptr(V), _ptr(out["O"]), _ptr(out["LSE"]), opt("O_hp"),
                           opt("ones"), opt("fired"), B, H, N, d, int(bool(causal)),
                           float(softmax_scale), int(variant),
                           float(DEFAULT_BETA if beta is None else beta),
                           float(DEFAULT_EPS if eps is None else eps),
                           (FWD_SINGLE_ROUNDING if single_rounding else 0) | (FWD_PV_E4M3 if pv_e4m3 else 0)
                           | (FWD_GUARD_UNDERFLOW if guard_underflow else 0),
                           _stream(stream))
    _check(st)
    return out


def attn_delta_hp(O_hp, dO, delta=None, stream=None):
    """delta_hp = rowsum(dO o O_hp), float32 [B,H,N], from the float32 O_hp of attn_fwd_opt."""
    B, H, N, d = _bhnd(dO, "dO")
    if O_hp.dtype != torch.float32 or not O_hp.is_cuda or not O_hp.is_contiguous() or tuple(O_hp.shape) != (B, H, N, d):
        raise ValueError("O_hp must be a contiguous CUDA float32 tensor shaped like dO")
    if delta is None:
        delta = torch.empty((B, H, N), dtype=torch.float32, device=dO.device)
    _check(_lib.attn_delta_hp(_ptr(O_hp), _ptr(dO), _ptr(delta), B, H, N, d, _stream(stream)))
    return delta


def attn_delta_recompute(Q, K, V, dO, LSE, causal, softmax_scale, delta=None, stream=None):
    """delta = rowsum(P o dP), recomputed in float32 from Q, K, V, dO and LSE."""
    B, H, N, d = _bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V), ("dO", dO)):
        if _bhnd(t, n) != (B, H, N, d):
            raise ValueError(f"{n} shape differs from Q")
    if delta is None:
        delta = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _check(_lib.attn_delta_recompute(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(LSE), _ptr(delta),
                                     B, H, N, d, int(bool(causal)), float(softmax_scale),
                                     _stream(stream)))
    return delta


def attn_delta(O, dO, delta=None, stream=None):
    """delta = rowsum(dO o O), float32 [B,H,N]."""
    B, H, N, d = _bhnd(O, "O")
    if _bhnd(dO, "dO") != (B, H, N, d):
        raise ValueError("dO shape differs from O")
    if delta is None:
        delta = torch.empty((B, H, N), dtype=torch.float32, device=O.device)
    _check(_lib.attn_delta(_ptr(O), _ptr(dO), _ptr(delta), B, H, N, d, _stream(stream)))
    return delta


def attn_bwd(Q, K, V, O, dO, LSE, causal, softmax_scale, variant=STANDARD,
             dQ=None, dK=None, dV=None, workspace=None, stream=None):
    """dQ, dK, dV = attention backward.  `workspace` (uint8 CUDA tensor) is allocated when absent;
    after the call its first B*H*N float32 hold delta."""
    B, H, N, d = _bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V), ("O", O), ("dO", dO)):
        if _bhnd(t, n) != (B, H, N, d):
            raise ValueError(f"{n} shape differs from Q")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    need = bwd_workspace_bytes(B, H, N, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    st = _lib.attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                       _ptr(dV), _ptr(workspace), workspace.numel(), B, H, N, d, int(bool(causal)),
                       float(softmax_scale), int(variant), _stream(stream))
    _check(st)
    return dQ, dK, dV


def attn_bwd_noalloc(Q, K, V, O, dO, LSE, causal, softmax_scale, dQ, dK, dV, variant=STANDARD, stream=None):
    """attn_bwd_noalloc of the C ABI: attn_bwd with delta in the library's own device array.  The
    outputs are the caller's (this wrapper allocates nothing either)."""
    B, H, N, d = _bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V), ("O", O), ("dO", dO), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        if _bhnd(t, n) != (B, H, N, d):
            raise ValueError(f"{n} shape differs from Q")
    _check(_lib.attn_bwd_noalloc(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                                 _ptr(dV), B, H, N, d, int(bool(causal)), float(softmax_scale), int(variant),
                                 _stream(stream)))
    return dQ, dK, dV


def attn_bwd_dkdv(Q, K, V, dO, LSE, delta, causal, softmax_scale, dK=None, dV=None, stream=None):
    """Stage 2 of the backward pass alone: dK, dV (delta from attn_delta)."""
    B, H, N, d = _bhnd(Q, "Q")
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    _check(_lib.attn_bwd_dkdv(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(LSE), _ptr(delta), _ptr(dK),
                              _ptr(dV), B, H, N, d, int(bool(causal)), float(softmax_scale),
                              _stream(stream)))
    return dK, dV


def attn_bwd_dq(Q, K, V, dO, LSE, delta, causal, softmax_scale, dQ=None, stream=None):
    """Stage 3 of the backward pass alone: dQ (delta from attn_delta)."""
    B, H, N, d = _bhnd(Q, "Q")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    _check(_lib.attn_bwd_dq(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(LSE), _ptr(delta), _ptr(dQ),
                            B, H, N, d, int(bool(causal)), float(softmax_scale), _stream(stream)))
    return dQ


def attn_bwd_dq_delta(Q, K, V, O, dO, LSE, causal, softmax_scale, dQ=None, delta=None, stream=None):
    """First stage of attn_bwd: dQ, and delta = rowsum(dO o O) formed on the way (returned too)."""
    B, H, N, d = _bhnd(Q, "Q")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    if delta is None:
        delta = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _check(_lib.attn_bwd_dq_delta(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ),
                                  _ptr(delta), B, H, N, d, int(bool(causal)), float(softmax_scale),
                                  _stream(stream)))
    return dQ, delta


def _strided_bhnd(t, name, like=None):
    """A CUDA bfloat16 tensor of logical shape [B,H,N,d] with a contiguous last dimension and any
    batch / head / row strides (e.g. a permuted view of a [B,N,H,d] buffer)."""
    if t.dtype != torch.bfloat16 or not t.is_cuda or t.dim() != 4 or t.stride(3) != 1:
        raise ValueError(f"{name} must be a CUDA bfloat16 tensor [B,H,N,d] whose last dimension is contiguous")
    if like is not None and (t.shape != like.shape or t.stride() != like.stride()):
        raise ValueError(f"{name} must have the shape and strides of Q")
    return t.shape, t.stride()


def attn_fwd_strided(Q, K, V, causal, softmax_scale, variant=STANDARD, beta=None, eps=None,
                     O=None, LSE=None, stream=None):
    """attn_fwd_strided of the C ABI.  Q, K, V (and O, when given) share one set of strides;
    O defaults to a tensor laid out like Q."""
    (B, H, N, d), (sb, sh, sn, _) = _strided_bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V)):
        _strided_bhnd(t, n, Q)
    O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device) if O is None else O
    _strided_bhnd(O, "O", Q)
    if LSE is None:
        LSE = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _check(_lib.attn_fwd_strided(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), sb, sh, sn, B, H, N, d,
                                 int(bool(causal)), float(softmax_scale), int(variant),
                                 float(DEFAULT_BETA if beta is None else beta),
                                 float(DEFAULT_EPS if eps is None else eps), _stream(stream)))
    return O, LSE


def attn_bwd_strided(Q, K, V, O, dO, LSE, causal, softmax_scale, variant=STANDARD,
                     dQ=None, dK=None, dV=None, workspace=None, stream=None):
    """attn_bwd_strided of the C ABI; every bf16 tensor shares Q's strides."""
    (B, H, N, d), (sb, sh, sn, _) = _strided_bhnd(Q, "Q")
    for n, t in (("K", K), ("V", V), ("O", O), ("dO", dO)):
        _strided_bhnd(t, n, Q)
    new = lambda: torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    dQ = new() if dQ is None else dQ
    dK = new() if dK is None else dK
    dV = new() if dV is None else dV
    for n, t in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        _strided_bhnd(t, n, Q)
    need = bwd_workspace_bytes(B, H, N, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    _check(_lib.attn_bwd_strided(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ),
                                 _ptr(dK), _ptr(dV), _ptr(workspace), workspace.numel(), sb, sh, sn,
                                 B, H, N, d, int(bool(causal)), float(softmax_scale), int(variant),
                                 _stream(stream)))
    return dQ, dK, dV


def attn_fwd_gqa(Q, K, V, causal, softmax_scale, variant=STANDARD, beta=None, eps=None, stream=None):
    """Grouped-query forward: Q [B,H,N,d], K and V [B,H_kv,N,d] (contiguous)."""
    B, H, N, d = _bhnd(Q, "Q")
    Bk, Hkv, Nk, dk = _bhnd(K, "K")
    if _bhnd(V, "V") != K.shape or (Bk, Nk, dk) != (B, N, d):
        raise ValueError("K and V must be [B,H_kv,N,d] with the batch, length and head size of Q")
    O = torch.empty_like(Q)
    LSE = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _check(_lib.attn_fwd_gqa(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), B, H, Hkv, N, d,
                             int(bool(causal)), float(softmax_scale), int(variant),
                             float(DEFAULT_BETA if beta is None else beta),
                             float(DEFAULT_EPS if eps is None else eps), _stream(stream)))
    return O, LSE


def attn_bwd_gqa(Q, K, V, O, dO, LSE, causal, softmax_scale, variant=STANDARD, workspace=None, stream=None):
    """Grouped-query backward: dQ like Q, dK and dV like K."""
    B, H, N, d = _bhnd(Q, "Q")
    Hkv = _bhnd(K, "K")[1]
    for n, t in (("O", O), ("dO", dO)):
        if _bhnd(t, n) != (B, H, N, d):
            raise ValueError(f"{n} shape differs from Q")
    if _bhnd(V, "V") != K.shape:
        raise ValueError("V shape differs from K")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(K)
    need = bwd_workspace_bytes(B, H, N, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    _check(_lib.attn_bwd_gqa(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                             _ptr(dV), _ptr(workspace), workspace.numel(), B, H, Hkv, N, d,
                             int(bool(causal)), float(softmax_scale), int(variant), _stream(stream)))
    return dQ, dK, dV


def attn_fwd_rect(Q, K, V, causal, softmax_scale, variant=STANDARD, beta=None, eps=None, stream=None):
    """Forward with different numbers of queries and keys: Q [B,H,Nq,d], K and V [B,H,Nk,d]
    (contiguous); the causal mask is aligned at the bottom right."""
    B, H, Nq, d = _bhnd(Q, "Q")
    Bk, Hk, Nk, dk = _bhnd(K, "K")
    if _bhnd(V, "V") != K.shape or (Bk, Hk, dk) != (B, H, d):
        raise ValueError("K and V must be [B,H,Nk,d] with the batch, heads and head size of Q")
    O = torch.empty_like(Q)
    LSE = torch.empty((B, H, Nq), dtype=torch.float32, device=Q.device)
    _check(_lib.attn_fwd_rect(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), B, H, Nq, Nk, d,
                              int(bool(causal)), float(softmax_scale), int(variant),
                              float(DEFAULT_BETA if beta is None else beta),
                              float(DEFAULT_EPS if eps is None else eps), _stream(stream)))
    return O, LSE


def attn_bwd_rect(Q, K, V, O, dO, LSE, causal, softmax_scale, variant=STANDARD, workspace=None, stream=None):
    """Backward of attn_fwd_rect: dQ like Q, dK and dV like K."""
    B, H, Nq, d = _bhnd(Q, "Q")
    Nk = _bhnd(K, "K")[2]
    for n, t in (("O", O), ("dO", dO)):
        if _bhnd(t, n) != (B, H, Nq, d):
            raise ValueError(f"{n} shape differs from Q")
    if _bhnd(V, "V") != K.shape or tuple(K.shape) != (B, H, Nk, d):
        raise ValueError("K and V must be [B,H,Nk,d] with the batch, heads and head size of Q")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(K)
    need = bwd_workspace_bytes(B, H, Nq, d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    _check(_lib.attn_bwd_rect(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE), _ptr(dQ), _ptr(dK),
                              _ptr(dV), _ptr(workspace), workspace.numel(), B, H, Nq, Nk, d,
                              int(bool(causal)), float(softmax_scale), int(variant), _stream(stream)))
    return dQ, dK, dV
