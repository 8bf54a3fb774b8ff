"""Thin Python binding of libosdn (argument marshalling only).

``osdn_precond_update``, ``osdn_fwd``, ``osdn_bwd``, ``osdn_workspace_bytes`` and
``osdn_strerror`` mirror the C entry points of ``include/osdn.h`` one to one: they take
torch tensors that already live on the GPU (PyTorch is used for device memory and
streams only), check dtype / contiguity / device, and pass raw pointers.  Every step of
the computation runs in the HIP library; there is no fallback of any kind: if the shared
object is missing this module raises.

``forward`` / ``backward`` are conveniences that allocate the outputs and the workspace.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libosdn.so")
_lib = None

OSDN_F32, OSDN_BF16 = 0, 1


class OsdnParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("T", ctypes.c_int32), ("H", ctypes.c_int32),
        ("K", ctypes.c_int32), ("V", ctypes.c_int32), ("chunk", ctypes.c_int32),
        ("io_dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("eta", ctypes.c_float),
        ("d_min", ctypes.c_float), ("d_max", ctypes.c_float), ("eps", ctypes.c_float),
        ("beta_aware", ctypes.c_int32), ("retention_per_channel", ctypes.c_int32),
        ("gate_per_channel", ctypes.c_int32),
        ("segments", ctypes.c_int32), ("p1_pieces", ctypes.c_int32), ("p1_piece_sweeps", ctypes.c_int32),
        ("p1_solved", ctypes.c_int32),
    ]


class OsdnError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libosdn error {status}: {osdn_strerror(status)}")


def lib():
    """Load libosdn.so (built in-tree by ``build.py``); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_13473_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, fp = ctypes.c_void_p, ctypes.c_void_p
        pp = ctypes.POINTER(OsdnParams)
        L.osdn_workspace_bytes.restype = ctypes.c_size_t
        L.osdn_workspace_bytes.argtypes = [pp, ctypes.c_int]
        L.osdn_debug_mask_offset.restype = ctypes.c_size_t
        L.osdn_debug_mask_offset.argtypes = [pp]
        L.osdn_strerror.restype = ctypes.c_char_p
        L.osdn_strerror.argtypes = [ctypes.c_int]
        L.osdn_precond_update.restype = ctypes.c_int
        L.osdn_precond_update.argtypes = [pp, vp, fp, fp, fp, vp, fp, fp, vp]
        L.osdn_fwd.restype = ctypes.c_int
        L.osdn_fwd.argtypes = [pp, vp, vp, vp, fp, fp, fp, fp, fp, vp, fp, fp, vp, ctypes.c_size_t, vp]
        L.osdn_fwd_noalloc.restype = ctypes.c_int
        L.osdn_fwd_noalloc.argtypes = [pp, vp, vp, vp, fp, fp, fp, fp, fp, vp, fp, fp, vp]
        L.osdn_bwd.restype = ctypes.c_int
        L.osdn_bwd.argtypes = [pp] + [vp] * 19 + [vp, ctypes.c_size_t, vp]
        ip = ctypes.POINTER(ctypes.c_int32)
        L.osdn_workspace_bytes_packed.restype = ctypes.c_size_t
        L.osdn_workspace_bytes_packed.argtypes = [pp, ip, ctypes.c_int32, ctypes.c_int]
        L.osdn_fwd_packed.restype = ctypes.c_int
        L.osdn_fwd_packed.argtypes = [pp, vp, vp, vp, fp, fp, fp, fp, fp, vp, fp, fp, ip, ctypes.c_int32, vp,
                                      ctypes.c_size_t, vp]
        L.osdn_bwd_packed.restype = ctypes.c_int
        L.osdn_bwd_packed.argtypes = [pp] + [vp] * 19 + [ip, ctypes.c_int32, vp, ctypes.c_size_t, vp]
        L.osdn_step.restype = ctypes.c_int
        L.osdn_step.argtypes = [pp, vp, vp, vp, fp, fp, fp, fp, fp, vp, fp, fp, vp]
        L.osdn_profile_enable.restype = None
        L.osdn_profile_enable.argtypes = [ctypes.c_int]
        L.osdn_profile_kernel_count.restype = ctypes.c_int
        L.osdn_profile_kernel_name.restype = ctypes.c_char_p
        L.osdn_profile_kernel_name.argtypes = [ctypes.c_int]
        L.osdn_profile_read.restype = ctypes.c_int
        L.osdn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int), ctypes.c_int]
        _lib = L
    return _lib


def osdn_profile_enable(on: bool) -> None:
    lib().osdn_profile_enable(int(bool(on)))


def osdn_profile_read() -> dict:
    """{kernel name: (summed milliseconds, launches)} since the previous read."""
    L = lib()
    n = L.osdn_profile_kernel_count()
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int * n)()
    _check(L.osdn_profile_read(ms, cnt, n))
    return {L.osdn_profile_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(n)}


def osdn_strerror(status: int) -> str:
    return lib().osdn_strerror(int(status)).decode()


def osdn_workspace_bytes(params: OsdnParams, for_backward: bool) -> int:
    return int(lib().osdn_workspace_bytes(ctypes.byref(params), int(bool(for_backward))))


def osdn_debug_mask_offset(params: OsdnParams) -> int:
    return int(lib().osdn_debug_mask_offset(ctypes.byref(params)))


def _io_torch_dtype(params: OsdnParams):
    return torch.bfloat16 if params.io_dtype == OSDN_BF16 else torch.float32


def _ptr(t, dtype, shape=None, name="tensor"):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA/HIP torch tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc):
    if rc != 0:
        raise OsdnError(rc)


def osdn_precond_update(params, k, beta, retention, d_in, k_tilde, d_out, d_ckpt=None, stream=None):
    p = params
    io, f32 = _io_torch_dtype(p), torch.float32
    _check(lib().osdn_precond_update(
        ctypes.byref(p),
        _ptr(k, io, (p.B, p.T, p.H, p.K), "k"), _ptr(beta, f32, (p.B, p.T, p.H), "beta"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, (p.B, p.H, p.K), "d_in"),
        _ptr(k_tilde, io, (p.B, p.T, p.H, p.K), "k_tilde"), _ptr(d_out, f32, (p.B, p.H, p.K), "d_out"),
        _ptr(d_ckpt, f32, None, "d_ckpt"), _stream_ptr(stream)))


def osdn_step(params, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, stream=None):
    p = params
    io, f32 = _io_torch_dtype(p), torch.float32
    bth, bthk, bthv = (p.B, p.T, p.H), (p.B, p.T, p.H, p.K), (p.B, p.T, p.H, p.V)
    _check(lib().osdn_step(
        ctypes.byref(p), _ptr(q, io, bthk, "q"), _ptr(k, io, bthk, "k"), _ptr(v, io, bthv, "v"),
        _ptr(beta, f32, bth, "beta"), _ptr(log_alpha, f32, _gate_shape(p), "log_alpha"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, (p.B, p.H, p.K), "d_in"),
        _ptr(S_in, f32, (p.B, p.H, p.V, p.K), "S_in"), _ptr(o, io, bthv, "o"),
        _ptr(S_out, f32, (p.B, p.H, p.V, p.K), "S_out"), _ptr(d_out, f32, (p.B, p.H, p.K), "d_out"),
        _stream_ptr(stream)))


def osdn_fwd(params, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, workspace,
             stream=None):
    p = params
    io, f32 = _io_torch_dtype(p), torch.float32
    bth, bthk, bthv = (p.B, p.T, p.H), (p.B, p.T, p.H, p.K), (p.B, p.T, p.H, p.V)
    _check(lib().osdn_fwd(
        ctypes.byref(p), _ptr(q, io, bthk, "q"), _ptr(k, io, bthk, "k"), _ptr(v, io, bthv, "v"),
        _ptr(beta, f32, bth, "beta"), _ptr(log_alpha, f32, _gate_shape(p), "log_alpha"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, (p.B, p.H, p.K), "d_in"),
        _ptr(S_in, f32, (p.B, p.H, p.V, p.K), "S_in"), _ptr(o, io, bthv, "o"),
        _ptr(S_out, f32, (p.B, p.H, p.V, p.K), "S_out"), _ptr(d_out, f32, (p.B, p.H, p.K), "d_out"),
        _ptr(workspace, torch.uint8, None, "workspace"), ctypes.c_size_t(workspace.numel()),
        _stream_ptr(stream)))


def osdn_fwd_noalloc(params, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, stream=None):
    p = params
    io, f32 = _io_torch_dtype(p), torch.float32
    bth, bthk, bthv = (p.B, p.T, p.H), (p.B, p.T, p.H, p.K), (p.B, p.T, p.H, p.V)
    _check(lib().osdn_fwd_noalloc(
        ctypes.byref(p), _ptr(q, io, bthk, "q"), _ptr(k, io, bthk, "k"), _ptr(v, io, bthv, "v"),
        _ptr(beta, f32, bth, "beta"), _ptr(log_alpha, f32, _gate_shape(p), "log_alpha"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, (p.B, p.H, p.K), "d_in"),
        _ptr(S_in, f32, (p.B, p.H, p.V, p.K), "S_in"), _ptr(o, io, bthv, "o"),
        _ptr(S_out, f32, (p.B, p.H, p.V, p.K), "S_out"), _ptr(d_out, f32, (p.B, p.H, p.K), "d_out"),
        _stream_ptr(stream)))


def osdn_bwd(params, q, k, v, beta, log_alpha, retention, d_in, S_in, dO, dS_out, dd_out,
             dq, dk, dv, dbeta, dlog_alpha, dretention, dd_in, dS_in, workspace, stream=None):
    p = params
    io, f32 = _io_torch_dtype(p), torch.float32
    bth, bthk, bthv = (p.B, p.T, p.H), (p.B, p.T, p.H, p.K), (p.B, p.T, p.H, p.V)
    bhk, bhvk = (p.B, p.H, p.K), (p.B, p.H, p.V, p.K)
    _check(lib().osdn_bwd(
        ctypes.byref(p), _ptr(q, io, bthk, "q"), _ptr(k, io, bthk, "k"), _ptr(v, io, bthv, "v"),
        _ptr(beta, f32, bth, "beta"), _ptr(log_alpha, f32, _gate_shape(p), "log_alpha"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, bhk, "d_in"),
        _ptr(S_in, f32, bhvk, "S_in"), _ptr(dO, io, bthv, "dO"), _ptr(dS_out, f32, bhvk, "dS_out"),
        _ptr(dd_out, f32, bhk, "dd_out"), _ptr(dq, io, bthk, "dq"), _ptr(dk, io, bthk, "dk"),
        _ptr(dv, io, bthv, "dv"), _ptr(dbeta, f32, bth, "dbeta"),
        _ptr(dlog_alpha, f32, _gate_shape(p), "dlog_alpha"), _ptr(dretention, f32, _ret_shape(p), "dretention"),
        _ptr(dd_in, f32, bhk, "dd_in"), _ptr(dS_in, f32, bhvk, "dS_in"),
        _ptr(workspace, torch.uint8, None, "workspace"), ctypes.c_size_t(workspace.numel()),
        _stream_ptr(stream)))


def _cu(cu_seqlens):
    """Host int32 array of n_seqs + 1 offsets from a sequence of ints."""
    vals = [int(x) for x in cu_seqlens]
    return (ctypes.c_int32 * len(vals))(*vals), len(vals) - 1


def osdn_workspace_bytes_packed(params: OsdnParams, cu_seqlens, for_backward: bool) -> int:
    cu, n = _cu(cu_seqlens)
    return int(lib().osdn_workspace_bytes_packed(ctypes.byref(params), cu, n, int(bool(for_backward))))


def osdn_fwd_packed(params, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, cu_seqlens,
                    workspace, stream=None):
    p = params
    cu, n = _cu(cu_seqlens)
    io, f32 = _io_torch_dtype(p), torch.float32
    bth, bthk, bthv = (p.B, p.T, p.H), (p.B, p.T, p.H, p.K), (p.B, p.T, p.H, p.V)
    _check(lib().osdn_fwd_packed(
        ctypes.byref(p), _ptr(q, io, bthk, "q"), _ptr(k, io, bthk, "k"), _ptr(v, io, bthv, "v"),
        _ptr(beta, f32, bth, "beta"), _ptr(log_alpha, f32, _gate_shape(p), "log_alpha"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, (n, p.H, p.K), "d_in"),
        _ptr(S_in, f32, (n, p.H, p.V, p.K), "S_in"), _ptr(o, io, bthv, "o"),
        _ptr(S_out, f32, (n, p.H, p.V, p.K), "S_out"), _ptr(d_out, f32, (n, p.H, p.K), "d_out"),
        cu, n, _ptr(workspace, torch.uint8, None, "workspace"), ctypes.c_size_t(workspace.numel()),
        _stream_ptr(stream)))


def osdn_bwd_packed(params, q, k, v, beta, log_alpha, retention, d_in, S_in, dO, dS_out, dd_out,
                    dq, dk, dv, dbeta, dlog_alpha, dretention, dd_in, dS_in, cu_seqlens, workspace, stream=None):
    p = params
    cu, n = _cu(cu_seqlens)
    io, f32 = _io_torch_dtype(p), torch.float32
    bth, bthk, bthv = (p.B, p.T, p.H), (p.B, p.T, p.H, p.K), (p.B, p.T, p.H, p.V)
    bhk, bhvk = (n, p.H, p.K), (n, p.H, p.V, p.K)
    _check(lib().osdn_bwd_packed(
        ctypes.byref(p), _ptr(q, io, bthk, "q"), _ptr(k, io, bthk, "k"), _ptr(v, io, bthv, "v"),
        _ptr(beta, f32, bth, "beta"), _ptr(log_alpha, f32, _gate_shape(p), "log_alpha"),
        _ptr(retention, f32, _ret_shape(p), "retention"), _ptr(d_in, f32, bhk, "d_in"),
        _ptr(S_in, f32, bhvk, "S_in"), _ptr(dO, io, bthv, "dO"), _ptr(dS_out, f32, bhvk, "dS_out"),
        _ptr(dd_out, f32, bhk, "dd_out"), _ptr(dq, io, bthk, "dq"), _ptr(dk, io, bthk, "dk"),
        _ptr(dv, io, bthv, "dv"), _ptr(dbeta, f32, bth, "dbeta"),
        _ptr(dlog_alpha, f32, _gate_shape(p), "dlog_alpha"), _ptr(dretention, f32, _ret_shape(p), "dretention"),
        _ptr(dd_in, f32, bhk, "dd_in"), _ptr(dS_in, f32, bhvk, "dS_in"),
        cu, n, _ptr(workspace, torch.uint8, None, "workspace"), ctypes.c_size_t(workspace.numel()),
        _stream_ptr(stream)))


# ------------------------------------------------------------- conveniences ----
@dataclass
class Hyper:
    scale: float | None = None   # None => K ** -0.5
    eta: float = 0.003
    d_min: float = 0.5
    d_max: float = 2.0
    eps: float = 1e-6
    beta_aware: bool = True
    # scheduling knobs of osdn_params (0: the library decides)
    segments: int = 0
    p1_pieces: int = 0
    p1_piece_sweeps: int = 0
    p1_solved: int = 0


def make_params(B, T, H, K, V, bf16: bool, hp: Hyper = Hyper(), retention_per_channel: bool = False,
                gate_per_channel: bool = False) -> OsdnParams:
    scale = float(K) ** -0.5 if hp.scale is None else float(hp.scale)
    return OsdnParams(B, T, H, K, V, 64, OSDN_BF16 if bf16 else OSDN_F32, scale, hp.eta, hp.d_min,
                      hp.d_max, hp.eps, int(hp.beta_aware), int(bool(retention_per_channel)),
                      int(bool(gate_per_channel)), int(hp.segments), int(hp.p1_pieces), int(hp.p1_piece_sweeps),
                      int(hp.p1_solved))


def _ret_shape(p: OsdnParams):
    return (p.B, p.T, p.H, p.K) if p.retention_per_channel else (p.B, p.T, p.H)


def _gate_shape(p: OsdnParams):
    return (p.B, p.T, p.H, p.K) if p.gate_per_channel else (p.B, p.T, p.H)


def _per_channel(retention) -> bool:
    return retention is not None and retention.dim() == 4


def alloc_workspace(params: OsdnParams, for_backward: bool, device="cuda") -> torch.Tensor:
    n = osdn_workspace_bytes(params, for_backward)
    if n == 0:
        raise OsdnError(-2)
    return torch.empty(n, dtype=torch.uint8, device=device)   # torch allocations are >= 256-byte aligned


def forward(q, k, v, beta, log_alpha=None, retention=None, d_in=None, S_in=None, hp: Hyper = Hyper(),
            for_backward: bool = False, workspace=None, cu_seqlens=None):
    """Allocate outputs (+ workspace) and call osdn_fwd (osdn_fwd_packed when cu_seqlens is
    given: B == 1, one carried entry per sequence).  Returns (o, S_out, d_out, ctx)."""
    B, T, H, K = k.shape
    V = v.shape[-1]
    p = make_params(B, T, H, K, V, k.dtype == torch.bfloat16, hp, _per_channel(retention), _per_channel(log_alpha))
    if cu_seqlens is not None:
        cu_seqlens = [int(x) for x in cu_seqlens]
    if workspace is None:
        if cu_seqlens is None:
            workspace = alloc_workspace(p, for_backward, k.device)
        else:
            n = osdn_workspace_bytes_packed(p, cu_seqlens, for_backward)
            if n == 0:
                raise OsdnError(-2)
            workspace = torch.empty(n, dtype=torch.uint8, device=k.device)
    nb = B if cu_seqlens is None else len(cu_seqlens) - 1
    o = torch.empty_like(v)
    S_out = torch.empty(nb, H, V, K, dtype=torch.float32, device=k.device)
    d_out = torch.empty(nb, H, K, dtype=torch.float32, device=k.device)
    if cu_seqlens is None:
        osdn_fwd(p, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, workspace)
    else:
        osdn_fwd_packed(p, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, cu_seqlens, workspace)
    ctx = dict(params=p, inputs=(q, k, v, beta, log_alpha, retention, d_in, S_in), workspace=workspace,
               cu_seqlens=cu_seqlens)
    return o, S_out, d_out, ctx


def backward(ctx, dO, dS_out=None, dd_out=None):
    """Allocate gradients and call osdn_bwd on the context returned by ``forward``."""
    p = ctx["params"]
    q, k, v, beta, log_alpha, retention, d_in, S_in = ctx["inputs"]
    cu = ctx.get("cu_seqlens")
    nb = p.B if cu is None else len(cu) - 1
    f32 = dict(dtype=torch.float32, device=k.device)
    g = {
        "dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v),
        "dbeta": torch.empty_like(beta),
        "dlog_alpha": torch.empty_like(log_alpha) if log_alpha is not None else None,
        "dretention": torch.empty_like(retention) if retention is not None else None,
        "dd_in": torch.empty(nb, p.H, p.K, **f32), "dS_in": torch.empty(nb, p.H, p.V, p.K, **f32),
    }
    if cu is None:
        osdn_bwd(p, q, k, v, beta, log_alpha, retention, d_in, S_in, dO, dS_out, dd_out,
                 g["dq"], g["dk"], g["dv"], g["dbeta"], g["dlog_alpha"], g["dretention"], g["dd_in"],
                 g["dS_in"], ctx["workspace"])
    else:
        osdn_bwd_packed(p, q, k, v, beta, log_alpha, retention, d_in, S_in, dO, dS_out, dd_out,
                        g["dq"], g["dk"], g["dv"], g["dbeta"], g["dlog_alpha"], g["dretention"], g["dd_in"],
                        g["dS_in"], cu, ctx["workspace"])
    return g


def step(q, k, v, beta, log_alpha=None, retention=None, d_in=None, S_in=None, hp: Hyper = Hyper(),
         in_place: bool = False):
    """Recurrent form for 1..64 tokens: returns (o, S_out, d_out); with in_place the state S_in
    is updated where it is (and returned)."""
    B, T, H, K = k.shape
    V = v.shape[-1]
    p = make_params(B, T, H, K, V, k.dtype == torch.bfloat16, hp, _per_channel(retention), _per_channel(log_alpha))
    f32 = dict(dtype=torch.float32, device=k.device)
    o = torch.empty_like(v)
    S_out = S_in if (in_place and S_in is not None) else torch.empty(B, H, V, K, **f32)
    d_out = torch.empty(B, H, K, **f32)
    osdn_step(p, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out)
    return o, S_out, d_out


def precond_update(k, beta, retention=None, d_in=None, hp: Hyper = Hyper(), want_ckpt: bool = False):
    """Allocate outputs and call osdn_precond_update.  Returns (k_tilde, d_out[, d_ckpt])."""
    B, T, H, K = k.shape
    p = make_params(B, T, H, K, 64, k.dtype == torch.bfloat16, hp, _per_channel(retention))
    kt = torch.empty_like(k)
    d_out = torch.empty(B, H, K, dtype=torch.float32, device=k.device)
    ck = torch.empty(B, H, T // 64, K, dtype=torch.float32, device=k.device) if want_ckpt else None
    osdn_precond_update(p, k, beta, retention, d_in, kt, d_out, ck)
    return (kt, d_out, ck) if want_ckpt else (kt, d_out)
