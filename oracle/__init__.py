"""OSDN CPU oracle (fp64, token by token) -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``osdn_oracle.c``.  Only ``tests/``, the smoke check
and the benchmark's ``cpu_baseline`` leg may import this package; the product
path (the HIP library and its Python binding) never does, and this package
imports nothing from it.

All arrays are numpy float64, C-contiguous, in the paper's layouts
(Appendix C, Listing 1): q,k ``[B,T,H,K]``; v,o ``[B,T,H,V]``; beta, log_alpha,
retention ``[B,T,H]`` (or ``[B,T,H,K]``: one retention per coordinate; log_alpha ``[B,T,H,K]``: one state gate
per key channel, the online-scaled KDA recurrence); d ``[B,H,K]``; S ``[B,H,V,K]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "osdn_oracle.c")
_LIB = os.path.join(_HERE, "libosdn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2 + OpenMP over the (b,h) chains)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _Params(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int), ("T", ctypes.c_int), ("H", ctypes.c_int),
        ("K", ctypes.c_int), ("V", ctypes.c_int),
        ("scale", ctypes.c_double), ("eta", ctypes.c_double),
        ("d_min", ctypes.c_double), ("d_max", ctypes.c_double),
        ("eps", ctypes.c_double), ("beta_aware", ctypes.c_int), ("gate_vec", ctypes.c_int),
        ("ret_vec", ctypes.c_int),
    ]


@dataclass
class Hyper:
    """Scalar arguments of the method (defaults: Appendix C, Listing 1)."""
    scale: float | None = None   # None => K ** -0.5
    eta: float = 0.003
    d_min: float = 0.5
    d_max: float = 2.0
    eps: float = 1e-6
    beta_aware: bool = True


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.osdn_oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().osdn_oracle_threads())


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _params(hp: Hyper, B, T, H, K, V, retention=None, log_alpha=None) -> _Params:
    scale = float(K) ** -0.5 if hp.scale is None else float(hp.scale)
    ret_vec = gate_vec = 0
    if retention is not None:
        assert retention.shape in ((B, T, H), (B, T, H, K)), retention.shape
        ret_vec = int(retention.ndim == 4)       # one retention per coordinate: diag(r_t)
    if log_alpha is not None:
        assert log_alpha.shape in ((B, T, H), (B, T, H, K)), log_alpha.shape
        gate_vec = int(log_alpha.ndim == 4)      # one state gate per key channel: Diag(alpha_t)
    return _Params(B, T, H, K, V, scale, hp.eta, hp.d_min, hp.d_max, hp.eps, int(hp.beta_aware), gate_vec,
                   ret_vec)


def precond(k, beta, retention=None, d_in=None, hp: Hyper = Hyper(), want_traj: bool = False):
    """Phase 1 alone: returns (k_tilde [B,T,H,K], d_out [B,H,K][, d_traj [B,T,H,K]])."""
    lib = _load()
    k, beta, retention, d_in = map(_f64, (k, beta, retention, d_in))
    B, T, H, K = k.shape
    P = _params(hp, B, T, H, K, 1, retention)
    kt = np.empty_like(k)
    d_out = np.empty((B, H, K))
    traj = np.empty_like(k) if want_traj else None
    rc = lib.osdn_oracle_precond(ctypes.byref(P), _p(k), _p(beta), _p(retention), _p(d_in),
                                 _p(kt), _p(d_out), _p(traj))
    assert rc == 0
    return (kt, d_out, traj) if want_traj else (kt, d_out)


def fwd(q, k, v, beta, log_alpha=None, retention=None, d_in=None, S_in=None, hp: Hyper = Hyper()):
    """Forward: returns (o [B,T,H,V], S_out [B,H,V,K], d_out [B,H,K])."""
    lib = _load()
    q, k, v, beta, log_alpha, retention, d_in, S_in = map(
        _f64, (q, k, v, beta, log_alpha, retention, d_in, S_in))
    B, T, H, K = k.shape
    V = v.shape[-1]
    P = _params(hp, B, T, H, K, V, retention, log_alpha)
    o = np.empty((B, T, H, V))
    S_out = np.empty((B, H, V, K))
    d_out = np.empty((B, H, K))
    rc = lib.osdn_oracle_fwd(ctypes.byref(P), _p(q), _p(k), _p(v), _p(beta), _p(log_alpha),
                             _p(retention), _p(d_in), _p(S_in), _p(o), _p(S_out), _p(d_out))
    assert rc == 0
    return o, S_out, d_out


def bwd(q, k, v, beta, dO, log_alpha=None, retention=None, d_in=None, S_in=None,
        dS_out=None, dd_out=None, hp: Hyper = Hyper(), mask_force=None, want_dbar: bool = False):
    """Backward of ``fwd``.  Returns a dict with dq, dk, dv, dbeta, dlog_alpha,
    dretention (None when the input was None), dd_in, dS_in.

    ``mask_force`` (int8 ``[B,T,H,K]``; 1 = inside, 0 = outside, negative = plain rule)
    overrides single decisions of the projection's derivative; ``want_dbar`` adds
    ``"dbar"``: every unprojected value r d_t + c s, ``[B,T,H,K]``."""
    lib = _load()
    q, k, v, beta, dO, log_alpha, retention, d_in, S_in, dS_out, dd_out = map(
        _f64, (q, k, v, beta, dO, log_alpha, retention, d_in, S_in, dS_out, dd_out))
    B, T, H, K = k.shape
    V = v.shape[-1]
    P = _params(hp, B, T, H, K, V, retention, log_alpha)
    g = {
        "dq": np.empty_like(q), "dk": np.empty_like(k), "dv": np.empty_like(v),
        "dbeta": np.empty_like(beta),
        "dlog_alpha": np.empty_like(log_alpha) if log_alpha is not None else None,
        "dretention": np.empty_like(retention) if retention is not None else None,
        "dd_in": np.empty((B, H, K)), "dS_in": np.empty((B, H, V, K)),
    }
    mf = None
    if mask_force is not None:
        mf = np.ascontiguousarray(mask_force, dtype=np.int8)
        assert mf.shape == (B, T, H, K)
    dbar = np.empty_like(k) if want_dbar else None
    rc = lib.osdn_oracle_bwd_masked(
        ctypes.byref(P), _p(q), _p(k), _p(v), _p(beta), _p(log_alpha),
        _p(retention), _p(d_in), _p(S_in), _p(dO), _p(dS_out), _p(dd_out),
        _p(g["dq"]), _p(g["dk"]), _p(g["dv"]), _p(g["dbeta"]),
        _p(g["dlog_alpha"]), _p(g["dretention"]), _p(g["dd_in"]), _p(g["dS_in"]),
        None if mf is None else mf.ctypes.data_as(ctypes.c_void_p), _p(dbar))
    assert rc == 0
    if want_dbar:
        g["dbar"] = dbar
    return g
