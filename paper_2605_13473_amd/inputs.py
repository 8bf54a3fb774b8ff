"""Seeded synthetic inputs for the OSDN hot path.

This module holds none of the method's arithmetic: it only draws tensors with
the shapes and value distributions of the benchmark configurations, from a
counter-based generator (Philox), so that the HIP library and the CPU checker
can be fed exactly the same arrays.  It imports neither of them.

Distributions (per configuration): q,k ~ N(0,1) then L2-normalised over the
feature axis; v ~ N(0,1); beta = sigmoid(N(0, beta_std)); log-gate
log alpha = -softplus(N(g_mean, 1)); optional retention r = sigmoid(N(6.9, 1))
(median ~0.999, the paper's "initialised near 0.999"); dO ~ N(0,1).
Draw order is fixed: [mu,] q, k, v, beta, g, r, dO.  With ``bf16=True`` q, k, v
and dO are rounded to the nearest bfloat16 (ties to even) and returned as
float32 arrays holding exactly those values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    T: int
    H: int
    K: int
    V: int
    bf16: bool = True
    gated: bool = True          # draw log_alpha (False => ungated OSDN)
    apf: bool = False           # draw a retention tensor
    beta_std: float = 1.0
    g_mean: float = 0.0
    shift_every: int = 0        # >0: add a fresh N(0,1) mean to k every so many tokens
    backward: bool = False      # the configuration also runs the backward pass
    chunk: int = 64


# The five benchmark configurations (index = position in the benchmark's list).
CONFIGS = (
    Config("tiny_fp32_fwd", B=1, T=256, H=2, K=64, V=64, bf16=False),
    Config("340M_fwd", B=8, T=2048, H=8, K=128, V=128),
    Config("1p3B_fwd_bwd", B=4, T=4096, H=16, K=128, V=128, backward=True),
    Config("long_context_apf_fwd", B=1, T=32768, H=16, K=128, V=128, apf=True, shift_every=4096),
    Config("wide_head_apf_fwd_bwd", B=2, T=8192, H=8, K=128, V=256, apf=True, beta_std=2.0,
           g_mean=-2.0, backward=True),
)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def _softplus(x):
    return np.logaddexp(0.0, x)


def _unit(x):
    return x / np.sqrt((x * x).sum(-1, keepdims=True))


def make_inputs(cfg: Config, seed: int = 0) -> dict:
    """Draw one batch for ``cfg``.  Returns float32 arrays (None where unused):
    q, k [B,T,H,K]; v, dO [B,T,H,V]; beta, log_alpha, retention [B,T,H]."""
    rng = np.random.Generator(np.random.Philox(seed))
    B, T, H, K, V = cfg.B, cfg.T, cfg.H, cfg.K, cfg.V
    f32 = np.float32
    mu = None
    if cfg.shift_every > 0:
        nseg = (T + cfg.shift_every - 1) // cfg.shift_every
        mu = rng.standard_normal((B, nseg, H, K), dtype=f32)
    q = _unit(rng.standard_normal((B, T, H, K), dtype=f32))
    k = rng.standard_normal((B, T, H, K), dtype=f32)
    if mu is not None:
        k = k + np.repeat(mu, cfg.shift_every, axis=1)[:, :T]
    k = _unit(k)
    v = rng.standard_normal((B, T, H, V), dtype=f32)
    beta = _sigmoid(cfg.beta_std * rng.standard_normal((B, T, H), dtype=f32)).astype(f32)
    g = (-_softplus(cfg.g_mean + rng.standard_normal((B, T, H), dtype=f32))).astype(f32)
    r = _sigmoid(6.9 + rng.standard_normal((B, T, H), dtype=f32)).astype(f32)
    dO = rng.standard_normal((B, T, H, V), dtype=f32)
    if cfg.bf16:
        q, k, v, dO = (round_to_bf16(a) for a in (q, k, v, dO))
    return {
        "q": q.astype(f32), "k": k.astype(f32), "v": v, "beta": beta,
        "log_alpha": g if cfg.gated else None,
        "retention": r if cfg.apf else None,
        "dO": dO,
    }


def make_stress_inputs(B, T, H, K, V, seed=0, bf16=False, peaky=True, gated=True,
                       retention=0.0, d_lo=0.5, d_hi=2.0, key_norms=None, tiny_key_frac=0.0):
    """Inputs that make the preconditioner move by O(1) (for use with a large eta):
    keys with a few large coordinates, an initial d drawn uniformly in
    [d_lo, d_hi], optional constant-mean retention.  Same draw-order discipline.
    key_norms = (lo, hi): keys are not normalised; every token's norm is drawn log-uniformly
    from [lo, hi], and a fraction tiny_key_frac of the tokens gets a norm of 1e-4 to 1e-3
    (squared norm below the usual floor eps = 1e-6); beta is then capped token by token so
    that the recurrence stays bounded.  These draws come last, so the other tensors (beta's cap
    aside) do not depend on them."""
    rng = np.random.Generator(np.random.Philox(seed))
    f32 = np.float32
    q = _unit(rng.standard_normal((B, T, H, K), dtype=f32))
    k = rng.standard_normal((B, T, H, K), dtype=f32)
    if peaky:
        k = k * (1.0 + 6.0 * (rng.random((B, T, H, K), dtype=f32) < 4.0 / K))
    k = _unit(k)
    v = rng.standard_normal((B, T, H, V), dtype=f32)
    beta = _sigmoid(rng.standard_normal((B, T, H), dtype=f32)).astype(f32)
    g = (-_softplus(rng.standard_normal((B, T, H), dtype=f32))).astype(f32)
    d_in = (d_lo + (d_hi - d_lo) * rng.random((B, H, K), dtype=f32)).astype(f32)
    S_in = (0.5 * rng.standard_normal((B, H, V, K), dtype=f32)).astype(f32)
    dO = rng.standard_normal((B, T, H, V), dtype=f32)
    r = None
    if retention > 0.0:
        r = np.clip(retention + 0.02 * rng.standard_normal((B, T, H), dtype=f32), 0.0, 1.0).astype(f32)
    if key_norms is not None:
        lo, hi = key_norms
        norm = np.exp(np.log(lo) + (np.log(hi) - np.log(lo)) * rng.random((B, T, H, 1), dtype=f32))
        tiny = rng.random((B, T, H, 1), dtype=f32) < tiny_key_frac
        norm = np.where(tiny, 1e-4 * (1.0 + 9.0 * rng.random((B, T, H, 1), dtype=f32)), norm)
        k = (k * norm).astype(f32)
        # keep the tokens with long keys from blowing the state up over a long sequence: the write
        # scales the state along k by 1 - beta <k, d k>, so beta is capped at 0.95 / (d_hi |k|^2)
        beta = np.minimum(beta, 0.95 / (d_hi * (norm[..., 0] ** 2))).astype(f32)
    if bf16:
        q, k, v, dO = (round_to_bf16(a) for a in (q, k, v, dO))
    return {
        "q": q.astype(f32), "k": k.astype(f32), "v": v, "beta": beta,
        "log_alpha": g if gated else None, "retention": r, "d_in": d_in, "S_in": S_in, "dO": dO,
    }
