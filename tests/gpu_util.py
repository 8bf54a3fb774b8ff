"""Helpers shared by the GPU parity tests: move seeded inputs to the device, call the HIP
library through its Python binding, run the CPU oracle on the same arrays, compare."""
import numpy as np
import torch

import oracle
from paper_2605_13473_amd import binding as ob

# Tolerances (stated by the benchmark spec; the normalisation is derived in the design doc):
#   fp32 I/O : max|gpu - oracle| <= 1e-4 * max|oracle|                (1e-4 relative)
#   bf16 I/O : max|gpu - oracle| <= 2e-2 * max(1, max|oracle|)        (2e-2 max-abs, fp32 state)
F32_REL = 1e-4
BF16_ABS = 2e-2


def to_dev(x, bf16):
    dt = torch.bfloat16 if bf16 else torch.float32
    out = {}
    for name, a in x.items():
        if a is None:
            out[name] = None
        else:
            t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
            out[name] = t.to(dt) if name in ("q", "k", "v", "dO") else t
    return out


def f64(x):
    return {n: (None if a is None else np.asarray(a, dtype=np.float64)) for n, a in x.items()}


def check(name, got, ref, bf16, scale_floor=1.0):
    got = got.detach().float().cpu().numpy().astype(np.float64) if isinstance(got, torch.Tensor) else got
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    err = np.abs(got - ref).max() if ref.size else 0.0
    mx = np.abs(ref).max() if ref.size else 0.0
    if bf16:
        tol = BF16_ABS * max(scale_floor, mx)
    else:
        tol = F32_REL * max(mx, 1e-30)
    assert err <= tol, f"{name}: max|err| {err:.3e} > tol {tol:.3e} (max|ref| {mx:.3e})"
    return err


def gpu_forward(x, hp: ob.Hyper, bf16, for_backward=False):
    t = to_dev(x, bf16)
    o, S, d, ctx = ob.forward(t["q"], t["k"], t["v"], t["beta"], t.get("log_alpha"), t.get("retention"),
                              t.get("d_in"), t.get("S_in"), hp, for_backward=for_backward)
    torch.cuda.synchronize()
    return o, S, d, ctx, t


def oracle_hp(hp: ob.Hyper) -> oracle.Hyper:
    return oracle.Hyper(scale=hp.scale, eta=hp.eta, d_min=hp.d_min, d_max=hp.d_max, eps=hp.eps,
                        beta_aware=hp.beta_aware)


def compare_forward(x, hp, bf16):
    o, S, d, ctx, t = gpu_forward(x, hp, bf16)
    y = f64(x)
    oo, oS, od = oracle.fwd(y["q"], y["k"], y["v"], y["beta"], y.get("log_alpha"), y.get("retention"),
                            y.get("d_in"), y.get("S_in"), oracle_hp(hp))
    check("o", o, oo, bf16)
    check("S_out", S, oS, bf16)
    check("d_out", d, od, False)          # d is fp32 arithmetic on both I/O types
    return o, S, d


def compare_backward(x, hp, bf16, dS_out=None, dd_out=None):
    o, S, d, ctx, t = gpu_forward(x, hp, bf16, for_backward=True)
    tdS = None if dS_out is None else torch.from_numpy(dS_out).cuda()
    tdd = None if dd_out is None else torch.from_numpy(dd_out).cuda()
    g = ob.backward(ctx, t["dO"], tdS, tdd)
    torch.cuda.synchronize()
    y = f64(x)
    og = oracle.bwd(y["q"], y["k"], y["v"], y["beta"], y["dO"], y.get("log_alpha"), y.get("retention"),
                    y.get("d_in"), y.get("S_in"),
                    dS_out=None if dS_out is None else dS_out.astype(np.float64),
                    dd_out=None if dd_out is None else dd_out.astype(np.float64), hp=oracle_hp(hp))
    errs = {}
    for name, ref in og.items():
        if ref is None:
            assert g[name] is None
            continue
        errs[name] = check(name, g[name], ref, bf16)
    return errs
