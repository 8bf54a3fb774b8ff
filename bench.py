#!/usr/bin/env python3
"""Benchmark of the OSDN hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input: osdn_fwd
followed by osdn_bwd on the 1.3B-shaped configuration (B=4, T=4096, H=16, d_k=d_v=128,
chunk 64, bf16 I/O, fp32 state and gates) -- the configuration the headline metric is quoted
on.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line with

  value       whole-job tokens/s (B*T*steps / wall time between two device synchronisations)
  roofline    the dominant kernel (largest share of the step), its algorithmic bytes or flops
              per launch divided by its mean launch duration, measured with HIP events on the
              stream the kernel runs on (second pass over the same steps, events enabled)
  cpu_baseline  the fp64 CPU oracle timed on a bounded sample of the same workload

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--config I]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_FLOPS = 2.5e15       # MI355X dense bf16 MFMA
PEAK_HBM_BYTES = 8.0e12        # MI355X HBM3E
PEAK_FP32_VALU = 157.3e12



def measured_traffic(config_index):
    """HBM bytes per step and kernel from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of
    this workload (bench.py cannot read performance counters itself): {kernel: bytes}, or {}."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_configs{config_index}_fwd_bwd.txt")
    out = {}
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 7 and f[0].replace("_", "").isalpha():
                try:
                    out[f[0]] = float(f[6]) * 1e6          # column "total MB"
                except ValueError:
                    pass
    except OSError:
        pass
    return out


def algorithmic_bytes(cfg, es, backward_pass):
    """Compulsory HBM bytes of one pass with perfect fusion, per token-head: every input and
    output once, nothing for intermediates or checkpoints (gates fp32).
    forward: q, k, v in, o out, beta and log alpha;  backward: q, k, v, dO in, dq, dk, dv out,
    beta, log alpha and their gradients;  retention and its gradient on top with APF."""
    K, V = cfg.K, cfg.V
    if not backward_pass:
        return (2 * K + 2 * V) * es + 8 + (4 if cfg.apf else 0)
    return (4 * K + 3 * V) * es + 16 + (8 if cfg.apf else 0)


FORWARD_KERNELS = ("precond_fwd", "chunk_prep", "state_fwd", "output_fwd")


def kernel_models(cfg, es):
    """Algorithmic work of each kernel per launch: (bound, amount, unit-per-second peak).
    bytes = compulsory HBM traffic of the kernel's own inputs and outputs (every tensor
    once); flops = MFMA flops of its contractions (triangular products at half)."""
    B, T, H, K, V, C = cfg.B, cfg.T, cfg.H, cfg.K, cfg.V, 64
    th = B * T * H                       # token-heads
    nch = th // C                        # chunk-heads
    g = 4                                # bytes of an fp32 gate
    m = {}
    # phase 1: read k, beta; write k~ ; sequential, bandwidth/latency bound
    m["precond_fwd"] = ("hbm", th * (2 * K * es + g))
    # phase 1 backward: masks (read k, write 8 B per chunk and coordinate), the sigma chain
    # (read k and dk~), the per-chunk outputs (read k, dk~, dk_read; write dk, dbeta, dr)
    m["precond_mask"] = ("hbm", th * (K * es + g) + nch * K * 8)
    m["precond_chain"] = ("hbm", th * (2 * K * es + 2 * g) + nch * K * (8 + 4))
    m["precond_post"] = ("hbm", th * (4 * K * es + 6 * g) + nch * K * 8)
    # solved form of the reverse sweep (only without retention): read k twice and dk~; write the
    # 64 x 64 fp32 inverse, rho0 and the chunk's sum of lambda per chunk
    m["precond_lin"] = ("hbm", th * 3 * K * es + nch * (C * C * 4 + C * 4 + K * 4 + K * 8))
    # chunk_prep: read k, k~, v, beta, g ; write T, -W^T, (rho k~)^T, U^T
    m["chunk_prep"] = ("hbm", th * (4 * K * es + 2 * V * es + C * es + 2 * g))
    # state_fwd: read -W^T, (rho k~)^T, U^T ; write E^T, S checkpoints ; 2 KV-class GEMMs
    m["state_fwd"] = ("hbm", th * (2 * K * es + 2 * V * es + g) + nch * V * K * es)
    # output_fwd: read q, k~, S ckpt, E^T ; write o (and P when a backward pass follows)
    m["output_fwd"] = ("hbm", th * (2 * K * es + 2 * V * es + g + (C * es if cfg.backward else 0)) + nch * V * K * es)
    # bwd_chain: read -W^T, (rho k~)^T, q, dO, P ; write dE^T, dS' checkpoints
    m["bwd_chain"] = ("hbm", th * (3 * K * es + 2 * V * es + C * es + g) + nch * V * K * es)
    # bwd_post: read q, k, k~, v, dO, E^T, dE^T, T, S and dS' ckpts ; write dq, dv, dk (read side), dk~, dbeta, dg
    m["bwd_post"] = ("hbm", th * (6 * K * es + 5 * V * es + C * es + 4 * g) + 2 * nch * V * K * es)
    flops = {
        "chunk_prep": th * (C * K + C * K + C * V + C * C / 3.0),               # Gram, W, U (half), inverse
        "state_fwd": th * 4 * K * V,
        "output_fwd": th * (C * K + 2 * K * V + C * V),
        "bwd_chain": th * (6 * K * V + C * V),
        "bwd_post": th * (C * V + 2 * K * V + 2 * C * V + 6 * K * V + 2 * C * K + 4 * C * K),
    }
    return m, flops


def copy_rate(torch, dev, gib=1, reps=5):
    """Measured rate of a plain device copy of `gib` GiB (bytes read + written per second, GB/s):
    what this machine's HBM sustains, next to the 8 TB/s peak the fractions are quoted against."""
    n = gib << 28
    src = torch.empty(n, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * 4 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def decode_bench(args, cfg):
    """osdn_step on [B,1,H,*]: every launch reads and writes the whole state once (HBM-bound)."""
    import torch
    from paper_2605_13473_amd import binding as ob
    B, H, K, V = args.decode_batch, cfg.H, cfg.K, cfg.V
    dev, dt = "cuda:0", torch.bfloat16 if cfg.bf16 else torch.float32
    g = torch.Generator(device=dev).manual_seed(0)
    rnd = lambda *shape: torch.randn(*shape, device=dev, generator=g)
    unit = lambda a: a / a.norm(dim=-1, keepdim=True)
    q, k, v = unit(rnd(B, 1, H, K)).to(dt), unit(rnd(B, 1, H, K)).to(dt), rnd(B, 1, H, V).to(dt)
    beta, la = torch.sigmoid(rnd(B, 1, H)), -torch.nn.functional.softplus(rnd(B, 1, H))
    ret = torch.sigmoid(6.9 + rnd(B, 1, H)) if cfg.apf else None
    S = 0.1 * rnd(B, H, V, K)
    d = [torch.ones(B, H, K, device=dev), torch.empty(B, H, K, device=dev)]
    o = torch.empty_like(v)
    p = ob.make_params(B, 1, H, K, V, cfg.bf16, ob.Hyper())

    def step(i):
        ob.osdn_step(p, q, k, v, beta, la, ret, d[i & 1], S, o, S, d[(i + 1) & 1])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ob.osdn_profile_enable(True)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms, n = ob.osdn_profile_read()["step"]
    ob.osdn_profile_enable(False)
    es = 2 if cfg.bf16 else 4
    nbytes = B * H * (2 * V * K * 4 + 2 * K * 4 + (2 * K + 2 * V) * es + 12)     # S and d in and out, q k v o, gates
    dur = ms / n * 1e-3
    print(json.dumps({
        "metric": "OSDN recurrent step (decode), tokens/s", "value": B * args.steps / (t1 - t0), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * (t1 - t0) / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"decode step: B={B} T=1 H={H} K={K} V={V}, state in place, "
                               f"{'bf16' if cfg.bf16 else 'f32'} I/O, fp32 state"},
        "roofline": {"bound": "hbm", "achieved": nbytes / dur / 1e9, "peak": PEAK_HBM_BYTES / 1e9, "unit": "GB/s",
                     "frac": nbytes / dur / PEAK_HBM_BYTES, "traffic": None, "kernel": "step", "kernel_ms": ms / n},
        "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--packed-tokens", type=int, default=0,
                    help="side workload, not the headline: the configuration's heads on ONE packed token axis of this "
                         "many tokens (the paper trains on 65536 per GPU), cut into documents of uneven length "
                         "capped at 4096 tokens, state and preconditioner reset at every boundary")
    ap.add_argument("--decode-batch", type=int, default=0,
                    help="side workload, not the headline: time osdn_step (one token per sequence and launch, state "
                         "updated in place) for this many sequences with the configuration's heads")
    ap.add_argument("--channel-gate", action="store_true",
                    help="side workload, not the headline: the configuration's shape with one state gate per key "
                         "channel (online-scaled KDA), log alpha = -softplus(N(-1,1)) per channel")
    ap.add_argument("--segments", type=int, default=0,
                    help="experiments: force the number of segments of the two-stream pipeline (osdn_params.segments; "
                         "0 = the library decides, 1 = every kernel alone on one stream)")
    ap.add_argument("--p1-solved", type=int, default=0,
                    help="experiments: osdn_params.p1_solved (1: reverse sweep in solved form where it applies, "
                         "-1: never, 0: the library decides)")
    ap.add_argument("--no-retention", action="store_true", help="experiments: drop the configuration's retention")
    ap.add_argument("--backward", action="store_true",
                    help="experiments: also run the backward pass of a configuration that is forward-only in the list")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain device copy of 1 GiB before the steps (the reference that scales "
                         "the rocprofv3 HBM byte counters; its rate is printed with every result anyway)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every (batch, head) chain is independent, "
              "so the path would shard over batch and heads without communication). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_13473_amd import binding as ob
    from paper_2605_13473_amd.inputs import CONFIGS, make_inputs

    cfg = CONFIGS[args.config]
    if args.backward and not cfg.backward:
        import dataclasses
        cfg = dataclasses.replace(cfg, backward=True, name=cfg.name + "_with_backward")
    if args.decode_batch > 0:
        return decode_bench(args, cfg)
    cu = None
    if args.packed_tokens > 0:
        import dataclasses
        cfg = dataclasses.replace(cfg, B=1, T=args.packed_tokens, name=cfg.name + "_packed")
        rng = np.random.Generator(np.random.Philox(1))
        cu = [0]
        while cu[-1] < cfg.T:       # document lengths: 1 + exponential of mean 1200, capped at 4096
            cu.append(min(cfg.T, cu[-1] + min(4096, 1 + int(rng.exponential(1200.0)))))
    if args.channel_gate:
        import dataclasses
        cfg = dataclasses.replace(cfg, name=cfg.name + "_channel_gate")
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    ob.lib()                                        # fail loudly if the HIP library is not built
    x = make_inputs(cfg, seed=0)
    dt = torch.bfloat16 if cfg.bf16 else torch.float32
    es = 2 if cfg.bf16 else 4
    dev = "cuda:0"
    tq, tk, tv, tdO = (torch.from_numpy(x[n]).to(dev).to(dt) for n in ("q", "k", "v", "dO"))
    tb = torch.from_numpy(x["beta"]).to(dev)
    tg = None if x["log_alpha"] is None else torch.from_numpy(x["log_alpha"]).to(dev)
    if args.channel_gate:
        gen = torch.Generator(device=dev).manual_seed(2)
        tg = -torch.nn.functional.softplus(torch.randn(cfg.B, cfg.T, cfg.H, cfg.K, device=dev, generator=gen) - 1.0)
    tr = None if x["retention"] is None or args.no_retention else torch.from_numpy(x["retention"]).to(dev)
    hp = ob.Hyper(segments=args.segments, p1_solved=args.p1_solved)
    p = ob.make_params(cfg.B, cfg.T, cfg.H, cfg.K, cfg.V, cfg.bf16, hp, gate_per_channel=args.channel_gate)
    if cu is None:
        ws = ob.alloc_workspace(p, cfg.backward, dev)
    else:
        ws = torch.empty(ob.osdn_workspace_bytes_packed(p, cu, cfg.backward), dtype=torch.uint8, device=dev)
    nb = cfg.B if cu is None else len(cu) - 1           # entries of the carried tensors
    f32 = dict(dtype=torch.float32, device=dev)
    o = torch.empty_like(tv)
    S_out = torch.empty(nb, cfg.H, cfg.V, cfg.K, **f32)
    d_out = torch.empty(nb, cfg.H, cfg.K, **f32)
    dq, dk, dv = torch.empty_like(tq), torch.empty_like(tk), torch.empty_like(tv)
    dbeta = torch.empty_like(tb)
    dg = None if tg is None else torch.empty_like(tg)
    dr = None if tr is None else torch.empty_like(tb)
    dd_in = torch.empty(nb, cfg.H, cfg.K, **f32)
    dS_in = torch.empty(nb, cfg.H, cfg.V, cfg.K, **f32)

    def step():
        if cu is not None:
            ob.osdn_fwd_packed(p, tq, tk, tv, tb, tg, tr, None, None, o, S_out, d_out, cu, ws)
            if cfg.backward:
                ob.osdn_bwd_packed(p, tq, tk, tv, tb, tg, tr, None, None, tdO, None, None, dq, dk, dv, dbeta, dg,
                                   dr, dd_in, dS_in, cu, ws)
            return
        ob.osdn_fwd(p, tq, tk, tv, tb, tg, tr, None, None, o, S_out, d_out, ws)
        if cfg.backward:
            ob.osdn_bwd(p, tq, tk, tv, tb, tg, tr, None, None, tdO, None, None, dq, dk, dv, dbeta, dg, dr,
                        dd_in, dS_in, ws)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                               # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1e3 * (t1 - t0) / args.steps
    tokens_per_s = cfg.B * cfg.T * args.steps / (t1 - t0)

    # per-kernel durations: same steps again, each kernel bracketed by HIP events on its stream
    ob.osdn_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = ob.osdn_profile_read()
    ob.osdn_profile_enable(False)
    # a kernel may be launched once per segment of the sequence: durations and work are
    # summed over the launches of one step (= launch-weighted average rate)
    per_kernel = {k: ms / args.steps for k, (ms, n) in prof.items() if n > 0}
    copies_ms = per_kernel.pop("pad", None)         # moving ragged / packed sequences onto chunk boundaries
    unfold_ms = per_kernel.pop("unfold", None)      # per-channel gates: gradients of the folded operands mapped back
    launches = {k: n // args.steps for k, (ms, n) in prof.items() if n > 0}
    dominant = max(per_kernel, key=per_kernel.get)
    models, flops = kernel_models(cfg, es)
    th = cfg.B * cfg.T * cfg.H                          # token-heads of one step
    dur = per_kernel[dominant] * 1e-3
    # algorithmic bytes of the pass the dominant kernel belongs to (perfect fusion: no
    # intermediates), over that kernel's time per step
    in_bwd = dominant not in FORWARD_KERNELS
    alg_bytes = th * algorithmic_bytes(cfg, es, in_bwd)
    own_io = models[dominant][1]                        # the kernel's own inputs and outputs, every tensor once
    roof = {"bound": "hbm", "achieved": alg_bytes / dur / 1e9, "peak": PEAK_HBM_BYTES / 1e9, "unit": "GB/s",
            "frac": alg_bytes / dur / PEAK_HBM_BYTES,
            "traffic": measured_traffic(args.config).get(dominant) if cu is None and not args.channel_gate else None,
            "kernel": dominant, "kernel_ms": per_kernel[dominant], "launches_per_step": launches[dominant],
            "algorithmic_bytes": alg_bytes,
            "algorithmic_bytes_of": ("backward" if in_bwd else "forward") + " pass, perfect fusion",
            "own_io_model": {"bytes": own_io, "GB/s": own_io / dur / 1e9, "frac": own_io / dur / PEAK_HBM_BYTES,
                             "note": "the kernel's own inputs and outputs once each, intermediates included"},
            "mfma_frac_of_kernel": flops.get(dominant, 0.0) / dur / PEAK_BF16_FLOPS if cfg.bf16 else None,
            "per_kernel_ms": {k: round(v, 4) for k, v in per_kernel.items()}}
    if copies_ms is not None:
        roof["per_kernel_ms"]["pad (copies)"] = round(copies_ms, 4)
    if unfold_ms is not None:
        roof["per_kernel_ms"]["unfold"] = round(unfold_ms, 4)

    # whole-path algorithmic flops (MFMA only) per token-head, for the %-of-peak figure
    K, V, C = cfg.K, cfg.V, 64
    f_fwd = 6 * K * V + 3 * C * K + 2 * C * V + C * C / 3.0
    f_bwd = 12 * K * V + 4 * C * K + 4 * C * V
    total_flops = th * (f_fwd + (f_bwd if cfg.backward else 0.0))
    mfma_peak_frac = total_flops / (ms_per_step * 1e-3) / PEAK_BF16_FLOPS
    path_bytes = th * (algorithmic_bytes(cfg, es, False) + (algorithmic_bytes(cfg, es, True) if cfg.backward else 0))
    path_hbm_frac = path_bytes / (ms_per_step * 1e-3) / PEAK_HBM_BYTES
    binding = "hbm" if path_bytes / PEAK_HBM_BYTES > total_flops / PEAK_BF16_FLOPS else "mfma"
    prop = torch.cuda.get_device_properties(0)
    device = {"name": prop.name, "compute_units": prop.multi_processor_count,
              "clock_mhz": getattr(prop, "clock_rate", 0) / 1e3 or None,
              "hbm_gib": round(prop.total_memory / 2 ** 30, 1), "copy_GBps": copy_rate(torch, dev)}

    cpu = None
    if not args.no_cpu_baseline and cu is None and not args.channel_gate:
        import oracle
        nthreads = oracle.threads()
        nch = min(cfg.B * cfg.H, 8 * nthreads)       # ~10-30 core-seconds of oracle work
        chains = [(i // cfg.H, i % cfg.H) for i in range(nch)]
        sub = {}
        for name in ("q", "k", "v", "dO", "beta", "log_alpha", "retention"):
            a = x[name]
            sub[name] = None if a is None else np.ascontiguousarray(
                np.stack([a[b, :, h] for b, h in chains], 1)[None]).astype(np.float64)
        ohp = oracle.Hyper()
        c0 = time.perf_counter()
        oracle.fwd(sub["q"], sub["k"], sub["v"], sub["beta"], sub["log_alpha"], sub["retention"], hp=ohp)
        if cfg.backward:
            oracle.bwd(sub["q"], sub["k"], sub["v"], sub["beta"], sub["dO"], sub["log_alpha"],
                       sub["retention"], hp=ohp)
        c1 = time.perf_counter()
        cpu = {"value": nch * cfg.T / cfg.H / (c1 - c0), "unit": "tokens/s", "cores": nthreads,
               "kind": "oracle",
               "sample": f"{nch} of {cfg.B * cfg.H} (batch, head) chains, full T={cfg.T}, "
                         f"{'fwd+bwd' if cfg.backward else 'fwd'}, fp64 token-by-token recurrence; "
                         f"tokens/s scaled by 1/H to whole-token units; {c1 - c0:.1f} s"}

    line = {
        "metric": "OSDN chunkwise fwd+bwd tokens/sec @ H=16,d=128,T=4096 bf16; % MFMA peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: B={cfg.B} T={cfg.T} H={cfg.H} "
                               f"K={cfg.K} V={cfg.V} chunk=64 {'fwd+bwd' if cfg.backward else 'fwd'}",
                   "global_batch": cfg.B, "seq_len": cfg.T, "apf": cfg.apf,
                   **({} if cu is None else {"packed_sequences": len(cu) - 1})},
        "mfma_peak_frac": mfma_peak_frac,
        "path_roofline": {"binding": binding, "algorithmic_bytes": path_bytes, "algorithmic_flops": total_flops,
                          "hbm_frac": path_hbm_frac, "mfma_frac": mfma_peak_frac,
                          "t_hbm_ms": 1e3 * path_bytes / PEAK_HBM_BYTES, "t_mfma_ms": 1e3 * total_flops / PEAK_BF16_FLOPS},
        "device": device,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
