"""GPU parity of the chunkwise forward and backward passes with one state gate per key channel
(the chunkwise UT form of online-scaled KDA) against the CPU oracle's token-by-token recurrence
and its hand-written reverse mode."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_13473_amd import binding as ob
from paper_2605_13473_amd.inputs import make_stress_inputs
from tests.gpu_util import check, compare_backward, compare_forward, f64, oracle_hp, to_dev

pytestmark = pytest.mark.gpu


def _inputs(B, T, H, K, V, seed, bf16, g_mean=-1.0, retention=0.95):
    x = make_stress_inputs(B, T, H, K, V, seed=seed, bf16=bf16, retention=retention)
    rng = np.random.default_rng(seed + 700)
    x["log_alpha"] = (-np.logaddexp(0.0, g_mean + rng.standard_normal((B, T, H, K)))).astype(np.float32)
    return x


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(1, 64, 1, 64, 64), (2, 192, 3, 64, 128), (1, 256, 2, 128, 192), (2, 100, 2, 128, 64)])
def test_forward(shape, bf16):
    """Whole and ragged lengths, K = 64 and 128, carried state, large eta (d moves by O(1))."""
    B, T, H, K, V = shape
    compare_forward(_inputs(B, T, H, K, V, seed=81, bf16=bf16), ob.Hyper(eta=0.5), bf16)


@pytest.mark.parametrize("bf16", [False, True])
def test_strong_decay(bf16):
    """Gates with mean log alpha about -0.8 per token: the cumulative decay of a channel reaches
    e^-50 and below inside a chunk, its inverse e^+50 in the scaled write keys."""
    x = _inputs(1, 256, 2, 128, 64, seed=82, bf16=bf16, g_mean=0.0)
    assert np.cumsum(x["log_alpha"][:, :64], axis=1).min() < -50
    compare_forward(x, ob.Hyper(eta=0.3), bf16)


@pytest.mark.parametrize("bf16", [False, True])
def test_decay_near_the_documented_limit(bf16):
    """The chunk path folds e^{+|G|} into the write keys, so the documented limit on a channel's
    cumulative log-decay inside a chunk is about -80 (the exponent range of fp32 and bf16).
    Gates scaled so that the strongest channel reaches -70 to -75: forward and backward still
    agree with the oracle, and nothing overflows."""
    x = _inputs(1, 192, 2, 64, 64, seed=83, bf16=bf16, g_mean=0.0)
    worst = np.cumsum(x["log_alpha"].reshape(1, 3, 64, 2, 64), axis=2).min()
    x["log_alpha"] = (x["log_alpha"] * np.float32(-72.5 / worst)).astype(np.float32)
    worst = np.cumsum(x["log_alpha"].reshape(1, 3, 64, 2, 64), axis=2).min()
    assert -75.0 < worst < -70.0
    compare_forward(x, ob.Hyper(eta=0.3), bf16)
    compare_backward(x, ob.Hyper(eta=0.3), bf16)


def test_equal_entries_reproduce_the_scalar_gate():
    B, T, H, K, V = 2, 192, 2, 128, 128
    x = make_stress_inputs(B, T, H, K, V, seed=83, retention=0.95)
    xv = dict(x)
    xv["log_alpha"] = np.ascontiguousarray(np.broadcast_to(x["log_alpha"][..., None], (B, T, H, K)))
    hp = ob.Hyper(eta=0.5)
    o1, S1, d1 = compare_forward(x, hp, False)
    o2, S2, d2 = compare_forward(xv, hp, False)
    assert torch.equal(d1, d2)
    assert (o1 - o2).abs().max() <= 1e-4 * o1.abs().max() and (S1 - S2).abs().max() <= 1e-4 * S1.abs().max()


def test_long_sequence_pipelined_and_per_channel_retention():
    """Enough chunks for the segment pipeline, retention per coordinate as well."""
    B, T, H, K, V = 1, 64 * 44, 2, 64, 64
    x = _inputs(B, T, H, K, V, seed=84, bf16=True)
    rng = np.random.default_rng(85)
    x["retention"] = np.clip(x["retention"][..., None] + 0.03 * rng.standard_normal((B, T, H, K)), 0, 1).astype(np.float32)
    compare_forward(x, ob.Hyper(eta=0.3), True)


def test_packed_sequences():
    from tests.test_gpu_packed import _cu, _oracle_per_sequence, _packed_inputs
    lens, H, K, V, bf16, hp = [70, 1, 129, 64, 200], 2, 128, 64, False, ob.Hyper(eta=0.5)
    x = _packed_inputs(lens, H, K, V, seed=86, bf16=bf16)
    rng = np.random.default_rng(87)
    x["log_alpha"] = (-np.logaddexp(0.0, -1.0 + rng.standard_normal((1, sum(lens), H, K)))).astype(np.float32)
    t = to_dev({n: x[n] for n in ("q", "k", "v", "beta", "log_alpha", "retention", "d_in", "S_in")}, bf16)
    o, S, d, _ = ob.forward(t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], t["retention"], t["d_in"], t["S_in"],
                            hp, cu_seqlens=_cu(lens))
    torch.cuda.synchronize()
    ref = _oracle_per_sequence(x, lens, hp, backward=False)
    check("o", o, ref["o"], bf16)
    check("S_out", S, ref["S_out"], bf16)
    check("d_out", d, ref["d_out"], False)


def test_prefill_then_decode_steps():
    """Chunkwise prefill of T tokens, then single-token steps, against one oracle run over all of them."""
    B, T, H, K, V, extra = 2, 130, 2, 128, 64, 3
    x = _inputs(B, T + extra, H, K, V, seed=88, bf16=False)
    hp = ob.Hyper(eta=0.5)
    t = to_dev(x, False)
    pre = lambda a: a[:, :T].contiguous()
    o, S, d, _ = ob.forward(pre(t["q"]), pre(t["k"]), pre(t["v"]), pre(t["beta"]), pre(t["log_alpha"]),
                            pre(t["retention"]), t["d_in"], t["S_in"], hp)
    outs = [o]
    for i in range(T, T + extra):
        c = lambda a: a[:, i:i + 1].contiguous()
        oi, S, d = ob.step(c(t["q"]), c(t["k"]), c(t["v"]), c(t["beta"]), c(t["log_alpha"]), c(t["retention"]), d, S, hp)
        outs.append(oi)
    torch.cuda.synchronize()
    y = f64(x)
    oo, oS, od = oracle.fwd(y["q"], y["k"], y["v"], y["beta"], y["log_alpha"], y["retention"], y["d_in"], y["S_in"],
                            oracle_hp(hp))
    check("o", torch.cat(outs, 1), oo, False)
    check("S_out", S, oS, False)
    check("d_out", d, od, False)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(1, 64, 1, 64, 64), (2, 192, 3, 64, 128), (1, 256, 2, 128, 192), (2, 100, 2, 128, 64)])
def test_backward(shape, bf16):
    """Every gradient, dlog_alpha per channel included, with terminal adjoints of S and d."""
    B, T, H, K, V = shape
    x = _inputs(B, T, H, K, V, seed=89, bf16=bf16)
    rng = np.random.default_rng(90)
    dS = rng.standard_normal((B, H, V, K)).astype(np.float32)
    dd = rng.standard_normal((B, H, K)).astype(np.float32)
    errs = compare_backward(x, ob.Hyper(eta=0.5), bf16, dS, dd)
    assert "dlog_alpha" in errs


def test_backward_strong_decay_and_long_sequence():
    """Cumulative channel decays down to e^-50 inside a chunk, enough chunks for the segment
    pipeline, per-coordinate retention as well."""
    B, T, H, K, V = 1, 64 * 44, 1, 64, 64
    x = _inputs(B, T, H, K, V, seed=91, bf16=False, g_mean=0.0)
    rng = np.random.default_rng(92)
    x["retention"] = np.clip(x["retention"][..., None] + 0.03 * rng.standard_normal((B, T, H, K)), 0, 1).astype(np.float32)
    compare_backward(x, ob.Hyper(eta=0.3), False)


def test_backward_packed_sequences():
    from tests.test_gpu_packed import _gpu_packed, _oracle_per_sequence, _packed_inputs
    lens, H, K, V, bf16, hp = [70, 1, 129, 64], 2, 64, 64, False, ob.Hyper(eta=0.5)
    x = _packed_inputs(lens, H, K, V, seed=93, bf16=bf16)
    rng = np.random.default_rng(94)
    x["log_alpha"] = (-np.logaddexp(0.0, -1.0 + rng.standard_normal((1, sum(lens), H, K)))).astype(np.float32)
    got, _ = _gpu_packed(x, lens, hp, bf16, backward=True)
    ref = _oracle_per_sequence(x, lens, hp, backward=True)
    for name, r in ref.items():
        check(name, got[name], r, False)
