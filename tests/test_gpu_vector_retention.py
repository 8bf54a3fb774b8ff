"""GPU parity with one retention value per coordinate (diag(r_t) in place of r_t I, the
vector-retention extension of the APF step) on every entry point, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_13473_amd import binding as ob
from paper_2605_13473_amd.inputs import make_stress_inputs
from tests.gpu_util import check, compare_backward, compare_forward, f64, oracle_hp, to_dev

pytestmark = pytest.mark.gpu


def _inputs(B, T, H, K, V, seed, bf16, spread=0.04):
    """Stress inputs whose scalar retention is spread out over the K coordinates."""
    x = make_stress_inputs(B, T, H, K, V, seed=seed, bf16=bf16, retention=0.95)
    rng = np.random.default_rng(seed + 500)
    r = x["retention"][..., None] + spread * rng.standard_normal((B, T, H, K)).astype(np.float32)
    x["retention"] = np.clip(r, 0.0, 1.0).astype(np.float32)
    return x


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("shape", [(1, 64, 1, 64, 64), (2, 192, 3, 64, 128), (1, 256, 2, 128, 192), (2, 100, 2, 128, 64)])
def test_forward_backward(shape, bf16):
    """Whole and ragged lengths, K = 64 and 128, large eta so that both faces of the box are hit."""
    B, T, H, K, V = shape
    x = _inputs(B, T, H, K, V, seed=71, bf16=bf16)
    hp = ob.Hyper(eta=0.5)
    compare_forward(x, hp, bf16)
    rng = np.random.default_rng(72)
    dS = rng.standard_normal((B, H, V, K)).astype(np.float32)
    dd = rng.standard_normal((B, H, K)).astype(np.float32)
    errs = compare_backward(x, hp, bf16, dS, dd)
    assert "dretention" in errs
    # the preconditioner really moved, and differently per coordinate
    _, _, traj = oracle.precond(x["k"], x["beta"], x["retention"], x["d_in"], oracle.Hyper(eta=0.5), want_traj=True)
    assert traj.max() - traj.min() > 0.5


def test_phase1_over_pieces_with_retention_per_coordinate():
    """The sweeps over pieces of the sequence (forced: 4 pieces per chain over 12 chunks) compose
    the piece maps with one retention per coordinate."""
    B, T, H, K, V = 1, 64 * 12, 2, 128, 64
    x = _inputs(B, T, H, K, V, seed=75, bf16=False)
    hp = ob.Hyper(eta=0.5, p1_pieces=4)
    compare_forward(x, hp, False)
    compare_backward(x, hp, False)


def test_equal_entries_reproduce_the_scalar_gate_bitwise():
    B, T, H, K, V = 2, 128, 2, 128, 64
    x = make_stress_inputs(B, T, H, K, V, seed=73, bf16=True, retention=0.95)
    hp = ob.Hyper(eta=0.5)
    t = to_dev(x, True)
    rv = t["retention"][..., None].expand(B, T, H, K).contiguous()
    a = ob.forward(t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], t["retention"], t["d_in"], t["S_in"], hp,
                   for_backward=True)
    b = ob.forward(t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], rv, t["d_in"], t["S_in"], hp,
                   for_backward=True)
    ga, gb = ob.backward(a[3], t["dO"]), ob.backward(b[3], t["dO"])
    torch.cuda.synchronize()
    for u, v in zip(a[:3], b[:3]):
        assert torch.equal(u, v)
    for name in ga:
        if name == "dretention":
            assert gb[name].shape == (B, T, H, K)
            ref = ga[name].double()
            assert (gb[name].double().sum(-1) - ref).abs().max() <= 1e-5 * ref.abs().max()
        else:
            assert torch.equal(ga[name], gb[name]), name


def test_precond_update_and_step():
    for bf16 in (False, True):
        x = _inputs(2, 40, 3, 128, 64, seed=74, bf16=bf16)
        t = to_dev(x, bf16)
        hp = ob.Hyper(eta=0.7)
        kt, d_out = ob.precond_update(t["k"], t["beta"], t["retention"], t["d_in"], hp)
        o, S, d = ob.step(t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], t["retention"], t["d_in"], t["S_in"], hp)
        torch.cuda.synchronize()
        okt, od = oracle.precond(x["k"], x["beta"], x["retention"], x["d_in"], oracle_hp(hp))
        check("k_tilde", kt, okt, bf16)
        check("d_out", d_out, od, False)
        y = f64(x)
        oo, oS, od2 = oracle.fwd(y["q"], y["k"], y["v"], y["beta"], y["log_alpha"], y["retention"], y["d_in"],
                                 y["S_in"], oracle_hp(hp))
        check("o", o, oo, bf16)
        check("S_out", S, oS, bf16)
        check("d_out(step)", d, od2, False)


def test_packed_sequences():
    """Per-coordinate retention on a packed axis of ragged sequences, against the oracle run on
    every sequence alone."""
    from tests.test_gpu_packed import _cu, _gpu_packed, _oracle_per_sequence, _packed_inputs
    lens, H, K, V, bf16, hp = [70, 1, 129, 64], 2, 64, 64, False, ob.Hyper(eta=0.5)
    x = _packed_inputs(lens, H, K, V, seed=75, bf16=bf16)
    rng = np.random.default_rng(76)
    x["retention"] = np.clip(x["retention"][..., None] + 0.04 * rng.standard_normal((1, sum(lens), H, K)),
                             0.0, 1.0).astype(np.float32)
    got, _ = _gpu_packed(x, lens, hp, bf16, backward=True)
    ref = _oracle_per_sequence(x, lens, hp, backward=True)
    for name, r in ref.items():
        check(name, got[name], r, False)


def test_argument_errors():
    p = ob.make_params(1, 64, 1, 64, 64, False)
    p.retention_per_channel = 2
    assert ob.osdn_workspace_bytes(p, False) == 0
    k = torch.zeros(1, 64, 1, 64, device="cuda")
    with pytest.raises(ValueError):         # shape of retention must match the flag
        ob.osdn_precond_update(ob.make_params(1, 64, 1, 64, 64, False, retention_per_channel=True), k,
                               torch.zeros(1, 64, 1, device="cuda"), torch.ones(1, 64, 1, device="cuda"), None,
                               torch.empty_like(k), torch.empty(1, 1, 64, device="cuda"))
