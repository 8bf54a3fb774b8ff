"""The entry point that allocates nothing (osdn_fwd_noalloc: scratch in a device array that is
part of the library) against osdn_fwd with a caller workspace, through the C-ABI: two calls in a
row, the second on a smaller input, so that the second runs over what the first left in the
shared scratch."""
import ctypes

import pytest
import torch

from paper_2605_13473_amd import binding as ob
from paper_2605_13473_amd.inputs import make_stress_inputs
from tests.gpu_util import check, to_dev

pytestmark = pytest.mark.gpu


def _both(shape, bf16, seed):
    B, T, H, K, V = shape
    x = make_stress_inputs(B, T, H, K, V, seed=seed, bf16=bf16, retention=0.97)
    t = to_dev(x, bf16)
    hp = ob.Hyper(eta=0.5, segments=1)          # the same single-stream schedule on both sides
    p = ob.make_params(B, T, H, K, V, bf16, hp)
    f32 = dict(dtype=torch.float32, device="cuda")
    new = lambda: (torch.full_like(t["v"], float("nan")), torch.full((B, H, V, K), float("nan"), **f32),
                   torch.full((B, H, K), float("nan"), **f32))
    o1, S1, d1 = new()
    ws = ob.alloc_workspace(p, False)
    ob.osdn_fwd(p, t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], t["retention"], t["d_in"], t["S_in"],
                o1, S1, d1, ws)
    o2, S2, d2 = new()
    before = torch.cuda.memory_allocated()
    ob.osdn_fwd_noalloc(p, t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], t["retention"], t["d_in"], t["S_in"],
                        o2, S2, d2)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    # same kernels, same schedule, same inputs: bit for bit; and to the parity tolerance by the same helper
    for name, a, b in (("o", o1, o2), ("S_out", S1, S2), ("d_out", d1, d2)):
        assert torch.equal(a, b), name
        check(name, b, a.float().cpu().numpy().astype("float64"), bf16 and name != "d_out")
    # and against the default (pipelined) schedule of osdn_fwd, to the parity tolerance
    o3, S3, d3 = new()
    p3 = ob.make_params(B, T, H, K, V, bf16, ob.Hyper(eta=0.5))
    ob.osdn_fwd(p3, t["q"], t["k"], t["v"], t["beta"], t["log_alpha"], t["retention"], t["d_in"], t["S_in"],
                o3, S3, d3, ob.alloc_workspace(p3, False))
    torch.cuda.synchronize()
    for name, a, b in (("o", o3, o2), ("S_out", S3, S2), ("d_out", d3, d2)):
        check(name, b, a.float().cpu().numpy().astype("float64"), bf16 and name != "d_out")


@pytest.mark.parametrize("bf16", [False, True])
def test_two_calls_in_a_row_second_smaller(bf16):
    _both((2, 640, 2, 128, 128), bf16, seed=101)
    _both((1, 200, 3, 64, 64), bf16, seed=102)          # smaller, ragged: over the first call's leftovers


def test_limit_and_argument_errors():
    L = ob.lib()
    fake = ctypes.c_void_p(0x1000)
    big = ob.make_params(4, 4096, 16, 128, 128, True)
    assert ob.osdn_workspace_bytes(big, False) > (64 << 20)
    rc = L.osdn_fwd_noalloc(ctypes.byref(big), fake, fake, fake, fake, None, None, None, None, fake, fake, fake, None)
    assert rc == -4 and "workspace" in ob.osdn_strerror(rc)
    bad = ob.make_params(1, 128, 1, 96, 64, False)
    assert L.osdn_fwd_noalloc(ctypes.byref(bad), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                              None) == -2
