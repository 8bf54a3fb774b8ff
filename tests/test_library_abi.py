"""CPU-side checks of the C-ABI library: it loads, exports every symbol include/osdn.h
declares, sizes its workspace, and rejects bad arguments before touching any pointer
(no compute is launched here, so no GPU is needed)."""
import ctypes
import os
import re

import pytest

from paper_2605_13473_amd import binding as ob

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "osdn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(osdn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ob.lib()
    names = _declared_symbols()
    assert {"osdn_fwd", "osdn_bwd", "osdn_precond_update", "osdn_step", "osdn_workspace_bytes",
            "osdn_fwd_packed", "osdn_bwd_packed", "osdn_workspace_bytes_packed", "osdn_strerror"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_workspace_size_and_shape_validation():
    p = ob.make_params(4, 4096, 16, 128, 128, True)
    fwd, bwd = ob.osdn_workspace_bytes(p, False), ob.osdn_workspace_bytes(p, True)
    assert 0 < fwd < bwd
    # at least k~ plus W, U, E^T and the per-chunk state
    assert fwd >= 4 * 4096 * 16 * 128 * 2 * 4
    # per-coordinate retention only matters for the padded copies of a ragged length
    assert ob.osdn_workspace_bytes(ob.make_params(4, 4096, 16, 128, 128, True, retention_per_channel=True), True) == bwd
    # a ragged length costs the padded copies of the caller's tensors on top
    q = ob.make_params(4, 4096 - 7, 16, 128, 128, True)
    assert ob.osdn_workspace_bytes(q, False) > fwd and ob.osdn_workspace_bytes(q, True) > bwd
    # H * max(K, V) must stay below 2^24 (32-bit byte offsets inside a chunk)
    for bad in (dict(T=0), dict(K=256), dict(K=96), dict(V=96), dict(chunk=32), dict(B=0), dict(H=40000, V=512)):
        q = ob.make_params(1, 128, 1, 64, 64, False)
        for k, v in bad.items():
            setattr(q, k, v)
        assert ob.osdn_workspace_bytes(q, False) == 0, bad


def test_argument_errors_before_any_pointer_is_used():
    L = ob.lib()
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    p = ob.make_params(1, 128, 1, 96, 64, False)          # K must be 64 or 128
    rc = L.osdn_fwd(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                    fake, ctypes.c_size_t(1 << 30), None)
    assert rc == -2 and "shape" in ob.osdn_strerror(rc)
    p = ob.make_params(1, 128, 1, 64, 64, False)
    p.io_dtype = 5
    assert L.osdn_fwd(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                      fake, ctypes.c_size_t(1 << 30), None) == -3
    p = ob.make_params(1, 128, 1, 64, 64, False, ob.Hyper(eta=-1.0))
    assert L.osdn_precond_update(ctypes.byref(p), fake, fake, None, None, fake, fake, None, None) == -5
    p = ob.make_params(1, 128, 1, 64, 64, False)
    p.retention_per_channel = 3                            # a flag: 0 or 1
    assert L.osdn_precond_update(ctypes.byref(p), fake, fake, None, None, fake, fake, None, None) == -5
    p = ob.make_params(1, 128, 1, 64, 64, False, gate_per_channel=True)     # then the gate is required
    assert L.osdn_fwd(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                      fake, ctypes.c_size_t(1 << 30), None) == -1
    args = [fake] * 19
    args[4] = None
    assert L.osdn_bwd(ctypes.byref(p), *args, fake, ctypes.c_size_t(1 << 30), None) == -1
    plain = ob.make_params(1, 128, 1, 64, 64, False)
    assert ob.osdn_workspace_bytes(p, False) > ob.osdn_workspace_bytes(plain, False)
    assert ob.osdn_workspace_bytes(p, True) > ob.osdn_workspace_bytes(plain, True)
    p = ob.make_params(1, 128, 1, 64, 64, False)
    assert L.osdn_fwd(ctypes.byref(p), None, fake, fake, fake, None, None, None, None, fake, fake, fake,
                      fake, ctypes.c_size_t(1 << 30), None) == -1
    # misaligned and too-small workspaces
    assert L.osdn_fwd(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                      ctypes.c_void_p(0x1010), ctypes.c_size_t(1 << 30), None) == -4
    assert L.osdn_fwd(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                      fake, ctypes.c_size_t(16), None) == -4
    # the recurrent step takes at most one chunk of tokens, and d_out apart from d_in
    p = ob.make_params(1, 65, 1, 64, 64, False)
    assert L.osdn_step(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake, None) == -2
    p = ob.make_params(1, 1, 1, 64, 64, False)
    assert L.osdn_step(ctypes.byref(p), fake, fake, fake, fake, None, None, fake, None, fake, fake, fake, None) == -1
    assert L.osdn_step(ctypes.byref(p), fake, fake, None, fake, None, None, None, None, fake, fake, fake, None) == -1
    # d_ckpt needs whole chunks
    p = ob.make_params(1, 7, 1, 64, 64, False)
    assert L.osdn_precond_update(ctypes.byref(p), fake, fake, None, None, fake, fake, fake, None) == -2
    # gradient outputs that must accompany optional inputs
    p = ob.make_params(1, 128, 1, 64, 64, False)
    args = [fake] * 19
    args[4] = fake      # log_alpha given ...
    args[15] = None     # ... but dlog_alpha missing
    assert L.osdn_bwd(ctypes.byref(p), *args, fake, ctypes.c_size_t(1 << 30), None) == -1


def test_packed_sequences_workspace_and_validation():
    p = ob.make_params(1, 128, 1, 64, 64, False)
    dense = ob.osdn_workspace_bytes(p, True)
    aligned = ob.osdn_workspace_bytes_packed(p, [0, 64, 128], True)
    assert dense <= aligned <= dense + 4096               # whole chunks: only the index tables on top
    # ragged sequences are padded to whole chunks each, and copied
    assert ob.osdn_workspace_bytes_packed(p, [0, 60, 128], True) > aligned
    # offsets must start at 0, end at T and ascend strictly (no empty sequence); packed means B == 1
    for bad in ([1, 64, 128], [0, 64, 100], [0, 64, 64, 128], [0, 128, 64, 128]):
        assert ob.osdn_workspace_bytes_packed(p, bad, True) == 0, bad
    assert ob.osdn_workspace_bytes_packed(ob.make_params(2, 128, 1, 64, 64, False), [0, 64, 128], True) == 0
    L = ob.lib()
    fake = ctypes.c_void_p(0x1000)
    cu = (ctypes.c_int32 * 3)(0, 64, 100)
    rc = L.osdn_fwd_packed(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                           cu, 2, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == -2
    rc = L.osdn_fwd_packed(ctypes.byref(p), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                           None, 2, fake, ctypes.c_size_t(1 << 30), None)
    assert rc == -1
    args = [fake] * 19
    assert L.osdn_bwd_packed(ctypes.byref(p), *args, cu, 2, fake, ctypes.c_size_t(1 << 30), None) == -2


def test_binding_rejects_cpu_tensors_and_wrong_dtypes():
    import torch
    p = ob.make_params(1, 64, 1, 64, 64, False)
    k = torch.zeros(1, 64, 1, 64)
    with pytest.raises(TypeError):
        ob.osdn_precond_update(p, k, k[..., 0], None, None, k.clone(), torch.zeros(1, 1, 64))


def test_scheduling_fields_and_mask_offset_query():
    """The scheduling knobs are plain fields of the parameter block (the library reads no
    environment variables): zeros mean "the library decides", out-of-range values are parameter
    errors reported before any pointer is used, and they never change the workspace size.  The
    diagnostic mask query is host-only and points inside the backward part of the workspace."""
    L = ob.lib()
    fake = ctypes.c_void_p(0x1000)
    base = ob.make_params(2, 4096, 2, 128, 128, True)
    assert (base.segments, base.p1_pieces, base.p1_piece_sweeps, base.p1_solved) == (0, 0, 0, 0)
    fwd, bwd = ob.osdn_workspace_bytes(base, False), ob.osdn_workspace_bytes(base, True)
    tuned = ob.make_params(2, 4096, 2, 128, 128, True, ob.Hyper(segments=3, p1_pieces=4, p1_piece_sweeps=2))
    assert (tuned.segments, tuned.p1_pieces, tuned.p1_piece_sweeps) == (3, 4, 2)
    assert ob.osdn_workspace_bytes(tuned, False) == fwd and ob.osdn_workspace_bytes(tuned, True) == bwd
    never = ob.make_params(2, 4096, 2, 128, 128, True, ob.Hyper(p1_pieces=-1, segments=1))
    assert ob.osdn_workspace_bytes(never, True) == bwd
    for bad in (dict(segments=-1), dict(p1_pieces=-2), dict(p1_piece_sweeps=-1), dict(p1_piece_sweeps=14),
                dict(p1_solved=2), dict(p1_solved=-2)):
        q = ob.make_params(2, 4096, 2, 128, 128, True, ob.Hyper(**bad))
        assert ob.osdn_workspace_bytes(q, False) == 0, bad
        assert L.osdn_fwd(ctypes.byref(q), fake, fake, fake, fake, None, None, None, None, fake, fake, fake,
                          fake, ctypes.c_size_t(1 << 40), None) == -5, bad
    off = ob.osdn_debug_mask_offset(base)
    assert fwd <= off and off % 256 == 0 and off + 2 * 2 * 64 * 128 * 8 <= bwd
    bad = ob.make_params(2, 4096, 2, 96, 128, True)
    assert ob.osdn_debug_mask_offset(bad) == 0
    # the environment is not consulted: a variable the library once read changes nothing
    os.environ["OSDN_SEGMENTS"] = "-7"
    try:
        assert ob.osdn_workspace_bytes(base, True) == bwd
    finally:
        del os.environ["OSDN_SEGMENTS"]


def test_precond_update_ignores_the_value_width():
    """osdn_precond_update has no value tensor: V takes no part in its shape checks."""
    L = ob.lib()
    fake = ctypes.c_void_p(0x1000)
    p = ob.make_params(1, 128, 40000, 64, 64, False)        # H * K * 256 < 2^32 ...
    p.V = 1 << 20                                           # ... whatever V holds
    p.eta = -1.0                                            # reaches the scalar checks: the shape passed
    assert L.osdn_precond_update(ctypes.byref(p), fake, fake, None, None, fake, fake, None, None) == -5
