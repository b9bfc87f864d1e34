"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/la.h declares, plans deterministically and rejects bad
arguments before enqueuing anything."""
import ctypes
import os
import re

import pytest

from paper_2405_17381_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "la.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(la_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_strerror_is_distinct_per_status():
    msgs = {binding.la_strerror(s) for s in range(0, -9, -1)}
    assert len(msgs) == 9
    assert binding.la_strerror(-99) == "unknown status"


@pytest.fixture(autouse=True)
def _default_switches():
    for name in ("lseg", "no_pair", "no_decay_skip", "f32_plain"):
        binding.debug_set(name, 0)
    yield
    for name in ("lseg", "no_pair", "no_decay_skip", "f32_plain"):
        binding.debug_set(name, 0)


def test_debug_switches_are_exported_but_not_public(monkeypatch):
    """The test / tuning switches live behind la_debug_set (csrc/la_debug.h), are absent from the
    public header, and the environment is never read."""
    lib = binding.load_library()
    for name in binding.DEBUG_EXPORTS:
        assert getattr(lib, name) is not None
        assert name not in _declared_symbols()
    assert binding.debug_get("lseg") == 0
    binding.debug_set("lseg", 128)
    assert binding.debug_get("lseg") == 128
    with pytest.raises(binding.LaError):
        binding.debug_set("no_such_switch", 1)
    assert binding.debug_get("no_such_switch") == -1
    binding.debug_set("lseg", 0)
    base = binding.la_plan(1, 2, 3000, 64, binding.LA_BF16)
    monkeypatch.setenv("LA_LSEG", "128")
    assert binding.la_plan(1, 2, 3000, 64, binding.LA_BF16) == base


def test_plan_and_workspace():
    # many scans: one segment, no scratch
    tile, L, S = binding.la_plan(32, 16, 2048, 128, binding.LA_BF16)
    assert (tile, S) == (32, 1) and L >= 2048
    assert binding.la_workspace_bytes(32, 16, 2048, 128, binding.LA_BF16, False) == 0
    # few scans, long sequence: segmented, scratch = scans * S * d*d * 4
    tile, L, S = binding.la_plan(1, 16, 65536, 128, binding.LA_BF16)
    assert S > 1 and L % tile == 0 and (S - 1) * L < 65536 <= S * L
    need = binding.la_workspace_bytes(1, 16, 65536, 128, binding.LA_BF16, False)
    assert need == 16 * S * 128 * 128 * 4
    # backward keeps forward states of (V,K) and reverse states of (dO,Q) side by side
    assert binding.la_workspace_bytes(1, 16, 65536, 128, binding.LA_BF16, True) == 2 * need
    # fp32 tile lengths
    assert binding.la_plan(1, 2, 256, 64, binding.LA_F32)[0] == 64
    assert binding.la_plan(1, 2, 256, 128, binding.LA_F32)[0] == 32
    # override
    with binding.debug(lseg=128):
        assert binding.la_plan(1, 2, 300, 64, binding.LA_BF16) == (32, 128, 3)
        with binding.debug(staged_scan=1):               # the register-staged family: 64-row blocks
            assert binding.la_plan(1, 2, 300, 64, binding.LA_BF16) == (64, 128, 3)
    # invalid problem: no scratch, error status from the plan
    assert binding.la_workspace_bytes(1, 1, 16, 96, binding.LA_BF16, False) == 0
    with pytest.raises(binding.LaError):
        binding.la_plan(1, 1, 16, 96, binding.LA_BF16)


def _raw_fwd(Q=4096, K=4096, V=4096, lam=(0.5,), O=4096, B=1, H=1, n=8, d=64, dt=1, ws=0, wsb=0):
    lib = binding.load_library()
    lam_arr = (ctypes.c_float * max(1, len(lam)))(*lam) if lam is not None else None
    return lib.la_fwd(Q, K, V, lam_arr, O, B, H, n, d, dt, ws, wsb, None)


def test_bad_arguments_are_rejected_without_a_gpu():
    """Every rejection happens before any HIP call, so fake (never
    dereferenced) pointers are enough to drive the checks."""
    assert _raw_fwd(d=96) == -2
    assert _raw_fwd(n=0) == -2
    assert _raw_fwd(H=257, lam=(0.5,) * 257) == -2
    assert _raw_fwd(n=2 ** 31 - 1) == -2                        # beyond LA_MAX_SEQ_LEN
    assert _raw_fwd(n=2 ** 30) == -2
    assert binding.la_workspace_bytes(1, 1, 2 ** 31 - 1, 64, binding.LA_BF16, False) == 0
    assert _raw_fwd(dt=7) == -3
    assert _raw_fwd(Q=0) == -1
    assert _raw_fwd(lam=None) == -1
    assert _raw_fwd(Q=4100) == -7
    for bad in (0.0, -0.1, 1.5, float("nan"), float("inf")):
        assert _raw_fwd(lam=(bad,)) == -4
    # segmented plan without scratch
    binding.debug_set("lseg", 64)
    assert _raw_fwd(n=256, ws=0, wsb=0) == -5
    assert _raw_fwd(n=256, ws=4096 + 8, wsb=1 << 30) == -5      # misaligned
    assert _raw_fwd(n=256, ws=4096, wsb=16) == -5               # too small
    lib = binding.load_library()
    lam_arr = (ctypes.c_float * 1)(0.5)
    assert lib.la_bwd(4096, 4096, 4096, lam_arr, 4096, 4096, 4096, 0,
                      1, 1, 8, 64, 1, 0, 0, None) == -1
    # more (scan, segment) workgroups than a grid can hold
    lam16 = (ctypes.c_float * 16)(*([0.5] * 16))
    assert lib.la_fwd(4096, 4096, 4096, lam16, 4096, 4000, 16, 1 << 20, 64, 1, 4096, 1 << 62, None) == -2


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 1, 8, 64)
    with pytest.raises(ValueError):
        binding.la_fwd(x, x, x, [0.5])


def test_inference_and_output_stage_entry_points_reject_bad_arguments():
    """la_fwd_state, la_decode_step, la_gate_norm_*: every rejection precedes any HIP call."""
    lib = binding.load_library()
    lam = (ctypes.c_float * 1)(0.5)
    P = 4096
    # la_fwd_state: misaligned state pointers, bad shape
    assert lib.la_fwd_state(P, P, P, lam, P, P + 4, 0, 1, 1, 8, 64, 1, 0, 0, None) == -7
    assert lib.la_fwd_state(P, P, P, lam, P, 0, P + 8, 1, 1, 8, 64, 1, 0, 0, None) == -7
    assert lib.la_fwd_state(P, P, P, lam, P, 0, 0, 1, 1, 8, 32, 1, 0, 0, None) == -2
    # la_decode_step: missing state, bad lambda, bad dtype
    assert lib.la_decode_step(P, P, P, lam, 0, P, 1, 1, 64, 1, None) == -1
    bad = (ctypes.c_float * 1)(2.0)
    assert lib.la_decode_step(P, P, P, bad, P, P, 1, 1, 64, 1, None) == -4
    assert lib.la_decode_step(P, P, P, lam, P, P, 1, 1, 64, 5, None) == -3
    # gate / norm stage: null, negative or non-finite eps, batch beyond the grid limit
    assert lib.la_gate_norm_fwd(P, 0, P, 0.0, 1, 1, 8, 64, 1, None) == -1
    assert lib.la_gate_norm_fwd(P, P, P, -1.0, 1, 1, 8, 64, 1, None) == -4
    assert lib.la_gate_norm_fwd(P, P, P, float("nan"), 1, 1, 8, 64, 1, None) == -4
    assert lib.la_gate_norm_fwd(P, P, P, 0.0, 70000, 1, 8, 64, 1, None) == -2
    assert lib.la_gate_norm_bwd(P, P, P, P, 0, 0.0, 1, 1, 8, 64, 1, None) == -1
    assert lib.la_gate_norm_bwd(P, P, P, P + 2, P, 0.0, 1, 1, 8, 64, 1, None) == -7
    # fused-activation entry points share the checks of la_fwd / la_bwd
    assert lib.la_fwd_swish(P, P, P, lam, 0, 1, 1, 8, 64, 1, 0, 0, None) == -1
    assert lib.la_fwd_swish(P, P, P, lam, P, 1, 1, 8, 96, 1, 0, 0, None) == -2
    assert lib.la_bwd_swish(P, P, P, lam, P, P, P + 4, P, 1, 1, 8, 64, 1, 0, 0, None) == -7
    # wide query / key feature: dk must be a multiple (1..4) of dv, dv in {64, 128}
    assert lib.la_fwd_wide(P, P, P, lam, P, 1, 1, 8, 96, 64, 1, 0, 0, None) == -2
    assert lib.la_fwd_wide(P, P, P, lam, P, 1, 1, 8, 640, 128, 1, 0, 0, None) == -2
    assert lib.la_fwd_wide(P, P, P, lam, P, 1, 1, 8, 64, 32, 1, 0, 0, None) == -2
    assert lib.la_fwd_wide(0, P, P, lam, P, 1, 1, 8, 128, 64, 1, 0, 0, None) == -1
    assert lib.la_bwd_wide(P, P, P, lam, P, P, 0, P, 1, 1, 8, 128, 64, 1, 0, 0, None) == -1
    # LRPE-d rotation: scratch query is host arithmetic; missing / small scratch, too many scans
    assert lib.la_lrpe_workspace_bytes(2, 3, 300, 64) == 2 * 3 * 3 * 64 * 4
    assert lib.la_lrpe_workspace_bytes(2, 3, 300, 96) == 0
    assert lib.la_lrpe_rotate_fwd(P, 0, P, 1, 1, 8, 64, 1, None) == -1
    assert lib.la_lrpe_rotate_fwd(P, P, P, 300, 300, 8, 64, 1, None) == -2
    assert lib.la_lrpe_rotate_bwd(P, P, P, P, P, 0, 0, 0, 1, 1, 8, 64, 1, None) == -5
    assert lib.la_lrpe_rotate_bwd(P, P, P, P, P, 0, P, 16, 1, 1, 8, 64, 1, None) == -5
    assert lib.la_lrpe_rotate_bwd(P, P, P, P, 0, 0, P, 1 << 20, 1, 1, 8, 64, 1, None) == -1
    # strided layouts: strides in multiples of 8 elements, rows at least d apart
    good = binding.LaLayout(8 * 64 * 2, 64, 2 * 64)
    short = binding.LaLayout(8 * 64, 64, 32)
    odd = binding.LaLayout(8 * 64 * 2 + 4, 64, 2 * 64)
    ref = ctypes.byref
    assert lib.la_fwd_strided(P, P, P, lam, P, ref(good), None, 1, 2, 8, 64, 1, 0, 0, None) == -1
    assert lib.la_fwd_strided(P, P, P, lam, P, ref(short), ref(good), 1, 2, 8, 64, 1, 0, 0, None) == -2
    assert lib.la_fwd_strided(P, P, P, lam, P, ref(good), ref(odd), 1, 2, 8, 64, 1, 0, 0, None) == -7
    assert lib.la_bwd_strided(P, P, P, lam, P, P, P, P, ref(good), ref(good), ref(short), 1, 2, 8, 64, 1, 0, 0, None) == -2
    # la_bwd_saved: a segmented problem needs the forward workspace
    with binding.debug(lseg=64):
        assert lib.la_bwd_saved(P, P, P, lam, P, P, P, P, 0, 1, 1, 256, 64, 1, P, 1 << 30, None) == -5
        assert lib.la_bwd_saved(P, P, P, lam, P, P, P, P, P + 8, 1, 1, 256, 64, 1, P, 1 << 30, None) == -5
    # la_fwd_static: a problem whose segment states exceed the static scratch is refused; bad
    # arguments are refused as in la_fwd (all before any HIP call)
    lam16 = (ctypes.c_float * 16)(*([0.9] * 16))
    with binding.debug(lseg=512):
        assert binding.la_workspace_bytes(2, 16, 131072, 128, 1, False) > binding.LA_STATIC_SCRATCH_BYTES
        assert lib.la_fwd_static(P, P, P, lam16, P, 2, 16, 131072, 128, 1, None) == -8
    # ... while every plan the library makes by itself fits
    for (B, H, n) in ((2, 16, 131072), (1, 255, 10 ** 6), (5, 51, 2 * 10 ** 6), (1, 1, 2 ** 30 - 1)):
        assert binding.la_workspace_bytes(B, H, n, 128, 1, False) <= binding.LA_STATIC_SCRATCH_BYTES
    assert lib.la_fwd_static(P, P, P, lam, P, 1, 1, 8, 96, 1, None) == -2
    assert lib.la_fwd_static(0, P, P, lam, P, 1, 1, 8, 64, 1, None) == -1
    assert lib.la_fwd_static(P, P + 2, P, lam, P, 1, 1, 8, 64, 1, None) == -7


def test_planner_properties():
    """For any valid shape: the segment length is a multiple of the tile, the segments cover the
    sequence exactly, many scans are never cut, few scans are cut until two workgroups per compute
    unit exist (or the 512-token floor is reached), and the scratch query matches the plan."""
    import random
    rng = random.Random(7)
    for _ in range(400):
        B = rng.choice([1, 2, 3, 8, 31, 64, 300])
        H = rng.choice([1, 2, 7, 16, 32, 256])
        n = rng.choice([1, 63, 64, 65, 511, 512, 513, 2048, 5000, 65536, 131072, 1000003])
        d = rng.choice([64, 128])
        dt = rng.choice([binding.LA_F32, binding.LA_BF16])
        tile, L, S = binding.la_plan(B, H, n, d, dt)
        assert tile in (32, 64) and L % tile == 0 and S >= 1
        assert (S - 1) * L < n <= S * L
        scans = B * H
        if scans >= 256:
            assert S == 1
        elif S > 1:
            assert L >= 512
            # (rounding the segment length up to the tile costs a few segments at most)
            assert scans * S >= 480 or L < 512 + tile
        need = binding.la_workspace_bytes(B, H, n, d, dt, False)
        assert need == (scans * S * d * d * 4 if S > 1 else 0)
        assert binding.la_workspace_bytes(B, H, n, d, dt, True) == 2 * need
