"""GPU parity: the HIP path (through the C ABI) against the CPU oracle,
element by element, on the same seeded inputs.

Tolerances (max|x - ref| / max|ref| per output tensor):
  fp32 path  <= 1e-4        bf16 path  <= 2e-2 on O and on every gradient.
For bf16 the oracle consumes the bf16-rounded inputs in fp64, so the measured
error is the kernels' internal rounding only.
"""
import os
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2405_17381_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(autouse=True)
def _need_gpu_and_clean_env(monkeypatch):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()                      # fail loudly if the HIP library is missing
    binding.debug_set("lseg", 0)
    yield
    torch.cuda.synchronize()


def _to_dev(xs, dtype):
    return [x.to(TDT[dtype]).cuda().contiguous() for x in xs]


def _ref_inputs(xs, dtype):
    """What the GPU actually sees, widened to fp64."""
    return [x.to(TDT[dtype]).to(torch.float64).numpy() for x in xs]


def _run_gpu(w, xs, lseg=None):
    if lseg is not None:
        binding.debug_set("lseg", lseg)
    try:
        Q, K, V, dO = _to_dev(xs, w.dtype)
        O = binding.la_fwd(Q, K, V, w.lambdas)
        dQ, dK, dV = binding.la_bwd(Q, K, V, w.lambdas, dO)
        torch.cuda.synchronize()
    finally:
        binding.debug_set("lseg", 0)
    return [t.to(torch.float64).cpu().numpy() for t in (O, dQ, dK, dV)]


def _compare(w, got, ref, tol, label):
    names = ("O", "dQ", "dK", "dV")
    worst = 0.0
    for nm, x, r in zip(names, got, ref):
        assert np.all(np.isfinite(x)), (label, nm, "non-finite output")
        err = oracle.rel_max_err(x, r)
        worst = max(worst, err)
        # per-head error: heads differ in lambda
        for h in range(r.shape[1]):
            eh = oracle.rel_max_err(x[:, h], r[:, h])
            assert eh <= 2 * tol, (label, nm, "head", h, eh)
        assert err <= tol, (label, nm, err)
    _say("  %s: worst rel err %.3e (tol %.0e)" % (label, worst, tol))
    return worst


def _full_case(w, lseg=None, use_left_product=False):
    label = "%s B%d H%d n%d d%d %s lseg=%s" % (w.name, w.B, w.H, w.n, w.d, w.dtype, lseg)
    _say("case " + label)
    xs = synth.draw(w)
    got = _run_gpu(w, xs, lseg)
    q, k, v, g = _ref_inputs(xs, w.dtype)
    if use_left_product:
        ref = (oracle.left_product_fwd(q, k, v, w.lambdas),) + oracle.left_product_bwd(q, k, v, w.lambdas, g)
    else:
        ref = (oracle.c_recurrence_fwd(q, k, v, w.lambdas),) + oracle.c_recurrence_bwd(q, k, v, w.lambdas, g)
    return _compare(w, got, ref, TOL[w.dtype], label)


# ---- configs[0]: fp32, B=1 H=2 n=256 d=64, lambda = (1.0, 0.99), block size 64 ------
def test_c1_fp32_against_both_oracle_forms():
    w = synth.workload("c1")
    assert binding.la_plan(w.B, w.H, w.n, w.d, binding.LA_F32)[0] == 64
    _full_case(w)
    _full_case(w, use_left_product=True)
    _full_case(w, lseg=64)          # four segments of one block each


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n,lseg", [(1, None), (63, None), (200, None), (333, 128), (512, 64)])
def test_fp32_ragged_and_segmented(d, n, lseg):
    lam = [1.0, 0.99, 0.5, 0.05, 1e-6]
    w = synth.custom(2, len(lam), n, d, lam, seed=1000 + n + d, dtype="f32")
    _full_case(w, lseg)


# ---- bf16 ----------------------------------------------------------------------------
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("n,lseg", [(1, None), (64, None), (65, None), (300, None), (1000, None),
                                    (640, 128), (1000, 256), (1337, 64)])
def test_bf16_ragged_and_segmented(d, n, lseg):
    lam = [1.0, 0.9999, 0.95, 0.6, 0.05, 1e-6]
    w = synth.custom(2, len(lam), n, d, lam, seed=2000 + n + d, dtype="bf16")
    _full_case(w, lseg)


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("n", [31, 32, 33, 95, 96, 97, 129])
def test_bf16_block_edges_of_the_direct_to_lds_kernels(n, d):
    """Sequence lengths around multiples of the 32-row block of the direct-to-LDS kernels (partial
    last block of the forward scan = partial first block of the reverse scans), whole and cut."""
    lam = [1.0, 0.999, 0.9, 0.3]
    w = synth.custom(3, len(lam), n, d, lam, seed=3100 + n, dtype="bf16")
    _full_case(w)
    if n > 64:
        _full_case(w, lseg=64)


def test_maximum_head_count_d128():
    """256 heads at d = 128: the backward pass's three-role launch carries three argument sets and
    the table of 256 decay rates in one dispatch packet."""
    H = 256
    lam = [float(0.5 + 0.5 * (h / (H - 1))) for h in range(H)]
    w = synth.custom(1, H, 100, 128, lam, seed=322, dtype="bf16")
    _full_case(w)


def test_c2_bf16_d64_full():
    _full_case(synth.workload("c2"))
    _full_case(synth.workload("c2"), lseg=512)


def test_result_independent_of_segmentation_bf16():
    """The block recurrence (App. C) makes the result independent of where
    the sequence is cut; on the GPU only the rounding may move."""
    lam = [1.0, 0.999, 0.9]
    w = synth.custom(1, 3, 2048, 128, lam, seed=77, dtype="bf16")
    xs = synth.draw(w)
    base = _run_gpu(w, xs, lseg=None)
    for lseg in (64, 512, 1024):
        other = _run_gpu(w, xs, lseg=lseg)
        for a, b in zip(base, other):
            assert oracle.rel_max_err(b, a) <= 1e-2, lseg


def test_decay_cutoff_of_the_prepass_is_invisible():
    """The segment-state pre-pass does not read rows whose decay weight is below
    2^-32 (bf16) or 2^-48 (fp32); against reading everything the fp32 state moves
    by far less than its own rounding, so outputs may differ only where that
    flips the rounding of a bf16 operand or output (2^-8 of one value)."""
    lam = [0.5, 0.9, 0.95, 0.98, 0.9999, 1.0]
    w = synth.custom(1, len(lam), 8192, 128, lam, seed=99, dtype="bf16")
    xs = synth.draw(w)
    cut = _run_gpu(w, xs, lseg=2048)
    binding.debug_set("no_decay_skip", 1)
    try:
        full = _run_gpu(w, xs, lseg=2048)
    finally:
        binding.debug_set("no_decay_skip", 0)
    for a, b in zip(cut, full):
        assert oracle.rel_max_err(a, b) <= 1e-3
        assert np.mean(a != b) <= 1e-3          # flips are rare
    q, k, v, g = _ref_inputs(xs, "bf16")
    ref = (oracle.c_recurrence_fwd(q, k, v, lam),) + oracle.c_recurrence_bwd(q, k, v, lam, g)
    _compare(w, cut, ref, TOL["bf16"], "decay cut-off, n=8192, L=2048")
    wf = synth.custom(1, len(lam), 1024, 64, lam, seed=98, dtype="f32")
    _full_case(wf, lseg=256)


def test_fp32_matrix_core_kernel_against_the_plain_fma_kernel():
    """d = 128 in fp32 runs on v_mfma_f32_32x32x2_f32; the "f32_plain" switch selects the literal FMA kernel.
    Two implementations of the same fp32 arithmetic: they differ by summation order only."""
    lam = [1.0, 0.999, 0.9, 0.3]
    w = synth.custom(2, 4, 777, 128, lam, seed=41, dtype="f32")
    xs = synth.draw(w)
    for lseg in (None, 256):
        mfma = _run_gpu(w, xs, lseg=lseg)
        binding.debug_set("f32_plain", 1)
        try:
            plain = _run_gpu(w, xs, lseg=lseg)
        finally:
            binding.debug_set("f32_plain", 0)
        for a, b in zip(mfma, plain):
            assert oracle.rel_max_err(a, b) <= 5e-6
            assert not np.array_equal(a, b)          # they really are different kernels


def test_bitwise_reproducible():
    w = synth.custom(2, 4, 1500, 128, [1.0, 0.99, 0.9, 0.5], seed=5, dtype="bf16")
    xs = synth.draw(w)
    a = _run_gpu(w, xs, lseg=256)
    b = _run_gpu(w, xs, lseg=256)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_outputs_are_fully_overwritten_and_neighbours_untouched():
    """Canaries: outputs pre-filled with NaN come back finite everywhere, and
    guard rows placed before and after each output buffer stay intact."""
    w = synth.custom(1, 2, 333, 128, [1.0, 0.97], seed=9, dtype="bf16")
    Q, K, V, dO = _to_dev(synth.draw(w), "bf16")
    n_el = Q.numel()
    guard = 4096
    bufs = []
    for _ in range(4):
        big = torch.full((n_el + 2 * guard,), float("nan"), dtype=torch.bfloat16, device="cuda")
        big[:guard] = 123.0
        big[-guard:] = 123.0
        bufs.append(big)
    outs = [b[guard:guard + n_el].view_as(Q) for b in bufs]
    binding.la_fwd(Q, K, V, w.lambdas, O=outs[0])
    binding.la_bwd(Q, K, V, w.lambdas, dO, dQ=outs[1], dK=outs[2], dV=outs[3])
    torch.cuda.synchronize()
    for big, o in zip(bufs, outs):
        assert torch.isfinite(o.float()).all()
        assert (big[:guard] == 123.0).all() and (big[-guard:] == 123.0).all()


# ---- full-size configs, in the launch configuration the benchmark times -----------------
def _full_size_case(w, chunk, slabwise=False):
    """Run the whole workload on the GPU into NaN-prefilled outputs and compare EVERY (b, h)
    scan of O, dQ, dK, dV with the compiled oracle recurrence, `chunk` scans at a time (bounds
    host memory).  Per output tensor the error is max|x - ref| / max|ref| over the whole tensor
    (<= tol); per scan it is taken against that scan's own max|ref| (<= 2 tol, heads differ in
    lambda).  The trilinearity invariant <dO,O> = <dQ,Q> = <dK,K> = <dV,V> is kept as a second,
    oracle-free check over the entire tensors, bounded tightly enough that one wrong head fails it."""
    label = "%s B%d H%d n%d d%d" % (w.name, w.B, w.H, w.n, w.d)
    tol = TOL[w.dtype]
    _say("case %s (all %d scans, %d at a time)" % (label, w.B * w.H, chunk))
    t0 = time.time()
    dt = TDT[w.dtype]
    if slabwise:
        Q, K, V, dO = synth.draw_slabwise(w, device="cuda", dtype=dt)
    else:
        Q, K, V, dO = _to_dev(synth.draw(w), w.dtype)
    _say("  inputs ready in %.1fs" % (time.time() - t0))
    outs = [torch.full_like(Q, float("nan")) for _ in range(4)]
    binding.la_fwd(Q, K, V, w.lambdas, O=outs[0])
    binding.la_bwd(Q, K, V, w.lambdas, dO, dQ=outs[1], dK=outs[2], dV=outs[3])
    torch.cuda.synchronize()
    _say("  plan (tile, L, S) = %s" % (binding.la_plan(w.B, w.H, w.n, w.d, binding.LA_BF16),))
    names = ("O", "dQ", "dK", "dV")
    for nm, t in zip(names, outs):
        assert torch.isfinite(t.float()).all(), (label, nm, "unwritten or non-finite output")
    scans = w.B * w.H
    flat_in = [x.view(scans, w.n, w.d) for x in (Q, K, V, dO)]
    flat_out = [x.view(scans, w.n, w.d) for x in outs]
    max_diff = [0.0] * 4                       # whole-tensor max|x - ref| and max|ref|
    max_ref = [0.0] * 4
    worst_scan = [(0.0, -1)] * 4               # per-scan relative error and where
    for lo in range(0, scans, chunk):
        hi = min(scans, lo + chunk)
        lam = [w.lambdas[s % w.H] for s in range(lo, hi)]
        # a chunk goes to the oracle as one batch of hi - lo "heads", each with its own lambda
        ins = [x[lo:hi].to(torch.float64).cpu().numpy()[None] for x in flat_in]
        ref = (oracle.c_recurrence_fwd(ins[0], ins[1], ins[2], lam),) + \
            oracle.c_recurrence_bwd(ins[0], ins[1], ins[2], lam, ins[3])
        for j in range(4):
            got = flat_out[j][lo:hi].to(torch.float64).cpu().numpy()[None]
            diff = np.abs(got - ref[j]).max(axis=(0, 2, 3))
            rmax = np.abs(ref[j]).max(axis=(0, 2, 3))
            max_diff[j] = max(max_diff[j], float(diff.max()))
            max_ref[j] = max(max_ref[j], float(rmax.max()))
            per = diff / np.maximum(rmax, 1e-300)
            k = int(per.argmax())
            if per[k] > worst_scan[j][0]:
                worst_scan[j] = (float(per[k]), lo + k)
            assert per[k] <= 2 * tol, (label, names[j], "scan", lo + k, "b,h", divmod(lo + k, w.H), per[k])
        if lo == 0 or hi == scans or (lo // chunk) % 8 == 0:
            _say("  scans %d..%d compared  [%.1fs]" % (lo, hi - 1, time.time() - t0))
    for j in range(4):
        err = max_diff[j] / max_ref[j]
        _say("  %-2s: rel err %.3e (tol %.0e); worst single scan %.3e at (b,h)=%s"
             % (names[j], err, tol, worst_scan[j][0], divmod(worst_scan[j][1], w.H)))
        assert err <= tol, (label, names[j], err)
    # trilinearity over everything, per head, accumulated in fp64 on the device.  The inner
    # products are sums of signed terms and can be small by cancellation, so the difference is
    # measured against the sum of |terms|: correct results give <= 1e-5 there, a head whose
    # gradient is noise of the right magnitude gives about 3e-4.
    O, dQ, dK, dV = outs

    def inner(x, y):
        return (x.double() * y.double()).sum(dim=(0, 2, 3))
    base = inner(dO, O)
    scale = (dO.double() * O.double()).abs().sum(dim=(0, 2, 3)).clamp_min(1e-30)
    for nm, gx, x in (("dQ", dQ, Q), ("dK", dK, K), ("dV", dV, V)):
        rel = ((inner(gx, x) - base).abs() / scale).max().item()
        _say("  <%s,%s> vs <dO,O>: %.2e of sum|terms|" % (nm, nm[1:], rel))
        assert rel <= 5e-5, (label, nm, rel)
    _say("  done in %.1fs" % (time.time() - t0))


@pytest.mark.parametrize("n", [2048, 4096, 8192, 16384, 32768, 65536])
def test_c3_sweep_point_every_scan(n):
    _full_size_case(synth.workload("c3_%d" % n), chunk=16)


def test_c2_layer_at_65536_tokens_every_scan():
    """C2's layer shape (d = 64, strong decay) at the size the benchmark's `c2_at_64k_tokens` entry times:
    32 x 32 scans of 2048 tokens, unsegmented, every scan against the oracle."""
    import math
    w = synth.custom(32, 32, 2048, 64, [math.exp(-(h + 1) / 32.0) for h in range(32)], seed=20240599,
                     dtype="bf16", name="c2_at_64k_tokens")
    _full_size_case(w, chunk=32)


def test_c4_silu_features_every_scan():
    _full_size_case(synth.workload("c4"), chunk=16)


def test_c5_long_context_every_scan():
    # 16 heads with lambda = 1 (no decay over 2048 blocks) and 16 slowly decaying ones
    _full_size_case(synth.workload("c5"), chunk=4, slabwise=True)


# ---- planner and limits --------------------------------------------------------------------
def test_maximum_head_count():
    H = 256
    lam = [float(0.5 + 0.5 * (h / (H - 1))) for h in range(H)]          # 0.5 .. 1.0
    w = synth.custom(1, H, 130, 64, lam, seed=321, dtype="bf16")
    _full_case(w)


@pytest.mark.parametrize("dtype,d,n", [("bf16", 128, 5000), ("f32", 64, 3000)])
def test_planner_segments_a_small_batch_by_itself(dtype, d, n):
    """Few scans: the planner cuts the sequences without any override."""
    lam = [1.0, 0.995, 0.9]
    dt = binding.LA_BF16 if dtype == "bf16" else binding.LA_F32
    tile, L, S = binding.la_plan(1, 3, n, d, dt)
    assert S > 1 and L >= 512
    w = synth.custom(1, 3, n, d, lam, seed=654 + n, dtype=dtype)
    _full_case(w)


@pytest.mark.parametrize("dtype,d,n,lseg", [("bf16", 128, 5000, None), ("bf16", 64, 1500, 256), ("f32", 128, 700, 128),
                                             ("f32", 64, 900, 256), ("bf16", 128, 300, None)])
def test_backward_reusing_the_forward_states(dtype, d, n, lseg):
    """la_bwd_saved takes the segment states la_fwd left in its workspace instead of recomputing
    them: same gradients as la_bwd (up to the rounding order of those states), and the oracle's."""
    lam = [1.0, 0.9995, 0.98, 0.6]
    w = synth.custom(1, 4, n, d, lam, seed=900 + n, dtype=dtype)
    xs = synth.draw(w)
    if lseg is not None:
        binding.debug_set("lseg", lseg)
    try:
        Q, K, V, dO = _to_dev(xs, dtype)
        dt = binding.LA_BF16 if dtype == "bf16" else binding.LA_F32
        need = binding.la_workspace_bytes(w.B, w.H, n, d, dt, False)
        fws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        O = binding.la_fwd(Q, K, V, w.lambdas, workspace=fws)
        keep = fws.clone()
        got = binding.la_bwd_saved(Q, K, V, w.lambdas, dO, fws if need else None)
        plain = binding.la_bwd(Q, K, V, w.lambdas, dO)
        torch.cuda.synchronize()
    finally:
        binding.debug_set("lseg", 0)
    assert torch.equal(fws, keep)                        # the forward workspace is only read
    q, k, v, g = _ref_inputs(xs, dtype)
    ref = oracle.c_recurrence_bwd(q, k, v, w.lambdas, g)
    for nm, a, b, r in zip(("dQ", "dK", "dV"), got, plain, ref):
        a64, b64 = a.double().cpu().numpy(), b.double().cpu().numpy()
        assert oracle.rel_max_err(a64, r) <= TOL[dtype], nm
        assert oracle.rel_max_err(a64, b64) <= (1e-5 if dtype == "f32" else 4e-3), nm
    assert torch.equal(got[1], plain[1]) and torch.equal(got[2], plain[2])     # dK, dV: same code path


def test_very_long_sequence_many_segments():
    """One batch, two heads, 300 000 tokens: the planner cuts each scan into about 250 segments
    (a ragged last one); lambda = 1 accumulates over all of them."""
    lam = [1.0, 0.9999]
    n = 300_000
    w = synth.custom(1, 2, n, 128, lam, seed=5, dtype="bf16")
    tile, L, S = binding.la_plan(1, 2, n, 128, binding.LA_BF16)
    assert S > 200 and n % L != 0
    _say("plan (tile, L, S) = %s" % ((tile, L, S),))
    _full_case(w)


@pytest.mark.parametrize("d", [128, 64])
def test_direct_to_lds_and_register_staged_block_scans_agree(d):
    """bf16 has two block-scan kernel families: the direct-to-LDS one (32-row blocks, the
    default) and the register-staged one (64-row blocks, "staged_scan" switch).  Same arithmetic
    up to block length and rounding points: they agree with each other far inside the tolerance,
    each agrees with the oracle, and they are different code (outputs not bit-identical)."""
    lam = [1.0, 0.9995, 0.97, 0.5]
    w = synth.custom(2, 4, 1337, d, lam, seed=4711, dtype="bf16")
    xs = synth.draw(w)
    q, k, v, g = _ref_inputs(xs, "bf16")
    ref = (oracle.c_recurrence_fwd(q, k, v, lam),) + oracle.c_recurrence_bwd(q, k, v, lam, g)
    for lseg in (None, 256):
        direct = _run_gpu(w, xs, lseg=lseg)
        binding.debug_set("staged_scan", 1)
        try:
            staged = _run_gpu(w, xs, lseg=lseg)
        finally:
            binding.debug_set("staged_scan", 0)
        _compare(w, direct, ref, TOL["bf16"], "direct-to-LDS, lseg=%s" % lseg)
        _compare(w, staged, ref, TOL["bf16"], "register-staged, lseg=%s" % lseg)
        for a, b in zip(direct, staged):
            assert oracle.rel_max_err(a, b) <= 1e-2
            assert not np.array_equal(a, b)
        # the backward pass's block scans as two launches (dQ, then the dK / dV pair) instead of one
        # launch of three roles: the same instructions on the same data, so the same bits
        with binding.debug(no_trio=1):
            split = _run_gpu(w, xs, lseg=lseg)
        for a, b in zip(direct, split):
            assert np.array_equal(a, b)


def test_prepass_wave_group_counts_agree():
    """The direct-to-LDS segment-state pre-pass splits a segment's blocks over G groups of four
    waves and adds the groups' partial states at the end (G = 4; 1 and 2 behind the
    "prepass_groups" switch).  Every count gives the oracle's result within the tolerance, with a
    ragged last block, a ragged last segment, segments shorter than G blocks, and a quickly
    decaying head whose cut-off leaves fewer blocks than groups; counts differ only by rounding
    order."""
    lam = [1.0, 0.9995, 0.97, 0.5]
    for n, lseg in ((1337, 256), (1000, 64), (4099, 2048)):
        w = synth.custom(2, 4, n, 128, lam, seed=99 + n, dtype="bf16")
        xs = synth.draw(w)
        q, k, v, g = _ref_inputs(xs, "bf16")
        ref = (oracle.c_recurrence_fwd(q, k, v, lam),) + oracle.c_recurrence_bwd(q, k, v, lam, g)
        runs = {}
        for groups in (4, 2, 1):
            _say("n=%d lseg=%d groups=%d" % (n, lseg, groups))
            with binding.debug(prepass_groups=0 if groups == 4 else groups):
                runs[groups] = _run_gpu(w, xs, lseg=lseg)
            _compare(w, runs[groups], ref, TOL["bf16"], "n=%d lseg=%d groups=%d" % (n, lseg, groups))
        for groups in (2, 1):
            for a, b in zip(runs[4], runs[groups]):
                assert oracle.rel_max_err(a, b) <= 8e-3          # a bf16 rounding step of the largest element


def _random_case(i):
    """Case i of a fixed pseudo-random list: shapes, decay rates and segment lengths nobody chose by hand."""
    rng = np.random.default_rng(9000 + i)
    dtype = ("bf16", "bf16", "f32")[i % 3]
    d = (128, 64)[(i // 3) % 2]
    B = int(rng.integers(1, 4))
    H = int(rng.integers(1, 7))
    n = int(rng.integers(1, 1600 if dtype == "bf16" else 700))
    kind = rng.random(H)
    lam = [1.0 if k < 0.15 else float(1.0 - 10.0 ** rng.uniform(-4.0, -0.3)) for k in kind]
    lseg = (None, 64, 128, 192, 512)[int(rng.integers(0, 5))]
    return dtype, d, B, H, n, lam, lseg


@pytest.mark.parametrize("i", range(24))
def test_pseudo_random_shapes(i):
    """24 seeded draws of (dtype, d, B, H, n, decay rates in (0.5, 1], forced segment length):
    O and all gradients against the oracle's recurrence."""
    dtype, d, B, H, n, lam, lseg = _random_case(i)
    _say("case %d: %s d=%d B=%d H=%d n=%d lseg=%s lambda=%s" % (i, dtype, d, B, H, n, lseg, ["%.5f" % x for x in lam]))
    w = synth.custom(B, H, n, d, lam, seed=9100 + i, dtype=dtype)
    xs = synth.draw(w)
    q, k, v, g = _ref_inputs(xs, dtype)
    ref = (oracle.c_recurrence_fwd(q, k, v, w.lambdas),) + oracle.c_recurrence_bwd(q, k, v, w.lambdas, g)
    got = _run_gpu(w, xs, lseg=lseg)
    _compare(w, got, ref, TOL[dtype], "case %d" % i)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_extreme_decay_rates(dtype, d):
    """Decay rates from 1e-6 (every power beyond the first few underflows to zero) to 1 (no decay) in one
    call, with and without forced segments: finite results, equal to the oracle within the tolerance."""
    lam = [1e-6, 1e-2, 0.2, 1.0]
    for n, lseg in ((300, None), (777, 128)):
        w = synth.custom(2, 4, n, d, lam, seed=4242 + n + d, dtype=dtype)
        xs = synth.draw(w)
        q, k, v, g = _ref_inputs(xs, dtype)
        ref = (oracle.c_recurrence_fwd(q, k, v, w.lambdas),) + oracle.c_recurrence_bwd(q, k, v, w.lambdas, g)
        got = _run_gpu(w, xs, lseg=lseg)
        _compare(w, got, ref, TOL[dtype], "%s d=%d n=%d lseg=%s" % (dtype, d, n, lseg))


def test_tensors_beyond_2_to_the_31_elements():
    """64 heads x 270 000 tokens x 128 features = 2.2e9 elements (4.4 GB) per tensor: element offsets
    of the later heads do not fit 32 bits.  Inputs drawn on the device; the first head, the head
    that straddles 2^31 elements and the last head are compared with the oracle over their whole
    length, O and all gradients; every output is checked to be fully written."""
    B, H, n, d = 1, 64, 270_000, 128
    assert H * n * d > 2 ** 31
    lam = [float(np.float32(0.9 + 0.0999 * h / (H - 1))) for h in range(H)]
    gen = torch.Generator(device="cuda").manual_seed(777)
    ins = [(torch.randn((B, H, n, d), generator=gen, device="cuda", dtype=torch.bfloat16) * s)
           for s in (0.088, 0.088, 0.088, 1.0)]
    outs = [torch.full((B, H, n, d), float("nan"), device="cuda", dtype=torch.bfloat16) for _ in range(4)]
    binding.la_fwd(ins[0], ins[1], ins[2], lam, O=outs[0])
    binding.la_bwd(ins[0], ins[1], ins[2], lam, ins[3], dQ=outs[1], dK=outs[2], dV=outs[3])
    torch.cuda.synchronize()
    _say("plan (tile, L, S) = %s" % (binding.la_plan(B, H, n, d, binding.LA_BF16),))
    for nm, t in zip(("O", "dQ", "dK", "dV"), outs):
        for h0 in range(0, H, 8):                        # in pieces: keeps the fp32 temporaries small
            assert not torch.isnan(t[:, h0:h0 + 8].float()).any(), (nm, "unwritten", h0)
    straddle = (2 ** 31) // (n * d)
    for h in (0, straddle, H - 1):
        q, k, v, g = [x[:, h:h + 1].to(torch.float64).cpu().numpy() for x in ins]
        ref = (oracle.c_recurrence_fwd(q, k, v, [lam[h]]),) + oracle.c_recurrence_bwd(q, k, v, [lam[h]], g)
        for nm, t, r in zip(("O", "dQ", "dK", "dV"), outs, ref):
            err = oracle.rel_max_err(t[:, h:h + 1].to(torch.float64).cpu().numpy(), r)
            _say("  head %d %s: rel err %.3e" % (h, nm, err))
            assert err <= TOL["bf16"], (h, nm, err)
