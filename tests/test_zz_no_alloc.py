"""la_fwd_static: la_fwd for callers that cannot allocate (HIP graph capture, serving loops).

Called through the raw C ABI.  Its kernels are la_fwd's, its segment states live in the
library's static device scratch, so its output must equal la_fwd's bit for bit, on two calls
in a row of which the second is smaller (the scratch keeps the first call's contents), and
both must meet the oracle's tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2405_17381_amd import binding, synth

pytestmark = pytest.mark.gpu


def _raw_static(Q, K, V, lam, O):
    lib = binding.load_library()
    B, H, n, d = Q.shape
    lam_arr = (ctypes.c_float * H)(*lam)
    stream = torch.cuda.current_stream().cuda_stream
    return lib.la_fwd_static(Q.data_ptr(), K.data_ptr(), V.data_ptr(), lam_arr, O.data_ptr(),
                             B, H, n, d, binding.LA_BF16 if Q.dtype == torch.bfloat16 else binding.LA_F32,
                             stream)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_static_scratch_forward_matches_la_fwd_twice_in_a_row(dtype, d):
    assert torch.cuda.is_available()
    binding.load_library()
    for name in ("lseg", "no_pair", "no_decay_skip", "f32_plain"):
        binding.debug_set(name, 0)
    lam = [1.0, 0.9995, 0.97, 0.5]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    tol = 2e-2 if dtype == "bf16" else 1e-4
    dt = binding.LA_BF16 if dtype == "bf16" else binding.LA_F32
    # first call: 8 segments per scan; second call, smaller: 3 segments, ragged tail
    for call, n in enumerate((4100, 1300)):
        print("la_fwd_static call %d: %s d=%d n=%d" % (call, dtype, d, n), flush=True)
        tile, L, S = binding.la_plan(1, 4, n, d, dt)
        assert S > 1, "the case must use the scratch"
        assert binding.la_workspace_bytes(1, 4, n, d, dt, False) <= binding.LA_STATIC_SCRATCH_BYTES
        w = synth.custom(1, 4, n, d, lam, seed=4242 + n, dtype=dtype)
        host = synth.draw(w)
        Q, K, V = [x.to(tdt).cuda().contiguous() for x in host[:3]]
        O = torch.full_like(Q, float("nan"))
        rc = _raw_static(Q, K, V, lam, O)
        assert rc == 0, binding.la_strerror(rc)
        want = binding.la_fwd(Q, K, V, lam)
        torch.cuda.synchronize()
        assert torch.isfinite(O.float()).all()
        assert torch.equal(O, want), "call %d differs from la_fwd" % call
        q, k, v = [x.to(tdt).to(torch.float64).numpy() for x in host[:3]]
        ref = oracle.c_recurrence_fwd(q, k, v, lam)
        err = oracle.rel_max_err(O.to(torch.float64).cpu().numpy(), ref)
        print("  rel err vs oracle %.3e (tol %.0e)" % (err, tol), flush=True)
        assert np.isfinite(err) and err <= tol


def test_static_scratch_forward_refuses_what_does_not_fit():
    binding.load_library()
    lam = [0.99] * 4
    Q = torch.zeros(1, 4, 70000, 128, dtype=torch.bfloat16, device="cuda")
    O = torch.full_like(Q, float("nan"))
    with binding.debug(lseg=64):                      # 1094 segments x 4 scans x 64 KiB > 64 MiB
        assert _raw_static(Q, Q, Q, lam, O) == -8
    torch.cuda.synchronize()
    assert torch.isnan(O.float()).all()                # nothing was enqueued
