"""GPU checks of la_fwd_strided / la_bwd_strided: same arithmetic as la_fwd / la_bwd on tensors
that are not contiguous [B, H, n, d], so the results must match those bit for bit, and (once,
independently) the oracle within the usual tolerance."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2405_17381_amd import binding

pytestmark = pytest.mark.gpu
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _token_major(B, H, n, d, dtype, seed, packed):
    """Q, K, V as [B, H, n, d] views of token-major storage: separate [B, n, H, d] tensors, or
    one packed [B, n, 3, H, d] tensor (what a fused QKV projection writes)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    if packed:
        qkv = (torch.randn((B, n, 3, H, d), generator=g) / d ** 0.5).to(TDT[dtype]).cuda()
        views = [qkv[:, :, j].permute(0, 2, 1, 3) for j in range(3)]
    else:
        views = [(torch.randn((B, n, H, d), generator=g) / d ** 0.5).to(TDT[dtype]).cuda().permute(0, 2, 1, 3)
                 for _ in range(3)]
    dO = torch.randn((B, n, H, d), generator=g).to(TDT[dtype]).cuda().permute(0, 2, 1, 3)
    return views + [dO]


@pytest.mark.parametrize("dtype,B,H,n,d,packed,lseg", [
    ("bf16", 2, 4, 1000, 128, False, None), ("bf16", 2, 4, 1000, 128, True, 256), ("bf16", 1, 3, 333, 64, True, None),
    ("f32", 2, 2, 300, 64, False, 128), ("f32", 1, 2, 150, 128, True, None), ("bf16", 1, 16, 4096, 128, False, 1024),
])
def test_strided_equals_contiguous(dtype, B, H, n, d, packed, lseg):
    """Same arithmetic in another layout: bit-identical to la_fwd / la_bwd on contiguous copies, in
    every kernel family (bf16 at d = 128: the direct-to-LDS kernels, and behind the "staged_scan"
    switch the register-staged ones; d = 64 and fp32: their only family)."""
    lam = [1.0, 0.999, 0.97, 0.9][:H] if H <= 4 else list(np.linspace(0.9, 1.0, H))
    Q, K, V, dO = _token_major(B, H, n, d, dtype, 7000 + n + d, packed)
    assert not Q.is_contiguous()
    if lseg is not None:
        binding.debug_set("lseg", lseg)
    try:
        cont = [x.contiguous() for x in (Q, K, V, dO)]
        for staged in (0, 1):
            with binding.debug(staged_scan=staged):
                O = binding.la_fwd_strided(Q, K, V, lam)
                dQ, dK, dV = binding.la_bwd_strided(Q, K, V, lam, dO)
                Oc = binding.la_fwd(cont[0], cont[1], cont[2], lam)
                dQc, dKc, dVc = binding.la_bwd(cont[0], cont[1], cont[2], lam, cont[3])
            torch.cuda.synchronize()
            assert O.stride() == Q.stride()              # outputs default to the inputs' layout
            for nm, a, b in (("O", O, Oc), ("dQ", dQ, dQc), ("dK", dK, dKc), ("dV", dV, dVc)):
                assert torch.equal(a.contiguous(), b), (nm, "staged_scan=%d" % staged)
    finally:
        binding.debug_set("lseg", 0)


def test_strided_against_oracle_and_mixed_layouts():
    """Token-major inputs, contiguous [B, H, n, d] outputs, gradients into a packed [B, n, 3, H, d] buffer."""
    B, H, n, d = 2, 3, 500, 128
    lam = [1.0, 0.98, 0.9]
    Q, K, V, dO = _token_major(B, H, n, d, "bf16", 71, packed=True)
    O = torch.empty((B, H, n, d), dtype=torch.bfloat16, device="cuda")
    grads = torch.full((B, n, 3, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dQ, dK, dV = [grads[:, :, j].permute(0, 2, 1, 3) for j in range(3)]
    binding.la_fwd_strided(Q, K, V, lam, O=O)
    binding.la_bwd_strided(Q, K, V, lam, dO, dQ=dQ, dK=dK, dV=dV)
    torch.cuda.synchronize()
    assert torch.isfinite(grads.float()).all()           # every element of the packed buffer was written
    q, k, v, g = [x.contiguous().to(torch.float64).cpu().numpy() for x in (Q, K, V, dO)]
    ref = (oracle.c_recurrence_fwd(q, k, v, lam),) + oracle.c_recurrence_bwd(q, k, v, lam, g)
    for nm, x, r in zip(("O", "dQ", "dK", "dV"), (O, dQ, dK, dV), ref):
        assert oracle.rel_max_err(x.contiguous().to(torch.float64).cpu().numpy(), r) <= 2e-2, nm
