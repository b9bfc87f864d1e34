"""GPU: the entry points under HIP graph capture.

The library's calls only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no memory-set or copy nodes), so a forward and a backward pass can be
captured once and replayed.  Each replay here runs on fresh inputs, with eager work and a
synchronisation between replays, and is compared bit for bit with the eager calls on the
same inputs (the kernels are deterministic) and, once, with the CPU oracle.
"""
import sys

import pytest
import torch

import oracle
from paper_2405_17381_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load_library()
    binding.debug_set("lseg", 0)
    yield
    torch.cuda.synchronize()


def _draw_bf16(w, seed):
    return [x.to(torch.bfloat16) for x in synth.draw(synth.custom(w.B, w.H, w.n, w.d, w.lambdas, seed=seed, dtype="bf16"))]


@pytest.mark.parametrize("shape", [(1, 4, 5000, 128), (3, 96, 200, 128), (2, 4, 777, 64)])
def test_captured_fwd_bwd_replays_match_eager(shape):
    """la_fwd + la_bwd captured into one graph: a segmented shape (pre-pass, segment scan and block
    scans in the graph), an unsegmented one (two launches) and d = 64.  Three replays on three
    different inputs, NaN-prefilled outputs, each equal to the eager result bit for bit."""
    B, H, n, d = shape
    lam = [1.0, 0.9995, 0.97, 0.5] * (H // 4)
    w = synth.custom(B, H, n, d, lam, seed=31, dtype="bf16")
    lam = w.lambdas                                      # as float32, what the C ABI takes
    tile, L, S = binding.la_plan(B, H, n, d, binding.LA_BF16)
    _say("shape %s plan (tile, L, S) = %s" % (shape, (tile, L, S)))
    dev = torch.device("cuda:0")
    static = [torch.zeros(B, H, n, d, dtype=torch.bfloat16, device=dev) for _ in range(4)]      # Q, K, V, dO
    outs = [torch.empty(B, H, n, d, dtype=torch.bfloat16, device=dev) for _ in range(4)]        # O, dQ, dK, dV
    ws_f = torch.empty(max(1, binding.la_workspace_bytes(B, H, n, d, binding.LA_BF16, False)), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(max(1, binding.la_workspace_bytes(B, H, n, d, binding.LA_BF16, True)), dtype=torch.uint8, device=dev)

    def run():
        binding.la_fwd(static[0], static[1], static[2], lam, O=outs[0], workspace=ws_f)
        binding.la_bwd(static[0], static[1], static[2], lam, static[3], dQ=outs[1], dK=outs[2], dV=outs[3],
                       workspace=ws_b)

    # eager warm-up on a side stream: every kernel's one-time set-up happens before the capture
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    torch.cuda.synchronize()

    for rep in range(3):
        xs = _draw_bf16(w, seed=100 + rep)
        for s, x in zip(static, xs):
            s.copy_(x)                                   # eager work between the replays
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [o.clone() for o in outs]
        for o in outs:
            o.fill_(float("nan"))
        run()                                            # the same calls, eagerly, on the same inputs
        torch.cuda.synchronize()
        for nm, a, b in zip(("O", "dQ", "dK", "dV"), got, outs):
            assert not torch.isnan(a.float()).any(), (rep, nm, "replay left NaN")
            assert torch.equal(a, b), (rep, nm, "replay differs from the eager call")
        if rep == 0 and B * H * n <= 40000:
            q, k, v, g = [x.to(torch.float64).numpy() for x in xs]
            ref = (oracle.c_recurrence_fwd(q, k, v, lam),) + oracle.c_recurrence_bwd(q, k, v, lam, g)
            for nm, a, r in zip(("O", "dQ", "dK", "dV"), got, ref):
                err = oracle.rel_max_err(a.to(torch.float64).cpu().numpy(), r)
                assert err <= TOL_BF16, (nm, err)
        _say("  replay %d equals the eager calls" % rep)


def test_captured_static_scratch_forward():
    """la_fwd_static is meant for callers under graph capture: captured after one eager call (its
    first use on a device looks up the scratch's address), replayed on fresh inputs, equal to la_fwd."""
    B, H, n, d = 1, 4, 6000, 128
    lam = [1.0, 0.9995, 0.97, 0.5]
    w = synth.custom(B, H, n, d, lam, seed=32, dtype="bf16")
    lam = w.lambdas
    assert binding.la_plan(B, H, n, d, binding.LA_BF16)[2] > 1
    dev = torch.device("cuda:0")
    Q, K, V = [torch.zeros(B, H, n, d, dtype=torch.bfloat16, device=dev) for _ in range(3)]
    O = torch.empty_like(Q)
    binding.la_fwd_static(Q, K, V, lam, O)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.la_fwd_static(Q, K, V, lam, O)
    torch.cuda.synchronize()
    for rep in range(3):
        xs = _draw_bf16(w, seed=200 + rep)
        for s, x in zip((Q, K, V), xs):
            s.copy_(x)
        O.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = binding.la_fwd(Q, K, V, lam)
        torch.cuda.synchronize()
        assert torch.equal(O, ref), rep
