#!/usr/bin/env python3
"""Benchmark: Lightning Attention fwd+bwd tokens/s on one MI355X.

Workload (`config.workload`): the bf16 sequence-length sweep at a fixed 65 536
tokens per batch, H=16, d=128, (B, n) in {(32,2K) ... (1,64K)}, per-head decay
geometric in [0.9, 0.9999].  One "step" is one forward + one backward pass of
the whole hot path at each of the six sweep points; `value` is total tokens
per second over the timed steps, with inputs resident in HBM.

Besides the headline the JSON line carries per-point figures (`sweep`), the
roofline of the dominant kernel (`roofline`) and the CPU oracle timed on the
host cores (`cpu_baseline`).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
H, D, TOKENS = 16, 128, 65536
POINTS = [(32, 2048), (16, 4096), (8, 8192), (4, 16384), (2, 32768), (1, 65536)]
# model flops per token per head, fwd + bwd, Alg. 5/6 at block length = d: 8d^2 + 22d^2
MODEL_FLOPS_PER_TOKEN_HEAD = 30 * D * D


def executed_flops_per_token_head(d, bk):
    """Matrix-core flops the bf16 kernels issue per token and head, fwd + bwd: four scans, each
    scores 2 bk d (the whole bk x bk tile of a 32-row block; three of four 32 x 32 tiles of a
    64-row block), intra 2 bk d (same tiles), inter 2 d^2 and state update 2 d^2."""
    tiles = 1.0 if bk == 32 else 0.75
    return 4 * (2 * tiles * 2 * bk * d + 4 * d * d)


def read_traffic_note():
    """HBM bytes per launch of the dominant kernel measured with rocprofv3
    --pmc (FETCH_SIZE, WRITE_SIZE), if a summary has been committed."""
    path = os.path.join(ROOT, "profiles", "scan_bf16_d128_c3_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].strip())
    except OSError:
        pass
    return None


def cpu_baseline():
    """The CPU oracle (compiled token recurrence, fp64, OpenMP over scans), as
    it stands, on a bounded sample of the same workload: the seeded (B=1, n=65536) sweep
    point of `synth`, rounded to bf16 as the GPU sees it."""
    import torch
    import oracle
    from paper_2405_17381_amd import synth
    w = synth.workload("c3_65536")
    xs = [x.to(torch.bfloat16).to(torch.float64).numpy() for x in synth.draw(w)]
    threads = oracle.oracle_threads()
    t0 = time.perf_counter()
    oracle.c_recurrence_fwd(xs[0], xs[1], xs[2], w.lambdas)
    oracle.c_recurrence_bwd(xs[0], xs[1], xs[2], w.lambdas, xs[3])
    dt = time.perf_counter() - t0
    return {
        "value": w.n / dt, "unit": "tokens/s", "cores": min(threads, H), "kind": "oracle",
        "sample": "the whole (B=1, n=65536) sweep point (one batch of 65536 tokens), all 16 heads, "
                  "d=128, seeded inputs of the test-suite's workload c3_65536, fwd+bwd token recurrence "
                  "in fp64; %.1f s wall on %d OpenMP threads (one thread per head)" % (dt, threads),
    }


def ablation(binding, torch, views, lam, ws):
    """Where the block scan's time goes: the same launches with work left out.  Every variant is
    selected by a debug switch of the library (csrc/la_debug.h); variants 1-4 of "ablate" give wrong
    results by design.  Medians of 20 single calls after 5 warm-up calls; every case is measured
    twice, interleaved, to show the run-to-run spread."""
    def med(fn):
        for _ in range(5):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        torch.cuda.synchronize()
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        return round(0.5 * (ms[9] + ms[10]), 4)

    cases = [("default (direct-to-LDS scan, 32-row blocks, non-temporal result stores)", {}),
             ("la_bwd as a dQ launch + a paired dK/dV launch (not one launch of three roles)", {"no_trio": 1}),
             ("register-staged scan and pre-pass (64-row blocks)", {"staged_scan": 1}),
             ("register-staged pre-pass only", {"staged_prepass": 1}),
             ("direct-to-LDS pre-pass with one group of four waves per workgroup (not four)", {"prepass_groups": 1}),
             ("ordinary result stores", {"store_policy": 2}),
             ("ablate 1: no result stores", {"ablate": 1}),
             ("ablate 2: loads, waits and barriers only", {"ablate": 2}),
             ("ablate 3: arithmetic only (no loads, no stores)", {"ablate": 3}),
             ("ablate 4: loads, barriers and result stores, no arithmetic", {"ablate": 4})]
    out = {"protocol": "median ms of 20 calls, two interleaved rounds; fwd = la_fwd, bwd = la_bwd, "
                       "fwd_bwd = the two back to back, sweep_step_ms = one fwd+bwd at each of the six "
                       "sweep points in turn (the benchmark's step); fwd_cold_ms / bwd_cold_ms = the call timed "
                       "after an untimed read-only pass over 1 GiB of other memory, so that it finds none of "
                       "the previous call's tiles in L2 or the Infinity Cache (and no dirty lines to write "
                       "back); H=16, d=128, bf16, 65536 tokens",
           "cases": []}
    junk = torch.zeros(1 << 28, dtype=torch.int32, device=ws.device)

    def med_cold(fn):
        for _ in range(3):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        torch.cuda.synchronize()
        for e0, e1 in evs:
            junk.sum()
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        return round(0.5 * (ms[9] + ms[10]), 4)

    fns = {}
    step_fns = []
    for B, n in ((32, 2048), (16, 4096), (8, 8192), (4, 16384), (2, 32768), (1, 65536)):
        t = views(B, n)
        step_fns.append(lambda t=t: (
            binding.la_fwd(t["Q"], t["K"], t["V"], lam, O=t["O"], workspace=ws),
            binding.la_bwd(t["Q"], t["K"], t["V"], lam, t["dO"], dQ=t["dQ"], dK=t["dK"], dV=t["dV"],
                           workspace=ws)))

    def sweep_step():
        for fn in step_fns:
            fn()

    for B, n in ((32, 2048), (1, 65536)):
        t = views(B, n)
        f = lambda t=t: binding.la_fwd(t["Q"], t["K"], t["V"], lam, O=t["O"], workspace=ws)
        b = lambda t=t: binding.la_bwd(t["Q"], t["K"], t["V"], lam, t["dO"], dQ=t["dQ"], dK=t["dK"],
                                       dV=t["dV"], workspace=ws)
        fns[(B, n)] = (f, b)
    med(fns[(32, 2048)][0])                                   # clocks up before the first case
    for rnd in range(2):
        for label, sw in cases:
            with binding.debug(**sw):
                row = {"case": label, "round": rnd}
                for (B, n), (f, b) in fns.items():
                    row["B%d_n%d" % (B, n)] = {"fwd_ms": med(f), "bwd_ms": med(b),
                                               "fwd_bwd_ms": med(lambda: (f(), b())),
                                               "fwd_cold_ms": med_cold(f), "bwd_cold_ms": med_cold(b)}
                row["sweep_step_ms"] = med(sweep_step)
            out["cases"].append(row)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--point", type=int, default=0,
                    help="profiling aid: restrict the step to the sweep point with this n")
    ap.add_argument("--sweep-only", action="store_true",
                    help="profiling aid: only the sweep (headline, per-point figures, roofline); none of the "
                         "side legs, so that a kernel trace holds the sweep's launches alone")
    ap.add_argument("--debug-switch", action="append", default=[], metavar="NAME=VALUE",
                    help="measurement aid: set a debug switch of the library (csrc/la_debug.h) for the whole "
                         "run, e.g. trio=0; may be given several times; recorded in the JSON line")
    ap.add_argument("--ablation", action="store_true",
                    help="measurement aid: instead of the benchmark, time the (32, 2048) and (1, 65536) points "
                         "with parts of the block scan left out or replaced (library debug switches) and "
                         "print one JSON line")
    ap.add_argument("--calib-copy", action="store_true",
                    help="profiling aid: also run a plain 256 MiB -> 256 MiB device copy per step, "
                         "whose FETCH_SIZE / WRITE_SIZE readings calibrate the HBM counters")
    args = ap.parse_args()
    global POINTS
    all_points = list(POINTS)
    if args.point:
        POINTS = [(B, n) for (B, n) in POINTS if n == args.point]
        assert POINTS, "no sweep point with n=%d" % args.point
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the hot path is a single-GPU kernel "
              "library; no collectives). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2405_17381_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load_library()
    for kv in args.debug_switch:
        name, val = kv.split("=", 1)
        binding.debug_set(name, int(val))
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    lam = synth.workload("c3_2048").lambdas

    numel = TOKENS * H * D
    gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 3)
    scale = 1.0 / (D ** 0.5)
    flat = {}
    for name in ("Q", "K", "V"):
        flat[name] = (torch.randn(numel, generator=gen, device=dev, dtype=torch.float32) * scale).to(torch.bfloat16)
    flat["dO"] = torch.randn(numel, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    for name in ("O", "dQ", "dK", "dV"):
        flat[name] = torch.empty(numel, device=dev, dtype=torch.bfloat16)
    ws_bytes = max(binding.la_workspace_bytes(B, H, n, D, binding.LA_BF16, True) for B, n in all_points)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def views(B, n):
        return {k: v.view(B, H, n, D) for k, v in flat.items()}

    def fwd_bwd(B, n):
        t = views(B, n)
        binding.la_fwd(t["Q"], t["K"], t["V"], lam, O=t["O"], workspace=ws)
        binding.la_bwd(t["Q"], t["K"], t["V"], lam, t["dO"], dQ=t["dQ"], dK=t["dK"], dV=t["dV"], workspace=ws)

    def step():
        for B, n in POINTS:
            fwd_bwd(B, n)
        if args.calib_copy:
            # an elementwise kernel that reads 256 MiB and writes 256 MiB
            torch.add(flat["Q"], 0, out=flat["O"])

    if args.ablation:
        print(json.dumps(ablation(binding, torch, views, lam, ws)), flush=True)
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_step = TOKENS * len(POINTS)
    value = tokens_per_step * args.steps / elapsed

    # ---- per sweep point: 5 warm-up + 20 timed iterations of la_fwd, of la_bwd and of the two back to
    # back, one pair of events per iteration on the stream the kernels run on; median and minimum -------
    def per_iteration_ms(fn, warm=5, iters=20):
        for _ in range(warm):
            fn()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        torch.cuda.synchronize()
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        return 0.5 * (ms[(iters - 1) // 2] + ms[iters // 2]), ms[0]

    sweep = []
    for B, n in POINTS:
        t = views(B, n)
        f = lambda: binding.la_fwd(t["Q"], t["K"], t["V"], lam, O=t["O"], workspace=ws)
        b = lambda: binding.la_bwd(t["Q"], t["K"], t["V"], lam, t["dO"], dQ=t["dQ"], dK=t["dK"],
                                   dV=t["dV"], workspace=ws)
        f_med, f_min = per_iteration_ms(f)
        b_med, b_min = per_iteration_ms(b)
        fb_med, fb_min = per_iteration_ms(lambda: (f(), b()))
        tps = TOKENS / (fb_med * 1e-3)
        tflops = tps * H * MODEL_FLOPS_PER_TOKEN_HEAD / 1e12
        bk, L, S = binding.la_plan(B, H, n, D, binding.LA_BF16)
        ex_tflops = tps * H * executed_flops_per_token_head(D, bk) / 1e12
        sweep.append({"B": B, "n": n, "fwd_ms": round(f_med, 4), "fwd_ms_min": round(f_min, 4),
                      "bwd_ms": round(b_med, 4), "bwd_ms_min": round(b_min, 4),
                      "fwd_bwd_ms": round(fb_med, 4), "fwd_bwd_ms_min": round(fb_min, 4),
                      "tokens_per_s": round(tps, 1), "model_tflops": round(tflops, 2),
                      "pct_mfma_bf16_peak": round(100.0 * tflops / MFMA_BF16_PEAK_TFLOPS, 2),
                      "executed_tflops": round(ex_tflops, 2),
                      "pct_mfma_bf16_peak_executed": round(100.0 * ex_tflops / MFMA_BF16_PEAK_TFLOPS, 2),
                      "algorithmic_TBps": round(28 * D * H * tps / 1e12, 3),
                      "block_len": bk, "segment_len": L, "segments": S})
    rates = [p["tokens_per_s"] for p in sweep]
    near_constant = {"min_over_max_tokens_per_s": round(min(rates) / max(rates), 3),
                     "target": "north_star: near-constant from 2K to 64K; proposed bound >= 0.8 (0.9 asked later)",
                     "note": "per-point rates from the median back-to-back fwd+bwd time of 20 iterations; the "
                             "four points with fewer than 256 (batch, head) scans pay the segment-state "
                             "pre-pass (extra reads of K, V / dO, Q), the first two do not"}
    if len(sweep) >= 2:
        # time per sequence against sequence length: least-squares slope in log-log (1 = linear in n)
        import math
        xs_ = [math.log(p["n"]) for p in sweep]
        ys_ = [math.log(p["fwd_bwd_ms"] / p["B"]) for p in sweep]
        mx, my = sum(xs_) / len(xs_), sum(ys_) / len(ys_)
        near_constant["loglog_slope_time_per_sequence_vs_n"] = round(
            sum((x - mx) * (y - my) for x, y in zip(xs_, ys_)) / sum((x - mx) ** 2 for x in xs_), 4)

    # ---- roofline of the dominant kernel: the block-scan kernel -------------------
    # One launch streams three [tokens, H, d] bf16 operands in and one out:
    # 4 * 2 * d bytes per token per head.
    binding.la_profile_enable(True)
    binding.la_profile_collect()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    scan_ms, launches = binding.la_profile_collect()
    binding.la_profile_enable(False)
    # Algorithmic bytes of the block-scan launches of one fwd+bwd at one sweep point:
    # O = scan(Q,K,V) and dQ = scan(dO,V,K) each read 3 and write 1 tensor; the dK / dV
    # pair reads Q,K,V,dO once and writes 2: (4 + 4 + 6) * d * 2 B = 28 d bytes per token
    # per head, in two launches (la_fwd's scan; la_bwd's dQ, dK, dV scans as one).
    alg_bytes_per_point = 28 * D * H * TOKENS
    alg_bytes = alg_bytes_per_point * len(POINTS) * args.steps
    achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
    per_launch = alg_bytes / max(launches, 1)
    roofline = {"bound": "hbm", "kernel": "la_scan_bf16_dma (block scan, d=128: la_fwd's launch and la_bwd's three-role launch)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic_note(),
                "launches": launches, "avg_launch_ms": round(scan_ms / max(launches, 1), 5),
                "algorithmic_bytes_per_launch": round(per_launch)}

    # ---- what the memory system delivers for the same access shape, no arithmetic ----------
    # torch.addcmul streams three 256 MiB bf16 tensors in and one out, like one block scan.
    for _ in range(3):
        torch.addcmul(flat["Q"], flat["K"], flat["V"], out=flat["O"])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        torch.addcmul(flat["Q"], flat["K"], flat["V"], out=flat["O"])
    e1.record()
    e1.synchronize()
    stream_gbs = 4 * 2 * numel / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9
    roofline["measured_stream_GBps"] = round(stream_gbs, 1)
    roofline["frac_of_measured_stream"] = round(achieved / stream_gbs, 4)

    decode = gate_norm = swish_fused = lrpe = fp32_path = saved_states = other_configs = graph_replay = token_major = None
    mfma_measured = None
    if not args.sweep_only:
        # ---- decode step (next row after the training path): B=8, H=32, d=128, bf16 ----------
        # One token per (batch, head) streams the fp32 d x d state in and out: 2 * 4 d^2 bytes.
        dB, dH = 8, 32
        dlam = synth.workload("c4").lambdas
        kv = torch.zeros(dB, dH, D, D, device=dev, dtype=torch.float32)
        qkv = [(torch.randn(dB, dH, D, device=dev) * scale).to(torch.bfloat16) for _ in range(3)]
        o1 = torch.empty_like(qkv[0])
        for _ in range(10):
            binding.la_decode_step(qkv[0], qkv[1], qkv[2], dlam, kv, o=o1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        dsteps = 200
        for _ in range(dsteps):
            binding.la_decode_step(qkv[0], qkv[1], qkv[2], dlam, kv, o=o1)
        e1.record()
        e1.synchronize()
        dec_ms = e0.elapsed_time(e1) / dsteps
        dec_bytes = 2 * 4 * D * D * dB * dH
        decode = {"workload": "la_decode_step, B=8, H=32, d=128, bf16 tokens, fp32 state in place",
                  "ms_per_step": round(dec_ms, 5), "tokens_per_s": round(dB / (dec_ms * 1e-3), 1),
                  "algorithmic_bytes_per_step": dec_bytes,
                  "achieved_GBps": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
                  "note": "includes launch overhead of one small kernel per step; 32 MiB of state per step"}

        # ---- gated SRMSNorm output stage (next row): same tensors as the (1, 65536) point ---------
        tg = views(1, TOKENS)
        leg_min = {}

        def _time(fn, it=20, key=None):
            """Median of `it` single-call timings after 5 warm-up calls (the sweep's protocol); the
            minimum is kept in `leg_min` under `key`."""
            med, mn = per_iteration_ms(fn, warm=5, iters=it)
            if key:
                leg_min[key] = round(mn, 4)
            return med
        gf = _time(lambda: binding.la_gate_norm_fwd(tg["O"], tg["V"], 0.0, Y=tg["dQ"]), key="gate_norm_fwd")
        gb = _time(lambda: binding.la_gate_norm_bwd(tg["O"], tg["V"], tg["dO"], 0.0, dO=tg["dK"], dU=tg["dV"]),
                   key="gate_norm_bwd")
        tensor_bytes = 2 * numel
        gate_norm = {"workload": "Y = SRMSNorm(O) * U and its backward, [1,16,65536,128] bf16",
                     "fwd_ms": round(gf, 4), "bwd_ms": round(gb, 4),
                     "fwd_ms_min": leg_min["gate_norm_fwd"], "bwd_ms_min": leg_min["gate_norm_bwd"],
                     "fwd_GBps": round(3 * tensor_bytes / (gf * 1e-3) / 1e9, 1),
                     "bwd_GBps": round(5 * tensor_bytes / (gb * 1e-3) / 1e9, 1),
                     "note": "algorithmic bytes: 3 tensors forward, 5 backward; HBM-bound"}

        # ---- Swish of the Q, K projections fused into the scans (next row) -------------------------
        swish = []
        for sB, sn in ((32, 2048), (1, TOKENS)):
            t = views(sB, sn)
            sf = _time(lambda: binding.la_fwd_swish(t["Q"], t["K"], t["V"], lam, O=t["O"], workspace=ws), key="sf")
            sb = _time(lambda: binding.la_bwd_swish(t["Q"], t["K"], t["V"], lam, t["dO"], dQp=t["dQ"], dKp=t["dK"],
                                                    dV=t["dV"], workspace=ws), key="sb")
            swish.append({"B": sB, "n": sn, "fwd_ms": round(sf, 4), "bwd_ms": round(sb, 4),
                          "fwd_ms_min": leg_min["sf"], "bwd_ms_min": leg_min["sb"],
                          "tokens_per_s": round(TOKENS / ((sf + sb) * 1e-3), 1),
                          "algorithmic_GBps": round(16 * tensor_bytes / ((sf + sb) * 1e-3) / 1e9, 1)})
        swish_fused = {"workload": "la_fwd_swish + la_bwd_swish, H=16, d=128, bf16, 65536 tokens",
                       "points": swish,
                       "note": "algorithmic bytes: 4 tensor passes forward, 12 backward (the two pre-activation "
                               "tiles of the phi' epilogue are extra reads); separate activation kernels would "
                               "add 10 passes to the plain path's 14"}

        # ---- LRPE-d layer (next row): rotation + attention over 2d-wide query / key features ----------
        lB, ln = 1, TOKENS
        t = views(lB, ln)
        theta = torch.rand((H, D), device=dev, dtype=torch.float32)
        qw = torch.empty((lB, H, ln, 2 * D), device=dev, dtype=torch.bfloat16)
        kw = torch.empty_like(qw)
        dqw = torch.empty_like(qw)
        dkw = torch.empty_like(qw)
        dth = torch.zeros((H, D), device=dev, dtype=torch.float32)
        lws = torch.empty(max(256, binding.la_lrpe_workspace_bytes(lB, H, ln, D)), dtype=torch.uint8, device=dev)
        rot_f = _time(lambda: binding.la_lrpe_rotate_fwd(t["Q"], theta, Xw=qw))
        binding.la_lrpe_rotate_fwd(t["K"], theta, Xw=kw)
        rot_b = _time(lambda: binding.la_lrpe_rotate_bwd(t["Q"], theta, dqw, dX=t["dQ"], dtheta=dth, workspace=lws))
        wf = _time(lambda: binding.la_fwd_wide(qw, kw, t["V"], lam, O=t["O"], workspace=ws))
        wb = _time(lambda: binding.la_bwd_wide(qw, kw, t["V"], lam, t["dO"], dQw=dqw, dKw=dkw, dV=t["dV"], workspace=ws))
        # forward with the non-square state in one kernel (whole sequences only) against the two
        # accumulated scans, at the (32, 2048) shape
        tw = views(32, 2048)
        qw2, kw2 = qw.view(32, H, 2048, 2 * D), kw.view(32, H, 2048, 2 * D)
        wf_one = _time(lambda: binding.la_fwd_wide(qw2, kw2, tw["V"], lam, O=tw["O"], workspace=ws))
        with binding.debug(wide_slices=1):
            wf_two = _time(lambda: binding.la_fwd_wide(qw2, kw2, tw["V"], lam, O=tw["O"], workspace=ws))
        layer_ms = 2 * rot_f + wf + wb + 2 * rot_b
        lrpe = {"workload": "LRPE-d attention layer, [1,16,65536,128] bf16: rotate Q and K (2d-wide features), "
                            "la_fwd_wide, la_bwd_wide, rotation backward for Q and K (with the theta gradient)",
                "rotate_fwd_ms": round(rot_f, 4), "rotate_bwd_ms": round(rot_b, 4),
                "rotate_fwd_GBps": round(3 * tensor_bytes / (rot_f * 1e-3) / 1e9, 1),
                "rotate_bwd_GBps": round(4 * tensor_bytes / (rot_b * 1e-3) / 1e9, 1),
                "wide_fwd_ms": round(wf, 4), "wide_bwd_ms": round(wb, 4),
                "wide_fwd_ms_32x2048_single_kernel": round(wf_one, 4),
                "wide_fwd_ms_32x2048_two_accumulated_scans": round(wf_two, 4),
                "layer_fwd_bwd_ms": round(layer_ms, 4),
                "tokens_per_s": round(TOKENS / (layer_ms * 1e-3), 1),
                "note": "wide attention = two accumulated scans over the cos and the sin half (twice the plain "
                        "path's traffic plus the accumulator re-reads); rotation: 1 tensor in, 2 out (forward), "
                        "3 in, 1 out (backward)"}

        # ---- training step that keeps the forward workspace: la_fwd + la_bwd_saved, (1, 65536) point -----
        t = views(1, TOKENS)
        fws = torch.empty(max(256, binding.la_workspace_bytes(1, H, TOKENS, D, binding.LA_BF16, False)),
                          dtype=torch.uint8, device=dev)
        def train_step():
            binding.la_fwd(t["Q"], t["K"], t["V"], lam, O=t["O"], workspace=fws)
            binding.la_bwd_saved(t["Q"], t["K"], t["V"], lam, t["dO"], fws, dQ=t["dQ"], dK=t["dK"], dV=t["dV"],
                                 workspace=ws)
        sv = _time(train_step, it=20, key="saved")
        saved_states = {"workload": "la_fwd + la_bwd_saved (backward reuses the forward pass's segment states: the "
                                    "training-step form), [1,16,65536,128] bf16",
                        "fwd_bwd_ms": round(sv, 4), "fwd_bwd_ms_min": leg_min["saved"],
                        "tokens_per_s": round(TOKENS / (sv * 1e-3), 1),
                        "plain_fwd_bwd_ms": sweep[-1]["fwd_bwd_ms"] if sweep[-1]["n"] == TOKENS else None,
                        "note": "not the headline: la_bwd takes no saved context by contract"}

        # ---- token-major tensors ([B, n, H, d], what the layer's projections write) through the strided
        # entry points: the same memory read as permuted views, no transpose --------------------------------
        token_major = []
        for sB, sn in ((32, 2048), (8, 8192), (1, TOKENS)):
            tm = {k: v.view(sB, sn, H, D).permute(0, 2, 1, 3) for k, v in flat.items()}
            tf = _time(lambda: binding.la_fwd_strided(tm["Q"], tm["K"], tm["V"], lam, O=tm["O"], workspace=ws), key="tmf")
            tb = _time(lambda: binding.la_bwd_strided(tm["Q"], tm["K"], tm["V"], lam, tm["dO"], dQ=tm["dQ"],
                                                      dK=tm["dK"], dV=tm["dV"], workspace=ws), key="tmb")
            tfb = _time(lambda: (binding.la_fwd_strided(tm["Q"], tm["K"], tm["V"], lam, O=tm["O"], workspace=ws),
                                 binding.la_bwd_strided(tm["Q"], tm["K"], tm["V"], lam, tm["dO"], dQ=tm["dQ"],
                                                        dK=tm["dK"], dV=tm["dV"], workspace=ws)), key="tmfb")
            cont = [p for p in sweep if p["n"] == sn]
            token_major.append({"B": sB, "n": sn, "fwd_ms": round(tf, 4), "bwd_ms": round(tb, 4),
                                "fwd_bwd_ms": round(tfb, 4), "fwd_bwd_ms_min": leg_min["tmfb"],
                                "tokens_per_s": round(TOKENS / (tfb * 1e-3), 1),
                                "contiguous_fwd_bwd_ms": cont[0]["fwd_bwd_ms"] if cont else None})

        # ---- the sweep step captured once into a HIP graph and replayed (same calls, same kernels; only
        # the launches are issued by the graph instead of one by one from the host) -------------------------
        if not args.calib_copy and not args.point:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            gr = _time(graph.replay, it=20, key="graph")
            ea = _time(step, it=20, key="eager")
            graph_replay = {"workload": "the headline step (fwd+bwd at the six sweep points) as one replay of a "
                                        "captured HIP graph",
                            "ms_per_step": round(gr, 4), "ms_per_step_min": leg_min["graph"],
                            "tokens_per_s": round(tokens_per_step / (gr * 1e-3), 1),
                            "eager_ms_per_step": round(ea, 4), "eager_ms_per_step_min": leg_min["eager"],
                            "note": "not the headline: the headline times the C-ABI calls issued one by one"}

        # ---- the other bf16 configurations (parity cases; timed here so that their rates come from the
        # same run and protocol): C2 (TNL-400M-shaped layer, d = 64), C4 (TNL-7B-shaped layer), C5 (one
        # 131072-token sequence, half of the heads without decay) ------------------------------------------
        other_configs = []
        # (plus C2's layer shape at the sweep's size: d = 64, 32 heads, 65536 tokens, bytes as at C3's first point)
        for name in ("c2", "c2_at_64k_tokens", "c4", "c5"):
            if name == "c2_at_64k_tokens":
                w = synth.custom(32, 32, 2048, 64, [math.exp(-(h + 1) / 32.0) for h in range(32)], seed=0,
                                 dtype="bf16", name=name)
            else:
                w = synth.workload(name)
            el = w.B * w.H * w.n * w.d
            gsc = 1.0 / (w.d ** 0.5)
            xs = [(torch.randn(el, generator=gen, device=dev, dtype=torch.float32) * gsc).to(torch.bfloat16)
                  .view(w.B, w.H, w.n, w.d) for _ in range(3)]
            if name == "c4":                                     # Q, K = silu(N(0,1)) / sqrt(d)
                for i in range(2):
                    xs[i] = (torch.nn.functional.silu(xs[i].float() / gsc) * gsc).to(torch.bfloat16)
            xs.append(torch.randn(el, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
                      .view(w.B, w.H, w.n, w.d))
            outs = [torch.empty_like(xs[0]) for _ in range(4)]
            need = binding.la_workspace_bytes(w.B, w.H, w.n, w.d, binding.LA_BF16, True)
            cws = ws if need <= ws.numel() else torch.empty(need, dtype=torch.uint8, device=dev)
            cf_ = lambda: binding.la_fwd(xs[0], xs[1], xs[2], w.lambdas, O=outs[0], workspace=cws)
            cb_ = lambda: binding.la_bwd(xs[0], xs[1], xs[2], w.lambdas, xs[3], dQ=outs[1], dK=outs[2], dV=outs[3],
                                         workspace=cws)
            f_med, f_min = per_iteration_ms(cf_)
            b_med, b_min = per_iteration_ms(cb_)
            fb_med, fb_min = per_iteration_ms(lambda: (cf_(), cb_()))
            tok = w.B * w.n
            tps = tok / (fb_med * 1e-3)
            bk, L, S = binding.la_plan(w.B, w.H, w.n, w.d, binding.LA_BF16)
            mt = tps * w.H * 30 * w.d * w.d / 1e12
            et = tps * w.H * executed_flops_per_token_head(w.d, bk) / 1e12
            other_configs.append({
                "config": name, "B": w.B, "H": w.H, "n": w.n, "d": w.d,
                "fwd_ms": round(f_med, 4), "fwd_ms_min": round(f_min, 4), "bwd_ms": round(b_med, 4),
                "bwd_ms_min": round(b_min, 4), "fwd_bwd_ms": round(fb_med, 4), "fwd_bwd_ms_min": round(fb_min, 4),
                "tokens_per_s": round(tps, 1), "algorithmic_TBps": round(28 * w.d * w.H * tps / 1e12, 3),
                "model_tflops": round(mt, 2), "pct_mfma_bf16_peak": round(100.0 * mt / MFMA_BF16_PEAK_TFLOPS, 2),
                "executed_tflops": round(et, 2),
                "pct_mfma_bf16_peak_executed": round(100.0 * et / MFMA_BF16_PEAK_TFLOPS, 2),
                "block_len": bk, "segment_len": L, "segments": S})
            del xs, outs, cws
        torch.cuda.empty_cache()

        # ---- what the matrix cores deliver with nothing in the way: the measured bf16 denominator -----
        sink = torch.zeros(1, device=dev, dtype=torch.float32)
        mf_iters, mf_wgs = 4000, 8 * 256
        mf_flops = binding.debug_mfma_rate(mf_wgs, mf_iters, sink)
        mf_med, mf_min = per_iteration_ms(lambda: binding.debug_mfma_rate(mf_wgs, mf_iters, sink), warm=3, iters=10)
        mf_tflops = mf_flops / (mf_med * 1e-3) / 1e12
        mfma_measured = {
            "kernel": "register-only loop of v_mfma_f32_32x32x16_bf16, 4 independent accumulator tiles per wave, "
                      "%d workgroups x 4 waves x %d iterations" % (mf_wgs, mf_iters),
            "ms": round(mf_med, 4), "ms_min": round(mf_min, 4), "measured_tflops": round(mf_tflops, 1),
            "published_tflops": MFMA_BF16_PEAK_TFLOPS,
            "implied_clock_GHz": round(mf_tflops * 1e12 / (256 * 4 * 1024.0) / 1e9, 3),
            "note": "implied clock = measured rate / (256 CUs x 4 SIMDs x 1024 flops per cycle), i.e. the clock at "
                    "which the published 2.5 PFLOP/s (at 2.4 GHz) scales to the measured rate",
            "sweep_pct_of_measured_model_flops": None, "sweep_pct_of_measured_executed_flops": None}

        # ---- fp32 path (matrix-core fp32 kernel at d = 128): the (32, 2048) point in fp32 ---------------
        fB, fn = 32, 2048
        ft = {k: flat[k][: fB * H * fn * D].float().view(fB, H, fn, D) for k in ("Q", "K", "V", "dO")}
        fo = [torch.empty_like(ft["Q"]) for _ in range(4)]
        ff = _time(lambda: binding.la_fwd(ft["Q"], ft["K"], ft["V"], lam, O=fo[0]))
        fb = _time(lambda: binding.la_bwd(ft["Q"], ft["K"], ft["V"], lam, ft["dO"], dQ=fo[1], dK=fo[2], dV=fo[3]))
        f_tps = fB * fn / ((ff + fb) * 1e-3)
        fp32_path = {"workload": "la_fwd + la_bwd in fp32, [32,16,2048,128]", "fwd_ms": round(ff, 4), "bwd_ms": round(fb, 4),
                     "tokens_per_s": round(f_tps, 1),
                     "model_tflops": round(f_tps * H * MODEL_FLOPS_PER_TOKEN_HEAD / 1e12, 2),
                     "executed_tflops": round(f_tps * H * (4 * (4 * 32 * D + 4 * D * D)) / 1e12, 2),
                     "note": "compute-bound (fp32 MFMA peak 157.3 TFLOP/s); executed flops = four scans of "
                             "4 BK d + 4 d^2 per token per head at BK = 32"}
        del ft, fo

    total_tflops = value * H * MODEL_FLOPS_PER_TOKEN_HEAD / 1e12
    total_ex_tflops = value * H * executed_flops_per_token_head(D, sweep[0]["block_len"]) / 1e12
    if mfma_measured:
        mf_tflops = mfma_measured["measured_tflops"]
        mfma_measured["sweep_pct_of_measured_model_flops"] = round(100.0 * total_tflops / mf_tflops, 2)
        mfma_measured["sweep_pct_of_measured_executed_flops"] = round(100.0 * total_ex_tflops / mf_tflops, 2)
    # The target of the benchmark spec (>= 40 % of the bf16 MFMA peak at d = 128, 30 d^2 model flops) needs
    # 28 d bytes per token per head to move at this rate:
    target_tps = 0.40 * MFMA_BF16_PEAK_TFLOPS * 1e12 / (H * MODEL_FLOPS_PER_TOKEN_HEAD)
    target = {"north_star": ">= 40 % of bf16 MFMA peak at d = 128, near-constant tokens/s from 2K to 64K",
              "met": bool(100.0 * total_tflops / MFMA_BF16_PEAK_TFLOPS >= 40.0),
              "tokens_per_s_needed": round(target_tps, 1),
              "HBM_TBps_needed_at_28d_bytes": round(28 * D * H * target_tps / 1e12, 2),
              "measured_stream_TBps": round(stream_gbs / 1e3, 2),
              "note": "the path moves 28 d bytes per token per head (14 tensor passes) and is HBM-bound; at the "
                      "rate a plain 3-in / 1-out streaming kernel reaches on this box the ceiling is "
                      "%.1f %% of the MFMA peak" % (100.0 * (stream_gbs * 1e9 / (28 * D * H)) * H *
                                                    MODEL_FLOPS_PER_TOKEN_HEAD / 1e12 / MFMA_BF16_PEAK_TFLOPS)}
    out = {
        "metric": "fwd+bwd tokens/s (causal linear attention with decay, bf16, d=128, seq-len sweep "
                  "2K-64K at 64K tokens per batch)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "debug_switches": args.debug_switch,
        "config": {"workload": ("" if not args.point else "PROFILING SUBSET n=%d of: " % args.point) +
                               "c3 sweep: (B,n) in {(32,2048),(16,4096),(8,8192),(4,16384),(2,32768),"
                               "(1,65536)}, H=16, d=128, lambda_h geometric in [0.9,0.9999]; one step = "
                               "fwd+bwd at all six points (393216 tokens)",
                   "tokens_per_step": tokens_per_step, "H": H, "d": D},
        "model_tflops": round(total_tflops, 2),
        "pct_mfma_bf16_peak": round(100.0 * total_tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "executed_tflops": round(total_ex_tflops, 2),
        "pct_mfma_bf16_peak_executed": round(100.0 * total_ex_tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "target": target,
        "mfma_measured": mfma_measured,
        "other_configs": other_configs,
        "sweep": sweep,
        "near_constant": near_constant,
        "roofline": roofline,
        "decode": decode,
        "gate_norm": gate_norm,
        "swish_fused": swish_fused,
        "lrpe_d": lrpe,
        "fp32_path": fp32_path,
        "saved_states": saved_states,
        "graph_replay": graph_replay,
        "token_major": {"workload": "la_fwd_strided + la_bwd_strided on [B, n, H, d] tensors (H=16, d=128, bf16, "
                                    "65536 tokens), beside the contiguous [B, H, n, d] figure of the same point",
                        "points": token_major} if token_major is not None else None,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
