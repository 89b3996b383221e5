#!/usr/bin/env python3
"""Benchmark of the FeF-DLLM verify step on one MI355X.

A step is one call of fef_verify_step (vocabulary head for draft and target rows, softmax,
draft sampling, accept tests, first rejection, residual sample, commit, re-mask) on one batch
of synthetic hidden states with the head W resident in HBM.  Prints ONE JSON line with the
whole-step throughput (verify positions per second = B*K / step time), the roofline fraction
of the dominant kernel (the vocabulary head, timed with HIP events recorded by the library
around that kernel on its stream) and the CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps 200] [--warmup 10] [--workload llada_b1]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


class HipEvents:
    """Raw HIP events (ctypes on libamdhip64) so the library can record them on its stream."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        e = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(e))
        assert rc == 0, f"hipEventCreate failed: {rc}"
        return e.value

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventSynchronize(b)
        assert rc == 0, f"hipEventSynchronize failed: {rc}"
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime failed: {rc}"
        return ms.value

    def destroy(self, e):
        self.hip.hipEventDestroy(e)


def head_bytes(wl, skinny, M, rowstream=False, tiled256=False, stream=False):
    """Algorithmic HBM bytes of one vocabulary-head launch over M rows: W once, H once, fp32
    logits written once, the per-tile (max, sum exp) partials."""
    esz = 2 if wl.dtype == "bf16" else 4
    nT = min(-(-wl.V // 16), 256) if skinny else -(-wl.V // 64)
    if tiled256:
        nT = -(-wl.V // 256)      # the 256 x 256 kernels merge their partials per workgroup tile
    if rowstream:
        nT = min(256, -(-(-(-wl.V // 16)) // 8))
    if stream:
        nT = min(256, -(-(-(-wl.V // 64)) // 4))   # the LDS-streaming kernel leaves one partial per row and workgroup
    return wl.V * wl.d * esz + M * wl.d * esz + M * wl.V * 4 + M * nT * 8


def cpu_baseline(wl, W, rounds, seed, budget_s=14.0, budget_1t_s=8.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same rounds: once with
    every thread the numerical library uses by default, once pinned to one thread."""
    import numpy as np
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import fef_oracle as O
    from paper_2605_14305_amd import synth
    W64 = synth.to_f64(W)
    nb = min(wl.B, max(1, 16 // wl.K))   # batched workloads: a leading subset of sequences
    h64 = [(synth.to_f64(hd[:nb]), synth.to_f64(ht[:nb])) for hd, ht in rounds]
    O.verify_step(h64[0][0], h64[0][1], W64, wl.K, wl.block, seed, temperature=wl.temperature)  # warm-up

    def timed(budget, cap):
        n, t0 = 0, time.perf_counter()
        while True:
            hd, ht = h64[n % len(h64)]
            O.verify_step(hd, ht, W64, wl.K, wl.block, seed, step=n, temperature=wl.temperature)
            n += 1
            el = time.perf_counter() - t0
            if el > budget or n >= cap:
                return n, el

    n, el = timed(budget_s, 64)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    with threadpool_limits(limits=1):
        n1, el1 = timed(budget_1t_s, 16)
    return {"value": nb * wl.K * n / el, "unit": "positions/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} verify steps of workload {wl.name} ({nb} of {wl.B} sequences, {nb * wl.K} positions each), "
                      f"numpy fp64, {el:.1f} s; host has {len(os.sched_getaffinity(0))} usable cores",
            "one_thread": {"value": nb * wl.K * n1 / el1, "unit": "positions/s", "cores": 1,
                           "sample": f"{n1} of the same steps with the numerical library pinned to one thread, {el1:.1f} s"}}


def acceptance_sweep(args, wl, Wd, dev):
    """The acceptance-rate sweep of the batched configuration: for draft/target correlations rho (0.999
    added to the stated three so that the mean overlap reaches ~0.95) and temperatures tau, `--sweep N` calls each; reports the mean overlap alpha = sum min(p, q) the calls
    return, the mean committed length they produce, the closed form (1 - alpha^K) / (1 - alpha) of
    Theorem 2 at that mean alpha, and the idealised acceleration S = E[C] / 2 (Corollary 2)."""
    import torch
    from paper_2605_14305_amd import binding as fb
    from paper_2605_14305_amd import synth
    vs = fb.VerifyStep(wl.B, wl.K, wl.block, wl.d, wl.V, dtype=wl.dtype, device=dev, diag=True)
    rows = []
    for rho in (0.5, 0.9, 0.99, 0.999):
        batches = [tuple(t.to(dev) for t in synth.make_hidden(wl.B, wl.K, wl.d, args.seed, rho, wl.sigma_h, wl.dtype, 0, r))
                   for r in range(8)]
        for tau in (0.5, 1.0):
            alpha_sum = torch.zeros((), dtype=torch.float64, device=dev)
            committed = torch.zeros((), dtype=torch.float64, device=dev)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.sweep):
                hd, ht = batches[i % len(batches)]
                tok, acc, _ = vs(hd, ht, Wd, args.seed, step=i, temperature=tau)
                alpha_sum += vs.diag["alpha"].double().mean()
                committed += torch.clamp(acc + 1, max=wl.K).double().mean()
            torch.cuda.synchronize()
            el = time.perf_counter() - t0
            a = float(alpha_sum.item()) / args.sweep
            ec = wl.K if a >= 1.0 else (1.0 - a ** wl.K) / (1.0 - a)
            rows.append({"rho": rho, "tau": tau, "calls": args.sweep, "mean_alpha": a,
                         "mean_committed": float(committed.item()) / args.sweep,
                         "theorem2_at_mean_alpha": ec, "S_ideal": ec / 2.0, "us_per_call": el / args.sweep * 1e6})
            print("rho %.3f tau %.1f: alpha %.3f  committed %.3f  (1-a^K)/(1-a) %.3f  S %.2f  %.0f us/call"
                  % (rho, tau, a, rows[-1]["mean_committed"], ec, ec / 2, rows[-1]["us_per_call"]), file=sys.stderr, flush=True)
    print(json.dumps({"metric": "acceptance sweep of the verify step (mean overlap, committed length, Theorem 2)",
                      "n_gpus": 1, "data": "synthetic", "dtype": wl.dtype,
                      "config": {"workload": wl.name, "B": wl.B, "K": wl.K, "block": wl.block, "d": wl.d, "V": wl.V,
                                 "logit_std": wl.logit_std, "diagnostics": "alpha of every slot"},
                      "rows": rows}), flush=True)


def bench_cross_entropy(args, wl, W, Wd, dev):
    """One step = one fef_head_cross_entropy call on R rows (head kernel without logits store,
    per-row log-sum-exp merge, loss sum)."""
    import numpy as np
    import torch
    from paper_2605_14305_amd import binding as fb
    from paper_2605_14305_amd import synth
    R = args.ce
    ce = fb.HeadCrossEntropy(R, wl.d, wl.V, dtype=wl.dtype, device=dev)
    g = torch.Generator().manual_seed(args.seed + 7)
    hs = [(torch.randn(R, wl.d, generator=g) * wl.sigma_h).to(Wd.dtype).to(dev) for _ in range(4)]
    labels = torch.randint(0, wl.V, (R,), generator=g, dtype=torch.int32).to(dev)
    ev = HipEvents()
    pairs = [(ev.create(), ev.create()) for _ in range(args.steps)]
    for i in range(args.warmup):
        ce(hs[i % 4], Wd, labels)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ce(hs[i % 4], Wd, labels, head_events=pairs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    head_s = sum(ev.elapsed_ms(a, b) for a, b in pairs) / len(pairs) / 1e3
    esz = 2 if wl.dtype == "bf16" else 4
    nT = min(256, -(-(-(-wl.V // 64)) // 4)) if R <= 128 else -(-wl.V // 256)   # per workgroup / per 256-token tile
    hb = wl.V * wl.d * esz + R * wl.d * esz + R * nT * 8 + R * 4       # no logits are written
    flops = 2.0 * R * wl.V * wl.d
    if hb / (HBM_PEAK_GBS * 1e9) >= flops / (MFMA_BF16_PEAK_TFLOPS * 1e12):
        ach = hb / head_s / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": None}
    else:
        ach = flops / head_s / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    roof.update({"kernel": "head_stream_kernel" if R <= 128 else ("head_tiled256_kernel" if R <= 256 else "head_tiled256w4_kernel"),
                 "avg_kernel_us": head_s * 1e6, "algorithmic_bytes": hb, "flops": flops, "events": "inline"})
    out = {"metric": "cross-entropy rows/s through the vocabulary head (forward, no logits written)",
           "value": R / (elapsed / args.steps), "unit": "rows/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
           "config": {"workload": f"ce_{wl.name}_r{R}", "R": R, "d": wl.d, "V": wl.V}, "roofline": roof}
    if not args.no_cpu_baseline:
        from oracle import ce_oracle as C
        W64 = synth.to_f64(W)
        n = min(R, 16)
        h64 = synth.to_f64(hs[0][:n])
        lab = labels[:n].cpu().numpy()
        t1 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t1 < 10.0 and reps < 16:
            C.cross_entropy(h64, W64, lab)
            reps += 1
        el = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": n * reps / el, "unit": "rows/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"{reps} x {n} rows, numpy fp64, {el:.1f} s"}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llada_b1")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="N",
                    help="instead of the benchmark, run the library's plain copy kernel N times on a "
                         "1 GiB buffer (profiler byte-counter calibration)")
    ap.add_argument("--split", action="store_true",
                    help="the method's own call order: a draft-only call, then a target-only call "
                         "(W is read twice); the roofline entry then describes the target call's head launch")
    ap.add_argument("--graph", action="store_true",
                    help="record the 16 distinct steps once into a HIP graph and time its replays "
                         "(the head-kernel events then come from a second, eager pass)")
    ap.add_argument("--ce", type=int, default=0, metavar="R",
                    help="instead of the verify step, time the cross-entropy use of the head (Algorithm 1's "
                         "token-level loss, forward only) on R rows of the workload's head shape")
    ap.add_argument("--sweep", type=int, default=0, metavar="N",
                    help="instead of the timed step, run the acceptance sweep (rho x tau, N calls each) on the "
                         "workload's shape and print its table as one JSON line")
    ap.add_argument("--events", choices=["inline", "separate"], default="separate",
                    help="record the head-kernel events in a second pass over the same steps (default: the timed "
                         "region then holds no event-carrying dispatch), or inside the timed steps")
    ap.add_argument("--mfma-leg", default="sweep_b64", metavar="WORKLOAD",
                    help="batched workload of the second timed leg printed under \"mfma\" when the main workload "
                         "is llada_b1 (same head shape); `none` skips it")
    ap.add_argument("--variant", default="auto", choices=["auto", "skinny", "tiled", "tiled256", "stream", "rowstream"],
                    help="head kernel (fef_gemm_variant); auto = the library's choice")
    ap.add_argument("--mfma-steps", type=int, default=48, help="timed steps of the second leg")
    ap.add_argument("--event-every", type=int, default=4, metavar="N",
                    help="with inline events, attach them to every N-th timed step (a dispatch with events "
                         "costs about 10 us of queue time, which would otherwise sit in every step)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; the verify step shards over sequences with no "
              "communication, and no multi-GPU figure is produced. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_14305_amd import binding as fb
    from paper_2605_14305_amd import synth

    wl = synth.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_probe:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.copy_probe):
            fb.fef_copy_probe(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_launches": args.copy_probe, "bytes_read": 1 << 30, "bytes_written": 1 << 30}))
        return
    W = synth.make_head(wl.V, wl.d, args.seed, wl.dtype)
    Wd = W.to(dev)
    if args.ce:
        return bench_cross_entropy(args, wl, W, Wd, dev)
    if args.sweep:
        return acceptance_sweep(args, wl, Wd, dev)
    out, rounds = time_verify(args, wl, Wd, dev, args.steps, args.warmup)
    line = {
        "metric": "verify-step positions/s at d=4096,V=126464 bf16; % HBM (B=1) / % MFMA (B>=32)",
        "value": out["positions_per_s"],
        "unit": "positions/s",
        "n_gpus": 1, "steps": out["steps"], "warmup": args.warmup,
        "ms_per_step": out["ms_per_step"],
        "committed_positions_per_s": out["committed_positions_per_s"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": out["config"],
        "roofline": out["roofline"],
    }
    # The batched half of the metric (rows through the head >> the bf16 ridge of ~312): a second,
    # shorter timed leg on the acceptance-sweep shape, same head W (same d, V, seed).
    if args.mfma_leg != "none" and wl.name == "llada_b1" and not (args.split or args.graph):
        wl2 = synth.WORKLOADS[args.mfma_leg]
        assert (wl2.d, wl2.V, wl2.dtype) == (wl.d, wl.V, wl.dtype), "the second leg reuses the resident head"
        out2, _ = time_verify(args, wl2, Wd, dev, args.mfma_steps, max(2, args.warmup // 3))
        line["mfma"] = {"workload": wl2.name, "steps": out2["steps"], "ms_per_step": out2["ms_per_step"],
                        "positions_per_s": out2["positions_per_s"],
                        "committed_positions_per_s": out2["committed_positions_per_s"],
                        "config": out2["config"], "roofline": out2["roofline"]}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, W, rounds, args.seed)
    print(json.dumps(line), flush=True)


def time_verify(args, wl, Wd, dev, steps, warmup):
    """Time `steps` calls of fef_verify_step on workload `wl` (head Wd resident) after `warmup`
    untimed ones; the head kernel's own duration comes from HIP events the library attaches to
    that dispatch, by default in a second pass over the same steps so that no event-carrying
    dispatch sits in the timed region.  Returns (result dict, host copies of the hidden states)."""
    import torch
    from paper_2605_14305_amd import binding as fb
    from paper_2605_14305_amd import synth
    n_rounds = 16   # distinct hidden-state batches, cycled, so only W could ever sit in a cache
    rounds = [synth.make_round(wl, args.seed, block_index=i // 8, step=i) for i in range(n_rounds)]
    rounds_d = [(hd.to(dev), ht.to(dev)) for hd, ht in rounds]

    vs = fb.VerifyStep(wl.B, wl.K, wl.block, wl.d, wl.V, dtype=wl.dtype, device=dev,
                       gemm_variant={"auto": fb.FEF_GEMM_AUTO, "skinny": fb.FEF_GEMM_SKINNY, "tiled": fb.FEF_GEMM_TILED,
                                     "tiled256": fb.FEF_GEMM_TILED256, "stream": fb.FEF_GEMM_STREAM,
                                     "rowstream": fb.FEF_GEMM_ROWSTREAM}[args.variant])
    p0 = vs._params()
    p0.phase = fb.FEF_PHASE_DRAFT if args.split else fb.FEF_PHASE_FUSED
    variant = fb.fef_select_gemm(p0, wl.K)
    ev = HipEvents()
    pairs = [(ev.create(), ev.create()) for _ in range(max(steps, 16))]

    def step(i, events=None):
        hd, ht = rounds_d[i % n_rounds]
        if args.split:
            vs(hd, None, Wd, args.seed, step=i, temperature=wl.temperature, phase=fb.FEF_PHASE_DRAFT)
            vs(None, ht, Wd, args.seed, step=i, temperature=wl.temperature, phase=fb.FEF_PHASE_TARGET,
               head_events=events)
        else:
            vs(hd, ht, Wd, args.seed, step=i, temperature=wl.temperature, head_events=events)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    inline = args.events == "inline" and not args.graph
    if args.graph:
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            for i in range(n_rounds):
                step(i)
        replays = max(1, steps // n_rounds)
        steps = replays * n_rounds
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        for i in range(steps):
            step(i, pairs[i] if inline and i % args.event_every == 0 else None)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    if not inline:
        for i in range(steps):
            step(i, pairs[i])
        torch.cuda.synchronize()
    sampled = range(0, steps, args.event_every) if inline else range(steps)
    head_ms = [ev.elapsed_ms(*pairs[i]) for i in sampled]
    head_avg_s = sum(head_ms) / len(head_ms) / 1e3
    for a, b in pairs:
        ev.destroy(a); ev.destroy(b)

    # Outside the timed region: positions committed by the same steps (the decisions are a function
    # of inputs and seed, so a second pass repeats them), and the rate of a plain read of W.
    committed = 0
    if not args.split:
        counts = []
        for i in range(steps):
            hd, ht = rounds_d[i % n_rounds]
            tok, _, _ = vs(hd, ht, Wd, args.seed, step=i, temperature=wl.temperature)
            counts.append((tok >= 0).sum())
        committed = int(torch.stack(counts).sum().item())
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        fb.fef_read_probe(Wd, sink)
    e0.record()
    for _ in range(10):
        fb.fef_read_probe(Wd, sink)
    e1.record()
    torch.cuda.synchronize()
    read_ceiling = Wd.numel() * Wd.element_size() * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    ms_per_step = elapsed / steps * 1e3
    positions = wl.B * wl.K
    M = positions if args.split else 2 * positions   # rows through one head launch
    hb = head_bytes(wl, variant == fb.FEF_GEMM_SKINNY, M, variant == fb.FEF_GEMM_ROWSTREAM,
                    variant == fb.FEF_GEMM_TILED256, variant == fb.FEF_GEMM_STREAM)
    flops = 2.0 * M * wl.V * wl.d
    hbm_time, mfma_time = hb / (HBM_PEAK_GBS * 1e9), flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if hbm_time >= mfma_time:
        ach = hb / head_avg_s / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None}
    else:
        ach = flops / head_avg_s / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    roof.update({"kernel": {fb.FEF_GEMM_SKINNY: "head_skinny_kernel" if M <= 16 else "head_skinny32_kernel",
                            fb.FEF_GEMM_TILED: "head_tiled_kernel",
                            fb.FEF_GEMM_TILED256: "head_tiled256_kernel" if M <= 256 else "head_tiled256w4_kernel",
                            fb.FEF_GEMM_STREAM: "head_stream_kernel",
                            fb.FEF_GEMM_ROWSTREAM: "head_rowstream_kernel",
                            fb.FEF_GEMM_F32: "head_f32_kernel"}[variant],
                 "avg_kernel_us": head_avg_s * 1e6, "algorithmic_bytes": hb, "flops": flops,
                 "events": "separate" if args.graph else args.events,
                 "event_samples": len(head_ms),
                 "plain_read_of_W_GBs": read_ceiling})
    if roof["bound"] == "hbm":
        roof["frac_of_plain_read"] = roof["achieved"] / read_ceiling
    # HBM-side bytes per launch are profiler counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) of an
    # earlier run of this same command, stored with the profiles; they are not measured in this run.
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            t = json.load(f).get(f"{roof['kernel']}:{wl.name}")
        if t:
            roof["traffic"] = t["hbm_bytes_per_launch"]
            roof["traffic_source"] = "profiles/traffic.json (stored rocprofv3 counter run of this kernel and workload)"
    out = {
        "steps": steps, "ms_per_step": ms_per_step, "positions_per_s": positions / (elapsed / steps),
        "committed_positions_per_s": committed / elapsed if committed else None,
        "config": {"workload": wl.name, "B": wl.B, "K": wl.K, "block": wl.block, "d": wl.d, "V": wl.V,
                   "rho": wl.rho, "logit_std": wl.logit_std, "temperature": wl.temperature,
                   "rows_through_head": M, "call_order": "draft+target" if args.split else "fused",
                   "launch": "hip graph replay" if args.graph else "stream"},
        "roofline": roof,
    }
    del vs
    torch.cuda.empty_cache()
    return out, rounds


if __name__ == "__main__":
    main()
