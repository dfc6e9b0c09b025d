#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

A *step* is one pass of the whole hot path (gate -> dispatch -> grouped expert FFN -> combine; the
headline layer is synchronous, i.e. every pair is transmitted and no refresh mask is computed) over
the 28 stacked layers of the DiT-MoE-XL-shaped workload (T = 4096 tokens, d = 1152, E = 8, top-2,
F = 4608, bf16), i.e. a full denoising step's MoE work.  Every layer has its own seeded weights,
activations and buffers, all resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Beside the headline the line carries, measured in the same run:
  * ``stages``: every stage as its own captured graph over the 28 layers' (cache-cold) buffers, so
    that launch gaps drop out; the row gather of dispatch is timed as the packed-buffer variant;
  * ``roofline``: the expert FFN (both grouped GEMMs of one moe_expert_ffn_rows call) against the
    bf16 MFMA peak, with the split per GEMM from events recorded between the two launches;
  * ``conditional_refresh``: the 512px Conditional Communication workload (T = 8192, two steps) at
    refresh fractions 25 / 50 / 75 / 100 %, with its per-stage HBM figures at 50 %;
  * ``ep_shard``: the grouped FFN over one expert-parallel shard's receive buffer (Zipf load);
  * ``cpu_baseline``: the oracle on bounded samples of the same workloads on the host cores.
"""
import argparse
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def kernel_sources_hash():
    """sha256 over the FFN kernel sources: ties a stored counter summary to the code it was taken on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2411_16786_amd", "csrc")
    for name in ("ffn.hip", "ffn_wide.hpp", "ffn_mfma.hpp"):
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=None, help="override the 28 layers (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the conditional-refresh sweep and the expert-parallel shard (headline and stages only)")
    ap.add_argument("--no-calibrate", action="store_true",
                    help="skip the two machine-ceiling microbenchmarks of the library (plain streaming copy at three "
                         "sizes; register-resident MFMA loop on random and on zero operands), reported under 'calibration'")
    ap.add_argument("--packed-dispatch", action="store_true",
                    help="materialise x_packed in moe_dispatch instead of gathering rows in the FFN's operand load")
    ap.add_argument("--n-shared", type=int, default=0,
                    help="add this many shared experts (always-fresh dense FFNs; DiT-MoE carries 2) to every layer; "
                         "the headline workload has none")
    ap.add_argument("--schedule", choices=["sync", "interweaved", "displaced", "dice"], default="sync",
                    help="step-level schedule of every layer (Algorithms 1-3); the headline workload is the synchronous "
                         "layer.  The asynchronous ones read the persistent combine buffer and run the expert call "
                         "whose results the next step collects on a second stream.  dice = the paper's combination: interweaved "
                         "in the shallow half of the layers, synchronous in the deep half (Selective Synchronization), "
                         "Algorithm 4 with stride 2 in every layer (Conditional Communication); launched eagerly")
    ap.add_argument("--workload", choices=["xl", "g", "s"], default="xl",
                    help="xl: DiT-MoE-XL shape x 28 layers (the headline workload); g: DiT-MoE-G shape (16 experts, "
                         "d=1792) x 40 layers; s: the small DiT-MoE-S-shaped layer (T=2048, d=384, 16 experts) x 12 layers")
    ap.add_argument("--tokens", type=int, default=None,
                    help="tokens per layer call instead of the workload's (smaller local batches; not the headline)")
    ap.add_argument("--eager", action="store_true", help="launch from Python every step instead of replaying a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no multi-GPU path); use --gpus 1")

    import numpy as np
    import torch

    from paper_2411_16786_amd import binding as B
    from paper_2411_16786_amd import workloads as WL

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    dev = "cuda"
    wl_cfg = {"xl": 3, "g": 6, "s": 2}[args.workload]
    c = WL.CONFIGS[wl_cfg]
    n_layers = args.layers or (12 if args.workload == "s" else c.layers)
    T, d, E, k, F = (args.tokens or c.T), c.d, c.E, c.k, c.F
    n_shared = args.n_shared
    N = T * (k + n_shared)          # (token, slot) pairs: k routed slots and one per shared expert
    headline = args.workload == "xl" and n_shared == 0 and args.tokens is None and args.schedule == "sync"
    extras = headline and not args.no_extras
    b = 2                           # bytes per bf16 element

    # ---- inputs: seeded on the host, uploaded once
    t_setup = time.time()
    ctx = B.Context(T, d, F, E, k, "bf16", n_shared=n_shared)
    workspace = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
    up = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(dev)
    layers = []
    n_cpu = 4 if args.workload == "xl" else 2      # layers kept on the host for the oracle's timed sample
    cpu_layers = []
    with ThreadPoolExecutor(max_workers=8) as pool:
        for first in range(0, n_layers, 8):        # generated and uploaded eight layers at a time (host memory)
            chunk = list(pool.map(lambda l: WL.make_layer(wl_cfg, layer=l, n_shared=n_shared, T=T),
                                  range(first, min(first + 8, n_layers))))
            for li in chunk:
                buf = B.LayerBuffers(ctx, dev, workspace=workspace)
                layers.append(dict(x=up(li.x), Wg=up(li.Wg), bg=None if li.bg is None else torch.from_numpy(li.bg).to(dev),
                                   W1=up(li.W1), W2=up(li.W2), buf=buf))
            if first == 0:
                cpu_layers = chunk[:n_cpu]
            del chunk
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    def graph_time(fn, reps=5):
        """Capture ``fn`` (a fixed launch sequence) as one HIP graph and return its mean replay time in ms."""
        fn()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    deferred = None
    step_no = [0]
    if args.schedule != "sync":
        from paper_2411_16786_amd import schedule as SCH
        deferred = torch.cuda.Stream()
        side_ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
        for L in layers:
            L["state"] = SCH.LayerState(ctx, dev, displaced=(args.schedule == "displaced"), workspace=workspace,
                                        side_workspace=side_ws)
            # one synchronous step fills the persistent buffers (and, for displaced, leaves a dispatch to wait on)
            SCH.moe_layer_step(SCH.SYNC, L["state"], L["x"], L["Wg"], L["bg"], L["W1"], None, L["W2"], None)
        torch.cuda.synchronize()

    def one_step():
        if deferred is None:
            for L in layers:
                B.moe_layer_forward(ctx, L["buf"], L["x"], L["Wg"], L["bg"], L["W1"], None, L["W2"], None,
                                    fuse_gather=not args.packed_dispatch)
            return
        if args.schedule == "dice":
            step_no[0] += 1
            pol = B.Policy(B.REFRESH_ALG4, step_t=step_no[0], stride_n=2)
            for i, L in enumerate(layers):
                sched = SCH.INTERWEAVED if 2 * i < len(layers) else SCH.SYNC
                SCH.moe_layer_step(sched, L["state"], L["x"], L["Wg"], L["bg"], L["W1"], None, L["W2"], None, policy=pol,
                                   side_stream=deferred if sched != SCH.SYNC else None)
        else:
            for L in layers:
                SCH.moe_layer_step(args.schedule, L["state"], L["x"], L["Wg"], L["bg"], L["W1"], None, L["W2"], None,
                                   side_stream=deferred)
        torch.cuda.current_stream().wait_stream(deferred)      # the step ends when its deferred expert calls have
        for L in layers:
            L["state"].commit_done = None
            L["buf"] = L["state"].buf                      # where this step's outputs are

    # ---- the headline: K steps, replayed as one HIP graph (the launch sequence is static)
    graph = None
    one_step()
    torch.cuda.synchronize()
    # (displaced alternates between two sets of layer buffers from step to step: launched eagerly)
    if not args.eager and args.schedule not in ("displaced", "dice"):
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        y_eager = layers[-1]["buf"].y.clone()
        with torch.cuda.graph(graph):
            one_step()
        for _ in range(2):
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(layers[-1]["buf"].y, y_eager), "graph replay differs from the eager result"
    run = graph.replay if graph is not None else one_step

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = T * n_layers * args.steps / elapsed

    # ---- every stage as its own captured graph over all layers (buffers of different layers: cache-cold)
    def stage_fns():
        def gate():
            for L in layers:
                ctx.moe_gate(L["x"], L["Wg"], L["bg"], L["buf"].scores, L["buf"].expert_idx)

        def dispatch_index():      # as in moe_layer_forward: index outputs only, the FFN gathers the rows itself
            for L in layers:
                bf = L["buf"]
                ctx.moe_dispatch(L["x"], bf.expert_idx, None, None, bf.counts, bf.offsets, bf.perm, bf.inv, bf.workspace)

        def dispatch_packed():     # the expert-parallel send buffer: index kernels + row gather
            for L in layers:
                bf = L["buf"]
                ctx.moe_dispatch(L["x"], bf.expert_idx, None, bf.x_packed, bf.counts, bf.offsets, bf.perm, bf.inv,
                                 bf.workspace)

        def expert_ffn():
            for L in layers:
                bf = L["buf"]
                ctx.moe_expert_ffn_rows(L["x"], bf.perm, bf.offsets, bf.seg_expert, N, L["W1"], None, L["W2"], None,
                                        bf.h_packed, bf.workspace)

        def combine():
            for L in layers:
                bf = L["buf"]
                ctx.moe_combine(bf.h_packed, bf.inv, bf.scores, None, None, None, False, bf.y)

        return [("gate", gate), ("dispatch", dispatch_index), ("dispatch_packed", dispatch_packed),
                ("expert_ffn", expert_ffn), ("combine", combine)]

    for L in layers:                       # the stage graphs run on the layers' own (synchronous) buffers
        L["buf"] = L.get("state").bufs[0] if "state" in L else L["buf"]
    avg = {name: graph_time(fn) / n_layers for name, fn in stage_fns()}
    avg["dispatch_gather"] = max(avg["dispatch_packed"] - avg["dispatch"], 1e-6)
    alg_bytes = {
        "gate": T * d * b + E * d * b + N * 8,
        "dispatch": 16 * N,                                   # index outputs only; the row gather rides in the FFN's operand load
        "dispatch_packed": T * d * b + N * d * b + 16 * N,    # each token row read once, every pair's row written
        "dispatch_gather": T * d * b + N * d * b + 4 * N,     # the gather kernel alone (by difference)
        "combine": N * d * b + T * d * b + N * 9,
    }
    ffn_flops = 4.0 * N * d * F
    ffn_tflops = ffn_flops / (avg["expert_ffn"] * 1e-3) / 1e12
    stages = {s: {"ms": round(v, 5)} for s, v in avg.items()}
    for s, nbytes in alg_bytes.items():
        gbs = nbytes / (avg[s] * 1e-3) / 1e9
        stages[s].update({"algorithmic_bytes": nbytes, "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)})
    stages["expert_ffn"].update({"flops": ffn_flops, "TFLOP/s": round(ffn_tflops, 1),
                                 "frac_mfma": round(ffn_tflops / PEAK_BF16_TFLOPS, 4)})

    # ---- the two GEMMs of the FFN call: an event recorded between the launches (eager pass, two rounds)
    per_kernel = None
    mids, ends = [], []
    for rnd in range(2):
        evs = []
        for L in layers:
            bf = L["buf"]
            e0, em, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            em.record()                                      # creates the handle that the library records again below
            ctx.moe_expert_ffn_between_event(em)
            e0.record()
            ctx.moe_expert_ffn_rows(L["x"], bf.perm, bf.offsets, bf.seg_expert, N, L["W1"], None, L["W2"], None,
                                    bf.h_packed, bf.workspace)
            e1.record()
            evs.append((e0, em, e1))
        ctx.moe_expert_ffn_between_event(None)
        torch.cuda.synchronize()
        if rnd == 1:
            mids = [e0.elapsed_time(em) for e0, em, _ in evs]
            ends = [em.elapsed_time(e1) for _, em, e1 in evs]
    g1_ms, g2_ms = float(np.mean(mids)), float(np.mean(ends))
    half = ffn_flops / 2
    per_kernel = {
        "GEMM1 (W1, bias, GELU; row gather in the operand load)": {
            "ms": round(g1_ms, 5), "TFLOP/s": round(half / (g1_ms * 1e-3) / 1e12, 1),
            "frac": round(half / (g1_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
        "GEMM2 (W2, bias)": {
            "ms": round(g2_ms, 5), "TFLOP/s": round(half / (g2_ms * 1e-3) / 1e12, 1),
            "frac": round(half / (g2_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
        "note": "events on the launch stream around and between the two launches of each call (eager, launch gaps included)"}

    traffic, traffic_note = None, "no counter summary for these kernel sources"
    tpath = os.path.join(ROOT, "profiles", "bench_xl28_hbm_traffic.txt")
    if os.path.exists(tpath) and headline:      # rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this same command (not live)
        stored_hash, stored = None, None
        for line in open(tpath):
            if line.startswith("ffn_traffic_bytes_per_call:"):
                stored = int(line.split(":")[1].split()[0])
            if line.startswith("kernel_sources_sha256_16:"):
                stored_hash = line.split(":")[1].strip()
        if stored is not None and stored_hash == kernel_sources_hash():
            traffic = stored
            traffic_note = ("HBM-side bytes per moe_expert_ffn_rows call from profiles/bench_xl28_hbm_traffic.txt "
                            f"(taken on kernel sources {stored_hash}, the ones that ran here)")
        elif stored is not None:
            traffic_note = (f"profiles/bench_xl28_hbm_traffic.txt was taken on kernel sources {stored_hash}, "
                            f"these are {kernel_sources_hash()}: not reported")
    roofline = {"kernel": "ffn_gemm_bf16_wide_kernel (GEMM1 + GEMM2 of one moe_expert_ffn_rows call)", "bound": "mfma",
                "achieved": round(ffn_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ffn_tflops / PEAK_BF16_TFLOPS, 4), "traffic": traffic, "traffic_note": traffic_note,
                "timing": f"mean over {n_layers} calls (one per layer, cold weights) replayed as one HIP graph, HIP events",
                "per_kernel": per_kernel}

    # ---- machine ceilings from the library's two microbenchmarks
    calibration = None
    if not args.no_calibrate:
        calibration = {"copy": [], "mfma": []}
        pool_bytes = 512 << 20
        src = torch.empty(pool_bytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for nbytes in (28385280, 75497472, 256 << 20):
            nrot = pool_bytes // nbytes
            def copies(nbytes=nbytes, nrot=nrot):
                for i in range(2 * nrot):
                    off = (i % nrot) * nbytes
                    B.moe_calibrate_copy(dst[off:off + nbytes], src[off:off + nbytes], 2048)
            ms = graph_time(copies) / (2 * nrot)
            calibration["copy"].append({"bytes_read_plus_written": 2 * nbytes, "us": round(ms * 1e3, 2),
                                        "GB/s": round(2 * nbytes / (ms * 1e-3) / 1e9, 1)})
        del src, dst
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
        iters, wgs = 4096, 256
        for name, ops in (("random bf16 operands", torch.randn(16 * 256 * 48, device=dev).to(torch.bfloat16)),
                          ("zero operands", torch.zeros(16 * 256 * 48, dtype=torch.bfloat16, device=dev))):
            ms = graph_time(lambda ops=ops: [B.moe_calibrate_mfma(ops, sink, iters, wgs) for _ in range(4)]) / 4
            flops = 2.0 * 32 * 32 * 16 * 8 * iters * 4 * wgs
            calibration["mfma"].append({"operands": name, "us": round(ms * 1e3, 1),
                                        "TFLOP/s": round(flops / (ms * 1e-3) / 1e12, 1)})
        # yardstick only: the vendor library's plain bf16 GEMM (through torch.matmul) at the two dense shapes of
        # this workload's FFN, i.e. one even segment, no gather, bias or GELU, the same operands every call
        rows = T * k
        calibration["library_gemm"] = []
        for name, n_, k_ in (("rows x F x d (the first GEMM's shape)", F, d), ("rows x d x F (the second GEMM's shape)", d, F)):
            a_ = torch.randn(rows, k_, device=dev).to(torch.bfloat16)
            w_ = (torch.randn(n_, k_, device=dev) * 0.02).to(torch.bfloat16)
            out_ = torch.empty(rows, n_, dtype=torch.bfloat16, device=dev)
            for _ in range(3):
                torch.matmul(a_, w_.t(), out=out_)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(20):
                torch.matmul(a_, w_.t(), out=out_)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 20
            calibration["library_gemm"].append({"shape": name, "rows": rows, "us": round(us, 1),
                                                "TFLOP/s": round(2.0 * rows * n_ * k_ / us * 1e-6, 1)})
            del a_, w_, out_

    # ---- Conditional Communication at the 512px shape (two consecutive diffusion steps), weights of the 28 layers
    cond = None
    cond_cpu = None
    if extras:
        c4 = WL.CONFIGS[4]
        assert (c4.d, c4.F, c4.E, c4.k) == (d, F, E, k)
        n_sets = 8
        ctx4 = B.Context(c4.T, c4.d, c4.F, c4.E, c4.k, "bf16")
        ws4 = torch.empty(ctx4.workspace_bytes(), dtype=torch.uint8, device=dev)
        sets = []
        li4 = None
        for i in range(n_sets):
            li = WL.make_layer(4, layer=i, with_experts=False)
            if i == 0:
                li4 = li
            sets.append(dict(x_prev=up(li.x), x_next=up(WL.next_step_x(4, li.x, layer=i)),
                             buf=B.LayerBuffers(ctx4, dev, with_cache=True, workspace=ws4)))
        N4 = c4.T * c4.k

        def layer_call(i, pol, which="x_next"):
            S, L = sets[i % n_sets], layers[i % n_layers]
            B.moe_layer_forward(ctx4, S["buf"], S[which], L["Wg"], None, L["W1"], None, L["W2"], None, policy=pol)

        cond = []
        for frac in (1.0, 0.75, 0.5, 0.25):
            n_units = int(frac * c4.T + 0.5)
            pol = B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=n_units)
            R = ctx4.moe_policy_refreshed_pairs(pol, c4.T)[0]
            for i in range(n_sets):                           # step t-1 fills the caches
                layer_call(i, B.Policy(B.REFRESH_ALL), "x_prev")
            ms = graph_time(lambda: [layer_call(i, pol) for i in range(n_layers)]) / n_layers
            entry = {"refresh_fraction": frac, "policy": "FRACTION_TOKEN", "refreshed_pairs": R,
                     "ms_per_layer": round(ms, 4), "tokens_per_s": round(c4.T / (ms * 1e-3), 1),
                     "ffn_flops_needed": 4.0 * R * c4.d * c4.F}
            if frac == 0.5:                                   # the stages of this step on their own (graphs over the sets)
                def st_refresh():
                    for i in range(n_layers):
                        bf = sets[i % n_sets]["buf"]
                        ctx4.moe_conditional_refresh(bf.scores, bf.expert_idx, pol, bf.mask, bf.n_refresh, bf.workspace)

                def st_dispatch():
                    for i in range(n_layers):
                        S = sets[i % n_sets]; bf = S["buf"]
                        ctx4.moe_dispatch(S["x_next"], bf.expert_idx, bf.mask, None, bf.counts, bf.offsets, bf.perm, bf.inv,
                                          bf.workspace)

                def st_dispatch_packed():
                    for i in range(n_layers):
                        S = sets[i % n_sets]; bf = S["buf"]
                        ctx4.moe_dispatch(S["x_next"], bf.expert_idx, bf.mask, bf.x_packed, bf.counts, bf.offsets, bf.perm,
                                          bf.inv, bf.workspace)

                def st_ffn():          # as in moe_layer_forward: the refreshed rows go straight into the cache
                    for i in range(n_layers):
                        S, L = sets[i % n_sets], layers[i % n_layers]; bf = S["buf"]
                        ctx4.moe_expert_ffn_commit(S["x_next"], bf.perm, bf.perm, bf.offsets, bf.seg_expert, R, L["W1"], None,
                                                   L["W2"], None, None, bf.mask, bf.H_cache, None, bf.workspace, T=c4.T)

                def st_combine():      # every row from the cache, scores written through
                    for i in range(n_layers):
                        bf = sets[i % n_sets]["buf"]
                        ctx4.moe_combine(None, bf.inv, bf.scores, bf.mask, bf.H_cache, bf.S_cache, False, bf.y)

                t = {n_: graph_time(f_) / n_layers for n_, f_ in (("refresh_mask", st_refresh), ("dispatch", st_dispatch),
                                                                   ("dispatch_packed", st_dispatch_packed),
                                                                   ("expert_ffn", st_ffn), ("combine", st_combine))}
                t["dispatch_gather"] = max(t["dispatch_packed"] - t["dispatch"], 1e-6)
                by = {"dispatch_gather": c4.T * c4.d * b + R * c4.d * b + 4 * N4,
                      # every pair's row read from the cache (the expert call wrote the fresh ones there), y written
                      "combine": N4 * c4.d * b + c4.T * c4.d * b + N4 * 9}
                st = {n_: {"ms": round(v, 5)} for n_, v in t.items()}
                for n_, nb in by.items():
                    gbs = nb / (t[n_] * 1e-3) / 1e9
                    st[n_].update({"algorithmic_bytes": nb, "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)})
                fl = 4.0 * R * c4.d * c4.F
                st["expert_ffn"].update({"TFLOP/s": round(fl / (t["expert_ffn"] * 1e-3) / 1e12, 1),
                                         "frac_mfma": round(fl / (t["expert_ffn"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)})
                entry["stages"] = st
            cond.append(entry)
        if not args.no_cpu_baseline:
            # the oracle on a bounded sample of this workload: two steps of the first 512 tokens, 50 % refreshed
            from oracle import moe_oracle as O
            Ts = 512
            lw = cpu_layers[0]
            xs0, xs1 = li4.x[:Ts], WL.next_step_x(4, li4.x)[:Ts]
            H = np.zeros((Ts, c4.k, c4.d)); S_ = np.zeros((Ts, c4.k))
            O.moe_layer(xs0, lw.Wg, None, lw.W1, None, lw.W2, None, c4.k, policy=O.REFRESH_ALL, H_cache=H, S_cache=S_)
            t1 = time.perf_counter()
            O.moe_layer(xs1, lw.Wg, None, lw.W1, None, lw.W2, None, c4.k, policy=O.REFRESH_FRACTION_TOKEN,
                        n_units=Ts // 2, H_cache=H, S_cache=S_)
            dt = time.perf_counter() - t1
            cond_cpu = {"value": round(Ts / dt, 2), "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
                        "sample": f"step t of the first {Ts} tokens at 50 % refresh (FRACTION_TOKEN), {dt:.2f} s"}
        del sets, ws4

    # ---- the receive side of an expert-parallel shard (segments ordered [source rank][local expert])
    ep_shard = None
    if extras:
        ep = WL.make_ep_shard()
        c5 = ep.cfg
        rows, W_ranks, E_loc = ep.x_recv.shape[0], ep.recv_counts.shape[0], ep.recv_counts.shape[1]
        ctx5 = B.Context(rows, c5.d, c5.F, E_loc, 1, "bf16")
        seg_offsets = torch.empty(W_ranks * E_loc + 1, dtype=torch.int32, device=dev)
        seg_expert = torch.empty(W_ranks * E_loc, dtype=torch.int32, device=dev)
        ctx5.moe_ep_segments(torch.from_numpy(np.ascontiguousarray(ep.recv_counts, dtype=np.int32)).to(dev),
                             seg_offsets, seg_expert)
        n_copies = 4                                              # 268 MB of weights per copy: cold in every call
        x5 = [up(ep.x_recv) for _ in range(n_copies)]
        W1_5 = [up(ep.W1) for _ in range(n_copies)]
        W2_5 = [up(ep.W2) for _ in range(n_copies)]
        h5 = torch.empty((rows, c5.d), dtype=torch.bfloat16, device=dev)
        ws5 = torch.empty(ctx5.workspace_bytes(), dtype=torch.uint8, device=dev)
        ms = graph_time(lambda: [ctx5.moe_expert_ffn(x5[i % n_copies], seg_offsets, seg_expert, rows, W1_5[i % n_copies], None,
                                                     W2_5[i % n_copies], None, h5, ws5) for i in range(2 * n_copies)]) / (2 * n_copies)
        ctx5.moe_expert_ffn_status(ws5)
        flops5 = 4.0 * rows * c5.d * c5.F
        ep_shard = {"rows": rows, "segments": W_ranks * E_loc, "rows_per_local_expert": ep.recv_counts.sum(axis=0).tolist(),
                    "ms_per_call": round(ms, 4), "rows_per_s": round(rows / (ms * 1e-3), 1), "flops": flops5,
                    "TFLOP/s": round(flops5 / (ms * 1e-3) / 1e12, 1),
                    "frac_mfma": round(flops5 / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        if not args.no_cpu_baseline:
            from oracle import moe_oracle as O
            so, se = O.ep_segments(ep.recv_counts)
            sel = np.random.Generator(np.random.PCG64(5)).choice(rows, size=384, replace=False).astype(np.int32)
            t1 = time.perf_counter()
            h_ref = O.expert_ffn(ep.x_recv, so, se, ep.W1, None, ep.W2, None, rows_sel=np.sort(sel))
            dt = time.perf_counter() - t1
            got = h5.float().cpu().numpy()[np.sort(sel)]
            rel = float(np.linalg.norm(got - h_ref) / np.linalg.norm(h_ref))
            assert rel <= 1e-2, f"expert-parallel shard output differs from the oracle: rel-L2 {rel:.3e}"
            ep_shard["cpu_baseline"] = {"value": round(len(sel) / dt, 2), "unit": "rows/s", "cores": O.num_threads(),
                                        "kind": "oracle",
                                        "sample": f"{len(sel)} sampled rows of the receive buffer, {dt:.2f} s; HIP rows vs "
                                                  f"the oracle: rel-L2 {rel:.2e}"}
        del x5, W1_5, W2_5, h5, ws5

    # ---- the CPU oracle on a bounded sample of the headline workload (whole layers)
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O
        for _ in range(1):
            run()                                       # the buffers hold the outputs of the timed path again
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        refs = [O.moe_layer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, k, n_shared=n_shared) for li in cpu_layers]
        cpu_s = time.perf_counter() - t1
        # the same layers through the HIP path (the buffers still hold the last timed pass): a live
        # parity check of exactly the code that was benchmarked
        worst = 0.0
        for L, ref in zip(layers, refs):
            got = L["buf"].y.float().cpu().numpy()
            # tokens whose k-th and (k+1)-th logits are closer than float accumulation resolves are
            # left out of the comparison (none at the seeds in use; the guard keeps the check honest)
            zs = -np.sort(-ref.z, axis=1)
            safe = np.min(zs[:, :k] - zs[:, 1:k + 1], axis=1) > 1e-4
            assert safe.mean() > 0.999
            assert np.array_equal(L["buf"].expert_idx.cpu().numpy()[safe, :k], ref.idx[safe]), "routing differs from the oracle"
            if safe.all() and n_shared == 0:
                assert np.array_equal(L["buf"].perm.cpu().numpy(), ref.perm), "permutation differs from the oracle"
            rel = float(np.linalg.norm(got[safe] - ref.y[safe]) / np.linalg.norm(ref.y[safe]))
            # max-abs 2e-2 is fit to |y| up to about 2; ungated shared experts push |y| past 4, where one
            # bf16 rounding of the output alone costs 1.6e-2, so with them the bound grows with max|y|
            abs_tol = 2e-2 * (max(1.0, float(np.abs(ref.y).max()) / 2.0) if n_shared else 1.0)
            worst_abs = float(np.abs(got[safe] - ref.y[safe]).max())
            assert rel <= 1e-2 and worst_abs <= abs_tol, \
                f"bench output differs from the oracle: rel-L2 {rel:.3e}, max-abs {worst_abs:.3e} (bound {abs_tol:.3e})"
            worst = max(worst, rel)
        n_lay = len(cpu_layers)
        cpu_baseline = {"value": round(T * n_lay / cpu_s, 2), "unit": "tokens/s (token passes through one MoE layer)",
                        "cores": O.num_threads(), "kind": "oracle",
                        "sample": f"layers 0..{n_lay - 1} of the same workload, whole layers (T={T}), {cpu_s:.2f} s; "
                                  f"HIP outputs of these layers vs the oracle: worst rel-L2 {worst:.2e}"}
        if cond_cpu is not None:
            cpu_baseline["conditional_refresh"] = cond_cpu

    out = {
        "metric": "MoE-layer tokens/sec at DiT-MoE-XL shape",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s (token passes through one MoE layer; T*layers per step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_layer": round(ms_per_step / n_layers, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": ("configs[2]: DiT-MoE-XL-shaped layer x 28 (T=4096, d=1152, E=8, top-2, F=4608)"
                                if args.workload == "xl" else
                                f"{'DiT-MoE-G' if args.workload == 'g' else 'configs[1]: DiT-MoE-S'}-shaped layer x {n_layers} "
                                f"(T={T}, d={d}, E={E}, top-{k}, F={F})")
                               + (f" + {n_shared} shared experts per layer" if n_shared else ""),
                   "layers": n_layers, "tokens": T, "launch": "eager" if graph is None else "hipGraph replay",
                   "refresh": ("full (synchronous layer)" if args.schedule != "dice" else
                               "Algorithm 4, stride 2: every second step transmits the top-1 pairs only"),
                   "schedule": args.schedule},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "stages": stages,
        "conditional_refresh": cond,
        "ep_shard": ep_shard,
        "calibration": calibration,
        "context": "the paper reports end-to-end DiT-MoE speedups of about 1.2x (1.26x at most) over synchronous expert "
                   "parallelism on 8 PCIe RTX 4090s, where the two all-to-alls take 62-79 % of a step (Section 3; "
                   "Experiments); another machine and another metric: context only, no baseline for this line",
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
