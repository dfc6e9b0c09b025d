#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

A *step* is one pass of the whole hot path (gate -> conditional-refresh mask -> dispatch ->
grouped expert FFN -> combine) over the 28 stacked layers of the DiT-MoE-XL-shaped workload
(T = 4096 tokens, d = 1152, E = 8, top-2, F = 4608, bf16), i.e. a full denoising step's MoE work.
Every layer has its own seeded weights, activations and buffers, all resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=None, help="override the 28 layers (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy five times (reference for scaling HBM counters)")
    ap.add_argument("--refresh-sweep", action="store_true",
                    help="also time the 512px conditional-communication workload (T=8192) at refresh fractions "
                         "25/50/75/100 %% and report it under 'conditional_refresh'")
    ap.add_argument("--ep-shard", action="store_true",
                    help="also time the grouped FFN over one expert-parallel shard's receive buffer (16384 rows from "
                         "four source ranks, four local experts under a Zipf load, d=2048, F=8192) and report it under "
                         "'ep_shard'")
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
    ap.add_argument("--workload", choices=["xl", "g"], default="xl",
                    help="xl: DiT-MoE-XL shape x 28 layers (the headline workload); g: DiT-MoE-G shape (16 experts, "
                         "d=1792) x 40 layers")
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
    wl_cfg = 3 if args.workload == "xl" else 6
    c = WL.CONFIGS[wl_cfg]
    n_layers = args.layers or c.layers
    T, d, E, k, F = (args.tokens or c.T), c.d, c.E, c.k, c.F
    n_shared = args.n_shared
    N = T * (k + n_shared)          # (token, slot) pairs: k routed slots and one per shared expert

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
                layers.append(dict(x=up(li.x), Wg=up(li.Wg), bg=torch.from_numpy(li.bg).to(dev), W1=up(li.W1),
                                   W2=up(li.W2), buf=buf))
            if first == 0:
                cpu_layers = chunk[:n_cpu]
            del chunk
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

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

    # ---- optional HIP graph of one step (the launch sequence is static)
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

    # ---- per-stage timing with events on the launch stream (eager, a few passes)
    stage_names = ["gate", "dispatch", "expert_ffn", "combine"]
    stage_ms = {s: [] for s in stage_names}
    n_passes = 3
    for _ in range(n_passes):
        for L in layers:
            buf = L["buf"]
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
            ev[0].record()
            ctx.moe_gate(L["x"], L["Wg"], L["bg"], buf.scores, buf.expert_idx)
            ev[1].record()
            # as in moe_layer_forward: dispatch writes the index outputs, the FFN gathers the rows itself
            ctx.moe_dispatch(L["x"], buf.expert_idx, None, None, buf.counts, buf.offsets, buf.perm,
                             buf.inv, buf.workspace)
            ev[2].record()
            ctx.moe_expert_ffn_rows(L["x"], buf.perm, buf.offsets, buf.seg_expert, N, L["W1"], None, L["W2"], None,
                                    buf.h_packed, buf.workspace)
            ev[3].record()
            ctx.moe_combine(buf.h_packed, buf.inv, buf.scores, None, None, None, False, buf.y)
            ev[4].record()
            L["ev"] = ev
        torch.cuda.synchronize()
        for L in layers:
            for i, s in enumerate(stage_names):
                stage_ms[s].append(L["ev"][i].elapsed_time(L["ev"][i + 1]))
    avg = {s: float(np.mean(v)) for s, v in stage_ms.items()}
    b = 2
    alg_bytes = {
        "gate": T * d * b + E * d * b + N * 8,
        "dispatch": 16 * N,          # index outputs only; the row gather rides in the FFN's operand load
        "combine": N * d * b + T * d * b + N * 9,
    }
    ffn_flops = 4.0 * N * d * F
    ffn_tflops = ffn_flops / (avg["expert_ffn"] * 1e-3) / 1e12
    stages = {s: {"ms": round(avg[s], 5)} for s in stage_names}
    for s, nbytes in alg_bytes.items():
        gbs = nbytes / (avg[s] * 1e-3) / 1e9
        stages[s].update({"algorithmic_bytes": nbytes, "GB/s": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4)})
    stages["expert_ffn"].update({"flops": ffn_flops, "TFLOP/s": round(ffn_tflops, 1),
                                 "frac_mfma": round(ffn_tflops / PEAK_BF16_TFLOPS, 4)})
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "bench_xl28_hbm_traffic.txt")
    if os.path.exists(tpath) and args.workload == "xl" and n_shared == 0:          # rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this same command (not live)
        for line in open(tpath):
            if line.startswith("ffn_traffic_bytes_per_call:"):
                traffic = int(line.split(":")[1].split()[0])
    roofline = {"kernel": "ffn_gemm_bf16_wide_kernel (GEMM1 + GEMM2 of one moe_expert_ffn_rows call)", "bound": "mfma",
                "achieved": round(ffn_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ffn_tflops / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                "traffic_note": "HBM-side bytes per moe_expert_ffn_rows call from profiles/bench_xl28_hbm_traffic.txt"}

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- optional: Conditional Communication at the 512px shape (two consecutive diffusion steps)
    cond = None
    if args.refresh_sweep:
        c4 = WL.CONFIGS[4]
        li4 = WL.make_layer(4)
        x_prev, x_next = up(li4.x), up(WL.next_step_x(4, li4.x))
        ctx4 = B.Context(c4.T, c4.d, c4.F, c4.E, c4.k, "bf16")
        buf4 = B.LayerBuffers(ctx4, dev, with_cache=True)
        w4 = (up(li4.Wg), None, up(li4.W1), None, up(li4.W2), None)
        cond = []
        for frac in (1.0, 0.75, 0.5, 0.25):
            n_units = int(frac * c4.T + 0.5)
            pol = B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=n_units)
            B.moe_layer_forward(ctx4, buf4, x_prev, *w4, policy=B.Policy(B.REFRESH_ALL))      # fills the cache
            for _ in range(3):
                B.moe_layer_forward(ctx4, buf4, x_next, *w4, policy=pol, max_rows=n_units * c4.k)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 20
            e0.record()
            for _ in range(reps):
                B.moe_layer_forward(ctx4, buf4, x_next, *w4, policy=pol, max_rows=n_units * c4.k)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            cond.append({"refresh_fraction": frac, "policy": "FRACTION_TOKEN", "refreshed_pairs": n_units * c4.k,
                         "ms_per_layer": round(ms, 4), "tokens_per_s": round(c4.T / (ms * 1e-3), 1),
                         "ffn_flops_needed": 4.0 * n_units * c4.k * c4.d * c4.F})
        del buf4, w4

    # ---- optional: the receive side of an expert-parallel shard (segments ordered [source rank][local expert])
    ep_shard = None
    if args.ep_shard:
        ep = WL.make_ep_shard()
        c5 = ep.cfg
        rows, W_ranks, E_loc = ep.x_recv.shape[0], ep.recv_counts.shape[0], ep.recv_counts.shape[1]
        ctx5 = B.Context(rows, c5.d, c5.F, E_loc, 1, "bf16")
        seg_offsets = torch.empty(W_ranks * E_loc + 1, dtype=torch.int32, device=dev)
        seg_expert = torch.empty(W_ranks * E_loc, dtype=torch.int32, device=dev)
        ctx5.moe_ep_segments(torch.from_numpy(np.ascontiguousarray(ep.recv_counts, dtype=np.int32)).to(dev),
                             seg_offsets, seg_expert)
        x5, W1_5, W2_5 = up(ep.x_recv), up(ep.W1), up(ep.W2)
        h5 = torch.empty((rows, c5.d), dtype=torch.bfloat16, device=dev)
        ws5 = torch.empty(ctx5.workspace_bytes(), dtype=torch.uint8, device=dev)
        call = lambda: ctx5.moe_expert_ffn(x5, seg_offsets, seg_expert, rows, W1_5, None, W2_5, None, h5, ws5)
        for _ in range(3):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        flops5 = 4.0 * rows * c5.d * c5.F
        ep_shard = {"rows": rows, "segments": W_ranks * E_loc, "rows_per_local_expert": ep.recv_counts.sum(axis=0).tolist(),
                    "ms_per_call": round(ms, 4), "rows_per_s": round(rows / (ms * 1e-3), 1), "flops": flops5,
                    "TFLOP/s": round(flops5 / (ms * 1e-3) / 1e12, 1),
                    "frac_mfma": round(flops5 / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del x5, W1_5, W2_5, h5, ws5

    # ---- the CPU oracle on a bounded sample of the same workload (layer 0, first tokens)
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O
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
                                f"DiT-MoE-G-shaped layer x {c.layers} (T={T}, d={d}, E={E}, top-{k}, F={F})")
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
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
