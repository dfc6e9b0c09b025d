"""GPU parity of the step-level schedules (Algorithms 1-3 with Algorithm 4 and Selective
Synchronization) against the schedule oracle, and of the expert call that writes into the
persistent combine buffer against the call that writes packed rows.

The stack runs on the GPU (layer l+1 reads x + y of layer l, added by torch in the storage type: a
stand-in for the block around the MoE layer, not part of the path).  The oracle is fed the GPU's own
layer inputs, layer by layer and step by step, and keeps its own buffers: which step's activations
reach which output is checked exactly, while rounding differences cannot pile up across layers."""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import moe_oracle as O
from oracle import schedule_oracle as SO
from paper_2411_16786_amd import binding as B
from paper_2411_16786_amd import schedule as S
from paper_2411_16786_amd import workloads as WL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def make_stack(seed, L, T, d, E, F, dtype, n_shared, steps, drift=0.2):
    layers = []
    for l in range(L):
        x, Wg, bg, W1, b1, W2, b2 = G.small_inputs(seed + l, T, d, E + n_shared, F, dtype, bias=True, w_std=0.03)
        layers.append(SO.Weights(Wg[:E].copy(), bg[:E].copy(), W1, b1, W2, b2))
    r = np.random.Generator(np.random.PCG64(seed + 100))
    xs = [WL.to_storage(r.standard_normal((T, d), dtype=np.float32), dtype)]
    for _ in range(steps - 1):
        xs.append(WL.to_storage(xs[-1] + np.float32(drift) * r.standard_normal((T, d), dtype=np.float32), dtype))
    return layers, xs


def policy_pair(kind, t, T, k):
    """The same Algorithm 4 arguments for the binding and for the oracle."""
    if kind == "all":
        return B.Policy(B.REFRESH_ALL), SO.PolicyArgs()
    if kind == "alg4":
        return (B.Policy(B.REFRESH_ALG4, step_t=t, stride_n=2),
                SO.PolicyArgs(policy=O.REFRESH_ALG4, step_t=t, stride_n=2))
    if kind == "alg4-fresh-scores":
        return (B.Policy(B.REFRESH_ALG4, step_t=t, stride_n=2, use_fresh_scores=True),
                SO.PolicyArgs(policy=O.REFRESH_ALG4, step_t=t, stride_n=2, use_fresh_scores=True))
    raise ValueError(kind)


def run_gpu_stack(ctx, layers_dev, xs, schedule, warmup, sync_layers, pol_kind, k, side):
    L = len(layers_dev)
    dtype = ctx.dtype_name
    T = xs[0].shape[0]
    side_stream = torch.cuda.Stream() if side else None
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    states = [S.LayerState(ctx, G.DEV, displaced=(schedule == S.DISPLACED), workspace=ws,
                           side_workspace=torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
                           if side else None) for _ in range(L)]
    trace = {}
    for t, x_np in enumerate(xs):
        # one input tensor per layer and step parity, so that a deferred expert call can still read it
        x = G.to_dev(x_np, dtype)
        keep = [x]
        for l in range(L):
            sched = S.SYNC if (t < warmup or l in sync_layers) else schedule
            pol, _ = policy_pair(pol_kind, t, T, k)
            if t < warmup:
                pol = B.Policy(B.REFRESH_ALL, use_fresh_scores=pol.use_fresh_scores)
            y = S.moe_layer_step(sched, states[l], x, *layers_dev[l], policy=pol, side_stream=side_stream)
            x_next = x + y
            trace[(t, l)] = (x, y.clone(), states[l].buf.expert_idx.clone())
            x = x_next
            keep.append(x)
        torch.cuda.synchronize()
        for l in range(L):
            trace[(t, l)] += (states[l].H.clone(), states[l].S.clone())
    return trace


CASES = [
    # name, dtype, L, T, d, E, F, k, n_shared, schedule, pol_kind, sync_layers
    ("interweaved-f32", "f32", 2, 96, 64, 4, 128, 2, 0, S.INTERWEAVED, "all", ()),
    ("interweaved-bf16-alg4", "bf16", 3, 512, 128, 8, 256, 2, 0, S.INTERWEAVED, "alg4", ()),
    ("interweaved-bf16-shared", "bf16", 3, 300, 128, 8, 256, 2, 2, S.INTERWEAVED, "alg4", ()),
    ("interweaved-selective-sync", "bf16", 4, 256, 128, 8, 256, 2, 0, S.INTERWEAVED, "all", (2, 3)),
    ("interweaved-fresh-scores", "bf16", 2, 256, 128, 8, 256, 2, 0, S.INTERWEAVED, "alg4-fresh-scores", ()),
    # expert width 1024: the second GEMM splits its reduction, with the scatter and with shared experts' segments
    ("interweaved-split-k-shared", "bf16", 2, 256, 192, 4, 1024, 2, 1, S.INTERWEAVED, "alg4", ()),
    ("displaced-f32", "f32", 2, 96, 64, 4, 128, 2, 0, S.DISPLACED, "all", ()),
    ("displaced-bf16-alg4", "bf16", 3, 512, 128, 8, 256, 2, 0, S.DISPLACED, "alg4", ()),
    ("displaced-bf16-shared", "bf16", 2, 300, 128, 8, 256, 2, 1, S.DISPLACED, "alg4", (1,)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_schedule_stack_against_the_oracle(case):
    name, dtype, L, T, d, E, F, k, ns, schedule, pol_kind, sync_layers = case
    steps, warmup = 5, 1
    layers, xs = make_stack(900 + len(name), L, T, d, E, F, dtype, ns, steps)
    say(f"schedule {name}: L={L} T={T} d={d} E={E}+{ns} F={F} steps={steps}")
    ctx = B.Context(T, d, F, E, k, dtype, n_shared=ns)
    layers_dev = [(G.to_dev(w.Wg, dtype), G.f32_dev(w.bg), G.to_dev(w.W1, dtype), G.f32_dev(w.b1),
                   G.to_dev(w.W2, dtype), G.f32_dev(w.b2)) for w in layers]
    trace = run_gpu_stack(ctx, layers_dev, xs, schedule, warmup, sync_layers, pol_kind, k, side=False)
    states = [SO.LayerState(T, k, d) for _ in range(L)]
    worst = 0.0
    for t in range(steps):
        for l in range(L):
            x_dev, y_dev, idx_dev, H_dev, S_dev = trace[(t, l)]
            x_in = G.to_np(x_dev)
            z = O.router_logits(x_in, layers[l].Wg, layers[l].bg)
            assert G.topk_margin(z, k) >= 2e-6, "near-tie in the routing of a recorded input: pick another seed"
            np.testing.assert_array_equal(G.to_np(idx_dev)[:, :k], O.topk(z, k))
            sched = SO.SYNC if (t < warmup or l in sync_layers) else schedule
            _, pol = policy_pair(pol_kind, t, T, k)
            if t < warmup:
                pol = SO.PolicyArgs(use_fresh_scores=pol.use_fresh_scores)
            y_ref = SO.layer_step(sched, states[l], x_in, layers[l], k, pol, n_shared=ns)
            G.assert_close_storage(G.to_np(y_dev), y_ref, dtype, f"{name} step {t} layer {l} y", wide_range=ns > 0)
            G.assert_close_storage(G.to_np(H_dev)[:, :k].reshape(T * k, d), states[l].H.reshape(T * k, d), dtype,
                                   f"{name} step {t} layer {l} combine buffer")
            np.testing.assert_allclose(G.to_np(S_dev)[:, :k], states[l].S, rtol=5e-5)
            worst = max(worst, np.linalg.norm(G.to_np(y_dev) - y_ref) / np.linalg.norm(y_ref))
    say(f"  worst rel-L2 of a layer output over {steps} steps x {L} layers: {worst:.2e}")
    # the deferred expert call on a second stream: same results bit for bit
    trace2 = run_gpu_stack(ctx, layers_dev, xs, schedule, warmup, sync_layers, pol_kind, k, side=True)
    for key, vals in trace.items():
        for a, b in zip(vals[1:], trace2[key][1:]):
            assert torch.equal(a, b), f"{name}: side-stream run differs at {key}"


@pytest.mark.parametrize("cfg,T,dtype", [(1, None, "f32"), (2, None, "bf16"), (3, None, "bf16"), (3, 700, "bf16")])
def test_commit_writes_the_rows_of_the_packed_call_into_the_pair_buffer(cfg, T, dtype):
    """moe_expert_ffn_commit against moe_expert_ffn_rows (itself checked against the oracle): the
    same h rows, bit for bit, at H[perm[r]]; pairs that were not dispatched keep their old rows; the
    scores of the dispatched pairs are committed.  Covers every tile shape the launcher picks."""
    li, _ = G.pick_layer(cfg, T=T)
    c = li.cfg
    Tn, k, d, E = li.x.shape[0], c.k, c.d, c.E
    say(f"commit: config {cfg} T={Tn}")
    ctx = B.Context(Tn, d, c.F, E, k, dtype)
    buf = B.LayerBuffers(ctx, G.DEV)
    x = G.to_dev(li.x, dtype)
    Wg, bg = G.to_dev(li.Wg, dtype), (G.f32_dev(li.bg) if li.bg is not None else None)
    W1, W2 = G.to_dev(li.W1, dtype), G.to_dev(li.W2, dtype)
    ctx.moe_gate(x, Wg, bg, buf.scores, buf.expert_idx, None, None)
    for pol in (B.Policy(B.REFRESH_ALL), B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=2),
                B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=Tn // 3)):
        ctx.moe_conditional_refresh(buf.scores, buf.expert_idx, pol, buf.mask, buf.n_refresh, buf.workspace)
        ctx.moe_dispatch(x, buf.expert_idx, buf.mask, None, buf.counts, buf.offsets, buf.perm, buf.inv, buf.workspace)
        rows = ctx.moe_policy_refreshed_pairs(pol, Tn)[0]
        ctx.moe_expert_ffn_rows(x, buf.perm, buf.offsets, buf.seg_expert, rows, W1, None, W2, None, buf.h_packed,
                                buf.workspace)
        H = torch.full((Tn, k, d), 3.0, dtype=ctx.torch_dtype, device=G.DEV)
        Sb = torch.full((Tn, k), 3.0, dtype=torch.float32, device=G.DEV)
        ctx.moe_expert_ffn_commit(x, buf.perm, buf.perm, buf.offsets, buf.seg_expert, rows, W1, None, W2, None,
                                  buf.scores, buf.mask, H, Sb, buf.workspace)
        torch.cuda.synchronize()
        R = int(buf.n_refresh.item())
        assert R == rows
        perm = G.to_np(buf.perm)[:R]
        Hn = G.to_np(H).reshape(Tn * k, d)
        np.testing.assert_array_equal(Hn[perm], G.to_np(buf.h_packed)[:R])
        rest = np.ones(Tn * k, bool); rest[perm] = False
        assert (Hn[rest] == 3.0).all()
        Sn, m = G.to_np(Sb), G.to_np(buf.mask)
        np.testing.assert_array_equal(Sn[m != 0], G.to_np(buf.scores)[m != 0])
        assert (Sn[m == 0] == 3.0).all()
