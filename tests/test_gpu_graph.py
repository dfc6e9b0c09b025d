"""The layer under HIP-graph capture: the library allocates nothing, never synchronises the host and
enqueues only kernels, so a caller may record one layer step into a graph and replay it.  Checked
here: every replay (not only the first) reproduces, bit for bit, what eager launches of the same
sequence produce -- with the caches of Conditional Communication (Algorithm 4) evolving from replay
to replay, the program's own eager work and synchronisations between the replays, and the result of
one sequence also compared with the oracle."""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import moe_oracle as O
from paper_2411_16786_amd import binding as B
from paper_2411_16786_amd import workloads as WL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _inputs(seed, T, d, steps, dtype, drift=0.2):
    r = np.random.Generator(np.random.PCG64(seed))
    xs = [WL.to_storage(r.standard_normal((T, d), dtype=np.float32), dtype)]
    for _ in range(steps - 1):
        xs.append(WL.to_storage(xs[-1] + np.float32(drift) * r.standard_normal((T, d), dtype=np.float32), dtype))
    return xs


CASES = [
    # name, T, d, E, k, F, dtype, n_shared, policy of the captured step
    ("bf16-half-of-the-tokens", 640, 384, 8, 2, 1536, "bf16", 0, lambda T, k: B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=T // 2)),
    ("bf16-algorithm-4-stride-2", 640, 384, 8, 2, 1536, "bf16", 0, lambda T, k: B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=2)),
    ("bf16-shared-expert-pairs", 384, 256, 4, 2, 1024, "bf16", 1, lambda T, k: B.Policy(B.REFRESH_FRACTION_PAIR, n_units=T * k // 2)),
    ("f32-quarter-of-the-tokens", 96, 64, 4, 2, 256, "f32", 0, lambda T, k: B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=T // 4)),
    ("bf16-synchronous", 512, 384, 16, 2, 1536, "bf16", 0, lambda T, k: None),
]


@pytest.mark.parametrize("name,T,d,E,k,F,dtype,n_shared,make_policy", CASES, ids=[c[0] for c in CASES])
def test_graph_replays_match_eager(name, T, d, E, k, F, dtype, n_shared, make_policy):
    steps = 5
    say(f"graph case {name}: T={T} d={d} E={E} k={k} F={F} {dtype} n_shared={n_shared}")
    x0, Wg, bg, W1, b1, W2, b2 = G.small_inputs(4242, T, d, E + n_shared, F, dtype, bias=True, w_std=0.04)
    Wg, bg = Wg[:E].copy(), bg[:E].copy()
    xs = _inputs(99, T, d, steps, dtype)
    policy = make_policy(T, k)

    def fresh_layer():
        L = G.GpuLayer(xs[0], Wg, bg, W1, b1, W2, b2, k, dtype, with_cache=True, n_shared=n_shared)
        L.forward(B.Policy(B.REFRESH_ALL), fuse_gather=True)          # a synchronous first step fills the caches
        return L

    # ---- eager sequence
    eager = fresh_layer()
    ys_eager, caches_eager = [], []
    for t in range(1, steps):
        y = eager.forward(policy, x=G.to_dev(xs[t], dtype), fuse_gather=True)
        ys_eager.append(y.clone())
        caches_eager.append(eager.buf.H_cache.clone())
    say("  eager sequence done")

    # ---- the same sequence as replays of one captured step that reads a fixed input buffer
    cap = fresh_layer()
    x_in = G.to_dev(xs[1], dtype).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                     # warm-up launch outside the capture
        scratch = G.GpuLayer(xs[0], Wg, bg, W1, b1, W2, b2, k, dtype, with_cache=True, n_shared=n_shared)
        B.moe_layer_forward(scratch.ctx, scratch.buf, x_in, scratch.Wg, scratch.bg, scratch.W1, scratch.b1,
                            scratch.W2, scratch.b2, B.Policy(B.REFRESH_ALL))
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.moe_layer_forward(cap.ctx, cap.buf, x_in, cap.Wg, cap.bg, cap.W1, cap.b1, cap.W2, cap.b2, policy)
    torch.cuda.synchronize()
    # the capture itself runs nothing: the caches still hold the first step
    say("  captured")
    for t in range(1, steps):
        x_in.copy_(G.to_dev(xs[t], dtype))                            # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        junk = (x_in.float() * 2).sum().item()                        # more eager work, and a host read
        assert np.isfinite(junk)
        assert torch.equal(cap.buf.y[:T], ys_eager[t - 1]), f"{name}: replay {t} differs from the eager step"
        assert torch.equal(cap.buf.H_cache, caches_eager[t - 1]), f"{name}: cache after replay {t} differs"
        say(f"  replay {t} equals the eager step")

    # ---- and the sequence is the right one: last step against the oracle fed the same history
    Hc = np.zeros((T, k, d))
    Sc = np.zeros((T, k))
    y_ref = None
    for t in range(steps):
        pol = B.Policy(B.REFRESH_ALL) if t == 0 else policy
        if pol is None:
            r = O.moe_layer(xs[t], Wg, bg, W1, b1, W2, b2, k, n_shared=n_shared)
        else:
            r = O.moe_layer(xs[t], Wg, bg, W1, b1, W2, b2, k, policy=pol.kind, step_t=pol.step_t,
                            stride_n=pol.stride_n, n_units=pol.n_units, H_cache=Hc, S_cache=Sc, n_shared=n_shared)
        y_ref = r.y
    G.assert_close_storage(G.to_np(cap.buf.y[:T]), y_ref, dtype, f"{name}: last replay vs oracle",
                           wide_range=n_shared > 0)
