"""Pins of the schedule oracle (Algorithms 1-3 with Algorithm 4, Selective Synchronization) against
what the paper states about them: the staleness each schedule introduces (Section 4.1: displaced =
1 step for dispatch + 1 for combine, interweaved = 0 + 1), which buffers each keeps, that shared
experts stay fresh, and fixed points.  The reference side of every pin is the single-layer oracle
(pinned on its own in test_oracle_pins.py) applied to the recorded input of the step the paper
names, or a per-token restatement; none re-runs the schedule code."""
import math

import numpy as np
import pytest

from oracle import moe_oracle as O
from oracle import schedule_oracle as SO


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def make_weights(seed, d=16, E=4, F=24, n_shared=0):
    r = rng(seed)
    n = E + n_shared
    return SO.Weights(Wg=r.standard_normal((E, d), dtype=np.float32) / np.float32(math.sqrt(d)),
                      bg=r.standard_normal(E, dtype=np.float32) * np.float32(0.5),
                      W1=r.standard_normal((n, F, d), dtype=np.float32) * np.float32(0.2),
                      b1=r.standard_normal((n, F), dtype=np.float32) * np.float32(0.1),
                      W2=r.standard_normal((n, d, F), dtype=np.float32) * np.float32(0.2),
                      b2=r.standard_normal((n, d), dtype=np.float32) * np.float32(0.1))


def trajectory(seed, steps, T=24, d=16, drift=0.3):
    r = rng(seed)
    xs = [r.standard_normal((T, d), dtype=np.float32)]
    for _ in range(steps - 1):
        xs.append(xs[-1] + np.float32(drift) * r.standard_normal((T, d), dtype=np.float32))
    return xs


def routed_layer(x, w, k):
    E = w.Wg.shape[0]
    return O.moe_layer(x, w.Wg, w.bg, w.W1[:E], w.b1[:E], w.W2[:E], w.b2[:E], k)


def test_single_layer_staleness_is_one_step_interweaved_two_steps_displaced():
    w, k = make_weights(1), 2
    xs = trajectory(2, 6)
    sync = [routed_layer(x, w, k).y for x in xs]
    T, d = xs[0].shape
    for schedule, lag in ((SO.INTERWEAVED, 1), (SO.DISPLACED, 2)):
        st = SO.LayerState(T, k, d)
        ys = [SO.layer_step(SO.SYNC if t == 0 else schedule, st, x, w, k) for t, x in enumerate(xs)]
        np.testing.assert_array_equal(ys[0], sync[0])                       # warm-up step is Algorithm 1
        for t in range(1, len(xs)):
            src = max(t - lag, 0)              # right after the warm-up only that step's results exist
            np.testing.assert_allclose(ys[t], sync[src], rtol=1e-13, atol=1e-15,
                                       err_msg=f"{schedule}: step {t} must show the layer output of step {src}")
            if t >= 2:
                assert not np.allclose(ys[t], sync[t], rtol=1e-3)           # and it is stale indeed


def test_buffers_kept_by_each_schedule():
    # interweaved keeps only the combined results; displaced also keeps the dispatched rows
    w, k = make_weights(3), 2
    xs = trajectory(4, 3)
    T, d = xs[0].shape
    st_i, st_d = SO.LayerState(T, k, d), SO.LayerState(T, k, d)
    for t, x in enumerate(xs):
        SO.layer_step(SO.SYNC if t == 0 else SO.INTERWEAVED, st_i, x, w, k)
        SO.layer_step(SO.SYNC if t == 0 else SO.DISPLACED, st_d, x, w, k)
    assert st_i.pending is None
    ref = routed_layer(xs[-1], w, k)
    np.testing.assert_array_equal(st_d.pending.x_d, ref.x_packed)            # this step's dispatch, for the next
    np.testing.assert_array_equal(st_d.pending.perm, ref.perm)
    # interweaved: the buffer already holds this step's expert outputs; displaced: the previous step's
    h_now = ref.h_packed[ref.inv.reshape(-1)].reshape(T, k, d)
    np.testing.assert_allclose(st_i.H, h_now, rtol=1e-13)
    prev = routed_layer(xs[-2], w, k)
    np.testing.assert_allclose(st_d.H, prev.h_packed[prev.inv.reshape(-1)].reshape(T, k, d), rtol=1e-13)
    np.testing.assert_array_equal(st_i.S, ref.s)
    np.testing.assert_array_equal(st_d.S, prev.s)
    with pytest.raises(ValueError):
        SO.layer_step(SO.DISPLACED, SO.LayerState(T, k, d), xs[0], w, k)     # nothing to wait for


def test_fresh_score_variant_scales_stale_outputs_with_this_steps_scores():
    w, k = make_weights(5), 2
    xs = trajectory(6, 3)
    T, d = xs[0].shape
    st = SO.LayerState(T, k, d)
    pol = SO.PolicyArgs(use_fresh_scores=True)
    ys = [SO.layer_step(SO.SYNC if t == 0 else SO.INTERWEAVED, st, x, w, k, pol) for t, x in enumerate(xs)]
    prev, now = routed_layer(xs[1], w, k), routed_layer(xs[2], w, k)
    h_prev = prev.h_packed[prev.inv.reshape(-1)].reshape(T, k, d)
    for i in range(T):                      # per token: slot j's stale output times slot j's score of this step
        want = sum(now.s[i, j] * h_prev[i, j] for j in range(k))
        np.testing.assert_allclose(ys[2][i], want, rtol=1e-13, atol=1e-15)


def test_interweaved_with_algorithm_4_mixes_one_step_and_older_entries():
    # stride 2: step 0 synchronous; step 1 transmits slot 0 only; step 2 transmits everything but
    # reads the buffer first: slot 0 from step 1, slot 1 still from step 0; step 3 sees step 2's
    w, k = make_weights(7), 2
    xs = trajectory(8, 4)
    T, d = xs[0].shape
    st = SO.LayerState(T, k, d)
    ys = []
    for t, x in enumerate(xs):
        pol = SO.PolicyArgs(policy=O.REFRESH_ALG4, step_t=t, stride_n=2)
        ys.append(SO.layer_step(SO.SYNC if t == 0 else SO.INTERWEAVED, st, x, w, k, pol))
    r = [routed_layer(x, w, k) for x in xs]
    h = [ri.h_packed[ri.inv.reshape(-1)].reshape(T, k, d) for ri in r]
    np.testing.assert_allclose(ys[1], r[0].y, rtol=1e-13, atol=1e-15)
    want2 = r[1].s[:, [0]] * h[1][:, 0] + r[0].s[:, [1]] * h[0][:, 1]
    np.testing.assert_allclose(ys[2], want2, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(ys[3], r[2].y, rtol=1e-13, atol=1e-15)


def test_displaced_with_algorithm_4_restated_by_hand():
    # stride 2, displaced: the expert at step t runs on the dispatch of step t-1 (its rows, its mask, its
    # scores) and that result is read at step t+1.  Step 0 synchronous (all pairs); dispatch of step 1
    # carries slot 0 only, of step 2 both slots, of step 3 slot 0 only.
    w, k = make_weights(13), 2
    xs = trajectory(14, 6)
    T, d = xs[0].shape
    st = SO.LayerState(T, k, d)
    ys = []
    for t, x in enumerate(xs):
        pol = SO.PolicyArgs(policy=O.REFRESH_ALG4, step_t=t, stride_n=2)
        ys.append(SO.layer_step(SO.SYNC if t == 0 else SO.DISPLACED, st, x, w, k, pol))
    r = [routed_layer(x, w, k) for x in xs]
    h = [ri.h_packed[ri.inv.reshape(-1)].reshape(T, k, d) for ri in r]
    part = lambda t, j: r[t].s[:, [j]] * h[t][:, j]
    close = lambda a, b: np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)
    close(ys[1], part(0, 0) + part(0, 1))          # nothing newer has arrived
    close(ys[2], part(0, 0) + part(0, 1))          # step 1 re-ran the dispatch of step 0
    close(ys[3], part(1, 0) + part(0, 1))          # step 2 ran the dispatch of step 1: slot 0 only
    close(ys[4], part(2, 0) + part(2, 1))          # step 3 ran the dispatch of step 2: both slots
    close(ys[5], part(3, 0) + part(2, 1))          # step 4 ran the dispatch of step 3: slot 0 only


def test_shared_experts_are_fresh_under_every_schedule():
    w, k, ns = make_weights(9, n_shared=2), 2, 2
    E = w.Wg.shape[0]
    xs = trajectory(10, 4)
    T, d = xs[0].shape
    for schedule, lag in ((SO.INTERWEAVED, 1), (SO.DISPLACED, 2)):
        st = SO.LayerState(T, k, d)
        ys = [SO.layer_step(SO.SYNC if t == 0 else schedule, st, x, w, k, n_shared=ns) for t, x in enumerate(xs)]
        t = 3
        fresh_shared = sum(O.expert_ffn(xs[t], [0, T], [E + e], w.W1, w.b1, w.W2, w.b2) for e in range(ns))
        np.testing.assert_allclose(ys[t], routed_layer(xs[t - lag], w, k).y + fresh_shared, rtol=1e-12, atol=1e-14)


def test_stack_fixed_point_selective_sync_and_warmup():
    k, L = 2, 3
    layers = [make_weights(20 + l) for l in range(L)]
    x0 = trajectory(30, 1)[0]
    # a constant input: the synchronous stack repeats itself, and every stale schedule reaches the
    # same output once the staleness has propagated through the layers
    steps = 2 + 2 * L + 1
    sync_out, _ = SO.run_stack([x0] * steps, layers, k, SO.SYNC)
    for schedule in (SO.INTERWEAVED, SO.DISPLACED):
        out, _ = SO.run_stack([x0] * steps, layers, k, schedule, warmup=1)
        np.testing.assert_array_equal(out[-1], sync_out[-1])
    # a moving input: stale schedules differ from the synchronous stack, warm-up steps do not
    xs = trajectory(31, 5)
    sync_out, _ = SO.run_stack(xs, layers, k, SO.SYNC)
    out_i, _ = SO.run_stack(xs, layers, k, SO.INTERWEAVED, warmup=2)
    np.testing.assert_array_equal(out_i[0], sync_out[0]); np.testing.assert_array_equal(out_i[1], sync_out[1])
    assert not np.allclose(out_i[3], sync_out[3], rtol=1e-3)
    # every layer synchronised = the synchronous stack; synchronising the deep layers only leaves
    # those layers exact functions of their (stale-fed) input
    out_all, _ = SO.run_stack(xs, layers, k, SO.INTERWEAVED, warmup=1, sync_layers=range(L))
    for a, b in zip(out_all, sync_out):
        np.testing.assert_array_equal(a, b)
    seen = {}
    SO.run_stack(xs, layers, k, SO.INTERWEAVED, warmup=1, sync_layers=(2,),
                 record=lambda t, l, x, y: seen.__setitem__((t, l), (x.copy(), y.copy())))
    for t in range(1, 5):
        x_in, y = seen[(t, 2)]
        np.testing.assert_array_equal(y, routed_layer(x_in, layers[2], k).y)       # deep layer: fresh
        x_in, y = seen[(t, 0)]
        x_prev, _ = seen[(t - 1, 0)]
        np.testing.assert_allclose(y, routed_layer(x_prev, layers[0], k).y, rtol=1e-13, atol=1e-15)   # shallow: 1 step stale
    # the stack itself: layer l+1 reads x + y of layer l (kept in float32), the step's result is the
    # last layer's x + y, and every step starts from the input given for it
    seen = {}
    outs, _ = SO.run_stack(xs, layers, k, SO.INTERWEAVED, warmup=1,
                           record=lambda t, l, x, y: seen.__setitem__((t, l), (x.copy(), y.copy())))
    for t in range(len(xs)):
        np.testing.assert_array_equal(seen[(t, 0)][0], xs[t])
        assert np.abs(seen[(t, 0)][1]).max() > 1e-3           # a residual of nothing would pin nothing
        for l in range(L):
            x_l, y_l = seen[(t, l)]
            nxt = (x_l.astype(np.float64) + y_l).astype(np.float32)
            np.testing.assert_array_equal(seen[(t, l + 1)][0] if l + 1 < L else outs[t], nxt)
    # errors of the two schedules against the synchronous stack: 1-step staleness hurts less than 2-step
    out_d, _ = SO.run_stack(xs, layers, k, SO.DISPLACED, warmup=1)
    out_i, _ = SO.run_stack(xs, layers, k, SO.INTERWEAVED, warmup=1)
    err = lambda o: np.mean([np.linalg.norm(a - b) for a, b in zip(o[2:], sync_out[2:])])
    assert err(out_i) < err(out_d)
