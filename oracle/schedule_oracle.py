"""CPU oracle of the step-level schedules: synchronous expert parallelism (Algorithm 1), displaced
expert parallelism (Algorithm 2) and interweaved parallelism (Algorithm 3), each with the
Conditional Communication decision of Algorithm 4 and with Selective Synchronization (Section 4.2,
"Selectively Synchronize Vulnerable Layers") as a per-layer choice of schedule.

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module.  It shares nothing with the GPU library.

On one device an "asynchronous all-to-all" moves nothing; what the schedules fix is WHICH step's
activations each operation sees.  A handle that is waited for in the same step carries this step's
data; a handle waited for in the next step (``h^prev``) carries the previous step's.  Each layer
keeps the state those handles imply:

  * ``H`` [T, k, d], ``S`` [T, k]: the combined expert outputs (and the router scores that go with
    them) that have arrived, i.e. what ``wait(h_c^prev)`` returns; the persistent combine buffer
    of Section 4.1.  Pairs that Algorithm 4 does not transmit keep their older entry.
  * ``pending`` (displaced only): the dispatch launched in the previous step, i.e. what
    ``wait(h_d^prev)`` returns.  Interweaved parallelism has no such buffer (Section 4.1: it
    stores only the combined results).

Everything is float64 and built from the routines of ``moe_oracle`` (router, Algorithm 4 mask,
dispatch, expert FFN, combine), taken in the order the algorithms list them.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import moe_oracle as O

SYNC, DISPLACED, INTERWEAVED = "sync", "displaced", "interweaved"


@dataclass
class Weights:
    Wg: np.ndarray
    bg: Optional[np.ndarray]
    W1: np.ndarray                 # E routed experts, then n_shared shared ones
    b1: Optional[np.ndarray]
    W2: np.ndarray
    b2: Optional[np.ndarray]


@dataclass
class Dispatched:
    """Result of one step's dispatch: the packed rows and the tables that describe them."""
    x_d: np.ndarray                # [R, d]
    offsets: np.ndarray            # [E + 1]
    perm: np.ndarray               # [R] pair ids
    s: np.ndarray                  # [T, k] router scores of that step
    mask: np.ndarray               # [T, k] Algorithm 4 decision of that step


class LayerState:
    def __init__(self, T: int, k: int, d: int):
        self.H = np.zeros((T, k, d))
        self.S = np.zeros((T, k))
        self.pending: Optional[Dispatched] = None


@dataclass
class PolicyArgs:
    policy: int = O.REFRESH_ALL
    step_t: int = 0
    stride_n: int = 1
    n_units: int = 0
    use_fresh_scores: bool = False


def _split(w: Weights, n_shared: int):
    E = np.asarray(w.Wg).shape[0]
    cut = lambda a, lo, hi: None if a is None else np.asarray(a)[lo:hi]
    routed = (cut(w.W1, 0, E), cut(w.b1, 0, E), cut(w.W2, 0, E), cut(w.b2, 0, E))
    shared = (cut(w.W1, E, E + n_shared), cut(w.b1, E, E + n_shared), cut(w.W2, E, E + n_shared),
              cut(w.b2, E, E + n_shared))
    return E, routed, shared


def _route(x, w: Weights, k: int, pol: PolicyArgs, renorm_topk: bool):
    """router + Algorithm 4 + dispatch of this step's activations."""
    E = np.asarray(w.Wg).shape[0]
    z = O.router_logits(x, w.Wg, w.bg)
    idx = O.topk(z, k)
    _, s = O.scores(z, idx, renorm_topk)
    mask, _ = O.refresh_mask(s, pol.policy, pol.step_t, pol.stride_n, pol.n_units)
    _, offsets, perm, _ = O.dispatch(idx, mask, E)
    return Dispatched(O.pack_rows(x, perm, k), offsets, perm, s, mask)


def _expert_and_arrive(st: LayerState, disp: Dispatched, routed, E: int):
    """x_e <- expert(x_d); async_combine(x_e): the rows land in the persistent buffer, where the
    next step's wait finds them, together with the scores of the step they were routed in."""
    W1, b1, W2, b2 = routed
    x_e = O.expert_ffn(disp.x_d, disp.offsets, np.arange(E, dtype=np.int32), W1, b1, W2, b2)
    T, k, d = st.H.shape
    Hf, Sf = st.H.reshape(T * k, d), st.S.reshape(T * k)
    Hf[disp.perm] = x_e
    Sf[disp.perm] = disp.s.reshape(T * k)[disp.perm]


def _scale(st: LayerState, s_now: np.ndarray, use_fresh_scores: bool) -> np.ndarray:
    """x <- scale(x_c, s) on the arrived buffer: the stale scores that belong to the buffered
    outputs (the paper's choice, "Expert Score Scaling") or this step's."""
    s = s_now if use_fresh_scores else st.S
    return (s[:, :, None] * st.H).sum(axis=1)


def layer_step(schedule: str, st: LayerState, x, w: Weights, k: int, pol: PolicyArgs = PolicyArgs(),
               n_shared: int = 0, renorm_topk: bool = False) -> np.ndarray:
    """One layer in one diffusion step under ``schedule``; returns the MoE output y [T, d]
    (float64) and advances ``st``.  The shared experts' dense result on this step's x is added
    under every schedule: they are replicated, hence never stale (supplement, "Influence of
    Shared Experts")."""
    E, routed, shared = _split(w, n_shared)
    y_shared = O.shared_experts(x, *shared) if n_shared else 0.0
    if schedule == SYNC:
        # Algorithm 1 (with Algorithm 4's reuse of cached outputs): everything within the step
        r = O.moe_layer(x, w.Wg, w.bg, *routed, k, renorm_topk=renorm_topk, policy=pol.policy, step_t=pol.step_t,
                        stride_n=pol.stride_n, n_units=pol.n_units, H_cache=st.H, S_cache=st.S,
                        use_fresh_scores=pol.use_fresh_scores)
        st.pending = Dispatched(r.x_packed, r.offsets, r.perm, r.s, r.mask)   # a later displaced step waits on it
        return r.y + y_shared
    now = _route(x, w, k, pol, renorm_topk)                  # [s, idx] <- router(x); h_d <- async_dispatch(x, idx)
    if schedule == INTERWEAVED:
        # Algorithm 3: x_c <- wait(h_c^prev) is what arrived before this step's expert ran ...
        y = _scale(st, now.s, pol.use_fresh_scores)
        # ... the dispatch is waited for within the step, the expert runs on THIS step's rows,
        # and its combine is collected in the next step
        _expert_and_arrive(st, now, routed, E)
        st.pending = None
        return y + y_shared
    if schedule == DISPLACED:
        # Algorithm 2: x_d <- wait(h_d^prev): the expert sees the previous step's dispatch;
        # x_c <- wait(h_c^prev): scale sees the combine launched in the previous step
        if st.pending is None:
            raise ValueError("displaced step without a previous dispatch (run a synchronous step first)")
        y = _scale(st, now.s, pol.use_fresh_scores)
        _expert_and_arrive(st, st.pending, routed, E)
        st.pending = now
        return y + y_shared
    raise ValueError(f"unknown schedule {schedule!r}")


def run_stack(x0_steps: Sequence[np.ndarray], layers: List[Weights], k: int, schedule: str, warmup: int = 1,
              sync_layers: Sequence[int] = (), policy_for_step=None, n_shared: int = 0, record=None):
    """A stack of MoE layers over several diffusion steps.  Layer l+1 reads x + y of layer l (a
    residual connection; attention is not part of this path).  The first ``warmup`` steps are
    synchronous (supplement, "Setup": all asynchronous methods start with synchronised steps),
    and so are the layers in ``sync_layers`` in every step (Selective Synchronization).
    ``policy_for_step(t)`` gives the Algorithm 4 arguments of step t (default: transmit all).
    Activations between layers are kept in float32 (the oracle's input type).
    Returns the stack output of every step; ``record(t, l, x, y)`` sees every layer call."""
    T, d = x0_steps[0].shape
    states = [LayerState(T, k, d) for _ in layers]
    outs = []
    for t, x in enumerate(x0_steps):
        x = np.asarray(x, np.float32)
        for l, w in enumerate(layers):
            sched = SYNC if (t < warmup or l in sync_layers) else schedule
            pol = policy_for_step(t) if policy_for_step else PolicyArgs()
            if t < warmup:
                pol = PolicyArgs(use_fresh_scores=pol.use_fresh_scores)
            y = layer_step(sched, states[l], x, w, k, pol, n_shared)
            if record:
                record(t, l, x, y)
            x = (x.astype(np.float64) + y).astype(np.float32)
        outs.append(x)
    return outs, states
