"""Step-level schedules of the MoE layer on one device: synchronous (Algorithm 1), displaced
(Algorithm 2) and interweaved (Algorithm 3) expert parallelism, each with Conditional
Communication (Algorithm 4) and, per layer, Selective Synchronization.

This module only sequences C-ABI calls (and, optionally, puts the deferred expert work on a second
stream); every arithmetic step runs in the library's kernels.  On one device an asynchronous
all-to-all moves nothing: what a schedule fixes is which step's activations each call sees.

  * The persistent combine buffer of Section 4.1 is ``LayerState.H`` / ``.S`` ([T, slots, d] expert
    outputs per (token, slot) pair and the scores that belong to them).  ``moe_combine`` reads it
    with a mask that refreshes nothing (routed slots; shared-expert slots stay fresh), and
    ``moe_expert_ffn_commit`` writes the expert outputs of the pairs Algorithm 4 transmits straight
    into it, after that read: they are what the next step's combine finds.
  * Interweaved: the expert runs on THIS step's rows (read from x through the permutation); 1-step
    staleness, no dispatch buffer.
  * Displaced: the expert runs on the PREVIOUS step's packed rows, kept in a second set of layer
    buffers; 2-step staleness.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as B

SYNC, DISPLACED, INTERWEAVED = "sync", "displaced", "interweaved"


class LayerState:
    """Buffers one layer keeps across diffusion steps."""

    def __init__(self, ctx: B.Context, device="cuda", displaced: bool = False,
                 workspace: Optional[torch.Tensor] = None, side_workspace: Optional[torch.Tensor] = None):
        self.ctx = ctx
        T, kc, d = ctx.T_max, ctx.slots, ctx.d
        self.H = torch.zeros((T, kc, d), dtype=ctx.torch_dtype, device=device)
        self.S = torch.zeros((T, kc), dtype=torch.float32, device=device)
        self.bufs = [B.LayerBuffers(ctx, device, workspace=workspace) for _ in range(2 if displaced else 1)]
        for b in self.bufs:                      # the caches of these buffers are the persistent ones
            b.H_cache, b.S_cache = self.H, self.S
        self.cur = 0
        self.pending = None                      # displaced: (buffers, T, routed rows) of the previous step's dispatch
        # mask that transmits nothing: routed slots 0, shared-expert slots 1
        self.mask_stale = torch.empty((T, kc), dtype=torch.uint8, device=device)
        self._n_tmp = torch.zeros(1, dtype=torch.int32, device=device)
        ctx.moe_conditional_refresh(self.S, None, B.Policy(B.REFRESH_NONE), self.mask_stale, self._n_tmp,
                                    self.bufs[0].workspace)
        self.side_workspace = side_workspace     # hidden activations of the deferred expert call (second stream)
        self.commit_done: Optional[torch.cuda.Event] = None

    @property
    def buf(self) -> B.LayerBuffers:
        return self.bufs[self.cur]


def moe_layer_step(schedule: str, st: LayerState, x, Wg, bg, W1, b1, W2, b2, policy: Optional[B.Policy] = None,
                   side_stream: Optional[torch.cuda.Stream] = None):
    """Enqueue one layer of one diffusion step under ``schedule``; returns y (a view of the layer's
    buffers, valid until the layer's next call).  ``policy`` None transmits every pair.

    With ``side_stream`` the deferred expert call of the asynchronous schedules runs there, after
    this layer's combine, so that it overlaps the following layers' work on the current stream;
    ``st`` then needs a ``side_workspace`` of its own, and x must stay unchanged until that call
    has run (interweaved reads its rows from x)."""
    ctx = st.ctx
    policy = policy if policy is not None else B.Policy(B.REFRESH_ALL)
    T = x.shape[0]
    E, k, ns = ctx.E, ctx.k, ctx.n_shared
    main = torch.cuda.current_stream()
    if st.commit_done is not None:               # the previous step's deferred expert call owns the buffers until done
        main.wait_event(st.commit_done)
        st.commit_done = None
    if schedule == DISPLACED or (schedule == SYNC and len(st.bufs) == 2):
        st.cur ^= 1                              # this step's dispatch must not overwrite the pending one
    buf = st.buf
    if schedule == SYNC:
        # Algorithm 1 with Algorithm 4's cache: the combine writes refreshed pairs through to H / S.
        # The dispatch is materialised when a displaced step may follow (it waits on this dispatch).
        y = B.moe_layer_forward(ctx, buf, x, Wg, bg, W1, b1, W2, b2, policy, fuse_gather=len(st.bufs) == 1)
        st.pending = (buf, T, ctx.moe_policy_refreshed_pairs(policy, T)[1])
        return y

    rows_routed = ctx.moe_policy_refreshed_pairs(policy, T)[1]
    ctx.moe_gate(x, Wg, bg, buf.scores[:T], buf.expert_idx[:T], buf.probs, buf.logits)
    ctx.moe_conditional_refresh(buf.scores[:T], buf.expert_idx[:T], policy, buf.mask[:T], buf.n_refresh, buf.workspace)
    packed = buf.x_packed if schedule == DISPLACED else None
    ctx.moe_dispatch(x, buf.expert_idx[:T], buf.mask[:T], packed, buf.counts, buf.offsets, buf.perm, buf.inv,
                     buf.workspace)
    if ns > 0:
        # shared experts: this step's x, within the step (they are replicated, never stale)
        # (max_rows bounds the packed row ids of the segments, which follow the routed rows)
        ctx.moe_expert_ffn_rows(x, buf.perm, buf.offsets[E:], buf.seg_expert[E:], rows_routed + T * ns, W1, b1, W2, b2,
                                buf.h_packed, buf.workspace)
    # x_c <- wait(h_c^prev); x <- scale(x_c, s): the routed slots come from the persistent buffer
    ctx.moe_combine(buf.h_packed, buf.inv, buf.scores[:T], st.mask_stale[:T], st.H, st.S,
                    bool(policy.use_fresh_scores), buf.y[:T])
    y = buf.y[:T]

    # the expert call whose results the next step collects
    if schedule == INTERWEAVED:
        src, src_T, src_rows = buf, T, rows_routed
        x_rows, row_pairs = x, buf.perm
    else:
        if st.pending is None:
            raise RuntimeError("displaced step without a previous dispatch (run a synchronous step first)")
        src, src_T, src_rows = st.pending
        x_rows, row_pairs = src.x_packed, None
    stream = side_stream if side_stream is not None else main
    workspace = st.side_workspace if side_stream is not None else buf.workspace
    if side_stream is not None:
        if st.side_workspace is None:
            raise RuntimeError("a side stream needs LayerState.side_workspace")
        side_stream.wait_stream(main)            # after this layer's combine has read H / S
    with torch.cuda.stream(stream):
        ctx.moe_expert_ffn_commit(x_rows, row_pairs, src.perm, src.offsets[:E + 1], src.seg_expert[:E], src_rows,
                                  W1, b1, W2, b2, src.scores[:src_T], src.mask[:src_T], st.H, st.S, workspace)
        if side_stream is not None:
            st.commit_done = torch.cuda.Event()
            st.commit_done.record(stream)
    st.pending = (buf, T, rows_routed)
    return y
