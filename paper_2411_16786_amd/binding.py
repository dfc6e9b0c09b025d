"""Thin Python binding of ``libdicemoe.so`` (see ``include/dice_moe.h``).

Argument marshalling only: every function takes torch tensors that live on the GPU, checks
device / dtype / contiguity, and passes their addresses to the C entry point of the same name.
PyTorch is used for device memory and streams, nothing else; there is no CPU fallback -- if the
library is missing the import of this module's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdicemoe.so")

MOE_F32, MOE_BF16 = 0, 1
REFRESH_ALL, REFRESH_ALG4, REFRESH_FRACTION_TOKEN, REFRESH_FRACTION_PAIR, REFRESH_NONE = range(5)
REFRESH_ALG4_HIGH, REFRESH_ALG4_RANDOM = 5, 6      # ablation variants (n_units carries RANDOM's seed)

MOE_OK = 0
MOE_ERR_NULL, MOE_ERR_SHAPE, MOE_ERR_DTYPE, MOE_ERR_POLICY = -1, -2, -3, -4
MOE_ERR_WORKSPACE, MOE_ERR_CACHE_COLD, MOE_ERR_HIP = -5, -6, -7

EXPORTS = ["moe_create", "moe_destroy", "moe_workspace_bytes", "moe_last_error", "moe_status_string",
           "moe_gate", "moe_policy_refreshed_pairs", "moe_conditional_refresh", "moe_dispatch", "moe_dispatch_noalloc", "moe_expert_ffn", "moe_expert_ffn_rows",
           "moe_expert_ffn_commit", "moe_expert_ffn_status", "moe_expert_ffn_between_event", "moe_calibrate_copy",
           "moe_calibrate_mfma", "moe_combine", "moe_ep_segments"]


class MoeShape(ctypes.Structure):
    _fields_ = [("T_max", ctypes.c_int32), ("d", ctypes.c_int32), ("F", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("renorm_topk", ctypes.c_int32), ("n_shared", ctypes.c_int32)]


class MoePolicy(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("step_t", ctypes.c_int32), ("stride_n", ctypes.c_int32),
                ("n_units", ctypes.c_int32), ("use_fresh_scores", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{text} (status {status})")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load the C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run paper_2411_16786_amd/build.py (hipcc, gfx950)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.moe_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(MoeShape)]
        L.moe_destroy.argtypes = [vp]
        L.moe_workspace_bytes.argtypes = [vp]
        L.moe_workspace_bytes.restype = ctypes.c_size_t
        L.moe_last_error.argtypes = [vp]
        L.moe_last_error.restype = ctypes.c_char_p
        L.moe_status_string.argtypes = [ctypes.c_int]
        L.moe_status_string.restype = ctypes.c_char_p
        L.moe_gate.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        L.moe_policy_refreshed_pairs.argtypes = [vp, ctypes.POINTER(MoePolicy), i32, ctypes.POINTER(i32),
                                                 ctypes.POINTER(i32)]
        L.moe_conditional_refresh.argtypes = [vp, vp, vp, i32, ctypes.POINTER(MoePolicy), vp, vp, vp, vp]
        L.moe_dispatch.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.moe_dispatch_noalloc.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.moe_expert_ffn.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.moe_expert_ffn_rows.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.moe_expert_ffn_commit.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        L.moe_expert_ffn_status.argtypes = [vp, vp, vp]
        L.moe_expert_ffn_between_event.argtypes = [vp, vp]
        L.moe_calibrate_copy.argtypes = [vp, vp, ctypes.c_size_t, i32, vp]
        L.moe_calibrate_mfma.argtypes = [vp, vp, i32, i32, vp]
        L.moe_combine.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp]
        L.moe_ep_segments.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        for name in EXPORTS:
            getattr(L, name)          # AttributeError if the library lacks a declared entry point
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


@dataclass
class Policy:
    kind: int = REFRESH_ALL
    step_t: int = 0
    stride_n: int = 1
    n_units: int = 0
    use_fresh_scores: bool = False

    def c(self) -> MoePolicy:
        return MoePolicy(self.kind, self.step_t, self.stride_n, self.n_units, int(self.use_fresh_scores))


class Context:
    """Owns one ``moe_ctx``; methods carry the names of the C entry points."""

    def __init__(self, T_max: int, d: int, F: int, E: int, k: int, dtype: str = "bf16",
                 renorm_topk: bool = False, n_shared: int = 0):
        self.T_max, self.d, self.F, self.E, self.k = T_max, d, F, E, k
        self.n_shared = n_shared
        self.slots = k + n_shared            # columns of every per-pair array
        self.experts = E + n_shared          # expert ids in use (shared experts last)
        self.dtype_name = dtype
        self.torch_dtype = {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]
        shape = MoeShape(T_max, d, F, E, k, MOE_BF16 if dtype == "bf16" else MOE_F32, int(renorm_topk), n_shared)
        self._h = ctypes.c_void_p()
        rc = lib().moe_create(ctypes.byref(self._h), ctypes.byref(shape))
        if rc != MOE_OK:
            raise MoeError(rc, "moe_create: " + lib().moe_status_string(rc).decode())

    def __del__(self):
        h = getattr(self, "_h", None)
        if h is not None and h.value:
            try:
                lib().moe_destroy(h)
            except Exception:          # interpreter shutdown: the module's globals may be gone already
                pass
            self._h = ctypes.c_void_p()

    def _check(self, rc: int):
        if rc != MOE_OK:
            raise MoeError(rc, lib().moe_last_error(self._h).decode() or lib().moe_status_string(rc).decode())

    def workspace_bytes(self) -> int:
        return lib().moe_workspace_bytes(self._h)

    def moe_policy_refreshed_pairs(self, policy: Policy, T: int):
        """(refreshed pairs incl. shared-expert slots, routed ones among them) for T tokens, from the
        library (Algorithm 4's count is the library's arithmetic, not the binding's)."""
        pol = policy.c()
        n_pairs, n_routed = ctypes.c_int32(), ctypes.c_int32()
        self._check(lib().moe_policy_refreshed_pairs(self._h, ctypes.byref(pol), T, ctypes.byref(n_pairs),
                                                     ctypes.byref(n_routed)))
        return n_pairs.value, n_routed.value

    def moe_gate(self, x, Wg, bg, scores, expert_idx, probs_all=None, logits=None):
        T = x.shape[0]
        self._check(lib().moe_gate(self._h, _ptr(x, self.torch_dtype), _ptr(Wg, self.torch_dtype),
                                   _ptr(bg, torch.float32), T, _ptr(scores, torch.float32),
                                   _ptr(expert_idx, torch.int32), _ptr(probs_all, torch.float32),
                                   _ptr(logits, torch.float32), _stream()))

    def moe_conditional_refresh(self, scores, expert_idx, policy: Policy, mask, n_refresh, workspace):
        T = scores.shape[0]
        pol = policy.c()
        self._check(lib().moe_conditional_refresh(self._h, _ptr(scores, torch.float32),
                                                  _ptr(expert_idx, torch.int32), T, ctypes.byref(pol),
                                                  _ptr(mask, torch.uint8), _ptr(n_refresh, torch.int32),
                                                  _ptr(workspace), _stream()))

    def moe_dispatch(self, x, expert_idx, mask, x_packed, counts, offsets, perm, inv, workspace):
        T = x.shape[0]
        self._check(lib().moe_dispatch(self._h, _ptr(x, self.torch_dtype), _ptr(expert_idx, torch.int32),
                                       _ptr(mask, torch.uint8), T, _ptr(x_packed, self.torch_dtype),
                                       _ptr(counts, torch.int32), _ptr(offsets, torch.int32),
                                       _ptr(perm, torch.int32), _ptr(inv, torch.int32), _ptr(workspace),
                                       _stream()))

    def moe_dispatch_noalloc(self, x, expert_idx, mask, x_packed, counts, offsets, perm, inv):
        T = expert_idx.shape[0]
        self._check(lib().moe_dispatch_noalloc(self._h, _ptr(x, self.torch_dtype), _ptr(expert_idx, torch.int32),
                                               _ptr(mask, torch.uint8), T, _ptr(x_packed, self.torch_dtype),
                                               _ptr(counts, torch.int32), _ptr(offsets, torch.int32),
                                               _ptr(perm, torch.int32), _ptr(inv, torch.int32), _stream()))

    def moe_expert_ffn(self, x_packed, seg_offsets, seg_expert, max_rows, W1, b1, W2, b2, h_packed, workspace):
        n_seg = seg_expert.shape[0]
        self._check(lib().moe_expert_ffn(self._h, _ptr(x_packed, self.torch_dtype),
                                         _ptr(seg_offsets, torch.int32), _ptr(seg_expert, torch.int32), n_seg,
                                         max_rows, _ptr(W1, self.torch_dtype), _ptr(b1, torch.float32),
                                         _ptr(W2, self.torch_dtype), _ptr(b2, torch.float32),
                                         _ptr(h_packed, self.torch_dtype), _ptr(workspace), _stream()))

    def moe_expert_ffn_rows(self, x, row_pairs, seg_offsets, seg_expert, max_rows, W1, b1, W2, b2, h_packed,
                            workspace):
        n_seg = seg_expert.shape[0]
        self._check(lib().moe_expert_ffn_rows(self._h, _ptr(x, self.torch_dtype), _ptr(row_pairs, torch.int32),
                                              _ptr(seg_offsets, torch.int32), _ptr(seg_expert, torch.int32), n_seg,
                                              max_rows, _ptr(W1, self.torch_dtype), _ptr(b1, torch.float32),
                                              _ptr(W2, self.torch_dtype), _ptr(b2, torch.float32),
                                              _ptr(h_packed, self.torch_dtype), _ptr(workspace), _stream()))

    def moe_expert_ffn_commit(self, x_rows, row_pairs, out_pairs, seg_offsets, seg_expert, max_rows, W1, b1, W2, b2,
                              scores, mask, H_buffer, S_buffer, workspace, T=None):
        n_seg = seg_expert.shape[0]
        T = scores.shape[0] if T is None else T
        self._check(lib().moe_expert_ffn_commit(self._h, _ptr(x_rows, self.torch_dtype), _ptr(row_pairs, torch.int32),
                                                _ptr(out_pairs, torch.int32), _ptr(seg_offsets, torch.int32),
                                                _ptr(seg_expert, torch.int32), n_seg, max_rows,
                                                _ptr(W1, self.torch_dtype), _ptr(b1, torch.float32),
                                                _ptr(W2, self.torch_dtype), _ptr(b2, torch.float32),
                                                _ptr(scores, torch.float32), _ptr(mask, torch.uint8), T,
                                                _ptr(H_buffer, self.torch_dtype), _ptr(S_buffer, torch.float32),
                                                _ptr(workspace), _stream()))

    def moe_expert_ffn_status(self, workspace):
        """Waits for the current stream; raises MoeError (MOE_ERR_SHAPE) if the last expert FFN call
        with this workspace was given a max_rows smaller than its segment table."""
        self._check(lib().moe_expert_ffn_status(self._h, _ptr(workspace), _stream()))

    def moe_expert_ffn_between_event(self, event):
        """``event``: a recorded-once ``torch.cuda.Event(enable_timing=True)`` (or None to stop)."""
        self._check(lib().moe_expert_ffn_between_event(self._h, None if event is None else event.cuda_event))

    def moe_combine(self, h_packed, inv, scores, mask, H_cache, S_cache, use_fresh_scores, y):
        T = scores.shape[0]
        self._check(lib().moe_combine(self._h, _ptr(h_packed, self.torch_dtype), _ptr(inv, torch.int32),
                                      _ptr(scores, torch.float32), _ptr(mask, torch.uint8), T,
                                      _ptr(H_cache, self.torch_dtype), _ptr(S_cache, torch.float32),
                                      int(bool(use_fresh_scores)), _ptr(y, self.torch_dtype), _stream()))

    def moe_ep_segments(self, recv_counts, seg_offsets, seg_expert):
        W, E_loc = recv_counts.shape
        self._check(lib().moe_ep_segments(self._h, _ptr(recv_counts, torch.int32), W, E_loc,
                                          _ptr(seg_offsets, torch.int32), _ptr(seg_expert, torch.int32),
                                          _stream()))


class LayerBuffers:
    """Device buffers of one MoE layer call, allocated once with torch (worst-case sizes)."""

    def __init__(self, ctx: Context, device="cuda", with_cache: bool = False, with_debug: bool = False,
                 workspace: Optional[torch.Tensor] = None):
        T, k, d, E = ctx.T_max, ctx.slots, ctx.d, ctx.experts
        N = T * k
        dt = ctx.torch_dtype
        dev = device
        self.scores = torch.empty((T, k), dtype=torch.float32, device=dev)
        self.expert_idx = torch.empty((T, k), dtype=torch.int32, device=dev)
        self.mask = torch.empty((T, k), dtype=torch.uint8, device=dev)
        self.n_refresh = torch.zeros(1, dtype=torch.int32, device=dev)
        self.x_packed = torch.zeros((N, d), dtype=dt, device=dev)
        self.h_packed = torch.zeros((N, d), dtype=dt, device=dev)
        self.counts = torch.empty(E, dtype=torch.int32, device=dev)
        self.offsets = torch.empty(E + 1, dtype=torch.int32, device=dev)
        self.perm = torch.empty(N, dtype=torch.int32, device=dev)
        self.inv = torch.empty(N, dtype=torch.int32, device=dev)
        self.seg_expert = torch.arange(E, dtype=torch.int32, device=dev)
        self.y = torch.empty((T, d), dtype=dt, device=dev)
        self.workspace = workspace if workspace is not None else torch.empty(
            ctx.workspace_bytes(), dtype=torch.uint8, device=dev)
        self.H_cache = torch.zeros((T, k, d), dtype=dt, device=dev) if with_cache else None
        self.S_cache = torch.zeros((T, k), dtype=torch.float32, device=dev) if with_cache else None
        self.probs = torch.empty((T, ctx.E), dtype=torch.float32, device=dev) if with_debug else None
        self.logits = torch.empty((T, ctx.E), dtype=torch.float32, device=dev) if with_debug else None


def moe_layer_forward(ctx: Context, buf: LayerBuffers, x, Wg, bg, W1, b1, W2, b2,
                      policy: Optional[Policy] = None, max_rows: Optional[int] = None, fuse_gather: bool = True,
                      rows_to_cache: Optional[bool] = None):
    """Enqueue one MoE layer (gate -> refresh -> dispatch -> expert FFN -> combine) on the current
    stream.  With ``policy`` None the layer is synchronous and touches no cache; otherwise the
    mask of ``policy`` is applied and ``buf`` must hold caches.  ``max_rows`` bounds the number of
    refreshed pairs (it sizes the FFN launch and picks its tile shape); by default it is the count
    the policy implies, T*k for the synchronous layer.  With ``fuse_gather`` (default) dispatch
    writes its index outputs only and the FFN reads the token rows through ``perm``; otherwise
    ``buf.x_packed`` is materialised first (the send buffer of the expert-parallel layout).  With
    ``rows_to_cache`` (default whenever there is a policy, the gather is fused and the shape has no
    shared experts) the expert call scatters the refreshed rows straight into ``buf.H_cache`` and the
    combine reads every row from there: same results bit for bit, ``buf.h_packed`` stays unwritten."""
    T = x.shape[0]
    N = T * ctx.slots
    if max_rows is None and policy is not None:
        max_rows = ctx.moe_policy_refreshed_pairs(policy, T)[0]
    ctx.moe_gate(x, Wg, bg, buf.scores[:T], buf.expert_idx[:T], buf.probs, buf.logits)
    mask = None
    if policy is not None:
        ctx.moe_conditional_refresh(buf.scores[:T], buf.expert_idx[:T], policy, buf.mask[:T], buf.n_refresh,
                                    buf.workspace)
        mask = buf.mask[:T]
    rows = N if max_rows is None else max_rows
    if rows_to_cache is None:
        rows_to_cache = policy is not None and fuse_gather and ctx.n_shared == 0
    if rows_to_cache:
        if policy is None or not fuse_gather or ctx.n_shared != 0:
            raise ValueError("rows_to_cache needs a policy (caches), the fused gather and no shared experts")
        ctx.moe_dispatch(x, buf.expert_idx[:T], mask, None, buf.counts, buf.offsets, buf.perm, buf.inv,
                         buf.workspace)
        ctx.moe_expert_ffn_commit(x, buf.perm, buf.perm, buf.offsets, buf.seg_expert, rows, W1, b1, W2, b2,
                                  None, mask, buf.H_cache, None, buf.workspace, T=T)
        ctx.moe_combine(None, buf.inv, buf.scores[:T], mask, buf.H_cache, buf.S_cache,
                        bool(policy.use_fresh_scores), buf.y[:T])
        return buf.y[:T]
    if fuse_gather:
        ctx.moe_dispatch(x, buf.expert_idx[:T], mask, None, buf.counts, buf.offsets, buf.perm, buf.inv,
                         buf.workspace)
        ctx.moe_expert_ffn_rows(x, buf.perm, buf.offsets, buf.seg_expert, rows, W1, b1, W2, b2, buf.h_packed,
                                buf.workspace)
    else:
        ctx.moe_dispatch(x, buf.expert_idx[:T], mask, buf.x_packed, buf.counts, buf.offsets, buf.perm, buf.inv,
                         buf.workspace)
        ctx.moe_expert_ffn(buf.x_packed, buf.offsets, buf.seg_expert, rows, W1, b1, W2, b2, buf.h_packed,
                           buf.workspace)
    use_fresh = bool(policy.use_fresh_scores) if policy is not None else False
    ctx.moe_combine(buf.h_packed, buf.inv, buf.scores[:T], mask,
                    buf.H_cache if policy is not None else None,
                    buf.S_cache if policy is not None else None, use_fresh, buf.y[:T])
    return buf.y[:T]


def moe_calibrate_copy(dst: torch.Tensor, src: torch.Tensor, workgroups: int):
    rc = lib().moe_calibrate_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), workgroups, _stream())
    if rc != MOE_OK:
        raise MoeError(rc, "moe_calibrate_copy")


def moe_calibrate_mfma(operands: torch.Tensor, sink: torch.Tensor, iters: int, workgroups: int):
    rc = lib().moe_calibrate_mfma(_ptr(operands), _ptr(sink, torch.float32), iters, workgroups, _stream())
    if rc != MOE_OK:
        raise MoeError(rc, "moe_calibrate_mfma")
