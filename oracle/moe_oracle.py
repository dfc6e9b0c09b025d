"""ctypes front end of the CPU oracle (``moe_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this module.  It shares nothing with
the GPU library and never imports it.

Every function here only marshals numpy arrays into the C routine of the same
name; the arithmetic lives in ``moe_oracle.c`` (double precision throughout),
which cites the passages of the paper each routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

REFRESH_ALL, REFRESH_ALG4, REFRESH_FRACTION_TOKEN, REFRESH_FRACTION_PAIR, REFRESH_NONE = range(5)
REFRESH_ALG4_HIGH, REFRESH_ALG4_RANDOM = 5, 6      # ablation variants: which slot stays fresh


def build(force: bool = False) -> str:
    """Compile ``moe_oracle.c`` with gcc into ``libmoe_oracle.so`` beside it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
             "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_refresh_mask.restype = ctypes.c_int
        _lib.oracle_dispatch.restype = ctypes.c_int
        _lib.oracle_combine.restype = ctypes.c_int
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def router_logits(x, Wg, bg=None) -> np.ndarray:
    x, Wg = _f32(x), _f32(Wg)
    bg = None if bg is None else _f32(bg)
    T, d = x.shape
    E = Wg.shape[0]
    assert Wg.shape == (E, d)
    z = np.empty((T, E), np.float64)
    lib().oracle_router_logits(_p(x), _p(Wg), _p(bg), T, d, E, _p(z))
    return z


def topk(z, k: int) -> np.ndarray:
    z = _f64(z)
    T, E = z.shape
    assert 1 <= k <= E
    idx = np.empty((T, k), np.int32)
    lib().oracle_topk(_p(z), T, E, k, _p(idx))
    return idx


def scores(z, idx, renorm_topk: bool = False):
    """Returns (p[T,E], s[T,k])."""
    z, idx = _f64(z), _i32(idx)
    T, E = z.shape
    k = idx.shape[1]
    p = np.empty((T, E), np.float64)
    s = np.empty((T, k), np.float64)
    lib().oracle_scores(_p(z), _p(idx), T, E, k, int(renorm_topk), _p(p), _p(s))
    return p, s


def refresh_mask(s, policy: int, step_t: int = 0, stride_n: int = 1, n_units: int = 0):
    """Returns (mask[T,k] uint8, R)."""
    s = _f64(s)
    T, k = s.shape
    mask = np.empty((T, k), np.uint8)
    R = lib().oracle_refresh_mask(_p(s), T, k, policy, step_t, stride_n, n_units, _p(mask))
    if R < 0:
        raise ValueError("invalid refresh policy arguments")
    return mask, R


def mix32(seed: int, token: int) -> int:
    """The counter-based draw of REFRESH_ALG4_RANDOM (see ``moe_oracle.c``)."""
    f = lib().oracle_mix32_export
    f.restype = ctypes.c_uint32
    f.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
    return int(f(seed & 0xFFFFFFFF, token & 0xFFFFFFFF))


def dispatch(idx, mask, E: int):
    """Returns (counts[E], offsets[E+1], perm[R], inv[T,k])."""
    idx = _i32(idx)
    T, k = idx.shape
    mask = None if mask is None else _u8(mask)
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.full(T * k, -1, np.int32)
    inv = np.empty((T, k), np.int32)
    R = lib().oracle_dispatch(_p(idx), _p(mask), T, k, E, _p(counts), _p(offsets), _p(perm), _p(inv))
    return counts, offsets, perm[:R].copy(), inv


def pack_rows(x, perm, k: int) -> np.ndarray:
    x, perm = _f32(x), _i32(perm)
    R, d = perm.shape[0], x.shape[1]
    out = np.empty((R, d), np.float32)
    lib().oracle_pack_rows(_p(x), _p(perm), R, k, d, _p(out))
    return out


def expert_ffn(x_packed, seg_offsets, seg_expert, W1, b1, W2, b2, rows_sel=None) -> np.ndarray:
    """h rows (float64) for every packed row, or only for ``rows_sel``."""
    x_packed, W1, W2 = _f32(x_packed), _f32(W1), _f32(W2)
    b1 = None if b1 is None else _f32(b1)
    b2 = None if b2 is None else _f32(b2)
    seg_offsets, seg_expert = _i32(seg_offsets), _i32(seg_expert)
    n_seg = seg_expert.shape[0]
    assert seg_offsets.shape[0] == n_seg + 1
    E, F, d = W1.shape
    assert W2.shape == (E, d, F) and x_packed.shape[1] == d
    assert seg_offsets[n_seg] <= x_packed.shape[0]
    if rows_sel is None:
        n = int(seg_offsets[n_seg])
        sel = None
    else:
        sel = _i32(rows_sel)
        n = sel.shape[0]
    h = np.zeros((n, d), np.float64)
    lib().oracle_expert_ffn(_p(x_packed), _p(seg_offsets), _p(seg_expert), n_seg, _p(W1), _p(b1),
                            _p(W2), _p(b2), d, F, _p(sel), n, _p(h))
    return h


def combine(h_packed, inv, s, mask, H_cache=None, S_cache=None, use_fresh_scores=False,
            tokens_sel=None) -> np.ndarray:
    """y rows (float64).  ``H_cache`` [T,k,d] / ``S_cache`` [T,k] (float64) are updated in place."""
    h_packed, inv, s = _f64(h_packed), _i32(inv), _f64(s)
    T, k = inv.shape
    d = h_packed.shape[1] if h_packed.ndim == 2 and h_packed.shape[0] > 0 else (
        H_cache.shape[2] if H_cache is not None else h_packed.shape[1])
    mask = None if mask is None else _u8(mask)
    for c in (H_cache, S_cache):
        assert c is None or (c.dtype == np.float64 and c.flags.c_contiguous)
    if tokens_sel is None:
        sel, n = None, T
    else:
        sel = _i32(tokens_sel)
        n = sel.shape[0]
    y = np.empty((n, d), np.float64)
    rc = lib().oracle_combine(_p(h_packed), _p(inv), _p(s), _p(mask), T, k, d, _p(H_cache),
                              _p(S_cache), int(use_fresh_scores), _p(sel), n, _p(y))
    if rc != 0:
        raise ValueError("a reused pair was met with no cache (cold cache)")
    return y


def shared_experts(x, W1s, b1s, W2s, b2s) -> np.ndarray:
    """Sum over the shared experts of their FFN applied to every token, float64 [T, d].

    The DiT-MoE layer carries, beside the routed experts, shared experts that see every token
    (Section 2, "Mixture-of-Experts"; Section 5.1, "Models and Datasets": two of them; supplement,
    "More details of MoE" and its figure).  Their result is added to the routed sum without a gate
    score, and it is computed anew in every step: it never takes part in Conditional Communication
    (supplement, "Influence of Shared Experts").  Written out as the definition, dense:
    out_i = sum_s ( W2s[s] gelu(W1s[s] x_i + b1s[s]) + b2s[s] ), GELU in its exact erf form.
    """
    from scipy.special import erf
    x = _f64(x)
    W1s, W2s = _f64(W1s), _f64(W2s)
    S, F, d = W1s.shape
    assert W2s.shape == (S, d, F) and x.shape[1] == d
    out = np.zeros((x.shape[0], d), np.float64)
    for e in range(S):
        u = x @ W1s[e].T
        if b1s is not None:
            u = u + _f64(b1s)[e][None, :]
        g = 0.5 * u * (1.0 + erf(u / np.sqrt(2.0)))
        h = g @ W2s[e].T
        if b2s is not None:
            h = h + _f64(b2s)[e][None, :]
        out += h
    return out


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def ep_segments(recv_counts):
    """Segment table of an expert-parallel receive buffer ordered [source rank][local expert]."""
    rc = _i32(recv_counts)
    W, E_loc = rc.shape
    seg_offsets = np.empty(W * E_loc + 1, np.int32)
    seg_expert = np.empty(W * E_loc, np.int32)
    lib().oracle_ep_segments(_p(rc), W, E_loc, _p(seg_offsets), _p(seg_expert))
    return seg_offsets, seg_expert


@dataclass
class LayerResult:
    z: np.ndarray
    idx: np.ndarray
    p: np.ndarray
    s: np.ndarray
    mask: np.ndarray
    R: int
    counts: np.ndarray
    offsets: np.ndarray
    perm: np.ndarray
    inv: np.ndarray
    x_packed: np.ndarray
    h_packed: np.ndarray
    y: np.ndarray
    y_shared: Optional[np.ndarray] = None


def moe_layer(x, Wg, bg, W1, b1, W2, b2, k: int, *, renorm_topk=False, policy=REFRESH_ALL,
              step_t=0, stride_n=1, n_units=0, H_cache=None, S_cache=None,
              use_fresh_scores=False, n_shared=0) -> LayerResult:
    """One MoE layer in the order of Algorithm 1, with the Algorithm 4 decision between router
    and dispatch.  Caches (float64) are updated in place when given.  With ``n_shared`` > 0 the
    weight arrays hold E routed experts followed by n_shared shared ones; the shared experts'
    dense result (``shared_experts``) is added to the routed y."""
    E = np.asarray(Wg).shape[0]
    if n_shared:
        assert np.asarray(W1).shape[0] == E + n_shared
        W1s, W2s = np.asarray(W1)[E:], np.asarray(W2)[E:]
        b1s = None if b1 is None else np.asarray(b1)[E:]
        b2s = None if b2 is None else np.asarray(b2)[E:]
        W1, W2 = np.asarray(W1)[:E], np.asarray(W2)[:E]
        b1 = None if b1 is None else np.asarray(b1)[:E]
        b2 = None if b2 is None else np.asarray(b2)[:E]
    z = router_logits(x, Wg, bg)
    idx = topk(z, k)
    p, s = scores(z, idx, renorm_topk)
    mask, R = refresh_mask(s, policy, step_t, stride_n, n_units)
    counts, offsets, perm, inv = dispatch(idx, mask, E)
    xp = pack_rows(x, perm, k)
    h = expert_ffn(xp, offsets, np.arange(E, dtype=np.int32), W1, b1, W2, b2)
    y = combine(h, inv, s, mask, H_cache, S_cache, use_fresh_scores)
    y_shared = None
    if n_shared:
        y_shared = shared_experts(x, W1s, b1s, W2s, b2s)
        y = y + y_shared
    return LayerResult(z, idx, p, s, mask, R, counts, offsets, perm, inv, xp, h, y, y_shared)
