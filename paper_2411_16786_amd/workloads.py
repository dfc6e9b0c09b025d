"""Seeded synthetic inputs for the five DiT-MoE-shaped workloads.

This module is shared by the GPU tests, the benchmark and the CPU oracle's tests.
It holds no arithmetic of the MoE layer itself: it only draws random tensors of
the shapes and distributions the workloads name, rounds them to the workload's
storage type and returns them as float32 arrays in which every value is exactly
representable in that type (so the same numbers can be uploaded as bf16 and
widened to double without any further rounding).

The paper evaluates on trained DiT-MoE checkpoints (DiT-MoE-XL: 8 experts x 28
layers, DiT-MoE-G: 16 experts x 40 layers; Section 5, Setups); neither weights nor
data are available here, so these tensors stand in for them, as the paper itself
does when it measures latency at other image sizes with re-initialised embeddings
(supplement, "Extending Image Sizes").

Weight layout follows a linear layer's weight (rows are output features):
Wg[E, d], W1[E, F, d], W2[E, d, F].
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class MoEConfig:
    cfg: int
    name: str
    dtype: str          # "f32" or "bf16": storage type of activations and weights
    T: int              # tokens on this device
    d: int              # hidden size
    E: int              # routed experts
    k: int              # activated experts per token (top-K)
    F: int              # expert FFN width
    layers: int = 1
    ep_world: int = 1   # emulated expert-parallel world size (config 5)
    notes: str = ""

    @property
    def N(self) -> int:
        return self.T * self.k


CONFIGS: Dict[int, MoEConfig] = {
    1: MoEConfig(1, "tiny-fp32", "f32", T=64, d=64, E=4, k=2, F=256,
                 notes="batch 1, 8x8 latent patches"),
    2: MoEConfig(2, "dit-moe-s", "bf16", T=2048, d=384, E=16, k=2, F=1536,
                 notes="batch 8 x 256 tokens, LayerNorm-ed inputs, near-uniform load"),
    3: MoEConfig(3, "dit-moe-xl", "bf16", T=4096, d=1152, E=8, k=2, F=4608, layers=28,
                 notes="batch 16 x 256 tokens, router bias gives uneven load, 28 layers"),
    4: MoEConfig(4, "xl-512px-conditional", "bf16", T=8192, d=1152, E=8, k=2, F=4608,
                 notes="batch 8 x 1024 tokens, two consecutive diffusion steps"),
    5: MoEConfig(5, "ep-shard-zipf", "bf16", T=8192, d=2048, E=16, k=2, F=8192, ep_world=4,
                 notes="4 local experts of a 4-way expert-parallel layout, Zipf(1.2) load"),
    # the paper's second model (Section 5.1): 16 experts x 40 layers.  The paper gives no widths;
    # d = 1792 is the published DiT-MoE-G/2 hidden size, F = 4d as in the other workloads.
    6: MoEConfig(6, "dit-moe-g", "bf16", T=4096, d=1792, E=16, k=2, F=7168, layers=40,
                 notes="batch 16 x 256 tokens, router bias gives uneven load, 40 layers"),
}


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of an array whose values are already exact in bf16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_round(a) if dtype == "bf16" else a


def _normal(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return to_storage(a, dtype)


def layer_seed(cfg: int, layer: int = 0, bump: int = 0) -> int:
    return 1000 * cfg + layer + 100000 * bump


def zipf_weights(n: int, s: float = 1.2) -> np.ndarray:
    w = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    return w / w.sum()


@dataclass
class LayerInputs:
    cfg: MoEConfig
    seed: int
    x: np.ndarray                     # [T, d]
    Wg: np.ndarray                    # [E, d]
    bg: Optional[np.ndarray]          # [E] float32 or None
    W1: np.ndarray                    # [E, F, d]
    W2: np.ndarray                    # [E, d, F]
    b1: Optional[np.ndarray] = None   # [E, F] float32 (None = zero)
    b2: Optional[np.ndarray] = None   # [E, d] float32 (None = zero)
    extra: dict = field(default_factory=dict)


def make_weights(c: MoEConfig, rng: np.random.Generator, E: Optional[int] = None):
    E = c.E if E is None else E
    W1 = _normal(rng, (E, c.F, c.d), 0.02, c.dtype)
    W2 = _normal(rng, (E, c.d, c.F), 0.02, c.dtype)
    return W1, W2


def make_layer(cfg: int, layer: int = 0, bump: int = 0, with_experts: bool = True,
               T: Optional[int] = None, n_shared: int = 0) -> LayerInputs:
    """Inputs of one MoE layer of workload ``cfg``.

    ``T`` may shrink the token count (same distributions) for tests that need a
    small case of a big workload's shape.  Draw order is fixed: x, Wg, bg, W1, W2.
    With ``n_shared`` > 0 the weights of that many shared experts (same shape and
    distribution as the routed ones, drawn from a generator of their own so that the
    routed values do not move) follow the routed experts in W1 and W2; the DiT-MoE
    models of Section 5.1 carry two.
    """
    c = CONFIGS[cfg]
    T = c.T if T is None else T
    seed = layer_seed(cfg, layer, bump)
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal((T, c.d), dtype=np.float32)
    if cfg == 2:
        # activations as they leave a LayerNorm without affine parameters
        x = x - x.mean(axis=1, keepdims=True)
        x = x / np.sqrt((x * x).mean(axis=1, keepdims=True))
    x = to_storage(x, c.dtype)
    Wg = _normal(rng, (c.E, c.d), 1.0 / np.sqrt(c.d), c.dtype)
    bg = None
    if cfg in (3, 6):
        bg = (rng.standard_normal(c.E, dtype=np.float32) * np.float32(0.5)).astype(np.float32)
    elif cfg == 5:
        # router bias = log of the Zipf(1.2) weights: expert load follows the Zipf law
        bg = np.log(zipf_weights(c.E, 1.2)).astype(np.float32)
    else:
        rng.standard_normal(1, dtype=np.float32)  # keep the stream position independent of bg
    if with_experts:
        W1, W2 = make_weights(c, rng)
        if n_shared > 0:
            rng_s = np.random.Generator(np.random.PCG64([seed, 0x5AED]))
            W1s, W2s = make_weights(c, rng_s, E=n_shared)
            W1 = np.concatenate([W1, W1s], axis=0)
            W2 = np.concatenate([W2, W2s], axis=0)
    else:
        W1 = W2 = None
    return LayerInputs(c, seed, x, Wg, bg, W1, W2)


def next_step_x(cfg: int, x_prev: np.ndarray, layer: int = 0, bump: int = 0) -> np.ndarray:
    """Activations of the following diffusion step: x_t = x_{t-1} + 0.1 * N(0, 1)."""
    c = CONFIGS[cfg]
    rng = np.random.Generator(np.random.PCG64(layer_seed(cfg, layer, bump) + 500))
    noise = rng.standard_normal(x_prev.shape, dtype=np.float32)
    return to_storage(x_prev + np.float32(0.1) * noise, c.dtype)


@dataclass
class EPShardInputs:
    cfg: MoEConfig
    seed: int
    x_recv: np.ndarray        # [rows, d] receive buffer ordered [source rank][local expert]
    recv_counts: np.ndarray   # [W, E_loc] int32
    row_expert: np.ndarray    # [rows] local expert of each row (for checks)
    W1: np.ndarray            # [E_loc, F, d]
    W2: np.ndarray            # [E_loc, d, F]


def make_ep_shard(rows: int = 16384, bump: int = 0, with_experts: bool = True) -> EPShardInputs:
    """Receive side of shard 0 in a 4-way expert-parallel layout of workload 5.

    Shard 0 holds the four hottest experts of a Zipf(1.2) load over 16.  Each received row's
    local expert is drawn from the Zipf weights restricted to ranks 1-4; its source rank is
    the row's draw index modulo the world size; rows are N(0,1).  The buffer is laid out
    [source rank][local expert] as an all-to-all would deliver it.
    """
    c = CONFIGS[5]
    W = c.ep_world
    E_loc = c.E // W
    seed = layer_seed(5, 0, bump) + 700
    rng = np.random.Generator(np.random.PCG64(seed))
    w = zipf_weights(c.E, 1.2)[:E_loc]
    w = w / w.sum()
    e_draw = rng.choice(E_loc, size=rows, p=w).astype(np.int32)
    src = (np.arange(rows) % W).astype(np.int32)
    order = np.lexsort((np.arange(rows), e_draw, src))      # by (src, local expert, draw index)
    row_expert = e_draw[order]
    recv_counts = np.zeros((W, E_loc), np.int32)
    np.add.at(recv_counts, (src, e_draw), 1)
    x_recv = _normal(rng, (rows, c.d), 1.0, c.dtype)
    if with_experts:
        W1, W2 = make_weights(c, rng, E=E_loc)
    else:
        W1 = W2 = None
    return EPShardInputs(c, seed, x_recv, recv_counts, row_expert, W1, W2)
