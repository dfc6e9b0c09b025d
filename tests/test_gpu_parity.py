"""Parity of the HIP path (through the C-ABI binding) against the CPU oracle, stage by stage and
end to end, on the same seeded inputs.  Integer results are bit-exact; floating-point results
are held to the tolerances of tests/gpu_util.py."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2411_16786_amd import binding as B
from paper_2411_16786_amd import workloads as WL

import gpu_util as G

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def poison(t: torch.Tensor):
    """Fill an output buffer with NaN before a run, so that assert_written can tell written rows."""
    t.fill_(float("nan"))


def assert_written(t: torch.Tensor, rows: int, what: str):
    """After a run into a poisoned buffer: every element of the first ``rows`` rows was written with a
    finite value, and no row beyond them was touched."""
    a = G.to_np(t)
    assert np.isfinite(a[:rows]).all(), f"{what}: rows left unwritten or not finite: {np.unique(np.nonzero(~np.isfinite(a[:rows]))[0])[:10]}"
    assert np.isnan(a[rows:]).all(), f"{what}: rows beyond the {rows} packed rows were written"


# ----------------------------------------------------------------------------- gate
GATE_CASES = [
    # (name, T, d, E, k, dtype, bias, renorm)
    ("tiny-f32", 64, 64, 4, 2, "f32", False, False),
    ("ragged-f32", 131, 80, 7, 3, "f32", True, True),
    ("s-bf16", 2048, 384, 16, 2, "bf16", False, False),
    ("xl-bf16", 1000, 1152, 8, 2, "bf16", True, False),
    ("k-equals-E", 70, 128, 5, 5, "bf16", True, False),
    ("E64-wide", 300, 2048, 64, 6, "bf16", True, False),     # router rows too large for LDS
    ("E32", 257, 256, 32, 4, "bf16", False, True),
    ("one-token", 1, 64, 4, 1, "f32", False, False),
]


@pytest.mark.parametrize("case", GATE_CASES, ids=[c[0] for c in GATE_CASES])
def test_gate_against_oracle(case):
    name, T, d, E, k, dtype, bias, renorm = case
    say(f"gate case {name}")
    x, Wg, bg, *_ = G.small_inputs(11, T, d, E, 64, dtype, bias=bias)
    ctx = B.Context(T, d, 64, E, k, dtype, renorm_topk=renorm)
    scores = torch.empty((T, k), dtype=torch.float32, device=G.DEV)
    idx = torch.empty((T, k), dtype=torch.int32, device=G.DEV)
    probs = torch.empty((T, E), dtype=torch.float32, device=G.DEV)
    logits = torch.empty((T, E), dtype=torch.float32, device=G.DEV)
    ctx.moe_gate(G.to_dev(x, dtype), G.to_dev(Wg, dtype), G.f32_dev(bg), scores, idx, probs, logits)
    torch.cuda.synchronize()
    z_gpu, idx_gpu, s_gpu, p_gpu = map(G.to_np, (logits, idx, scores, probs))

    z = O.router_logits(x, Wg, bg)
    assert np.abs(z_gpu - z).max() <= 2e-5 * max(1.0, np.abs(z).max())
    # integer stage of the oracle on the GPU's own float logits: must agree bit for bit
    idx_on_gpu_logits = O.topk(z_gpu.astype(np.float64), k)
    np.testing.assert_array_equal(idx_gpu, idx_on_gpu_logits)
    # softmax / scores of the oracle on the same routing
    p, s = O.scores(z, idx_gpu, renorm_topk=renorm)
    np.testing.assert_allclose(p_gpu, p, rtol=5e-5, atol=1e-9)
    np.testing.assert_allclose(s_gpu, s, rtol=5e-5, atol=1e-9)
    # wherever double logits leave no near-tie, the routing from x itself agrees too
    idx_ref = O.topk(z, k)
    zs = -np.sort(-z, axis=1)
    kk = min(k + 1, E)
    safe = np.min(zs[:, :kk - 1] - zs[:, 1:kk], axis=1) > 1e-4 if kk >= 2 else np.ones(T, bool)
    assert safe.mean() > 0.98
    np.testing.assert_array_equal(idx_gpu[safe], idx_ref[safe])


def test_gate_exact_ties_go_to_the_lower_expert():
    # duplicated router rows give exactly equal logits
    T, d, E, k = 40, 64, 6, 3
    x, Wg, bg, *_ = G.small_inputs(12, T, d, E, 64, "bf16", bias=False)
    Wg[3] = Wg[1]
    Wg[5] = Wg[0]
    ctx = B.Context(T, d, 64, E, k, "bf16")
    scores = torch.empty((T, k), dtype=torch.float32, device=G.DEV)
    idx = torch.empty((T, k), dtype=torch.int32, device=G.DEV)
    logits = torch.empty((T, E), dtype=torch.float32, device=G.DEV)
    ctx.moe_gate(G.to_dev(x, "bf16"), G.to_dev(Wg, "bf16"), None, scores, idx, None, logits)
    torch.cuda.synchronize()
    z_gpu = G.to_np(logits)
    assert (z_gpu[:, 3] == z_gpu[:, 1]).all() and (z_gpu[:, 5] == z_gpu[:, 0]).all()
    np.testing.assert_array_equal(G.to_np(idx), O.topk(z_gpu.astype(np.float64), k))


@pytest.mark.parametrize("dtype,E,k,n_shared", [("bf16", 4, 2, 20), ("bf16", 16, 2, 3), ("bf16", 20, 3, 5), ("f32", 4, 1, 20)])
def test_gate_writes_every_shared_slot(dtype, E, k, n_shared):
    # the shared experts' slots follow the k routed ones: expert ids E .. E+n_shared-1, score 1
    T, d = 50, 64
    say(f"gate with shared slots: {dtype} E={E} k={k} n_shared={n_shared}")
    x, Wg, bg, *_ = G.small_inputs(14, T, d, E, 64, dtype, bias=True)
    ctx = B.Context(T, d, 64, E, k, dtype, n_shared=n_shared)
    slots = k + n_shared
    scores = torch.full((T, slots), -3.0, dtype=torch.float32, device=G.DEV)
    idx = torch.full((T, slots), -3, dtype=torch.int32, device=G.DEV)
    logits = torch.empty((T, E), dtype=torch.float32, device=G.DEV)
    ctx.moe_gate(G.to_dev(x, dtype), G.to_dev(Wg, dtype), G.f32_dev(bg), scores, idx, None, logits)
    torch.cuda.synchronize()
    idx_gpu, s_gpu, z_gpu = G.to_np(idx), G.to_np(scores), G.to_np(logits)
    np.testing.assert_array_equal(idx_gpu[:, :k], O.topk(z_gpu.astype(np.float64), k))
    np.testing.assert_array_equal(idx_gpu[:, k:], np.broadcast_to(E + np.arange(n_shared), (T, n_shared)))
    np.testing.assert_array_equal(s_gpu[:, k:], 1.0)
    _, s = O.scores(O.router_logits(x, Wg, bg), idx_gpu[:, :k])
    np.testing.assert_allclose(s_gpu[:, :k], s, rtol=5e-5, atol=1e-9)


# ----------------------------------------------------------------------------- refresh mask
def gpu_mask(ctx, s_dev, policy):
    T, k = s_dev.shape
    mask = torch.full((T, k), 7, dtype=torch.uint8, device=G.DEV)
    n = torch.full((1,), -5, dtype=torch.int32, device=G.DEV)
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    ctx.moe_conditional_refresh(s_dev, None, policy, mask, n, ws)
    torch.cuda.synchronize()
    return G.to_np(mask), int(n.item())


@pytest.mark.parametrize("T,k", [(1, 2), (63, 2), (1024, 2), (1025, 2), (2049, 3), (8192, 2), (5000, 1),
                                 (16384, 2), (16385, 2), (20011, 2)])
def test_refresh_mask_bit_exact(T, k):
    say(f"refresh mask T={T} k={k}")
    r = np.random.Generator(np.random.PCG64(100 + T))
    s = np.sort(r.random((T, k), dtype=np.float32), axis=1)[:, ::-1].copy()
    if T > 100:                      # exact ties across the selection boundary
        s[T // 3: T // 3 + 40, 0] = s[T // 3, 0]
        s[5:25, k - 1] = s[5, k - 1]
    ctx = B.Context(T, 64, 64, 4, k, "f32") if k <= 4 else None
    s_dev = G.f32_dev(s)
    s64 = s.astype(np.float64)
    pols = [B.Policy(B.REFRESH_ALL), B.Policy(B.REFRESH_NONE)]
    for t in range(4):
        for n in (1, 2, 3):
            pols.append(B.Policy(B.REFRESH_ALG4, step_t=t, stride_n=n))
            # ablation variants: lowest activated slot / a drawn slot stays fresh (n_units = seed)
            pols.append(B.Policy(B.REFRESH_ALG4_HIGH, step_t=t, stride_n=n))
            pols.append(B.Policy(B.REFRESH_ALG4_RANDOM, step_t=t, stride_n=n, n_units=1000 * n + t))
    pols.append(B.Policy(B.REFRESH_ALG4_RANDOM, step_t=1, stride_n=2, n_units=-7))       # seed taken modulo 2^32
    for n_units in sorted({0, 1, T // 4, T // 3 + 17 if T > 100 else T // 2, T // 2, (3 * T) // 4, T - 1, T} - {-1}):
        if 0 <= n_units <= T:
            pols.append(B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=n_units))
    for n_units in sorted({0, 1, T // 2, T - 1, T, T + 1, T + T // 3, T * k - 1, T * k}):
        if 0 <= n_units <= T * k:
            pols.append(B.Policy(B.REFRESH_FRACTION_PAIR, n_units=n_units))
    for pol in pols:
        m_gpu, n_gpu = gpu_mask(ctx, s_dev, pol)
        m_ref, R = O.refresh_mask(s64, pol.kind, pol.step_t, pol.stride_n, pol.n_units)
        np.testing.assert_array_equal(m_gpu, m_ref, err_msg=str(pol))
        assert n_gpu == R == int(m_ref.sum()), pol


# ----------------------------------------------------------------------------- dispatch
@pytest.mark.parametrize("T,E,k,d,dtype,masked", [
    (64, 4, 2, 64, "f32", False),
    (301, 8, 2, 128, "bf16", True),
    (2048, 16, 2, 384, "bf16", False),
    (1000, 64, 6, 64, "bf16", True),
    (4096, 8, 2, 1152, "bf16", False),
    (8192, 8, 2, 1152, "bf16", True),
    (17, 3, 3, 64, "f32", True),
    (1, 4, 2, 64, "bf16", False),
    # pair counts that take each launch shape of the index kernels: one workgroup with 1, 2, 4, 8 steps per
    # wave (up to 2048 pairs), then count + place over several workgroups with 1, 2, 4, 8 steps, and a
    # grid beyond 256 workgroups
    (100, 4, 2, 64, "bf16", True),
    (250, 8, 2, 64, "bf16", False),
    (500, 8, 2, 64, "bf16", True),
    (1000, 8, 2, 64, "bf16", True),
    (1024, 8, 2, 64, "bf16", False),
    (1025, 8, 2, 64, "bf16", True),
    (5003, 8, 2, 64, "bf16", True),
    (12001, 8, 2, 64, "bf16", True),
    (20480, 16, 2, 64, "bf16", False),
    (40000, 8, 2, 64, "bf16", True),
    (70000, 64, 2, 64, "bf16", True),
    (150000, 8, 2, 64, "bf16", False),
    (300000, 5, 2, 64, "bf16", True),
    (400000, 64, 3, 64, "bf16", True),          # 586 workgroups, 64 experts: the scan kernel between count and place
])
def test_dispatch_bit_exact(T, E, k, d, dtype, masked):
    say(f"dispatch T={T} E={E} k={k} d={d} {dtype} masked={masked}")
    r = np.random.Generator(np.random.PCG64(200 + T + E))
    x = WL.to_storage(r.standard_normal((T, d), dtype=np.float32), dtype)
    # skewed routing, distinct experts per token
    z = r.standard_normal((T, E)) + np.log(WL.zipf_weights(E, 1.2))
    idx = O.topk(z, k)
    mask = (r.random((T, k)) < 0.5).astype(np.uint8) if masked else None
    ctx = B.Context(T, d, 64, E, k, dtype)
    buf = B.LayerBuffers(ctx, G.DEV)
    buf.x_packed.fill_(-77.0)
    ctx.moe_dispatch(G.to_dev(x, dtype), G.i32_dev(idx), None if mask is None else G.u8_dev(mask),
                     buf.x_packed, buf.counts, buf.offsets, buf.perm, buf.inv, buf.workspace)
    torch.cuda.synchronize()
    counts, offsets, perm, inv = O.dispatch(idx, mask, E)
    R = perm.shape[0]
    np.testing.assert_array_equal(G.to_np(buf.counts), counts)
    np.testing.assert_array_equal(G.to_np(buf.offsets), offsets)
    perm_gpu = G.to_np(buf.perm)
    np.testing.assert_array_equal(perm_gpu[:R], perm)
    assert (perm_gpu[R:] == -1).all()
    np.testing.assert_array_equal(G.to_np(buf.inv).reshape(T, k), inv)
    xp = G.to_np(buf.x_packed)
    np.testing.assert_array_equal(xp[:R], O.pack_rows(x, perm, k))       # rows copied bit for bit
    assert (xp[R:] == -77.0).all()                                       # rows beyond R untouched


def test_dispatch_nothing_refreshed():
    T, E, k, d = 100, 4, 2, 64
    idx = O.topk(np.random.default_rng(1).standard_normal((T, E)), k)
    ctx = B.Context(T, d, 64, E, k, "bf16")
    buf = B.LayerBuffers(ctx, G.DEV)
    x = torch.zeros((T, d), dtype=torch.bfloat16, device=G.DEV)
    ctx.moe_dispatch(x, G.i32_dev(idx), G.u8_dev(np.zeros((T, k), np.uint8)), buf.x_packed, buf.counts,
                     buf.offsets, buf.perm, buf.inv, buf.workspace)
    torch.cuda.synchronize()
    assert G.to_np(buf.counts).sum() == 0 and (G.to_np(buf.offsets) == 0).all()
    assert (G.to_np(buf.perm) == -1).all() and (G.to_np(buf.inv) == -1).all()


# ----------------------------------------------------------------------------- expert FFN
FFN_CASES = [
    # (name, rows per segment, d, F, dtype, bias)
    ("f32-tiny", [30, 0, 41, 57], 64, 256, "f32", False),
    ("f32-bias-ragged", [1, 65, 64, 130], 48, 80, "f32", True),
    ("bf16-ragged", [129, 0, 300, 1, 127, 256], 128, 320, "bf16", True),
    ("bf16-s-shape", [200, 310, 64, 450], 384, 1536, "bf16", False),
    ("bf16-one-row", [1], 64, 64, "bf16", True),
]


@pytest.mark.parametrize("case", FFN_CASES, ids=[c[0] for c in FFN_CASES])
def test_expert_ffn_against_oracle(case):
    name, seg_rows, d, F, dtype, bias = case
    say(f"ffn case {name}")
    E = len(seg_rows)
    rows = int(sum(seg_rows))
    _, _, _, W1, b1, W2, b2 = G.small_inputs(31, 4, d, E, F, dtype, bias=bias)
    r = np.random.Generator(np.random.PCG64(32))
    xp = WL.to_storage(r.standard_normal((rows, d), dtype=np.float32), dtype)
    # segments in a permuted expert order: the segment table, not the position, picks the expert
    seg_expert = np.roll(np.arange(E, dtype=np.int32), 1)
    seg_offsets = np.concatenate([[0], np.cumsum(seg_rows)]).astype(np.int32)
    ctx = B.Context(rows + 8, d, F, E, 1, dtype)
    h = torch.full((rows + 8, d), 9.0, dtype=ctx.torch_dtype, device=G.DEV)
    xp_dev = torch.zeros((rows + 8, d), dtype=ctx.torch_dtype, device=G.DEV)
    xp_dev[:rows] = G.to_dev(xp, dtype)
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    ctx.moe_expert_ffn(xp_dev, G.i32_dev(seg_offsets), G.i32_dev(seg_expert), rows + 8, G.to_dev(W1, dtype),
                       G.f32_dev(b1), G.to_dev(W2, dtype), G.f32_dev(b2), h, ws)
    torch.cuda.synchronize()
    h_gpu = G.to_np(h)
    h_ref = O.expert_ffn(xp, seg_offsets, seg_expert, W1, b1, W2, b2)
    G.assert_close_storage(h_gpu[:rows], h_ref, dtype, name)
    assert (h_gpu[rows:] == 9.0).all()          # rows outside every segment are left untouched


# Shapes that take each launch configuration of the wide-tile bf16 kernel (tile shape, number of
# stages, workgroups per compute unit are chosen from rows and widths), checked on sampled rows:
# the first and last rows of every segment (tile and segment boundaries) plus random ones.
WIDE_FFN_CASES = [
    # (name, rows per segment, d, F)
    ("xl-8192-rows", [1391, 612, 1204, 893, 1347, 701, 1120, 924], 1152, 4608),   # 128x192 x2 / 256x192
    ("xl-4096-rows", [695, 306, 602, 446, 673, 350, 560, 464], 1152, 4608),       # 128x192 x2 / three stages
    ("xl-2048-rows", [300, 200, 310, 250, 280, 190, 270, 248], 1152, 4608),       # second GEMM: K split in two
    ("xl-700-rows", [3, 250, 0, 129, 64, 1, 192, 61], 1152, 4608),                # second GEMM: K split in three
    ("column-tails", [700, 0, 1033, 515, 390, 462], 1088, 1600),                  # widths not multiples of 192
    # short reductions in the first GEMM: one, two, three and four 64-deep steps (pipeline prologue / tail paths)
    ("k-64", [900, 411, 1200, 777], 64, 1536),
    ("k-128", [900, 411, 1200, 777], 128, 1536),
    ("k-192", [900, 411, 1200, 777], 192, 1536),
    ("k-256", [900, 411, 1200, 777], 256, 1536),
    ("k-256-few-rows", [90, 41, 300, 77], 256, 4608),                             # three stages at four steps
    # second GEMM on 256 x 192 tiles with the shortest reductions its four-deep weight ring takes (five and
    # six 64-deep steps), and one step less (three-deep ring)
    ("k2-320", [1391, 612, 1204, 893, 1347, 701, 1120, 924], 1152, 320),
    ("k2-384", [1391, 612, 1204, 893, 1347, 701, 1120, 924], 1152, 384),
    ("k2-256", [1391, 612, 1204, 893, 1347, 701, 1120, 924], 1152, 256),
    # tile-to-XCD dealing: one hot expert whose tiles spill over to the other XCDs' spare slots; many
    # segments that share five experts (three XCDs own nothing); more segments than a wavefront has
    # lanes (row-band order instead); sixteen experts, two per XCD
    ("hot-expert", [5000, 100, 0, 100, 37, 100, 263, 2592], 384, 1536),
    ("forty-segments-five-experts", [150 + 37 * (g % 7) for g in range(40)], 384, 1536, [g % 5 for g in range(40)]),
    ("eighty-segments", [64 + 11 * (g % 9) for g in range(80)], 384, 1536, [g % 8 for g in range(80)]),
    ("sixteen-experts", [512 + 90 * ((g * 5) % 7) - 200 * (g % 2) for g in range(16)], 384, 1536),
]


@pytest.mark.parametrize("case", WIDE_FFN_CASES, ids=[c[0] for c in WIDE_FFN_CASES])
def test_expert_ffn_wide_tiles_on_sampled_rows(case):
    name, seg_rows, d, F = case[:4]
    say(f"wide ffn case {name}")
    dtype = "bf16"
    seg_expert = np.asarray(case[4], np.int32) if len(case) > 4 else np.roll(np.arange(len(seg_rows), dtype=np.int32), 3)
    E = int(seg_expert.max()) + 1
    rows = int(sum(seg_rows))
    # weights of the order of 1/sqrt(fan-in), as in the workloads: outputs of order one, for which the
    # absolute bf16 tolerance is written
    _, _, _, W1, b1, W2, b2 = G.small_inputs(51, 4, d, E, F, dtype, bias=True, w_std=0.02)
    r = np.random.Generator(np.random.PCG64(52))
    xp = WL.to_storage(r.standard_normal((rows, d), dtype=np.float32), dtype)
    seg_offsets = np.concatenate([[0], np.cumsum(seg_rows)]).astype(np.int32)
    ctx = B.Context(rows + 8, d, F, E, 1, dtype)
    h = torch.full((rows + 8, d), 9.0, dtype=ctx.torch_dtype, device=G.DEV)
    xp_dev = torch.zeros((rows + 8, d), dtype=ctx.torch_dtype, device=G.DEV)
    xp_dev[:rows] = G.to_dev(xp, dtype)
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    ctx.moe_expert_ffn(xp_dev, G.i32_dev(seg_offsets), G.i32_dev(seg_expert), rows, G.to_dev(W1, dtype),
                       G.f32_dev(b1), G.to_dev(W2, dtype), G.f32_dev(b2), h, ws)
    torch.cuda.synchronize()
    h_gpu = G.to_np(h)
    edge = []
    for g in range(len(seg_rows)):
        lo, hi = int(seg_offsets[g]), int(seg_offsets[g + 1])
        edge += [q for q in (lo, lo + 1, hi - 2, hi - 1) if lo <= q < hi]
    sel = np.unique(np.concatenate([np.array(edge, dtype=np.int64), r.integers(0, rows, 160)])).astype(np.int32)
    h_ref = O.expert_ffn(xp, seg_offsets, seg_expert, W1, b1, W2, b2, rows_sel=sel)
    G.assert_close_storage(h_gpu[sel], h_ref, dtype, name)
    assert (h_gpu[rows:] == 9.0).all()          # rows outside every segment are left untouched
    assert np.isfinite(h_gpu[:rows]).all() and (h_gpu[:rows] != 9.0).any(axis=1).all()   # every row written


# ----------------------------------------------------------------------------- combine
@pytest.mark.parametrize("T,k,d,dtype", [(64, 2, 64, "f32"), (333, 3, 128, "bf16"), (4096, 2, 1152, "bf16"),
                                         (50, 1, 64, "f32"), (100, 6, 192, "bf16"), (77, 4, 64, "bf16")])
def test_combine_against_oracle_on_the_same_rows(T, k, d, dtype):
    say(f"combine T={T} k={k} d={d} {dtype}")
    r = np.random.Generator(np.random.PCG64(40 + T))
    N = T * k
    h = WL.to_storage(r.standard_normal((N, d), dtype=np.float32), dtype)
    s = r.random((T, k), dtype=np.float32)
    inv = r.permutation(N).astype(np.int32).reshape(T, k)
    ctx = B.Context(T, d, 64, max(k, 4), k, dtype)
    y = torch.empty((T, d), dtype=ctx.torch_dtype, device=G.DEV)
    ctx.moe_combine(G.to_dev(h, dtype), G.i32_dev(inv), G.f32_dev(s), None, None, None, False, y)
    torch.cuda.synchronize()
    y_ref = O.combine(h.astype(np.float64), inv, s.astype(np.float64), None)
    G.assert_close_storage(G.to_np(y), y_ref, dtype, "combine", end_to_end=False)

    # with a mask: fresh rows from the packed buffer, reused rows and scores from the cache
    mask = (r.random((T, k)) < 0.5).astype(np.uint8)
    Hc = WL.to_storage(r.standard_normal((T, k, d), dtype=np.float32), dtype)
    Sc = r.random((T, k), dtype=np.float32)
    for use_fresh in (False, True):
        Hc_dev, Sc_dev = G.to_dev(Hc, dtype), G.f32_dev(Sc)
        ctx.moe_combine(G.to_dev(h, dtype), G.i32_dev(inv), G.f32_dev(s), G.u8_dev(mask), Hc_dev, Sc_dev,
                        use_fresh, y)
        torch.cuda.synchronize()
        Hc64, Sc64 = Hc.astype(np.float64), Sc.astype(np.float64)
        y_ref = O.combine(h.astype(np.float64), inv, s.astype(np.float64), mask, Hc64, Sc64, use_fresh)
        G.assert_close_storage(G.to_np(y), y_ref, dtype, "combine+cache", end_to_end=False)
        # write-through is a copy: bit-exact; untouched entries unchanged
        np.testing.assert_array_equal(G.to_np(Hc_dev), Hc64.astype(np.float32))
        np.testing.assert_array_equal(G.to_np(Sc_dev), Sc64.astype(np.float32))


# ----------------------------------------------------------------------------- whole layer
def check_layer(li_x, Wg, bg, W1, b1, W2, b2, k, dtype, name, renorm=False):
    g = G.GpuLayer(li_x, Wg, bg, W1, b1, W2, b2, k, dtype, renorm=renorm)
    y = G.to_np(g.forward())
    ref = O.moe_layer(li_x, Wg, bg, W1, b1, W2, b2, k, renorm_topk=renorm)
    np.testing.assert_array_equal(G.to_np(g.buf.expert_idx), ref.idx)
    np.testing.assert_array_equal(G.to_np(g.buf.counts), ref.counts)
    np.testing.assert_array_equal(G.to_np(g.buf.offsets), ref.offsets)
    np.testing.assert_array_equal(G.to_np(g.buf.perm)[:ref.R], ref.perm)
    np.testing.assert_array_equal(G.to_np(g.buf.inv).reshape(ref.inv.shape), ref.inv)
    np.testing.assert_allclose(G.to_np(g.buf.scores), ref.s, rtol=5e-5)
    G.assert_close_storage(G.to_np(g.buf.h_packed)[:ref.R], ref.h_packed, dtype, name + " h")
    G.assert_close_storage(y, ref.y, dtype, name + " y")
    # determinism: a second run is bit-identical
    y2 = G.to_np(g.forward())
    np.testing.assert_array_equal(y, y2)
    return g, ref


def test_layer_config1_tiny_fp32():
    li, _ = G.pick_layer(1)
    say(f"config 1 seed {li.seed}")
    check_layer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, 2, "f32", "cfg1")


def test_layer_config1_invariant_variants():
    # k = E (dense sum), identical experts, renormalised scores, biases
    x, Wg, bg, W1, b1, W2, b2 = G.small_inputs(51, 64, 64, 4, 256, "f32", bias=True)
    check_layer(x, Wg, bg, W1, b1, W2, b2, 4, "f32", "k=E")
    check_layer(x, Wg, bg, W1, b1, W2, b2, 2, "f32", "renorm", renorm=True)
    W1[:] = W1[0]; W2[:] = W2[0]; b1[:] = b1[0]; b2[:] = b2[0]
    g, ref = check_layer(x, Wg, bg, W1, b1, W2, b2, 2, "f32", "identical experts")
    one = O.expert_ffn(x, [0, 64], [0], W1, b1, W2, b2)
    G.assert_close_storage(G.to_np(g.buf.y), one * ref.s.sum(axis=1, keepdims=True), "f32", "expert(x)*sum(gates)")


def test_layer_config2_small_bf16():
    li, _ = G.pick_layer(2)
    say(f"config 2 seed {li.seed}")
    g, ref = check_layer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, 2, "bf16", "cfg2")
    load = ref.counts / ref.counts.mean()
    assert load.max() < 1.5          # near-uniform load


@pytest.mark.parametrize("cfg,T", [(1, None), (2, None), (3, None), (3, 1500)])
def test_layer_forward_with_the_gather_folded_into_the_ffn(cfg, T):
    """moe_layer_forward's default path (dispatch writes indices only, the first GEMM reads token rows
    through perm) against the path that materialises x_packed: bit-identical h rows and y, for the
    synchronous layer and for an Algorithm 4 off-step; and y against the oracle where it runs in full."""
    li, _ = G.pick_layer(cfg, T=T)
    c = li.cfg
    say(f"fused gather: config {cfg} T={li.x.shape[0]} seed {li.seed}")
    dtype, k = c.dtype, c.k
    Tn = li.x.shape[0]
    ctx = B.Context(Tn, c.d, c.F, c.E, k, dtype)
    dev = lambda a: G.to_dev(a, dtype)
    args = (dev(li.Wg), G.f32_dev(li.bg) if li.bg is not None else None, dev(li.W1), None, dev(li.W2), None)
    x0 = dev(li.x)
    x1 = dev(WL.next_step_x(cfg, li.x))
    out = {}
    for fused in (True, False):
        buf = B.LayerBuffers(ctx, G.DEV, with_cache=True)
        buf.x_packed.fill_(-5.0)
        y_sync = B.moe_layer_forward(ctx, buf, x0, *args, fuse_gather=fused).clone()
        torch.cuda.synchronize()
        R = int(G.to_np(buf.offsets)[-1])
        h_sync = G.to_np(buf.h_packed)[:R].copy()
        if fused:
            assert (G.to_np(buf.x_packed) == -5.0).all()        # never materialised
        B.moe_layer_forward(ctx, buf, x0, *args, policy=B.Policy(B.REFRESH_ALL), fuse_gather=fused, rows_to_cache=False)
        y_off = B.moe_layer_forward(ctx, buf, x1, *args, policy=B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=2),
                                    fuse_gather=fused, rows_to_cache=False).clone()
        torch.cuda.synchronize()
        R1 = int(G.to_np(buf.offsets)[-1])
        assert R1 == Tn                                          # slot 0 of every token
        out[fused] = (G.to_np(y_sync), h_sync, G.to_np(y_off), G.to_np(buf.h_packed)[:R1].copy())
    for a, b_ in zip(out[True], out[False]):
        np.testing.assert_array_equal(a, b_)
    if cfg in (1, 2):
        ref = O.moe_layer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, k)
        G.assert_close_storage(out[True][0], ref.y, dtype, f"cfg{cfg} fused y")


def sampled_layer_check(g, ref_idx_stage, li, k, name, n_rows=96, n_tok=64, seed=0):
    """Full-size check: integer stages in full, FFN rows and output tokens on a sample."""
    c = li.cfg
    z, idx, s, counts, offsets, perm, inv = ref_idx_stage
    np.testing.assert_array_equal(G.to_np(g.buf.expert_idx), idx)
    np.testing.assert_array_equal(G.to_np(g.buf.counts), counts)
    np.testing.assert_array_equal(G.to_np(g.buf.offsets), offsets)
    R = perm.shape[0]
    np.testing.assert_array_equal(G.to_np(g.buf.perm)[:R], perm)
    np.testing.assert_array_equal(G.to_np(g.buf.inv).reshape(inv.shape), inv)
    np.testing.assert_allclose(G.to_np(g.buf.scores), s, rtol=5e-5)
    xp_gpu = G.to_np(g.buf.x_packed)[:R]
    np.testing.assert_array_equal(xp_gpu, li.x[perm // k])
    r = np.random.Generator(np.random.PCG64(seed))
    # sampled tokens: all their pairs go through the oracle's expert, then its combine
    toks = np.sort(r.choice(li.x.shape[0], size=n_tok, replace=False)).astype(np.int32)
    # always include the first and last row of every expert's segment (tile edges, ragged tails)
    edge_rows = np.unique(np.concatenate([offsets[:-1][counts > 0], offsets[1:][counts > 0] - 1]))
    rows = np.unique(np.concatenate([inv[toks].reshape(-1), edge_rows,
                                     r.choice(R, size=n_rows, replace=False)])).astype(np.int32)
    h_ref = O.expert_ffn(xp_gpu, offsets, np.arange(c.E), li.W1, None, li.W2, None, rows_sel=rows)
    h_gpu = G.to_np(g.buf.h_packed)
    G.assert_close_storage(h_gpu[rows], h_ref, c.dtype, name + " h rows")
    h_sparse = np.zeros((R, c.d))
    h_sparse[rows] = h_ref
    y_ref = O.combine(h_sparse, inv, s, None, tokens_sel=toks)
    G.assert_close_storage(G.to_np(g.buf.y)[toks], y_ref, c.dtype, name + " y tokens")


def oracle_index_stages(li, k, z=None):
    z = O.router_logits(li.x, li.Wg, li.bg) if z is None else z
    idx = O.topk(z, k)
    _, s = O.scores(z, idx)
    counts, offsets, perm, inv = O.dispatch(idx, None, li.cfg.E)
    return z, idx, s, counts, offsets, perm, inv


@pytest.mark.parametrize("layer", [0, 27])
def test_layer_config3_xl_full_size_sampled(layer):
    li, z = G.pick_layer(3, layer=layer)
    say(f"config 3 layer {layer} seed {li.seed}")
    g = G.GpuLayer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, 2, "bf16")
    poison(g.buf.h_packed); poison(g.buf.y)
    g.forward()
    assert_written(g.buf.h_packed, li.cfg.N, "cfg3 h_packed"); assert_written(g.buf.y, li.cfg.T, "cfg3 y")
    st = oracle_index_stages(li, 2, z)
    load = st[3] / st[3].mean()
    say(f"  expert load max/mean = {load.max():.2f}")
    assert 1.2 < load.max() < 4.0            # moderately uneven
    sampled_layer_check(g, st, li, 2, f"cfg3 layer {layer}", seed=layer)


def test_layer_dit_moe_g_shape_full_size_sampled():
    """The paper's second model shape (Section 5.1: 16 experts; 40 layers of it in the benchmark):
    one full-size layer, integer stages in full, FFN rows and outputs on a sample."""
    li, z = G.pick_layer(6)
    say(f"DiT-MoE-G shape, seed {li.seed}")
    g = G.GpuLayer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, 2, "bf16")
    poison(g.buf.h_packed); poison(g.buf.y)
    g.forward()
    assert_written(g.buf.h_packed, li.cfg.N, "dit-moe-g h_packed"); assert_written(g.buf.y, li.cfg.T, "dit-moe-g y")
    st = oracle_index_stages(li, 2, z)
    sampled_layer_check(g, st, li, 2, "dit-moe-g", n_rows=48, n_tok=32, seed=6)


@pytest.mark.parametrize("T", [4096, 1024, 300])
def test_layer_is_bit_reproducible_at_the_xl_widths(T):
    """No floating-point atomics anywhere and every reduction in a fixed order (the split second GEMM
    included): two runs of the layer give the same bits, also when other work ran in between."""
    li, _ = G.pick_layer(3, T=T)
    g = G.GpuLayer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, 2, "bf16")
    y1 = g.forward(fuse_gather=True).clone()
    h1 = g.buf.h_packed.clone()
    g.buf.h_packed.fill_(0); g.buf.y.fill_(0); g.buf.workspace.fill_(7)
    y2 = g.forward(fuse_gather=True)
    assert torch.equal(y1, y2) and torch.equal(h1, g.buf.h_packed)


# ----------------------------------------------------------------------------- shared experts
def shared_reference_tables(ref, E, n_shared):
    """Per-pair arrays of a layer with shared experts, from the oracle's routed result: the shared
    slots follow the k routed ones (expert E+s, score 1, always refreshed), and the permutation is
    the oracle's own stable sort run on those extended arrays."""
    T = ref.idx.shape[0]
    idx = np.concatenate([ref.idx, np.broadcast_to(E + np.arange(n_shared, dtype=np.int32), (T, n_shared))], axis=1)
    s = np.concatenate([ref.s, np.ones((T, n_shared))], axis=1)
    mask = np.concatenate([ref.mask, np.ones((T, n_shared), np.uint8)], axis=1)
    counts, offsets, perm, inv = O.dispatch(idx, mask, E + n_shared)
    return idx, s, mask, counts, offsets, perm, inv


def check_shared_tables(g, ref, E, n_shared, with_mask):
    idx, s, mask, counts, offsets, perm, inv = shared_reference_tables(ref, E, n_shared)
    R = perm.shape[0]
    np.testing.assert_array_equal(G.to_np(g.buf.expert_idx), idx)
    np.testing.assert_allclose(G.to_np(g.buf.scores), s, rtol=5e-5)
    np.testing.assert_array_equal(G.to_np(g.buf.scores)[:, -n_shared:], 1.0)
    if with_mask:
        np.testing.assert_array_equal(G.to_np(g.buf.mask), mask)
        assert int(g.buf.n_refresh.item()) == R == ref.R + n_shared * idx.shape[0]
    np.testing.assert_array_equal(G.to_np(g.buf.counts), counts)
    np.testing.assert_array_equal(G.to_np(g.buf.offsets), offsets)
    np.testing.assert_array_equal(G.to_np(g.buf.perm)[:R], perm)
    np.testing.assert_array_equal(G.to_np(g.buf.inv).reshape(inv.shape), inv)
    return offsets, perm, inv


@pytest.mark.parametrize("dtype,T,d,E,F,k,n_shared", [("f32", 64, 64, 4, 256, 2, 2), ("f32", 77, 64, 5, 128, 1, 1),
                                                     ("bf16", 1000, 128, 8, 512, 2, 2), ("bf16", 333, 64, 6, 256, 3, 3)])
@pytest.mark.parametrize("fused", [False, True])
def test_shared_experts_synchronous_layer_full_parity(dtype, T, d, E, F, k, n_shared, fused):
    """A layer with shared experts (Section 5.1, "Models and Datasets"; supplement, "More details of
    MoE"): routed tables, the shared slots, every h row and y against the oracle."""
    x, Wg, bg, W1, b1, W2, b2 = G.small_inputs(71, T, d, E + n_shared, F, dtype, bias=True, w_std=0.03)
    Wg, bg = Wg[:E].copy(), bg[:E].copy()
    say(f"shared experts: {dtype} T={T} d={d} E={E}+{n_shared} F={F} k={k} fused={fused}")
    z = O.router_logits(x, Wg, bg)
    assert G.topk_margin(z, k) >= 1e-5
    g = G.GpuLayer(x, Wg, bg, W1, b1, W2, b2, k, dtype, n_shared=n_shared)
    y = G.to_np(g.forward(fuse_gather=fused))
    ref = O.moe_layer(x, Wg, bg, W1, b1, W2, b2, k, n_shared=n_shared)
    offsets, perm, inv = check_shared_tables(g, ref, E, n_shared, with_mask=False)
    # every packed row, shared experts' rows included, through the oracle's per-row routine
    xp = x[perm // (k + n_shared)]
    if not fused:
        np.testing.assert_array_equal(G.to_np(g.buf.x_packed)[:perm.shape[0]], xp)
    h_ref = O.expert_ffn(xp, offsets, np.arange(E + n_shared), W1, b1, W2, b2)
    G.assert_close_storage(G.to_np(g.buf.h_packed)[:perm.shape[0]], h_ref, dtype, "h rows")
    G.assert_close_storage(y, ref.y, dtype, "y with shared experts", wide_range=True)
    share = np.linalg.norm(ref.y_shared) / np.linalg.norm(ref.y)
    say(f"  shared experts carry {100 * share:.0f}% of |y|")
    assert share > 0.2                      # the check would notice a missing shared term


def test_shared_experts_stay_fresh_under_conditional_refresh():
    """Two steps with caches: the routed pairs follow the policy, the shared experts are recomputed
    in every step (supplement, "Influence of Shared Experts") and never enter the caches."""
    dtype, T, d, E, F, k, n_shared = "bf16", 1024, 128, 8, 256, 2, 2
    x0, Wg, bg, W1, b1, W2, b2 = G.small_inputs(73, T, d, E + n_shared, F, dtype, bias=True, w_std=0.03)
    Wg, bg = Wg[:E].copy(), bg[:E].copy()
    policies = [B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=2), B.Policy(B.REFRESH_ALG4, step_t=2, stride_n=2),
                B.Policy(B.REFRESH_NONE), B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=T // 4),
                B.Policy(B.REFRESH_FRACTION_PAIR, n_units=T + T // 2),
                B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=T // 2, use_fresh_scores=True)]
    assert G.topk_margin(O.router_logits(x0, Wg, bg), k) >= 1e-5
    # step-t activations: seeded, the seed bumped until routing has no near-tie and no policy's
    # selection boundary (last admitted / first rejected importance score) is closer than 1e-6, so
    # that float and double scores must take the same decision
    for bump in range(50):
        r = np.random.Generator(np.random.PCG64(74 + 1000 * bump))
        x1 = WL.to_storage(x0 + np.float32(0.2) * r.standard_normal(x0.shape, dtype=np.float32), dtype)
        z1 = O.router_logits(x1, Wg, bg)
        s1 = O.scores(z1, O.topk(z1, k))[1]
        if G.topk_margin(z1, k) >= 1e-5 and min(G.selection_gap(s1, p_.kind, p_.n_units) for p_ in policies) >= 1e-6:
            break
    else:
        raise AssertionError("no step-t seed with clear selection boundaries found")
    say(f"  step-t seed bump {bump}")
    g = G.GpuLayer(x0, Wg, bg, W1, b1, W2, b2, k, dtype, with_cache=True, n_shared=n_shared)
    x1_dev = G.to_dev(x1, dtype)
    kc = k + n_shared
    H0 = np.zeros((T, k, d)); S0 = np.zeros((T, k))
    r0 = O.moe_layer(x0, Wg, bg, W1, b1, W2, b2, k, n_shared=n_shared, H_cache=H0, S_cache=S0)
    for fused in (False, True):
        for pol in policies:
            g.buf.H_cache.fill_(7.0); g.buf.S_cache.fill_(7.0)
            y0 = G.to_np(g.forward(B.Policy(B.REFRESH_ALL), fuse_gather=fused))
            G.assert_close_storage(y0, r0.y, dtype, "step0 y", wide_range=True)
            Hc0, Sc0 = G.to_np(g.buf.H_cache).copy(), G.to_np(g.buf.S_cache).copy()
            # shared slots of the caches are never written
            assert (Hc0[:, k:] == 7.0).all() and (Sc0[:, k:] == 7.0).all()
            G.assert_close_storage(Hc0[:, :k].reshape(T * k, d), H0.reshape(T * k, d), dtype, "step0 cache")
            y1 = G.to_np(g.forward(pol, x=x1_dev, fuse_gather=fused))
            H, S = H0.copy(), S0.copy()
            r1 = O.moe_layer(x1, Wg, bg, W1, b1, W2, b2, k, n_shared=n_shared, policy=pol.kind, step_t=pol.step_t,
                             stride_n=pol.stride_n, n_units=pol.n_units, H_cache=H, S_cache=S,
                             use_fresh_scores=pol.use_fresh_scores)
            s_gpu = G.to_np(g.buf.scores)[:, :k].astype(np.float64)
            m_from_gpu_scores, R = O.refresh_mask(s_gpu, pol.kind, pol.step_t, pol.stride_n, pol.n_units)
            m_gpu = G.to_np(g.buf.mask)
            np.testing.assert_array_equal(m_gpu[:, :k], m_from_gpu_scores, err_msg=str(pol))
            np.testing.assert_array_equal(m_gpu[:, k:], 1)
            assert int(g.buf.n_refresh.item()) == R + n_shared * T == g.ctx.moe_policy_refreshed_pairs(pol, T)[0]
            # the selection boundaries are clear (seed check above), so double scores give the same
            # mask; if they ever do not, everything after the decision is compared against the oracle
            # fed the GPU's mask (the decision itself was checked just above)
            y_ref = r1.y
            if not np.array_equal(m_gpu[:, :k], r1.mask):
                say(f"  {pol}: float and double scores disagree; oracle fed the GPU's mask")
                H, S = H0.copy(), S0.copy()
                y_ref, perm_ref, inv_ref, R_ref = G.oracle_layer_given_mask(x1, Wg, bg, W1, b1, W2, b2, k, m_gpu[:, :k].copy(),
                                                                            H, S, pol.use_fresh_scores, n_shared=n_shared)
                r1.mask, r1.R = m_gpu[:, :k].copy(), R_ref
            check_shared_tables(g, r1, E, n_shared, with_mask=True)
            G.assert_close_storage(y1, y_ref, dtype, f"step1 y {pol}", wide_range=True)
            G.assert_close_storage(G.to_np(g.buf.H_cache)[:, :k].reshape(T * k, d), H.reshape(T * k, d), dtype,
                                   "cache")
            np.testing.assert_allclose(G.to_np(g.buf.S_cache)[:, :k], S, rtol=5e-5)
            keep = m_gpu == 0
            np.testing.assert_array_equal(G.to_np(g.buf.H_cache)[keep], Hc0[keep])
            np.testing.assert_array_equal(G.to_np(g.buf.S_cache)[keep], Sc0[keep])
            assert (G.to_np(g.buf.H_cache)[:, k:] == 7.0).all()
            say(f"  fused={fused} {pol}: R={R}+{n_shared * T}")


def test_shared_experts_config3_xl_full_size_sampled():
    """DiT-MoE-XL shape with its two shared experts at full size: integer stages in full, y on
    sampled tokens (routed rows by the oracle's per-row routine, shared part by its dense definition)."""
    n_shared = 2
    li, z = G.pick_layer(3, n_shared=n_shared)
    c, k = li.cfg, li.cfg.k
    E, T = c.E, c.T
    say(f"config 3 with {n_shared} shared experts, seed {li.seed}")
    g = G.GpuLayer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, k, "bf16", n_shared=n_shared)
    g.forward(fuse_gather=True)
    idx = O.topk(z, k)
    _, s = O.scores(z, idx)

    class RoutedOnly:                       # the fields shared_reference_tables reads
        pass
    ref = RoutedOnly()
    ref.idx, ref.s, ref.mask, ref.R = idx, s, np.ones((T, k), np.uint8), T * k
    offsets, perm, inv = check_shared_tables(g, ref, E, n_shared, with_mask=False)
    r = np.random.Generator(np.random.PCG64(5))
    toks = np.sort(r.choice(T, size=48, replace=False)).astype(np.int32)
    kc = k + n_shared
    rows = np.unique(inv[toks][:, :k].reshape(-1)).astype(np.int32)
    xp = li.x[perm // kc]
    h_ref = O.expert_ffn(xp, offsets, np.arange(E + n_shared), li.W1, None, li.W2, None, rows_sel=rows)
    G.assert_close_storage(G.to_np(g.buf.h_packed)[rows], h_ref, "bf16", "routed h rows")
    h_sparse = np.zeros((perm.shape[0], c.d))
    h_sparse[rows] = h_ref
    y_routed = O.combine(h_sparse, inv[:, :k].copy(), s, None, tokens_sel=toks)
    y_shared = O.shared_experts(li.x[toks], li.W1[E:], None, li.W2[E:], None)
    G.assert_close_storage(G.to_np(g.buf.y)[toks], y_routed + y_shared, "bf16", "y tokens", wide_range=True)
    # the shared experts' own rows: one dense FFN each
    for e in range(n_shared):
        rows_s = inv[toks][:, k + e]
        one = O.shared_experts(li.x[toks], li.W1[E + e:E + e + 1], None, li.W2[E + e:E + e + 1], None)
        G.assert_close_storage(G.to_np(g.buf.h_packed)[rows_s], one, "bf16", f"shared expert {e} rows", wide_range=True)


# ----------------------------------------------------------------------------- conditional refresh, two steps
def run_two_steps(T, policies, cfg=4):
    """Seeded two-step inputs: step-t activations free of routing near-ties and, for every fraction
    policy in ``policies``, with a gap of at least 1e-6 between the last admitted and the first
    rejected importance score (float and double scores then take the same decision); the seed is
    bumped until both hold."""
    li, _ = G.pick_layer(cfg, T=T)
    c = li.cfg
    k = c.k
    for bump in range(50):
        x1 = WL.next_step_x(cfg, li.x, bump=bump)
        z1 = O.router_logits(x1, li.Wg, li.bg)
        s1 = O.scores(z1, O.topk(z1, k))[1]
        gap = min([G.selection_gap(s1, p_.kind, p_.n_units) for p_ in policies] + [np.inf])
        if G.topk_margin(z1, k) >= 1e-4 and gap >= 1e-6:
            break
    else:
        raise AssertionError("no step-t seed with clear routing and selection boundaries found")
    say(f"two steps: T={T} seed {li.seed} step bump {bump}, smallest selection gap {gap:.2e}")
    return li, x1, z1


def test_conditional_refresh_two_steps_small_full_parity():
    T = 1024
    policies = [B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=int(np.floor(f * T + 0.5))) for f in (0.25, 0.5, 0.75, 1.0)]
    policies += [B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=2), B.Policy(B.REFRESH_FRACTION_PAIR, n_units=T),
                 B.Policy(B.REFRESH_NONE), B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=T // 2, use_fresh_scores=True)]
    li, x1, z1 = run_two_steps(T, policies)
    c, k, d = li.cfg, li.cfg.k, li.cfg.d
    # shrink the expert width so that the oracle runs every row in seconds
    F = 256
    W1 = li.W1[:, :F, :].copy()
    W2 = li.W2[:, :, :F].copy()
    g = G.GpuLayer(li.x, li.Wg, li.bg, W1, None, W2, None, k, "bf16", with_cache=True)
    x1_dev = G.to_dev(x1, "bf16")

    def oracle_step0():
        H = np.zeros((T, k, d)); S = np.zeros((T, k))
        r0 = O.moe_layer(li.x, li.Wg, li.bg, W1, None, W2, None, k, policy=O.REFRESH_ALL, H_cache=H, S_cache=S)
        return r0, H, S

    r0, H0, S0 = oracle_step0()
    sync1 = O.moe_layer(x1, li.Wg, li.bg, W1, None, W2, None, k)
    changed = (sync1.idx != r0.idx).any(axis=1).mean()
    say(f"  routing changed for {100 * changed:.1f}% of tokens between the two steps")

    for pol in policies:
        # step t-1: synchronous, fills the cache
        y0 = G.to_np(g.forward(B.Policy(B.REFRESH_ALL)))
        G.assert_close_storage(y0, r0.y, "bf16", "step0 y")
        Hc0, Sc0 = G.to_np(g.buf.H_cache).copy(), G.to_np(g.buf.S_cache).copy()
        G.assert_close_storage(Hc0.reshape(T * k, d), H0.reshape(T * k, d), "bf16", "step0 cache")
        # step t: partial refresh
        y1 = G.to_np(g.forward(pol, x=x1_dev))
        H, S = H0.copy(), S0.copy()
        r1 = O.moe_layer(x1, li.Wg, li.bg, W1, None, W2, None, k, policy=pol.kind, step_t=pol.step_t,
                         stride_n=pol.stride_n, n_units=pol.n_units, H_cache=H, S_cache=S,
                         use_fresh_scores=pol.use_fresh_scores)
        # the mask from the GPU's own float scores, by the oracle: bit-exact
        s_gpu = G.to_np(g.buf.scores).astype(np.float64)
        m_ref_gpu_scores, R = O.refresh_mask(s_gpu, pol.kind, pol.step_t, pol.stride_n, pol.n_units)
        m_gpu = G.to_np(g.buf.mask)
        np.testing.assert_array_equal(m_gpu, m_ref_gpu_scores, err_msg=str(pol))
        assert int(g.buf.n_refresh.item()) == R
        # The selection boundary is clear (seed check in run_two_steps), so double scores give the same
        # decision.  Should they ever not, the decision has been checked above on the scores it was
        # taken from, and everything after it is compared against the oracle fed that mask: a full
        # comparison runs either way.
        y_ref, perm_ref, inv_ref = r1.y, r1.perm, r1.inv
        if not np.array_equal(m_gpu, r1.mask):
            say(f"  {pol}: float and double scores disagree on {(m_gpu != r1.mask).sum()} mask bytes; oracle fed the GPU's mask")
            H, S = H0.copy(), S0.copy()
            y_ref, perm_ref, inv_ref, _ = G.oracle_layer_given_mask(x1, li.Wg, li.bg, W1, None, W2, None, k, m_gpu, H, S,
                                                                    pol.use_fresh_scores)
        np.testing.assert_array_equal(G.to_np(g.buf.perm)[:R], perm_ref)
        np.testing.assert_array_equal(G.to_np(g.buf.inv).reshape(T, k), inv_ref)
        G.assert_close_storage(y1, y_ref, "bf16", f"step1 y {pol}")
        G.assert_close_storage(G.to_np(g.buf.H_cache).reshape(T * k, d), H.reshape(T * k, d), "bf16", "cache")
        np.testing.assert_allclose(G.to_np(g.buf.S_cache), S, rtol=5e-5)
        # untouched cache entries are unchanged bit for bit
        keep = m_gpu == 0
        np.testing.assert_array_equal(G.to_np(g.buf.H_cache)[keep], Hc0[keep])
        np.testing.assert_array_equal(G.to_np(g.buf.S_cache)[keep], Sc0[keep])
        rel = np.linalg.norm(r1.y - sync1.y) / np.linalg.norm(sync1.y)
        say(f"  {pol}: R={R}, rel-L2 of the approximation vs the synchronous step = {rel:.4f}")
        if pol.kind == B.REFRESH_NONE:
            np.testing.assert_array_equal(y1, y0)            # fraction 0: the cache, bit for bit
        if pol.kind == B.REFRESH_FRACTION_TOKEN and pol.n_units == T:
            y_sync = G.to_np(g.forward(None, x=x1_dev))       # fraction 1: the synchronous layer, bit for bit
            np.testing.assert_array_equal(y1, y_sync)


def test_conditional_refresh_config4_full_size_sampled():
    T4 = WL.CONFIGS[4].T
    li, x1, z1 = run_two_steps(T4, [B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=int(np.floor(f * T4 + 0.5)))
                                    for f in (0.5, 0.25, 0.75, 1.0)])
    c, k, T = li.cfg, li.cfg.k, li.cfg.T
    g = G.GpuLayer(li.x, li.Wg, li.bg, li.W1, None, li.W2, None, k, "bf16", with_cache=True)
    x1_dev = G.to_dev(x1, "bf16")
    st0 = oracle_index_stages(li, k)
    r = np.random.Generator(np.random.PCG64(4))
    for f in (0.5, 0.25, 0.75, 1.0):
        n_units = int(np.floor(f * T + 0.5))
        g.forward(B.Policy(B.REFRESH_ALL))
        if f == 0.5:
            sampled_layer_check(g, st0, li, k, "cfg4 step t-1", n_rows=32, n_tok=32)
        Hc0 = G.to_np(g.buf.H_cache).copy()
        Sc0 = G.to_np(g.buf.S_cache).copy()
        poison(g.buf.h_packed); poison(g.buf.y)
        y1 = G.to_np(g.forward(B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=n_units), x=x1_dev))
        assert_written(g.buf.h_packed, n_units * k, f"cfg4 f={f} h_packed"); assert_written(g.buf.y, T, f"cfg4 f={f} y")
        # integer stages on the GPU's float scores
        s_gpu = G.to_np(g.buf.scores).astype(np.float64)
        idx_gpu = G.to_np(g.buf.expert_idx)
        np.testing.assert_array_equal(idx_gpu, O.topk(z1, k))
        mask, R = O.refresh_mask(s_gpu, O.REFRESH_FRACTION_TOKEN, n_units=n_units)
        np.testing.assert_array_equal(G.to_np(g.buf.mask), mask)
        assert int(g.buf.n_refresh.item()) == R == n_units * k
        counts, offsets, perm, inv = O.dispatch(idx_gpu, mask, c.E)
        np.testing.assert_array_equal(G.to_np(g.buf.counts), counts)
        np.testing.assert_array_equal(G.to_np(g.buf.perm)[:R], perm)
        np.testing.assert_array_equal(G.to_np(g.buf.inv).reshape(T, k), inv)
        # sampled tokens, refreshed and reused alike
        toks = np.sort(r.choice(T, size=48, replace=False)).astype(np.int32)
        rows = inv[toks].reshape(-1)
        rows = np.unique(rows[rows >= 0]).astype(np.int32)
        xp = G.to_np(g.buf.x_packed)[:R]
        np.testing.assert_array_equal(xp, x1[perm // k])
        h_ref = O.expert_ffn(xp, offsets, np.arange(c.E), li.W1, None, li.W2, None, rows_sel=rows)
        G.assert_close_storage(G.to_np(g.buf.h_packed)[rows], h_ref, "bf16", f"cfg4 f={f} h rows")
        h_sparse = np.zeros((max(R, 1), c.d)); h_sparse[rows] = h_ref
        H64, S64 = Hc0.astype(np.float64), Sc0.astype(np.float64)
        y_ref = O.combine(h_sparse, inv, s_gpu, mask, H64, S64, False, tokens_sel=toks)
        G.assert_close_storage(y1[toks], y_ref, "bf16", f"cfg4 f={f} y tokens")
        keep = mask == 0
        np.testing.assert_array_equal(G.to_np(g.buf.H_cache)[keep], Hc0[keep])
        say(f"  cfg4 f={f}: R={R}")


# ----------------------------------------------------------------------------- expert-parallel shard (config 5)
def test_ep_shard_config5_receive_side_sampled():
    ep = WL.make_ep_shard()
    c = ep.cfg
    rows, E_loc, W = ep.x_recv.shape[0], 4, 4
    say(f"config 5 receive side: rows={rows} recv_counts=\n{ep.recv_counts}")
    ctx = B.Context(rows, c.d, c.F, E_loc, 1, "bf16")
    seg_offsets = torch.empty(W * E_loc + 1, dtype=torch.int32, device=G.DEV)
    seg_expert = torch.empty(W * E_loc, dtype=torch.int32, device=G.DEV)
    ctx.moe_ep_segments(G.i32_dev(ep.recv_counts), seg_offsets, seg_expert)
    so_ref, se_ref = O.ep_segments(ep.recv_counts)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(G.to_np(seg_offsets), so_ref)
    np.testing.assert_array_equal(G.to_np(seg_expert), se_ref)
    h = torch.empty((rows + 16, c.d), dtype=torch.bfloat16, device=G.DEV)
    poison(h)
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    x_dev, W1_dev, W2_dev = G.to_dev(ep.x_recv, "bf16"), G.to_dev(ep.W1, "bf16"), G.to_dev(ep.W2, "bf16")
    ctx.moe_expert_ffn(x_dev, seg_offsets, seg_expert, rows, W1_dev, None, W2_dev, None, h, ws)
    torch.cuda.synchronize()
    ctx.moe_expert_ffn_status(ws)
    assert_written(h, rows, "cfg5 h")
    # self-consistency (expert-parallelism figure: the segment layout must not matter): the same rows
    # regrouped expert-major, four segments instead of sixteen, give the same bits row for row
    order = np.argsort(ep.row_expert, kind="stable")
    counts_e = np.bincount(ep.row_expert, minlength=E_loc)
    off_e = G.i32_dev(np.concatenate([[0], np.cumsum(counts_e)]))
    h2 = torch.empty((rows, c.d), dtype=torch.bfloat16, device=G.DEV)
    poison(h2)
    ctx.moe_expert_ffn(x_dev[torch.from_numpy(order).to(G.DEV)].contiguous(), off_e,
                       torch.arange(E_loc, dtype=torch.int32, device=G.DEV), rows, W1_dev, None, W2_dev, None, h2, ws)
    torch.cuda.synchronize()
    assert torch.equal(h2, h[:rows][torch.from_numpy(order).to(G.DEV)]), "segment layout changed the result"
    r = np.random.Generator(np.random.PCG64(5))
    edge = np.unique(np.concatenate([so_ref[:-1], so_ref[1:] - 1]))
    sel = np.unique(np.concatenate([edge, r.choice(rows, size=24, replace=False)])).astype(np.int32)
    h_ref = O.expert_ffn(ep.x_recv, so_ref, se_ref, ep.W1, None, ep.W2, None, rows_sel=sel)
    G.assert_close_storage(G.to_np(h)[sel], h_ref, "bf16", "cfg5 h rows")
    load = ep.recv_counts.sum(axis=0)
    say(f"  rows per local expert {load.tolist()}")


def test_ep_shard_config5_source_side_gate_and_dispatch():
    li, z = G.pick_layer(5, with_experts=False)
    c = li.cfg
    say(f"config 5 source side seed {li.seed}")
    ctx = B.Context(c.T, c.d, c.F, c.E, c.k, "bf16")
    buf = B.LayerBuffers(ctx, G.DEV, workspace=torch.empty(1 << 20, dtype=torch.uint8, device=G.DEV))   # dispatch scratch only
    x = G.to_dev(li.x, "bf16")
    ctx.moe_gate(x, G.to_dev(li.Wg, "bf16"), G.f32_dev(li.bg), buf.scores, buf.expert_idx)
    ctx.moe_dispatch(x, buf.expert_idx, None, buf.x_packed, buf.counts, buf.offsets, buf.perm, buf.inv, buf.workspace)
    torch.cuda.synchronize()
    idx = O.topk(z, c.k)
    counts, offsets, perm, inv = O.dispatch(idx, None, c.E)
    np.testing.assert_array_equal(G.to_np(buf.expert_idx), idx)
    np.testing.assert_array_equal(G.to_np(buf.counts), counts)
    np.testing.assert_array_equal(G.to_np(buf.perm), perm)
    np.testing.assert_array_equal(G.to_np(buf.x_packed), li.x[perm // c.k])
    send_counts = counts.reshape(c.ep_world, c.E // c.ep_world)      # [destination rank][local expert]
    say(f"  send counts per destination rank {send_counts.sum(axis=1).tolist()}, "
        f"hottest expert / mean = {counts.max() / counts.mean():.2f}")
    assert counts.max() / counts.mean() > 3.0                          # Zipf-skewed load
    # destination rank r's slice of the send buffer is contiguous
    for rnk in range(c.ep_world):
        lo, hi = offsets[rnk * 4], offsets[(rnk + 1) * 4]
        assert ((idx.reshape(-1)[perm[lo:hi]] // 4) == rnk).all()


def test_ep_round_trip_four_ranks_against_the_oracle_layer():
    """Both all-to-alls of expert parallelism on one device (expert-parallelism figure; Algorithm 1,
    dispatch and combine): four emulated source ranks route and pack their own tokens, every shard's
    receive buffer is the concatenation, in rank order, of the slices the sources' HIP dispatch
    produced for it (host-side slicing stands in for the transfer), the shard runs the grouped FFN
    over the [source][local expert] segments, the results travel back into each source's packed
    order and through its combine.  Every source's y must equal the oracle's plain layer on that
    source's tokens: the sharding is invisible in the result."""
    c = WL.CONFIGS[5]
    W, k, d, F, E = c.ep_world, c.k, c.d, c.F, c.E
    E_loc = E // W
    T_src = 96
    base = WL.make_layer(5, layer=0, T=T_src)                     # the layer's weights (Zipf router bias)
    xs = []
    for rnk in range(W):
        for bump in range(20):
            xr = WL.make_layer(5, layer=rnk, bump=bump, with_experts=False, T=T_src).x
            if G.topk_margin(O.router_logits(xr, base.Wg, base.bg), k) >= 1e-4:
                break
        xs.append(xr)
    say(f"EP round trip: {W} ranks x {T_src} tokens, d={d} F={F} E={E}")
    ctx_src = B.Context(T_src, d, F, E, k, "bf16")
    Wg_dev, bg_dev = G.to_dev(base.Wg, "bf16"), G.f32_dev(base.bg)
    ws_small = torch.empty(1 << 16, dtype=torch.uint8, device=G.DEV)      # router and dispatch only: no hidden activations
    # ---- source side: router and dispatch with a packed send buffer
    src = []
    for rnk in range(W):
        buf = B.LayerBuffers(ctx_src, G.DEV, workspace=ws_small)
        x_dev = G.to_dev(xs[rnk], "bf16")
        ctx_src.moe_gate(x_dev, Wg_dev, bg_dev, buf.scores, buf.expert_idx)
        ctx_src.moe_dispatch(x_dev, buf.expert_idx, None, buf.x_packed, buf.counts, buf.offsets, buf.perm, buf.inv, ws_small)
        poison(buf.h_packed)
        src.append(buf)
    torch.cuda.synchronize()
    offs = [G.to_np(b_.offsets) for b_ in src]
    cnts = [G.to_np(b_.counts) for b_ in src]
    # ---- every shard: receive, grouped FFN over [source][local expert], send back
    for sh in range(W):
        lo_e, hi_e = sh * E_loc, (sh + 1) * E_loc
        pieces = [src[rnk].x_packed[offs[rnk][lo_e]:offs[rnk][hi_e]] for rnk in range(W)]
        recv = torch.cat(pieces, dim=0).contiguous()
        rows = recv.shape[0]
        recv_counts = np.array([[cnts[rnk][e] for e in range(lo_e, hi_e)] for rnk in range(W)], np.int32)
        assert recv_counts.sum() == rows
        say(f"  shard {sh}: {rows} rows, recv_counts {recv_counts.tolist()}")
        if rows == 0:
            continue
        ctx_sh = B.Context(rows, d, F, E_loc, 1, "bf16")
        seg_offsets = torch.empty(W * E_loc + 1, dtype=torch.int32, device=G.DEV)
        seg_expert = torch.empty(W * E_loc, dtype=torch.int32, device=G.DEV)
        ctx_sh.moe_ep_segments(G.i32_dev(recv_counts), seg_offsets, seg_expert)
        h_recv = torch.empty((rows, d), dtype=torch.bfloat16, device=G.DEV)
        poison(h_recv)
        ws = torch.empty(ctx_sh.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
        ctx_sh.moe_expert_ffn(recv, seg_offsets, seg_expert, rows, G.to_dev(base.W1[lo_e:hi_e], "bf16"), None,
                              G.to_dev(base.W2[lo_e:hi_e], "bf16"), None, h_recv, ws)
        torch.cuda.synchronize()
        ctx_sh.moe_expert_ffn_status(ws)
        assert_written(h_recv, rows, f"shard {sh} h")
        pos = 0
        for rnk in range(W):                                     # the return trip: same slices, other direction
            n = int(offs[rnk][hi_e] - offs[rnk][lo_e])
            src[rnk].h_packed[offs[rnk][lo_e]:offs[rnk][hi_e]] = h_recv[pos:pos + n]
            pos += n
        assert pos == rows
    # ---- home ranks: combine, and the whole trip against the oracle's layer
    for rnk in range(W):
        buf = src[rnk]
        assert_written(buf.h_packed, T_src * k, f"rank {rnk} returned rows")
        ctx_src.moe_combine(buf.h_packed, buf.inv, buf.scores, None, None, None, False, buf.y)
        torch.cuda.synchronize()
        ref = O.moe_layer(xs[rnk], base.Wg, base.bg, base.W1, None, base.W2, None, k)
        np.testing.assert_array_equal(G.to_np(buf.expert_idx), ref.idx)
        np.testing.assert_array_equal(G.to_np(buf.counts), ref.counts)
        np.testing.assert_array_equal(G.to_np(buf.perm), ref.perm)
        np.testing.assert_array_equal(G.to_np(buf.inv).reshape(T_src, k), ref.inv)
        G.assert_close_expert_rows(G.to_np(buf.h_packed), ref.h_packed, f"rank {rnk} h")
        G.assert_close_storage(G.to_np(buf.y), ref.y, "bf16", f"rank {rnk} y")


def test_expert_ffn_reports_a_max_rows_below_the_segment_table():
    """The FFN launch is sized from the host's max_rows; a segment table that holds more rows leaves
    rows uncomputed, and moe_expert_ffn_status must say so (and say nothing after a correct call)."""
    d, F, dtype = 128, 256, "bf16"
    seg_rows = [300, 200, 100]
    rows = sum(seg_rows)
    _, _, _, W1, b1, W2, b2 = G.small_inputs(91, 4, d, 3, F, dtype, bias=False)
    ctx = B.Context(rows, d, F, 3, 1, dtype)
    xp = torch.zeros((rows, d), dtype=torch.bfloat16, device=G.DEV)
    h = torch.empty((rows, d), dtype=torch.bfloat16, device=G.DEV)
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    so = G.i32_dev(np.concatenate([[0], np.cumsum(seg_rows)]))
    se = torch.arange(3, dtype=torch.int32, device=G.DEV)
    args = (G.to_dev(W1, dtype), None, G.to_dev(W2, dtype), None, h, ws)
    for max_rows, ok in ((rows, True), (rows - 1, False), (100, False), (0, False), (rows, True)):
        ctx.moe_expert_ffn(xp, so, se, max_rows, *args)
        if ok:
            ctx.moe_expert_ffn_status(ws)
        else:
            with pytest.raises(B.MoeError) as e:
                ctx.moe_expert_ffn_status(ws)
            assert e.value.status == B.MOE_ERR_SHAPE and str(rows) in str(e.value) and str(max_rows) in str(e.value)
    # float path
    ctx32 = B.Context(rows, d, F, 3, 1, "f32")
    ws32 = torch.empty(ctx32.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    x32 = torch.zeros((rows, d), dtype=torch.float32, device=G.DEV)
    h32 = torch.empty((rows, d), dtype=torch.float32, device=G.DEV)
    a32 = (G.to_dev(W1, "f32"), None, G.to_dev(W2, "f32"), None, h32, ws32)
    ctx32.moe_expert_ffn(x32, so, se, rows - 7, *a32)
    with pytest.raises(B.MoeError):
        ctx32.moe_expert_ffn_status(ws32)
    ctx32.moe_expert_ffn(x32, so, se, rows, *a32)
    ctx32.moe_expert_ffn_status(ws32)


@pytest.mark.parametrize("cfg,T", [(1, None), (2, None), (3, 1500)])
def test_expert_rows_written_straight_into_the_cache_give_the_same_bits(cfg, T):
    """The default path of a layer with a cache (Algorithm 4, "reuse stale h"; Section 4.1, persistent
    combine buffer): the expert call scatters the refreshed rows into H_cache itself and the combine reads
    every row from there.  Against the path through h_packed with write-through: y, H_cache and S_cache
    bit for bit over two steps and five policies, and h_packed never written."""
    li, _ = G.pick_layer(cfg, T=T)
    c = li.cfg
    dtype, k = c.dtype, c.k
    Tn = li.x.shape[0]
    say(f"rows to cache: config {cfg} T={Tn}")
    ctx = B.Context(Tn, c.d, c.F, c.E, k, dtype)
    dev = lambda a: G.to_dev(a, dtype)
    args = (dev(li.Wg), G.f32_dev(li.bg) if li.bg is not None else None, dev(li.W1), None, dev(li.W2), None)
    x0, x1 = dev(li.x), dev(WL.next_step_x(cfg, li.x))
    pols = [B.Policy(B.REFRESH_ALG4, step_t=1, stride_n=2), B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=Tn // 3),
            B.Policy(B.REFRESH_FRACTION_PAIR, n_units=Tn + Tn // 4), B.Policy(B.REFRESH_NONE),
            B.Policy(B.REFRESH_FRACTION_TOKEN, n_units=Tn // 2, use_fresh_scores=True)]
    for pol in pols:
        out = {}
        for direct in (False, True):
            buf = B.LayerBuffers(ctx, G.DEV, with_cache=True)
            poison(buf.h_packed)
            y0 = B.moe_layer_forward(ctx, buf, x0, *args, policy=B.Policy(B.REFRESH_ALL), rows_to_cache=direct).clone()
            y1 = B.moe_layer_forward(ctx, buf, x1, *args, policy=pol, rows_to_cache=direct).clone()
            torch.cuda.synchronize()
            ctx.moe_expert_ffn_status(buf.workspace)
            if direct:
                assert torch.isnan(buf.h_packed).all()          # the packed output buffer is not used at all
            out[direct] = (y0, y1, buf.H_cache.clone(), buf.S_cache.clone())
        for a, b_, name in zip(out[False], out[True], ("y step 0", "y step 1", "H_cache", "S_cache")):
            assert torch.equal(a, b_), f"{name} differs under {pol}"


def test_measurement_aids_run_and_do_what_they_say():
    """The library's calibration kernels and the between-GEMMs event (measurement aids of the C-ABI): the
    copy is exact, the MFMA loop runs, and the event recorded between the two GEMMs of an expert FFN call
    splits the call's time into two positive parts that add up to the whole."""
    src = torch.arange(1 << 22, dtype=torch.int32, device=G.DEV)
    dst = torch.zeros_like(src)
    B.moe_calibrate_copy(dst, src, 512)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    ops = torch.randn(16 * 256 * 48, device=G.DEV).to(torch.bfloat16)
    sink = torch.zeros(4, dtype=torch.float32, device=G.DEV)
    B.moe_calibrate_mfma(ops, sink, 64, 32)
    torch.cuda.synchronize()
    assert (sink == 0).all()

    d, F, rows = 256, 512, 2048
    _, _, _, W1, b1, W2, b2 = G.small_inputs(93, 4, d, 2, F, "bf16", bias=False)
    ctx = B.Context(rows, d, F, 2, 1, "bf16")
    xp = torch.zeros((rows, d), dtype=torch.bfloat16, device=G.DEV)
    h = torch.empty((rows, d), dtype=torch.bfloat16, device=G.DEV)
    ws = torch.empty(ctx.workspace_bytes(), dtype=torch.uint8, device=G.DEV)
    so = G.i32_dev(np.array([0, 1000, rows]))
    se = torch.arange(2, dtype=torch.int32, device=G.DEV)
    e0, em, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    em.record()
    ctx.moe_expert_ffn_between_event(em)
    e0.record()
    ctx.moe_expert_ffn(xp, so, se, rows, G.to_dev(W1, "bf16"), None, G.to_dev(W2, "bf16"), None, h, ws)
    e1.record()
    ctx.moe_expert_ffn_between_event(None)
    torch.cuda.synchronize()
    a, b_, whole = e0.elapsed_time(em), em.elapsed_time(e1), e0.elapsed_time(e1)
    assert a > 0 and b_ > 0 and abs(a + b_ - whole) < 0.05 * whole + 1e-3
    # and once the hook is removed the event is left alone
    ctx.moe_expert_ffn(xp, so, se, rows, G.to_dev(W1, "bf16"), None, G.to_dev(W2, "bf16"), None, h, ws)
    torch.cuda.synchronize()
    assert abs(e0.elapsed_time(em) - a) < 1e-6
