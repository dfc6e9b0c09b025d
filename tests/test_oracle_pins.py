"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin is independent of the oracle's own
code: library sorts and matmuls, closed forms, brute force in Python, invariants, and the
truth table of Algorithm 4 written out by hand under tests/golden/.
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import erf as sp_erf

from oracle import moe_oracle as O
from paper_2411_16786_amd import workloads as WL

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def np_gelu(u):
    return 0.5 * u * (1.0 + sp_erf(u / math.sqrt(2.0)))


def np_expert(x, W1, b1, W2, b2):
    """Two library matmuls (double): the textbook 2-layer MLP with exact GELU."""
    u = x.astype(np.float64) @ W1.astype(np.float64).T
    if b1 is not None:
        u = u + b1.astype(np.float64)
    h = np_gelu(u) @ W2.astype(np.float64).T
    if b2 is not None:
        h = h + b2.astype(np.float64)
    return h


# ----------------------------------------------------------------------------- router
def test_router_logits_match_library_matmul():
    r = rng(1)
    x = r.standard_normal((37, 29), dtype=np.float32)
    Wg = r.standard_normal((5, 29), dtype=np.float32)
    bg = r.standard_normal(5, dtype=np.float32)
    z = O.router_logits(x, Wg, bg)
    ref = x.astype(np.float64) @ Wg.astype(np.float64).T + bg.astype(np.float64)
    np.testing.assert_allclose(z, ref, rtol=1e-13, atol=1e-13)
    # no bias: a dropped or doubled bias term would show
    np.testing.assert_allclose(O.router_logits(x, Wg), ref - bg.astype(np.float64), rtol=1e-13, atol=1e-13)
    # a transposed operand would fail on a non-symmetric case
    x1 = np.zeros((1, 29), np.float32); x1[0, 3] = 2.0
    np.testing.assert_array_equal(O.router_logits(x1, Wg)[0], 2.0 * Wg[:, 3].astype(np.float64))


def test_topk_matches_full_library_sort():
    r = rng(2)
    for E, k in [(4, 2), (8, 2), (16, 2), (16, 5), (7, 7), (3, 1)]:
        z = r.standard_normal((200, E))
        # inject exact ties
        z[::3, E // 2] = z[::3, 0]
        z[::5, :] = np.round(z[::5, :])
        idx = O.topk(z, k)
        # library: lexsort by (-z, expert id): last key is primary
        for i in range(z.shape[0]):
            order = np.lexsort((np.arange(E), -z[i]))
            np.testing.assert_array_equal(idx[i], order[:k])


def test_topk_exhaustive_tie_patterns():
    for E in (2, 3, 4):
        rows = np.array(list(itertools.product([0.0, 1.0, 2.0], repeat=E)))
        for k in range(1, E + 1):
            idx = O.topk(rows, k)
            for i, row in enumerate(rows):
                want = sorted(range(E), key=lambda e: (-row[e], e))[:k]
                assert list(idx[i]) == want


def test_softmax_properties():
    r = rng(3)
    z = r.standard_normal((50, 8)) * 3
    idx = O.topk(z, 2)
    p, s = O.scores(z, idx)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)
    assert (p > 0).all()
    # shift invariance
    p2, s2 = O.scores(z + 123.25, idx)
    np.testing.assert_allclose(p2, p, rtol=1e-12)
    # ratio of two probabilities is exp of the logit difference
    np.testing.assert_allclose(p[:, 1] / p[:, 4], np.exp(z[:, 1] - z[:, 4]), rtol=1e-12)
    # scores are the probabilities at the selected experts, in rank order
    np.testing.assert_array_equal(s, np.take_along_axis(p, idx.astype(np.int64), axis=1))
    assert (s[:, 0] >= s[:, 1]).all()
    # large logits do not overflow
    pb, _ = O.scores(z + 1e4, idx)
    assert np.isfinite(pb).all()


def test_softmax_two_experts_is_logistic():
    r = rng(4)
    z = r.standard_normal((64, 2)) * 2
    idx = O.topk(z, 1)
    p, _ = O.scores(z, idx)
    np.testing.assert_allclose(p[:, 0], 1.0 / (1.0 + np.exp(z[:, 1] - z[:, 0])), rtol=1e-13)


def test_scores_renormalised_over_topk():
    r = rng(5)
    z = r.standard_normal((40, 6))
    idx = O.topk(z, 3)
    p, s = O.scores(z, idx, renorm_topk=True)
    np.testing.assert_allclose(s.sum(axis=1), 1.0, atol=1e-13)
    _, s_raw = O.scores(z, idx)
    np.testing.assert_allclose(s, s_raw / s_raw.sum(axis=1, keepdims=True), rtol=1e-13)


# ----------------------------------------------------------------------------- dispatch
@pytest.mark.parametrize("masked", [False, True])
def test_dispatch_is_a_bijection_in_expert_then_token_order(masked):
    r = rng(6)
    T, E, k = 301, 8, 2
    z = r.standard_normal((T, E))
    idx = O.topk(z, k)
    mask = (r.random((T, k)) < 0.6).astype(np.uint8) if masked else None
    counts, offsets, perm, inv = O.dispatch(idx, mask, E)
    live = np.ones(T * k, bool) if mask is None else mask.reshape(-1).astype(bool)
    R = int(live.sum())
    assert perm.shape[0] == R and counts.sum() == R and offsets[-1] == R
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    # bijection onto the refreshed pairs
    assert sorted(perm.tolist()) == np.nonzero(live)[0].tolist()
    flat_inv = inv.reshape(-1)
    np.testing.assert_array_equal(flat_inv[perm], np.arange(R))
    assert (flat_inv[~live] == -1).all()
    # order: expert ids non-decreasing, token ids increasing inside an expert
    e_of_row = idx.reshape(-1)[perm]
    assert (np.diff(e_of_row) >= 0).all()
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert (idx.reshape(-1)[seg] == e).all()
        assert (np.diff(seg // k) > 0).all()
    # the same permutation from a library stable sort
    pairs = np.nonzero(live)[0]
    want = pairs[np.argsort(idx.reshape(-1)[pairs], kind="stable")]
    np.testing.assert_array_equal(perm, want)
    np.testing.assert_array_equal(counts, np.bincount(idx.reshape(-1)[pairs], minlength=E))
    # rows are copied bit for bit
    x = r.standard_normal((T, 16), dtype=np.float32)
    xp = O.pack_rows(x, perm, k)
    np.testing.assert_array_equal(xp, x[perm // k])


def test_dispatch_empty_and_single_expert():
    idx = np.zeros((5, 1), np.int32)
    counts, offsets, perm, inv = O.dispatch(idx, np.zeros((5, 1), np.uint8), 3)
    assert counts.tolist() == [0, 0, 0] and perm.shape[0] == 0 and (inv == -1).all()
    counts, offsets, perm, inv = O.dispatch(idx, None, 3)
    assert counts.tolist() == [5, 0, 0] and perm.tolist() == [0, 1, 2, 3, 4]


# ----------------------------------------------------------------------------- expert FFN
def test_gelu_closed_form_values_through_a_1x1_expert():
    # with d = F = 1 and unit weights the expert is gelu itself; gelu(u) = u * Phi(u)
    xs = np.array([[0.0], [1.0], [-1.0], [2.0], [-3.0]], np.float32)
    one = np.ones((1, 1, 1), np.float32)
    h = O.expert_ffn(xs, [0, 5], [0], one, None, one, None)[:, 0]
    phi = lambda u: 0.5 * (1.0 + math.erf(u / math.sqrt(2.0)))
    want = [0.0, 0.8413447460685429, -0.15865525393145707, 1.9544997361036416, -3.0 * phi(-3.0)]
    np.testing.assert_allclose(h, want, rtol=1e-14, atol=1e-16)
    # gelu(u) - gelu(-u) = u
    np.testing.assert_allclose(h[1] - h[2], 1.0, rtol=1e-14)


def test_single_expert_reduces_to_two_library_matmuls():
    r = rng(7)
    n, d, F = 23, 12, 40
    x = r.standard_normal((n, d), dtype=np.float32)
    W1 = r.standard_normal((1, F, d), dtype=np.float32) * 0.3
    W2 = r.standard_normal((1, d, F), dtype=np.float32) * 0.3
    b1 = r.standard_normal((1, F), dtype=np.float32)
    b2 = r.standard_normal((1, d), dtype=np.float32)
    h = O.expert_ffn(x, [0, n], [0], W1, b1, W2, b2)
    np.testing.assert_allclose(h, np_expert(x, W1[0], b1[0], W2[0], b2[0]), rtol=1e-12, atol=1e-13)
    h0 = O.expert_ffn(x, [0, n], [0], W1, None, W2, None)
    np.testing.assert_allclose(h0, np_expert(x, W1[0], None, W2[0], None), rtol=1e-12, atol=1e-13)
    # zero weights leave only the output bias
    hz = O.expert_ffn(x, [0, n], [0], W1 * 0, b1 * 0, W2 * 0, b2)
    np.testing.assert_array_equal(hz, np.broadcast_to(b2[0].astype(np.float64), (n, d)))


def test_grouped_ffn_uses_each_segments_expert_and_row_selection():
    r = rng(8)
    d, F, E = 8, 24, 3
    offs = np.array([0, 4, 4, 11], np.int32)          # expert 1 gets no rows
    x = r.standard_normal((11, d), dtype=np.float32)
    W1 = r.standard_normal((E, F, d), dtype=np.float32)
    W2 = r.standard_normal((E, d, F), dtype=np.float32)
    h = O.expert_ffn(x, offs, [0, 1, 2], W1, None, W2, None)
    np.testing.assert_allclose(h[:4], np_expert(x[:4], W1[0], None, W2[0], None), rtol=1e-12)
    np.testing.assert_allclose(h[4:], np_expert(x[4:], W1[2], None, W2[2], None), rtol=1e-12)
    sel = np.array([10, 0, 5], np.int32)
    hs = O.expert_ffn(x, offs, [0, 1, 2], W1, None, W2, None, rows_sel=sel)
    np.testing.assert_array_equal(hs, h[sel])


# ----------------------------------------------------------------------------- whole layer
def small_layer(seed, T=48, d=16, E=4, F=32, bias=True):
    r = rng(seed)
    x = r.standard_normal((T, d), dtype=np.float32)
    Wg = r.standard_normal((E, d), dtype=np.float32) / np.float32(math.sqrt(d))
    bg = r.standard_normal(E, dtype=np.float32) * np.float32(0.5) if bias else None
    W1 = r.standard_normal((E, F, d), dtype=np.float32) * np.float32(0.2)
    W2 = r.standard_normal((E, d, F), dtype=np.float32) * np.float32(0.2)
    b1 = r.standard_normal((E, F), dtype=np.float32) * np.float32(0.1) if bias else None
    b2 = r.standard_normal((E, d), dtype=np.float32) * np.float32(0.1) if bias else None
    return x, Wg, bg, W1, b1, W2, b2


def test_k_equals_E_is_the_dense_gate_weighted_sum():
    x, Wg, bg, W1, b1, W2, b2 = small_layer(9)
    E = Wg.shape[0]
    res = O.moe_layer(x, Wg, bg, W1, b1, W2, b2, k=E)
    # no routing code at all: softmax by numpy, every expert on every token
    z = x.astype(np.float64) @ Wg.astype(np.float64).T + bg.astype(np.float64)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    dense = sum(p[:, [e]] * np_expert(x, W1[e], b1[e], W2[e], b2[e]) for e in range(E))
    np.testing.assert_allclose(res.y, dense, rtol=1e-11, atol=1e-13)


def test_identical_experts_give_expert_times_sum_of_gates():
    x, Wg, bg, W1, b1, W2, b2 = small_layer(10)
    W1[:] = W1[0]; W2[:] = W2[0]; b1[:] = b1[0]; b2[:] = b2[0]
    res = O.moe_layer(x, Wg, bg, W1, b1, W2, b2, k=2)
    want = np_expert(x, W1[0], b1[0], W2[0], b2[0]) * res.s.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(res.y, want, rtol=1e-11, atol=1e-13)


def test_top2_layer_against_a_per_token_python_restatement():
    x, Wg, bg, W1, b1, W2, b2 = small_layer(11, T=20)
    res = O.moe_layer(x, Wg, bg, W1, b1, W2, b2, k=2)
    z = x.astype(np.float64) @ Wg.astype(np.float64).T + bg.astype(np.float64)
    for i in range(x.shape[0]):
        order = sorted(range(Wg.shape[0]), key=lambda e: (-z[i, e], e))[:2]
        pe = np.exp(z[i] - z[i].max()); pe /= pe.sum()
        yi = sum(pe[e] * np_expert(x[i:i + 1], W1[e], b1[e], W2[e], b2[e])[0] for e in order)
        np.testing.assert_allclose(res.y[i], yi, rtol=1e-11, atol=1e-13)


def test_equation_1_gradient_of_output_norm():
    # d||y_i|| / d h_i^e = s_i^e y_i / ||y_i||   (Section 4.3, Equation 1)
    r = rng(12)
    T, k, d = 6, 2, 10
    h = r.standard_normal((T * k, d))
    s = r.random((T, k))
    inv = np.arange(T * k, dtype=np.int32).reshape(T, k)
    y = O.combine(h, inv, s, None)
    eps = 1e-6
    for (i, j, c) in [(0, 0, 0), (2, 1, 3), (5, 1, 9)]:
        hp = h.copy(); hp[i * k + j, c] += eps
        hm = h.copy(); hm[i * k + j, c] -= eps
        num = (np.linalg.norm(O.combine(hp, inv, s, None)[i]) -
               np.linalg.norm(O.combine(hm, inv, s, None)[i])) / (2 * eps)
        ana = s[i, j] * y[i, c] / np.linalg.norm(y[i])
        assert abs(num - ana) < 1e-8


# ----------------------------------------------------------------------------- refresh mask
def test_alg4_truth_table_from_the_paper():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "alg4_truth_table.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) > 20
    for t, n, j, want in [[int(v) for v in r_] for r_ in rows]:
        k = max(j + 1, 2)
        s = np.linspace(0.9, 0.1, 3 * k).reshape(3, k)
        mask, R = O.refresh_mask(s, O.REFRESH_ALG4, step_t=t, stride_n=n)
        assert (mask[:, j] == want).all(), (t, n, j)
        assert R == int(mask.sum())


def test_alg4_special_cases():
    r = rng(13)
    s = np.sort(r.random((100, 2)), axis=1)[:, ::-1].copy()
    for t in range(6):
        m1, R1 = O.refresh_mask(s, O.REFRESH_ALG4, step_t=t, stride_n=1)
        assert m1.all() and R1 == 200            # n = 1: every step is synchronous
        m2, R2 = O.refresh_mask(s, O.REFRESH_ALG4, step_t=t, stride_n=2)
        if t % 2:
            assert R2 == 100 and m2[:, 0].all() and not m2[:, 1].any()
        else:
            assert m2.all()
    # the pair form at n_units = T is the off-step of Algorithm 4
    mp, Rp = O.refresh_mask(s, O.REFRESH_FRACTION_PAIR, n_units=100)
    m2, _ = O.refresh_mask(s, O.REFRESH_ALG4, step_t=1, stride_n=2)
    np.testing.assert_array_equal(mp, m2)
    mp, Rp = O.refresh_mask(s, O.REFRESH_FRACTION_PAIR, n_units=200)
    assert mp.all() and Rp == 200


def test_ablation_variants_of_algorithm_4():
    # "High Score" / "Random" rows of the ablation table: same budget as Algorithm 4 (one slot per
    # token on off-steps, everything on t mod n == 0), another choice of the slot that stays fresh
    r = rng(41)
    T, k = 4000, 3
    s = -np.sort(-r.random((T, k)), axis=1)
    for kind in (O.REFRESH_ALG4, O.REFRESH_ALG4_HIGH, O.REFRESH_ALG4_RANDOM):
        on, R_on = O.refresh_mask(s, kind, step_t=4, stride_n=2, n_units=123)
        assert R_on == T * k and on.all()
        off, R_off = O.refresh_mask(s, kind, step_t=3, stride_n=2, n_units=123)
        assert R_off == T and (off.sum(axis=1) == 1).all()
    low, _ = O.refresh_mask(s, O.REFRESH_ALG4, 3, 2)
    high, _ = O.refresh_mask(s, O.REFRESH_ALG4_HIGH, 3, 2)
    assert low[:, 0].all() and high[:, k - 1].all()
    # HIGH deprioritises high scores: the fresh pair is the token's smallest activated score, LOW's the largest
    assert (s[high == 1] == s.min(axis=1)).all() and (s[low == 1] == s.max(axis=1)).all()
    # RANDOM: the slot is a function of (seed, token) only, roughly uniform over the slots, and
    # different seeds disagree on about (k-1)/k of the tokens
    a, _ = O.refresh_mask(s, O.REFRESH_ALG4_RANDOM, 3, 2, n_units=123)
    a2, _ = O.refresh_mask(s[::-1].copy(), O.REFRESH_ALG4_RANDOM, 5, 2, n_units=123)
    np.testing.assert_array_equal(a, a2)                       # scores and step do not enter
    b, _ = O.refresh_mask(s, O.REFRESH_ALG4_RANDOM, 3, 2, n_units=124)
    share = a.mean(axis=0)
    assert np.all(np.abs(share - 1.0 / k) < 0.03), share
    differ = (a.argmax(axis=1) != b.argmax(axis=1)).mean()
    assert abs(differ - (k - 1) / k) < 0.04
    for i in (0, 1, 77, T - 1):
        assert a[i].argmax() == O.mix32(123, i) % k
    # the mixer: zero is its fixed point, it is a bijection (no collisions on a sample), and one
    # flipped input bit flips about half of the output bits
    assert O.mix32(0, 0) == 0
    # published outputs of the MurmurHash3 32-bit finaliser for the inputs 1, 2 and 2^32 - 1 (they fix the
    # shifts and both multipliers), and the seed enters as seed * 0x9E3779B9 added to the token, mod 2^32
    assert O.mix32(0, 1) == 0x514E28B7 and O.mix32(0, 2) == 0x30F4C306 and O.mix32(0, 0xFFFFFFFF) == 0x81F16F39
    assert O.mix32(1, 0) == O.mix32(0, 0x9E3779B9) and O.mix32(3, 5) == O.mix32(0, (3 * 0x9E3779B9 + 5) % 2**32)
    vals = {O.mix32(7, i) for i in range(20000)}
    assert len(vals) == 20000
    flips = [bin(O.mix32(7, i) ^ O.mix32(7, i ^ 1)).count("1") for i in range(2000)]
    assert 14 < np.mean(flips) < 18
    with pytest.raises(ValueError):
        O.refresh_mask(s, O.REFRESH_ALG4_HIGH, 1, 0)


def test_fraction_masks_against_brute_force_sort_and_nesting():
    r = rng(14)
    T, k = 257, 2
    s = np.sort(r.random((T, k)), axis=1)[:, ::-1].copy()
    s[10:60, 0] = s[5, 0]            # exact ties: lower token index must win
    s[100:130, 1] = s[99, 1]
    prev_tok = np.zeros((T, k), np.uint8)
    prev_pair = np.zeros((T, k), np.uint8)
    for n_units in [0, 1, 7, 30, 64, 128, 200, 257]:
        m, R = O.refresh_mask(s, O.REFRESH_FRACTION_TOKEN, n_units=n_units)
        order = sorted(range(T), key=lambda i: (-s[i, 0], i))[:n_units]
        want = np.zeros((T, k), np.uint8); want[order, :] = 1
        np.testing.assert_array_equal(m, want)
        assert R == n_units * k
        assert (m >= prev_tok).all(); prev_tok = m
    for n_units in [0, 1, 50, 257, 258, 300, 514]:
        m, R = O.refresh_mask(s, O.REFRESH_FRACTION_PAIR, n_units=n_units)
        order = sorted(((j, -s[i, j], i) for i in range(T) for j in range(k)))[:n_units]
        want = np.zeros((T, k), np.uint8)
        for j, _, i in order:
            want[i, j] = 1
        np.testing.assert_array_equal(m, want)
        assert R == n_units
        assert (m >= prev_pair).all(); prev_pair = m
    with pytest.raises(ValueError):
        O.refresh_mask(s, O.REFRESH_FRACTION_TOKEN, n_units=T + 1)
    with pytest.raises(ValueError):
        O.refresh_mask(s, O.REFRESH_ALG4, step_t=1, stride_n=0)


# ----------------------------------------------------------------------------- cache / refresh fractions
def two_steps(seed=15):
    x0, Wg, bg, W1, b1, W2, b2 = small_layer(seed, T=40)
    r = rng(seed + 1)
    x1 = x0 + np.float32(0.1) * r.standard_normal(x0.shape, dtype=np.float32)
    return x0, x1, (Wg, bg, W1, b1, W2, b2)


def test_full_refresh_equals_synchronous_layer_and_fills_cache():
    x0, x1, w = two_steps()
    T, d, k = x0.shape[0], x0.shape[1], 2
    H = np.full((T, k, d), np.nan); S = np.full((T, k), np.nan)
    r0 = O.moe_layer(x0, *w, k=k, policy=O.REFRESH_ALL, H_cache=H, S_cache=S)
    plain = O.moe_layer(x0, *w, k=k)
    np.testing.assert_array_equal(r0.y, plain.y)
    # after a synchronous step the cache reproduces the output
    np.testing.assert_allclose((S[:, :, None] * H).sum(axis=1), r0.y, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(H.reshape(T * k, d), r0.h_packed[r0.inv.reshape(-1)])
    np.testing.assert_array_equal(S, r0.s)
    # FRACTION_TOKEN with every token = synchronous layer, bit for bit
    r1 = O.moe_layer(x1, *w, k=k, policy=O.REFRESH_FRACTION_TOKEN, n_units=T, H_cache=H.copy(), S_cache=S.copy())
    np.testing.assert_array_equal(r1.y, O.moe_layer(x1, *w, k=k).y)


def test_zero_refresh_returns_the_cache_untouched():
    x0, x1, w = two_steps(17)
    T, d, k = x0.shape[0], x0.shape[1], 2
    H = np.zeros((T, k, d)); S = np.zeros((T, k))
    r0 = O.moe_layer(x0, *w, k=k, H_cache=H, S_cache=S)
    H0, S0 = H.copy(), S.copy()
    r1 = O.moe_layer(x1, *w, k=k, policy=O.REFRESH_NONE, H_cache=H, S_cache=S)
    np.testing.assert_array_equal(r1.y, r0.y)
    np.testing.assert_array_equal(H, H0); np.testing.assert_array_equal(S, S0)
    assert r1.R == 0 and r1.perm.shape[0] == 0
    # with the fresh-score variant the cached rows are scaled by this step's scores instead
    r2 = O.moe_layer(x1, *w, k=k, policy=O.REFRESH_NONE, H_cache=H, S_cache=S, use_fresh_scores=True)
    np.testing.assert_allclose(r2.y, (r1.s[:, :, None] * H0).sum(axis=1), rtol=1e-13, atol=1e-15)


def test_partial_refresh_blends_fresh_and_cached_pairs():
    x0, x1, w = two_steps(19)
    T, d, k = x0.shape[0], x0.shape[1], 2
    H = np.zeros((T, k, d)); S = np.zeros((T, k))
    r0 = O.moe_layer(x0, *w, k=k, H_cache=H, S_cache=S)
    H0, S0 = H.copy(), S.copy()
    sync1 = O.moe_layer(x1, *w, k=k)
    r1 = O.moe_layer(x1, *w, k=k, policy=O.REFRESH_ALG4, step_t=1, stride_n=2, H_cache=H, S_cache=S)
    assert r1.R == T and r1.mask[:, 0].all() and not r1.mask[:, 1].any()
    # restated per token: slot 0 fresh from the synchronous step-1 layer, slot 1 from step 0
    h_sync = sync1.h_packed[sync1.inv.reshape(-1)].reshape(T, k, d)
    want = sync1.s[:, [0]] * h_sync[:, 0] + S0[:, [1]] * H0[:, 1]
    np.testing.assert_allclose(r1.y, want, rtol=1e-12, atol=1e-14)
    # write-through: refreshed rows replaced, the others unchanged bit for bit
    np.testing.assert_array_equal(H[:, 1], H0[:, 1]); np.testing.assert_array_equal(S[:, 1], S0[:, 1])
    np.testing.assert_allclose(H[:, 0], h_sync[:, 0], rtol=1e-13)
    np.testing.assert_array_equal(S[:, 0], sync1.s[:, 0])
    # a reused pair with no cache is an error
    with pytest.raises(ValueError):
        O.moe_layer(x1, *w, k=k, policy=O.REFRESH_ALG4, step_t=1, stride_n=2)


# ----------------------------------------------------------------------------- shared experts
def shared_weights(seed, S, d, F, bias=True):
    r = rng(seed)
    W1s = r.standard_normal((S, F, d), dtype=np.float32) * np.float32(0.2)
    W2s = r.standard_normal((S, d, F), dtype=np.float32) * np.float32(0.2)
    b1s = r.standard_normal((S, F), dtype=np.float32) * np.float32(0.1) if bias else None
    b2s = r.standard_normal((S, d), dtype=np.float32) * np.float32(0.1) if bias else None
    return W1s, b1s, W2s, b2s


def test_shared_experts_closed_forms():
    # d = F = 1, unit weights: each shared expert is gelu itself, so S of them give S * gelu(x)
    xs = np.array([[0.0], [1.0], [-1.0], [2.0]], np.float32)
    ones = np.ones((3, 1, 1), np.float32)
    out = O.shared_experts(xs, ones, None, ones, None)[:, 0]
    np.testing.assert_allclose(out, 3 * np.array([0.0, 0.8413447460685429, -0.15865525393145707,
                                                  1.9544997361036416]), rtol=1e-14, atol=1e-16)
    # zero weights leave the sum of the output biases; a bias on the hidden layer goes through gelu
    W1s, b1s, W2s, b2s = shared_weights(31, 2, 6, 10)
    x = rng(32).standard_normal((9, 6), dtype=np.float32)
    out = O.shared_experts(x, W1s * 0, b1s * 0, W2s * 0, b2s)
    np.testing.assert_allclose(out, np.broadcast_to(b2s.astype(np.float64).sum(axis=0), (9, 6)), rtol=1e-15)
    W2row = np.zeros((1, 1, 2), np.float32); W2row[0, 0] = [1.0, 0.0]
    out = O.shared_experts(np.zeros((1, 1), np.float32), np.zeros((1, 2, 1), np.float32),
                           np.array([[1.0, -1.0]], np.float32), W2row, None)
    np.testing.assert_allclose(out, [[0.8413447460685429]], rtol=1e-14)   # picks gelu(b1[0]) only


def test_shared_experts_against_the_segmented_c_routine_and_a_scalar_loop():
    # the dense numpy definition against (a) the C per-row routine run with one segment of all
    # rows per shared expert, (b) scalar Python loops with math.erf
    W1s, b1s, W2s, b2s = shared_weights(33, 2, 7, 13)
    T, d, F = 11, 7, 13
    x = rng(34).standard_normal((T, d), dtype=np.float32)
    out = O.shared_experts(x, W1s, b1s, W2s, b2s)
    via_c = sum(O.expert_ffn(x, [0, T], [e], W1s, b1s, W2s, b2s) for e in range(2))
    np.testing.assert_allclose(out, via_c, rtol=1e-12, atol=1e-14)
    for i in (0, 5, 10):
        for c in (0, 3, 6):
            acc = 0.0
            for e in range(2):
                acc += float(b2s[e, c])
                for f in range(F):
                    u = float(b1s[e, f]) + sum(float(W1s[e, f, q]) * float(x[i, q]) for q in range(d))
                    acc += float(W2s[e, c, f]) * 0.5 * u * (1.0 + math.erf(u / math.sqrt(2.0)))
            assert abs(out[i, c] - acc) <= 1e-12 * max(1.0, abs(acc))


def test_layer_with_shared_experts_adds_them_ungated_and_always_fresh():
    x0, x1, w = two_steps(23)
    Wg, bg, W1, b1, W2, b2 = w
    T, d, k, E = x0.shape[0], x0.shape[1], 2, Wg.shape[0]
    W1s, b1s, W2s, b2s = shared_weights(35, 2, d, W1.shape[1])
    cat = lambda a, b: np.concatenate([a, b], axis=0)
    wS = (Wg, bg, cat(W1, W1s), cat(b1, b1s), cat(W2, W2s), cat(b2, b2s))
    plain = O.moe_layer(x0, *w, k=k)
    both = O.moe_layer(x0, *wS, k=k, n_shared=2)
    # routing is untouched; y grows by the plain sum of the two dense FFNs (library matmuls)
    np.testing.assert_array_equal(both.idx, plain.idx); np.testing.assert_array_equal(both.s, plain.s)
    add = np_expert(x0, W1s[0], b1s[0], W2s[0], b2s[0]) + np_expert(x0, W1s[1], b1s[1], W2s[1], b2s[1])
    np.testing.assert_allclose(both.y, plain.y + add, rtol=1e-12, atol=1e-13)
    # a shared expert is a routed expert that every token selects with score 1: with one routed
    # expert and k = 1 the softmax score is 1, so sharing that expert's weights doubles the output
    one = O.moe_layer(x0, Wg[:1], bg[:1], W1[:1], b1[:1], W2[:1], b2[:1], k=1)
    two = O.moe_layer(x0, Wg[:1], bg[:1], cat(W1[:1], W1[:1]), cat(b1[:1], b1[:1]), cat(W2[:1], W2[:1]),
                      cat(b2[:1], b2[:1]), k=1, n_shared=1)
    np.testing.assert_allclose(two.y, 2.0 * one.y, rtol=1e-12, atol=1e-14)
    # staleness stays with the routed experts: with nothing refreshed the routed part is the
    # cache's, the shared part is this step's
    H = np.zeros((T, k, d)); S = np.zeros((T, k))
    r0 = O.moe_layer(x0, *wS, k=k, n_shared=2, H_cache=H, S_cache=S)
    r1 = O.moe_layer(x1, *wS, k=k, n_shared=2, policy=O.REFRESH_NONE, H_cache=H, S_cache=S)
    assert r1.R == 0
    add1 = np_expert(x1, W1s[0], b1s[0], W2s[0], b2s[0]) + np_expert(x1, W1s[1], b1s[1], W2s[1], b2s[1])
    np.testing.assert_allclose(r1.y, (r0.y - r0.y_shared) + add1, rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------- expert-parallel layout
def test_ep_receive_layout_and_segmented_ffn():
    r = rng(21)
    W, E, k, T, d, F = 4, 8, 2, 64, 8, 16
    E_loc = E // W
    W1 = r.standard_normal((E, F, d), dtype=np.float32) * np.float32(0.3)
    W2 = r.standard_normal((E, d, F), dtype=np.float32) * np.float32(0.3)
    shard = 1
    send_slices, send_counts = [], np.zeros((W, W, E_loc), np.int32)
    for src in range(W):
        x = r.standard_normal((T, d), dtype=np.float32)
        idx = O.topk(r.standard_normal((T, E)), k)
        counts, offsets, perm, inv = O.dispatch(idx, None, E)
        xp = O.pack_rows(x, perm, k)
        # experts are block-partitioned, so the packed order is already (dest rank, local expert)
        send_counts[src] = counts.reshape(W, E_loc)
        lo, hi = offsets[shard * E_loc], offsets[(shard + 1) * E_loc]
        send_slices.append(xp[lo:hi])
    recv = np.concatenate(send_slices)                      # what the all-to-all delivers
    recv_counts = send_counts[:, shard, :]
    seg_offsets, seg_expert = O.ep_segments(recv_counts)
    assert seg_offsets[-1] == recv.shape[0]
    np.testing.assert_array_equal(seg_expert, np.tile(np.arange(E_loc), W))
    np.testing.assert_array_equal(np.diff(seg_offsets), recv_counts.reshape(-1))
    Wl1, Wl2 = W1[shard * E_loc:(shard + 1) * E_loc], W2[shard * E_loc:(shard + 1) * E_loc]
    h_seg = O.expert_ffn(recv, seg_offsets, seg_expert, Wl1, None, Wl2, None)
    # regroup expert-major and run the plain per-expert grouping: same rows, same values
    row_e = np.repeat(seg_expert, np.diff(seg_offsets))
    order = np.argsort(row_e, kind="stable")
    offs_e = np.concatenate([[0], np.cumsum(np.bincount(row_e, minlength=E_loc))]).astype(np.int32)
    h_grp = O.expert_ffn(recv[order], offs_e, np.arange(E_loc), Wl1, None, Wl2, None)
    np.testing.assert_array_equal(h_seg[order], h_grp)
    for q in (0, recv.shape[0] // 2, recv.shape[0] - 1):
        e = row_e[q]
        np.testing.assert_allclose(h_seg[q], np_expert(recv[q:q + 1], Wl1[e], None, Wl2[e], None)[0], rtol=1e-12)


# ----------------------------------------------------------------------------- workload generators
def test_workload_generators_are_seeded_and_storage_exact():
    a = WL.make_layer(2, T=64)
    b = WL.make_layer(2, T=64)
    np.testing.assert_array_equal(a.x, b.x); np.testing.assert_array_equal(a.W1, b.W1)
    for arr in (a.x, a.Wg, a.W1, a.W2):
        np.testing.assert_array_equal(WL.bf16_round(arr), arr)       # already exact in bf16
    # LayerNorm-ed rows (before rounding): zero mean, unit variance
    assert abs(a.x.mean(axis=1)).max() < 1e-2 and abs((a.x ** 2).mean(axis=1) - 1).max() < 1e-2
    c1 = WL.make_layer(1)
    assert c1.x.shape == (64, 64) and c1.W1.shape == (4, 256, 64) and c1.W2.shape == (4, 64, 256)
    assert abs(c1.W1.std() - 0.02) < 1e-3
    # bf16 rounding is round-to-nearest-even
    v = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], np.float32)
    np.testing.assert_array_equal(WL.bf16_round(v), np.array([1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7], np.float32))
    ep = WL.make_ep_shard(rows=512, with_experts=False)
    assert ep.recv_counts.sum() == 512 and ep.recv_counts.shape == (4, 4)
    assert (ep.recv_counts.sum(axis=1) == 128).all()
    so, se = O.ep_segments(ep.recv_counts)
    np.testing.assert_array_equal(np.repeat(se, np.diff(so)), ep.row_expert)
