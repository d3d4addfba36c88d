"""Pins of the fp64 CPU oracle against things that are NOT the oracle: published known-answer
vectors, a library routine, closed forms, invariants and special cases that reduce to dense
attention.  None of these tests needs a GPU."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def topk_rows(scores, k):
    """deterministic top-k (value descending, index ascending), ascending output -- numpy only"""
    order = np.argsort(-scores, axis=-1, kind="stable")[..., :k]
    return np.sort(order, axis=-1).astype(np.int32)


# ------------------------------------------------------------------------------------------------
# Philox and the noise
# ------------------------------------------------------------------------------------------------
def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = oracle.philox4x32_10(w[:4], w[4:6])
        assert [int(x) for x in out] == w[6:]
        n += 1
    assert n == 3


def test_noise_is_a_24bit_integer_over_2_23_with_uniform_moments():
    ws = np.array([oracle.noise_unit(7, bh, i, j) for bh in range(2) for i in range(40) for j in range(250)])
    assert ws.min() >= -1.0 and ws.max() < 1.0
    scaled = ws * 2.0**23
    assert np.all(scaled == np.round(scaled))  # exact integers
    n = ws.size
    assert abs(ws.mean()) < 4.0 / math.sqrt(3 * n)  # sd of U[-1,1) is 1/sqrt(3)
    assert abs(ws.var() - 1.0 / 3.0) < 0.01
    # the four words of one Philox call serve key blocks 4c..4c+3; the next call is independent
    assert len(np.unique(ws)) > 0.99 * n


def test_noise_depends_on_every_coordinate_and_on_both_seed_words():
    base = oracle.noise_unit(5, 1, 2, 3)
    assert base == oracle.noise_unit(5, 1, 2, 3)
    others = [oracle.noise_unit(6, 1, 2, 3), oracle.noise_unit(5 + (1 << 32), 1, 2, 3), oracle.noise_unit(5, 0, 2, 3),
              oracle.noise_unit(5, 1, 3, 3), oracle.noise_unit(5, 1, 2, 2), oracle.noise_unit(5, 1, 2, 7)]
    assert all(o != base for o in others)


def _round_to_f32(x: Fraction) -> np.float32:
    """correctly rounded (nearest) binary32 of an exact rational, checked against both neighbours"""
    c = np.float32(float(x))
    best = c
    for cand in (np.nextafter(c, np.float32(-np.inf)), np.nextafter(c, np.float32(np.inf))):
        if abs(Fraction(float(cand)) - x) < abs(Fraction(float(best)) - x):
            best = cand
    return best


def test_noisy_score_is_one_correctly_rounded_fma():
    g = rng(0)
    s = g.standard_normal((1, 8, 8)).astype(np.float32)
    amp = np.float32(0.3)
    _, noisy = oracle.route(s, 2, seed=11, amp=float(amp), return_noisy=True)
    inexact_product = 0
    for i in range(8):
        for j in range(8):
            w = oracle.noise_unit(11, 0, i, j)
            exact = Fraction(float(amp)) * Fraction(w) + Fraction(float(s[0, i, j]))
            want = _round_to_f32(exact)
            if Fraction(float(np.float32(float(amp) * w))) != Fraction(float(amp)) * Fraction(w):
                inexact_product += 1
            assert noisy[0, i, j] == want
    assert inexact_product > 0  # the case where fma and mul-then-add can differ occurs


# ------------------------------------------------------------------------------------------------
# k from the keep ratio
# ------------------------------------------------------------------------------------------------
def test_topk_count_rounding_and_clamps():
    assert oracle.topk_count(16, 0.25) == 4
    assert oracle.topk_count(512, 0.20) == 102  # 102.4
    assert oracle.topk_count(1182, 0.15) == 177  # 177.3 : the 85 % sparsity rows of Table 1
    assert oracle.topk_count(1154, 0.05) == 58  # 57.7
    assert oracle.topk_count(10, 0.25) == 3  # 2.5 rounds up
    assert oracle.topk_count(100, 1e-9) == 1
    assert oracle.topk_count(100, 1.0) == 100


# ------------------------------------------------------------------------------------------------
# dense attention (Eq.1) against a library routine
# ------------------------------------------------------------------------------------------------
def test_dense_matches_torch_sdpa_float64():
    g = rng(1)
    q, k, v = (g.standard_normal((3, 70, 16)) for _ in range(3))
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None])[0].numpy()
    got, lse = oracle.dense_attention(q, k, v, return_lse=True)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    logits = torch.from_numpy(q) @ torch.from_numpy(k).transpose(1, 2) / math.sqrt(16)
    np.testing.assert_allclose(lse, torch.logsumexp(logits, -1).numpy(), rtol=0, atol=1e-12)
    # a row subset gives the same rows
    rows = np.array([0, 13, 69], np.int32)
    np.testing.assert_array_equal(oracle.dense_attention(q, k, v, q_rows=rows), got[:, rows])
    # a non-default scale is honoured
    want2 = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], scale=0.7)[0].numpy()
    np.testing.assert_allclose(oracle.dense_attention(q, k, v, scale=0.7), want2, rtol=0, atol=1e-13)


def test_dense_softmax_rows_sum_to_one():
    g = rng(2)
    q, k = g.standard_normal((2, 50, 8)), g.standard_normal((2, 50, 8))
    v = np.ones((2, 50, 8))
    np.testing.assert_allclose(oracle.dense_attention(q, k, v), 1.0, rtol=0, atol=1e-14)
    # V = one-hot of the key position recovers the attention matrix itself
    vv = np.zeros((1, 6, 6))
    vv[0] = np.eye(6)
    p = oracle.dense_attention(q[:1, :6, :6], k[:1, :6, :6], vv)
    assert np.all(p > 0)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)


# ------------------------------------------------------------------------------------------------
# pooling, scores, statistics
# ------------------------------------------------------------------------------------------------
def test_block_mean_and_scores_match_numpy_including_ragged_tail_and_bias():
    g = rng(3)
    n, b, d = 45, 8, 4  # 6 blocks, the last with 5 tokens
    q, k = g.standard_normal((2, n, d)), g.standard_normal((2, n, d))
    qm = np.stack([q[:, s:s + b].mean(1) for s in range(0, n, b)], 1)
    km = np.stack([k[:, s:s + b].mean(1) for s in range(0, n, b)], 1)
    np.testing.assert_allclose(oracle.block_mean(k, b), km, atol=1e-15)
    want = np.einsum("hid,hjd->hij", qm, km) / math.sqrt(d)
    np.testing.assert_allclose(oracle.block_scores(q, k, b), want, atol=1e-14)
    bias = g.standard_normal((2, 6))
    np.testing.assert_allclose(oracle.block_scores(q, k, b, scale=0.3, key_bias=bias),
                               want * math.sqrt(d) * 0.3 + bias[:, None, :], atol=1e-14)


def test_H_of_a_two_token_block_closed_form():
    # Eq.5 on a block {1,2}: H = (k1-kbar)^T v1 + (k2-kbar)^T v2 = 1/2 (k1-k2)^T (v1-v2)
    g = rng(4)
    k, v = g.standard_normal((1, 2, 5)), g.standard_normal((1, 2, 5))
    st = oracle.kv_stats(k, v, block=2, group=1, want_hj=True)
    want = 0.5 * np.outer(k[0, 0] - k[0, 1], v[0, 0] - v[0, 1])
    np.testing.assert_allclose(st["hj"][0, 0], want, atol=1e-15)
    np.testing.assert_allclose(st["hg"][0, 0], want, atol=1e-15)
    assert abs(want[1, 3] - want[3, 1]) > 1e-3  # not symmetric: a transposed H would fail
    np.testing.assert_allclose(st["vs"][0, 0], v[0].sum(0), atol=1e-15)
    np.testing.assert_allclose(st["kbar"][0, 0], k[0].mean(0), atol=1e-15)


def test_group_means_and_global_mean_of_H():
    g = rng(5)
    n, b, d = 7 * 4 + 2, 4, 3  # 8 blocks, ragged tail of 2 tokens
    k, v = g.standard_normal((2, n, d)), g.standard_normal((2, n, d))
    hj = oracle.kv_stats(k, v, b, 1, want_hj=True)["hj"]
    # Eq.5 via the algebraically equal form  K^T V - b_j kbar^T vbar
    for j in range(8):
        kb, vb = k[0, 4 * j:4 * j + 4], v[0, 4 * j:4 * j + 4]
        np.testing.assert_allclose(hj[0, j], kb.T @ vb - len(kb) * np.outer(kb.mean(0), vb.mean(0)), atol=1e-13)
    hg3 = oracle.kv_stats(k, v, b, 3)["hg"]  # groups {0,1,2},{3,4,5},{6,7}
    assert hg3.shape == (2, 3, d, d)
    np.testing.assert_allclose(hg3[:, 0], hj[:, 0:3].mean(1), atol=1e-14)
    np.testing.assert_allclose(hg3[:, 2], hj[:, 6:8].mean(1), atol=1e-14)  # short last group: mean over 2
    np.testing.assert_allclose(oracle.kv_stats(k, v, b, 100)["hg"][:, 0], hj.mean(1), atol=1e-14)  # Eq.6


def test_proposition1_group_mean_minimises_within_group_squares():
    g = rng(6)
    n, b, d, G = 64 * 4, 4, 6, 8
    k, v = g.standard_normal((1, n, d)), g.standard_normal((1, n, d))
    st = oracle.kv_stats(k, v, b, G, want_hj=True)
    hglob = st["hj"][0].mean(0)
    for gi in range(st["hg"].shape[1]):
        blk = st["hj"][0, gi * G:(gi + 1) * G]
        within = ((blk - st["hg"][0, gi]) ** 2).sum()
        assert within <= ((blk - hglob) ** 2).sum() + 1e-12  # Eq.19
        for _ in range(3):  # Eq.18, any matrix C
            c = st["hg"][0, gi] + 0.1 * g.standard_normal((d, d))
            assert within <= ((blk - c) ** 2).sum()


def test_lemma1_bound_holds():
    g = rng(7)
    n, b, d, G, ksel = 40 * 4, 4, 5, 8, 6
    q, k, v = (g.standard_normal((1, n, d)) for _ in range(3))
    st = oracle.kv_stats(k, v, b, G, want_hj=True)
    for t in (0, 17, 159):
        sel = np.sort(g.choice(40, ksel, replace=False)).astype(np.int32)
        r, bound = oracle.lemma1(q[0, t] / math.sqrt(d), st["kbar"][0], st["hj"][0], st["hg"][0], G, sel)
        assert 0 < r <= bound * (1 + 1e-12)


def _lemma1_by_hand(q_scaled, k, v, b, G, sel, group_of=None):
    """Appendix "Error Analysis", Lemma 1, evaluated in numpy straight from K and V (no oracle call):
    R = sum_{j in U} alpha_j (H_j - Hbar^{(g(j))}),  M = max_{j in U} ||H_j - Hbar^{(g(j))}||_F,  sum_{j in U} alpha_j,
    alpha_j = exp(q~ . Kbar_j) divided by its largest value over U (a common factor of both sides of the bound)."""
    n, d = k.shape
    nb = -(-n // b)
    blocks = [slice(j * b, min((j + 1) * b, n)) for j in range(nb)]
    kbar = np.stack([k[s].mean(0) for s in blocks])
    hj = np.stack([(k[s] - k[s].mean(0)).T @ v[s] for s in blocks])  # Eq.5
    group_of = group_of or (lambda j: j // G)
    members = {}
    for j in range(nb):
        members.setdefault(j // G, []).append(j)  # Eq.12: consecutive blocks, the last group short
    hbar = {g: np.mean([hj[j] for j in js], axis=0) for g, js in members.items()}
    unsel = [j for j in range(nb) if j not in set(int(x) for x in sel)]
    z = np.array([q_scaled @ kbar[j] for j in unsel])
    alpha = np.exp(z - z.max())
    dev = [hj[j] - hbar[group_of(j)] for j in unsel]
    R = sum(a * dv for a, dv in zip(alpha, dev))
    return np.sqrt((R * R).sum()), max(np.sqrt((dv * dv).sum()) for dv in dev) * alpha.sum()


def test_lemma1_values_against_direct_evaluation():
    """both outputs of oracle.lemma1 against the definition written out from K and V: four groups, the last one
    short (3 blocks of 8) and its last block ragged; a wrong group assignment changes the value by far more than
    the tolerance, so the comparison can fail"""
    g = rng(70)
    b, d, G, ksel = 4, 5, 8, 5
    n = 26 * b + 3  # 27 blocks: groups of 8, 8, 8, 3; tail block of 3 tokens
    q, k, v = (g.standard_normal((1, n, d)) for _ in range(3))
    st = oracle.kv_stats(k, v, b, G, want_hj=True)
    assert st["hg"].shape[1] == 4
    for t in (0, 50, n - 1):
        sel = np.sort(g.choice(27, ksel, replace=False)).astype(np.int32)
        qs = q[0, t] / math.sqrt(d)
        r, bound = oracle.lemma1(qs, st["kbar"][0], st["hj"][0], st["hg"][0], G, sel)
        want_r, want_bound = _lemma1_by_hand(qs, k[0], v[0], b, G, sel)
        np.testing.assert_allclose(r, want_r, rtol=1e-12)
        np.testing.assert_allclose(bound, want_bound, rtol=1e-12)
        # sensitivity: the same evaluation with the group boundaries off by one block, or with every block compared
        # with the next group's mean, is nowhere near
        wrong_r, _ = _lemma1_by_hand(qs, k[0], v[0], b, G, sel, group_of=lambda j: min((j + 1) // G, 3))
        assert abs(wrong_r - want_r) > 1e-3 * want_r
        wrong_r, wrong_bound = _lemma1_by_hand(qs, k[0], v[0], b, G, sel, group_of=lambda j: (j // G + 1) % 4)
        assert abs(wrong_r - want_r) > 1e-3 * want_r and abs(wrong_bound - want_bound) > 1e-3 * want_bound
    # with every deviation zero the residual vanishes: one group per block
    st1 = oracle.kv_stats(k, v, b, 1, want_hj=True)
    r, bound = oracle.lemma1(q[0, 0] / math.sqrt(d), st1["kbar"][0], st1["hj"][0], st1["hg"][0], 1, np.array([2], np.int32))
    assert r < 1e-13 and bound < 1e-13


# ------------------------------------------------------------------------------------------------
# the piecewise attention
# ------------------------------------------------------------------------------------------------
def _all_blocks(BH, NB):
    return np.broadcast_to(np.arange(NB, dtype=np.int32), (BH, NB, NB)).copy()


def _random_routing(g, BH, NB, k):
    return np.stack([[np.sort(g.choice(NB, k, replace=False)) for _ in range(NB)] for _ in range(BH)]).astype(np.int32)


@pytest.mark.parametrize("n,b", [(64, 8), (61, 8)])
def test_keep_everything_equals_dense(n, b):
    g = rng(8)
    q, k, v = (g.standard_normal((2, n, 8)) for _ in range(3))
    NB = oracle.n_blocks(n, b)
    res = oracle.pasa_attention(q, k, v, _all_blocks(2, NB), b, group=4, return_all=True)
    want, lse = oracle.dense_attention(q, k, v, return_lse=True)
    np.testing.assert_allclose(res["o"], want, rtol=0, atol=1e-13)
    np.testing.assert_allclose(res["lse"], lse, rtol=0, atol=1e-12)
    assert np.all(res["parts"][:, :, 1:] == 0)


def test_weights_sum_to_one_and_constant_v_is_reproduced():
    g = rng(9)
    n, b, d = 93, 8, 6  # 12 blocks, tail of 5
    q, k = g.standard_normal((2, n, d)), g.standard_normal((2, n, d))
    c = g.standard_normal(d)
    v = np.broadcast_to(c, (2, n, d)).copy()
    idx = _random_routing(g, 2, 12, 3)
    for G in (1, 4, 32):
        res = oracle.pasa_attention(q, k, v, idx, b, group=G, return_all=True)
        np.testing.assert_allclose(res["wsum"].sum(-1), 1.0, atol=1e-14)
        assert np.all(res["wsum"] > 0)
        np.testing.assert_allclose(res["o"], np.broadcast_to(c, (2, n, d)), atol=1e-13)
        np.testing.assert_allclose(res["parts"][:, :, 2], 0.0, atol=1e-13)  # H_j = 0 when V is constant


@pytest.mark.parametrize("n", [96, 91])
def test_block_constant_keys_make_the_approximation_exact(n):
    # if every key of a block equals the block mean, the Taylor expansion has no remainder and
    # H_j = 0: the piecewise output equals dense attention for ANY routing, ragged tail included
    g = rng(10)
    b, d = 8, 5
    NB = oracle.n_blocks(n, b)
    q, v = g.standard_normal((2, n, d)), g.standard_normal((2, n, d))
    k = np.repeat(g.standard_normal((2, NB, d)), b, axis=1)[:, :n]
    want, lse = oracle.dense_attention(q, k, v, return_lse=True)
    for ksel, G in ((1, 1), (3, 4), (NB - 1, 32)):
        idx = _random_routing(g, 2, NB, ksel)
        got = oracle.pasa_attention(q, k, v, idx, b, group=G, return_all=True)
        np.testing.assert_allclose(got["o"], want, rtol=0, atol=1e-13)
        np.testing.assert_allclose(got["lse"], lse, rtol=0, atol=1e-12)


def test_first_order_term_removes_the_linear_error():
    # keys = block centroid + eps*delta with zero-mean delta.  With per-block statistics (G=1) the
    # error against dense attention is O(eps^2); with the zeroth-order term alone it is O(eps).
    g = rng(11)
    n, b, d = 64, 8, 4
    q, v = g.standard_normal((1, n, d)), g.standard_normal((1, n, d))
    cent = np.repeat(g.standard_normal((1, 8, d)), b, axis=1)
    delta = g.standard_normal((1, 8, b, d))
    delta -= delta.mean(2, keepdims=True)
    delta = delta.reshape(1, n, d)
    idx = _random_routing(g, 1, 8, 1)
    err0, err1 = [], []
    for eps in (1e-2, 1e-3):
        k = cent + eps * delta
        want = oracle.dense_attention(q, k, v)
        err1.append(np.abs(oracle.pasa_attention(q, k, v, idx, b, group=1, terms=3) - want).max())
        err0.append(np.abs(oracle.pasa_attention(q, k, v, idx, b, group=1, terms=1) - want).max())
    slope0 = math.log10(err0[0] / err0[1])
    slope1 = math.log10(err1[0] / err1[1])
    assert 0.9 < slope0 < 1.1, (err0, slope0)
    assert 1.9 < slope1 < 2.1, (err1, slope1)


def test_first_order_sign_and_orientation_by_direct_evaluation():
    # one unselected block of two tokens, everything written out by hand
    g = rng(12)
    d = 3
    q = g.standard_normal((1, 4, d))
    k = g.standard_normal((1, 4, d))
    v = g.standard_normal((1, 4, d))
    idx = np.array([[[0], [0]]], np.int32)  # both query blocks select key block 0; block 1 unselected
    res = oracle.pasa_attention(q, k, v, idx, block=2, group=1, scale=1.0, return_all=True)
    t = 3
    qt = q[0, t]
    e = np.exp(k[0, :2] @ qt)
    kb = k[0, 2:].mean(0)
    a = math.exp(kb @ qt)
    H = 0.5 * np.outer(k[0, 2] - k[0, 3], v[0, 2] - v[0, 3])
    num = e @ v[0, :2] + a * v[0, 2:].sum(0) + a * (qt @ H)
    den = e.sum() + 2 * a
    np.testing.assert_allclose(res["o"][0, t], num / den, atol=1e-14)
    np.testing.assert_allclose(res["parts"][0, t, 2], a * (qt @ H) / den, atol=1e-14)
    assert np.abs(qt @ H - H @ qt).max() > 1e-3


def test_single_group_reproduces_the_global_formula_and_G1_the_per_block_one():
    g = rng(13)
    n, b, d = 80, 8, 4
    q, k, v = (g.standard_normal((1, n, d)) for _ in range(3))
    idx = _random_routing(g, 1, 10, 3)
    st = oracle.kv_stats(k, v, b, 1, want_hj=True)
    hbar = st["hj"][0].mean(0)  # Eq.6
    sc = 1 / math.sqrt(d)
    o_glob = oracle.pasa_attention(q, k, v, idx, b, group=10_000)
    o_blk = oracle.pasa_attention(q, k, v, idx, b, group=1)
    for t in (0, 33, 79):
        qt = q[0, t] * sc
        S = set(idx[0, t // b].tolist())
        U = [j for j in range(10) if j not in S]
        ex = np.concatenate([np.arange(j * b, (j + 1) * b) for j in sorted(S)])
        e = np.exp(k[0, ex] @ qt)
        al = np.exp(st["kbar"][0, U] @ qt)
        den = e.sum() + b * al.sum()
        num7 = e @ v[0, ex] + al @ st["vs"][0, U] + (qt @ hbar) * al.sum()  # Eq.7
        np.testing.assert_allclose(o_glob[0, t], num7 / den, atol=1e-13)
        num13 = e @ v[0, ex] + al @ st["vs"][0, U] + sum(a * (qt @ st["hj"][0, j]) for a, j in zip(al, U))  # Eq.13
        np.testing.assert_allclose(o_blk[0, t], num13 / den, atol=1e-13)


def test_identical_blocks_inside_a_group_make_grouping_lossless():
    g = rng(14)
    b, d, G = 4, 3, 4
    # 3 groups, each made of 4 copies of one block
    kb, vb = g.standard_normal((1, 3, b, d)), g.standard_normal((1, 3, b, d))
    k = np.repeat(kb, G, axis=1).reshape(1, 3 * G * b, d)
    v = np.repeat(vb, G, axis=1).reshape(1, 3 * G * b, d)
    q = g.standard_normal(k.shape)
    idx = _random_routing(g, 1, 12, 2)
    np.testing.assert_allclose(oracle.pasa_attention(q, k, v, idx, b, group=G),
                               oracle.pasa_attention(q, k, v, idx, b, group=1), atol=1e-13)
    # ... and it differs from the single global matrix
    assert np.abs(oracle.pasa_attention(q, k, v, idx, b, group=G) - oracle.pasa_attention(q, k, v, idx, b, group=99)).max() > 1e-4


def test_group_zero_is_keep_or_drop_and_q_block_subset():
    g = rng(15)
    n, b, d = 48, 8, 4
    q, k, v = (g.standard_normal((1, n, d)) for _ in range(3))
    idx = _random_routing(g, 1, 6, 2)
    got = oracle.pasa_attention(q, k, v, idx, b, group=0)
    for i in range(6):  # dense attention restricted to the selected keys (Eq.3)
        cols = np.concatenate([np.arange(j * b, (j + 1) * b) for j in idx[0, i]])
        want = oracle.dense_attention(q[:, i * b:(i + 1) * b], k[:, cols], v[:, cols])
        # dense_attention needs equal lengths for q and k: evaluate row by row instead
        for t in range(i * b, (i + 1) * b):
            e = np.exp(k[0, cols] @ q[0, t] / math.sqrt(d))
            np.testing.assert_allclose(got[0, t], (e @ v[0, cols]) / e.sum(), atol=1e-14)
    sub = oracle.pasa_attention(q, k, v, idx, b, group=2, q_blocks=[1, 4])
    full = oracle.pasa_attention(q, k, v, idx, b, group=2)
    np.testing.assert_array_equal(sub[:, 8:16], full[:, 8:16])
    np.testing.assert_array_equal(sub[:, 32:40], full[:, 32:40])
    assert np.isnan(sub[:, 0:8]).all()


# ------------------------------------------------------------------------------------------------
# routing
# ------------------------------------------------------------------------------------------------
def test_zero_amplitude_is_deterministic_topk():
    g = rng(16)
    s = g.standard_normal((3, 37, 37)).astype(np.float32)
    s[0, 0, 5] = s[0, 0, 9] = s[0, 0].max() + 1  # a tie at the top: lower index first
    s[1, 2, :] = 0.25  # a fully tied row selects the first k blocks
    for k in (1, 7, 37):
        got = oracle.route(s, k, seed=3, amp=0.0)
        np.testing.assert_array_equal(got, topk_rows(s, k))
    assert oracle.route(s, 1, seed=3, amp=0.0)[0, 0, 0] == 5
    np.testing.assert_array_equal(oracle.route(s, 4, 3, 0.0)[1, 2], [0, 1, 2, 3])


def test_negative_zero_ties_with_positive_zero_and_negatives_rank_below():
    s = np.zeros((1, 4, 4), np.float32)
    s[0, :, 1] = -0.0
    s[0, :, 0] = -1.0
    s[0, 3, :] = [-3.0, -2.0, -0.5, -1.0]
    got = oracle.route(s, 2, 0, 0.0)
    np.testing.assert_array_equal(got[0, 0], [1, 2])  # -0 ties with +0: lower index first
    np.testing.assert_array_equal(got[0, 3], [2, 3])  # among negatives the larger value wins


def test_noisy_routing_is_topk_of_the_noisy_scores_and_is_seeded():
    g = rng(17)
    s = g.standard_normal((2, 64, 64)).astype(np.float32)
    idx, noisy = oracle.route(s, 9, seed=1234, amp=0.5, return_noisy=True)
    np.testing.assert_array_equal(idx, topk_rows(noisy, 9))
    assert np.all(np.diff(idx, axis=-1) > 0)
    assert np.abs(noisy - s).max() <= 0.5 and np.abs(noisy - s).max() > 0.4
    np.testing.assert_array_equal(idx, oracle.route(s, 9, seed=1234, amp=0.5))
    assert (oracle.route(s, 9, seed=1235, amp=0.5) != idx).any()
    assert (oracle.route(s, 9, seed=1234, amp=0.0) != idx).any()
    # head identity comes from bh_ids, not from the position in the batch
    np.testing.assert_array_equal(oracle.route(s[1:], 9, 1234, 0.5, bh_ids=[1]), idx[1:])
    assert (oracle.route(s[1:], 9, 1234, 0.5) != idx[1:]).any()


def test_huge_amplitude_selects_every_block_equally_often():
    s = np.linspace(-1, 1, 32, dtype=np.float32)[None, None, :].repeat(32, 1)
    counts = np.zeros(32)
    for seed in range(200):
        idx = oracle.route(s, 8, seed=seed, amp=1e6)
        counts += np.bincount(idx.ravel(), minlength=32)
    freq = counts / (200 * 32)
    np.testing.assert_allclose(freq, 8 / 32, atol=0.03)


# ------------------------------------------------------------------------------------------------
# covariance-aware routing prior (Eq.8, second term)
# ------------------------------------------------------------------------------------------------
def _brute_force_prior(K, V, b, G, eps):
    """Eq.5, Eq.12 and the norm written with Python loops over tokens and matrix elements (tiny inputs only)"""
    n, d = len(K), len(K[0])
    NB = -(-n // b)
    H = []
    for j in range(NB):
        rows = range(j * b, min((j + 1) * b, n))
        kbar = [sum(K[r][c] for r in rows) / len(rows) for c in range(d)]
        H.append([[sum((K[r][a] - kbar[a]) * V[r][c] for r in rows) for c in range(d)] for a in range(d)])
    G = min(G, NB)
    out = []
    for j in range(NB):
        members = range((j // G) * G, min((j // G + 1) * G, NB))
        ss = 0.0
        for a in range(d):
            for c in range(d):
                mean = sum(H[m][a][c] for m in members) / len(members)
                ss += (H[j][a][c] - mean) ** 2
        out.append(math.log(math.sqrt(ss) + eps))
    return np.array(out)


@pytest.mark.parametrize("G", [1, 2, 3, 100])
def test_key_prior_against_brute_force(G):
    g = rng(31)
    n, d, b = 23, 4, 4  # 6 blocks, the last one of 3 tokens; G=3: two full groups; G=2: three; G=100: one
    K, V = g.standard_normal((n, d)), g.standard_normal((n, d))
    got = oracle.key_prior(K[None], V[None], b, G, eps=1e-6)[0]
    np.testing.assert_allclose(got, _brute_force_prior(K.tolist(), V.tolist(), b, G, 1e-6), rtol=1e-10, atol=1e-10)


def test_key_prior_special_cases():
    g = rng(32)
    n, d, b = 64, 8, 8
    K, V = g.standard_normal((n, d)), g.standard_normal((n, d))
    # a group of one block is its own mean: the norm vanishes and only eps is left
    np.testing.assert_allclose(oracle.key_prior(K[None], V[None], b, 1, eps=1e-3), math.log(1e-3), atol=1e-9)
    # identical blocks inside a group: same
    Kr, Vr = np.tile(K[:b], (8, 1)), np.tile(V[:b], (8, 1))
    np.testing.assert_allclose(oracle.key_prior(Kr[None], Vr[None], b, 4, eps=1e-3), math.log(1e-3), atol=1e-6)
    # H is linear in V and invariant to a constant shift of K: beta(K + c, s V) = beta(K, V) + log s  (eps = 0)
    b0 = oracle.key_prior(K[None], V[None], b, 4, eps=0.0)
    b1 = oracle.key_prior((K + 3.0)[None], (2.5 * V)[None], b, 4, eps=0.0)
    np.testing.assert_allclose(b1, b0 + math.log(2.5), atol=1e-9)
    # one block differs from seven identical ones: closed form from H of the odd block
    Ko, Vo = Kr.copy(), Vr.copy()
    Vo[:b] = g.standard_normal((b, d))
    st = oracle.kv_stats(Ko[None], Vo[None], b, 8, want_hj=True)
    delta = st["hj"][0, 0] - st["hj"][0, 1]
    fro = np.linalg.norm(delta)
    want = np.array([math.log(fro * 7 / 8)] + [math.log(fro / 8)] * 7)
    np.testing.assert_allclose(oracle.key_prior(Ko[None], Vo[None], b, 8, eps=0.0)[0], want, atol=1e-9)


# ------------------------------------------------------------------------------------------------
# curvature-aware budget (Eq.9-11) and its L1 signal
# ------------------------------------------------------------------------------------------------
def test_budget_schedule_hand_example_and_invariants():
    # 10 steps, 20 % dense -> steps 0,1 dense; signal on the sparse steps 1,1,2,4,1,1,3,3 (mean 2)
    l1 = np.array([[9.0, 9.0, 1, 1, 2, 4, 1, 1, 3, 3]])
    got = oracle.budget_schedule(l1, rho=0.2, dense_fraction=0.2)
    np.testing.assert_allclose(got, [1, 1, 0.1, 0.1, 0.2, 0.4, 0.1, 0.1, 0.3, 0.3], rtol=1e-15)
    # the paper's budget identity: the sparse densities sum to rho * |T_sparse| (no cap active)
    g = rng(41)
    l1 = g.uniform(0.5, 1.5, size=(10, 50))
    r = oracle.budget_schedule(l1, 0.15)
    assert np.all(r[:10] == 1.0) and abs(r[10:].sum() - 0.15 * 40) < 1e-12
    # a flat signal gives the uniform budget; scaling the signal changes nothing; prompts are averaged
    np.testing.assert_allclose(oracle.budget_schedule(np.full((3, 20), 7.0), 0.3)[4:], 0.3, rtol=1e-15)
    np.testing.assert_allclose(oracle.budget_schedule(123.0 * l1, 0.15), r, rtol=1e-12)
    np.testing.assert_allclose(oracle.budget_schedule(l1.mean(axis=0, keepdims=True), 0.15), r, rtol=1e-12)
    # the cap: a spike cannot ask for more than every block
    spike = np.ones((1, 10)); spike[0, 5] = 100.0
    assert oracle.budget_schedule(spike, 0.5, dense_fraction=0.0).max() == 1.0


def test_l1_distance_closed_forms():
    g = rng(42)
    a = g.standard_normal(1001)
    assert oracle.l1_distance(a, a) == 0.0
    assert abs(oracle.l1_distance(a, a + 0.25) - 0.25) < 1e-15
    assert abs(oracle.l1_distance([1, -2, 3, 0], [0, 0, 0, 4]) - (1 + 2 + 3 + 4) / 4) < 1e-15
    b, c = g.standard_normal(1001), g.standard_normal(1001)
    assert oracle.l1_distance(a, b) == oracle.l1_distance(b, a)
    assert oracle.l1_distance(a, c) <= oracle.l1_distance(a, b) + oracle.l1_distance(b, c) + 1e-15

# ---- Gumbel variant of the routing bias ----------------------------------------------------------------------

def test_numpy_philox_agrees_with_the_c_routine_and_the_published_vectors():
    rng = np.random.default_rng(3)
    for _ in range(50):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64)
        got = [int(x) for x in oracle._philox4x32_10_np(*ctr, *key)]
        assert got == [int(x) for x in oracle.philox4x32_10(ctr.astype(np.uint32), key.astype(np.uint32))]
    # Random123's known-answer vector for the all-ones counter and key
    ones = 0xFFFFFFFF
    assert [int(x) for x in oracle._philox4x32_10_np(ones, ones, ones, ones, ones, ones)] == \
        [0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD]


def test_gumbel_routing_uses_the_same_philox_word_as_the_uniform_bias():
    """route() with zero scores and amplitude 1 returns w = ((int32)x >> 8) 2^-23; route_gumbel's u is built from
    x >> 9 of the same word, so floor((w 2^23 mod 2^24) / 2) must be u 2^23 - 0.5"""
    s = np.zeros((2, 9, 9), np.float32)
    _, w = oracle.route(s, 1, 0xABCDEF0123, 1.0, return_noisy=True)
    _, r = oracle.route_gumbel(s, 1, 0xABCDEF0123, 1.0, return_noisy=True)
    top24 = np.mod(np.round(w.astype(np.float64) * 2**23).astype(np.int64), 2**24)
    u = np.exp(-np.exp(-r))
    np.testing.assert_allclose(u * 2**23 - 0.5, top24 // 2, atol=1e-6)
    assert (u > 0).all() and (u < 1).all()


def test_gumbel_zero_temperature_is_deterministic_topk():
    rng = np.random.default_rng(5)
    s = rng.standard_normal((2, 17, 17)).astype(np.float32)
    np.testing.assert_array_equal(oracle.route_gumbel(s, 5, 99, 0.0), oracle.route(s, 5, 99, 0.0))


def test_gumbel_top1_samples_the_softmax_and_top2_the_plackett_luce_law():
    """Gumbel-max: argmax_j (s_j + tau g_j) ~ softmax(s / tau); the top-k set is a sample without replacement"""
    logits = np.array([0.3, -0.4, 1.1, 0.0])
    tau = 0.7
    BH = 6000
    s = np.broadcast_to(logits.astype(np.float32), (BH, 4, 4)).copy()
    p = np.exp(logits.astype(np.float32).astype(np.float64) / tau)
    p /= p.sum()
    n = BH * 4
    top1 = oracle.route_gumbel(s, 1, 2024, tau).reshape(-1)
    freq = np.bincount(top1, minlength=4) / n
    assert np.abs(freq - p).max() < 4.5 * np.sqrt(0.25 / n)
    top2 = oracle.route_gumbel(s, 2, 2025, tau).reshape(-1, 2)
    for a in range(4):
        for b in range(a + 1, 4):
            want = p[a] * p[b] / (1 - p[a]) + p[b] * p[a] / (1 - p[b])
            got = np.mean((top2[:, 0] == a) & (top2[:, 1] == b))
            assert abs(got - want) < 4.5 * np.sqrt(0.25 / n), (a, b, got, want)


def test_gumbel_variates_have_the_textbook_moments():
    s = np.zeros((4, 64, 64), np.float32)
    _, g = oracle.route_gumbel(s, 1, 7, 1.0, return_noisy=True)
    n = g.size
    assert abs(g.mean() - 0.5772156649) < 5 * np.sqrt(np.pi**2 / 6 / n)
    assert abs(g.var() - np.pi**2 / 6) < 0.1
