"""Pins of the CPU oracle against things other than itself.

The paper prints no score, index or merged value for the reduction path, so the
pins are: closed forms worked out by hand from Eq. 1-5, invariants, special
cases that reduce to a textbook result, brute force in pure Python on tiny
inputs, and an independent numpy evaluation as a third opinion.  Each pin is
chosen so that one plausible mistake (dropped term, wrong sign or index,
transposed operand, wrong tie rule) fails it.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import vscan_oracle as vo

LN = math.log


# ----------------------------------------------------------------------------
# Scoring, Eq. 1-2 ([CLS] row)
# ----------------------------------------------------------------------------
def _cls_case(n_patch, heads=1, dh=2):
    """q_CLS = [1, 0]; k_j = [ln(j+1), 7] for patch j=0..n-1, CLS key = [ln 4, -3]:
    with scale 1 the logits are ln(j+1), so softmax_j = (j+1) / sum."""
    S = n_patch + 1
    q = np.zeros((1, 1, heads, S, dh), np.float32)
    k = np.zeros((1, 1, heads, S, dh), np.float32)
    q[..., 0, 0] = 1.0
    q[..., 1:, :] = 5.0           # other query rows must not matter in [CLS] mode
    k[..., 0, :] = [LN(4.0), -3.0]
    for j in range(n_patch):
        k[..., 1 + j, :] = [LN(j + 1.0), 7.0]
    return q, k


def test_cls_scores_closed_form_visual_domain():
    q, k = _cls_case(3)
    s = vo.encoder_scores(q, k, has_cls=1, mode=0, domain=0, scale=1.0)
    np.testing.assert_allclose(s[0, 0], [1 / 6, 2 / 6, 3 / 6], rtol=1e-6)


def test_cls_scores_closed_form_all_keys_domain():
    # the CLS key joins the softmax (logit ln 4) and its column is dropped
    q, k = _cls_case(3)
    s = vo.encoder_scores(q, k, has_cls=1, mode=0, domain=1, scale=1.0)
    np.testing.assert_allclose(s[0, 0], [1 / 10, 2 / 10, 3 / 10], rtol=1e-6)


def test_cls_scores_scale_is_applied_to_logits():
    q, k = _cls_case(3)
    s = vo.encoder_scores(q, k, has_cls=1, mode=0, domain=0, scale=2.0)
    np.testing.assert_allclose(s[0, 0], [1 / 14, 4 / 14, 9 / 14], rtol=1e-6)


def test_cls_scores_head_mean():
    # head 0: p = (1,2,3)/6; head 1 has q = 0 -> uniform 1/3; Eq. 2 averages them
    q, k = _cls_case(3, heads=2)
    q[0, 0, 1, 0, :] = 0.0
    s = vo.encoder_scores(q, k, has_cls=1, mode=0, domain=0, scale=1.0)
    want = 0.5 * (np.array([1, 2, 3]) / 6 + 1 / 3)
    np.testing.assert_allclose(s[0, 0], want, rtol=1e-6)


def test_cls_scores_default_scale_is_inverse_sqrt_head_dim():
    # dh = 4, scale 1/2: logits ln(j+1)/2 -> p ~ sqrt(j+1)
    S = 4
    q = np.zeros((1, 1, 1, S, 4), np.float32)
    k = np.zeros((1, 1, 1, S, 4), np.float32)
    q[0, 0, 0, 0, 2] = 1.0
    for j in range(3):
        k[0, 0, 0, 1 + j, 2] = LN(j + 1.0)
    s = vo.encoder_scores(q, k, has_cls=1, mode=0)
    w = np.sqrt([1.0, 2.0, 3.0])
    np.testing.assert_allclose(s[0, 0], w / w.sum(), rtol=1e-6)


def test_scores_sum_to_one_and_uniform_for_zero_query():
    rng = np.random.default_rng(3)
    q = rng.normal(size=(2, 3, 4, 10, 8)).astype(np.float32)
    k = rng.normal(size=(2, 3, 4, 10, 8)).astype(np.float32)
    for mode, has_cls in ((0, 1), (1, 1), (1, 0)):
        s = vo.encoder_scores(q, k, has_cls=has_cls, mode=mode, domain=0)
        np.testing.assert_allclose(s.sum(-1), 1.0, rtol=1e-12)
        s0 = vo.encoder_scores(np.zeros_like(q), k, has_cls=has_cls, mode=mode, domain=0)
        np.testing.assert_allclose(s0, 1.0 / s0.shape[-1], rtol=1e-12)
    # with the CLS key in the domain the patch scores sum to less than one
    s = vo.encoder_scores(q, k, has_cls=1, mode=0, domain=1)
    assert np.all(s.sum(-1) < 1.0)


def _numpy_softmax(z):
    z = z - z.max(-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(-1, keepdims=True)


def test_scores_against_numpy_third_opinion():
    rng = np.random.default_rng(11)
    B, C, H, S, dh = 2, 2, 3, 9, 5
    q = rng.normal(size=(B, C, H, S, dh)).astype(np.float32)
    k = rng.normal(size=(B, C, H, S, dh)).astype(np.float32)
    scale = 1 / math.sqrt(dh)
    z = np.einsum("bchid,bchjd->bchij", q.astype(np.float64), k.astype(np.float64)) * scale
    # [CLS] row, visual keys only / all keys
    want = _numpy_softmax(z[..., 0, 1:]).mean(2)
    np.testing.assert_allclose(vo.encoder_scores(q, k, 1, 0, 0), want, rtol=1e-10)
    want = _numpy_softmax(z[..., 0, :])[..., 1:].mean(2)
    np.testing.assert_allclose(vo.encoder_scores(q, k, 1, 0, 1), want, rtol=1e-10)
    # mean attention received: patch queries, patch keys; column mean incl. diagonal
    want = _numpy_softmax(z[..., 1:, 1:]).mean(3).mean(2)
    np.testing.assert_allclose(vo.encoder_scores(q, k, 1, 1, 0), want, rtol=1e-10)
    want = _numpy_softmax(z[..., 1:, :])[..., 1:].mean(3).mean(2)
    np.testing.assert_allclose(vo.encoder_scores(q, k, 1, 1, 1), want, rtol=1e-10)
    want = _numpy_softmax(z).mean(3).mean(2)
    np.testing.assert_allclose(vo.encoder_scores(q, k, 0, 1, 0), want, rtol=1e-10)


def test_mean_received_closed_form():
    # q_i = [a_i, 0], a = (0, 1, 2); k_j = [ln(j+1), 9]; scale 1
    # row i: p_ij = (j+1)^a_i / sum_j (j+1)^a_i  ->  rows (1,1,1)/3, (1,2,3)/6, (1,4,9)/14
    q = np.zeros((1, 1, 1, 3, 2), np.float32)
    k = np.zeros((1, 1, 1, 3, 2), np.float32)
    for i, a in enumerate((0.0, 1.0, 2.0)):
        q[0, 0, 0, i] = [a, 0.0]
    for j in range(3):
        k[0, 0, 0, j] = [LN(j + 1.0), 9.0]
    s = vo.encoder_scores(q, k, has_cls=0, mode=1, domain=0, scale=1.0)
    want = (np.array([1, 1, 1]) / 3 + np.array([1, 2, 3]) / 6 + np.array([1, 4, 9]) / 14) / 3
    np.testing.assert_allclose(s[0, 0], want, rtol=1e-6)


# ----------------------------------------------------------------------------
# Selection, Eq. 2-3 and the footnote
# ----------------------------------------------------------------------------
def _py_select(sl, sg, gh, gw, wr, wc, kl, kg):
    """Pure-Python statement of the rule, using sorted()."""
    N, W = gh * gw, wr * wc
    kw = kl // W
    taken = set()
    for wy, wx in itertools.product(range(wr), range(wc)):
        toks = [r * gw + c for r in range(gh) for c in range(gw)
                if (r * wr) // gh == wy and (c * wc) // gw == wx]
        toks.sort(key=lambda i: (-sl[i], i))
        taken.update(toks[:kw])
    rest = sorted((i for i in range(N) if i not in taken), key=lambda i: (-sg[i], i))
    taken.update(rest[:kg + kl - kw * W])
    return sorted(taken)


def test_select_all_ties_closed_form():
    # 4x4 grid, 2x2 windows of 2x2 tokens, one local token per window, two global.
    # window firsts: 0, 2, 8, 10; then the two lowest remaining indices: 1, 3.
    s = np.full((1, 1, 16), 1 / 16)
    kept = vo.select(s, s, 4, 4, 2, 2, 4, 2)
    assert kept.tolist() == [[0, 1, 2, 3, 8, 10]]


def test_select_local_has_priority_over_global():
    # tokens 0 and 1 (same window) hold the two best scores.  Local takes the best
    # of each window (0, 2, 8, 10 with the scores below); the single global token is
    # then the best remaining one, token 1, not a repeat of token 0.
    s = np.arange(16, dtype=np.float64)[::-1].copy() / 100.0
    kept = vo.select(s.reshape(1, 1, 16), s.reshape(1, 1, 16), 4, 4, 2, 2, 4, 1)
    assert kept.tolist() == [[0, 1, 2, 8, 10]]


def test_select_uses_local_scores_in_windows_and_global_scores_after():
    sg = np.arange(16, dtype=np.float64).reshape(1, 1, 16)          # favours high indices
    sl = np.arange(16, dtype=np.float64)[::-1].copy().reshape(1, 1, 16)  # favours low indices
    kept = vo.select(sl, sg, 4, 4, 2, 2, 4, 2)
    # local by sl: 0, 2, 8, 10; global by sg among the rest: 15, 14
    assert kept.tolist() == [[0, 2, 8, 10, 14, 15]]


def test_select_remainder_of_local_budget_goes_to_global():
    s = np.arange(16, dtype=np.float64).reshape(1, 1, 16)
    # kl = 5 over 4 windows: one per window (5, 7, 13, 15), remainder 1 joins kg = 1:
    # global takes the best two of the rest: 14, 12
    kept = vo.select(s, s, 4, 4, 2, 2, 5, 1)
    assert kept.tolist() == [[5, 7, 12, 13, 14, 15]]


@pytest.mark.parametrize("gh,gw,wr,wc,kl,kg", [(4, 4, 2, 2, 4, 3), (6, 6, 3, 3, 9, 5),
                                              (5, 7, 2, 3, 6, 4), (8, 8, 1, 1, 7, 9),
                                              (6, 6, 2, 2, 0, 10), (6, 6, 2, 2, 12, 0)])
def test_select_brute_force_with_ties(gh, gw, wr, wc, kl, kg):
    rng = np.random.default_rng(gh * 100 + gw)
    B, C, N = 3, 2, gh * gw
    # few distinct values -> many exact ties
    sg = rng.integers(0, 5, size=(B, C, N)).astype(np.float64) / 8
    sl = rng.integers(0, 5, size=(B, C, N)).astype(np.float64) / 8
    kept = vo.select(sl, sg, gh, gw, wr, wc, kl, kg)
    assert kept.shape == (B, C * (kl + kg))
    for b in range(B):
        want = []
        for c in range(C):
            want += [c * N + i for i in _py_select(sl[b, c], sg[b, c], gh, gw, wr, wc, kl, kg)]
        assert kept[b].tolist() == want
        assert len(set(want)) == len(want)


def test_select_windows_of_a_grid_that_does_not_divide():
    """5 x 7 grid, 2 x 3 windows, written out by hand from the partition rule (token (r, c) lies
    in window (floor(2 r / 5), floor(3 c / 7))): rows 0-2 | 3-4, columns 0-2 | 3-4 | 5-6, i.e.

        0 0 0 1 1 2 2
        0 0 0 1 1 2 2
        0 0 0 1 1 2 2
        3 3 3 4 4 5 5
        3 3 3 4 4 5 5

    Base scores grow with the token index, so a window's best tokens are its last ones unless a
    planted score says otherwise.  The planted pairs straddle every boundary of the partition:
    (2,0) | (3,0) across the row boundary, (0,2) | (0,3) and (0,4) | (0,5) across the column
    boundaries.  Two per window:
      window 0: (2,0) = 14 and (0,2) = 2      window 1: (0,3) = 3 and (0,4) = 4
      window 2: (0,5) = 5 and its last token (2,6) = 20
      window 3: (3,0) = 21 and its last token (4,2) = 30
      window 4: last two tokens (4,3) = 31, (4,4) = 32      window 5: (4,5) = 33, (4,6) = 34
    and one global token, the best of the rest: (4,1) = 29.
    Any other partition (even splits 2 + 3 rows or 2 + 2 + 3 columns, the window counts of
    the two axes swapped) puts two of the planted scores into one window or separates a pair
    the wrong way and picks a different set."""
    s = 0.001 * np.arange(35, dtype=np.float64)
    for (r, c), v in {(2, 0): 100.0, (3, 0): 99.0, (0, 2): 98.0, (0, 3): 97.0, (0, 4): 96.0,
                      (0, 5): 95.0}.items():
        s[r * 7 + c] = v
    s = s.reshape(1, 1, 35)
    kept = vo.select(s, s, 5, 7, 2, 3, 12, 0)
    assert kept.tolist() == [[2, 3, 4, 5, 14, 20, 21, 30, 31, 32, 33, 34]]
    kept = vo.select(s, s, 5, 7, 2, 3, 12, 1)
    assert kept.tolist() == [[2, 3, 4, 5, 14, 20, 21, 29, 30, 31, 32, 33, 34]]
    # the transposed case (7 x 5 grid, 3 x 2 windows), planted at the mirrored positions
    t = 0.001 * np.arange(35, dtype=np.float64)
    for (r, c), v in {(0, 2): 100.0, (0, 3): 99.0, (2, 0): 98.0, (3, 0): 97.0, (4, 0): 96.0,
                      (5, 0): 95.0}.items():
        t[r * 5 + c] = v
    # rows 0-2 | 3-4 | 5-6, columns 0-2 | 3-4:
    #   window 0 (rows 0-2, cols 0-2): (0,2) = 2, (2,0) = 10     window 1 (rows 0-2, cols 3-4): (0,3) = 3, last (2,4) = 14
    #   window 2 (rows 3-4, cols 0-2): (3,0) = 15, (4,0) = 20    window 3 (rows 3-4, cols 3-4): (4,3) = 23, (4,4) = 24
    #   window 4 (rows 5-6, cols 0-2): (5,0) = 25, last (6,2) = 32   window 5 (rows 5-6, cols 3-4): (6,3) = 33, (6,4) = 34
    t = t.reshape(1, 1, 35)
    kept = vo.select(t, t, 7, 5, 3, 2, 12, 0)
    assert kept.tolist() == [[2, 3, 10, 14, 15, 20, 23, 24, 25, 32, 33, 34]]


def test_select_rejects_budget_larger_than_window():
    s = np.zeros((1, 1, 16))
    with pytest.raises(ValueError):
        vo.select(s, s, 4, 4, 2, 2, 20, 0)      # 5 per 4-token window


# ----------------------------------------------------------------------------
# Assignment and merging, "Token Merging" paragraph and Eq. 4
# ----------------------------------------------------------------------------
def test_assign_uses_cosine_not_dot_product():
    # u = (1, 0).  slot 0 = (10, 10): dot 10, cos 0.707.  slot 1 = (0.9, 0.1): dot 0.9,
    # cos 0.994.  Cosine similarity picks slot 1.
    x = np.array([[[10, 10], [0.9, 0.1], [1, 0]]], np.float32)
    a = vo.assign(x, np.array([[0, 1]], np.int32))
    assert a.tolist() == [[0, 1, 1]]


def test_assign_is_invariant_to_positive_rescaling():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(2, 40, 6)).astype(np.float32)
    kept = np.sort(rng.permutation(40)[:7]).astype(np.int32)[None].repeat(2, 0)
    a = vo.assign(x, kept)
    x2 = x * rng.uniform(0.5, 4.0, size=(2, 40, 1)).astype(np.float32)
    assert np.array_equal(vo.assign(x2, kept), a)


def test_assign_ties_go_to_lowest_slot_and_duplicates_match():
    # slots 0 and 2 are exact duplicates; token 3 equals them -> slot 0.
    # token 4 is a positive multiple of slot 1 -> cos = 1 -> slot 1.
    x = np.array([[[1, 2, 3], [-1, 0.5, 2], [1, 2, 3], [1, 2, 3], [-2, 1, 4]]], np.float32)
    a = vo.assign(x, np.array([[0, 1, 2]], np.int32))
    assert a.tolist() == [[0, 1, 2, 0, 1]]


def test_assign_brute_force():
    rng = np.random.default_rng(17)
    B, T, D, K = 2, 30, 5, 6
    x = rng.normal(size=(B, T, D)).astype(np.float32)
    kept = np.stack([np.sort(rng.permutation(T)[:K]) for _ in range(B)]).astype(np.int32)
    a = vo.assign(x, kept)
    xd = x.astype(np.float64)
    for b in range(B):
        for u in range(T):
            if u in kept[b]:
                assert a[b, u] == list(kept[b]).index(u)
                continue
            best, best_c = None, None
            for s in range(K):
                xs = xd[b, kept[b, s]]
                c = float(xd[b, u] @ xs) / (math.sqrt(float(xd[b, u] @ xd[b, u])) *
                                             math.sqrt(float(xs @ xs)))
                if best is None or c > best_c:
                    best, best_c = s, c
            assert a[b, u] == best
    pairs_u = np.array([0 * T + 3, 1 * T + 4])
    pairs_s = np.array([0 * T + kept[0, 2], 1 * T + kept[1, 0]])
    got = vo.cos_pairs(x.reshape(-1, D), pairs_u, pairs_s)
    for g, u, s in zip(got, pairs_u, pairs_s):
        a_, b_ = xd.reshape(-1, D)[u], xd.reshape(-1, D)[s]
        assert abs(g - a_ @ b_ / math.sqrt((a_ @ a_) * (b_ @ b_))) < 1e-14


def test_merge_hand_example():
    # Eq. 4 with D = 1: slot 0 = token 0 with members {1, 2}; slot 1 = token 3 alone
    x = np.array([[[1.0], [2.0], [3.0], [10.0]]], np.float32)
    m, cnt = vo.merge(x, np.array([[0, 3]], np.int32), np.array([[0, 0, 0, 1]], np.int32))
    assert m[0, :, 0].tolist() == [2.0, 10.0]
    assert cnt.tolist() == [[3, 1]]


def test_merge_invariants():
    rng = np.random.default_rng(23)
    B, T, D, K = 3, 50, 8, 9
    x = rng.normal(size=(B, T, D)).astype(np.float32)
    kept = np.stack([np.sort(rng.permutation(T)[:K]) for _ in range(B)]).astype(np.int32)
    a = vo.assign(x, kept)
    m, cnt = vo.merge(x, kept, a)
    # every token is in exactly one group; group sizes add up to T
    assert np.all(cnt.sum(1) == T)
    assert np.array_equal(cnt, np.stack([np.bincount(a[b], minlength=K) for b in range(B)]))
    # merged means preserve the feature sum
    np.testing.assert_allclose((m * cnt[..., None]).sum(1), x.astype(np.float64).sum(1),
                               rtol=1e-12, atol=1e-12)
    # keep everything -> identity
    all_idx = np.arange(T, dtype=np.int32)[None].repeat(B, 0)
    a_id = vo.assign(x, all_idx)
    assert np.array_equal(a_id, all_idx)
    m_id, _ = vo.merge(x, all_idx, a_id)
    assert np.array_equal(m_id, x.astype(np.float64))
    # identical features everywhere -> merged equals that feature, all in slot 0
    xc = np.tile(x[:, :1], (1, T, 1))
    a_c = vo.assign(xc, kept)
    for b in range(B):
        dropped = np.setdiff1d(np.arange(T), kept[b])
        assert np.all(a_c[b, dropped] == 0)
    m_c, _ = vo.merge(xc, kept, a_c)
    np.testing.assert_allclose(m_c, np.tile(x[:, :1], (1, K, 1)).astype(np.float64), rtol=1e-15)


# ----------------------------------------------------------------------------
# Stage 2, Eq. 5 and the KV-cache remark
# ----------------------------------------------------------------------------
def test_llm_scores_closed_form_gqa_and_query_mean():
    # Hq = 4, Hkv = 2, Tq = 1, V = 3.  kv head 0 keys give logits ln(j+1); kv head 1 keys
    # give ln((j+1)^2).  Query heads 0,1 -> kv 0; heads 2,3 -> kv 1.  Heads 1 and 3 have
    # q = 0 (uniform).  Mean over the four heads.
    S, vs, V = 6, 1, 3
    q = np.zeros((1, 4, 1, 2), np.float32)
    k = np.full((1, 2, S, 2), 50.0, np.float32)       # non-visual keys would dominate
    q[0, 0, 0] = [1, 0]
    q[0, 2, 0] = [1, 0]
    for j in range(V):
        k[0, 0, vs + j] = [LN(j + 1.0), 3]
        k[0, 1, vs + j] = [2 * LN(j + 1.0), -3]
    s = vo.llm_scores(q, k, vs, V, domain=0, scale=1.0)
    want = (np.array([1, 2, 3]) / 6 + np.array([1, 4, 9]) / 14 + 2 / 3) / 4
    np.testing.assert_allclose(s[0], want, rtol=1e-6)
    np.testing.assert_allclose(s.sum(), 1.0, rtol=1e-12)


def test_llm_scores_causal_domain_lengths():
    # q = 0 -> uniform over the causal row.  S = 6, Tq = 2: the two queries sit at
    # positions 4 and 5 and see 5 and 6 keys; each visual token gets (1/5 + 1/6)/2.
    q = np.zeros((1, 2, 2, 3), np.float32)
    k = np.random.default_rng(1).normal(size=(1, 1, 6, 3)).astype(np.float32)
    s = vo.llm_scores(q, k, 1, 3, domain=1)
    np.testing.assert_allclose(s[0], [11 / 60] * 3, rtol=1e-12)


def test_llm_scores_against_numpy_third_opinion():
    rng = np.random.default_rng(29)
    B, Hq, Hkv, Tq, S, dh, vs, V = 2, 6, 2, 3, 20, 4, 5, 9
    q = rng.normal(size=(B, Hq, Tq, dh)).astype(np.float32)
    k = rng.normal(size=(B, Hkv, S, dh)).astype(np.float32)
    kk = np.repeat(k.astype(np.float64), Hq // Hkv, axis=1)
    z = np.einsum("bhtd,bhjd->bhtj", q.astype(np.float64), kk) / math.sqrt(dh)
    want = _numpy_softmax(z[..., vs:vs + V]).mean((1, 2))
    np.testing.assert_allclose(vo.llm_scores(q, k, vs, V, 0), want, rtol=1e-10)
    want = np.zeros((B, V))
    for t in range(Tq):
        n = S - Tq + t + 1
        want += _numpy_softmax(z[:, :, t, :n])[..., vs:vs + V].mean(1) / Tq
    np.testing.assert_allclose(vo.llm_scores(q, k, vs, V, 1), want, rtol=1e-10)


def test_topk_ties_and_brute_force():
    assert vo.topk(np.full((1, 7), 0.25), 3).tolist() == [[0, 1, 2]]
    rng = np.random.default_rng(31)
    s = rng.integers(0, 4, size=(5, 33)).astype(np.float64)
    for keep in (0, 1, 10, 33):
        kept = vo.topk(s, keep)
        for b in range(5):
            want = sorted(sorted(range(33), key=lambda i: (-s[b, i], i))[:keep])
            assert kept[b].tolist() == want


def test_compact_hand_example_and_identity():
    # rows are labelled by their position; S = 8, prefix 2, V = 4, text 2, keep {1, 3}
    B, G, S, W = 2, 3, 8, 2
    t = np.arange(B * G * S * W, dtype=np.float32).reshape(B, G, S, W)
    kept = np.array([[1, 3], [0, 2]], np.int32)
    out = vo.compact(t, kept, 2, 4)
    assert out.shape == (B, G, 6, W)
    assert np.array_equal(out[0], t[0][:, [0, 1, 3, 5, 6, 7]])
    assert np.array_equal(out[1], t[1][:, [0, 1, 2, 4, 6, 7]])
    ident = vo.compact(t, np.arange(4, dtype=np.int32)[None].repeat(B, 0), 2, 4)
    assert np.array_equal(ident, t)
    h = np.arange(B * S * W, dtype=np.float32).reshape(B, S, W)
    assert np.array_equal(vo.compact(h, kept, 2, 4)[0], h[0][[0, 1, 3, 5, 6, 7]])


# ----------------------------------------------------------------------------
# End-to-end invariants on a realistic small workload
# ----------------------------------------------------------------------------
def test_encoder_end_to_end_invariants():
    from paper_2505_22654_amd import workloads as wl
    shape = wl.EncoderShape(dtype=wl.BF16, batch=2, n_segments=2, grid_h=12, grid_w=12,
                            has_cls=1, score_mode=0, heads=4, head_dim=16, feat_dim=64,
                            win_rows=3, win_cols=3, keep_global=10, keep_local=9)
    inp = wl.encoder_inputs(shape, seed=99)
    r = vo.encoder_reduce(shape, inp["q"], inp["k"], inp["x"])
    T, K, N = shape.tokens_per_image, shape.keep, shape.n_tokens
    for b in range(shape.batch):
        kept = r["kept"][b]
        assert np.all(np.diff(kept) > 0) and kept.min() >= 0 and kept.max() < T
        # per-segment budget
        assert np.array_equal(np.bincount(kept // N, minlength=2), [19, 19])
        dropped = np.setdiff1d(np.arange(T), kept)
        assert len(dropped) + len(kept) == T
        assert np.array_equal(r["assign"][b, kept], np.arange(K))
        assert r["assign"][b].min() >= 0 and r["assign"][b].max() < K
    np.testing.assert_allclose((r["merged"] * r["counts"][..., None]).sum(1),
                               inp["x"].astype(np.float64).sum(1), rtol=1e-10, atol=1e-9)
    # keep == N on one segment is the identity
    shape_id = wl.EncoderShape(dtype=wl.F32, batch=1, n_segments=1, grid_h=4, grid_w=4,
                               has_cls=1, score_mode=0, heads=2, head_dim=8, feat_dim=16,
                               win_rows=2, win_cols=2, keep_global=8, keep_local=8)
    inp = wl.encoder_inputs(shape_id, seed=5)
    r = vo.encoder_reduce(shape_id, inp["q"], inp["k"], inp["x"])
    assert r["kept"].tolist() == [list(range(16))]
    assert np.array_equal(r["merged"][0], inp["x"][0].astype(np.float64))


def test_llm_end_to_end_invariants():
    from paper_2505_22654_amd import workloads as wl
    shape = wl.LlmShape(dtype=wl.BF16, batch=2, prefix=3, vis_len=20, text=5, n_query=2,
                        q_heads=4, kv_heads=2, head_dim=8, hidden=16, keep=7)
    inp = wl.llm_inputs(shape, seed=7)
    r = vo.llm_prune(shape, **inp)
    S, So = shape.seq_len, shape.seq_out
    assert r["k"].shape == (2, 2, So, 8) and r["hidden"].shape == (2, So, 16)
    for b in range(2):
        rows = list(range(3)) + [3 + int(j) for j in r["kept"][b]] + list(range(23, S))
        assert np.array_equal(r["hidden"][b], inp["hidden"][b][rows])
        assert np.array_equal(r["v"][b], inp["v"][b][:, rows])
    # uniform keys -> all scores tie -> the first `keep` visual tokens stay
    inp["k"][:] = 1.0
    r = vo.llm_prune(shape, **inp)
    assert r["kept"].tolist() == [list(range(7))] * 2


# ---- Eq. 5 written out from the hidden states -------------------------------------------------

def test_scores_from_hidden_agree_with_projected_form():
    """Projecting first (in fp64, handed to the C oracle as fp32) and scoring from the hidden
    states directly are the same definition; they agree to fp32 rounding of the projections."""
    from paper_2505_22654_amd import workloads as wl
    shape = wl.LlmShape(dtype=wl.BF16, batch=2, prefix=3, vis_len=40, text=6, n_query=2,
                        q_heads=4, kv_heads=2, head_dim=16, hidden=48, keep=10)
    x = wl.llm_inputs(shape, 77)["hidden"]
    w = wl.llm_weights(shape, 77)
    got = vo.llm_scores_from_hidden(x, w["w_q"], w["w_k"], shape.vis_start, shape.vis_len,
                                    shape.n_query, shape.q_heads, shape.kv_heads, shape.head_dim)
    x64 = x.astype(np.float64)
    B, S, _ = x.shape
    q = (x64[:, S - 2:] @ w["w_q"].astype(np.float64).T).reshape(B, 2, 4, 16).transpose(0, 2, 1, 3)
    k = (x64 @ w["w_k"].astype(np.float64).T).reshape(B, S, 2, 16).transpose(0, 2, 1, 3)
    want = vo.llm_scores(q.astype(np.float32), k.astype(np.float32), shape.vis_start,
                         shape.vis_len)
    np.testing.assert_allclose(got, want, rtol=5e-6)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-12)
    # the all-keys reading: causal rows, one key fewer for the earlier of the two queries
    got = vo.llm_scores_from_hidden(x, w["w_q"], w["w_k"], shape.vis_start, shape.vis_len,
                                    shape.n_query, shape.q_heads, shape.kv_heads, shape.head_dim,
                                    domain=1)
    want = vo.llm_scores(q.astype(np.float32), k.astype(np.float32), shape.vis_start,
                         shape.vis_len, 1)
    np.testing.assert_allclose(got, want, rtol=5e-6)


def test_scores_from_hidden_closed_form():
    """Identity projections on one head: the score of token j is softmax_j(x_last . x_j * scale);
    with x_j = a_j * e_0 and x_last = e_0 that is softmax(a * scale)."""
    V, Dh = 7, 4
    a = np.log(np.arange(1, V + 1))           # softmax(a) = (j+1) / sum
    x = np.zeros((1, V + 1, Dh))
    x[0, :V, 0] = a
    x[0, V, 0] = 1.0                            # the last token
    eye = np.eye(Dh)
    got = vo.llm_scores_from_hidden(x, eye, eye, 0, V, 1, 1, 1, Dh, scale=1.0)
    # all-keys domain: the last token's own key (logit 1) joins the denominator
    got_all = vo.llm_scores_from_hidden(x, eye, eye, 0, V, 1, 1, 1, Dh, domain=1, scale=1.0)
    np.testing.assert_allclose(got_all[0], np.arange(1, V + 1) / (np.arange(1, V + 1).sum() + np.e),
                               rtol=1e-12)
    # two query positions, both e_0: the earlier one does not see the later one's key, so its
    # denominator lacks one e; the score is the mean of the two rows
    x3 = np.zeros((1, V + 2, Dh)); x3[0, :V, 0] = a; x3[0, V:, 0] = 1.0
    got2q = vo.llm_scores_from_hidden(x3, eye, eye, 0, V, 2, 1, 1, Dh, domain=1, scale=1.0)
    tot = np.arange(1, V + 1).sum()
    np.testing.assert_allclose(got2q[0], np.arange(1, V + 1) * 0.5 * (1 / (tot + np.e) + 1 / (tot + 2 * np.e)),
                               rtol=1e-12)
    np.testing.assert_allclose(got[0], np.arange(1, V + 1) / np.arange(1, V + 1).sum(), rtol=1e-12)
    # a transposed weight would contract the wrong axis: a non-symmetric W_K catches it
    wk = np.zeros((Dh, Dh)); wk[0, 1] = 1.0    # key feature 0 reads hidden feature 1
    x2 = np.zeros((1, V + 1, Dh)); x2[0, :V, 1] = a; x2[0, V, 0] = 1.0
    got2 = vo.llm_scores_from_hidden(x2, eye, wk, 0, V, 1, 1, 1, Dh, scale=1.0)
    np.testing.assert_allclose(got2[0], np.arange(1, V + 1) / np.arange(1, V + 1).sum(), rtol=1e-12)


def test_scores_from_hidden_gqa_and_queries():
    """Grouped heads read the kv head floor(h * Hkv / Hq); several query positions are averaged."""
    rng = np.random.default_rng(5)
    B, S, Dh, Hq, Hkv, dh, V, Tq = 1, 9, 6, 4, 2, 3, 5, 2
    x = rng.standard_normal((B, S, Dh)); wq = rng.standard_normal((Hq * dh, Dh)); wk = rng.standard_normal((Hkv * dh, Dh))
    got = vo.llm_scores_from_hidden(x, wq, wk, 1, V, Tq, Hq, Hkv, dh)
    want = np.zeros(V)
    for h in range(Hq):
        for t in range(Tq):
            qv = wq[h * dh:(h + 1) * dh] @ x[0, S - Tq + t]
            g = h // (Hq // Hkv)
            kv = x[0, 1:1 + V] @ wk[g * dh:(g + 1) * dh].T
            l = kv @ qv / np.sqrt(dh)
            e = np.exp(l - l.max()); want += e / e.sum()
    np.testing.assert_allclose(got[0], want / (Hq * Tq), rtol=1e-12)


# ---- Eq. 1-2 written out from the encoder's hidden states ------------------------------------

def test_encoder_scores_from_hidden_agree_with_projected_form():
    from paper_2505_22654_amd import workloads as wl
    shape = wl.EncoderShape(dtype=wl.BF16, batch=2, n_segments=2, grid_h=5, grid_w=4, has_cls=1,
                            score_mode=0, heads=3, head_dim=8, feat_dim=24, win_rows=1,
                            win_cols=1, keep_global=4, keep_local=0)
    inp = wl.encoder_hidden_inputs(shape, 31)
    x = inp["hidden"].astype(np.float64)
    B, C, S, D = x.shape
    q = (x @ inp["w_q"].astype(np.float64).T).reshape(B, C, S, 3, 8).transpose(0, 1, 3, 2, 4)
    k = (x @ inp["w_k"].astype(np.float64).T).reshape(B, C, S, 3, 8).transpose(0, 1, 3, 2, 4)
    for domain in (0, 1):
        got = vo.encoder_scores_from_hidden(inp["hidden"], inp["w_q"], inp["w_k"], 3, 8, domain)
        want = vo.encoder_scores(q.astype(np.float32), k.astype(np.float32), 1, 0, domain)
        np.testing.assert_allclose(got, want, rtol=5e-6)
    np.testing.assert_allclose(
        vo.encoder_scores_from_hidden(inp["hidden"], inp["w_q"], inp["w_k"], 3, 8, 0).sum(axis=2),
        1.0, rtol=1e-12)


def test_encoder_scores_from_hidden_closed_form():
    """One head, identity-like weights: the [CLS] row e_0 against patch rows a_j e_1 with a key
    weight that reads hidden feature 1 into key feature 0 (a transposed weight would give a
    uniform score instead)."""
    N, D = 6, 4
    a = np.log(np.arange(1, N + 1))
    x = np.zeros((1, 1, N + 1, D))
    x[0, 0, 0, 0] = 1.0
    x[0, 0, 1:, 1] = a
    wq = np.eye(D)
    wk = np.zeros((D, D)); wk[0, 1] = 1.0
    got = vo.encoder_scores_from_hidden(x, wq, wk, 1, D, 0, scale=1.0)
    np.testing.assert_allclose(got[0, 0], np.arange(1, N + 1) / np.arange(1, N + 1).sum(), rtol=1e-12)
    # all keys: the [CLS] key has logit 0 and adds exp(0) = 1 to the denominator
    got = vo.encoder_scores_from_hidden(x, wq, wk, 1, D, 1, scale=1.0)
    np.testing.assert_allclose(got[0, 0], np.arange(1, N + 1) / (np.arange(1, N + 1).sum() + 1.0),
                               rtol=1e-12)


# ---- mean attention received, written out from the encoder's hidden states -------------------

@pytest.mark.parametrize("has_cls", [0, 1])
def test_encoder_mean_scores_from_hidden_agree_with_projected_form(has_cls):
    """Projecting on the host and calling the C oracle's mean mode gives the same scores (two
    routes: numpy on hidden states, C loops on Q and K), with and without a [CLS] row, both key
    domains; every column sum of row-softmaxes adds up to 1 over the patch columns in domain 0."""
    from paper_2505_22654_amd import workloads as wl
    shape = wl.EncoderShape(dtype=wl.BF16, batch=2, n_segments=2, grid_h=5, grid_w=4, has_cls=has_cls,
                            score_mode=1, heads=3, head_dim=8, feat_dim=24, win_rows=1,
                            win_cols=1, keep_global=4, keep_local=0)
    inp = wl.encoder_hidden_inputs(shape, 37)
    x = inp["hidden"].astype(np.float64)
    B, C, S, D = x.shape
    q = (x @ inp["w_q"].astype(np.float64).T).reshape(B, C, S, 3, 8).transpose(0, 1, 3, 2, 4)
    k = (x @ inp["w_k"].astype(np.float64).T).reshape(B, C, S, 3, 8).transpose(0, 1, 3, 2, 4)
    for domain in ((0, 1) if has_cls else (0,)):
        got = vo.encoder_mean_scores_from_hidden(inp["hidden"], inp["w_q"], inp["w_k"], 3, 8, has_cls,
                                                 domain)
        want = vo.encoder_scores(q.astype(np.float32), k.astype(np.float32), has_cls, 1, domain)
        np.testing.assert_allclose(got, want, rtol=5e-6)
    s0 = vo.encoder_mean_scores_from_hidden(inp["hidden"], inp["w_q"], inp["w_k"], 3, 8, has_cls, 0)
    np.testing.assert_allclose(s0.sum(axis=2), 1.0, rtol=1e-12)


def test_encoder_mean_scores_from_hidden_closed_form():
    """One head; every query reads hidden feature 0 (all ones), every key hidden feature 1 (= a_j)
    into feature 0: all rows have logits a_j = ln(j+1), so every row-softmax - and their mean - is
    (j+1)/sum.  With a key weight transposed the logits would not depend on j.  Then a [CLS] row
    with key logit 0 in the all-keys domain adds 1 to every denominator."""
    N, D = 5, 4
    a = np.log(np.arange(1, N + 1))
    x = np.zeros((1, 1, N, D))
    x[0, 0, :, 0] = 1.0
    x[0, 0, :, 1] = a
    wq = np.zeros((D, D)); wq[0, 0] = 1.0
    wk = np.zeros((D, D)); wk[0, 1] = 1.0
    want = np.arange(1, N + 1) / np.arange(1, N + 1).sum()
    got = vo.encoder_mean_scores_from_hidden(x, wq, wk, 1, D, 0, 0, scale=1.0)
    np.testing.assert_allclose(got[0, 0], want, rtol=1e-12)
    xc = np.concatenate([np.zeros((1, 1, 1, D)), x], axis=2)   # [CLS] row of zeros: key logit 0
    got = vo.encoder_mean_scores_from_hidden(xc, wq, wk, 1, D, 1, 1, scale=1.0)
    np.testing.assert_allclose(got[0, 0], np.arange(1, N + 1) / (np.arange(1, N + 1).sum() + 1.0),
                               rtol=1e-12)
    # patch-only domain with the same [CLS] row present: it takes no part
    got = vo.encoder_mean_scores_from_hidden(xc, wq, wk, 1, D, 1, 0, scale=1.0)
    np.testing.assert_allclose(got[0, 0], want, rtol=1e-12)


def test_encoder_mean_scores_from_hidden_query_dependence():
    """Two queries with different logit gains: the mean of two different softmax rows, by hand."""
    D = 2
    x = np.array([[[[1.0, 0.0], [2.0, 1.0]]]])          # two patch tokens
    wq = np.array([[1.0, 0.0], [0.0, 0.0]])              # q_i = (x_i0, 0)
    wk = np.array([[0.0, 1.0], [0.0, 0.0]])              # k_j = (x_j1, 0)
    # logits l_ij = x_i0 * x_j1: row 0 = (0, 1), row 1 = (0, 2)
    r0 = np.exp([0.0, 1.0]) / np.exp([0.0, 1.0]).sum()
    r1 = np.exp([0.0, 2.0]) / np.exp([0.0, 2.0]).sum()
    got = vo.encoder_mean_scores_from_hidden(x, wq, wk, 1, D, 0, 0, scale=1.0)
    np.testing.assert_allclose(got[0, 0], (r0 + r1) / 2, rtol=1e-12)
