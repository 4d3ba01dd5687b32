"""Pins for the CPU oracle (no GPU needed).

Each test fixes the oracle against something other than itself: the brute-force
definition of eviction error (Sec. 3.1), Theorems 3.1 / 3.2, the H2O sum theorem
(App. "H2O scores"), closed forms that follow from the score formula (Sec. 3.1-3.3),
or a library routine that computes the same thing in a special case.
"""
import itertools

import numpy as np
import pytest
import scipy.ndimage
import scipy.special
import torch

RNG = np.random.default_rng(1234)


def _weights(n):
    w = RNG.random(n) ** 3 + 1e-3
    return w / w.sum()


# ---- closed-form score == the definition (Theorem 3.2) ------------------------

@pytest.mark.parametrize("n,d", [(2, 3), (5, 4), (17, 8), (64, 16)])
def test_closed_form_equals_bruteforce_removal(oracle, n, d):
    w = _weights(n)
    v = RNG.standard_normal((n, d)) * np.exp(0.5 * RNG.standard_normal((n, 1)))
    c, w_out, o = oracle.caote_scores(w * 7.5, v)          # any positive scale of h
    e = oracle.bruteforce_eviction_error(w, v)
    np.testing.assert_allclose(w_out, w, rtol=1e-13)
    np.testing.assert_allclose(c, e, rtol=1e-10, atol=1e-14)
    # the brute force itself against an independent numpy evaluation of Eq. (eviction error)
    for j in (0, n - 1):
        keep = np.arange(n) != j
        o2 = (w[keep] / w[keep].sum()) @ v[keep]
        assert np.isclose(np.linalg.norm(w @ v - o2), e[j], rtol=1e-12)


@pytest.mark.parametrize("n,d", [(3, 4), (24, 8), (48, 32)])
def test_single_query_score_equals_literal_token_deletion(oracle, n, d):
    """Generation case (W = 1, one head): delete key/value j, redo the softmax."""
    q = RNG.standard_normal((1, d))
    k = RNG.standard_normal((n, d))
    v = RNG.standard_normal((n, d))
    scale = 1.0 / np.sqrt(d)
    e = oracle.bruteforce_delete_token(q[0], k, v, scale)
    for wic in (0, 1):   # with W = 1 the causal window mask hides nothing
        c, h, a = oracle.score_one(q, k, v, None, 1, 1, scale, wic, oracle.BASE_NONE)
        np.testing.assert_allclose(c, e, rtol=1e-9, atol=1e-14)
        # TOVA: the scores already sum to one (Sec. 3.2), so h == w == alpha
        assert np.isclose(h.sum(), 1.0, rtol=1e-13)
    # and literal deletion, redone here with a library softmax
    s = (k @ q[0]) * scale
    alpha = scipy.special.softmax(s)
    j = n // 2
    keep = np.arange(n) != j
    o2 = scipy.special.softmax(s[keep]) @ v[keep]
    assert np.isclose(np.linalg.norm(alpha @ v - o2), e[j], rtol=1e-11)


def test_theorem_3_1_renormalised_weights(oracle):
    """alpha'_i = alpha_i / (1 - alpha_j) after evicting j."""
    n, d = 12, 8
    q = RNG.standard_normal((1, d))
    k = RNG.standard_normal((n, d))
    A = oracle.window_attention(q, k, 1, 1, 0.3, 0)[0]
    for j in (0, 5, n - 1):
        keep = np.arange(n) != j
        A2 = oracle.window_attention(q, k[keep], 1, 1, 0.3, 0)[0]
        np.testing.assert_allclose(A2, A[keep] / (1.0 - A[j]), rtol=1e-12)


# ---- attention slice -----------------------------------------------------------

def test_attention_matches_library_softmax_no_mask(oracle):
    G, W, n, d = 3, 4, 37, 16
    q = RNG.standard_normal((G * W, d))
    k = RNG.standard_normal((n, d))
    A = oracle.window_attention(q, k, G, W, 0.25, 0)
    ref = scipy.special.softmax(0.25 * q @ k.T, axis=1)
    np.testing.assert_allclose(A, ref, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(A.sum(axis=1), 1.0, rtol=1e-13)
    a = oracle.column_sums(A)
    np.testing.assert_allclose(a, ref.sum(axis=0), rtol=1e-12)
    assert np.isclose(a.sum(), G * W, rtol=1e-12)       # sum_j a_j = number of rows


def test_attention_window_causal_mask_against_torch(oracle):
    """Window keys are the last W cache rows; inside the window attention is causal."""
    G, W, n, d = 2, 5, 23, 8
    q = RNG.standard_normal((G, W, d))
    k = RNG.standard_normal((n, d))
    A = oracle.window_attention(q.reshape(G * W, d), k, G, W, 0.5, 1).reshape(G, W, n)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    logits = 0.5 * torch.einsum("gwd,nd->gwn", tq, tk)
    pos_q = (n - W) + torch.arange(W)
    mask = torch.arange(n)[None, :] > pos_q[:, None]
    ref = torch.softmax(logits.masked_fill(mask[None], float("-inf")), dim=-1).numpy()
    np.testing.assert_allclose(A, ref, rtol=1e-12, atol=1e-300)
    assert (A[:, :, :][:, mask.numpy()] == 0.0).all()


def test_h2o_sum_theorem_full_causal(oracle):
    """App. 'H2O scores': with b+1 tokens pushed through together (W = N, causal),
    the H2O scores sum to b+1, the first row attends only to itself and the last
    token's score is its own diagonal weight."""
    n, d = 19, 8
    x = RNG.standard_normal((n, d))
    k = RNG.standard_normal((n, d))
    v = RNG.standard_normal((n, d))
    A = oracle.window_attention(x, k, 1, n, 1.0, 1)
    assert A[0, 0] == 1.0 and (np.triu(A, 1) == 0.0).all()
    c, h, a = oracle.score_one(x, k, v, None, 1, n, 1.0, 1, oracle.BASE_H2O)
    assert np.isclose(h.sum(), n, rtol=1e-12)
    assert np.isclose(h[-1], A[-1, -1], rtol=1e-13)
    np.testing.assert_allclose(h, A.sum(axis=0), rtol=1e-12)


def test_zero_keys_give_uniform_weights_and_shift_invariance(oracle):
    G, W, n, d = 2, 3, 11, 4
    q = RNG.standard_normal((G * W, d))
    A = oracle.window_attention(q, np.zeros((n, d)), G, W, 1.0, 0)
    np.testing.assert_allclose(A, 1.0 / n, rtol=1e-14)
    k = RNG.standard_normal((n, d))
    u = RNG.standard_normal(d) * 5            # adds q_r.u to every logit of row r
    A1 = oracle.window_attention(q, k, G, W, 1.0, 1)
    A2 = oracle.window_attention(q, k + u, G, W, 1.0, 1)
    np.testing.assert_allclose(A1, A2, rtol=1e-9, atol=1e-300)


def test_row_without_visible_key_is_an_error(oracle):
    with pytest.raises(ValueError):
        oracle.window_attention(np.ones((4, 2)), np.ones((3, 2)), 1, 4, 1.0, 1)  # N < W


# ---- base scores ---------------------------------------------------------------

def test_h2o_accumulates_previous_attention(oracle):
    G, W, n, d = 2, 2, 9, 4
    q, k, v = RNG.standard_normal((G * W, d)), RNG.standard_normal((n, d)), RNG.standard_normal((n, d))
    h_in = RNG.random(n)
    c0, h0, a = oracle.score_one(q, k, v, None, G, W, 1.0, 1, oracle.BASE_H2O)
    c1, h1, _ = oracle.score_one(q, k, v, h_in, G, W, 1.0, 1, oracle.BASE_H2O)
    np.testing.assert_allclose(h0, a, rtol=0)
    np.testing.assert_allclose(h1, h_in + a, rtol=1e-15)
    assert np.isclose(h1.sum() - h_in.sum(), G * W, rtol=1e-12)
    # the scores follow the general formula with w = h / sum(h)
    w = h1 / h1.sum()
    o = w @ v
    np.testing.assert_allclose(c1, w / (1 - w) * np.linalg.norm(v - o, axis=1), rtol=1e-12)


def test_snapkv_pooling_against_library_max_filter(oracle):
    n, W = 40, 6
    a = RNG.random(n)
    lo, hi = 0, n - W
    h = oracle.base_score(a, None, oracle.BASE_SNAPKV, 7, lo, hi)
    ref = scipy.ndimage.maximum_filter1d(a[lo:hi], size=7, mode="constant", cval=-np.inf)
    np.testing.assert_array_equal(h[lo:hi], ref)
    np.testing.assert_array_equal(h[hi:], a[hi:])       # protected rows untouched
    assert (h[lo:hi] >= a[lo:hi]).all()
    # a spike spreads to exactly [j-3, j+3]
    spike = np.zeros(n)
    spike[15] = 1.0
    hs = oracle.base_score(spike, None, oracle.BASE_SNAPKV, 7, 0, n - W)
    assert np.array_equal(np.nonzero(hs)[0], np.arange(12, 19))
    # a spike just outside the scored range does not leak in; one at the edge is clipped
    spike = np.zeros(n)
    spike[hi] = 1.0
    spike[2] = 0.5
    hs = oracle.base_score(spike, None, oracle.BASE_SNAPKV, 7, 2, hi)
    assert (hs[hi - 3:hi] == 0.0).all() and hs[hi] == 1.0
    assert np.array_equal(np.nonzero(hs[:hi])[0], np.arange(2, 6))
    # with a protected head the head rows neither pool nor are pooled into
    hs = oracle.base_score(a, None, oracle.BASE_SNAPKV, 5, 4, hi)
    ref = scipy.ndimage.maximum_filter1d(a[4:hi], size=5, mode="constant", cval=-np.inf)
    np.testing.assert_array_equal(hs[4:hi], ref)
    np.testing.assert_array_equal(hs[:4], a[:4])


def test_snapkv_pool_width_one_is_base_none_with_protected_tail(oracle):
    G, W, n, d = 2, 4, 33, 8
    q, k, v = RNG.standard_normal((G * W, d)), RNG.standard_normal((n, d)), RNG.standard_normal((n, d))
    c0, h0, _ = oracle.score_one(q, k, v, None, G, W, 0.4, 1, oracle.BASE_NONE, 1, 0, W)
    c1, h1, _ = oracle.score_one(q, k, v, None, G, W, 0.4, 1, oracle.BASE_SNAPKV, 1, 0, W)
    np.testing.assert_array_equal(c0, c1)
    assert np.isinf(c1[n - W:]).all() and np.isfinite(c1[:n - W]).all()
    # protected rows take no part in the normalisation or in o
    w = h1[:n - W] / h1[:n - W].sum()
    o = w @ v[:n - W]
    np.testing.assert_allclose(c1[:n - W], w / (1 - w) * np.linalg.norm(v[:n - W] - o, axis=1),
                               rtol=1e-12)


# ---- score values: closed forms -------------------------------------------------

def test_normalisation_and_weighted_residual_identity(oracle):
    n, d = 50, 12
    h = RNG.random(n) * 3
    v = RNG.standard_normal((n, d))
    c, w, o = oracle.caote_scores(h, v)
    assert np.isclose(w.sum(), 1.0, rtol=1e-14)
    np.testing.assert_allclose(w, h / h.sum(), rtol=1e-14)
    np.testing.assert_allclose(o, (h / h.sum()) @ v, rtol=1e-12)
    np.testing.assert_allclose(w @ (v - o), 0.0, atol=1e-14)


def test_equal_values_give_zero_scores(oracle):
    n, d = 9, 5
    v = np.tile(RNG.standard_normal(d), (n, 1))
    c, _, _ = oracle.caote_scores(_weights(n), v)
    np.testing.assert_allclose(c, 0.0, atol=1e-15)


def test_uniform_weights_reduce_to_fastcaote(oracle):
    """w = 1/N  =>  c_j = ||v_j - mean(v)|| / (N-1), which is the FastCAOTE score."""
    n, d = 21, 6
    v = RNG.standard_normal((n, d))
    c, _, o = oracle.caote_scores(np.ones(n), v)
    ref = np.linalg.norm(v - v.mean(axis=0), axis=1) / (n - 1)
    np.testing.assert_allclose(c, ref, rtol=1e-12)
    cf, _, of = oracle.caote_scores(np.ones(n), v, fast=True)
    np.testing.assert_allclose(cf, ref, rtol=1e-12)
    np.testing.assert_allclose(of, v.mean(axis=0), rtol=1e-12, atol=1e-15)


def test_fastcaote_uses_plain_mean_with_general_weights(oracle):
    n, d = 14, 5
    w = _weights(n)
    v = RNG.standard_normal((n, d))
    cf, _, _ = oracle.caote_scores(w, v, fast=True)
    ref = w / (1 - w) * np.linalg.norm(v.mean(axis=0) - v, axis=1)
    np.testing.assert_allclose(cf, ref, rtol=1e-12)


def test_two_token_closed_form(oracle):
    p = 0.3
    v = RNG.standard_normal((2, 7))
    c, _, _ = oracle.caote_scores(np.array([p, 1 - p]), v)
    dist = np.linalg.norm(v[0] - v[1])
    np.testing.assert_allclose(c, [p * dist, (1 - p) * dist], rtol=1e-12)


def test_monotone_in_weight_at_fixed_distance(oracle):
    """Tokens at the same distance from o are ranked by their weight."""
    d = 4
    u = RNG.standard_normal(d)
    u /= np.linalg.norm(u)
    # four tokens on a sphere around the origin in symmetric pairs, so o = 0 regardless
    v = np.stack([u, -u, 2 * u[::-1], -2 * u[::-1]])
    w = np.array([0.1, 0.1, 0.4, 0.4])
    c, _, o = oracle.caote_scores(w, v)
    np.testing.assert_allclose(o, 0.0, atol=1e-16)
    np.testing.assert_allclose(c, w / (1 - w) * np.array([1, 1, 2, 2]), rtol=1e-12)
    ws = np.linspace(0.01, 0.9, 30)
    f = ws / (1 - ws)
    assert (np.diff(f) > 0).all()


def test_score_zero_iff_zero_weight_or_value_at_output(oracle):
    n, d = 6, 3
    v = RNG.standard_normal((n, d))
    h = RNG.random(n)
    h[2] = 0.0
    c, w, o = oracle.caote_scores(h, v)
    assert c[2] == 0.0 and (np.delete(c, 2) > 0).all()
    v2 = v.copy()
    # put token 4 exactly at the output: o = sum_{i != 4} w_i v_i / (1 - w_4)
    keep = np.arange(n) != 4
    v2[4] = (w[keep] @ v[keep]) / (1 - w[4])
    c2, _, o2 = oracle.caote_scores(h, v2)
    assert c2[4] < 1e-15 and np.allclose(o2, v2[4])


def test_protected_rows_and_degenerate_sets(oracle):
    n, d = 8, 3
    v = RNG.standard_normal((n, d))
    h = RNG.random(n)
    c, w, _ = oracle.caote_scores(h, v, lo=2, hi=6)
    assert np.isinf(c[:2]).all() and np.isinf(c[6:]).all() and np.isfinite(c[2:6]).all()
    assert w[:2].sum() == 0 and np.isclose(w.sum(), 1.0)
    c, _, _ = oracle.caote_scores(h, v, lo=3, hi=4)     # a single scored token is never evicted
    assert np.isinf(c).all()
    c, _, _ = oracle.caote_scores(np.zeros(n), v)       # no attention mass anywhere
    assert (c == 0).all()


def test_joint_score_reduces_to_single_and_matches_two_token_removal(oracle):
    n, d = 10, 4
    w = _weights(n)
    v = RNG.standard_normal((n, d))
    c, _, o = oracle.caote_scores(w, v)
    for j in range(n):
        assert np.isclose(oracle.joint_eviction_error(w, v, [j]), c[j], rtol=1e-12)
    for i, j in itertools.combinations(range(4), 2):
        keep = np.ones(n, bool)
        keep[[i, j]] = False
        o2 = (w[keep] / w[keep].sum()) @ v[keep]
        assert np.isclose(oracle.joint_eviction_error(w, v, [i, j]), np.linalg.norm(o - o2), rtol=1e-11)


def _removal_error(w, v, gone):
    """Joint error by its definition: take the tokens out, renormalise, measure the change."""
    keep = np.ones(len(w), bool)
    keep[list(gone)] = False
    if not keep.any() or w[keep].sum() <= 0:
        return np.inf
    return np.linalg.norm(w @ v - (w[keep] / w[keep].sum()) @ v[keep])


def test_joint_error_matches_removal_of_larger_sets(oracle):
    n, d = 9, 5
    w = _weights(n)
    v = RNG.standard_normal((n, d))
    for m in (3, 4, 6):
        for gone in itertools.islice(itertools.combinations(range(n), m), 12):
            assert np.isclose(oracle.joint_eviction_error(w, v, list(gone)), _removal_error(w, v, gone),
                              rtol=1e-10)


def test_greedy_joint_eviction_step_by_step_against_real_removal(oracle):
    """Every step of the greedy evicts the candidate whose real removal, together with what
    is already gone, changes the output least (App. B), and reports that change."""
    n, d, m = 12, 4, 7
    for trial in range(4):
        w = _weights(n)
        v = RNG.standard_normal((n, d)) * np.exp(RNG.standard_normal((n, 1)))
        order, err = oracle.greedy_joint_evict(w, v, m)
        assert len(set(order.tolist())) == m
        gone = []
        for t in range(m):
            cand = {j: _removal_error(w, v, gone + [j]) for j in range(n) if j not in gone}
            best = min(cand.values())
            assert np.isclose(cand[int(order[t])], best, rtol=1e-10), (trial, t)
            assert np.isclose(err[t], best, rtol=1e-9)
            gone.append(int(order[t]))
        # and the reported errors are the general m-token formula on the evicted prefix
        for t in range(m):
            assert np.isclose(err[t], oracle.joint_eviction_error(w, v, order[:t + 1]), rtol=1e-10)
        # the per-step candidate table: the m-token formula for S + j, NaN for what is gone
        c = oracle.joint_candidates(w, v, order[:3])
        assert np.isnan(c[order[:3]]).all()
        for j in range(n):
            if j not in order[:3]:
                assert np.isclose(c[j], _removal_error(w, v, list(order[:3]) + [j]), rtol=1e-10)


def test_greedy_joint_first_step_is_the_single_token_choice(oracle):
    n, d = 40, 8
    w = _weights(n)
    v = RNG.standard_normal((n, d))
    c, _, _ = oracle.caote_scores(w, v)
    order, err = oracle.greedy_joint_evict(w, v, 1)
    assert order[0] == np.argmin(c) and np.isclose(err[0], c.min(), rtol=1e-12)


def test_greedy_joint_finds_a_cancelling_pair(oracle):
    """Two tokens whose weighted offsets from the output are opposite cancel exactly: after
    one of them is gone the other is the next to go and the joint error drops to zero,
    although a third token has a smaller single-token score than the second."""
    n, d = 8, 6
    w = _weights(n)
    v = RNG.standard_normal((n, d))
    x = np.zeros(d)
    x[0] = 1e-3                                          # tiny offset: token 0 goes first
    # tokens 0 and 1: w0 (o - v0) = -w1 (o - v1) = -x; the others are re-centred so that o = 0
    rest = np.arange(2, n)
    v[rest] -= (w[rest] @ v[rest]) / w[rest].sum()
    v[0] = x / w[0]
    v[1] = -x / w[1]
    assert np.allclose(w @ v, 0, atol=1e-15)
    c, _, _ = oracle.caote_scores(w, v)
    assert np.argmin(c) in (0, 1)
    order, err = oracle.greedy_joint_evict(w, v, 2)
    assert set(order.tolist()) == {0, 1}
    assert err[1] < 1e-12 and err[0] > 1e-4


def test_greedy_joint_protected_rows_ties_and_exhaustion(oracle):
    n, d = 10, 3
    v = RNG.standard_normal((n, d))
    h = RNG.random(n)
    _, w, _ = oracle.caote_scores(h, v, lo=2, hi=8)
    order, _ = oracle.greedy_joint_evict(w, v, 6, lo=2, hi=8)      # every scored token goes
    assert sorted(order.tolist()) == list(range(2, 8))
    # identical tokens tie: the higher index leaves first
    v2 = np.tile(RNG.standard_normal((1, d)), (n, 1))
    v2[0] += 1.0
    w2 = np.full(n, 1.0 / n)
    order, _ = oracle.greedy_joint_evict(w2, v2, 3)
    assert order.tolist() == [9, 8, 7]
    with pytest.raises(ValueError):
        oracle.greedy_joint_evict(w, v, 7, lo=2, hi=8)


# ---- selection and compaction -----------------------------------------------------

def test_select_against_lexsort(oracle):
    n = 200
    c = np.round(RNG.random(n), 2)                     # many ties
    c[[3, 77, 150]] = np.inf
    for b in (1, 3, 50, 199, 200):
        idx = oracle.select_one(c, b)
        order = np.lexsort((np.arange(n), -c))         # score desc, index asc
        ref = np.sort(order[:b])
        np.testing.assert_array_equal(idx, ref)
    idx = oracle.select_one(c, 3)
    np.testing.assert_array_equal(idx, [3, 77, 150])   # protected first
    idx = oracle.select_one(c, 205)
    np.testing.assert_array_equal(idx[:200], np.arange(200))
    assert (idx[200:] == -1).all()


def test_select_tie_keeps_lower_index(oracle):
    c = np.array([1.0, 2.0, 1.0, 1.0, 3.0])
    np.testing.assert_array_equal(oracle.select_one(c, 3), [0, 1, 4])
    np.testing.assert_array_equal(oracle.select_one(c, 4), [0, 1, 2, 4])


def test_compact_stable_and_swap_last(oracle):
    n = 12
    rows = RNG.integers(0, 2 ** 15, size=(n, 5)).astype(np.uint16)
    idx = np.array([0, 1, 4, 5, 9, 11], dtype=np.int32)
    out, m = oracle.compact_one(rows, idx, "stable")
    assert m == 6
    np.testing.assert_array_equal(out[:6], rows[idx])
    np.testing.assert_array_equal(out[6:], rows[6:])   # beyond the new length: untouched
    out, m = oracle.compact_one(rows, np.arange(n, dtype=np.int32), "stable")
    np.testing.assert_array_equal(out, rows)
    # evict-one: the last row drops into the hole
    for jstar in (0, 5, n - 1):
        idx = np.delete(np.arange(n, dtype=np.int32), jstar)
        out, m = oracle.compact_one(rows, idx, "swap_last")
        assert m == n - 1
        ref = rows.copy()
        ref[jstar] = rows[n - 1]
        np.testing.assert_array_equal(out[:n - 1], ref[:n - 1])
    with pytest.raises(ValueError):
        oracle.compact_one(rows, np.arange(n - 2, dtype=np.int32), "swap_last")
    # padded (-1) index lists: all tokens kept, nothing moves
    idx = np.concatenate([np.arange(n), [-1, -1]]).astype(np.int32)
    out, m = oracle.compact_one(rows, idx, "stable")
    assert m == n
    np.testing.assert_array_equal(out, rows)


def test_compact_fill_moves_only_rows_from_beyond_the_new_length(oracle):
    """Hole-filling compaction against its statement written with numpy set operations: kept rows
    below the new length stay, the kept rows from beyond it drop into the freed positions, both in
    ascending order.  Special cases that reduce to the other two modes."""
    for seed, (n, n_keep) in enumerate([(12, 6), (40, 13), (40, 39), (40, 1), (300, 150), (300, 20), (64, 32)]):
        rng = np.random.default_rng(4100 + seed)
        rows = rng.integers(0, 2 ** 31, size=(n, 3)).astype(np.uint32)
        idx = np.sort(rng.choice(n, size=n_keep, replace=False)).astype(np.int32)
        out, m = oracle.compact_one(rows, idx, "fill")
        assert m == n_keep
        holes = np.array(sorted(set(range(n_keep)) - set(idx.tolist())), dtype=np.int64)
        movers = idx[idx >= n_keep]
        assert len(holes) == len(movers)
        ref = rows.copy()
        ref[holes] = rows[movers]
        np.testing.assert_array_equal(out, ref)              # rows at and beyond n_keep untouched too
        stay = idx[idx < n_keep]
        np.testing.assert_array_equal(out[stay], rows[stay])
        # the rows below the new length are exactly the kept rows, each once
        assert sorted(map(tuple, out[:n_keep])) == sorted(map(tuple, rows[idx]))
    n = 12
    rows = RNG.integers(0, 2 ** 15, size=(n, 5)).astype(np.uint16)
    for jstar in (0, 5, n - 1):                              # one evicted token: swap_last
        idx = np.delete(np.arange(n, dtype=np.int32), jstar)
        a, _ = oracle.compact_one(rows, idx, "fill")
        b, _ = oracle.compact_one(rows, idx, "swap_last")
        np.testing.assert_array_equal(a, b)
    idx = np.arange(6, 12, dtype=np.int32)                   # every kept row from beyond: stable
    a, _ = oracle.compact_one(rows, idx, "fill")
    b, _ = oracle.compact_one(rows, idx, "stable")
    np.testing.assert_array_equal(a, b)
    idx = np.arange(6, dtype=np.int32)                       # the first rows kept: nothing moves
    a, m = oracle.compact_one(rows, idx, "fill")
    assert m == 6
    np.testing.assert_array_equal(a, rows)
    idx = np.concatenate([np.arange(n), [-1, -1]]).astype(np.int32)   # nothing evicted
    a, m = oracle.compact_one(rows, idx, "fill")
    assert m == n
    np.testing.assert_array_equal(a, rows)


# ---- the batched wrapper only loops ----------------------------------------------

def test_batched_wrapper_matches_single_instances(oracle):
    from paper_2504_14051_amd import synth
    wl = synth.tiny().with_(batch=2, n_q_heads=4, n_kv_heads=2, context=96, window=4, budget=40,
                            head_dim=16)
    lens = np.array([96, 70], dtype=np.int32)
    cache = synth.make_cache(wl, seq_lens=lens, base_init="random")
    c, h, a = oracle.score_batched(cache.q.double().numpy(), cache.K.double().numpy(),
                                   cache.V.double().numpy(), cache.base.numpy(), lens,
                                   n_kv_heads=2, window=4, scale=wl.softmax_scale,
                                   window_in_cache=1, base=oracle.BASE_H2O, threads=2)
    b, hk, N = 1, 1, 70
    q1 = cache.q[b, 2:4].double().numpy().reshape(8, 16)
    c1, h1, a1 = oracle.score_one(q1, cache.K[b, hk, :N].double().numpy(),
                                  cache.V[b, hk, :N].double().numpy(),
                                  cache.base[b, hk, :N].numpy(), 2, 4, wl.softmax_scale, 1,
                                  oracle.BASE_H2O)
    np.testing.assert_array_equal(c[b, hk, :N], c1)
    np.testing.assert_array_equal(h[b, hk, :N], h1)
    assert np.isnan(c[b, hk, N:]).all()
    kept = oracle.select_batched(c, lens, 40)
    np.testing.assert_array_equal(kept[b, hk], oracle.select_one(c1, 40))


# ---- row normalisers handed over by the caller (App. C: the attention weights exist already) --

def _masked_logits(q, k, W, scale, wic):
    R, N = q.shape[0], k.shape[0]
    s = (q @ k.T) * scale
    if wic:
        i = np.arange(R) % W
        vis = np.arange(N)[None, :] < (N - W + i + 1)[:, None]
        s = np.where(vis, s, -np.inf)
    return s


@pytest.mark.parametrize("G,W,N,d,wic", [(1, 1, 9, 4, 0), (2, 3, 17, 8, 1), (4, 8, 40, 16, 1), (7, 2, 33, 8, 0)])
def test_row_lse_is_the_library_logsumexp(oracle, G, W, N, d, wic):
    q = RNG.standard_normal((G * W, d))
    k = RNG.standard_normal((N, d)) * 2.0
    scale = 0.7 / np.sqrt(d)
    s = _masked_logits(q, k, W, scale, wic)
    np.testing.assert_allclose(oracle.row_lse(q, k, G, W, scale, wic),
                               scipy.special.logsumexp(s, axis=1), rtol=1e-13)


@pytest.mark.parametrize("G,W,N,d,wic", [(2, 3, 17, 8, 1), (4, 4, 64, 16, 1), (1, 5, 21, 8, 0)])
def test_given_lse_reproduces_the_softmax_and_the_scores(oracle, G, W, N, d, wic):
    q = RNG.standard_normal((G * W, d))
    k = RNG.standard_normal((N, d))
    v = RNG.standard_normal((N, d))
    scale = 1.0 / np.sqrt(d)
    s = _masked_logits(q, k, W, scale, wic)
    lse = scipy.special.logsumexp(s, axis=1)                    # the caller's normalisers
    A = oracle.window_attention_given_lse(q, k, G, W, scale, wic, lse)
    np.testing.assert_allclose(A, scipy.special.softmax(s, axis=1), rtol=1e-12, atol=1e-300)
    for base, h_in in ((oracle.BASE_NONE, None), (oracle.BASE_H2O, RNG.random(N)),
                       (oracle.BASE_SNAPKV, None)):
        kw = dict(pool_kernel=3, n_protect_tail=W if base == oracle.BASE_SNAPKV else 0)
        c0, h0, a0 = oracle.score_one(q, k, v, h_in, G, W, scale, wic, base, **kw)
        c1, h1, a1 = oracle.score_one(q, k, v, h_in, G, W, scale, wic, base, lse=lse, **kw)
        np.testing.assert_allclose(a1, a0, rtol=1e-12)
        np.testing.assert_allclose(h1, h0, rtol=1e-12)
        np.testing.assert_allclose(c1, c0, rtol=1e-9, atol=1e-14)


def test_shifted_lse_scales_the_attention_mass(oracle):
    """lse + log 2 halves every column sum: nothing is renormalised behind the caller's back.
    Without an accumulator the scores do not change (w = h / sum h); with one they follow
    h = h_in + a / 2."""
    G, W, N, d = 2, 4, 30, 8
    q = RNG.standard_normal((G * W, d))
    k = RNG.standard_normal((N, d))
    v = RNG.standard_normal((N, d))
    scale = 1.0 / np.sqrt(d)
    lse = oracle.row_lse(q, k, G, W, scale, 1)
    c0, h0, a0 = oracle.score_one(q, k, v, None, G, W, scale, 1, oracle.BASE_NONE, lse=lse)
    c1, h1, a1 = oracle.score_one(q, k, v, None, G, W, scale, 1, oracle.BASE_NONE, lse=lse + np.log(2.0))
    np.testing.assert_allclose(a1, a0 / 2, rtol=1e-13)
    np.testing.assert_allclose(c1, c0, rtol=1e-10)
    assert np.isclose(a0.sum(), G * W, rtol=1e-12) and np.isclose(a1.sum(), G * W / 2, rtol=1e-12)
    h_in = RNG.random(N)
    c2, h2, a2 = oracle.score_one(q, k, v, h_in, G, W, scale, 1, oracle.BASE_H2O, lse=lse + np.log(2.0))
    np.testing.assert_allclose(h2, h_in + a0 / 2, rtol=1e-13)
    c3, _, _ = oracle.caote_scores(h_in + a0 / 2, v)
    np.testing.assert_allclose(c2, c3, rtol=1e-12)
