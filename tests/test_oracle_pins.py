"""Pins for the CPU oracle: everything here checks ``oracle/`` against something other than
itself — a hand-worked rational example, closed forms, invariants, library routines and
brute force.  CPU only."""
import itertools
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import wkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------------------
# hand-worked rational example (Eq. 1-4)
# ---------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def rational():
    with open(os.path.join(GOLDEN, "rational_example.json")) as f:
        return json.load(f)


def _fr(xs):
    return np.array([float(Fraction(x)) for x in xs])


def test_rational_example_scores(rational):
    g = rational
    keys = np.log(np.array(g["c"], dtype=np.float64))[:, None]          # d = 1
    q = np.array([g["q_head_a"], g["q_head_b"]], dtype=np.float64)[:, :, None]
    # row sums of the un-normalised weights pin the causal mask: 18, 64 / 48, 22
    for head, sums in ((0, g["row_sums_head_a"]), (1, g["row_sums_head_b"])):
        A = O.attention_probs(q[head], keys, scale=1.0)
        for i, z in enumerate(sums):
            j = 2  # c_2 = 3 : A[i, 2] = 3^q / Z
            assert A[i, j] == pytest.approx(3.0 ** q[head, i, 0] / float(Fraction(z)), rel=1e-13)
        assert A[0, 8] == 0.0          # the first observation query cannot see the last key
    t = O.token_scores(q, keys, scale=1.0)
    np.testing.assert_allclose(t, _fr(g["t"]), rtol=1e-13)
    for p in (1, 2, 3):
        s = O.window_scores(t, g["omega"], p)
        np.testing.assert_allclose(s, _fr(g[f"s_p{p}"]), rtol=1e-13)


def test_rational_example_selection(rational):
    g = rational
    keys = np.log(np.array(g["c"], dtype=np.float64))[:, None]
    q = np.array([g["q_head_a"], g["q_head_b"]], dtype=np.float64)[:, :, None]
    _, _, sel, idx = O.select_indices(q, keys, g["omega"], 3, 2, scale=1.0)
    assert sel.tolist() == g["selected_p3_k2"]
    assert idx.tolist() == g["tok_idx_p3_k2"]
    _, _, sel, idx = O.select_indices(q, keys, g["omega"], 2, 1, scale=1.0)
    assert sel.tolist() == g["selected_p2_k1"]
    assert idx.tolist() == g["tok_idx_p2_k1"]


def test_default_scale_is_inverse_sqrt_d():
    # d = 4 -> 1/sqrt(d) = 1/2: keys 2*ln(c) e_0 and a query e_0 give weights c again.
    c = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    keys = np.zeros((5, 4)); keys[:, 0] = 2.0 * np.log(c)
    q = np.zeros((1, 4)); q[0, 0] = 1.0
    A = O.attention_probs(q, keys)
    np.testing.assert_allclose(A[0], c / c.sum(), rtol=1e-13)


# ---------------------------------------------------------------------------------------
# invariants and closed forms (Eq. 1-2)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,alpha,d", [(40, 8, 16), (97, 5, 8), (33, 32, 4)])
def test_rows_sum_to_one_and_mask(n, alpha, d):
    r = _rng(1)
    A = O.attention_probs(r.standard_normal((alpha, d)), r.standard_normal((n, d)) * 3)
    np.testing.assert_allclose(A.sum(1), 1.0, rtol=1e-13)
    for i in range(alpha):
        assert np.all(A[i, n - alpha + i + 1:] == 0.0)
        assert np.all(A[i, : n - alpha + i + 1] > 0.0)


@pytest.mark.parametrize("n,alpha,G", [(64, 8, 2), (129, 16, 4)])
def test_zero_queries_give_harmonic_numbers(n, alpha, G):
    # Q = 0: each observation query spreads uniformly over the keys it sees, so
    # t_j = G * (H_n - H_{n-alpha}) for every review token.
    r = _rng(2)
    t = O.token_scores(np.zeros((G, alpha, 8)), r.standard_normal((n, 8)))
    H = lambda m: sum(Fraction(1, i) for i in range(1, m + 1))
    np.testing.assert_allclose(t, G * float(H(n) - H(n - alpha)), rtol=1e-13)


def test_two_level_keys_closed_form():
    # keys in S have logit x, the others 0 => A_ij = e^x / (|S_vis| e^x + vis - |S_vis|)
    n, alpha, d, x = 50, 6, 9, 1.7
    S = [3, 10, 11, 46, 48]
    q = np.zeros((alpha, d)); q[:, 0] = 1.0
    keys = np.zeros((n, d)); keys[S, 0] = x * math.sqrt(d)        # q.k/sqrt(d) = x
    A = O.attention_probs(q, keys)
    for i in range(alpha):
        vis = n - alpha + i + 1
        s_vis = sum(1 for j in S if j < vis)
        Z = s_vis * math.exp(x) + (vis - s_vis)
        for j in range(vis):
            want = (math.exp(x) if j in S else 1.0) / Z
            assert A[i, j] == pytest.approx(want, rel=1e-13)


def test_mass_conservation():
    # summed over ALL keys (review context + observation window) the probabilities of the
    # G*alpha observation rows add to G*alpha; t holds the review-context part of it.
    r = _rng(3)
    G, alpha, n, d = 3, 7, 60, 12
    q = r.standard_normal((G, alpha, d)); K = r.standard_normal((n, d))
    t = O.token_scores(q, K)
    tail = sum(O.attention_probs(q[g], K)[:, n - alpha:].sum() for g in range(G))
    assert t.sum() + tail == pytest.approx(G * alpha, rel=1e-13)
    assert t.shape == (n - alpha,)


def test_matches_torch_sdpa_with_identity_values():
    # softmax(QK^T/sqrt(d)) @ I = A : a library routine on the same inputs.
    r = _rng(4)
    alpha, n, d = 8, 48, 16
    q = r.standard_normal((alpha, d)); K = r.standard_normal((n, d))
    mask = torch.arange(n)[None, :] <= (n - alpha + torch.arange(alpha))[:, None]
    A_lib = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None], torch.from_numpy(K)[None, None],
        torch.eye(n, dtype=torch.float64)[None, None], attn_mask=mask[None, None])[0, 0].numpy()
    np.testing.assert_allclose(O.attention_probs(q, K), A_lib, rtol=1e-11, atol=1e-15)


def test_lse_matches_scipy_logsumexp_and_recovers_probs():
    # the hand-over form of the normaliser: a library log-sum-exp over the visible keys, and
    # exp(logit - lse) must be the probability of Eq. 1
    from scipy.special import logsumexp
    rng = np.random.default_rng(11)
    n, alpha, d = 53, 6, 8
    q = rng.standard_normal((alpha, d)) * 3.0
    k = rng.standard_normal((n, d)) * 3.0
    lse = O.softmax_lse(q, k)
    A = O.attention_probs(q, k)
    for i in range(alpha):
        vis = n - alpha + i + 1
        logits = (k[:vis] @ q[i]) / math.sqrt(d)
        assert lse[i] == pytest.approx(logsumexp(logits), rel=1e-13)
        np.testing.assert_allclose(np.exp(logits - lse[i]), A[i, :vis], rtol=1e-12)
    # explicit scale
    np.testing.assert_allclose(O.softmax_lse(q, k, scale=0.5), O.softmax_lse(q * 0.5 * math.sqrt(d), k), rtol=1e-13)


def test_lse_of_zero_queries_is_log_of_visible_count():
    n, alpha, d = 40, 5, 4
    k = np.random.default_rng(3).standard_normal((n, d))
    lse = O.softmax_lse(np.zeros((alpha, d)), k)
    np.testing.assert_allclose(lse, np.log(n - alpha + 1 + np.arange(alpha)), rtol=1e-14)


def test_scalar_rederivation_tiny():
    # brute force with scalar loops and math.exp, written term by term from Eq. 1-2.
    r = _rng(5)
    G, alpha, n, d = 2, 3, 11, 4
    q = r.standard_normal((G, alpha, d)); K = r.standard_normal((n, d))
    t = [0.0] * (n - alpha)
    for g in range(G):
        for i in range(alpha):
            last_visible = n - alpha + i
            e = []
            for j in range(last_visible + 1):
                dot = sum(q[g, i, c] * K[j, c] for c in range(d))
                e.append(math.exp(dot / math.sqrt(d)))
            Z = sum(e)
            for j in range(n - alpha):
                t[j] += e[j] / Z
    np.testing.assert_allclose(O.token_scores(q, K), t, rtol=1e-12)


def test_scores_depend_on_head_sum_not_mean_or_single_head():
    r = _rng(6)
    q = r.standard_normal((4, 5, 8)); K = r.standard_normal((30, 8))
    t = O.token_scores(q, K)
    parts = [O.token_scores(q[g:g + 1], K) for g in range(4)]
    np.testing.assert_allclose(t, sum(parts), rtol=1e-13)


# ---------------------------------------------------------------------------------------
# Eq. 3-4 against library pooling routines
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("omega", [4, 8, 16, 32])
def test_pool_mean_and_max_special_cases(omega):
    t = _rng(7).random(omega * 13)
    np.testing.assert_allclose(O.window_scores(t, omega, omega), t.reshape(-1, omega).mean(1), rtol=1e-13)
    mp = torch.nn.functional.max_pool1d(torch.from_numpy(t)[None, None], omega, omega)[0, 0].numpy()
    np.testing.assert_allclose(O.window_scores(t, omega, 1), mp, rtol=0)


@pytest.mark.parametrize("omega,p", [(8, 3), (16, 8), (32, 16), (8, 7)])
def test_pool_top_p_matches_torch_topk(omega, p):
    t = _rng(8).random(omega * 9)
    want = torch.from_numpy(t).view(-1, omega).topk(p, dim=1).values.sum(1).numpy() / p
    np.testing.assert_allclose(O.window_scores(t, omega, p), want, rtol=1e-13)


def test_pool_p_larger_than_window_is_mean():
    t = _rng(9).random(24)
    np.testing.assert_allclose(O.window_scores(t, 8, 20), t.reshape(-1, 8).mean(1), rtol=1e-13)


def test_pool_partial_tail_window_by_hand():
    t = np.array([1.0, 5.0, 2.0, 4.0, 3.0, 9.0, 7.0])          # omega=3 -> {1,5,2},{4,3,9},{7}
    np.testing.assert_allclose(O.window_scores(t, 3, 3), [8 / 3, 16 / 3, 7 / 3])
    np.testing.assert_allclose(O.window_scores(t, 3, 2), [7 / 2, 13 / 2, 7 / 2])
    np.testing.assert_allclose(O.window_scores(t, 3, 1), [5.0, 9.0, 7.0])
    assert len(O.window_scores(np.arange(17.0), 8, 8)) == 3      # ceil(17/8)


# ---------------------------------------------------------------------------------------
# selection: brute force over every subset, argsort, ties, invariants
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("nw,k,seed", [(10, 3, 0), (12, 5, 1), (9, 9, 2), (11, 1, 3), (8, 0, 4)])
def test_selection_is_the_max_sum_subset(nw, k, seed):
    s = _rng(100 + seed).random(nw)
    best = max(itertools.combinations(range(nw), k), key=lambda c: sum(s[list(c)]))
    assert O.select_windows(s, k).tolist() == sorted(best)
    assert sorted(np.argsort(s)[::-1][:k].tolist()) == O.select_windows(s, k).tolist()


def test_selection_ties_prefer_lower_index():
    s = np.array([0.5, 0.9, 0.5, 0.5, 0.1, 0.9])
    assert O.select_windows(s, 2).tolist() == [1, 5]
    assert O.select_windows(s, 3).tolist() == [0, 1, 5]
    assert O.select_windows(s, 4).tolist() == [0, 1, 2, 5]


def test_end_to_end_micro_brute_force():
    # L=48, w_obs=8, win=4 -> 10 windows; the selected set must be the best of all C(10,k).
    r = _rng(11)
    G, alpha, n, d, omega = 2, 8, 48, 8, 4
    q = r.standard_normal((G, alpha, d)); K = r.standard_normal((n, d)) * 2
    for p, k in ((4, 3), (2, 4), (1, 2)):
        t, s, sel, idx = O.select_indices(q, K, omega, p, k)
        best = max(itertools.combinations(range(len(s)), k), key=lambda c: sum(s[list(c)]))
        assert sel.tolist() == sorted(best)
        # invariants: count, sorted, contiguous inside windows, observation window appended
        assert len(idx) == k * omega + alpha
        assert np.all(np.diff(idx) > 0)
        for m, w in enumerate(sel):
            assert idx[m * omega:(m + 1) * omega].tolist() == list(range(w * omega, (w + 1) * omega))
        assert idx[-alpha:].tolist() == list(range(n - alpha, n))


def test_token_indices_partial_tail_window():
    # n - alpha = 10, omega = 4: windows {0..3},{4..7},{8,9}
    idx = O.token_indices([0, 2], 4, 13, 3)
    assert idx.tolist() == [0, 1, 2, 3, 8, 9, 10, 11, 12]


# ---------------------------------------------------------------------------------------
# group sharing and gather (Section 2.2.2)
# ---------------------------------------------------------------------------------------
def test_group_uses_first_layer_only_and_gathers_every_layer():
    r = _rng(12)
    G, alpha, n, d, gamma = 2, 4, 40, 8, 3
    q = r.standard_normal((G, alpha, d))
    Ks = [r.standard_normal((n, d)) for _ in range(gamma)]
    Vs = [r.standard_normal((n, d)) for _ in range(gamma)]
    t, s, sel, idx, k_out, v_out = O.compress_group(q, Ks, Vs, 4, 4, 3)
    # changing the other layers' keys must not move the indices
    Ks2 = [Ks[0]] + [r.standard_normal((n, d)) for _ in range(gamma - 1)]
    assert O.compress_group(q, Ks2, Vs, 4, 4, 3)[3].tolist() == idx.tolist()
    for l in range(gamma):
        want_k = torch.index_select(torch.from_numpy(Ks[l]), 0, torch.from_numpy(idx)).numpy()
        want_v = torch.index_select(torch.from_numpy(Vs[l]), 0, torch.from_numpy(idx)).numpy()
        assert np.array_equal(k_out[l], want_k) and np.array_equal(v_out[l], want_v)


def test_planted_aligned_span_is_selected():
    # keys aligned with the mean observation query inside one window-aligned span must win.
    r = _rng(13)
    G, alpha, n, d, omega = 4, 16, 1040, 32, 16
    q = r.standard_normal((G, alpha, d)) + 1.0
    K = r.standard_normal((n, d))
    qhat = q.reshape(-1, d).mean(0); qhat /= np.linalg.norm(qhat)
    K[320:384] = math.sqrt(d) * qhat
    _, s, sel, _ = O.select_indices(q, K, omega, omega, 8)
    assert {20, 21, 22, 23} <= set(sel.tolist())


# ---------------------------------------------------------------------------------------
# Eq. 5-7 closed forms
# ---------------------------------------------------------------------------------------
def test_decode_step_matches_torch_sdpa():
    rng = np.random.default_rng(21)
    n, d, G = 37, 16, 3
    q = rng.standard_normal((G, d)); kk = rng.standard_normal((n, d)); vv = rng.standard_normal((n, d))
    kn = rng.standard_normal(d); vn = rng.standard_normal(d)
    out, K, V = O.decode_step(q, kk, vv, kn, vn)
    assert K.shape == (n + 1, d) and np.array_equal(K[-1], kn) and np.array_equal(V[-1], vn) and np.array_equal(K[:n], kk)
    tq = torch.from_numpy(q)[None, :, None, :]                      # [1, G, 1, d]: G heads, one query each
    tk = torch.from_numpy(K)[None, None].expand(1, G, n + 1, d)
    tv = torch.from_numpy(V)[None, None].expand(1, G, n + 1, d)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0].numpy()
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-14)
    out2, _, _ = O.decode_step(q, kk, vv, kn, vn, scale=0.3)
    want2 = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.3)[0, :, 0].numpy()
    np.testing.assert_allclose(out2, want2, rtol=1e-12, atol=1e-14)


def test_decode_step_closed_forms():
    rng = np.random.default_rng(22)
    n, d = 9, 8
    kk = rng.standard_normal((n, d)); vv = rng.standard_normal((n, d)); kn = rng.standard_normal(d); vn = rng.standard_normal(d)
    # a zero query weighs every token equally: the output is the mean of all n+1 values
    out, _, V = O.decode_step(np.zeros((2, d)), kk, vv, kn, vn)
    np.testing.assert_allclose(out, np.broadcast_to(V.mean(axis=0), (2, d)), rtol=1e-13)
    # an empty retained cache: the token attends to itself only
    out, _, _ = O.decode_step(rng.standard_normal((2, d)), np.zeros((0, d)), np.zeros((0, d)), kn, vn)
    np.testing.assert_allclose(out, np.broadcast_to(vn, (2, d)), rtol=1e-15)
    # a query far along one key: the output tends to that key's value
    q = 200.0 * kk[4][None, :] / np.linalg.norm(kk[4])
    kk2 = kk.copy(); kk2[4] *= 10.0
    out, _, _ = O.decode_step(q, kk2, vv, kn, vn, scale=1.0)
    np.testing.assert_allclose(out[0], vv[4], atol=1e-9)


def test_jaccard_closed_forms_and_numpy():
    assert O.jaccard([], []) == 1.0
    assert O.jaccard([1, 2, 3], [1, 2, 3]) == 1.0
    assert O.jaccard([1, 2, 3], [4, 5]) == 0.0
    assert O.jaccard(range(0, 8), range(4, 12)) == pytest.approx(4 / 12)          # half of each shared
    rng = np.random.default_rng(31)
    for _ in range(20):
        a = np.unique(rng.integers(0, 200, size=rng.integers(0, 80)))
        b = np.unique(rng.integers(0, 200, size=rng.integers(0, 80)))
        inter, union = len(np.intersect1d(a, b)), len(np.union1d(a, b))
        want = 1.0 if union == 0 else inter / union
        assert O.jaccard(a, b) == pytest.approx(want, rel=1e-15)
        assert O.jaccard(a, b) == O.jaccard(b, a)


@pytest.mark.parametrize("H,lam,total", [(4, 14, 8192.0), (8, 14, 4096.0 * 8), (7, 3, 1000.0)])
def test_group_budgets_closed_forms(H, lam, total):
    b = O.group_budgets(total, H, lam)
    assert b.sum() == pytest.approx(total, rel=1e-13)                    # Eq. 5
    assert b[-1] == pytest.approx(total / (lam * H), rel=1e-13)          # Eq. 6
    assert b[0] / b[-1] == pytest.approx(2 * lam - 1, rel=1e-12)         # follows from Eq. 6
    np.testing.assert_allclose(np.diff(b), np.diff(b)[0], rtol=1e-10)    # Eq. 7: arithmetic
