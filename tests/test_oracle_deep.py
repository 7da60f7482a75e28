"""Pins for the eviction-path oracle against closed forms, library routines,
brute force and invariants (no GPU, no HIP library)."""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

SCALE = 1.0 / np.sqrt(128.0)


def test_single_query_is_textbook_softmax(oracle):
    # h_n = l_w = 1, no divisor: the score of context key a is the softmax weight of
    # the one window query (last position, sees every key) on a (Eq. 1).
    rng = np.random.default_rng(1)
    l, d = 97, 128
    K = rng.standard_normal((l, d))
    q = rng.standard_normal((1, 1, d))
    got = oracle.deep_scores(q, K, SCALE, norm_mode=1)
    want = sp_softmax((K @ q[0, 0]) * SCALE)[: l - 1]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)


def test_zero_queries_closed_form(oracle):
    # Q = 0: every visible key gets weight 1/(p+1) for the query at position p, so
    # ac'_a = sum_b 1/(l_c+b+1) / (l-a)  (Eq. 1-3).
    l, lw, hn, d = 200, 8, 4, 16
    rng = np.random.default_rng(2)
    K = rng.standard_normal((l, d))
    Q = np.zeros((hn, lw, d))
    lc = l - lw
    h = sum(1.0 / (lc + b + 1) for b in range(lw))
    got = oracle.deep_scores(Q, K, 0.3, norm_mode=0)
    np.testing.assert_allclose(got, h / (l - np.arange(lc)), rtol=1e-13)
    got1 = oracle.deep_scores(Q, K, 0.3, norm_mode=1)
    np.testing.assert_allclose(got1, np.full(lc, h), rtol=1e-13)
    # paper divisor favours late tokens: top-k = the last k context tokens, then the window
    _, kept = oracle.deep_unit(Q, K, 0.3, P=1, budget=lw + 10, norm_mode=0)
    assert kept.tolist() == list(range(lc - 10, l))
    # without the divisor all tie -> lowest indices first
    _, kept = oracle.deep_unit(Q, K, 0.3, P=1, budget=lw + 10, norm_mode=1)
    assert kept.tolist() == list(range(10)) + list(range(lc, l))


def test_attention_mass_and_causal_mask(oracle):
    # Every softmax row sums to 1; with the plain window sum the context scores of one
    # head add up to l_w minus the mass the window queries put on window keys.  A dense
    # numpy/scipy evaluation with an explicit mask matrix gives the reference.
    rng = np.random.default_rng(3)
    l, lw, d = 60, 5, 32
    K = rng.standard_normal((l, d))
    Q = rng.standard_normal((1, lw, d))
    lc = l - lw
    logits = (Q[0] @ K.T) * 0.2
    pos = lc + np.arange(lw)[:, None]
    logits = np.where(np.arange(l)[None, :] <= pos, logits, -np.inf)
    A = sp_softmax(logits, axis=1)
    got = oracle.deep_scores(Q, K, 0.2, norm_mode=1)
    np.testing.assert_allclose(got, A[:, :lc].sum(0), rtol=1e-12)
    assert abs(got.sum() + A[:, lc:].sum() - lw) < 1e-12
    got0 = oracle.deep_scores(Q, K, 0.2, norm_mode=0)
    np.testing.assert_allclose(got0, A[:, :lc].sum(0) / (l - np.arange(lc)), rtol=1e-12)


def test_group_mean_is_mean_of_single_heads(oracle):
    # Eq. 3 is linear in the heads: the group score is the mean of the one-head scores,
    # with query head g of the group at index g (head h_n*i+g of the model).
    rng = np.random.default_rng(4)
    l, lw, hn, d = 80, 6, 4, 24
    K = rng.standard_normal((l, d))
    Q = rng.standard_normal((hn, lw, d))
    got = oracle.deep_scores(Q, K, 0.25)
    singles = [oracle.deep_scores(Q[g:g + 1], K, 0.25) for g in range(hn)]
    np.testing.assert_allclose(got, np.mean(singles, axis=0), rtol=1e-13)
    same = oracle.deep_scores(np.repeat(Q[:1], hn, axis=0), K, 0.25)
    np.testing.assert_allclose(same, singles[0], rtol=1e-13)


def test_scores_invariant_to_key_shift_along_query(oracle):
    # softmax is shift invariant: adding c*q/|q|^2 ... to every key adds the same
    # constant to a row's logits only if all rows share q; use one query row.
    rng = np.random.default_rng(5)
    l, d = 50, 16
    K = rng.standard_normal((l, d))
    q = rng.standard_normal((1, 1, d))
    base = oracle.deep_scores(q, K, 0.5, norm_mode=1)
    shifted = oracle.deep_scores(q, K + 3.0 * q[0, 0] / (q[0, 0] @ q[0, 0]), 0.5, norm_mode=1)
    np.testing.assert_allclose(base, shifted, rtol=1e-10)


def test_maxpool(oracle):
    x = np.array([1, 5, 2, 0, 0, 0, 0, 3], dtype=np.float64)
    assert oracle.maxpool(x, 3).tolist() == [5, 5, 5, 2, 0, 0, 3, 3]
    assert oracle.maxpool(x, 1).tolist() == x.tolist()
    rng = np.random.default_rng(6)
    for n, P in [(1, 7), (3, 7), (50, 7), (64, 15), (33, 5)]:
        x = rng.standard_normal(n)
        r = (P - 1) // 2
        padded = np.concatenate([np.full(r, -np.inf), x, np.full(r, -np.inf)])
        want = np.lib.stride_tricks.sliding_window_view(padded, P).max(axis=1)
        got = oracle.maxpool(x, P)
        assert np.array_equal(got, want)
        assert np.all(got >= x)
    assert np.array_equal(oracle.maxpool(np.full(9, 2.5), 7), np.full(9, 2.5))


def test_topk_bruteforce_and_ties(oracle):
    rng = np.random.default_rng(7)
    for n, k in [(1, 1), (10, 0), (10, 10), (100, 17), (257, 64)]:
        p = rng.standard_normal(n)
        p[rng.integers(0, n, size=n // 3)] = 0.5          # many exact ties
        want = np.sort(np.lexsort((np.arange(n), -p))[:k])
        assert np.array_equal(oracle.topk(p, k), want)
    # all equal -> lowest indices
    assert oracle.topk(np.ones(20), 5).tolist() == [0, 1, 2, 3, 4]
    # plateau of pooled values at the boundary: lowest indices of the plateau win
    p = np.array([0.1, 0.9, 0.9, 0.9, 0.9, 0.2, 1.0, 0.05])
    assert oracle.topk(p, 3).tolist() == [1, 2, 6]


def test_deep_unit_invariants(oracle):
    rng = np.random.default_rng(8)
    l, lw, hn, d = 300, 16, 4, 128
    K = rng.standard_normal((l, d))
    Q = rng.standard_normal((hn, lw, d))
    lc = l - lw
    for budget in [lw, lw + 1, 64, l - 1, l, l + 50]:
        pooled, kept = oracle.deep_unit(Q, K, SCALE, P=7, budget=budget)
        assert len(kept) == min(budget, l)                       # kept count == budget
        assert np.all(np.diff(kept) > 0)                         # ascending, unique
        assert kept[-lw:].tolist() == list(range(lc, l))         # whole window kept
        ctx = kept[:-lw]
        out = np.setdiff1d(np.arange(lc), ctx)
        if len(ctx) and len(out):
            assert pooled[ctx].min() >= pooled[out].max()
            t = pooled[ctx].min()
            tied_in = ctx[pooled[ctx] == t]
            tied_out = out[pooled[out] == t]
            if len(tied_in) and len(tied_out):
                assert tied_in.max() < tied_out.min()            # ties: lowest index first
    with pytest.raises(ValueError):
        oracle.deep_unit(Q, K, SCALE, P=7, budget=lw - 1)


def test_layer_ratio_pins(oracle):
    # alpha printed as 0.525 for beta 0.05; mean over layers equals r_c; at r_c = alpha
    # both cases of Eq. 5 give the endpoints (1, beta).
    gold = dict(line.split() for line in open(__file__.rsplit("/", 1)[0] + "/golden/hyperparameters.txt")
                if line.strip() and not line.startswith("#"))
    beta, alpha = float(gold["beta"]), float(gold["alpha"])
    assert abs((1 + beta) / 2 - alpha) < 1e-15
    l, lw, m = 8192, 32, 32
    lc = l - lw
    for rc in [0.1, 0.3, alpha, 0.6, 0.9, 1.0]:
        r = (rc * lc + lw) / l
        out = oracle.layer_ratios(r, l, lw, m, beta)
        assert abs(out.mean() - rc) < 1e-12
        assert np.all(np.diff(out) <= 1e-15)
        assert out.min() >= beta - 1e-12 and out.max() <= 1 + 1e-12
    r = (alpha * lc + lw) / l
    out = oracle.layer_ratios(r, l, lw, m, beta)
    assert abs(out[0] - 1.0) < 1e-12 and abs(out[-1] - beta) < 1e-12
    just_above = oracle.layer_ratios(((alpha + 1e-9) * lc + lw) / l, l, lw, m, beta)
    assert abs(just_above[0] - 1.0) < 1e-6 and abs(just_above[-1] - beta) < 1e-6


def test_layer_budget_pins(oracle):
    # Eq. 7 by hand: l_c = 1000, window 32, three layers, r_c = 0.3007 (between beta and alpha):
    # r_c(0) = 2 r_c - beta = 0.5514, r_c(2) = beta = 0.05, r_c(1) = their mean 0.3007
    # -> k = floor(551.4), floor(300.7), floor(50.0 +- an ulp); the window is added to each
    l, lw, m, beta = 1032, 32, 3, 0.05
    r = (0.3007 * 1000 + lw) / l
    b = oracle.layer_budgets(r, l, lw, m, beta)
    assert b[0] == 32 + 551 and b[1] == 32 + 300 and b[2] in (32 + 49, 32 + 50)
    # above alpha: r_c = 0.8004 -> r_c(0) = 1, r_c(2) = 0.6008, r_c(1) = 0.8004 -> 1000, 800, 600
    b = oracle.layer_budgets((0.8004 * 1000 + lw) / l, l, lw, m, beta)
    assert b[0] in (32 + 999, 32 + 1000) and b[1] == 32 + 800 and b[2] == 32 + 600
    # r = 1 keeps everything in every layer; one layer gets the mean
    assert np.array_equal(oracle.layer_budgets(1.0, 5000, 64, 7, beta), np.full(7, 5000))
    assert oracle.layer_budgets((0.25 * 900 + 100.5) / 1000, 1000, 100, 1, beta)[0] == 100 + 225
    # beta = 0: the last layer keeps the window alone, never less (the printed Eq. 6 in doubles
    # ends an ulp below zero for these arguments)
    b = oracle.layer_budgets(0.33344103305169476, 52801, 92, 19, 0.0)
    assert b[-1] == 92 and b.min() == 92
    # floor never exceeds the share: the budgets sum to at most the requested total
    for rc in (0.07, 0.31, 0.77):
        b = oracle.layer_budgets((rc * 8160 + 32) / 8192, 8192, 32, 32, beta)
        want = 32 * (rc * 8160 + 32)
        assert want - 32 - 1e-6 <= b.sum() <= want + 1e-6
