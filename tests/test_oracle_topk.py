"""Pins of the oracle's fixed-budget thresholds (CPU only)."""
import itertools

import numpy as np
import pytest

from oracle import kvzap_oracle as O


def _kept_nonwindow(S, tau, w):
    res = O.prune(S, tau, w)
    B, H, T = S.shape
    return [[set(int(t) for t in res.idx[b][h] if t < T - w) for h in range(H)] for b in range(B)]


def test_per_head_topk_equals_an_argsort_topk_when_scores_are_distinct():
    rng = np.random.default_rng(0)
    B, H, T, w = 2, 3, 200, 16
    S = rng.standard_normal((B, H, T))
    for k in (1, 7, 50, 183):
        tau = O.topk_threshold(S, w, k, per_layer=False)
        kept = _kept_nonwindow(S, tau, w)
        for b in range(B):
            for h in range(H):
                want = set(np.argsort(-S[b, h, :T - w], kind="stable")[:k].tolist())
                assert kept[b][h] == want and len(want) == k


def test_per_layer_topk_shares_one_budget_across_heads():
    rng = np.random.default_rng(1)
    B, H, T, w, k = 2, 4, 120, 8, 150
    S = rng.standard_normal((B, H, T)) * np.array([0.5, 1.0, 2.0, 4.0])[None, :, None]
    tau = O.topk_threshold(S, w, k, per_layer=True)
    assert (tau == tau[:, :1]).all()                      # one threshold per sequence
    kept = _kept_nonwindow(S, tau, w)
    for b in range(B):
        sizes = [len(x) for x in kept[b]]
        assert sum(sizes) == k                            # the budget, exactly (no ties)
        flat = S[b, :, :T - w]
        kept_vals = np.concatenate([flat[h, sorted(kept[b][h])] for h in range(H)])
        mask = np.ones(flat.shape, bool)
        for h in range(H):
            mask[h, sorted(kept[b][h])] = False
        assert kept_vals.min() > flat[mask].max()         # every kept score beats every dropped one
        assert sizes[3] > sizes[0]                        # the wide head takes more of the budget


def test_limits_window_and_padding():
    rng = np.random.default_rng(2)
    S = rng.standard_normal((2, 2, 40))
    assert np.isposinf(O.topk_threshold(S, 8, 0, False)).all()
    assert np.isneginf(O.topk_threshold(S, 8, 32, False)).all()       # population is 32
    assert np.isneginf(O.topk_threshold(S, 8, 64, True)).all()        # pooled: 64
    assert np.isfinite(O.topk_threshold(S, 8, 63, True)).all()
    assert np.isneginf(O.topk_threshold(S, 50, 1, False)).all()       # window covers everything
    # k = 0 keeps exactly the window, k >= population keeps everything
    r0 = O.prune(S, O.topk_threshold(S, 8, 0, False), 8)
    assert (r0.lengths == 8).all()
    rall = O.prune(S, O.topk_threshold(S, 8, 32, False), 8)
    assert (rall.lengths == 40).all()
    # right-padded batch: the population ends at T_b - window
    tau = O.topk_threshold(S, 8, 5, False, seq_lens=[40, 20])
    want = np.sort(S[1, 0, :12])[::-1][4]
    assert tau[1, 0] == want
    res = O.prune(S, tau, 8, seq_lens=[40, 20])
    assert res.lengths[1].tolist() == [13, 13]


def test_ties_and_nan():
    S = np.array([[[3.0, 1.0, 3.0, np.nan, 2.0, 3.0, 0.0, 9.0, 9.0]]])     # window = last 2
    tau = O.topk_threshold(S, 2, 2, False)
    assert tau[0, 0] == 3.0
    kept = _kept_nonwindow(S, tau, 2)[0][0]
    assert kept == {0, 2, 5}                              # all three tied entries, not two
    assert np.isneginf(O.topk_threshold(S, 2, 6, False)[0, 0])    # 6 non-NaN entries
    res = O.prune(S, O.topk_threshold(S, 2, 6, False), 2)
    assert 3 not in res.idx[0][0]                         # NaN is never kept outside the window


def test_nested_in_k_and_brute_force():
    rng = np.random.default_rng(3)
    S = rng.standard_normal((1, 2, 9))
    w = 2
    prev = None
    for k in range(0, 9):
        kept = _kept_nonwindow(S, O.topk_threshold(S, w, k, False), w)[0]
        if prev is not None:
            assert all(prev[h] <= kept[h] for h in range(2))
        prev = kept
        # brute force: among all subsets of size min(k, 7) of a head's 7 non-window positions,
        # the kept set is the one with the largest score sum
        for h in range(2):
            kk = min(k, 7)
            best = max(itertools.combinations(range(7), kk), key=lambda c: S[0, h, list(c)].sum())
            assert kept[h] == set(best)


def test_scalar_threshold_behaviour_is_unchanged_by_the_array_form():
    rng = np.random.default_rng(4)
    S = rng.standard_normal((2, 3, 50))
    a = O.prune(S, 0.1, 5)
    b = O.prune(S, np.full((2, 3), 0.1), 5)
    assert (a.lengths == b.lengths).all()
    assert all(np.array_equal(x, y) for ra, rb in zip(a.idx, b.idx) for x, y in zip(ra, rb))
