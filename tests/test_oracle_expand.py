"""Pins for the equal-growth expansion oracle (CPU only)."""
import json
import os

import numpy as np
import pytest
import scipy.special

import oracle
import ygg_workloads as wl


def _grow(seed, B, D, W, V, sigma=3.0, logits_fn=None):
    N = 1 + D * W
    parent = np.full((B, N), -7, np.int32)
    token = np.full((B, N), -7, np.int32)
    cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 5, 0.0
    margins, all_logits = [], []
    for d in range(1, D + 1):
        F = 1 if d == 1 else W
        if logits_fn:
            x = logits_fn(d, F)
        else:
            x = np.stack([wl.draft_logits(seed, d, F, V, sub=b) for b in range(B)]) * np.float32(sigma / 3.0)
        all_logits.append(x)
        margins.append(oracle.expand(D, W, d, x, parent, token, cum))
    return parent, token, cum, margins, all_logits


def _independent_step(x, cum_front, W):
    """Library log-softmax (scipy, float64) + numpy lexsort over every candidate."""
    F, V = x.shape
    s = cum_front.astype(np.float64)[:, None] + scipy.special.log_softmax(x.astype(np.float64), axis=1)
    flat = np.arange(F * V)
    order = np.lexsort((flat, -s.ravel()))[:W]
    return order // V, order % V, s.ravel()[order]


@pytest.mark.parametrize("B,D,W,V", [(1, 3, 4, 50), (3, 4, 5, 17), (2, 2, 8, 300)])
def test_matches_independent_sort_of_all_candidates(B, D, W, V):
    parent, token, cum, margins, logits = _grow(31, B, D, W, V)
    for b in range(B):
        for d in range(1, D + 1):
            base_prev = 0 if d == 1 else 1 + (d - 2) * W
            base = 1 + (d - 1) * W
            F = 1 if d == 1 else W
            p, v, s = _independent_step(logits[d - 1][b], cum[b, base_prev:base_prev + F], W)
            assert np.array_equal(parent[b, base:base + W], base_prev + p)
            assert np.array_equal(token[b, base:base + W], v)
            np.testing.assert_allclose(cum[b, base:base + W], s, rtol=0, atol=2e-6)
            assert margins[d - 1][b] > 1e-9   # well-conditioned seeds only


def test_structure_invariants():
    B, D, W, V = 2, 5, 6, 200
    parent, token, cum, _, _ = _grow(32, B, D, W, V)
    N = 1 + D * W
    for b in range(B):
        assert parent[b, 0] == -1
        for d in range(1, D + 1):
            base = 1 + (d - 1) * W
            lo = 0 if d == 1 else base - W
            hi = 0 if d == 1 else base - 1
            blk = slice(base, base + W)
            assert ((parent[b, blk] >= lo) & (parent[b, blk] <= hi)).all()      # exactly W nodes per depth
            assert len({(int(p), int(t)) for p, t in zip(parent[b, blk], token[b, blk])}) == W
            assert (np.diff(cum[b, blk]) <= 0).all()                             # emitted best first
        for i in range(1, N):
            assert cum[b, i] <= cum[b, parent[b, i]] <= 0.0                      # log-probs only decrease
        assert ((token[b] >= 0) & (token[b] < V)).all()


def test_width_one_is_the_greedy_chain():
    B, D, V = 2, 6, 40
    parent, token, cum, _, logits = _grow(33, B, D, 1, V)
    for b in range(B):
        run = 0.0
        for d in range(1, D + 1):
            x = logits[d - 1][b, 0].astype(np.float64)
            assert parent[b, d] == d - 1
            assert token[b, d] == int(np.argmax(x))
            run += x.max() - scipy.special.logsumexp(x)
            assert abs(cum[b, d] - run) < 1e-5


def test_scores_of_one_row_sum_to_the_parent_probability():
    F, V = 5, 1000
    x = wl.draft_logits(34, 2, F, V)
    cum_front = -np.abs(wl.rng(34, 99).standard_normal(F)).astype(np.float32)
    s = oracle.expand_scores(x, cum_front)
    np.testing.assert_allclose(np.exp(s).sum(1), np.exp(cum_front.astype(np.float64)), rtol=1e-12)
    # a constant shift of a row's logits changes nothing
    x2 = x.copy()
    x2[2] += np.float32(8.0)
    s2 = oracle.expand_scores(x2, cum_front)
    np.testing.assert_allclose(s2[2], s[2], atol=1e-5)   # (fp32 shift rounds the inputs)
    assert np.array_equal(s2[[0, 1, 3, 4]], s[[0, 1, 3, 4]])


def test_selected_set_is_a_threshold_set():
    D, W, V = 3, 4, 60
    parent, token, cum, _, logits = _grow(35, 1, D, W, V)
    for d in range(2, D + 1):
        base_prev, base = 1 + (d - 2) * W, 1 + (d - 1) * W
        s = oracle.expand_scores(logits[d - 1][0], cum[0, base_prev:base_prev + W].copy())
        chosen = np.zeros(s.shape, bool)
        chosen[parent[0, base:base + W] - base_prev, token[0, base:base + W]] = True
        assert chosen.sum() == W
        assert s[chosen].min() >= s[~chosen].max()


def test_ties_go_to_the_lower_flat_index():
    # depth 1: duplicated maxima inside one row
    V, W, D = 8, 3, 2
    row = np.array([[[1.0, 5.0, 5.0, 0.0, 5.0, 5.0, -1.0, 2.0]]], np.float32)
    def fn(d, F):
        if d == 1:
            return row
        # depth 2: identical rows under parents whose cum is identical -> equal scores across rows
        return np.tile(np.array([0.0, 3.0, 1.0, 3.0, 0.0, 0.0, 0.0, 0.0], np.float32), (1, F, 1))
    parent, token, cum, margins, _ = _grow(0, 1, D, W, V, logits_fn=fn)
    assert token[0, 1:4].tolist() == [1, 2, 4]
    assert cum[0, 1] == cum[0, 2] == cum[0, 3]
    assert parent[0, 4:7].tolist() == [1, 1, 2] and token[0, 4:7].tolist() == [1, 3, 1]
    assert margins[0][0] == 0.0 and margins[1][0] == 0.0


def test_handworked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "expand_handworked.json")))
    W, D = g["width"], g["depth"]
    def fn(d, F):
        if d == 1:
            return (np.log(np.array(g["step1_probs"])) + g["step1_shift"]).astype(np.float32)[None]
        return (np.log(np.array(g["step2_probs"])) + np.array(g["step2_shift"])[:, None]).astype(np.float32)[None]
    parent, token, cum, margins, _ = _grow(0, 1, D, W, g["vocab"], logits_fn=fn)
    assert parent[0].tolist() == g["expected_parent"]
    assert token[0, 1:].tolist() == g["expected_token_tail"]
    np.testing.assert_allclose(np.exp(cum[0].astype(np.float64)), g["expected_path_prob"], rtol=g["tolerance"])
    r = g["expected_margin_ratio_step2"]
    assert abs(margins[1][0] - np.log(r[0] / r[1])) < g["tolerance"]


def test_rejects_bad_depth():
    with pytest.raises(ValueError):
        oracle.expand(2, 2, 3, np.zeros((1, 2, 4), np.float32), np.zeros((1, 5), np.int32),
                      np.zeros((1, 5), np.int32), np.zeros((1, 5), np.float32))
