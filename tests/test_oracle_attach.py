"""Pins for the oracle of equal growth with free attachment (CPU only)."""
import json
import os

import numpy as np
import pytest
import scipy.special

import oracle
import ygg_workloads as wl


def _new_tree(B, D, W):
    N = 1 + D * W
    parent = np.full((B, N), -7, np.int32)
    token = np.full((B, N), -7, np.int32)
    cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 5, 0.0
    return parent, token, cum


def _rows(seed, t, B, F, V, sigma):
    return np.stack([wl.draft_logits(seed, t, F, V, sub=b) for b in range(B)]) * np.float32(sigma / 3.0)


def _grow(seed, B, D, W, V, sigma=3.0, logits_fn=None):
    parent, token, cum = _new_tree(B, D, W)
    pool = oracle.attach_pool(B, D, W)
    margins, logits, pools = [], [], []
    for t in range(1, D + 1):
        F = 1 if t == 1 else W
        x = logits_fn(t, F) if logits_fn else _rows(seed, t, B, F, V, sigma)
        logits.append(x)
        margins.append(oracle.attach(D, W, t, x, parent, token, cum, pool))
        pools.append({k: v.copy() for k, v in pool.items()})
    return parent, token, cum, margins, logits, pools


def _independent(logits, D, W, keep=None):
    """The definition again, from library pieces: scipy log-softmax, numpy argsort for the offers, Python's
    sorted() on tuples for the pool.  keep(t) optionally truncates the pool to its best keep(t) entries
    after step t.  One sequence; returns parent, token, score lists and the pool after every step."""
    V = logits[0].shape[-1]
    parent, token, score = [-1], [None], [0.0]
    cum32 = [np.float32(0.0)]
    pool, pools = [], []
    for t in range(1, D + 1):
        new_nodes = [0] if t == 1 else list(range(1 + (t - 2) * W, 1 + (t - 1) * W))
        for r, node in enumerate(new_nodes):
            x = logits[t - 1][r]
            lp = scipy.special.log_softmax(x.astype(np.float64))
            best = np.lexsort((np.arange(V), -x.astype(np.float64)))[:W]
            for v in best:
                pool.append((-(float(cum32[node]) + lp[v]), node * V + int(v)))
        pool = sorted(pool)
        for neg, flat in pool[:W]:
            parent.append(flat // V)
            token.append(flat % V)
            score.append(-neg)
            cum32.append(np.float32(-neg))
        pool = pool[W:]
        if keep is not None:
            pool = pool[:keep(t)]
        pools.append(list(pool))
    return parent, token, score, pools


@pytest.mark.parametrize("B,D,W,V,sigma", [(1, 3, 4, 50, 3.0), (3, 4, 5, 17, 1.0), (2, 5, 3, 300, 6.0), (1, 6, 2, 9, 0.3)])
def test_matches_independent_pool_of_all_offers(B, D, W, V, sigma):
    parent, token, cum, margins, logits, pools = _grow(41, B, D, W, V, sigma)
    for b in range(B):
        p, tk, s, ref_pools = _independent([x[b] for x in logits], D, W)
        assert np.array_equal(parent[b], p)
        assert np.array_equal(token[b, 1:], tk[1:])
        np.testing.assert_allclose(cum[b], s, rtol=0, atol=2e-6)
        for t in range(D):
            n = pools[t]["count"][b]
            assert n == len(ref_pools[t]) == t * W * (W - 1)   # offers W + t*W*W minus (t+1)*W taken
            assert [(int(a) * V + int(c)) for a, c in zip(pools[t]["node"][b, :n], pools[t]["token"][b, :n])] == \
                [flat for _, flat in ref_pools[t]]
            np.testing.assert_allclose(pools[t]["score"][b, :n], [-neg for neg, _ in ref_pools[t]], rtol=0, atol=1e-12)
        assert all(m[b] > 1e-9 for m in margins)


@pytest.mark.parametrize("sigma", [0.05, 1.0, 8.0])
def test_pool_may_be_cut_to_the_slots_still_to_fill(sigma):
    """An entry of rank r needs r // W more steps before it can be taken, and later offers only push it
    down: keeping the best W*(D-t) entries after step t changes nothing (the bounded device-side pool)."""
    D, W, V = 6, 3, 40
    for seed in range(5):
        logits = [_rows(100 + seed, t, 1, 1 if t == 1 else W, V, sigma)[0] for t in range(1, D + 1)]
        full = _independent(logits, D, W)
        cut = _independent(logits, D, W, keep=lambda t: W * (D - t))
        assert full[0] == cut[0] and full[1] == cut[1] and full[2] == cut[2]
        for t in range(D):
            assert cut[3][t] == full[3][t][:W * (D - t - 1)]


def test_structure_invariants_and_free_attachment():
    B, D, W, V = 2, 6, 4, 120
    parent, token, cum, _, _, pools = _grow(42, B, D, W, V, sigma=1.0)
    N = 1 + D * W
    older_parent = 0
    for b in range(B):
        assert parent[b, 0] == -1
        depth = np.zeros(N, np.int64)
        for i in range(1, N):
            step = (i - 1) // W + 1
            assert 0 <= parent[b, i] < 1 + (step - 1) * W          # a node of an earlier step
            depth[i] = depth[parent[b, i]] + 1
            assert depth[i] <= step
            assert cum[b, i] <= cum[b, parent[b, i]] + 1e-7          # log-probabilities only add negatives
            older_parent += int(step >= 2 and parent[b, i] < 1 + (step - 2) * W)
        for t in range(1, D + 1):
            sl = slice(1 + (t - 1) * W, 1 + t * W)
            assert np.all(np.diff(cum[b, sl]) <= 0)                  # selection order
            n = pools[t - 1]["count"][b]
            if n:
                assert pools[t - 1]["score"][b, 0] <= cum[b, sl][-1] + 1e-7   # nothing left behind beats a taken one
                assert np.all(np.diff(pools[t - 1]["score"][b, :n]) <= 0)
        pairs = {(int(parent[b, i]), int(token[b, i])) for i in range(1, N)}
        assert len(pairs) == N - 1                                   # no (parent, token) pair twice
    assert older_parent > 0   # with a flat drafter some leaves do hang under nodes older than the last step


def test_width_one_is_the_greedy_chain_and_equals_the_frontier_rule():
    B, D, W, V = 2, 5, 1, 64
    parent, token, cum, _, logits, pools = _grow(43, B, D, W, V)
    p2, t2, c2 = _new_tree(B, D, W)
    for d in range(1, D + 1):
        oracle.expand(D, W, d, logits[d - 1], p2, t2, c2)
    assert np.array_equal(parent, p2) and np.array_equal(token, t2) and np.array_equal(cum, c2)
    assert np.array_equal(parent[0], np.arange(-1, D))
    for b in range(B):
        for d in range(D):
            assert token[b, d + 1] == int(np.argmax(logits[d][b, 0]))
    assert all(np.all(pl["count"] == 0) for pl in pools)


def test_single_step_equals_the_frontier_rule():
    B, D, W, V = 3, 1, 6, 90
    parent, token, cum, _, logits, _ = _grow(44, B, D, W, V)
    p2, t2, c2 = _new_tree(B, D, W)
    oracle.expand(D, W, 1, logits[0], p2, t2, c2)
    assert np.array_equal(parent, p2) and np.array_equal(token, t2) and np.array_equal(cum, c2)


def test_equal_scores_go_to_the_lower_node_then_token():
    D, W, V = 2, 2, 6
    def fn(t, F):
        x = np.zeros((1, F, V), np.float32)   # uniform rows: every offer of a step has the same score
        return x
    parent, token, cum, margins, _, pools = _grow(0, 1, D, W, V, logits_fn=fn)
    assert list(token[0, 1:3]) == [0, 1]
    assert list(parent[0, 3:5]) == [1, 1] and list(token[0, 3:5]) == [0, 1]   # node 1's offers precede node 2's
    assert list(pools[1]["node"][0, :2]) == [2, 2] and list(pools[1]["token"][0, :2]) == [0, 1]
    assert margins[1][0] == 0.0


def test_handworked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "attach_handworked.json")))
    V, W, D = g["vocab"], g["width"], g["depth"]
    parent, token, cum = _new_tree(1, D, W)
    pool = oracle.attach_pool(1, D, W)
    for t in range(1, D + 1):
        x = np.log(np.array(g["step_probs"][t - 1], np.float64)).astype(np.float32)[None]
        oracle.attach(D, W, t, x, parent, token, cum, pool)
    assert list(parent[0]) == g["expected_parent"]
    assert list(token[0, 1:]) == g["expected_token_tail"]
    np.testing.assert_allclose(np.exp(cum[0].astype(np.float64)), g["expected_path_prob"], rtol=g["tolerance"])
    n = int(pool["count"][0])
    assert n == len(g["expected_pool_node"])
    assert list(pool["node"][0, :n]) == g["expected_pool_node"] and list(pool["token"][0, :n]) == g["expected_pool_token"]
    np.testing.assert_allclose(np.exp(pool["score"][0, :n]), g["expected_pool_prob"], rtol=g["tolerance"])


def test_rejects_bad_arguments_and_small_pools():
    parent, token, cum = _new_tree(1, 2, 2)
    pool = oracle.attach_pool(1, 2, 2)
    x = np.zeros((1, 1, 8), np.float32)
    with pytest.raises(ValueError):
        oracle.attach(2, 2, 3, np.zeros((1, 2, 8), np.float32), parent, token, cum, pool)   # step beyond D
    with pytest.raises(ValueError):
        oracle.attach(2, 9, 1, np.zeros((1, 1, 8), np.float32), *_new_tree(1, 2, 9), oracle.attach_pool(1, 2, 9))  # W > V
    small = {k: (v[:, :1].copy() if v.ndim == 2 else v.copy()) for k, v in pool.items()}
    with pytest.raises(ValueError):
        oracle.attach(2, 2, 1, x, parent, token, cum, small)           # pool cannot hold the root's offers
