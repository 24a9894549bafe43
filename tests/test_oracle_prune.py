"""Pins for the verification-width pruning oracle (CPU only)."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
import ygg_workloads as wl


def _brute(parent, value):
    """Every set of nodes that contains the root and is closed under 'parent of': best total by size, and the argmax sets."""
    N = len(parent)
    best = [-np.inf] * (N + 1)
    sets = [None] * (N + 1)
    best[0] = 0.0
    for mask in range(1, 1 << N, 2):            # odd masks contain node 0
        nodes = [i for i in range(N) if mask >> i & 1]
        if any(not (mask >> parent[i] & 1) for i in nodes if i):
            continue
        tot = float(sum(value[i] for i in nodes))
        k = len(nodes)
        if tot > best[k] + 1e-15:
            best[k], sets[k] = tot, [set(nodes)]
        elif abs(tot - best[k]) <= 1e-15:
            sets[k].append(set(nodes))
    return best, sets


def _is_valid(parent, keep, want):
    idx = np.flatnonzero(keep)
    return len(idx) == want and (want == 0 or (keep[0] and all(keep[parent[i]] for i in idx if i)))


@pytest.mark.parametrize("seed", range(8))
def test_dp_equals_enumeration_of_all_connected_sets(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(2, 13))
    parent = wl.random_topological_tree(seed, N).astype(np.int32)
    value = rng.random(N) ** 3 * (10.0 if seed % 2 else 1.0)     # arbitrary, not monotone along paths
    ref, sets = _brute(parent, value)
    for want in range(0, N + 1):
        best, keep = oracle.subtree_dp(parent, value, want)
        np.testing.assert_allclose(best, ref, rtol=0, atol=1e-12)
        assert _is_valid(parent, keep, want)
        assert abs(value[keep].sum() - ref[want]) <= 1e-12
        if want and len(sets[want]) == 1:
            assert set(np.flatnonzero(keep)) == sets[want][0]


def test_monotone_values_reduce_to_the_largest_values():
    """If a child is never worth more than its parent, the k most valuable nodes are already connected:
    the DP must agree with a plain sort (this is what the device kernel relies on)."""
    for seed in range(6):
        rng = np.random.default_rng(100 + seed)
        N = 60
        parent = wl.random_topological_tree(seed, N).astype(np.int32)
        value = np.ones(N)
        for i in range(1, N):
            value[i] = value[parent[i]] * rng.random()
        order = np.lexsort((np.arange(N), -value))
        for want in (1, 2, 7, 30, 59, 60):
            best, keep = oracle.subtree_dp(parent, value, want)
            assert set(np.flatnonzero(keep)) == set(order[:want])
            np.testing.assert_allclose(best[1:], np.cumsum(value[order]), rtol=1e-13)


def test_chain_and_star():
    N = 9
    chain = wl.chain_tree(N).astype(np.int32)
    v = np.array([1, 9, 1, 9, 1, 9, 1, 9, 1], np.float64)
    best, keep = oracle.subtree_dp(chain, v, 4)
    assert list(np.flatnonzero(keep)) == [0, 1, 2, 3]                 # a chain can only keep a prefix
    np.testing.assert_allclose(best, np.concatenate([[0], np.cumsum(v)]))
    star = np.array([-1] + [0] * (N - 1), np.int32)
    best, keep = oracle.subtree_dp(star, v, 4)
    assert keep[0] and keep.sum() == 4 and v[keep].sum() == 1 + 27      # the root and the three best leaves


def _grown(cfg_seed, B, D, W, V, sigma):
    N = 1 + D * W
    parent = np.full((B, N), -1, np.int32); token = np.zeros((B, N), np.int32); cum = np.zeros((B, N), np.float32)
    pool = oracle.attach_pool(B, D, W)
    for t in range(1, D + 1):
        F = 1 if t == 1 else W
        x = np.stack([wl.draft_logits(cfg_seed, t, F, V, sub=b) for b in range(B)]) * np.float32(sigma / 3.0)
        oracle.attach(D, W, t, x, parent, token, cum, pool)
    return parent, token, cum


def test_prune_outputs_are_a_renumbered_subtree():
    B, D, W, V = 3, 5, 4, 200
    parent, token, cum = _grown(7, B, D, W, V, 1.0)
    N = 1 + D * W
    t_ver = np.concatenate([[0.0], np.where(np.arange(1, N + 1) <= 8, 1.0, 1.0 + 0.2 * (np.arange(1, N + 1) - 8))])
    for w in (1, 5, 12, N):
        r = oracle.prune(w, parent, token, cum, t_ver, 0.5)
        for b in range(B):
            kept = r["kept_nodes"][b]
            assert kept[0] == 0 and np.all(np.diff(kept) > 0)
            assert r["new_parent"][b, 0] == -1
            for k in range(1, w):
                assert kept[r["new_parent"][b, k]] == parent[b, kept[k]]     # same edges, new numbers
                assert r["new_parent"][b, k] < k
            assert np.array_equal(r["new_token"][b], token[b, kept])
            p = np.exp(cum[b].astype(np.float64))
            np.testing.assert_allclose(r["expected_len"][b], p[kept].sum(), rtol=1e-13)
            # path probabilities shrink along every path: the kept set is the w most probable nodes
            assert p[kept].min() >= np.delete(p, kept).max(initial=0.0) - 1e-15
            obj = r["best_curve"][b, 1:] / (0.5 + t_ver[1:])
            assert r["best_width"][b] == 1 + int(np.argmax(obj))
            np.testing.assert_allclose(r["best_curve"][b, 1:], np.cumsum(np.sort(p)[::-1]), rtol=1e-13)


def test_best_width_follows_the_verifier_latency_curve():
    """Flat verifier latency -> verify everything; latency growing faster than the expected length -> verify little."""
    parent, token, cum = _grown(9, 1, 4, 4, 100, 1.0)
    N = parent.shape[1]
    flat = np.concatenate([[0.0], np.ones(N)])
    steep = np.concatenate([[0.0], 1.0 + 10.0 * np.arange(N)])
    assert oracle.prune(3, parent, token, cum, flat, 1.0)["best_width"][0] == N
    assert oracle.prune(3, parent, token, cum, steep, 1.0)["best_width"][0] == 1


def test_handworked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "prune_handworked.json")))
    parent = np.array(g["parent"], np.int32)
    N = len(parent)
    best, keep = oracle.subtree_dp(parent, np.array(g["general_values"]), 4)
    np.testing.assert_allclose(best, g["general_best"], atol=g["tolerance"])
    assert list(np.flatnonzero(keep)) == g["general_keep4"]
    best, _ = oracle.subtree_dp(parent, np.array(g["path_prob"]), 3)
    np.testing.assert_allclose(best, g["path_best"], atol=g["tolerance"])
    cum = np.log(np.array(g["path_prob"])).astype(np.float32)[None]
    token = np.arange(10, 10 + N, dtype=np.int32)[None]
    r = oracle.prune(5, parent[None], token, cum, np.array(g["t_verifier"]), g["t_draft"])
    assert list(r["kept_nodes"][0]) == g["keep5_nodes"] and list(r["new_parent"][0]) == g["keep5_new_parent"]
    assert list(r["new_token"][0]) == [10 + i for i in g["keep5_nodes"]]
    assert r["best_width"][0] == g["expected_best_width"]
    np.testing.assert_allclose(r["expected_len"][0], g["path_best"][5], rtol=1e-6)


def test_rejects_bad_trees():
    with pytest.raises(ValueError):
        oracle.subtree_dp(np.array([-1, 1, 0], np.int32), np.ones(3), 2)     # parent[1] = 1 is not an earlier node
    with pytest.raises(ValueError):
        oracle.subtree_dp(np.array([-1, 0], np.int32), np.ones(2), 3)        # more nodes wanted than there are
