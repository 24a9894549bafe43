"""Pins for the greedy acceptance + K/V compaction oracle (CPU only)."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
import ygg_workloads as wl


def _kv(seed, layers, B, N, cap, Hkv=2, Dh=4, dtype="bf16"):
    mk = lambda s, n: wl.normal(seed, s, (layers, B, n, Hkv, Dh), dtype)
    return mk(5, N), mk(6, N), mk(3, cap), mk(4, cap)


def _enumerate_paths(parent, token, tstar):
    """Every root->node path, independently: a path is accepted if each edge's child token equals
    the verifier's token at the edge's parent.  Returns the longest, lowest last index on ties."""
    N = len(parent)
    best = [0]
    for i in range(N):
        path, a = [], i
        while a != -1:
            path.append(a)
            a = parent[a]
        path = path[::-1]
        ok = all(token[c] == tstar[p] for p, c in zip(path[:-1], path[1:]))
        if ok and len(path) > len(best):
            best = path
    return best


@pytest.mark.parametrize("seed", range(6))
def test_matches_enumeration_of_all_paths(seed):
    B, D, W, V, layers = 3, 4, 3, 12, 2
    N = 1 + D * W
    parent = np.stack([wl.level_tree(40 + seed, D, W, "dirichlet", 0.5, sub=b) for b in range(B)])
    token = np.stack([wl.node_tokens(40 + seed, parent[b], V, sub=b) for b in range(B)])
    logits = np.stack([wl.target_logits(40 + seed, parent[b], token[b], V, 0.8, sub=b) for b in range(B)])
    lens = np.array([3, 0, 5], np.int32)
    cap = 5 + D + 1
    kt, vt, kc, vc = _kv(seed, layers, B, N, cap)
    kc0, vc0, lens0 = kc.copy(), vc.copy(), lens.copy()
    r = oracle.accept_compact(D + 1, parent, token, kt, vt, kc, vc, lens, target_logits=logits)
    for b in range(B):
        tstar = logits[b].argmax(1)                      # numpy argmax: first maximum
        assert np.array_equal(r["tstar"][b], tstar)
        path = _enumerate_paths(parent[b].tolist(), token[b].tolist(), tstar.tolist())
        n = len(path)
        assert r["accept_len"][b] == n and 1 <= n <= D + 1
        assert r["accept_path"][b, :n].tolist() == path and (r["accept_path"][b, n:] == -1).all()
        assert r["bonus_token"][b] == tstar[path[-1]]
        # maximality: no child of the last accepted node carries the bonus token
        kids = np.nonzero(parent[b] == path[-1])[0]
        assert not any(token[b, k] == r["bonus_token"][b] for k in kids)
        assert lens[b] == lens0[b] + n
        for layer in range(layers):
            L = lens0[b]
            assert np.array_equal(kc[layer, b, L:L + n], kt[layer, b, path])
            assert np.array_equal(vc[layer, b, L:L + n], vt[layer, b, path])
            assert np.array_equal(kc[layer, b, :L], kc0[layer, b, :L]) and np.array_equal(kc[layer, b, L + n:], kc0[layer, b, L + n:])
            assert np.array_equal(vc[layer, b, :L], vc0[layer, b, :L]) and np.array_equal(vc[layer, b, L + n:], vc0[layer, b, L + n:])
    assert any(r["accept_len"] > 1)


def test_full_agreement_on_a_chain_accepts_everything_and_none_accepts_root_only():
    D, V = 5, 30
    N = D + 1
    parent = wl.chain_tree(N)[None]
    token = np.arange(10, 10 + N, dtype=np.int32)[None]
    kt, vt, kc, vc = _kv(1, 1, 1, N, 20, dtype="f32")
    tstar = np.concatenate([token[0, 1:], [3]]).astype(np.int32)[None]
    lens = np.array([7], np.int32)
    r = oracle.accept_compact(N, parent, token, kt, vt, kc, vc, lens, target_tokens=tstar)
    assert r["accept_len"][0] == D + 1 and r["accept_path"][0].tolist() == list(range(N)) and r["bonus_token"][0] == 3
    assert lens[0] == 7 + N and np.array_equal(kc[0, 0, 7:7 + N], kt[0, 0])
    lens = np.array([7], np.int32)
    r = oracle.accept_compact(N, parent, token, kt, vt, kc, vc, lens, target_tokens=np.full((1, N), 29, np.int32))
    assert r["accept_len"][0] == 1 and r["accept_path"][0].tolist() == [0] + [-1] * D and r["bonus_token"][0] == 29


def test_argmax_takes_the_first_maximum():
    parent = np.array([[-1, 0, 0]], np.int32)
    token = np.array([[0, 4, 2]], np.int32)
    x = np.zeros((1, 3, 6), np.float32)
    x[0, 0, [2, 4]] = 9.0          # tie between tokens 2 and 4 -> 2, so node 2 matches, node 1 does not
    x[0, 2, [5, 1]] = 1.0          # bonus after node 2: first maximum is 1
    kt, vt, kc, vc = _kv(2, 1, 1, 3, 6)
    r = oracle.accept_compact(2, parent, token, kt, vt, kc, vc, np.array([1], np.int32), target_logits=x)
    assert r["tstar"][0].tolist() == [2, 0, 1]
    assert r["accept_path"][0].tolist() == [0, 2] and r["bonus_token"][0] == 1


def test_equal_depth_matches_resolve_to_lower_index():
    # two children of the root with the same token (hand-made; the generator never does this)
    parent = np.array([[-1, 0, 0, 1, 2]], np.int32)
    token = np.array([[1, 7, 7, 8, 8]], np.int32)
    tstar = np.array([[7, 8, 8, 0, 0]], np.int32)
    kt, vt, kc, vc = _kv(3, 1, 1, 5, 8)
    r = oracle.accept_compact(3, parent, token, kt, vt, kc, vc, np.array([0], np.int32), target_tokens=tstar)
    assert r["accept_path"][0].tolist() == [0, 1, 3]


def test_general_topological_tree_and_capacity_errors():
    parent = wl.random_topological_tree(44, 12)[None]
    token = wl.node_tokens(44, parent[0], 9)[None]
    tstar = wl.rng(44, 77).integers(0, 9, size=(1, 12)).astype(np.int32)
    kt, vt, kc, vc = _kv(4, 1, 1, 12, 16)
    r = oracle.accept_compact(12, parent, token, kt, vt, kc, vc, np.array([2], np.int32), target_tokens=tstar)
    path = _enumerate_paths(parent[0].tolist(), token[0].tolist(), tstar[0].tolist())
    assert r["accept_path"][0, :len(path)].tolist() == path
    with pytest.raises(ValueError):   # cache too small for the accepted path
        oracle.accept_compact(12, parent, token, kt, vt, kc, vc, np.array([16], np.int32), target_tokens=tstar)
    with pytest.raises(ValueError):   # both or neither target given
        oracle.accept_compact(12, parent, token, kt, vt, kc, vc, np.array([0], np.int32))


def test_handworked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "accept_handworked.json")))
    parent = np.array([g["parent_idx"]], np.int32)
    token = np.array([g["token_ids"]], np.int32)
    tstar = np.array([g["target_tokens"]], np.int32)
    N = parent.shape[1]
    kt, vt, kc, vc = _kv(5, 1, 1, N, 10)
    lens = np.array([4], np.int32)
    r = oracle.accept_compact(g["path_cols"], parent, token, kt, vt, kc, vc, lens, target_tokens=tstar)
    assert r["accept_len"][0] == g["expected_accept_len"]
    assert r["accept_path"][0].tolist() == g["expected_path"]
    assert r["bonus_token"][0] == g["expected_bonus"]
    assert lens[0] == 4 + g["expected_accept_len"]
    assert np.array_equal(kc[0, 0, 4:7], kt[0, 0, [0, 1, 4]])
