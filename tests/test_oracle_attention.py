"""Pins for the attention oracle (CPU only).

Each test checks the fp64 oracle against something other than itself: a hand-worked
fixture, closed forms, a library routine (torch SDPA in float64), or an independent
sequential per-path implementation written here in numpy.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import ygg_workloads as wl


def _case(seed, B=2, N=9, Hq=4, Hkv=2, Dh=8, L=(5, 11), dtype="f32", tree="random", scale=0.37):
    """Small random attention problem.  Returns dict of arrays + scale."""
    cap = max(L) + 3
    def nrm(stream, shape):
        return wl.normal(seed, stream, shape, dtype)
    if tree == "chain":
        parent = np.stack([wl.chain_tree(N) for _ in range(B)])
    elif tree == "level":
        W = (N - 1) // 2
        assert 1 + 2 * W == N
        parent = np.stack([wl.level_tree(seed, 2, W, "uniform", 0.0, sub=b) for b in range(B)])
    else:
        parent = np.stack([wl.random_topological_tree(seed, N, sub=b) for b in range(B)])
    return dict(q=nrm(2, (B, N, Hq, Dh)), k_cache=nrm(3, (B, cap, Hkv, Dh)), v_cache=nrm(4, (B, cap, Hkv, Dh)),
                k_tree=nrm(5, (B, N, Hkv, Dh)), v_tree=nrm(6, (B, N, Hkv, Dh)),
                seq_lens=np.array(L[:B], np.int32), parent_idx=parent, scale=scale)


def _run(c):
    return oracle.tree_attention(c["q"], c["k_cache"], c["v_cache"], c["seq_lens"], c["k_tree"], c["v_tree"],
                                 c["parent_idx"], c["scale"])


def _sequential_path_attention(c, b, i, h):
    """Independent statement: lay the prefix and the root->i path out as one ordinary sequence and
    run plain single-query softmax attention for its last token."""
    f = wl.storage_to_f64
    Hq, Hkv = c["q"].shape[2], c["k_tree"].shape[2]
    kv = h // (Hq // Hkv)
    L = int(c["seq_lens"][b])
    path = []
    a = i
    while a != -1:
        path.append(a)
        a = int(c["parent_idx"][b, a])
    path = path[::-1]
    K = np.concatenate([f(c["k_cache"][b, :L, kv]), f(c["k_tree"][b, path, kv])], axis=0)
    V = np.concatenate([f(c["v_cache"][b, :L, kv]), f(c["v_tree"][b, path, kv])], axis=0)
    qv = f(c["q"][b, i, h])
    s = (K @ qv) * np.float64(c["scale"])
    w = np.exp(s - s.max())
    return (w / w.sum()) @ V, s.max() + np.log(w.sum())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("tree", ["random", "level", "chain"])
def test_each_node_equals_sequential_attention_along_its_path(dtype, tree):
    c = _case(11, dtype=dtype, tree=tree)
    out, lse = _run(c)
    B, N, Hq, _ = c["q"].shape
    for b in range(B):
        for i in range(N):
            for h in range(Hq):
                ref, ref_lse = _sequential_path_attention(c, b, i, h)
                np.testing.assert_allclose(out[b, i, h], ref, rtol=0, atol=1e-12)
                assert abs(lse[b, i, h] - ref_lse) < 1e-12


def test_row_function_matches_full_function():
    c = _case(12, B=2, N=7, Hq=6, Hkv=2)
    out, lse = _run(c)
    for (b, i, h) in [(0, 0, 0), (1, 6, 5), (0, 3, 4)]:
        row, l, _ = oracle.attention_row(c["q"], c["k_cache"], c["v_cache"], c["seq_lens"], c["k_tree"],
                                         c["v_tree"], c["parent_idx"], c["scale"], b, i, h)
        assert np.array_equal(row, out[b, i, h]) and l == lse[b, i, h]


@pytest.mark.parametrize("G", [1, 4])
def test_width_one_tree_is_causal_attention_library_routine(G):
    """W = 1: the tree is a chain, so the N tree queries are the last N positions of an ordinary
    causal sequence of length L+N.  Checked against torch's SDPA (float64, explicit mask)."""
    Hkv, N, L, Dh = 2, 6, 10, 16
    c = _case(13, B=1, N=N, Hq=Hkv * G, Hkv=Hkv, Dh=Dh, L=(L,), tree="chain", scale=1.0 / np.sqrt(Dh))
    out, _ = _run(c)
    f = wl.storage_to_f64
    K = torch.from_numpy(np.concatenate([f(c["k_cache"][0, :L]), f(c["k_tree"][0])], 0))  # [L+N,Hkv,Dh]
    V = torch.from_numpy(np.concatenate([f(c["v_cache"][0, :L]), f(c["v_tree"][0])], 0))
    Q = torch.from_numpy(f(c["q"][0]))                                                     # [N,Hq,Dh]
    K = K.permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    V = V.permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    Q = Q.permute(1, 0, 2)[None]
    mask = torch.ones(N, L + N, dtype=torch.bool).tril(diagonal=L)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask, scale=float(c["scale"]))
    ref = ref[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out[0], ref, rtol=0, atol=1e-12)


def test_probabilities_sum_to_one_and_mask_is_ancestors_only():
    c = _case(14, B=2, N=12, L=(7, 3))
    for b in range(2):
        L = int(c["seq_lens"][b])
        for i in range(12):
            _, _, p = oracle.attention_row(c["q"], c["k_cache"], c["v_cache"], c["seq_lens"], c["k_tree"],
                                           c["v_tree"], c["parent_idx"], c["scale"], b, i, 1, want_probs=True)
            assert abs(p.sum() - 1.0) < 1e-14
            anc = set()
            a = i
            while a != -1:
                anc.add(a)
                a = int(c["parent_idx"][b, a])
            for t in range(12):
                assert (p[L + t] > 0) == (t in anc)
                if t not in anc:
                    assert p[L + t] == 0.0
            assert (p[:L] > 0).all()


def test_zero_query_gives_mean_of_visible_values_and_log_count():
    c = _case(15, B=2, N=9, L=(4, 9))
    c["q"] = np.zeros_like(c["q"])
    out, lse = _run(c)
    f = wl.storage_to_f64
    for b in range(2):
        L = int(c["seq_lens"][b])
        for i in range(9):
            path, a = [], i
            while a != -1:
                path.append(a)
                a = int(c["parent_idx"][b, a])
            for h in range(4):
                kv = h // 2
                vis = np.concatenate([f(c["v_cache"][b, :L, kv]), f(c["v_tree"][b, path, kv])], 0)
                np.testing.assert_allclose(out[b, i, h], vis.mean(0), atol=1e-13)
                assert abs(lse[b, i, h] - np.log(L + len(path))) < 1e-13


def test_empty_prefix_root_returns_its_own_value_exactly():
    c = _case(16, B=1, N=7, L=(0,))
    out, lse = _run(c)
    f = wl.storage_to_f64
    for h in range(4):
        assert np.array_equal(out[0, 0, h], f(c["v_tree"][0, 0, h // 2]))
    # every other node: convex combination of ancestor values only
    for i in range(1, 7):
        path, a = [], i
        while a != -1:
            path.append(a)
            a = int(c["parent_idx"][0, a])
        ref, _ = _sequential_path_attention(c, 0, i, 0)
        np.testing.assert_allclose(out[0, i, 0], ref, atol=1e-13)
        lo = f(c["v_tree"][0, path, 0]).min(0) - 1e-12
        hi = f(c["v_tree"][0, path, 0]).max(0) + 1e-12
        assert ((out[0, i, 0] >= lo) & (out[0, i, 0] <= hi)).all()


def test_single_node_tree_is_plain_decode_attention():
    c = _case(17, B=1, N=1, L=(9,), tree="chain")
    out, _ = _run(c)
    ref, _ = _sequential_path_attention(c, 0, 0, 3)
    np.testing.assert_allclose(out[0, 0, 3], ref, atol=1e-13)


def test_constant_values_give_that_constant():
    c = _case(18)
    for name in ("v_cache", "v_tree"):
        c[name] = np.full_like(c[name], 1.25) if c[name].dtype == np.float32 else c[name]
    out, _ = _run(c)
    np.testing.assert_allclose(out, 1.25, atol=1e-14)


def test_non_ancestor_keys_and_values_do_not_matter():
    c = _case(19, B=1, N=10, L=(6,))
    out0, lse0 = _run(c)
    i = 9
    anc, a = set(), i
    while a != -1:
        anc.add(a)
        a = int(c["parent_idx"][0, a])
    other = [t for t in range(10) if t not in anc]
    assert other
    c["k_tree"][0, other] *= 3.0
    c["v_tree"][0, other] += 7.0
    out1, lse1 = _run(c)
    assert np.array_equal(out0[0, i], out1[0, i]) and np.array_equal(lse0[0, i], lse1[0, i])
    # ... while an ancestor's value does
    c["v_tree"][0, 0] += 1.0
    out2, _ = _run(c)
    assert np.abs(out2[0, i] - out1[0, i]).max() > 1e-6


def test_relabelling_siblings_permutes_rows():
    c = _case(20, B=1, N=7, L=(5,), tree="level")   # depth 2, width 3
    out0, _ = _run(c)
    perm = np.array([0, 3, 1, 2, 6, 4, 5])          # new index k holds old node perm[k]; keeps levels
    inv = np.argsort(perm)
    c2 = dict(c)
    for name in ("q", "k_tree", "v_tree"):
        c2[name] = np.ascontiguousarray(c[name][:, perm])
    old_parent = c["parent_idx"][0]
    c2["parent_idx"] = np.array([[-1 if old_parent[perm[k]] < 0 else inv[old_parent[perm[k]]] for k in range(7)]],
                                np.int32)
    out1, _ = _run(c2)
    np.testing.assert_allclose(out1[0], out0[0, perm], atol=1e-14)


def test_prefix_split_and_lse_merge_reproduces_direct_result():
    """Partial results over two disjoint key ranges merged with
    m* = max m_s, l* = sum l_s e^{m_s-m*}, O = sum O_s l_s e^{m_s-m*} / l* equal the direct result."""
    c = _case(21, B=1, N=6, L=(12,), Hq=2, Hkv=1)
    out, lse = _run(c)
    h, cut, L = 1, 5, 12
    # part A: prefix rows [0,cut) plus the tree
    a = dict(c)
    a["seq_lens"] = np.array([cut], np.int32)
    outA, lseA = _run(a)
    for i in range(6):
        # part B: prefix rows [cut, L): rows cut..L-2 as a prefix, row L-1 as the root of a one-node tree
        bcase = dict(
            q=np.ascontiguousarray(c["q"][:, i:i + 1]),
            k_cache=np.ascontiguousarray(c["k_cache"][:, cut:L - 1]), v_cache=np.ascontiguousarray(c["v_cache"][:, cut:L - 1]),
            k_tree=np.ascontiguousarray(c["k_cache"][:, L - 1:L]), v_tree=np.ascontiguousarray(c["v_cache"][:, L - 1:L]),
            seq_lens=np.array([L - 1 - cut], np.int32), parent_idx=np.array([[-1]], np.int32), scale=c["scale"])
        outB, lseB = _run(bcase)
        m = max(lseA[0, i, h], lseB[0, 0, h])
        wa, wb = np.exp(lseA[0, i, h] - m), np.exp(lseB[0, 0, h] - m)
        merged = (wa * outA[0, i, h] + wb * outB[0, 0, h]) / (wa + wb)
        np.testing.assert_allclose(merged, out[0, i, h], atol=1e-13)
        assert abs(m + np.log(wa + wb) - lse[0, i, h]) < 1e-13


def test_scale_and_gqa_head_mapping_are_respected():
    c = _case(22, B=1, N=5, Hq=6, Hkv=3, L=(8,), scale=1.0)
    out1, _ = _run(c)
    c["scale"] = 0.25
    out2, _ = _run(c)
    assert np.abs(out1 - out2).max() > 1e-3
    # heads 2g and 2g+1 share kv head g: with identical queries they must give identical rows
    c["q"][:, :, 1] = c["q"][:, :, 0]
    c["q"][:, :, 2] = c["q"][:, :, 0]
    out3, _ = _run(c)
    assert np.array_equal(out3[:, :, 0], out3[:, :, 1])
    assert not np.array_equal(out3[:, :, 0], out3[:, :, 2])


def test_handworked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "attention_handworked.json")))
    a = np.log(np.array(g["prefix_a"] + g["tree_a"], np.float64)).astype(np.float32)
    L, N = len(g["prefix_a"]), len(g["tree_a"])
    zeros = lambda n: np.zeros(n, np.float32)
    k_cache = np.stack([a[:L], zeros(L)], -1).reshape(1, L, 1, 2)
    k_tree = np.stack([a[L:], zeros(N)], -1).reshape(1, N, 1, 2)
    v_cache = np.array(g["prefix_v"], np.float32).reshape(1, L, 1, 2)
    v_tree = np.array(g["tree_v"], np.float32).reshape(1, N, 1, 2)
    q = np.tile(np.array([1.0, 0.0], np.float32), (1, N, 1, 1))
    out, lse = oracle.tree_attention(q, k_cache, v_cache, np.array([L], np.int32), k_tree, v_tree,
                                     np.array([g["parent_idx"]], np.int32), g["scale"])
    np.testing.assert_allclose(out[0, :, 0], np.array(g["expected_out"]), atol=g["tolerance"])
    np.testing.assert_allclose(np.exp(lse[0, :, 0]), np.array(g["expected_exp_lse"]), rtol=g["tolerance"])


def test_rejects_non_topological_tree():
    c = _case(23, B=1, N=4, L=(3,))
    c["parent_idx"] = np.array([[-1, 2, 0, 1]], np.int32)
    with pytest.raises(ValueError):
        _run(c)
