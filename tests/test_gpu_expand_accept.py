"""GPU parity of equal-growth expansion and greedy acceptance + compaction against the CPU oracle:
indices, paths, lengths and cache bytes must match bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev, workspace

pytestmark = pytest.mark.gpu


def _cfg(B, D, W, V, dtype="bf16", Hkv=2, Dh=64, seed=5):
    return wl.Config("case", B, 2 * Hkv, Hkv, Dh, dtype, 16, (), D, W, V, (0.6,), "dirichlet", 0.5, 1, seed)


def _expand_both(cfg, logits_fn=None, check_margin=True):
    B, N, D, W = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width
    parent = np.full((B, N), -9, np.int32); token = np.full((B, N), -9, np.int32); cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 1, 0.0
    gp, gt, gc = to_dev(parent.copy()), to_dev(token.copy()), to_dev(cum.copy())
    shape = shape_of(cfg)
    ws = workspace(shape, ygg.OP_EXPAND)
    for d in range(1, D + 1):
        x = logits_fn(d) if logits_fn else wl.expansion_inputs(cfg, d)
        margin = oracle.expand(D, W, d, x, parent, token, cum)
        if check_margin:
            assert margin.min() > 1e-9, "ill-conditioned seed: pick another"
        ygg.equal_growth_expand(shape, d, to_dev(x), gp, gt, gc, ws)
    torch.cuda.synchronize()
    assert np.array_equal(gp.cpu().numpy(), parent)
    assert np.array_equal(gt.cpu().numpy(), token)
    got, ref = gc.cpu().numpy().astype(np.float64), cum.astype(np.float64)
    assert np.array_equal(np.isneginf(got), np.isneginf(ref))
    fin = np.isfinite(ref)
    assert np.abs(got[fin] - ref[fin]).max() <= 1e-5
    return parent, token, cum


@pytest.mark.parametrize("B,D,W,V", [(1, 3, 4, 1000), (2, 4, 8, 4097), (3, 2, 1, 50), (1, 2, 64, 9000),
                                     (2, 5, 16, 32000), (1, 3, 7, 13), (4, 3, 5, 4096), (1, 8, 8, 32000), (1, 16, 8, 32000),
                                     (1, 2, 40, 128256), (1, 2, 64, 128256)])   # the last two: > 1024 chunk lists per sequence
def test_expand_shapes(B, D, W, V):
    _expand_both(_cfg(B, D, W, V))


def test_expand_ties_resolve_to_lower_flat_index():
    cfg = _cfg(1, 2, 3, 5000)
    def fn(d):
        F = 1 if d == 1 else 3
        x = np.zeros((1, F, 5000), np.float32)
        if d == 1:
            x[0, 0, [7, 4100, 4999, 12]] = 5.0          # four equal maxima in two chunks -> tokens 7, 12, 4100
        else:
            x[0, :, 100] = 2.0                           # identical rows under parents with identical cum
            x[0, :, 4500] = 2.0
        return x
    parent, token, _ = _expand_both(cfg, logits_fn=fn, check_margin=False)
    assert token[0, 1:4].tolist() == [7, 12, 4100]
    assert parent[0, 4:7].tolist() == [1, 1, 2] and token[0, 4:7].tolist() == [100, 4500, 100]


def test_expand_masked_vocabulary_entries():
    cfg = _cfg(2, 2, 4, 300)
    def fn(d):
        x = wl.expansion_inputs(cfg, d)
        x[:, :, 5:] = -np.inf if d == 1 else x[:, :, 5:]   # depth 1: only five finite logits
        return x
    _expand_both(cfg, logits_fn=fn)


def test_expand_is_deterministic():
    cfg = _cfg(2, 3, 8, 20000)
    a = _expand_both(cfg)
    b = _expand_both(cfg)
    assert all(np.array_equal(x.view(np.int32), y.view(np.int32)) for x, y in zip(a, b))


def _accept_both(cfg, parent, token, layers, lens, logits=None, tstar=None, depth=None, codes=False):
    B, N = parent.shape
    D = cfg.depth if depth is None else depth
    max_len = int(lens.max())
    cap = max_len + D + 1
    mk = lambda s, n: wl.normal(cfg.seed, s, (layers, B, n, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    if codes:   # K/V held as 8-bit codes: compaction moves bytes, any byte pattern will do
        mk = lambda s, n: wl.rng(cfg.seed, s).integers(0, 256, size=(layers, B, n, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint8)
    kt, vt, kc, vc = mk(5, N), mk(6, N), mk(3, cap), mk(4, cap)
    lens = lens.astype(np.int32).copy()
    g = [to_dev(a.copy()) for a in (kt, vt, kc, vc, lens)]
    ref = oracle.accept_compact(D + 1, parent, token, kt, vt, kc, vc, lens, target_logits=logits, target_tokens=tstar)
    shape = shape_of(cfg, max_seq_len=max_len, kv_capacity=cap, n_nodes=N)
    shape.depth = D
    if codes:
        shape.kv_dtype = ygg.FP8_E4M3
    alen = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    apath = torch.full((B, D + 1), -5, dtype=torch.int32, device=DEV)
    bonus = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    ygg.accept_and_compact(shape, layers, to_dev(parent), to_dev(token), g[0], g[1], g[2], g[3], g[4], alen, apath, bonus,
                           target_logits=None if logits is None else to_dev(logits),
                           target_tokens=None if tstar is None else to_dev(tstar),
                           workspace=workspace(shape, ygg.OP_ACCEPT))
    torch.cuda.synchronize()
    assert np.array_equal(alen.cpu().numpy(), ref["accept_len"])
    assert np.array_equal(apath.cpu().numpy(), ref["accept_path"])
    assert np.array_equal(bonus.cpu().numpy(), ref["bonus_token"])
    assert np.array_equal(g[4].cpu().numpy(), lens)
    back = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()
    assert np.array_equal(back(g[2]), kc) and np.array_equal(back(g[3]), vc)
    return ref


@pytest.mark.parametrize("B,D,W,V,dtype,layers", [(1, 3, 4, 1000, "f32", 2), (3, 6, 8, 32000, "bf16", 3),
                                                  (2, 4, 5, 4099, "bf16", 1), (16, 5, 3, 517, "bf16", 2),
                                                  (1, 2, 2, 70000, "f32", 0)])
def test_accept_shapes(B, D, W, V, dtype, layers):
    cfg = _cfg(B, D, W, V, dtype=dtype)
    parent = wl.trees(cfg); token = wl.tokens(cfg, parent)
    logits = wl.acceptance_inputs(wl.scaled(cfg, agree=(0.8,)), parent, token)
    lens = wl.rng(cfg.seed, 50).integers(0, 40, size=B)
    ref = _accept_both(cfg, parent, token, layers, lens, logits=logits)
    assert ref["accept_len"].max() > 1


def test_accept_compacts_8bit_caches():
    cfg = _cfg(3, 5, 4, 2000, Dh=128)
    parent = wl.trees(cfg); token = wl.tokens(cfg, parent)
    logits = wl.acceptance_inputs(wl.scaled(cfg, agree=(0.8,)), parent, token)
    ref = _accept_both(cfg, parent, token, 2, np.array([7, 0, 33]), logits=logits, codes=True)
    assert ref["accept_len"].max() > 1


def test_accept_argmax_ties_across_chunks_and_precomputed_tokens():
    cfg = _cfg(1, 2, 2, 40000)
    parent = np.array([[-1, 0, 0, 1, 2]], np.int32)
    token = np.array([[0, 30000, 5, 9, 39999]], np.int32)
    x = np.zeros((1, 5, 40000), np.float32)
    x[0, 0, [5, 30000]] = 3.0           # tie in different chunks -> 5: node 2 matches
    x[0, 2, [39999, 39998]] = 1.0       # -> 39998: node 4 does not match
    ref = _accept_both(cfg, parent, token, 1, np.array([3]), logits=x)
    assert ref["accept_path"][0].tolist() == [0, 2, -1] and ref["bonus_token"][0] == 39998
    ref2 = _accept_both(cfg, parent, token, 1, np.array([3]), tstar=ref["tstar"])
    assert np.array_equal(ref2["accept_path"], ref["accept_path"])


def test_accept_general_tree_full_chain_and_root_only():
    N = 40
    cfg = _cfg(1, N - 1, 1, 64)
    parent = wl.random_topological_tree(9, N)[None]
    token = wl.node_tokens(9, parent[0], 64)[None]
    tstar = wl.rng(9, 60).integers(0, 64, size=(1, N)).astype(np.int32)
    _accept_both(cfg, parent, token, 2, np.array([11]), tstar=tstar, depth=N - 1)
    chain = wl.chain_tree(N)[None]
    tok = np.arange(N, dtype=np.int32)[None]
    full = np.concatenate([tok[0, 1:], [7]]).astype(np.int32)[None]
    ref = _accept_both(cfg, chain, tok, 1, np.array([0]), tstar=full, depth=N - 1)
    assert ref["accept_len"][0] == N
    ref = _accept_both(cfg, chain, tok, 1, np.array([5]), tstar=np.full((1, N), 63, np.int32), depth=N - 1)
    assert ref["accept_len"][0] == 1


def test_accept_largest_tree_fully_accepted_chain():
    """N = 1024 nodes as one chain, every draft token right: 1024 rows move into the cache of every layer."""
    N = 1024
    cfg = _cfg(2, N - 1, 1, 2000)
    chain = np.stack([wl.chain_tree(N), wl.chain_tree(N)])
    tok = np.stack([np.arange(N), np.arange(N)[::-1]]).astype(np.int32)
    full = np.concatenate([tok[:, 1:], [[7], [8]]], axis=1).astype(np.int32)
    full[1, 500] = 1999                                   # sequence 1 stops after 501 nodes
    ref = _accept_both(cfg, chain, tok, 2, np.array([3, 0]), tstar=full, depth=N - 1)
    assert ref["accept_len"].tolist() == [N, 501] and ref["bonus_token"].tolist() == [7, 1999]
