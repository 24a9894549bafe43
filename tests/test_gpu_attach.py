"""GPU parity of equal growth with free attachment against the CPU oracle: the tree arrays and the
carried pool must match after every step (indices bit for bit, scores to rounding)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev, workspace

pytestmark = pytest.mark.gpu

POOL_REC = np.dtype([("score", "<f8"), ("node", "<i4"), ("token", "<i4")])


def _cfg(B, D, W, V, seed=5):
    return wl.Config("case", B, 4, 2, 64, "bf16", 16, (), D, W, V, (0.6,), "dirichlet", 0.5, 1, seed)


def read_pool(pool_t, B, D, W):
    """Device pool bytes -> list of (count, records) per sequence (layout documented in include/ygg.h)."""
    cap = W * max(D - 1, 1)
    raw = pool_t.cpu().numpy()
    stride = 16 + cap * 16
    out = []
    for b in range(B):
        rec = raw[b * stride:(b + 1) * stride]
        count = int(rec[:4].view(np.int32)[0])
        out.append((count, rec[16:].view(POOL_REC)))
    return out


def attach_both(cfg, logits_fn=None, check_margin=True, sigma=1.0):
    B, N, D, W, V = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width, cfg.vocab
    parent = np.full((B, N), -9, np.int32); token = np.full((B, N), -9, np.int32); cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 1, 0.0
    gp, gt, gc = to_dev(parent.copy()), to_dev(token.copy()), to_dev(cum.copy())
    shape = shape_of(cfg)
    ws = workspace(shape, ygg.OP_ATTACH)
    nbytes = ygg.attach_pool_bytes(shape)
    assert nbytes >= B * (16 + W * max(D - 1, 1) * 16)
    gpool = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=DEV)   # step 1 must not rely on its contents
    pool = oracle.attach_pool(B, D, W)
    for t in range(1, D + 1):
        x = logits_fn(t) if logits_fn else wl.expansion_inputs(cfg, t) * np.float32(sigma)
        margin = oracle.attach(D, W, t, x, parent, token, cum, pool)
        ygg.equal_growth_attach(shape, t, to_dev(x), gp, gt, gc, gpool, ws)
        torch.cuda.synchronize()
        sl = slice(0, 1 + t * W)
        assert np.array_equal(gp.cpu().numpy()[:, sl], parent[:, sl]), f"parents differ at step {t}"
        assert np.array_equal(gt.cpu().numpy()[:, sl], token[:, sl]), f"tokens differ at step {t}"
        got, ref = gc.cpu().numpy()[:, sl].astype(np.float64), cum[:, sl].astype(np.float64)
        assert np.array_equal(np.isneginf(got), np.isneginf(ref))
        fin = np.isfinite(ref)
        assert np.abs(got[fin] - ref[fin]).max() <= 1e-5
        keep = W * (D - t)
        for b, (count, rec) in enumerate(read_pool(gpool, B, D, W)):
            n_ref = int(pool["count"][b])
            assert count == min(keep, n_ref), (t, b, count, keep, n_ref)
            if check_margin and n_ref:
                s = pool["score"][b, :min(n_ref, count + 1)]
                gaps = -np.diff(s[np.isfinite(s)])
                assert margin[b] > 1e-9 and (gaps.size == 0 or gaps[gaps > 0].min(initial=1.0) > 1e-10), "ill-conditioned seed"
            assert np.array_equal(rec["node"][:count], pool["node"][b, :count]), f"pool nodes differ at step {t}"
            assert np.array_equal(rec["token"][:count], pool["token"][b, :count]), f"pool tokens differ at step {t}"
            rs, gs = pool["score"][b, :count], rec["score"][:count]
            assert np.array_equal(np.isneginf(gs), np.isneginf(rs))
            f = np.isfinite(rs)
            assert f.sum() == 0 or np.abs(gs[f] - rs[f]).max() <= 1e-9
    return parent, token, cum


@pytest.mark.parametrize("B,D,W,V", [(1, 3, 4, 1000), (2, 4, 8, 4097), (3, 2, 1, 50), (2, 5, 16, 32000), (1, 3, 7, 13),
                                     (1, 6, 8, 32000), (1, 4, 32, 20000), (1, 2, 56, 9000), (4, 3, 5, 4096), (1, 1, 6, 700), (1, 8, 8, 32000), (1, 16, 8, 32000),
                                     # > 1024 list entries per row, and a pool sort over 4096 slots (the widest the call accepts)
                                     (1, 2, 40, 128256), (1, 2, 60, 128256)])
def test_attach_shapes(B, D, W, V):
    attach_both(_cfg(B, D, W, V))


@pytest.mark.parametrize("sigma", [0.05, 3.0])
def test_attach_flat_and_peaked_drafters(sigma):
    """A flat drafter hangs many leaves under old nodes (the pool is used hard); a peaked one rarely does."""
    parent, _, _ = attach_both(_cfg(2, 6, 6, 5000, seed=11), sigma=sigma)
    W = 6
    old = sum(int(parent[b, i] < 1 + ((i - 1) // W - 1) * W) for b in range(2) for i in range(1 + W, parent.shape[1]))
    assert (old > 0) if sigma < 1 else True


def test_attach_equal_scores_resolve_to_lower_node_then_token():
    cfg = _cfg(1, 3, 3, 5000)
    def fn(t):
        F = 1 if t == 1 else 3
        x = np.zeros((1, F, 5000), np.float32)
        x[0, :, [7, 4100, 4999, 12]] = 5.0      # four equal maxima in two chunks: every row offers tokens 7, 12, 4100
        return x
    parent, token, _ = attach_both(cfg, logits_fn=fn, check_margin=False)
    assert token[0, 1:4].tolist() == [7, 12, 4100]
    assert parent[0, 4:7].tolist() == [1, 1, 1] and token[0, 4:7].tolist() == [7, 12, 4100]


def test_attach_masked_vocabulary_entries():
    cfg = _cfg(2, 3, 4, 300)
    def fn(t):
        x = wl.expansion_inputs(cfg, t)
        if t == 1:
            x[:, :, 3:] = -np.inf     # the root can offer three finite tokens only: the fourth node has cum = -inf
        return x
    attach_both(cfg, logits_fn=fn, check_margin=False)


def test_attach_is_deterministic():
    cfg = _cfg(2, 4, 8, 20000)
    a = attach_both(cfg)
    b = attach_both(cfg)
    assert all(np.array_equal(x.view(np.int32), y.view(np.int32)) for x, y in zip(a, b))


def test_attach_tree_feeds_attention_and_acceptance():
    """The grown tree is a general topological tree (depth != step): attention and acceptance take it as is."""
    from gpu_util import run_attention
    cfg = wl.Config("case", 1, 8, 2, 128, "bf16", 200, (), 4, 6, 3000, (0.6,), "dirichlet", 0.5, 1, 77)
    parent, token, _ = attach_both(cfg)
    lens = np.array([200], np.int32)
    host = wl.attention_inputs(cfg, lens=lens)
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], lens, host["k_tree"],
                                             host["v_tree"], parent, cfg.softmax_scale)
    out, lse = run_attention(shape_of(cfg, max_seq_len=200), host, parent)
    assert np.abs(out - ref_out).max() <= 2e-2 and np.abs(lse - ref_lse).max() <= 1e-3
    from test_gpu_expand_accept import _accept_both
    logits = wl.acceptance_inputs(cfg, parent, token)
    _accept_both(cfg, parent, token, 2, lens, logits=logits)
