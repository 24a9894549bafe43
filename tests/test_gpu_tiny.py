"""GPU parity on the tiny fp32 configuration: every step of the path against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, run_attention, shape_of, to_dev, workspace

pytestmark = pytest.mark.gpu


def test_tiny_attention_fp32():
    cfg = wl.CONFIGS[1]
    parent = wl.trees(cfg)
    host = wl.attention_inputs(cfg)
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"],
                                             host["k_tree"], host["v_tree"], parent, cfg.softmax_scale)
    out, lse = run_attention(shape_of(cfg), host, parent)
    assert np.abs(out - ref_out).max() <= 1e-5
    assert np.abs(lse - ref_lse).max() <= 1e-5


def test_tiny_expand_all_depths():
    cfg = wl.CONFIGS[1]
    B, N, D, W = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width
    parent = np.full((B, N), -9, np.int32); token = np.full((B, N), -9, np.int32); cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 7, 0.0
    g_parent, g_token, g_cum = to_dev(parent.copy()), to_dev(token.copy()), to_dev(cum.copy())
    shape = shape_of(cfg)
    ws = workspace(shape, ygg.OP_EXPAND)
    for d in range(1, D + 1):
        x = wl.expansion_inputs(cfg, d)
        margin = oracle.expand(D, W, d, x, parent, token, cum)
        assert margin.min() > 1e-9
        ygg.equal_growth_expand(shape, d, to_dev(x), g_parent, g_token, g_cum, ws)
    torch.cuda.synchronize()
    assert np.array_equal(g_parent.cpu().numpy(), parent)
    assert np.array_equal(g_token.cpu().numpy(), token)
    assert np.abs(g_cum.cpu().numpy().astype(np.float64) - cum.astype(np.float64)).max() <= 1e-5


def test_tiny_accept_and_compact():
    cfg = wl.CONFIGS[1]
    B, N, D = cfg.batch, cfg.n_nodes, cfg.depth
    parent = wl.trees(cfg); token = wl.tokens(cfg, parent)
    logits = wl.acceptance_inputs(cfg, parent, token)
    layers = 2
    cap = cfg.kv_capacity
    mk = lambda s, n: wl.normal(cfg.seed, s, (layers, B, n, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    kt, vt, kc, vc = mk(5, N), mk(6, N), mk(3, cap), mk(4, cap)
    lens = wl.seq_lens(cfg).copy()
    g = dict(kt=to_dev(kt), vt=to_dev(vt), kc=to_dev(kc.copy()), vc=to_dev(vc.copy()), lens=to_dev(lens.copy()))
    ref = oracle.accept_compact(D + 1, parent, token, kt, vt, kc, vc, lens, target_logits=logits)
    shape = shape_of(cfg)
    alen = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    apath = torch.full((B, D + 1), -5, dtype=torch.int32, device=DEV)
    bonus = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    ygg.accept_and_compact(shape, layers, to_dev(parent), to_dev(token), g["kt"], g["vt"], g["kc"], g["vc"], g["lens"],
                           alen, apath, bonus, target_logits=to_dev(logits), workspace=workspace(shape, ygg.OP_ACCEPT))
    torch.cuda.synchronize()
    assert np.array_equal(alen.cpu().numpy(), ref["accept_len"])
    assert np.array_equal(apath.cpu().numpy(), ref["accept_path"])
    assert np.array_equal(bonus.cpu().numpy(), ref["bonus_token"])
    assert np.array_equal(g["lens"].cpu().numpy(), lens)
    assert np.array_equal(g["kc"].cpu().numpy(), kc) and np.array_equal(g["vc"].cpu().numpy(), vc)
