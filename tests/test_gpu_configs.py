"""GPU parity at the full sizes of the five workload configurations, in the launch configuration the
benchmark times (same shapes, same plan).  Attention is compared on every output row and every
log-sum-exp of a whole layer (the oracle runs its rows in parallel: about 20 s for the widest tree);
expansion indices, accepted paths and compacted cache bytes are compared exactly everywhere."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, run_attention, shape_of, to_dev, workspace

pytestmark = pytest.mark.gpu


def _gates(cfg, out, lse, ref_out, ref_lse):
    err = np.abs(out - ref_out)
    if cfg.dtype == "f32":
        assert err.max() <= 1e-5 and np.abs(lse - ref_lse).max() <= 1e-5
    else:
        assert err.max() <= 2e-2 and err.mean() <= 1e-2, (err.max(), err.mean())
        rms = np.sqrt((ref_out ** 2).mean())
        assert np.sqrt((err ** 2).mean()) <= 0.02 * rms, (np.sqrt((err ** 2).mean()), rms)
        assert np.abs(lse - ref_lse).max() <= 1e-3
        # no row tile, key split or kv head may hide behind the averages: the same relative bound per node
        row_rms = np.sqrt((err ** 2).mean(axis=(2, 3)))                     # [B, N]
        assert (row_rms <= 0.05 * rms).all(), float(row_rms.max() / rms)
    assert np.isfinite(out).all() and np.isfinite(lse).all()


@pytest.mark.parametrize("config,layer", [(1, 0), (2, 0), (2, 31), (3, 0), (3, 17), (4, 0), (4, 31), (5, 0)])
def test_attention_full_size(config, layer):
    """Every output row and every log-sum-exp of the layer against the oracle."""
    cfg = wl.CONFIGS[config]
    lens = wl.seq_lens(cfg)
    parent = wl.trees(cfg)
    host = wl.attention_inputs(cfg, layer=layer, lens=lens)
    out, lse = run_attention(shape_of(cfg), host, parent)
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], lens, host["k_tree"],
                                             host["v_tree"], parent, cfg.softmax_scale)
    _gates(cfg, out, lse, ref_out, ref_lse)


@pytest.mark.parametrize("config,layer", [(2, 0), (3, 5), (5, 0)])
def test_attention_full_size_8bit_kv(config, layer):
    """The bf16 configurations at full size with K/V stored as E4M3 codes (same draws, quantised per kv head);
    every row of the layer."""
    cfg = wl.CONFIGS[config]
    lens = wl.seq_lens(cfg)
    parent = wl.trees(cfg)
    host = wl.attention_inputs_fp8kv(cfg, layer=layer, lens=lens)
    shape = shape_of(cfg)
    shape.kv_dtype = ygg.FP8_E4M3
    d = {k: to_dev(np.ascontiguousarray(v)) for k, v in host.items()}
    out_t = torch.full_like(d["q"], float("nan"))
    lse_t = torch.full(d["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ygg.tree_attention_fp8kv(shape, d["q"], d["k_cache"], d["v_cache"], d["seq_lens"], d["k_tree"], d["v_tree"],
                             d["k_scale"], d["v_scale"], to_dev(parent), out_t, lse_t, workspace(shape, ygg.OP_ATTENTION))
    torch.cuda.synchronize()
    out, lse = out_t.double().cpu().numpy(), lse_t.double().cpu().numpy()
    ref_out, ref_lse = oracle.tree_attention_fp8kv(host["q"], host["k_cache"], host["v_cache"], lens, host["k_tree"],
                                                   host["v_tree"], host["k_scale"], host["v_scale"], parent,
                                                   cfg.softmax_scale)
    _gates(cfg, out, lse, ref_out, ref_lse)


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_expansion_full_size(config):
    cfg = wl.CONFIGS[config]
    B, N, D, W = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width
    parent = np.full((B, N), -9, np.int32); token = np.full((B, N), -9, np.int32); cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 1, 0.0
    gp, gt, gc = to_dev(parent.copy()), to_dev(token.copy()), to_dev(cum.copy())
    shape = shape_of(cfg)
    ws = workspace(shape, ygg.OP_EXPAND)
    for d in range(1, D + 1):
        x = wl.expansion_inputs(cfg, d)
        margin = oracle.expand(D, W, d, x, parent, token, cum)
        assert margin.min() > 1e-9
        ygg.equal_growth_expand(shape, d, to_dev(x), gp, gt, gc, ws)
    torch.cuda.synchronize()
    assert np.array_equal(gp.cpu().numpy(), parent) and np.array_equal(gt.cpu().numpy(), token)
    assert np.abs(gc.cpu().numpy().astype(np.float64) - cum).max() <= 1e-5
    for d in range(1, D + 1):   # exactly W nodes per depth, each hanging off the previous depth
        blk = parent[:, 1 + (d - 1) * W: 1 + d * W]
        lo, hi = (0, 0) if d == 1 else (1 + (d - 2) * W, (d - 1) * W)
        assert ((blk >= lo) & (blk <= hi)).all()


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_free_attachment_full_size(config):
    """Equal growth with free attachment on the same draft logits: tree and pool after every step."""
    from test_gpu_attach import attach_both
    cfg = wl.CONFIGS[config]
    parent, _, _ = attach_both(cfg)
    W = cfg.width
    for i in range(1, cfg.n_nodes):    # a leaf hangs under any node grown in an earlier step
        assert np.all((parent[:, i] >= 0) & (parent[:, i] < 1 + ((i - 1) // W) * W))


@pytest.mark.parametrize("config,layers", [(1, 2), (2, 4), (3, 2), (4, 1), (5, 1)])
def test_acceptance_full_size(config, layers):
    cfg = wl.CONFIGS[config]
    B, N, D = cfg.batch, cfg.n_nodes, cfg.depth
    parent = wl.trees(cfg); token = wl.tokens(cfg, parent)
    logits = wl.acceptance_inputs(cfg, parent, token)
    lens = wl.seq_lens(cfg).copy()
    cap = cfg.kv_capacity
    kt = np.stack([wl.attention_inputs(cfg, layer=l, lens=lens)["k_tree"] for l in range(layers)])
    vt = np.stack([wl.attention_inputs(cfg, layer=l, lens=lens)["v_tree"] for l in range(layers)])
    shp = (layers, B, cap, cfg.n_kv_heads, cfg.head_dim)
    kc = wl.normal(cfg.seed, 3, shp, cfg.dtype); vc = wl.normal(cfg.seed, 4, shp, cfg.dtype)
    g = [to_dev(a) for a in (kt, vt, kc, vc, lens)]
    ref = oracle.accept_compact(D + 1, parent, token, kt, vt, kc, vc, lens, target_logits=logits)
    shape = shape_of(cfg)
    alen = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    apath = torch.full((B, D + 1), -5, dtype=torch.int32, device=DEV)
    bonus = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    ygg.accept_and_compact(shape, layers, to_dev(parent), to_dev(token), g[0], g[1], g[2], g[3], g[4], alen, apath,
                           bonus, target_logits=to_dev(logits), workspace=workspace(shape, ygg.OP_ACCEPT))
    torch.cuda.synchronize()
    assert np.array_equal(alen.cpu().numpy(), ref["accept_len"])
    assert np.array_equal(apath.cpu().numpy(), ref["accept_path"])
    assert np.array_equal(bonus.cpu().numpy(), ref["bonus_token"])
    assert np.array_equal(g[4].cpu().numpy(), lens)
    assert 1 <= ref["accept_len"].min() and ref["accept_len"].max() <= D + 1
    back = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()
    assert np.array_equal(back(g[2]), kc) and np.array_equal(back(g[3]), vc)


def test_whole_step_on_the_tiny_configuration_with_the_grown_tree():
    """expand (D steps) -> attention over the grown tree -> accept, chained on the device."""
    cfg = wl.CONFIGS[1]
    B, N, D, W = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width
    parent = np.full((B, N), -1, np.int32); token = np.zeros((B, N), np.int32); cum = np.zeros((B, N), np.float32)
    token[:, 0] = 11
    gp, gt, gc = to_dev(parent.copy()), to_dev(token.copy()), to_dev(cum.copy())
    shape = shape_of(cfg)
    ws = workspace(shape, ygg.OP_EXPAND)
    for d in range(1, D + 1):
        x = wl.expansion_inputs(cfg, d)
        oracle.expand(D, W, d, x, parent, token, cum)
        ygg.equal_growth_expand(shape, d, to_dev(x), gp, gt, gc, ws)
    host = wl.attention_inputs(cfg)
    ref_out, _ = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"], host["k_tree"],
                                       host["v_tree"], parent, cfg.softmax_scale)
    torch.cuda.synchronize()
    out, _ = run_attention(shape, host, gp.cpu().numpy())
    assert np.abs(out - ref_out).max() <= 1e-5
    logits = wl.acceptance_inputs(cfg, parent, token)
    tstar = logits.argmax(-1).astype(np.int32)
    kt, vt = host["k_tree"][None].copy(), host["v_tree"][None].copy()
    kc, vc, lens = host["k_cache"][None].copy(), host["v_cache"][None].copy(), host["seq_lens"].copy()
    ref = oracle.accept_compact(D + 1, parent, token, kt, vt, kc, vc, lens, target_tokens=tstar)
    g = [to_dev(a) for a in (kt, vt, host["k_cache"][None].copy(), host["v_cache"][None].copy(), host["seq_lens"].copy())]
    alen = torch.zeros((B,), dtype=torch.int32, device=DEV); apath = torch.zeros((B, D + 1), dtype=torch.int32, device=DEV)
    bonus = torch.zeros((B,), dtype=torch.int32, device=DEV)
    ygg.accept_and_compact(shape, 1, gp, gt, g[0], g[1], g[2], g[3], g[4], alen, apath, bonus,
                           target_logits=to_dev(logits), workspace=workspace(shape, ygg.OP_ACCEPT))
    torch.cuda.synchronize()
    assert np.array_equal(apath.cpu().numpy(), ref["accept_path"]) and np.array_equal(g[2].cpu().numpy(), kc)
