"""The calls only enqueue kernels and never synchronise, so a whole verification step can be captured
once as a HIP graph and replayed.  Every replay must reproduce the eager result bit for bit, also when
the program launches other work and synchronises between the replays."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev, workspace

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16).cpu().numpy() if t.dtype == torch.bfloat16 else t.cpu().numpy()


@pytest.mark.parametrize("growth", ["frontier", "attach"])
@pytest.mark.parametrize("which", ["tiny_fp32", "bf16_matrix_cores", "8bit_kv"])
def test_captured_step_replays_like_the_eager_step(which, growth):
    if which == "tiny_fp32":
        cfg, layers = wl.CONFIGS[1], 2
    else:
        cfg, layers = wl.scaled(wl.CONFIGS[2], prefix_len=700, depth=4, width=8, vocab=6000, n_q_heads=8, n_kv_heads=8,
                                seed=31), 3
    B, N, D, W = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width
    shape = shape_of(cfg)
    codes = which == "8bit_kv"
    if codes:
        shape.kv_dtype = ygg.FP8_E4M3
    cap = cfg.kv_capacity
    lens_h = wl.seq_lens(cfg)
    draft = [to_dev(wl.expansion_inputs(cfg, d)) for d in range(1, D + 1)]
    per_layer = [(wl.attention_inputs_fp8kv if codes else wl.attention_inputs)(cfg, layer=l, lens=lens_h)
                 for l in range(layers)]
    if codes:
        k_scale, v_scale = (to_dev(np.stack([h[k] for h in per_layer])) for k in ("k_scale", "v_scale"))
    stack = lambda k: to_dev(np.stack([h[k] for h in per_layer]))
    q, k_tree, v_tree = stack("q"), stack("k_tree"), stack("v_tree")
    k_cache0, v_cache0 = stack("k_cache"), stack("v_cache")
    k_cache, v_cache = k_cache0.clone(), v_cache0.clone()
    lens0 = to_dev(lens_h); lens = lens0.clone()
    parent0 = np.full((B, N), -1, np.int32); token0 = np.zeros((B, N), np.int32); token0[:, 0] = 9
    parent, token = to_dev(parent0.copy()), to_dev(token0.copy())
    cum = torch.zeros((B, N), dtype=torch.float32, device=DEV)
    out = torch.empty_like(q)
    # a target whose argmax agrees with the drafted tree now and then; the tree is only known on the device
    target = to_dev(wl.normal(cfg.seed, 77, (B, N, cfg.vocab), "f32"))
    alen = torch.zeros((B,), dtype=torch.int32, device=DEV)
    apath = torch.zeros((B, D + 1), dtype=torch.int32, device=DEV)
    bonus = torch.zeros((B,), dtype=torch.int32, device=DEV)
    ws = {op: workspace(shape, op, layers) for op in (ygg.OP_ATTENTION, ygg.OP_EXPAND, ygg.OP_ACCEPT, ygg.OP_ATTACH)}
    pool = torch.zeros(ygg.attach_pool_bytes(shape), dtype=torch.uint8, device=DEV)

    def step():
        lens.copy_(lens0); k_cache.copy_(k_cache0); v_cache.copy_(v_cache0)
        for d in range(1, D + 1):
            if growth == "frontier":
                ygg.equal_growth_expand(shape, d, draft[d - 1], parent, token, cum, ws[ygg.OP_EXPAND])
            else:
                ygg.equal_growth_attach(shape, d, draft[d - 1], parent, token, cum, pool, ws[ygg.OP_ATTACH])
        for l in range(layers):
            if codes:
                ygg.tree_attention_fp8kv(shape, q[l], k_cache[l], v_cache[l], lens, k_tree[l], v_tree[l], k_scale[l],
                                         v_scale[l], parent, out[l], None, ws[ygg.OP_ATTENTION])
            else:
                ygg.tree_attention(shape, q[l], k_cache[l], v_cache[l], lens, k_tree[l], v_tree[l], parent, out[l], None,
                                   ws[ygg.OP_ATTENTION])
        ygg.accept_and_compact(shape, layers, parent, token, k_tree, v_tree, k_cache, v_cache, lens, alen, apath, bonus,
                               target_logits=target, workspace=ws[ygg.OP_ACCEPT])

    results = lambda: [_bits(t).copy() for t in (parent, token, cum, out, alen, apath, bonus, lens, k_cache, v_cache)]
    step(); step()
    torch.cuda.synchronize()
    eager = results()
    # the eager tree equals the oracle's (the rest of the path is covered by the parity tests)
    p_ref, t_ref, c_ref = parent0.copy(), token0.copy(), np.zeros((B, N), np.float32)
    o_pool = oracle.attach_pool(B, D, W)
    for d in range(1, D + 1):
        x = draft[d - 1].cpu().numpy()
        if growth == "frontier":
            oracle.expand(D, W, d, x, p_ref, t_ref, c_ref)
        else:
            oracle.attach(D, W, d, x, p_ref, t_ref, c_ref, o_pool)
    assert np.array_equal(eager[0], p_ref) and np.array_equal(eager[1], t_ref)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    scratch = torch.empty(1 << 20, dtype=torch.float32, device=DEV)
    for rep in range(4):
        for t in (parent, token, cum, out, alen, apath, bonus):   # wipe the outputs: a replay must rewrite them
            t.fill_(-3 if t.dtype in (torch.int32,) else 0)
        parent.copy_(to_dev(parent0)); token.copy_(to_dev(token0)); cum.zero_()
        scratch.normal_(); float(scratch.sum())                   # unrelated eager work and a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("parent", "token", "cum", "out", "accept_len", "accept_path", "bonus", "seq_lens", "k_cache",
                               "v_cache"), results(), eager):
            assert np.array_equal(a, b), f"replay {rep}: {name} differs from the eager step"
