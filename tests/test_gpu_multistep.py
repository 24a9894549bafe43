"""Several verification steps in a row, chained on the device: the lengths and the caches that one step's acceptance
leaves behind are what the next step's attention reads, with no value ever brought back to the host in between.
The oracle replays the same steps on the CPU; everything must agree at the end and after every step."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev, to_f64, workspace

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.cpu().numpy()


@pytest.mark.parametrize("which", ["fp32_vector_path", "bf16_matrix_cores_ragged_batch", "8bit_kv_ragged_batch"])
def test_three_steps_chained_on_the_device(which):
    steps = 3
    if which == "fp32_vector_path":
        base = wl.scaled(wl.CONFIGS[1], prefix_len=40)
        lens0 = np.array([40], np.int32)
    else:
        base = wl.Config("case", 3, 8, 2, 128, "bf16", 0, (5, 300), 4, 6, 5000, (0.7,), "dirichlet", 0.5, 1, 61)
        lens0 = np.array([300, 5, 131], np.int32)
    B, N, D, W, V = base.batch, base.n_nodes, base.depth, base.width, base.vocab
    layers = 2
    max_len = int(lens0.max()) + steps * (D + 1)
    cap = max_len + D + 1
    cfg = wl.scaled(base, prefix_len=max_len, prefix_range=())
    shape = shape_of(cfg, max_seq_len=max_len, kv_capacity=cap)
    codes = which.startswith("8bit")   # K/V as E4M3 codes: what compaction appends is what the next attention decodes

    mk = lambda stream, n: wl.normal(cfg.seed, stream, (layers, B, n, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    if codes:
        shape.kv_dtype = ygg.FP8_E4M3
        mk = lambda stream, n: wl.f64_to_fp8_e4m3_bits(
            wl.normal(cfg.seed, stream, (layers, B, n, cfg.n_kv_heads, cfg.head_dim), "f32").astype(np.float64) * 64.0)
        k_scale = np.array([1 / 64.0, 1 / 50.0], np.float32)
        v_scale = np.array([1 / 70.0, 1 / 64.0], np.float32)
        g_ks, g_vs = to_dev(k_scale), to_dev(v_scale)
    kc, vc = mk(3, cap), mk(4, cap)
    lens = lens0.copy()
    g_kc, g_vc, g_lens = to_dev(kc.copy()), to_dev(vc.copy()), to_dev(lens.copy())
    ws = {op: workspace(shape, op, layers) for op in (ygg.OP_ATTENTION, ygg.OP_EXPAND, ygg.OP_ACCEPT)}
    tol = 1e-5 if cfg.dtype == "f32" else 2e-2
    total_accepted = 0
    for step in range(steps):
        seed = cfg.seed + 100 * step
        # drafting: grow the tree from this step's draft logits
        parent = np.full((B, N), -1, np.int32); token = np.zeros((B, N), np.int32); cum = np.zeros((B, N), np.float32)
        token[:, 0] = 7 + step
        g_parent, g_token, g_cum = to_dev(parent.copy()), to_dev(token.copy()), to_dev(cum.copy())
        for d in range(1, D + 1):
            x = np.stack([wl.draft_logits(seed, d, 1 if d == 1 else W, V, sub=b) for b in range(B)])
            oracle.expand(D, W, d, x, parent, token, cum)
            ygg.equal_growth_expand(shape, d, to_dev(x), g_parent, g_token, g_cum, ws[ygg.OP_EXPAND])
        # verification: every layer attends over what the previous steps left in the cache
        q = wl.normal(seed, 11, (layers, B, N, cfg.n_q_heads, cfg.head_dim), cfg.dtype)
        kt, vt = mk(500 + step, N), mk(600 + step, N)
        g_q, g_kt, g_vt = to_dev(q), to_dev(kt), to_dev(vt)
        g_out = torch.empty_like(g_q)
        for l in range(layers):
            if codes:
                ygg.tree_attention_fp8kv(shape, g_q[l], g_kc[l], g_vc[l], g_lens, g_kt[l], g_vt[l], g_ks, g_vs, g_parent,
                                         g_out[l], None, ws[ygg.OP_ATTENTION])
            else:
                ygg.tree_attention(shape, g_q[l], g_kc[l], g_vc[l], g_lens, g_kt[l], g_vt[l], g_parent, g_out[l], None,
                                   ws[ygg.OP_ATTENTION])
        if codes:
            ref_out = np.stack([oracle.tree_attention_fp8kv(q[l], kc[l], vc[l], lens, kt[l], vt[l], k_scale, v_scale, parent,
                                                            cfg.softmax_scale)[0] for l in range(layers)])
        else:
            ref_out = np.stack([oracle.tree_attention(q[l], kc[l], vc[l], lens, kt[l], vt[l], parent, cfg.softmax_scale)[0]
                                for l in range(layers)])
        # acceptance: the target agrees with the draft now and then; lengths and caches advance on the device
        target = wl.acceptance_inputs(wl.scaled(cfg, seed=seed), parent, token)
        ref = oracle.accept_compact(D + 1, parent, token, kt, vt, kc, vc, lens, target_logits=target)
        alen = torch.zeros((B,), dtype=torch.int32, device=DEV)
        apath = torch.zeros((B, D + 1), dtype=torch.int32, device=DEV)
        bonus = torch.zeros((B,), dtype=torch.int32, device=DEV)
        ygg.accept_and_compact(shape, layers, g_parent, g_token, g_kt, g_vt, g_kc, g_vc, g_lens, alen, apath, bonus,
                               target_logits=to_dev(target), workspace=ws[ygg.OP_ACCEPT])
        torch.cuda.synchronize()   # the checks below read back; the calls above never needed a value from the device
        assert np.array_equal(g_parent.cpu().numpy(), parent) and np.array_equal(g_token.cpu().numpy(), token)
        assert np.abs(to_f64(g_out) - ref_out).max() <= tol, f"step {step}"
        assert np.array_equal(alen.cpu().numpy(), ref["accept_len"]) and np.array_equal(apath.cpu().numpy(), ref["accept_path"])
        assert np.array_equal(bonus.cpu().numpy(), ref["bonus_token"])
        assert np.array_equal(g_lens.cpu().numpy(), lens)
        assert np.array_equal(_bits(g_kc), kc) and np.array_equal(_bits(g_vc), vc), f"cache differs after step {step}"
        total_accepted += int(ref["accept_len"].sum())
    assert np.array_equal(lens, lens0 + (lens - lens0)) and (lens - lens0).sum() == total_accepted
    assert total_accepted > steps * B    # some draft tokens were accepted beyond the root
