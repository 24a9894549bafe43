"""GPU parity of verification-width pruning against the oracle's bottom-up tree DP."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev

pytestmark = pytest.mark.gpu


def _grow(cfg, rule, sigma=1.0):
    B, N, D, W = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width
    parent = np.full((B, N), -1, np.int32); token = np.zeros((B, N), np.int32); cum = np.zeros((B, N), np.float32)
    token[:, 0] = 1
    pool = oracle.attach_pool(B, D, W)
    for t in range(1, D + 1):
        x = wl.expansion_inputs(cfg, t) * np.float32(sigma)
        if rule == "attach":
            oracle.attach(D, W, t, x, parent, token, cum, pool)
        else:
            oracle.expand(D, W, t, x, parent, token, cum)
    return parent, token, cum


def _latency(N, knee, slope):
    n = np.arange(N + 1, dtype=np.float64)
    return np.where(n <= knee, 1.0, 1.0 + slope * (n - knee)).astype(np.float32)


def prune_both(cfg, parent, token, cum, w, t_ver, t_draft):
    B, N = parent.shape
    ref = oracle.prune(w, parent, token, cum, t_ver.astype(np.float64), t_draft)
    shape = shape_of(cfg, n_nodes=N)
    kept = torch.full((B, w), -5, dtype=torch.int32, device=DEV)
    npar = torch.full((B, w), -5, dtype=torch.int32, device=DEV)
    ntok = torch.full((B, w), -5, dtype=torch.int32, device=DEV)
    elen = torch.full((B,), float("nan"), dtype=torch.float32, device=DEV)
    bw = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    ygg.prune_for_verification(shape, w, to_dev(parent), to_dev(token), to_dev(cum), kept, npar, ntok, elen, bw,
                               t_verifier=to_dev(t_ver), t_draft=t_draft)
    torch.cuda.synchronize()
    kept, npar, ntok, elen, bw = (x.cpu().numpy() for x in (kept, npar, ntok, elen, bw))
    for b in range(B):
        p = np.exp(cum[b].astype(np.float64))
        srt = np.sort(p)[::-1]
        unique = w == N or srt[w - 1] - srt[w] > 1e-12
        k = kept[b]
        # always: a valid renumbered subtree of the optimal value
        assert k[0] == 0 and np.all(np.diff(k) > 0) and npar[b, 0] == -1
        for j in range(1, w):
            assert 0 <= npar[b, j] < j and k[npar[b, j]] == parent[b, k[j]]
        assert np.array_equal(ntok[b], token[b, k])
        assert abs(p[k].sum() - ref["expected_len"][b]) <= 1e-9 * max(1.0, ref["expected_len"][b])
        assert abs(elen[b] - ref["expected_len"][b]) <= 2e-6 * max(1.0, ref["expected_len"][b])
        if unique:
            assert np.array_equal(k, ref["kept_nodes"][b]) and np.array_equal(npar[b], ref["new_parent"][b])
        obj = ref["best_curve"][b, 1:] / (t_draft + t_ver[1:].astype(np.float64))
        top2 = np.sort(obj)[-2:] if N > 1 else np.array([0.0, 1.0])
        if top2[1] - top2[0] > 1e-9 * top2[1]:
            assert bw[b] == ref["best_width"][b]
        else:
            assert abs(obj[bw[b] - 1] - top2[1]) <= 1e-9 * top2[1]
    return kept, npar, ntok


@pytest.mark.parametrize("config,rule", [(1, "frontier"), (1, "attach"), (2, "frontier"), (2, "attach"), (3, "attach"),
                                         (4, "frontier"), (4, "attach"), (5, "attach")])
def test_prune_on_the_drafted_trees_of_every_configuration(config, rule):
    cfg = wl.CONFIGS[config]
    parent, token, cum = _grow(cfg, rule)
    N = cfg.n_nodes
    t_ver = _latency(N, knee=max(2, N // 4), slope=0.05)
    for w in sorted({1, 2, max(1, N // 3), N - 1, N}):
        prune_both(cfg, parent, token, cum, w, t_ver, t_draft=0.7)


@pytest.mark.parametrize("knee,slope,t_draft", [(0, 0.0, 1.0), (0, 50.0, 1.0), (16, 0.02, 0.1), (4, 0.3, 3.0)])
def test_best_width_follows_the_latency_curve(knee, slope, t_draft):
    cfg = wl.Config("case", 3, 4, 2, 64, "bf16", 16, (), 6, 8, 3000, (0.6,), "dirichlet", 0.5, 1, 21)
    parent, token, cum = _grow(cfg, "attach", sigma=0.5)
    prune_both(cfg, parent, token, cum, 9, _latency(cfg.n_nodes, knee, slope), t_draft)


def test_prune_handles_equal_values_and_dead_branches():
    cfg = wl.Config("case", 1, 4, 2, 64, "bf16", 16, (), 3, 3, 50, (0.6,), "dirichlet", 0.5, 1, 22)
    parent = np.array([[-1, 0, 0, 0, 1, 1, 2, 4, 4, 6]], np.int32)
    token = np.arange(10, dtype=np.int32)[None]
    # node 1 is certain (same value as the root), nodes 4 and 5 tie, node 3 and its would-be subtree are impossible
    cum = np.array([[0.0, 0.0, -1.0, -np.inf, -0.5, -0.5, -1.0, -0.5, -2.0, -3.0]], np.float32)
    t_ver = _latency(10, 3, 0.1)
    for w in range(1, 11):
        kept, _, _ = prune_both(cfg, parent, token, cum, w, t_ver, 0.5)
        if w < 10:
            assert 3 not in kept[0]
    kept, _, _ = prune_both(cfg, parent, token, cum, 4, t_ver, 0.5)
    assert list(kept[0]) == [0, 1, 4, 5]      # 0 and 1 (certain), then 4 before 5 before 7 among the -0.5 ties


def test_pruned_tree_feeds_attention():
    from gpu_util import run_attention
    cfg = wl.Config("case", 2, 8, 2, 128, "bf16", 300, (), 4, 8, 3000, (0.6,), "dirichlet", 0.5, 1, 23)
    parent, token, cum = _grow(cfg, "attach")
    w = 17
    kept, npar, _ = prune_both(cfg, parent, token, cum, w, _latency(cfg.n_nodes, 8, 0.05), 0.5)
    lens = np.array([300, 123], np.int32)
    full = wl.attention_inputs(cfg, lens=lens)
    host = dict(full)
    for name in ("q", "k_tree", "v_tree"):        # the verifier runs on the kept tokens only
        host[name] = np.stack([full[name][b][kept[b]] for b in range(cfg.batch)])
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], lens, host["k_tree"],
                                             host["v_tree"], npar, cfg.softmax_scale)
    # a node of the pruned tree sees exactly what it saw in the full tree: same ancestors, same prefix
    full_out, _ = oracle.tree_attention(full["q"], full["k_cache"], full["v_cache"], lens, full["k_tree"],
                                        full["v_tree"], parent, cfg.softmax_scale)
    for b in range(cfg.batch):
        assert np.abs(ref_out[b] - full_out[b][kept[b]]).max() <= 1e-12
    out, lse = run_attention(shape_of(cfg, max_seq_len=300, n_nodes=w), host, npar)
    assert np.abs(out - ref_out).max() <= 2e-2 and np.abs(lse - ref_lse).max() <= 1e-3
