"""Randomized parity over shapes the hand-picked cases do not name: one fixed seed, so the run is repeatable.

Attention (bf16 / fp32, batches of 1 to 6 ragged sequences incl. empty prefixes, level trees and arbitrary topological
ones, 1 to 8 kv heads x group sizes 1 to 8) against the oracle at the contractual bounds, with poisoned workspaces
draft
growth by both rules, pruning and acceptance bit for bit.  The same generators, with more seeds and wider ranges, were run
by hand against the kernels
this is the part that stays in the suite.
"""
import numpy as np
import pytest

import oracle
import ygg_workloads as wl
from gpu_util import run_attention, shape_of
from test_gpu_attach import attach_both
from test_gpu_expand_accept import _accept_both, _expand_both
from test_gpu_prune import _latency, prune_both

pytestmark = pytest.mark.gpu


def test_random_attention_shapes(n_cases=120):
    rng = np.random.default_rng(20251223)
    for it in range(n_cases):
        Hkv = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 2, 4, 8]))
        Hq = Hkv * G
        D = int(rng.integers(1, 9))
        W = int(rng.integers(1, 17))
        if (1 + D * W) > 300: W = 300 // D
        B = int(rng.integers(1, 7))
        maxL = int(rng.choice([0, 1, 50, 64, 200, 777, 2000, 5000]))
        lens = [int(rng.integers(0, maxL + 1)) for _ in range(B)]
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        Dh = 128 if rng.random() < (0.7 if dtype == "bf16" else 0.5) else 64
        cfg = wl.Config("case", B, Hq, Hkv, Dh, dtype, max(maxL, 1), (), D, W, 100, (0.5,), "dirichlet", 0.5, 1, 1000 + it)
        la = np.asarray(lens, np.int32)
        host = wl.attention_inputs(cfg, lens=la)
        parent = wl.trees(cfg) if rng.random() < 0.7 else np.stack([wl.random_topological_tree(it * 7 + b, cfg.n_nodes) for b in range(B)]).astype(np.int32)
        depth = cfg.n_nodes - 1
        shape = shape_of(cfg, max_seq_len=max(maxL, 1), kv_capacity=max(maxL, 1) + depth + 1)
        shape.depth = depth
        # the generator sized the cache for cfg.kv_capacity; rebuild caches with the capacity passed
        cap = shape.kv_capacity
        for k in ("k_cache", "v_cache"):
            full = wl.normal(cfg.seed, 3 if k == "k_cache" else 4, (B, cap, Hkv, Dh), dtype)
            full[:, :min(cap, host[k].shape[1])] = host[k][:, :min(cap, host[k].shape[1])]
            host[k] = full
        ref, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], la, host["k_tree"], host["v_tree"], parent, cfg.softmax_scale)
        out, lse = run_attention(shape, host, parent, poison=0xFF if it % 2 else 0xA5)
        err = np.abs(out - ref).max()
        tol = 1e-5 if dtype == "f32" else 2e-2
        print(f"shape {it}: B{B} Hq{Hq} Hkv{Hkv} Dh{Dh} {dtype} D{D} W{W} lens{lens} err {err:.2e}", flush=True)
        assert err <= tol and np.abs(lse - ref_lse).max() <= (1e-5 if dtype == "f32" else 1e-3)


def test_random_growth_pruning_and_acceptance_shapes(n_cases=24):
    rng = np.random.default_rng(20251224)
    for it in range(n_cases):
        B = int(rng.integers(1, 4))
        D = int(rng.integers(1, 7))
        W = int(rng.integers(1, 33))
        V = int(rng.choice([W + 3, 500, 4096, 4097, 9000, 33000]))
        V = max(V, W)
        cfg = wl.Config("case", B, 4, 2, 64, "bf16", 16, (), D, W, V, (0.6,), "dirichlet", 0.5, 1, 2000 + it)
        print(f"grow {it}: B{B} D{D} W{W} V{V}", flush=True)
        parent, token, cum = _expand_both(cfg)
        p2, t2, c2 = attach_both(cfg)
        N = cfg.n_nodes
        for w in sorted({1, max(1, N // 2), N}):
            prune_both(cfg, p2, t2, c2, w, _latency(N, max(1, N // 3), 0.07), 0.4)
        lens = rng.integers(0, 30, size=B)
        logits = wl.acceptance_inputs(wl.scaled(cfg, agree=(0.8,)), parent, token)
        _accept_both(cfg, parent, token, int(rng.integers(0, 3)), lens, logits=logits)
