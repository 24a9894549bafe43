#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
  D calls of ygg_equal_growth_expand, n_layers calls of ygg_tree_attention (one per layer, each
  layer with its own Q/K/V buffers), one call of ygg_accept_and_compact over all layers.
Inputs are seeded, synthetic and already resident in HBM when the timed region starts.

Prints ONE JSON line: the verify-step time per layer (whole step / n_layers), the roofline of the
dominant kernel (tree attention, timed with dispatch-bound HIP events on its own stream) and the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
FP32_VALU_PEAK_TFLOPS = 157.3


def attention_work(cfg, lens, kv_bytes=None):
    """Algorithmic bytes and flops of one tree-attention layer (kv_bytes: bytes of a stored K/V element
    when it differs from the element size of Q and O)."""
    e = 4 if cfg.dtype == "f32" else 2
    ekv = e if kv_bytes is None else kv_bytes
    N, Hq, Hkv, Dh, B = cfg.n_nodes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.batch
    sumL = int(np.sum(lens))
    nbytes = 2 * sumL * Hkv * Dh * ekv + 2 * B * N * Hkv * Dh * ekv + 2 * B * N * Hq * Dh * e
    flops = 4 * N * Hq * Dh * (sumL + B * N)
    return nbytes, flops


# HBM bytes per launch of the attention main kernel (fetched + written), from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs
# scaled by a streaming kernel of known size; a benchmark run cannot collect counters itself, so the figures measured with
# the commands recorded in profiles/attn_mfma_hbm_traffic.md are carried here, per workload configuration.
MEASURED_TRAFFIC_BYTES = {2: 26_075_033, 3: 37_865_267, 4: 177_698_509, 5: 329_497_497}


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload configuration 1..5")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attention-only", action="store_true", help="time only the attention calls of a step")
    ap.add_argument("--tree", default="", help="override the tree of the configuration: D,W (N = 1 + D*W nodes)")
    ap.add_argument("--heads", default="", help="override the head counts of the configuration: Hq,Hkv")
    ap.add_argument("--prefix", type=int, default=0, help="override the KV prefix length of the configuration (all sequences)")
    ap.add_argument("--batch", type=int, default=0, help="override the number of sequences of the configuration")
    ap.add_argument("--growth", choices=["frontier", "attach"], default="frontier",
                    help="draft-step rule: children of the previous depth only (default, the metric's definition) "
                         "or free attachment anywhere in the partial tree")
    ap.add_argument("--kv", choices=["native", "fp8"], default="native",
                    help="fp8: K/V stored as 8-bit E4M3 codes with per-kv-head scales (bf16 configurations, head_dim 128)")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every call from the host instead of replaying one captured HIP graph per step")
    ap.add_argument("--plan", default="", help="tuning: force the attention launch plan, waves,rblocks,nsplit,kshares (0 = library's choice)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB streaming kernel, dst = 2*src (reference point for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the design notes say how the path would shard",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_23858_amd as ygg
    import ygg_workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    ygg.load_library()  # fails loudly if libygg.so is missing
    if args.plan:
        ygg.set_attention_plan(*(int(x) for x in args.plan.split(",")))
    dev = "cuda:0"
    cfg = wl.CONFIGS[args.config]
    variant = ""
    if args.tree:
        d_, w_ = (int(x) for x in args.tree.split(","))
        cfg = wl.scaled(cfg, depth=d_, width=w_)
        variant += f" with tree {d_}x{w_}"
    if args.heads:
        hq_, hkv_ = (int(x) for x in args.heads.split(","))
        cfg = wl.scaled(cfg, n_q_heads=hq_, n_kv_heads=hkv_)
        variant += f" with heads {hq_}/{hkv_}"
    if args.prefix:
        cfg = wl.scaled(cfg, prefix_len=args.prefix, prefix_range=())
        variant += f" with prefix {args.prefix}"
    if args.batch:
        cfg = wl.scaled(cfg, batch=args.batch)
        variant += f" with batch {args.batch}"
    kv8 = args.kv == "fp8"
    if kv8:
        if cfg.dtype != "bf16" or cfg.head_dim != 128:
            print("bench.py: --kv fp8 needs a bf16 configuration with head_dim 128", file=sys.stderr)
            sys.exit(2)
        variant += " with 8-bit K/V"
    n_layers = args.layers or cfg.n_layers
    B, N, D, W, V = cfg.batch, cfg.n_nodes, cfg.depth, cfg.width, cfg.vocab
    Hkv, Dh, cap = cfg.n_kv_heads, cfg.head_dim, cfg.kv_capacity
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16

    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    # ---------------- inputs (host generator, then resident in HBM)
    lens_h = wl.seq_lens(cfg)
    parent_h = wl.trees(cfg)
    token_h = wl.tokens(cfg, parent_h)
    q = torch.empty((n_layers, B, N, cfg.n_q_heads, Dh), dtype=tdt, device=dev)
    kvdt = torch.uint8 if kv8 else tdt
    k_cache = torch.empty((n_layers, B, cap, Hkv, Dh), dtype=kvdt, device=dev)
    v_cache = torch.empty_like(k_cache)
    k_tree = torch.empty((n_layers, B, N, Hkv, Dh), dtype=kvdt, device=dev)
    v_tree = torch.empty_like(k_tree)
    k_scale = torch.ones((n_layers, Hkv), dtype=torch.float32, device=dev)
    v_scale = torch.ones_like(k_scale)
    layer0 = None
    for layer in range(n_layers):
        h = (wl.attention_inputs_fp8kv if kv8 else wl.attention_inputs)(cfg, layer=layer, lens=lens_h)
        if layer == 0:
            layer0 = h
        q[layer], k_cache[layer], v_cache[layer] = up(h["q"]), up(h["k_cache"]), up(h["v_cache"])
        k_tree[layer], v_tree[layer] = up(h["k_tree"]), up(h["v_tree"])
        if kv8:
            k_scale[layer], v_scale[layer] = up(h["k_scale"]), up(h["v_scale"])
    out = torch.empty_like(q)
    draft_h = [wl.expansion_inputs(cfg, d) for d in range(1, D + 1)]
    draft = [up(x) for x in draft_h]
    target_h = wl.acceptance_inputs(cfg, parent_h, token_h)
    target = up(target_h)
    parent, token = up(parent_h), up(token_h)
    lens0 = up(lens_h)
    lens = lens0.clone()
    e_parent = torch.full((B, N), -1, dtype=torch.int32, device=dev)
    e_token = torch.zeros((B, N), dtype=torch.int32, device=dev)
    e_cum = torch.zeros((B, N), dtype=torch.float32, device=dev)
    accept_len = torch.zeros((B,), dtype=torch.int32, device=dev)
    accept_path = torch.zeros((B, D + 1), dtype=torch.int32, device=dev)
    bonus = torch.zeros((B,), dtype=torch.int32, device=dev)

    shape = ygg.Shape(batch=B, n_q_heads=cfg.n_q_heads, n_kv_heads=Hkv, head_dim=Dh, depth=D, width=W, n_nodes=N,
                      vocab=V, kv_dtype=2 if kv8 else 0 if cfg.dtype == "f32" else 1, softmax_scale=cfg.softmax_scale,
                      kv_capacity=cap, max_seq_len=cfg.max_prefix)
    ws = [ygg.new_workspace(shape, op, n_layers, device=dev) for op in (ygg.OP_ATTENTION, ygg.OP_EXPAND, ygg.OP_ACCEPT)]

    ws_attach = pool = None
    if args.growth == "attach":
        ws_attach = ygg.new_workspace(shape, ygg.OP_ATTACH, device=dev)
        pool = torch.empty(ygg.attach_pool_bytes(shape), dtype=torch.uint8, device=dev)

    def attention_pass():
        for layer in range(n_layers):
            if kv8:
                ygg.tree_attention_fp8kv(shape, q[layer], k_cache[layer], v_cache[layer], lens, k_tree[layer],
                                         v_tree[layer], k_scale[layer], v_scale[layer], parent, out[layer], None, ws[0])
            else:
                ygg.tree_attention(shape, q[layer], k_cache[layer], v_cache[layer], lens, k_tree[layer], v_tree[layer],
                                   parent, out[layer], None, ws[0])

    def step():
        lens.copy_(lens0)   # acceptance advances seq_lens; every step starts from the same state
        for d in range(1, D + 1):
            if pool is None:
                ygg.equal_growth_expand(shape, d, draft[d - 1], e_parent, e_token, e_cum, ws[1])
            else:
                ygg.equal_growth_attach(shape, d, draft[d - 1], e_parent, e_token, e_cum, pool, ws_attach)
        attention_pass()
        ygg.accept_and_compact(shape, n_layers, parent, token, k_tree, v_tree, k_cache, v_cache, lens,
                               accept_len, accept_path, bonus, target_logits=target, workspace=ws[2])

    if args.calibrate_copy:  # 256 MiB read + 256 MiB written by a plain elementwise kernel (dst = 2 * src)
        src = torch.ones(256 * 1024 * 1024 // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    body = attention_pass if args.attention_only else step
    # All shapes are static and no call synchronises, so one step is captured once as a HIP graph and
    # replayed: the timed region then holds the kernels of K whole steps and no per-launch host work.
    eager_body = body
    host_us_per_step = None
    if not args.no_graph:
        for _ in range(2):
            eager_body()   # first launches (module load, kernel attributes) stay outside the capture
        torch.cuda.synchronize()
        t_h = time.perf_counter()
        eager_body()
        host_us_per_step = (time.perf_counter() - t_h) * 1e6  # host time to enqueue one step eagerly
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager_body()
        body = graph.replay
    for _ in range(args.warmup):
        body()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        body()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    # the same K steps once more, each between its own pair of events: the median over steps, beside the mean above
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        body()
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_per_step_median = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])

    # ---------------- the three calls on their own (graph replays), with their algorithmic rates
    def replay_us(fn, reps=20, inner=10):
        # `inner` back-to-back calls per graph, so that the gap between two graph launches is not billed to a short call
        def many():
            for _ in range(inner):
                fn()
        if args.no_graph:
            run = many
        else:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                many()
            run = g.replay
        for _ in range(3):
            run()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        for _ in range(reps):
            run()
        a1.record()
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) * 1e3 / (reps * inner)

    def grow_all():
        for d in range(1, D + 1):
            if pool is None:
                ygg.equal_growth_expand(shape, d, draft[d - 1], e_parent, e_token, e_cum, ws[1])
            else:
                ygg.equal_growth_attach(shape, d, draft[d - 1], e_parent, e_token, e_cum, pool, ws_attach)

    def accept_only():
        lens.copy_(lens0)
        ygg.accept_and_compact(shape, n_layers, parent, token, k_tree, v_tree, k_cache, v_cache, lens,
                               accept_len, accept_path, bonus, target_logits=target, workspace=ws[2])

    w_keep = max(1, (3 * N) // 4)
    p_kept = torch.zeros((B, w_keep), dtype=torch.int32, device=dev)
    p_par, p_tok = torch.zeros_like(p_kept), torch.zeros_like(p_kept)
    p_len = torch.zeros((B,), dtype=torch.float32, device=dev)
    p_best = torch.zeros((B,), dtype=torch.int32, device=dev)
    t_ver = torch.linspace(1.0, 2.0, N + 1, dtype=torch.float32, device=dev)

    def prune_only():   # pruning of the tree the growth calls left in e_parent / e_token / e_cum
        ygg.prune_for_verification(shape, w_keep, e_parent, e_token, e_cum, p_kept, p_par, p_tok, p_len, p_best,
                                   t_verifier=t_ver, t_draft=1.0)

    ops = None
    if not args.attention_only:
        grow_us = replay_us(grow_all)
        acc_us = replay_us(accept_only)
        att_us = replay_us(attention_pass, inner=1)
        grow_bytes = sum(int(x.numel()) * 4 for x in draft)           # every draft logit read once
        acc_bytes = int(target.numel()) * 4                            # every target logit read once
        ops = {"growth_us_per_draft_step": round(grow_us / D, 2), "growth_gbps": round(grow_bytes / (grow_us * 1e-6) / 1e9, 1),
               "accept_us_per_call": round(acc_us, 2), "accept_argmax_gbps": round(acc_bytes / (acc_us * 1e-6) / 1e9, 1),
               "attention_us_per_layer": round(att_us / n_layers, 2),
               "prune_us_per_call": round(replay_us(prune_only), 2), "prune_keeps": w_keep}

    # ---------------- dominant kernel: same launches again with dispatch-bound events
    ygg.profile_begin(args.steps * n_layers)
    for _ in range(args.steps):
        eager_body()
    kern_us, kern_n = ygg.profile_end()
    nbytes, flops = attention_work(cfg, lens_h, kv_bytes=1 if kv8 else None)
    t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
    if cfg.dtype == "f32":
        bound, peak, unit, ach = "alu", FP32_VALU_PEAK_TFLOPS, "TFLOP/s", flops / (kern_us * 1e-6) / 1e12
    elif flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) > t_hbm:
        bound, peak, unit, ach = "mfma", MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", flops / (kern_us * 1e-6) / 1e12
    else:
        bound, peak, unit, ach = "hbm", HBM_PEAK_GBS, "GB/s", nbytes / (kern_us * 1e-6) / 1e9
    roofline = {"bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                "traffic": None if variant else MEASURED_TRAFFIC_BYTES.get(args.config), "kernel": "tree attention main kernel", "kernel_us": round(kern_us, 3),
                "launches_timed": kern_n, "algorithmic_bytes": nbytes, "flops": flops,
                "frac_of_hbm_peak": round(nbytes / (kern_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                "frac_of_mfma_bf16_peak": None if cfg.dtype == "f32" else round(flops / (kern_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "gbps": round(nbytes / (kern_us * 1e-6) / 1e9, 1), "tflops": round(flops / (kern_us * 1e-6) / 1e12, 2)}

    # ---------------- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        rows_all = B * N * cfg.n_q_heads
        # attention: time a sample of output rows of layer 0 sized for roughly 10 s, scale to all rows and layers
        t = time.perf_counter()
        probe = min(rows_all, 4 * threads)
        rs = np.random.default_rng(0).choice(rows_all, size=probe, replace=False)
        def run_rows(sel):
            # the oracle's full routine parallelises over rows; sampled rows go through the row routine
            for r in sel:
                b_, i_, h_ = r // (N * cfg.n_q_heads), (r // cfg.n_q_heads) % N, r % cfg.n_q_heads
                if kv8:
                    oracle.attention_row_fp8kv(layer0["q"], layer0["k_cache"], layer0["v_cache"], lens_h, layer0["k_tree"],
                                               layer0["v_tree"], layer0["k_scale"], layer0["v_scale"], parent_h,
                                               cfg.softmax_scale, int(b_), int(i_), int(h_))
                else:
                    oracle.attention_row(layer0["q"], layer0["k_cache"], layer0["v_cache"], lens_h, layer0["k_tree"],
                                         layer0["v_tree"], parent_h, cfg.softmax_scale, int(b_), int(i_), int(h_))
        run_rows(rs)
        per_row_serial = (time.perf_counter() - t) / probe
        est_full = per_row_serial * rows_all / threads
        if est_full <= 20.0:
            t = time.perf_counter()
            if kv8:
                oracle.tree_attention_fp8kv(layer0["q"], layer0["k_cache"], layer0["v_cache"], lens_h, layer0["k_tree"],
                                            layer0["v_tree"], layer0["k_scale"], layer0["v_scale"], parent_h,
                                            cfg.softmax_scale)
            else:
                oracle.tree_attention(layer0["q"], layer0["k_cache"], layer0["v_cache"], lens_h, layer0["k_tree"],
                                      layer0["v_tree"], parent_h, cfg.softmax_scale)
            t_attn_layer = time.perf_counter() - t
            attn_note = "attention: all rows of layer 0 (OpenMP over rows)"
        else:
            t_attn_layer = est_full
            attn_note = (f"attention: {probe} sampled rows of layer 0 run serially, scaled to {rows_all} rows "
                         f"and {threads} threads")
        # expansion: all D steps; acceptance: argmax + match + compaction of one layer
        p2 = np.full((B, N), -1, np.int32); t2 = np.zeros((B, N), np.int32); c2 = np.zeros((B, N), np.float32)
        t = time.perf_counter()
        for d in range(1, D + 1):
            oracle.expand(D, W, d, draft_h[d - 1], p2, t2, c2)
        t_expand = time.perf_counter() - t
        kt1 = np.ascontiguousarray(layer0["k_tree"][None]); vt1 = np.ascontiguousarray(layer0["v_tree"][None])
        kc1 = np.ascontiguousarray(layer0["k_cache"][None]); vc1 = np.ascontiguousarray(layer0["v_cache"][None])
        t = time.perf_counter()
        oracle.accept_compact(D + 1, parent_h, token_h, kt1, vt1, kc1, vc1, lens_h.copy(), target_logits=target_h)
        t_accept = time.perf_counter() - t
        if args.attention_only:
            cpu_step = n_layers * t_attn_layer
        else:
            cpu_step = t_expand + n_layers * t_attn_layer + t_accept
        cpu = {"value": round(cpu_step / n_layers * 1e6, 1), "unit": "us/layer", "cores": threads, "cpu_model": cpu_model(), "kind": "oracle",
               "sample": f"{attn_note}; expansion: all {D} steps; acceptance: argmax+match+1-layer compaction; "
                         f"step = expand + {n_layers} x attention layer + accept",
               "attention_layer_s": round(t_attn_layer, 4), "expand_s": round(t_expand, 4),
               "accept_s": round(t_accept, 4)}

    rec = {
        # the headline metric's first part is `value`; its second part (achieved HBM TB/s and MFMA % of the attention
        # main kernel) is spelled out in the two fields after `unit` and in `roofline`
        "metric": "verify-step µs per layer + achieved HBM TB/s and MFMA % for tree attention",
        "value": round(ms_per_step * 1e3 / n_layers, 3), "unit": "µs/layer",
        "value_definition": "one whole verification step (D growth calls + `layers` attention calls + accept/compact) divided by layers",
        "attention_hbm_tb_s": round(nbytes / (kern_us * 1e-6) / 1e12, 3),
        "attention_mfma_pct_of_bf16_dense_peak": None if cfg.dtype == "f32" else round(100 * flops / (kern_us * 1e-6) / (MFMA_BF16_PEAK_TFLOPS * 1e12), 2),
        "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "ms_per_step_median": round(ms_per_step_median, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}] {cfg.name}{variant}", "batch": B, "q_heads": cfg.n_q_heads,
                   "kv_heads": Hkv, "head_dim": Dh, "prefix": cfg.prefix_len or list(cfg.prefix_range),
                   "tree": f"depth {D} x width {W} + root = {N} nodes", "vocab": V, "layers": n_layers,
                   "scope": "attention only" if args.attention_only else "full step"},
        "wall_ms_timed_region": round(wall_ms, 2),
        "growth": args.growth,
        "calls": ops,
        "launch": "eager" if args.no_graph else "hip-graph replay of one captured step",
        "host_enqueue_us_per_step_eager": None if host_us_per_step is None else round(host_us_per_step, 1),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
