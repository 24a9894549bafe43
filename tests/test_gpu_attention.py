"""GPU parity of tree attention against the CPU oracle, through the C ABI.

bf16 cases: the contractual bound (2e-2 max-abs, 1e-2 mean-abs) cannot see a wrong ancestor mask
on N(0,1) inputs, so every case also has to pass two tighter gates: error relative to the
oracle's RMS <= 2 % and LSE within 1e-3; the short-prefix and tree-heavy cases make the tree keys
carry most of the softmax mass.
"""
import numpy as np
import pytest

import oracle
import ygg_workloads as wl
from gpu_util import run_attention, shape_of

pytestmark = pytest.mark.gpu


def _cfg(B, Hq, Hkv, D, W, dtype="bf16", Dh=128, seed=77):
    return wl.Config("case", B, Hq, Hkv, Dh, dtype, 0, (), D, W, 100, (0.5,), "dirichlet", 0.5, 1, seed)


def _inputs(cfg, lens, max_len, parent=None, tree_gain=1.0):
    lens = np.asarray(lens, np.int32)
    cfg = wl.scaled(cfg, prefix_len=int(max_len))
    host = wl.attention_inputs(cfg, lens=lens)
    if parent is None:
        parent = wl.trees(cfg)
    if tree_gain != 1.0:   # make the tree's own keys dominate the softmax
        k = wl.storage_to_f64(host["k_tree"]) * tree_gain
        host["k_tree"] = wl.to_storage(k.astype(np.float32), cfg.dtype)
    return cfg, host, parent


def _check(cfg, host, parent, max_len, n_nodes=None, depth=None):
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"],
                                             host["k_tree"], host["v_tree"], parent, cfg.softmax_scale)
    shape = shape_of(cfg, max_seq_len=int(max_len), n_nodes=n_nodes)
    if depth is not None:
        shape.depth = depth
        shape.kv_capacity = max(shape.kv_capacity, int(max_len) + depth + 1)
    out, lse = run_attention(shape, host, parent)
    err = np.abs(out - ref_out)
    if cfg.dtype == "f32":
        assert err.max() <= 1e-5, err.max()
        assert np.abs(lse - ref_lse).max() <= 1e-5
    else:
        # 2e-2 everywhere, except where that is less than one bf16 unit in the last place of the exact value (2^-7 of it
        # at most, i.e. for outputs above 2.56): the output is stored in bf16 (half a unit) and so are the softmax weights
        # (a quarter more when one key holds all the mass).  N(0,1) values average far below that; only the tree-heavy
        # cases, whose rows copy single V rows, can reach it.
        bound = np.maximum(2e-2, 2.0 ** -7 * np.abs(ref_out))
        worst = np.unravel_index(np.argmax(err - bound), err.shape)
        assert (err <= bound).all() and err.mean() <= 1e-2, (err[worst], ref_out[worst], out[worst], err.mean())
        rms = np.sqrt((ref_out ** 2).mean())
        assert np.sqrt((err ** 2).mean()) <= 0.02 * rms, (np.sqrt((err ** 2).mean()), rms)
        assert np.abs(lse - ref_lse).max() <= 1e-3, np.abs(lse - ref_lse).max()


# (B, Hq, Hkv, D, W, lens, max_len): query rows per kv head R = (1+D*W)*Hq/Hkv select the workgroup shape
BF16_CASES = [
    (1, 4, 4, 3, 4, [128], 128),            # R = 13, one key split
    (2, 8, 8, 6, 8, [300, 1], 300),         # R = 49, ragged batch
    (1, 8, 2, 4, 6, [130], 130),            # R = 100
    (2, 8, 2, 8, 4, [200, 77], 333),        # R = 132, max_seq_len above every length
    (1, 16, 2, 5, 6, [257], 257),           # R = 248
    (1, 8, 2, 10, 9, [65], 65),             # R = 364
    (1, 4, 1, 10, 15, [190], 190),          # R = 604
    (1, 8, 8, 6, 8, [1500], 1500),          # several key splits, partial last tile
    (3, 8, 2, 3, 4, [700, 0, 64], 700),     # several splits with an empty and a one-tile sequence
    (1, 40, 40, 8, 8, [1024], 1024),        # 13B-shaped layer (40 heads) with the paper's best static tree, 8 x 8
    (1, 40, 40, 16, 8, [333], 333),         # ... and its fixed baseline tree, 16 x 8 (R = 129)
    (1, 2, 2, 33, 31, [100], 100),          # the largest tree, N = 1024: ancestor masks of 32 words per node
    (1, 8, 1, 1023, 1, [40], 40),           # N = 1024 as one chain (depth 1023) under one kv head: R = 8192
]


@pytest.mark.parametrize("case", BF16_CASES, ids=lambda c: f"B{c[0]}_Hq{c[1]}_Hkv{c[2]}_D{c[3]}W{c[4]}_L{max(c[5])}")
def test_bf16_shapes(case):
    B, Hq, Hkv, D, W, lens, max_len = case
    cfg, host, parent = _inputs(_cfg(B, Hq, Hkv, D, W), lens, max_len)
    _check(cfg, host, parent, max_len)


# Batches of wide trees (more than 128 query rows per kv head) run "balanced": the key tiles of all sequences are laid end
# to end and cut into equal runs, so a workgroup may serve the tail of one sequence, whole short ones and the head of
# another.  (B, Hq, Hkv, D, W, lens, max_len)
RAGGED_BATCHES = [
    (5, 16, 2, 6, 8, [900, 0, 64, 1500, 333], 1500),          # R = 392, two row tiles; an empty and a one-tile prefix
    (2, 16, 2, 6, 8, [700, 700], 700),                        # equal lengths: every run lies inside one sequence
    (3, 16, 2, 6, 8, [0, 0, 0], 64),                          # fewer key tiles than runs
    (4, 8, 1, 8, 16, [2000, 15, 15, 15], 2048),               # one long sequence spans nearly every run; R = 1032
    (16, 8, 2, 6, 8, [37 * i % 601 for i in range(16)], 640), # many short sequences per run; R = 196
    (7, 32, 4, 5, 6, [511, 512, 513, 1, 1023, 1024, 1025], 1100),   # lengths around tile boundaries; R = 248
    (2, 8, 2, 10, 12, [3000, 100], 3000),                     # R = 484: a sequence whose length equals max_seq_len
    (6, 16, 4, 8, 12, [38, 13, 16, 23, 2, 21], 50),           # lengths far below the bound: the grid holds more runs than
                                                              # there are tiles, and sequences of two or three tiles
]


@pytest.mark.parametrize("case", RAGGED_BATCHES, ids=lambda c: f"B{c[0]}_Hq{c[1]}_Hkv{c[2]}_D{c[3]}W{c[4]}_L{max(c[5])}")
@pytest.mark.parametrize("gain", [1.0, 4.0])
def test_bf16_ragged_batches_in_balanced_runs(case, gain):
    import paper_2512_23858_amd as ygg
    B, Hq, Hkv, D, W, lens, max_len = case
    cfg, host, parent = _inputs(_cfg(B, Hq, Hkv, D, W, seed=123), lens, max_len, tree_gain=gain)
    plan = ygg.attention_plan(shape_of(cfg, max_seq_len=int(max_len)))
    assert plan["matrix_cores"] and plan["key_shares"] == 1 and plan["key_splits"] * Hkv * plan["row_tiles"] <= 256
    _check(cfg, host, parent, max_len)


@pytest.mark.parametrize("L", [0, 1, 31, 32, 33, 63, 64, 65])
@pytest.mark.parametrize("gain", [1.0, 4.0])
def test_bf16_short_prefix_and_tree_heavy(L, gain):
    cfg, host, parent = _inputs(_cfg(1, 8, 2, 5, 7, seed=91), [L], max(L, 1), tree_gain=gain)
    _check(cfg, host, parent, max(L, 1))


@pytest.mark.parametrize("v_scale", [2.0 ** -20, 2.0 ** 18])
def test_bf16_split_partials_keep_their_precision_for_any_range_of_v(v_scale):
    """Several key splits and V far outside what fp16 could hold as such (about 2.6e5) or far below its normal range:
    the split partials are stored relative to each row's own magnitude, so the error bounds simply scale with V."""
    cfg, host, parent = _inputs(_cfg(1, 8, 2, 6, 8, seed=95), [1500], 1500)
    for name in ("v_cache", "v_tree"):   # a power of two: exact in bf16
        host[name] = wl.to_storage((wl.storage_to_f64(host[name]) * v_scale).astype(np.float32), cfg.dtype)
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"],
                                             host["k_tree"], host["v_tree"], parent, cfg.softmax_scale)
    import paper_2512_23858_amd as ygg
    shape = shape_of(cfg, max_seq_len=1500)
    assert ygg.attention_plan(shape)["key_splits"] > 1
    out, lse = run_attention(shape, host, parent)
    assert np.isfinite(out).all()
    err = np.abs(out - ref_out) / v_scale
    assert err.max() <= 2e-2 and err.mean() <= 1e-2, (err.max(), err.mean())
    assert np.abs(lse - ref_lse).max() <= 1e-3


@pytest.mark.parametrize("lens,max_len", [([700], 700), ([900, 130, 415], 900)])
def test_bf16_scores_far_above_and_below_the_softmax_reference(lens, max_len):
    """The kernel keeps a per-row softmax reference that only moves when a block's weights outgrow it by 2^30.  Here
    the first keys of the prefix score far above the bulk (everything after them underflows against the reference
    they set) and the tree's own keys, which come last, far above those again (the reference has to move mid-stream,
    with the accumulated output rescaled)."""
    cfg, host, parent = _inputs(_cfg(len(lens), 8, 2, 6, 8, seed=96), lens, max_len, tree_gain=14.0)
    k = wl.storage_to_f64(host["k_cache"])
    k[:, :40] *= 9.0
    host["k_cache"] = wl.to_storage(k.astype(np.float32), cfg.dtype)
    _check(cfg, host, parent, max_len)


def test_bf16_chain_and_general_tree():
    N = 45
    for parent in (wl.chain_tree(N)[None], wl.random_topological_tree(5, N)[None]):
        cfg, host, _ = _inputs(_cfg(1, 8, 4, 4, 11, seed=92), [150], 150, parent=parent, tree_gain=3.0)
        _check(cfg, host, parent, 150, depth=N - 1)


def test_bf16_single_node_tree():
    cfg = wl.Config("decode", 2, 8, 2, 128, "bf16", 0, (), 0, 1, 100, (0.5,), "uniform", 0.0, 1, 93)
    cfg, host, parent = _inputs(cfg, [100, 259], 259)
    _check(cfg, host, parent, 259)


@pytest.mark.parametrize("case", [(1, 4, 4, 3, 4, [128], 128, 64), (2, 8, 2, 4, 6, [200, 77], 200, 128),
                                  (1, 8, 8, 6, 8, [1500], 1500, 128), (1, 4, 2, 5, 7, [0], 1, 64)],
                         ids=["tiny", "gqa_ragged", "splits", "empty_prefix"])
def test_fp32_shapes(case):
    B, Hq, Hkv, D, W, lens, max_len, Dh = case
    cfg, host, parent = _inputs(_cfg(B, Hq, Hkv, D, W, dtype="f32", Dh=Dh, seed=94), lens, max_len)
    _check(cfg, host, parent, max_len)


# head_dim 64 on the matrix cores: every workgroup shape (by query rows per kv head), classic key splits and balanced runs,
# an empty prefix, a partial last tile.  (B, Hq, Hkv, D, W, lens, max_len)
BF16_HEAD_DIM_64 = [
    (1, 4, 2, 3, 4, [90], 90),                                # R = 26: two wavefronts in a pair
    (2, 8, 8, 6, 8, [300, 1], 300),                           # R = 49: four wavefronts in pairs, ragged batch
    (1, 8, 2, 4, 6, [130], 130),                              # R = 100: eight wavefronts in pairs
    (1, 12, 2, 5, 5, [1500], 1500),                           # R = 156: 192-row shape, several key splits, partial last tile
    (1, 16, 2, 5, 6, [257], 257),                             # R = 248: 256-row shape
    (1, 4, 1, 10, 15, [0], 1),                                # R = 604: three row tiles, tree keys only
    (1, 12, 12, 8, 8, [2048], 2048),                          # a draft-model-sized layer (12 heads of 64), 8 x 8 tree
    (5, 16, 2, 6, 8, [900, 0, 64, 1500, 333], 1500),          # balanced runs, R = 392
    (6, 16, 4, 8, 12, [38, 13, 16, 23, 2, 21], 50),           # balanced runs, more runs than tiles
    (1, 2, 2, 33, 31, [100], 100),                            # N = 1024
]


@pytest.mark.parametrize("case", BF16_HEAD_DIM_64, ids=lambda c: f"B{c[0]}_Hq{c[1]}_Hkv{c[2]}_D{c[3]}W{c[4]}_L{max(c[5])}")
@pytest.mark.parametrize("gain", [1.0, 4.0])
def test_bf16_head_dim_64_shapes(case, gain):
    import paper_2512_23858_amd as ygg
    B, Hq, Hkv, D, W, lens, max_len = case
    cfg, host, parent = _inputs(_cfg(B, Hq, Hkv, D, W, Dh=64, seed=95), lens, max_len, tree_gain=gain)
    assert ygg.attention_plan(shape_of(cfg, max_seq_len=int(max_len)))["matrix_cores"]
    _check(cfg, host, parent, max_len)


@pytest.mark.parametrize("L", [0, 1, 31, 32, 33, 63, 64, 65])
def test_bf16_head_dim_64_short_prefix(L):
    cfg, host, parent = _inputs(_cfg(1, 8, 2, 5, 7, Dh=64, seed=96), [L], max(L, 1), tree_gain=4.0)
    _check(cfg, host, parent, max(L, 1))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_empty_key_splits_ignore_whatever_the_workspace_holds(dtype):
    """A sequence much shorter than max_seq_len leaves key splits empty: their slots of the workspace are never
    written and may hold NaN bit patterns, which the merge must not touch."""
    cfg, host, parent = _inputs(_cfg(3, 8, 2, 3, 4, dtype=dtype, seed=96), [700, 0, 64], 700)
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"],
                                             host["k_tree"], host["v_tree"], parent, cfg.softmax_scale)
    shape = shape_of(cfg, max_seq_len=700)
    out, lse = run_attention(shape, host, parent, poison=0xFF)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.abs(out - ref_out).max() <= tol


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_is_deterministic(dtype):
    """Same inputs, two launches with differently poisoned workspaces: outputs and LSE agree bit for bit (the key splits
    are merged in a fixed order and nothing is accumulated with atomics)."""
    cfg, host, parent = _inputs(_cfg(2, 8, 2, 6, 8, dtype=dtype, seed=97), [1500, 321], 1500)
    shape = shape_of(cfg, max_seq_len=1500)
    a_out, a_lse = run_attention(shape, host, parent, poison=0xA5)
    b_out, b_lse = run_attention(shape, host, parent, poison=0x00)
    assert np.array_equal(a_out, b_out) and np.array_equal(a_lse, b_lse)


@pytest.mark.parametrize("dtype,Dh", [("bf16", 128), ("f32", 64)])
def test_empty_cache_with_null_cache_pointers(dtype, Dh):
    """First step after an empty prompt: max_seq_len = 0, so the caches may be NULL; every node sees only its
    ancestors and itself."""
    import torch
    import paper_2512_23858_amd as ygg
    from gpu_util import DEV, to_dev, to_f64, workspace
    cfg, host, parent = _inputs(_cfg(2, 8, 4, 4, 5, dtype=dtype, Dh=Dh), [0, 0], 0)
    ref_out, ref_lse = oracle.tree_attention(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"],
                                             host["k_tree"], host["v_tree"], parent, cfg.softmax_scale)
    shape = shape_of(cfg, max_seq_len=0)
    d = {k: to_dev(np.ascontiguousarray(v)) for k, v in host.items()}
    out = torch.full_like(d["q"], float("nan"))
    lse = torch.full(d["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ygg.tree_attention(shape, d["q"], None, None, d["seq_lens"], d["k_tree"], d["v_tree"], to_dev(parent), out, lse,
                       workspace(shape, ygg.OP_ATTENTION))
    torch.cuda.synchronize()
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.abs(to_f64(out) - ref_out).max() <= tol
    assert np.abs(to_f64(lse) - ref_lse).max() <= (1e-5 if dtype == "f32" else 1e-3)
