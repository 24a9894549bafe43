"""GPU parity of tree attention with 8-bit (E4M3) K/V against the CPU oracle, through the C ABI.

The kernel widens the codes to bf16 exactly, so the bounds are those of the bf16 kernel: 2e-2
max-abs, 1e-2 mean-abs, and the two tighter gates (error <= 2 % of the oracle's RMS, LSE within
1e-3) that can see a wrong ancestor mask, a wrong scale or a code converted in the wrong order.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev, to_f64, workspace

pytestmark = pytest.mark.gpu


def _cfg(B, Hq, Hkv, D, W, seed=91):
    return wl.Config("case", B, Hq, Hkv, 128, "bf16", 0, (), D, W, 100, (0.5,), "dirichlet", 0.5, 1, seed)


def _inputs(cfg, lens, max_len, parent=None):
    lens = np.asarray(lens, np.int32)
    cfg = wl.scaled(cfg, prefix_len=int(max_len))
    host = wl.attention_inputs_fp8kv(cfg, lens=lens)
    return cfg, host, (wl.trees(cfg) if parent is None else parent)


def _shape(cfg, max_len, n_nodes=None, depth=None):
    shape = shape_of(cfg, max_seq_len=int(max_len), n_nodes=n_nodes)
    shape.kv_dtype = ygg.FP8_E4M3
    if depth is not None:
        assert cfg.batch == 1, "a capacity other than the arrays' is only harmless for a single sequence"
        shape.depth = depth
        shape.kv_capacity = max(shape.kv_capacity, int(max_len) + depth + 1)
    return shape


def _run(shape, host, parent, poison=0xA5):
    d = {k: to_dev(np.ascontiguousarray(v)) for k, v in host.items()}
    par = to_dev(np.ascontiguousarray(parent))
    out = torch.full_like(d["q"], float("nan"))
    lse = torch.full(d["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(shape, ygg.OP_ATTENTION, poison=poison)
    ygg.tree_attention_fp8kv(shape, d["q"], d["k_cache"], d["v_cache"], d["seq_lens"], d["k_tree"], d["v_tree"],
                             d["k_scale"], d["v_scale"], par, out, lse, ws)
    torch.cuda.synchronize()
    return to_f64(out), to_f64(lse)


def _oracle(cfg, host, parent):
    return oracle.tree_attention_fp8kv(host["q"], host["k_cache"], host["v_cache"], host["seq_lens"], host["k_tree"],
                                       host["v_tree"], host["k_scale"], host["v_scale"], parent, cfg.softmax_scale)


def _check(cfg, host, parent, max_len, n_nodes=None, depth=None):
    ref_out, ref_lse = _oracle(cfg, host, parent)
    out, lse = _run(_shape(cfg, max_len, n_nodes, depth), host, parent)
    err = np.abs(out - ref_out)
    assert err.max() <= 2e-2 and err.mean() <= 1e-2, (err.max(), err.mean())
    rms = np.sqrt((ref_out ** 2).mean())
    assert np.sqrt((err ** 2).mean()) <= 0.02 * rms, (np.sqrt((err ** 2).mean()), rms)
    assert np.abs(lse - ref_lse).max() <= 1e-3, np.abs(lse - ref_lse).max()


# (B, Hq, Hkv, D, W, lens, max_len): R = (1+D*W)*Hq/Hkv picks 2 or 4 computing wavefronts, paired or not
CASES = [
    (1, 4, 4, 3, 4, [128], 128),            # R = 13: two wavefronts in a pair, one key split
    (2, 8, 8, 6, 8, [300, 1], 300),         # R = 49: four wavefronts in pairs, ragged batch
    (1, 8, 2, 4, 6, [130], 130),            # R = 100: four wavefronts, 128 rows
    (2, 8, 2, 8, 4, [200, 77], 333),        # R = 132: two row tiles, max_seq_len above every length
    (1, 16, 2, 5, 6, [257], 257),           # R = 248
    (1, 8, 2, 10, 9, [65], 65),             # R = 364: three row tiles
    (3, 4, 2, 2, 3, [1000, 513, 64], 1000), # several key splits per sequence, short tree
    (1, 8, 8, 6, 8, [1024], 1024),          # the 7B-shaped tree on a reduced head count
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"B{c[0]}_Hq{c[1]}_Hkv{c[2]}_D{c[3]}W{c[4]}_L{max(c[5])}")
def test_shapes(case):
    B, Hq, Hkv, D, W, lens, max_len = case
    cfg, host, parent = _inputs(_cfg(B, Hq, Hkv, D, W), lens, max_len)
    _check(cfg, host, parent, max_len)


@pytest.mark.parametrize("L", [0, 1, 31, 63, 64, 65, 191, 449])
def test_short_prefix_and_tile_boundaries(L):
    """Prefix lengths around the 64-key tiles: the tree keys straddle tiles, splits end raggedly, and with
    few tiles the loaders' look-ahead reaches past the end of the split."""
    cfg, host, parent = _inputs(_cfg(2, 8, 4, 5, 7, seed=5 + L), [L, max(L - 3, 0)], L)
    _check(cfg, host, parent, L)


def test_chain_general_tree_and_single_node():
    cfg, host, _ = _inputs(_cfg(1, 8, 4, 12, 1), [150], 150)
    _check(cfg, host, wl.chain_tree(13)[None], 150)
    cfg, host, _ = _inputs(_cfg(1, 4, 2, 4, 5), [99], 99)
    _check(cfg, host, wl.random_topological_tree(3, 21)[None], 99)
    cfg = wl.scaled(_cfg(1, 8, 8, 0, 1), prefix_len=200)
    host = wl.attention_inputs_fp8kv(cfg, lens=np.array([200], np.int32))
    _check(cfg, host, np.array([[-1]], np.int32), 200, n_nodes=1, depth=0)


def test_largest_tree():
    N = 1024
    cfg = wl.scaled(_cfg(1, 4, 2, 1, 1), prefix_len=300)
    cfg = wl.scaled(cfg, depth=31, width=33)
    assert cfg.n_nodes == N
    host = wl.attention_inputs_fp8kv(cfg, lens=np.array([300], np.int32))
    _check(cfg, host, wl.random_topological_tree(11, N)[None], 300, depth=N - 1)


def test_every_code_and_distinct_scales():
    """All 254 finite codes occur in K and V, scales differ per kv head and between K and V (one of them a
    power of two, one far from 1): a code widened wrongly, or a scale taken from the wrong head or
    tensor, moves the result by far more than the bound."""
    cfg, host, parent = _inputs(_cfg(1, 8, 4, 3, 5), [260], 260)
    r = np.random.default_rng(3)
    finite = np.delete(np.arange(256, dtype=np.uint8), [0x7F, 0xFF])
    for name in ("k_cache", "v_cache", "k_tree", "v_tree"):
        codes = r.choice(finite, size=host[name].shape)
        if name[0] == "k":   # keep the scores moderate: small magnitudes dominate, every code still present
            small = r.choice(finite[(finite & 0x7F) < 0x48], size=host[name].shape)
            codes = np.where(r.random(host[name].shape) < 0.97, small, codes)
        host[name] = codes.astype(np.uint8)
    for kind in "kv":
        assert np.unique(np.concatenate([host[kind + "_cache"].ravel(), host[kind + "_tree"].ravel()])).size == 254
    host["k_scale"] = np.array([0.25, 0.11, 0.4, 0.07], np.float32)
    host["v_scale"] = np.array([0.003, 0.02, 2.0 ** -7, 0.011], np.float32)
    ref_out, ref_lse = _oracle(cfg, host, parent)
    out, lse = _run(_shape(cfg, 260), host, parent)
    err = np.abs(out - ref_out)
    rms = np.sqrt((ref_out ** 2).mean())
    assert np.sqrt((err ** 2).mean()) <= 0.02 * rms and err.max() <= 0.1 * rms + 2e-2, (err.max(), rms)
    assert np.abs(lse - ref_lse).max() <= 2e-3


def test_matches_bf16_kernel_on_dequantised_inputs():
    """With power-of-two scales the dequantised K/V are exact bf16 numbers: the bf16 entry point on them and
    the 8-bit entry point on the codes do the same matrix work and may differ only where a scale enters
    the fp32 arithmetic, i.e. by a rounding of the bf16 result."""
    cfg, host, parent = _inputs(_cfg(2, 8, 4, 6, 8), [700, 333], 700)
    host["k_scale"] = np.array([2.0 ** -6, 2.0 ** -7, 2.0 ** -6, 2.0 ** -5], np.float32)
    host["v_scale"] = np.array([2.0 ** -7, 2.0 ** -6, 2.0 ** -8, 2.0 ** -6], np.float32)
    out8, lse8 = _run(_shape(cfg, 700), host, parent)
    deq = {}
    for name in ("k_cache", "v_cache", "k_tree", "v_tree"):
        x = oracle.fp8_e4m3_decode(host[name]) * host[name[0] + "_scale"].astype(np.float64)[None, None, :, None]
        deq[name] = wl.to_storage(x.astype(np.float32), "bf16")
        assert np.array_equal(wl.storage_to_f64(deq[name]), x)
    d = {k: to_dev(np.ascontiguousarray(v)) for k, v in {**deq, "q": host["q"], "seq_lens": host["seq_lens"]}.items()}
    shape = shape_of(cfg, max_seq_len=700)
    out = torch.full_like(d["q"], float("nan"))
    lse = torch.full(d["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ygg.tree_attention(shape, d["q"], d["k_cache"], d["v_cache"], d["seq_lens"], d["k_tree"], d["v_tree"],
                       to_dev(parent), out, lse, workspace(shape, ygg.OP_ATTENTION))
    torch.cuda.synchronize()
    out16, lse16 = to_f64(out), to_f64(lse)
    assert np.abs(out8 - out16).max() <= 2.0 ** -7 * max(1.0, np.abs(out16).max())
    assert np.abs(lse8 - lse16).max() <= 1e-5


def test_empty_key_splits_ignore_whatever_the_workspace_holds():
    """One long and one empty sequence: the short one's key splits past its end write 'absent' markers, and
    the combine must not pick up the NaN bytes the workspace was filled with."""
    cfg, host, parent = _inputs(_cfg(2, 8, 8, 3, 4), [900, 0], 900)
    ref_out, ref_lse = _oracle(cfg, host, parent)
    out, lse = _run(_shape(cfg, 900), host, parent, poison=0xFF)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert np.abs(out - ref_out).max() <= 2e-2 and np.abs(lse - ref_lse).max() <= 1e-3


def test_is_deterministic():
    cfg, host, parent = _inputs(_cfg(2, 8, 2, 6, 8), [640, 100], 640)
    a = _run(_shape(cfg, 640), host, parent)
    b = _run(_shape(cfg, 640), host, parent)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_empty_cache_with_null_cache_pointers():
    cfg, host, parent = _inputs(_cfg(2, 8, 4, 4, 5), [0, 0], 0)
    ref_out, ref_lse = _oracle(cfg, host, parent)
    shape = _shape(cfg, 0)
    d = {k: to_dev(np.ascontiguousarray(v)) for k, v in host.items()}
    out = torch.full_like(d["q"], float("nan"))
    lse = torch.full(d["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV)
    ygg.tree_attention_fp8kv(shape, d["q"], None, None, d["seq_lens"], d["k_tree"], d["v_tree"], d["k_scale"], d["v_scale"],
                             to_dev(parent), out, lse, workspace(shape, ygg.OP_ATTENTION))
    torch.cuda.synchronize()
    assert np.abs(to_f64(out) - ref_out).max() <= 2e-2 and np.abs(to_f64(lse) - ref_lse).max() <= 1e-3
