"""Seeded synthetic inputs for the tree-verification hot path.

This module holds *no* arithmetic of the method: it only draws random tensors with the
shapes, value distributions and tree structure of the five workload configurations and
converts storage formats.  Both the CPU oracle's tests and the GPU tests/benchmark take
their inputs from here, so the two sides always see identical bytes.

Random numbers come from numpy's counter-based Philox generator keyed by
(seed, stream) so that any tensor can be regenerated independently of the others.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

# stream ids (second half of the Philox key)
_S_TREE, _S_TOKENS, _S_Q, _S_KC, _S_VC, _S_KT, _S_VT, _S_DRAFT, _S_TARGET, _S_PLANT, _S_LENS, _S_AGREE = range(12)


@dataclass(frozen=True)
class Config:
    """One workload configuration (shapes follow the public Llama architectures)."""
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" or "bf16" (storage type of Q/K/V/O)
    prefix_len: int       # fixed KV prefix length, or 0 if ragged
    prefix_range: tuple   # (lo, hi) inclusive for ragged batches, else ()
    depth: int
    width: int
    vocab: int
    agree: tuple          # (p,) or (lo, hi) per-sequence uniform range
    parents: str          # "uniform" or "dirichlet"
    alpha: float
    n_layers: int         # layers timed back to back
    seed: int

    @property
    def n_nodes(self) -> int:
        return 1 + self.depth * self.width

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_prefix(self) -> int:
        return self.prefix_range[1] if self.prefix_range else self.prefix_len

    @property
    def kv_capacity(self) -> int:
        return self.max_prefix + self.depth + 1

    @property
    def softmax_scale(self) -> float:
        return float(np.float32(1.0) / np.sqrt(np.float32(self.head_dim)))


CONFIGS = {
    1: Config("tiny-f32", 1, 4, 4, 64, "f32", 128, (), 3, 4, 1000, (0.7,), "uniform", 0.0, 1, 1000),
    2: Config("llama2-7b-layer", 1, 32, 32, 128, "bf16", 1024, (), 6, 8, 32000, (0.7,), "dirichlet", 0.5, 32, 2000),
    3: Config("llama3-8b-gqa", 1, 32, 8, 128, "bf16", 4096, (), 8, 16, 128256, (0.6,), "dirichlet", 0.5, 32, 3000),
    4: Config("long-context-wide-tree", 1, 32, 8, 128, "bf16", 32768, (), 10, 32, 128256, (0.6,), "dirichlet", 0.3, 32, 4000),
    5: Config("batched-70b-gqa", 16, 64, 8, 128, "bf16", 0, (512, 8192), 6, 8, 32000, (0.4, 0.8), "dirichlet", 0.5, 1, 5000),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a configuration with some fields replaced (used for small test cases)."""
    return replace(cfg, **kw)


def rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 20) + sub, stream]))


# ---------------------------------------------------------------- storage formats

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_fp8_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round to the 8-bit E4M3 format (4 exponent bits, bias 7, 3 mantissa bits, subnormals, no
    infinities; round-to-nearest-even, magnitudes above 448 saturate), returned as uint8 codes."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), 448.0)
    _, ex = np.frexp(a)                                   # a = f * 2^ex, f in [0.5, 1)
    e = np.maximum(ex - 1, -6)                            # exponent of the binade; subnormals share -6
    r = np.rint(np.ldexp(a, 3 - e))                       # multiples of the binade's quantum 2^(e-3)
    up = r >= 16                                          # rounded up into the next binade
    e = np.where(up, e + 1, e)
    r = np.where(up, 8.0, r)
    code = np.where(r < 8, r, (e + 7) * 8 + (r - 8)).astype(np.uint8)   # r < 8 only for subnormals
    return code | (np.signbit(x).astype(np.uint8) << np.uint8(7))


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    return x.astype(np.float32) if dtype == "f32" else f32_to_bf16_bits(x)


def storage_to_f64(a: np.ndarray) -> np.ndarray:
    return a.astype(np.float64) if a.dtype == np.float32 else bf16_bits_to_f64(a)


def normal(seed: int, stream: int, shape, dtype: str, sub: int = 0, sigma: float = 1.0) -> np.ndarray:
    x = rng(seed, stream, sub).standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return to_storage(x, dtype)


# ---------------------------------------------------------------- trees

def level_tree(seed: int, depth: int, width: int, parents: str, alpha: float, sub: int = 0) -> np.ndarray:
    """parent_idx[N] of a level-structured tree: node 0 is the root (-1), depth-d nodes sit at
    1+(d-1)W .. d*W.  Depth-1 nodes hang off the root.  For d >= 2 each node draws its parent
    among the depth d-1 slots: uniformly, or from Cat(pi) with pi ~ Dirichlet(alpha) so that
    child counts are skewed.  Children keep their draw order."""
    g = rng(seed, _S_TREE, sub)
    n = 1 + depth * width
    parent = np.empty(n, np.int32)
    parent[0] = -1
    for d in range(1, depth + 1):
        base = 1 + (d - 1) * width
        if d == 1:
            parent[base:base + width] = 0
            continue
        prev = base - width
        if parents == "uniform":
            slots = g.integers(0, width, size=width)
        else:
            pi = g.dirichlet(np.full(width, alpha))
            slots = g.choice(width, size=width, p=pi)
        parent[base:base + width] = prev + slots
    return parent


def chain_tree(n: int) -> np.ndarray:
    """Width-1 tree: node i's parent is i-1."""
    return np.arange(-1, n - 1, dtype=np.int32)


def random_topological_tree(seed: int, n: int, sub: int = 0) -> np.ndarray:
    """Any tree with parent[i] < i (not level structured)."""
    g = rng(seed, _S_TREE, sub)
    parent = np.empty(n, np.int32)
    parent[0] = -1
    for i in range(1, n):
        parent[i] = g.integers(0, i)
    return parent


def node_tokens(seed: int, parent: np.ndarray, vocab: int, sub: int = 0) -> np.ndarray:
    """token_ids[N]: root uniform; the children of one parent carry distinct tokens."""
    g = rng(seed, _S_TOKENS, sub)
    n = parent.shape[0]
    tok = np.empty(n, np.int32)
    tok[0] = g.integers(0, vocab)
    for p in range(n):
        kids = np.nonzero(parent == p)[0]
        if kids.size:
            tok[kids] = g.choice(vocab, size=kids.size, replace=False)
    return tok


def target_logits(seed: int, parent: np.ndarray, tokens: np.ndarray, vocab: int, agree: float,
                  sub: int = 0) -> np.ndarray:
    """[N,V] fp32 ~ N(0,1).  For every node with at least one child, with probability `agree`
    one child (uniform) is chosen and its token's logit is raised to rowmax + 1, making the
    draft token the row's argmax.  Leaves are never planted."""
    n = parent.shape[0]
    x = rng(seed, _S_TARGET, sub).standard_normal(size=(n, vocab), dtype=np.float32)
    g = rng(seed, _S_PLANT, sub)
    for i in range(n):
        kids = np.nonzero(parent == i)[0]
        u = g.random()
        pick = g.integers(0, max(kids.size, 1))
        if kids.size and u < agree:
            x[i, tokens[kids[pick]]] = x[i].max() + np.float32(1.0)
    return x


def draft_logits(seed: int, depth_step: int, rows: int, vocab: int, sub: int = 0) -> np.ndarray:
    """[rows,V] fp32 ~ N(0, 3^2) for draft step `depth_step` (1-based)."""
    x = rng(seed, _S_DRAFT, sub * 64 + depth_step).standard_normal(size=(rows, vocab), dtype=np.float32)
    x *= np.float32(3.0)
    return x


# ---------------------------------------------------------------- whole workloads

def seq_lens(cfg: Config) -> np.ndarray:
    if cfg.prefix_range:
        lo, hi = cfg.prefix_range
        return rng(cfg.seed, _S_LENS).integers(lo, hi + 1, size=cfg.batch).astype(np.int32)
    return np.full(cfg.batch, cfg.prefix_len, np.int32)


def agree_rates(cfg: Config) -> np.ndarray:
    if len(cfg.agree) == 2:
        return rng(cfg.seed, _S_AGREE).uniform(cfg.agree[0], cfg.agree[1], size=cfg.batch)
    return np.full(cfg.batch, cfg.agree[0])


def trees(cfg: Config) -> np.ndarray:
    """parent_idx [B,N] int32."""
    return np.stack([level_tree(cfg.seed, cfg.depth, cfg.width, cfg.parents, cfg.alpha, sub=b)
                     for b in range(cfg.batch)])


def tokens(cfg: Config, parent_idx: np.ndarray) -> np.ndarray:
    return np.stack([node_tokens(cfg.seed, parent_idx[b], cfg.vocab, sub=b) for b in range(cfg.batch)])


def attention_inputs(cfg: Config, layer: int = 0, lens: np.ndarray | None = None) -> dict:
    """Q, prefix K/V cache, tree K/V for one layer (seed = cfg.seed + layer).  Cache rows at or
    beyond a sequence's length are filled too (with the same distribution): a correct
    implementation never reads them."""
    s = cfg.seed + layer
    B, N, Hq, Hkv, Dh, cap = cfg.batch, cfg.n_nodes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.kv_capacity
    return dict(
        q=normal(s, _S_Q, (B, N, Hq, Dh), cfg.dtype),
        k_cache=normal(s, _S_KC, (B, cap, Hkv, Dh), cfg.dtype),
        v_cache=normal(s, _S_VC, (B, cap, Hkv, Dh), cfg.dtype),
        k_tree=normal(s, _S_KT, (B, N, Hkv, Dh), cfg.dtype),
        v_tree=normal(s, _S_VT, (B, N, Hkv, Dh), cfg.dtype),
        seq_lens=seq_lens(cfg) if lens is None else lens,
    )


def attention_inputs_fp8kv(cfg: Config, layer: int = 0, lens: np.ndarray | None = None) -> dict:
    """The same draws as attention_inputs with K and V stored as E4M3 codes: one scale per kv head
    and tensor kind (K, V), chosen so that the head's largest magnitude over cache and tree maps to
    448; code = round(x / scale).  Q keeps cfg.dtype."""
    s = cfg.seed + layer
    B, N, Hq, Hkv, Dh, cap = cfg.batch, cfg.n_nodes, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.kv_capacity
    out = dict(q=normal(s, _S_Q, (B, N, Hq, Dh), cfg.dtype), seq_lens=seq_lens(cfg) if lens is None else lens)
    for name, sc, st in (("k", _S_KC, _S_KT), ("v", _S_VC, _S_VT)):
        cache = normal(s, sc, (B, cap, Hkv, Dh), "f32")
        tree = normal(s, st, (B, N, Hkv, Dh), "f32")
        amax = np.maximum(np.abs(cache).max(axis=(0, 1, 3)), np.abs(tree).max(axis=(0, 1, 3)))
        scale = (amax / np.float32(448.0)).astype(np.float32)
        bc = scale.astype(np.float64)[None, :, None]

        def quantise(x):   # in slices of 1024 tokens: the float64 temporaries stay small
            codes = np.empty(x.shape, np.uint8)
            flat_x, flat_c = x.reshape(-1, Hkv, Dh), codes.reshape(-1, Hkv, Dh)
            for lo in range(0, flat_x.shape[0], 1024):
                flat_c[lo:lo + 1024] = f64_to_fp8_e4m3_bits(flat_x[lo:lo + 1024] / bc)
            return codes
        out[name + "_cache"] = quantise(cache)
        out[name + "_tree"] = quantise(tree)
        out[name + "_scale"] = scale
    return out


def expansion_inputs(cfg: Config, d: int) -> np.ndarray:
    """draft logits [B,F_d,V] for draft step d (F_1 = 1, else W)."""
    rows = 1 if d == 1 else cfg.width
    return np.stack([draft_logits(cfg.seed, d, rows, cfg.vocab, sub=b) for b in range(cfg.batch)])


def acceptance_inputs(cfg: Config, parent_idx: np.ndarray, token_ids: np.ndarray) -> np.ndarray:
    """target logits [B,N,V] with the per-sequence agreement rate planted."""
    p = agree_rates(cfg)
    return np.stack([target_logits(cfg.seed, parent_idx[b], token_ids[b], cfg.vocab, float(p[b]), sub=b)
                     for b in range(cfg.batch)])
