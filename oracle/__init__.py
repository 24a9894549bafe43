"""fp64 CPU oracle for the tree-verification hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling around ``ygg_oracle.c`` (which holds all the arithmetic and
cites the paper passages it follows).  Only ``tests/``, the smoke check and the
CPU-baseline leg of the benchmark may import this package; the GPU library and its
Python binding never do.

bf16 tensors are passed as ``numpy.uint16`` arrays (the upper half of an fp32 word),
fp32 tensors as ``numpy.float32``.  All results are ``float64`` / ``int32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ygg_oracle.c")
_LIB = os.path.join(_HERE, "libygg_oracle.so")

F32, BF16, FP8_E4M3 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def build_sanitized() -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (for the opt-in sanitizer test; a process
    that loads it needs libasan preloaded and finds it through YGG_ORACLE_LIB)."""
    out = os.path.join(_HERE, "libygg_oracle_san.so")
    subprocess.check_call(
        ["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", "-o", out, _SRC, "-lm"]
    )
    return out


_lib = None


def _load():
    global _lib
    if _lib is None:
        # YGG_ORACLE_LIB: another build of this same source (the sanitizer test's), never anything else
        _lib = ctypes.CDLL(os.environ.get("YGG_ORACLE_LIB") or build())
        for name in (
            "ygg_oracle_attention_row",
            "ygg_oracle_tree_attention",
            "ygg_oracle_attention_row_fp8kv",
            "ygg_oracle_tree_attention_fp8kv",
            "ygg_oracle_fp8_e4m3_decode",
            "ygg_oracle_expand_scores",
            "ygg_oracle_expand",
            "ygg_oracle_accept_compact",
        ):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    """Threads the oracle's row-parallel loops run on (OpenMP's maximum for this process)."""
    lib = _load()
    lib.ygg_oracle_max_threads.restype = ctypes.c_int
    return int(lib.ygg_oracle_max_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.uint8:
        return FP8_E4M3
    raise TypeError(f"expected float32, uint16 (bf16 bits) or uint8 (E4M3 codes), got {a.dtype}")


def _ptr(a):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be C-contiguous"
    return ctypes.c_void_p(a.ctypes.data)


def _i32(x):
    return ctypes.c_int32(int(x))


def _attn_common(q, k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx):
    B, N, Hq, Dh = q.shape
    Bc, cap, Hkv, Dhc = k_cache.shape
    assert (Bc, Dhc) == (B, Dh) and v_cache.shape == k_cache.shape
    assert k_tree.shape == (B, N, Hkv, Dh) and v_tree.shape == k_tree.shape
    assert parent_idx.shape == (B, N) and parent_idx.dtype == np.int32
    assert seq_lens.shape == (B,) and seq_lens.dtype == np.int32
    dt = _dtype_code(q)
    for a in (k_cache, v_cache, k_tree, v_tree):
        assert _dtype_code(a) == dt
    return B, N, Hq, Hkv, Dh, cap, dt


def attention_row(q, k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx, scale, b, i, h,
                  want_probs=False):
    """One output row: returns (out[Dh], lse, probs[L+N] or None)."""
    B, N, Hq, Hkv, Dh, cap, dt = _attn_common(q, k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx)
    out = np.empty(Dh, np.float64)
    lse = ctypes.c_double(0.0)
    probs = np.empty(int(seq_lens[b]) + N, np.float64) if want_probs else None
    rc = _load().ygg_oracle_attention_row(
        _i32(B), _i32(N), _i32(Hq), _i32(Hkv), _i32(Dh), ctypes.c_int(dt), ctypes.c_double(float(scale)),
        ctypes.c_int64(cap), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(k_tree),
        _ptr(v_tree), _ptr(parent_idx), _i32(b), _i32(i), _i32(h), _ptr(out), ctypes.byref(lse), _ptr(probs))
    if rc != 0:
        raise ValueError(f"ygg_oracle_attention_row failed with {rc}")
    return out, lse.value, probs


def fp8_e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """Values of E4M3 codes (uint8) as float64 (NaN for the two NaN codes)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, np.float64)
    rc = _load().ygg_oracle_fp8_e4m3_decode(_ptr(codes), ctypes.c_int64(codes.size), _ptr(out))
    if rc != 0:
        raise ValueError(f"ygg_oracle_fp8_e4m3_decode failed with {rc}")
    return out


def _attn_common_fp8kv(q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale, v_scale, parent_idx):
    B, N, Hq, Dh = q.shape
    Bc, cap, Hkv, Dhc = k_cache.shape
    assert (Bc, Dhc) == (B, Dh) and v_cache.shape == k_cache.shape
    assert k_tree.shape == (B, N, Hkv, Dh) and v_tree.shape == k_tree.shape
    assert parent_idx.shape == (B, N) and parent_idx.dtype == np.int32
    assert seq_lens.shape == (B,) and seq_lens.dtype == np.int32
    for a in (k_cache, v_cache, k_tree, v_tree):
        assert a.dtype == np.uint8
    for s in (k_scale, v_scale):
        assert s.dtype == np.float32 and s.shape == (Hkv,)
    return B, N, Hq, Hkv, Dh, cap, _dtype_code(q)


def attention_row_fp8kv(q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale, v_scale, parent_idx, scale,
                        b, i, h):
    """One output row with K/V stored as E4M3 codes and per-kv-head scales: (out[Dh], lse)."""
    B, N, Hq, Hkv, Dh, cap, dt = _attn_common_fp8kv(q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale,
                                                    v_scale, parent_idx)
    out = np.empty(Dh, np.float64)
    lse = ctypes.c_double(0.0)
    rc = _load().ygg_oracle_attention_row_fp8kv(
        _i32(B), _i32(N), _i32(Hq), _i32(Hkv), _i32(Dh), ctypes.c_int(dt), ctypes.c_double(float(scale)),
        ctypes.c_int64(cap), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(k_tree),
        _ptr(v_tree), _ptr(k_scale), _ptr(v_scale), _ptr(parent_idx), _i32(b), _i32(i), _i32(h), _ptr(out),
        ctypes.byref(lse), _ptr(None))
    if rc != 0:
        raise ValueError(f"ygg_oracle_attention_row_fp8kv failed with {rc}")
    return out, lse.value


def tree_attention_fp8kv(q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale, v_scale, parent_idx, scale):
    """All rows with K/V stored as E4M3 codes: (out[B,N,Hq,Dh] float64, lse[B,N,Hq] float64)."""
    B, N, Hq, Hkv, Dh, cap, dt = _attn_common_fp8kv(q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale,
                                                    v_scale, parent_idx)
    out = np.empty((B, N, Hq, Dh), np.float64)
    lse = np.empty((B, N, Hq), np.float64)
    rc = _load().ygg_oracle_tree_attention_fp8kv(
        _i32(B), _i32(N), _i32(Hq), _i32(Hkv), _i32(Dh), ctypes.c_int(dt), ctypes.c_double(float(scale)),
        ctypes.c_int64(cap), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(k_tree),
        _ptr(v_tree), _ptr(k_scale), _ptr(v_scale), _ptr(parent_idx), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"ygg_oracle_tree_attention_fp8kv failed with {rc}")
    return out, lse


def tree_attention(q, k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx, scale):
    """All rows: returns (out[B,N,Hq,Dh] float64, lse[B,N,Hq] float64)."""
    B, N, Hq, Hkv, Dh, cap, dt = _attn_common(q, k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx)
    out = np.empty((B, N, Hq, Dh), np.float64)
    lse = np.empty((B, N, Hq), np.float64)
    rc = _load().ygg_oracle_tree_attention(
        _i32(B), _i32(N), _i32(Hq), _i32(Hkv), _i32(Dh), ctypes.c_int(dt), ctypes.c_double(float(scale)),
        ctypes.c_int64(cap), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(k_tree),
        _ptr(v_tree), _ptr(parent_idx), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"ygg_oracle_tree_attention failed with {rc}")
    return out, lse


def expand_scores(logits, cum_front):
    """s(p,v) for one sequence: logits [F,V] float32, cum_front [F] float32 -> [F,V] float64."""
    F, V = logits.shape
    assert logits.dtype == np.float32 and cum_front.dtype == np.float32 and cum_front.shape == (F,)
    scores = np.empty((F, V), np.float64)
    rc = _load().ygg_oracle_expand_scores(_i32(F), _i32(V), _ptr(logits), _ptr(cum_front), _ptr(scores))
    if rc != 0:
        raise ValueError(f"ygg_oracle_expand_scores failed with {rc}")
    return scores


def expand(D, W, d, draft_logits, parent_idx, token_ids, cum_logprob):
    """One draft step, in place on parent_idx/token_ids/cum_logprob [B,N]; returns margin[B]."""
    B, F, V = draft_logits.shape
    N = 1 + D * W
    assert F == (1 if d == 1 else W)
    assert draft_logits.dtype == np.float32 and cum_logprob.dtype == np.float32
    assert parent_idx.dtype == np.int32 and token_ids.dtype == np.int32
    assert parent_idx.shape == (B, N) and token_ids.shape == (B, N) and cum_logprob.shape == (B, N)
    margin = np.empty(B, np.float64)
    rc = _load().ygg_oracle_expand(_i32(B), _i32(D), _i32(W), _i32(V), _i32(d), _ptr(draft_logits),
                                   _ptr(parent_idx), _ptr(token_ids), _ptr(cum_logprob), _ptr(margin))
    if rc != 0:
        raise ValueError(f"ygg_oracle_expand failed with {rc}")
    return margin


def attach_pool(B, D, W):
    """Empty pool state for attach(): room for every offer of all D steps."""
    cap = W + (D - 1) * W * W
    return {"score": np.zeros((B, cap), np.float64), "node": np.zeros((B, cap), np.int32),
            "token": np.zeros((B, cap), np.int32), "count": np.zeros(B, np.int32)}


def attach(D, W, t, draft_logits, parent_idx, token_ids, cum_logprob, pool):
    """One draft step of equal growth with free attachment, in place on the tree arrays and the pool; returns margin[B]."""
    B, F, V = draft_logits.shape
    N = 1 + D * W
    assert F == (1 if t == 1 else W)
    assert draft_logits.dtype == np.float32 and cum_logprob.dtype == np.float32
    assert parent_idx.dtype == np.int32 and token_ids.dtype == np.int32
    assert parent_idx.shape == (B, N) and token_ids.shape == (B, N) and cum_logprob.shape == (B, N)
    cap = pool["score"].shape[1]
    assert pool["score"].dtype == np.float64 and pool["node"].dtype == np.int32 and pool["token"].dtype == np.int32
    assert pool["node"].shape == (B, cap) and pool["token"].shape == (B, cap) and pool["count"].shape == (B,)
    margin = np.empty(B, np.float64)
    rc = _load().ygg_oracle_attach(_i32(B), _i32(D), _i32(W), _i32(V), _i32(t), _ptr(draft_logits),
                                   _ptr(parent_idx), _ptr(token_ids), _ptr(cum_logprob), _ptr(pool["score"]),
                                   _ptr(pool["node"]), _ptr(pool["token"]), _ptr(pool["count"]), _i32(cap), _ptr(margin))
    if rc != 0:
        raise ValueError(f"ygg_oracle_attach failed with {rc}")
    return margin


def subtree_dp(parent, value, want):
    """Bottom-up tree DP: best[k] for k = 0..N and one optimal set of `want` nodes (bool mask)."""
    N = parent.shape[0]
    assert parent.dtype == np.int32 and value.dtype == np.float64 and value.shape == (N,)
    best = np.empty(N + 1, np.float64)
    keep = np.zeros(N, np.uint8)
    rc = _load().ygg_oracle_subtree_dp(_i32(N), _ptr(parent), _ptr(value), _i32(want), _ptr(best), _ptr(keep))
    if rc != 0:
        raise ValueError(f"ygg_oracle_subtree_dp failed with {rc}")
    return best, keep.astype(bool)


def prune(w, parent_idx, token_ids, cum_logprob, t_verifier=None, t_draft=0.0):
    """Verification-width pruning of a batch of trees to w nodes each; see ygg_oracle_prune."""
    B, N = parent_idx.shape
    assert parent_idx.dtype == np.int32 and token_ids.dtype == np.int32 and cum_logprob.dtype == np.float32
    assert token_ids.shape == (B, N) and cum_logprob.shape == (B, N)
    if t_verifier is not None:
        assert t_verifier.dtype == np.float64 and t_verifier.shape == (N + 1,)
    out = dict(kept_nodes=np.empty((B, w), np.int32), new_parent=np.empty((B, w), np.int32),
               new_token=np.empty((B, w), np.int32), expected_len=np.empty(B, np.float64),
               best_width=np.zeros(B, np.int32), best_curve=np.empty((B, N + 1), np.float64))
    rc = _load().ygg_oracle_prune(_i32(B), _i32(N), _i32(w), _ptr(parent_idx), _ptr(token_ids), _ptr(cum_logprob),
                                  _ptr(t_verifier) if t_verifier is not None else None, ctypes.c_double(float(t_draft)),
                                  _ptr(out["kept_nodes"]), _ptr(out["new_parent"]), _ptr(out["new_token"]),
                                  _ptr(out["expected_len"]), _ptr(out["best_width"]), _ptr(out["best_curve"]))
    if rc != 0:
        raise ValueError(f"ygg_oracle_prune failed with {rc}")
    if t_verifier is None:
        out["best_width"] = None
    return out


def validate(depth, vocab, max_seq_len, parent_idx=None, seq_lens=None, token_ids=None, logits=None):
    """Per-sequence violation flags of the data-dependent calling contract (see ygg_oracle_validate)."""
    ref = next(a for a in (parent_idx, token_ids, seq_lens, logits) if a is not None)
    B = ref.shape[0]
    N = parent_idx.shape[1] if parent_idx is not None else (token_ids.shape[1] if token_ids is not None else 1)
    rows = 0
    if logits is not None:
        assert logits.dtype == np.float32 and logits.ndim == 3 and logits.shape[2] == vocab
        rows = logits.shape[1]
    for a in (parent_idx, seq_lens, token_ids):
        assert a is None or a.dtype == np.int32
    flags = np.zeros(B, np.int32)
    rc = _load().ygg_oracle_validate(_i32(B), _i32(N), _i32(depth), _i32(vocab), _i32(max_seq_len), _ptr(parent_idx),
                                     _ptr(seq_lens), _ptr(token_ids), _ptr(logits), _i32(rows), _ptr(flags))
    if rc != 0:
        raise ValueError(f"ygg_oracle_validate failed with {rc}")
    return flags


def accept_compact(path_cols, parent_idx, token_ids, k_tree, v_tree, k_cache, v_cache, seq_lens,
                   target_logits=None, target_tokens=None):
    """Greedy acceptance + compaction; k_cache, v_cache and seq_lens are updated in place.

    k_tree, v_tree [layers,B,N,Hkv,Dh]; k_cache, v_cache [layers,B,cap,Hkv,Dh].
    Returns dict(accept_len[B], accept_path[B,path_cols], bonus_token[B], tstar[B,N]).
    """
    B, N = parent_idx.shape
    layers, Bt, Nt, Hkv, Dh = k_tree.shape
    assert (Bt, Nt) == (B, N) and v_tree.shape == k_tree.shape
    cap = k_cache.shape[2]
    assert k_cache.shape == (layers, B, cap, Hkv, Dh) and v_cache.shape == k_cache.shape
    dt = _dtype_code(k_tree)
    assert _dtype_code(k_cache) == dt and _dtype_code(v_cache) == dt and _dtype_code(v_tree) == dt
    V = 0
    if target_logits is not None:
        assert target_logits.dtype == np.float32 and target_logits.shape[:2] == (B, N)
        V = target_logits.shape[2]
    if target_tokens is not None:
        assert target_tokens.dtype == np.int32 and target_tokens.shape == (B, N)
    accept_len = np.empty(B, np.int32)
    accept_path = np.empty((B, path_cols), np.int32)
    bonus = np.empty(B, np.int32)
    tstar = np.empty((B, N), np.int32)
    rc = _load().ygg_oracle_accept_compact(
        _i32(B), _i32(N), _i32(V), _i32(path_cols), _i32(layers), _i32(Hkv), _i32(Dh), ctypes.c_int(dt),
        ctypes.c_int64(cap), _ptr(target_logits), _ptr(target_tokens), _ptr(parent_idx), _ptr(token_ids),
        _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(accept_len),
        _ptr(accept_path), _ptr(bonus), _ptr(tstar))
    if rc != 0:
        raise ValueError(f"ygg_oracle_accept_compact failed with {rc}")
    return dict(accept_len=accept_len, accept_path=accept_path, bonus_token=bonus, tstar=tstar)
