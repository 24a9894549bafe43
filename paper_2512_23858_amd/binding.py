"""ctypes binding of include/ygg.h: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks dtypes/contiguity,
passes raw device pointers and the current HIP stream to the C ABI, and raises on a non-zero
status.  There is no CPU or PyTorch fallback: if libygg.so is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
OP_ATTENTION, OP_EXPAND, OP_ACCEPT, OP_ATTACH = 0, 1, 2, 3
F32, BF16, FP8_E4M3 = 0, 1, 2


class _CShape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("depth", ctypes.c_int32), ("width", ctypes.c_int32),
        ("n_nodes", ctypes.c_int32), ("vocab", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("kv_capacity", ctypes.c_int64), ("max_seq_len", ctypes.c_int32),
    ]


@dataclass
class Shape:
    """Mirror of ygg_shape (see include/ygg.h for the meaning of every field)."""
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    depth: int
    width: int
    n_nodes: int
    vocab: int
    kv_dtype: int
    softmax_scale: float
    kv_capacity: int
    max_seq_len: int

    def c(self) -> _CShape:
        return _CShape(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.depth, self.width,
                       self.n_nodes, self.vocab, self.kv_dtype, self.softmax_scale, self.kv_capacity,
                       self.max_seq_len)


_lib = None


def lib_path() -> str:
    return os.path.join(_PKG, "libygg.so")


def load_library() -> ctypes.CDLL:
    """Loads libygg.so (built by paper_2512_23858_amd/build.py).  Raises if it is not there."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} not found: build it with `python -m paper_2512_23858_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(path)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        shp = ctypes.POINTER(_CShape)
        lib.ygg_workspace_bytes.restype = sz
        lib.ygg_workspace_bytes.argtypes = [shp, i32, i32]
        lib.ygg_status_string.restype = ctypes.c_char_p
        lib.ygg_status_string.argtypes = [i32]
        lib.ygg_tree_attention.restype = i32
        lib.ygg_tree_attention.argtypes = [shp] + [vp] * 9 + [vp, sz, vp]
        lib.ygg_tree_attention_fp8kv.restype = i32
        lib.ygg_tree_attention_fp8kv.argtypes = [shp] + [vp] * 11 + [vp, sz, vp]
        lib.ygg_equal_growth_expand.restype = i32
        lib.ygg_equal_growth_expand.argtypes = [shp, i32] + [vp] * 4 + [vp, sz, vp]
        lib.ygg_equal_growth_expand_static.restype = i32
        lib.ygg_equal_growth_expand_static.argtypes = [shp, i32] + [vp] * 4 + [vp]
        lib.ygg_attach_pool_bytes.restype = sz
        lib.ygg_attach_pool_bytes.argtypes = [shp]
        lib.ygg_equal_growth_attach.restype = i32
        lib.ygg_equal_growth_attach.argtypes = [shp, i32] + [vp] * 4 + [vp, sz, vp, sz, vp]
        lib.ygg_prune_for_verification.restype = i32
        lib.ygg_prune_for_verification.argtypes = [shp, i32] + [vp] * 4 + [ctypes.c_float] + [vp] * 5 + [vp]
        lib.ygg_debug_validate.restype = i32
        lib.ygg_debug_validate.argtypes = [shp] + [vp] * 4 + [i32, vp, vp]
        lib.ygg_accept_and_compact.restype = i32
        lib.ygg_accept_and_compact.argtypes = [shp, i32] + [vp] * 12 + [vp, sz, vp]
        lib.ygg_init.restype = i32
        lib.ygg_init.argtypes = []
        lib.ygg_debug_set_attention_plan.restype = i32
        lib.ygg_debug_set_attention_plan.argtypes = [i32, i32, i32, i32]
        lib.ygg_debug_attention_plan.restype = i32
        lib.ygg_debug_attention_plan.argtypes = [shp, ctypes.POINTER(i32)]
        lib.ygg_debug_tree_attention_main.restype = i32
        lib.ygg_debug_tree_attention_main.argtypes = [shp] + [vp] * 9 + [vp, sz, vp]
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load_library().ygg_status_string(code).decode()


def workspace_bytes(shape: Shape, op: int, n_layers: int = 0) -> int:
    cs = shape.c()
    return int(load_library().ygg_workspace_bytes(ctypes.byref(cs), op, n_layers))


def new_workspace(shape: Shape, op: int, n_layers: int = 0, device="cuda:0"):
    """Allocates a workspace for (shape, op) through torch (contents undefined, as the library expects)."""
    n = workspace_bytes(shape, op, n_layers)
    if n == 0:
        raise ValueError("invalid shape for a workspace")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _dev(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed: {status_string(rc)} (status {rc})")


def _kv_torch_dtype(shape: Shape):
    """Element type of the K/V tensors (8-bit codes travel as uint8)."""
    return {F32: torch.float32, BF16: torch.bfloat16, FP8_E4M3: torch.uint8}[shape.kv_dtype]


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _dev(workspace, None, "workspace"), workspace.numel() * workspace.element_size()


def tree_attention(shape: Shape, q, k_cache, v_cache, seq_lens, k_tree, v_tree, parent_idx, out, lse=None,
                   workspace=None, main_kernel_only=False):
    """ygg_tree_attention: writes `out` (and `lse` if given) on the current stream.
    main_kernel_only: the measurement hook ygg_debug_tree_attention_main (no merge of the key splits)."""
    dt = _kv_torch_dtype(shape)
    cs = shape.c()
    wsp, wsn = _ws(workspace)
    fn = load_library().ygg_debug_tree_attention_main if main_kernel_only else load_library().ygg_tree_attention
    rc = fn(
        ctypes.byref(cs), _dev(q, dt, "q"), _dev(k_cache, dt, "k_cache"), _dev(v_cache, dt, "v_cache"),
        _dev(seq_lens, torch.int32, "seq_lens"), _dev(k_tree, dt, "k_tree"), _dev(v_tree, dt, "v_tree"),
        _dev(parent_idx, torch.int32, "parent_idx"), _dev(out, dt, "out"), _dev(lse, torch.float32, "lse"),
        wsp, wsn, _stream())
    _check(rc, "ygg_tree_attention")
    return out


def tree_attention_fp8kv(shape: Shape, q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale, v_scale, parent_idx,
                         out, lse=None, workspace=None):
    """ygg_tree_attention_fp8kv: K/V as uint8 E4M3 codes with per-kv-head fp32 scales, Q and out bf16."""
    cs = shape.c()
    wsp, wsn = _ws(workspace)
    u8, bf = torch.uint8, torch.bfloat16
    rc = load_library().ygg_tree_attention_fp8kv(
        ctypes.byref(cs), _dev(q, bf, "q"), _dev(k_cache, u8, "k_cache"), _dev(v_cache, u8, "v_cache"),
        _dev(seq_lens, torch.int32, "seq_lens"), _dev(k_tree, u8, "k_tree"), _dev(v_tree, u8, "v_tree"),
        _dev(k_scale, torch.float32, "k_scale"), _dev(v_scale, torch.float32, "v_scale"),
        _dev(parent_idx, torch.int32, "parent_idx"), _dev(out, bf, "out"), _dev(lse, torch.float32, "lse"),
        wsp, wsn, _stream())
    _check(rc, "ygg_tree_attention_fp8kv")
    return out


def equal_growth_expand(shape: Shape, d: int, draft_logits, parent_idx, token_ids, cum_logprob, workspace=None):
    """ygg_equal_growth_expand: fills the depth-d slots of parent_idx/token_ids/cum_logprob."""
    cs = shape.c()
    wsp, wsn = _ws(workspace)
    rc = load_library().ygg_equal_growth_expand(
        ctypes.byref(cs), d, _dev(draft_logits, torch.float32, "draft_logits"),
        _dev(parent_idx, torch.int32, "parent_idx"), _dev(token_ids, torch.int32, "token_ids"),
        _dev(cum_logprob, torch.float32, "cum_logprob"), wsp, wsn, _stream())
    _check(rc, "ygg_equal_growth_expand")


def equal_growth_expand_static(shape: Shape, d: int, draft_logits, parent_idx, token_ids, cum_logprob):
    """ygg_equal_growth_expand_static: the same draft step on the library's built-in scratch (no workspace)."""
    cs = shape.c()
    rc = load_library().ygg_equal_growth_expand_static(
        ctypes.byref(cs), d, _dev(draft_logits, torch.float32, "draft_logits"),
        _dev(parent_idx, torch.int32, "parent_idx"), _dev(token_ids, torch.int32, "token_ids"),
        _dev(cum_logprob, torch.float32, "cum_logprob"), _stream())
    _check(rc, "ygg_equal_growth_expand_static")


def attach_pool_bytes(shape: Shape) -> int:
    cs = shape.c()
    return int(load_library().ygg_attach_pool_bytes(ctypes.byref(cs)))


def equal_growth_attach(shape: Shape, t: int, draft_logits, parent_idx, token_ids, cum_logprob, pool, workspace=None):
    """ygg_equal_growth_attach: draft step t with free attachment; fills nodes 1+(t-1)W .. tW and updates `pool`."""
    cs = shape.c()
    wsp, wsn = _ws(workspace)
    pp, pn = _ws(pool)
    rc = load_library().ygg_equal_growth_attach(
        ctypes.byref(cs), t, _dev(draft_logits, torch.float32, "draft_logits"),
        _dev(parent_idx, torch.int32, "parent_idx"), _dev(token_ids, torch.int32, "token_ids"),
        _dev(cum_logprob, torch.float32, "cum_logprob"), pp, pn, wsp, wsn, _stream())
    _check(rc, "ygg_equal_growth_attach")


def prune_for_verification(shape: Shape, w_verify: int, parent_idx, token_ids, cum_logprob, kept_nodes, new_parent,
                           new_token, expected_len=None, best_width=None, t_verifier=None, t_draft: float = 0.0):
    """ygg_prune_for_verification: keeps the w_verify most valuable nodes as a renumbered tree."""
    cs = shape.c()
    i32t = torch.int32
    rc = load_library().ygg_prune_for_verification(
        ctypes.byref(cs), w_verify, _dev(parent_idx, i32t, "parent_idx"), _dev(token_ids, i32t, "token_ids"),
        _dev(cum_logprob, torch.float32, "cum_logprob"), _dev(t_verifier, torch.float32, "t_verifier"),
        ctypes.c_float(t_draft), _dev(kept_nodes, i32t, "kept_nodes"), _dev(new_parent, i32t, "new_parent"),
        _dev(new_token, i32t, "new_token"), _dev(expected_len, torch.float32, "expected_len"),
        _dev(best_width, i32t, "best_width"), _stream())
    _check(rc, "ygg_prune_for_verification")


def debug_validate(shape: Shape, flags, parent_idx=None, seq_lens=None, token_ids=None, logits=None):
    """ygg_debug_validate: per-sequence violation bit masks into `flags` ([B] int32 on the GPU)."""
    cs = shape.c()
    rows = 0 if logits is None else int(logits.shape[1])
    rc = load_library().ygg_debug_validate(
        ctypes.byref(cs), _dev(parent_idx, torch.int32, "parent_idx"), _dev(seq_lens, torch.int32, "seq_lens"),
        _dev(token_ids, torch.int32, "token_ids"), _dev(logits, torch.float32, "logits"), rows,
        _dev(flags, torch.int32, "flags"), _stream())
    _check(rc, "ygg_debug_validate")


def accept_and_compact(shape: Shape, n_layers: int, parent_idx, token_ids, k_tree, v_tree, k_cache, v_cache,
                       seq_lens, accept_len, accept_path, bonus_token, target_logits=None, target_tokens=None,
                       workspace=None):
    """ygg_accept_and_compact: updates the caches and seq_lens in place, fills the three outputs."""
    dt = _kv_torch_dtype(shape)
    cs = shape.c()
    wsp, wsn = _ws(workspace)
    rc = load_library().ygg_accept_and_compact(
        ctypes.byref(cs), n_layers, _dev(target_logits, torch.float32, "target_logits"),
        _dev(target_tokens, torch.int32, "target_tokens"), _dev(parent_idx, torch.int32, "parent_idx"),
        _dev(token_ids, torch.int32, "token_ids"), _dev(k_tree, dt, "k_tree"), _dev(v_tree, dt, "v_tree"),
        _dev(k_cache, dt, "k_cache"), _dev(v_cache, dt, "v_cache"), _dev(seq_lens, torch.int32, "seq_lens"),
        _dev(accept_len, torch.int32, "accept_len"), _dev(accept_path, torch.int32, "accept_path"),
        _dev(bonus_token, torch.int32, "bonus_token"), wsp, wsn, _stream())
    _check(rc, "ygg_accept_and_compact")


def attention_plan(shape: Shape) -> dict:
    """ygg_debug_attention_plan: the launch plan of tree_attention for this shape (host only)."""
    cs = shape.c()
    out = (ctypes.c_int32 * 5)()
    _check(load_library().ygg_debug_attention_plan(ctypes.byref(cs), out), "ygg_debug_attention_plan")
    return dict(matrix_cores=bool(out[0]), waves=out[1], key_shares=out[2], row_tiles=out[3], key_splits=out[4])


def init():
    """ygg_init: prepares the current device up front (otherwise done by the first launching call)."""
    _check(load_library().ygg_init(), "ygg_init")


def set_attention_plan(waves: int = 0, rblocks: int = 0, nsplit: int = 0, kshares: int = 0):
    """ygg_debug_set_attention_plan: tuning override of the attention launch plan (all zero: none)."""
    _check(load_library().ygg_debug_set_attention_plan(waves, rblocks, nsplit, kshares), "ygg_debug_set_attention_plan")
