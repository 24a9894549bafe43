"""Helpers shared by the GPU parity tests: host arrays -> device tensors, and calls through the
C ABI binding.  Expected values always come from the CPU oracle, never from the GPU path."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_23858_amd as ygg
import ygg_workloads as wl

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> cuda tensor; uint16 arrays are bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def shape_of(cfg: wl.Config, max_seq_len=None, kv_capacity=None, n_nodes=None) -> ygg.Shape:
    return ygg.Shape(
        batch=cfg.batch, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
        depth=cfg.depth, width=cfg.width, n_nodes=cfg.n_nodes if n_nodes is None else n_nodes, vocab=cfg.vocab,
        kv_dtype=ygg.binding.F32 if cfg.dtype == "f32" else ygg.binding.BF16,
        softmax_scale=cfg.softmax_scale,
        kv_capacity=cfg.kv_capacity if kv_capacity is None else kv_capacity,
        max_seq_len=cfg.max_prefix if max_seq_len is None else max_seq_len)


def workspace(shape: ygg.Shape, op: int, n_layers: int = 0, poison: int = 0xA5) -> torch.Tensor:
    n = ygg.workspace_bytes(shape, op, n_layers)
    assert n > 0, "invalid shape for workspace query"
    # poison the workspace: kernels must not rely on its contents (0xFF bytes read as NaN)
    return torch.full((n,), poison, dtype=torch.uint8, device=DEV)


def run_attention(shape: ygg.Shape, host: dict, parent_idx: np.ndarray, want_lse=True, poison: int = 0xA5):
    """host: dict with q,k_cache,v_cache,k_tree,v_tree,seq_lens (numpy).  Returns (out f64, lse f64)."""
    d = {k: to_dev(np.ascontiguousarray(v)) for k, v in host.items()}
    par = to_dev(np.ascontiguousarray(parent_idx))
    out = torch.full_like(d["q"], float("nan"))
    lse = torch.full(d["q"].shape[:3], float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    ws = workspace(shape, ygg.OP_ATTENTION, poison=poison)
    ygg.tree_attention(shape, d["q"], d["k_cache"], d["v_cache"], d["seq_lens"], d["k_tree"], d["v_tree"], par,
                       out, lse, ws)
    torch.cuda.synchronize()
    return to_f64(out), (to_f64(lse) if want_lse else None)
