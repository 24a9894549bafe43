"""GPU parity of the debug validator against the oracle's contract checker: flags bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import DEV, shape_of, to_dev

pytestmark = pytest.mark.gpu


def _run(cfg, depth, max_len, parent=None, lens=None, token=None, logits=None):
    shape = shape_of(cfg, max_seq_len=max_len, kv_capacity=max_len + depth + 1)
    shape.depth = depth
    flags = torch.full((cfg.batch,), -1, dtype=torch.int32, device=DEV)
    dev = lambda a: None if a is None else to_dev(np.ascontiguousarray(a))
    ygg.debug_validate(shape, flags, dev(parent), dev(lens), dev(token), dev(logits))
    torch.cuda.synchronize()
    ref = oracle.validate(depth, cfg.vocab, max_len, parent, lens, token, logits)
    got = flags.cpu().numpy()
    assert np.array_equal(got, ref), (got, ref)
    return got


def test_validator_matches_the_oracle_on_good_and_broken_inputs():
    B, D, W, V = 5, 4, 6, 9000
    cfg = wl.Config("case", B, 4, 2, 64, "bf16", 64, (), D, W, V, (0.6,), "dirichlet", 0.5, 1, 51)
    N = cfg.n_nodes
    parent = np.stack([wl.level_tree(51, D, W, "dirichlet", 0.5, sub=b) for b in range(B)]).astype(np.int32)
    token = (np.arange(B * N, dtype=np.int32).reshape(B, N) * 37) % V
    lens = np.array([0, 64, 10, 3, 33], np.int32)
    logits = wl.normal(51, 9, (B, 3, V), "f32")
    assert not _run(cfg, D, 64, parent, lens, token, logits).any()
    p = parent.copy(); p[1, 7] = 7; p[3, 0] = 2; p[4, 2] = -1
    l = lens.copy(); l[0] = 65; l[2] = -4
    t = token.copy(); t[1, N - 1] = V; t[4, 0] = -1
    x = logits.copy(); x[2, 1, 4097] = np.nan; x[3, 2, V - 1] = -np.inf; x[4, 0, 0] = np.nan
    got = _run(cfg, D, 64, p, l, t, x)
    assert list(got) == [2, 1 | 8, 2 | 16, 1, 1 | 8 | 16]
    assert list(_run(cfg, D - 1, 64, parent)) == [4] * B          # the trees are exactly D deep
    assert list(_run(cfg, D, 64, lens=lens)) == [0] * B            # any subset of the inputs


def test_validator_on_the_largest_tree():
    N = 1024
    cfg = wl.Config("case", 2, 2, 2, 64, "bf16", 16, (), 33, 31, 100, (0.6,), "dirichlet", 0.5, 1, 52)
    assert cfg.n_nodes == N
    parent = np.stack([wl.chain_tree(N), wl.random_topological_tree(3, N)]).astype(np.int32)
    _run(cfg, 1023, 16, parent)
    assert _run(cfg, 1022, 16, parent)[0] == 4
