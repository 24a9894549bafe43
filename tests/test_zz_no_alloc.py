"""The allocation-free draft step (ygg_equal_growth_expand_static) against the workspace-taking one,
through the C ABI: the same trees bit for bit, two runs in a row on the library's built-in scratch,
the second on a smaller input, with no device allocation made while the calls are enqueued."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2512_23858_amd as ygg
import ygg_workloads as wl
from gpu_util import shape_of, to_dev, workspace

pytestmark = pytest.mark.gpu


def _cfg(B, D, W, V, seed):
    return wl.Config("case", B, 4, 2, 64, "bf16", 16, (), D, W, V, (0.6,), "dirichlet", 0.5, 1, seed)


def _grow(cfg, static):
    B, N, D = cfg.batch, cfg.n_nodes, cfg.depth
    parent = np.full((B, N), -9, np.int32); token = np.full((B, N), -9, np.int32); cum = np.full((B, N), np.nan, np.float32)
    parent[:, 0], token[:, 0], cum[:, 0] = -1, 1, 0.0
    gp, gt, gc = to_dev(parent), to_dev(token), to_dev(cum)
    shape = shape_of(cfg)
    logits = [to_dev(wl.expansion_inputs(cfg, d)) for d in range(1, D + 1)]
    ws = None if static else workspace(shape, ygg.OP_EXPAND)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    for d in range(1, D + 1):
        if static:
            ygg.equal_growth_expand_static(shape, d, logits[d - 1], gp, gt, gc)
        else:
            ygg.equal_growth_expand(shape, d, logits[d - 1], gp, gt, gc, ws)
    if static:
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before   # torch's allocator was not asked either
    torch.cuda.synchronize()
    return gp.cpu().numpy(), gt.cpu().numpy(), gc.cpu().numpy()


def test_static_scratch_expand_equals_the_workspace_one_twice_in_a_row():
    big = _cfg(3, 4, 16, 50000, seed=11)      # several chunks per row, three sequences
    small = _cfg(1, 3, 4, 1000, seed=12)      # then a smaller input on the same scratch
    for cfg in (big, small, big):
        ref = _grow(cfg, static=False)
        got = _grow(cfg, static=True)
        assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
        assert np.array_equal(got[2].view(np.int32), ref[2].view(np.int32))      # same kernels: same bits


def test_static_scratch_rejects_shapes_beyond_its_size():
    lib = ygg.load_library()
    too_big = shape_of(_cfg(64, 2, 64, 128256, seed=1))                       # 64 x 64 rows x 32 chunks of lists
    assert ygg.workspace_bytes(too_big, ygg.OP_EXPAND) > 4 << 20
    cs = too_big.c()
    rc = lib.ygg_equal_growth_expand_static(ctypes.byref(cs), 1, *[ctypes.c_void_p(0x1000)] * 4, None)
    assert rc == 4 and ygg.status_string(rc).startswith("workspace")
