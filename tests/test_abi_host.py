"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, and turns every host-checkable mistake into a status code
before any kernel is launched."""
import ctypes
import os
import re

import pytest

import paper_2512_23858_amd as ygg
from paper_2512_23858_amd.binding import _CShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE = 0, 1, 2, 3, 4


def _shape(**kw):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, depth=3, width=4, n_nodes=13, vocab=1000,
                kv_dtype=1, softmax_scale=0.0884, kv_capacity=200, max_seq_len=128)
    base.update(kw)
    return ygg.Shape(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ygg.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ygg_[a-z_]+)\s*\(", header))
    assert {"ygg_tree_attention", "ygg_equal_growth_expand", "ygg_accept_and_compact", "ygg_workspace_bytes",
            "ygg_status_string"} <= declared
    lib = ygg.load_library()
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in ygg.h but not exported"


def test_status_strings_are_distinct():
    names = {ygg.status_string(i) for i in range(6)}
    assert len(names) == 6 and ygg.status_string(99) == "unknown status"


def test_workspace_sizes():
    s = _shape()
    for op in (ygg.OP_ATTENTION, ygg.OP_EXPAND, ygg.OP_ACCEPT, ygg.OP_ATTACH):
        n = ygg.workspace_bytes(s, op)
        assert n > 0 and n % 256 == 0
    assert ygg.workspace_bytes(s, 7) == 0
    assert ygg.workspace_bytes(_shape(n_q_heads=7), ygg.OP_ATTENTION) == 0          # Hq % Hkv != 0
    assert ygg.workspace_bytes(_shape(kv_capacity=130), ygg.OP_ATTENTION) == 0      # < max_seq_len + D + 1
    # the attention workspace holds one partial per split and query row: Dh fp16 values and three floats (matrix-core
    # kernels) or Dh + 2 floats (vector kernel)
    big = _shape(max_seq_len=32768, kv_capacity=32800)
    rows = big.batch * big.n_nodes * big.n_q_heads
    per_row = 128 * 2 + 12 if ygg.attention_plan(big)["matrix_cores"] else (128 + 2) * 4
    assert ygg.workspace_bytes(big, ygg.OP_ATTENTION) >= ygg.attention_plan(big)["key_splits"] * rows * per_row


def _call_attention(shape, ptrs, ws=None, ws_bytes=0):
    lib = ygg.load_library()
    cs = shape.c() if shape is not None else None
    args = [ctypes.c_void_p(p) for p in ptrs]
    return lib.ygg_tree_attention(ctypes.byref(cs) if cs is not None else None, *args,
                                  ctypes.c_void_p(ws), ctypes.c_size_t(ws_bytes), None)


FAKE = 0x1000  # never dereferenced on the host: every case below fails validation first


def test_attention_rejects_bad_arguments_on_the_host():
    good = [FAKE] * 8 + [0]   # q kc vc lens kt vt parent out, lse = NULL
    assert _call_attention(None, good) == ERR_NULL
    for i in (0, 3, 4, 5, 6, 7):
        bad = list(good)
        bad[i] = 0
        assert _call_attention(_shape(), bad) == ERR_NULL
    assert _call_attention(_shape(n_q_heads=6, n_kv_heads=4), good) == ERR_SHAPE
    assert _call_attention(_shape(batch=0), good) == ERR_SHAPE
    assert _call_attention(_shape(kv_capacity=100), good) == ERR_SHAPE
    assert _call_attention(_shape(head_dim=96), good) == ERR_UNSUPPORTED
    assert _call_attention(_shape(kv_dtype=5), good) == ERR_UNSUPPORTED
    assert _call_attention(_shape(n_nodes=5000), good) == ERR_UNSUPPORTED
    for bad_scale in (0.0, -0.125, float("inf"), float("nan")):     # row maxima are taken before scaling
        assert _call_attention(_shape(softmax_scale=bad_scale), good) == ERR_SHAPE
    need = ygg.workspace_bytes(_shape(), ygg.OP_ATTENTION)
    assert _call_attention(_shape(), good, ws=0, ws_bytes=need) == ERR_WORKSPACE           # missing
    assert _call_attention(_shape(), good, ws=0x1010, ws_bytes=need) == ERR_WORKSPACE      # misaligned
    assert _call_attention(_shape(), good, ws=0x1000, ws_bytes=need - 1) == ERR_WORKSPACE  # too small


def test_8bit_kv_attention_rejects_bad_arguments_on_the_host():
    lib = ygg.load_library()

    def call(shape, ptrs, ws=0x1000, ws_bytes=1 << 30):
        cs = shape.c()
        return lib.ygg_tree_attention_fp8kv(ctypes.byref(cs), *[ctypes.c_void_p(p) for p in ptrs],
                                            ctypes.c_void_p(ws), ctypes.c_size_t(ws_bytes), None)
    good = [FAKE] * 10 + [0]   # q kc vc lens kt vt k_scale v_scale parent out, lse = NULL
    s8 = _shape(kv_dtype=2)
    for i in (0, 3, 4, 5, 6, 7, 8, 9):
        bad = list(good)
        bad[i] = 0
        assert call(s8, bad) == ERR_NULL
    assert call(_shape(kv_dtype=1), good) == ERR_UNSUPPORTED                 # codes need kv_dtype FP8_E4M3
    assert call(_shape(kv_dtype=2, head_dim=64), good) == ERR_UNSUPPORTED
    assert call(s8, good, ws_bytes=16) == ERR_WORKSPACE
    assert _call_attention(s8, [FAKE] * 8 + [0], ws=0x1000, ws_bytes=1 << 30) == ERR_UNSUPPORTED   # no scales there
    # a K/V slab of one sequence is addressed with 32-bit byte offsets
    huge = _shape(kv_dtype=1, n_kv_heads=8, max_seq_len=3_000_000, kv_capacity=3_000_010)
    assert _call_attention(huge, [FAKE] * 8 + [0], ws=0x1000, ws_bytes=1 << 40) == ERR_UNSUPPORTED
    # 8-bit K/V: at most four computing wavefronts (the loaders take the other slots), in pairs for small trees
    for n_nodes, depth, width, exp in ((13, 3, 4, dict(waves=4, key_shares=2, row_tiles=1)),     # R = 52
                                       (5, 1, 4, dict(waves=2, key_shares=2, row_tiles=1)),      # R = 20
                                       (129, 8, 16, dict(waves=4, key_shares=1, row_tiles=5))):  # R = 516
        got = ygg.attention_plan(_shape(kv_dtype=2, n_nodes=n_nodes, depth=depth, width=width))
        assert got["matrix_cores"] and all(got[k] == v for k, v in exp.items()), got


def test_expand_rejects_bad_arguments_on_the_host():
    lib = ygg.load_library()

    def call(shape, d, ptrs, ws=0x1000, ws_bytes=1 << 30):
        cs = shape.c()
        return lib.ygg_equal_growth_expand(ctypes.byref(cs), d, *[ctypes.c_void_p(p) for p in ptrs],
                                           ctypes.c_void_p(ws), ctypes.c_size_t(ws_bytes), None)
    good = [FAKE] * 4
    assert call(_shape(), 0, good) == ERR_SHAPE            # d out of range
    assert call(_shape(), 4, good) == ERR_SHAPE
    assert call(_shape(n_nodes=14), 1, good) == ERR_SHAPE  # N != 1 + D*W
    assert call(_shape(width=65, n_nodes=196), 1, good) == ERR_UNSUPPORTED
    assert call(_shape(vocab=2, width=4), 1, good) == ERR_SHAPE   # fewer candidates than slots at depth 1
    assert call(_shape(vocab=600000, width=64, n_nodes=193), 2, good) == ERR_UNSUPPORTED   # too many chunk lists
    assert call(_shape(), 1, [0] + good[1:]) == ERR_NULL
    assert call(_shape(), 1, good, ws_bytes=16) == ERR_WORKSPACE


def test_attach_rejects_bad_arguments_on_the_host():
    lib = ygg.load_library()

    def call(shape, t, ptrs, pool=0x2000, pool_bytes=1 << 30, ws=0x1000, ws_bytes=1 << 30):
        cs = shape.c()
        return lib.ygg_equal_growth_attach(ctypes.byref(cs), t, *[ctypes.c_void_p(p) for p in ptrs],
                                           ctypes.c_void_p(pool), ctypes.c_size_t(pool_bytes),
                                           ctypes.c_void_p(ws), ctypes.c_size_t(ws_bytes), None)
    good = [FAKE] * 4
    assert call(_shape(), 0, good) == ERR_SHAPE            # step out of range
    assert call(_shape(), 4, good) == ERR_SHAPE
    assert call(_shape(n_nodes=14), 1, good) == ERR_SHAPE  # N != 1 + D*W
    assert call(_shape(vocab=3, width=4), 1, good) == ERR_SHAPE          # a row cannot offer W tokens
    assert call(_shape(width=64, n_nodes=193, vocab=9000), 2, good) == ERR_UNSUPPORTED   # W*W offers + pool > 4096 entries
    assert call(_shape(vocab=600000, width=32, n_nodes=97), 2, good) == ERR_UNSUPPORTED  # a row's chunk lists > 4096 entries
    assert call(_shape(), 1, [0] + good[1:]) == ERR_NULL
    assert call(_shape(), 1, good, pool=0) == ERR_NULL
    assert call(_shape(), 1, good, pool=0x2008) == ERR_WORKSPACE          # pool not 16-byte aligned
    assert call(_shape(), 1, good, pool_bytes=64) == ERR_WORKSPACE
    assert call(_shape(), 1, good, ws_bytes=16) == ERR_WORKSPACE
    s = _shape()
    assert ygg.attach_pool_bytes(s) >= s.batch * (16 + s.width * (s.depth - 1) * 16)
    assert ygg.workspace_bytes(s, ygg.OP_ATTACH) > ygg.workspace_bytes(s, ygg.OP_EXPAND)


def test_prune_rejects_bad_arguments_on_the_host():
    lib = ygg.load_library()

    def call(shape, w, ins, t_ver, outs, extra, t_draft=1.0):
        cs = shape.c()
        return lib.ygg_prune_for_verification(ctypes.byref(cs), w, *[ctypes.c_void_p(p) for p in ins],
                                              ctypes.c_void_p(t_ver), ctypes.c_float(t_draft),
                                              *[ctypes.c_void_p(p) for p in outs + extra], None)
    ins, outs = [FAKE] * 3, [FAKE] * 3
    assert call(_shape(), 0, ins, FAKE, outs, [FAKE, FAKE]) == ERR_SHAPE      # width out of range
    assert call(_shape(), 14, ins, FAKE, outs, [FAKE, FAKE]) == ERR_SHAPE
    assert call(_shape(), 5, ins, FAKE, outs, [FAKE, FAKE], t_draft=-1.0) == ERR_SHAPE
    assert call(_shape(), 5, [0] + ins[1:], FAKE, outs, [FAKE, FAKE]) == ERR_NULL
    assert call(_shape(), 5, ins, FAKE, [0] + outs[1:], [FAKE, FAKE]) == ERR_NULL
    assert call(_shape(), 5, ins, 0, outs, [FAKE, FAKE]) == ERR_NULL           # best_width wanted without a latency table
    assert call(_shape(n_nodes=2000, depth=3, width=4), 5, ins, FAKE, outs, [FAKE, FAKE]) in (ERR_SHAPE, ERR_UNSUPPORTED)


def test_validator_rejects_bad_arguments_on_the_host():
    lib = ygg.load_library()
    cs = _shape().c()
    f = lambda flags, rows, logits: lib.ygg_debug_validate(ctypes.byref(cs), *[ctypes.c_void_p(FAKE)] * 3, ctypes.c_void_p(logits),
                                                           rows, ctypes.c_void_p(flags), None)
    assert f(0, 1, FAKE) == ERR_NULL
    assert f(FAKE, 0, FAKE) == ERR_SHAPE      # logits without a row count
    bad = _shape(n_nodes=0).c()
    assert lib.ygg_debug_validate(ctypes.byref(bad), None, None, None, None, 0, ctypes.c_void_p(FAKE), None) == ERR_SHAPE


def test_accept_rejects_bad_arguments_on_the_host():
    lib = ygg.load_library()

    def call(shape, n_layers, ptrs, ws=0x1000, ws_bytes=1 << 30):
        cs = shape.c()
        return lib.ygg_accept_and_compact(ctypes.byref(cs), n_layers, *[ctypes.c_void_p(p) for p in ptrs],
                                          ctypes.c_void_p(ws), ctypes.c_size_t(ws_bytes), None)
    # target_logits target_tokens parent token kt vt kc vc lens alen apath bonus
    good = [FAKE, 0] + [FAKE] * 10
    assert call(_shape(), 1, [FAKE, FAKE] + good[2:]) == ERR_NULL      # both targets
    assert call(_shape(), 1, [0, 0] + good[2:]) == ERR_NULL            # neither
    assert call(_shape(), -1, good) == ERR_SHAPE
    bad = list(good)
    bad[6] = 0
    assert call(_shape(), 1, bad) == ERR_NULL                          # cache missing while n_layers > 0
    assert call(_shape(), 1, good, ws_bytes=8) == ERR_WORKSPACE
    assert call(_shape(head_dim=100), 1, good) == ERR_UNSUPPORTED


def test_shape_struct_layout_matches_header():
    # 10 x int32/float (4 bytes each) + padding to 8 + int64 + int32 + tail padding
    assert ctypes.sizeof(_CShape) == 56
    assert _CShape.kv_capacity.offset == 40 and _CShape.max_seq_len.offset == 48


def test_attention_plans_of_the_five_configurations():
    """The launch shapes the measurements were taken with (a change here is a performance change)."""
    import ygg_workloads as wl
    want = {1: dict(matrix_cores=False),
            2: dict(matrix_cores=True, waves=4, key_shares=2, row_tiles=1, key_splits=6),
            3: dict(matrix_cores=True, waves=6, key_shares=1, row_tiles=3, key_splits=10),
            4: dict(matrix_cores=True, waves=8, key_shares=1, row_tiles=6, key_splits=5),
            # a batch: 16 equal runs of the concatenated key tiles per (kv head, row tile) = 256 workgroups
            5: dict(matrix_cores=True, waves=8, key_shares=1, row_tiles=2, key_splits=16)}
    for c, exp in want.items():
        cfg = wl.CONFIGS[c]
        s = ygg.Shape(batch=cfg.batch, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                      depth=cfg.depth, width=cfg.width, n_nodes=cfg.n_nodes, vocab=cfg.vocab,
                      kv_dtype=0 if cfg.dtype == "f32" else 1, softmax_scale=cfg.softmax_scale,
                      kv_capacity=cfg.kv_capacity, max_seq_len=cfg.max_prefix)
        got = ygg.attention_plan(s)
        for k, v in exp.items():
            assert got[k] == v, (c, k, got)
    # the workspace follows the plan: one record per split and query row (Dh fp16 values + three floats, or Dh + 2 floats)
    s2 = _shape(max_seq_len=4096, kv_capacity=4200)
    p = ygg.attention_plan(s2)
    rows = s2.batch * s2.n_nodes * s2.n_q_heads
    per_row = 128 * 2 + 12 if p["matrix_cores"] else (128 + 2) * 4
    need = p["key_splits"] * rows * per_row
    assert need <= ygg.workspace_bytes(s2, ygg.OP_ATTENTION) < need + 3 * 256
    # head_dim 64 in bf16 runs on the matrix cores too (fp32 storage stays on the vector path)
    s3 = _shape(head_dim=64, max_seq_len=4096, kv_capacity=4200)
    p3 = ygg.attention_plan(s3)
    assert p3["matrix_cores"] and not ygg.attention_plan(_shape(head_dim=64, kv_dtype=0))["matrix_cores"]
    need = p3["key_splits"] * rows * (64 * 2 + 12)
    assert need <= ygg.workspace_bytes(s3, ygg.OP_ATTENTION) < need + 3 * 256


def test_plan_override_is_explicit_and_removable():
    """The tuning override is a call, not an environment variable, and leaves no trace once removed."""
    import os
    s = _shape(max_seq_len=4096, kv_capacity=4200)
    base = ygg.attention_plan(s)
    os.environ["YGG_ATTN_PLAN"] = "8,1,3,2"
    try:
        assert ygg.attention_plan(s) == base            # the environment is not consulted
    finally:
        del os.environ["YGG_ATTN_PLAN"]
    ygg.set_attention_plan(nsplit=3)
    try:
        forced = ygg.attention_plan(s)
        assert forced["key_splits"] == 3 and forced["waves"] == base["waves"]
        ygg.set_attention_plan(waves=2, rblocks=1, kshares=2)
        assert ygg.attention_plan(s)["waves"] == 2 and ygg.attention_plan(s)["key_shares"] == 2
        ygg.set_attention_plan(waves=5, rblocks=1, kshares=1)   # unknown shape: ignored
        assert ygg.attention_plan(s)["waves"] == base["waves"]
    finally:
        ygg.set_attention_plan()
    assert ygg.attention_plan(s) == base
