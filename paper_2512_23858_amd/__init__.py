"""MI355X (gfx950) tree-verification hot path of Yggdrasil-style speculative decoding.

The work is done by hand-written HIP kernels behind a C ABI (include/ygg.h, built into
libygg.so).  This package is only the thin Python binding with the same entry points;
PyTorch is used for device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    Shape,
    accept_and_compact,
    attach_pool_bytes,
    attention_plan,
    debug_validate,
    equal_growth_attach,
    equal_growth_expand,
    equal_growth_expand_static,
    init,
    lib_path,
    load_library,
    new_workspace,
    prune_for_verification,
    set_attention_plan,
    status_string,
    tree_attention,
    tree_attention_fp8kv,
    workspace_bytes,
    OP_ATTENTION,
    OP_EXPAND,
    OP_ACCEPT,
    OP_ATTACH,
    F32,
    BF16,
    FP8_E4M3,
)
