"""MI355X-native SpecExec verification hot path: thin Python binding over libspecexec_mi.so.

The library (hand-written HIP for gfx950, C ABI declared in include/specexec_mi.h) does all the
work; this package only marshals torch tensors into pointers.  There is no fallback path: if
the shared library has not been built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    lib, SxError, ModelWeights, verify_tree, verify_tree_workspace, verify_tree_range, commit_kv, specexec_round, RoundBuffers, draft_tree, accept_walk, expand_topk, expand_topk_static,
    row_logsoftmax_topk, gemm_bf16, gemm_w4a16_bf16, qkv_rope_bf16, tree_attention_bf16, check_status, status_string, version,
    LIB_PATH, EXPORTS, profile_enable, profile_select, profile_disable, profile_read, KERNEL_CLASSES,
)
