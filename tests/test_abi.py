"""The C ABI without a GPU: the library loads, exports every function the header declares, and
turns host-visible mistakes into status codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sx():
    import paper_2406_02532_amd as m
    return m


def test_every_declared_symbol_is_exported(sx):
    hdr = open(os.path.join(ROOT, "include", "specexec_mi.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sx_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(sx.EXPORTS)
    raw = C.CDLL(sx.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def test_version_and_status_strings(sx):
    assert sx.version() >= 1
    for code in range(0, -7, -1):
        assert sx.status_string(code) != "unknown status"
    assert sx.status_string(-99) == "unknown status"


def test_workspace_queries(sx):
    from workloads import CONFIGS, ModelCfg
    for name in ("C1", "C2", "C3", "C5"):
        c = CONFIGS[name]
        assert sx.verify_tree_workspace(c["cfg"], c["P"], c["T"]) > 0
    bad = ModelCfg(1, 4096, 32, 32, 64, 11008, 32000, dtype="bf16")       # bf16 path needs head_dim 128
    assert sx.verify_tree_workspace(bad, 16, 16) == 0
    assert sx.lib.sx_expand_topk_workspace(2048, 32000, 32, 2048) >= 3 * 2048 * 32 * 4
    assert sx.lib.sx_accept_walk_workspace(64, 1024) >= 4096
    assert sx.lib.sx_tree_attention_workspace(2048, 64, 8) > 0
    assert sx.lib.sx_tree_attention_workspace(2048, 64, 7) == 0


def test_host_side_errors_return_codes(sx):
    L = sx.lib
    one = C.c_void_p(256)      # a non-null, aligned fake address; these calls fail before any launch
    assert L.sx_expand_topk(None, one, 4, 100, 2, 4, one, one, one, one, one, 1 << 20, None) == -1
    assert L.sx_expand_topk(one, one, 4, 100, 200, 4, one, one, one, one, one, 1 << 20, None) == -2    # k > V
    assert L.sx_expand_topk(one, one, 4, 100, 2, 100000, one, one, one, one, one, 1 << 20, None) == -2  # B too large
    assert L.sx_expand_topk(one, one, 4, 100, 2, 4, one, one, one, one, None, 0, None) == -3
    assert L.sx_expand_topk(one, one, 4, 100, 2, 4, one, one, one, one, C.c_void_p(264), 1 << 20, None) == -3  # misaligned
    assert L.sx_expand_topk(one, one, 4, 100, 2, 4, one, one, one, one, one, 16, None) == -3
    assert L.sx_expand_topk_static(one, one, 4097, 32000, 16, 64, one, one, one, one, None) == -2      # > 65536 candidates
    assert L.sx_expand_topk_static(one, one, 4, 100, 2, 4, one, None, one, one, None) == -1
    assert L.sx_accept_walk(one, None, one, one, 4, 100, 0.6, 1.5, 1, 0, one, one, one, one, 1 << 20, None) == -2
    assert L.sx_accept_walk(one, None, one, one, 4, 1 << 20, 0.6, 0.9, 1, 0, one, one, one, one, 1 << 20, None) == -2
    assert L.sx_accept_walk(one, None, None, one, 4, 100, 0.6, 0.9, 1, 0, one, one, one, one, 1 << 20, None) == -1
    assert L.sx_gemm_bf16(one, one, None, one, 8, 8, 100, 0, None) == -2          # K % 64 != 0
    assert L.sx_gemm_bf16(one, one, None, one, 8, 8, 128, 2, None) == -1          # SwiGLU needs W2
    assert L.sx_gemm_bf16(one, one, None, one, 256, 262144, 8192, 0, None) == -2  # W of 4 GiB: 32-bit offsets would wrap
    assert L.sx_gemm_bf16(one, one, None, one, 64, 262144, 8192, 0, None) == -2   # the same through the narrow-tile kernel
    assert L.sx_gemm_bf16(one, one, None, one, 65536, 64, 32768, 1, None) == -2   # X of 4 GiB
    assert L.sx_gemm_bf16_workspace() >= 1024 + 256 * 256 * 4
    assert L.sx_gemm_bf16_ws(one, one, None, one, 8, 8, 128, 0, C.c_void_p(264), 1 << 20, None) == -3   # misaligned workspace
    assert L.sx_gemm_bf16_ws(one, one, None, one, 8, 8, 100, 0, one, 1 << 20, None) == -2               # K % 64 != 0
    assert L.sx_verify_tree(None, None, None, 0, one, one, 4, one, None, None, one, 1 << 20, None) == -1
    assert L.sx_row_logsoftmax_topk(one, 4, 100, 300, one, one, None) == -2
