"""CPU oracle for the SpecExec verification hot path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy restatements of what the path computes, written from the paper
(Alg. 1, Alg. 2, App. A, App. D) and the standard Llama-style decoder definition.  It
shares no code with the HIP library and never imports it; only tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import this package.  The product path must
never route through it.

Parity status: every function here is pinned by tests that do not depend on this code
(library routines, closed forms, brute force, hand-worked fixtures); see
tests/test_oracle_*.py.
"""
from .model import (  # noqa: F401
    tree_depths, ancestors, rmsnorm, rope, tree_attention, verify_tree, path_forward,
    round_bf16,
)
from .generate import specexec_generate  # noqa: F401
from .draft import create_draft_tree  # noqa: F401
from .sampling import (  # noqa: F401
    uniform01, sample_token, accept_walk, sequential_sample, warped_distribution, trial_uniform, specinfer_walk,
)
from .quant import unpack_w4, dequantize_w4, gemm_w4a16  # noqa: F401
from .expand import log_softmax, row_topk, expand_topk  # noqa: F401
