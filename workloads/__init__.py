"""Seeded synthetic inputs shared by the tests, the oracle-side checks and the benchmark.

Nothing in this package performs the method's arithmetic (no decoder forward, no
log-softmax/top-k selection results, no sampling): it only manufactures inputs --
weights, prefix KV, token trees, logit matrices -- from integer seeds, so that the CPU
oracle and the HIP library can be handed the very same bytes.
"""
from .gen import (  # noqa: F401
    ModelCfg, CONFIGS, hash_normal, gen_weights, gen_prefix_kv, gen_tokens,
    gen_uniform_tree, gen_best_first_tree, gen_chain_tree, gen_expand_inputs, gen_w4,
    gen_crafted_logits, tree_stats,
)
