"""Seeded synthetic inputs shared by the tests, the oracle-side checks and the benchmark.

This package manufactures inputs -- weights, prefix KV, token trees, logit matrices -- from
integer seeds, so that the CPU oracle and the HIP library can be handed the very same bytes.
It runs no decoder forward and no sampling, and neither side takes a result from it.  One
generator does hold a small piece of arithmetic of the method's kind: gen_best_first_tree
shapes its trees with a log-softmax and a best-first search over random logits (a stand-in
for a draft model's search).  Its output is only ever an *input* (any topologically ordered
tree is a legal one); no expected value of a test comes from it.
"""
from .gen import (  # noqa: F401
    ModelCfg, CONFIGS, hash_normal, gen_weights, gen_layer, gen_model_ends, gen_prefix_kv, gen_tokens,
    gen_uniform_tree, gen_best_first_tree, gen_chain_tree, gen_expand_inputs, gen_w4, gen_w4_layers,
    gen_crafted_logits, tree_stats,
)
