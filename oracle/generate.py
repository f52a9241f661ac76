"""Oracle (test infrastructure): the outer loop of Alg. 1 -- verify a tree, walk it, let the accepted
tokens join the context, repeat -- in the plainest form: nothing is cached between rounds, the
prefix keys and values are recomputed from scratch by an ordinary causal forward every round.

What pins it: Sect. 4.1.  Whatever trees are offered, the tokens this loop emits are the ones
token-by-token sampling from the target model emits with the same seed (`sequential_sample`), because
the uniform that decides the token at an absolute position is a function of (seed, position) alone.
"""
from __future__ import annotations

import numpy as np

from .model import path_forward, verify_tree
from .sampling import accept_walk


def specexec_generate(cfg, w, prompt, n_rounds, tree_fn, temperature, top_p, seed, return_cache=False):
    """prompt: token ids, at least one; its last token is the root of the first tree (the "bonus"
    token whose successor is not yet known), the tokens before it are the prefix.
    tree_fn(context, round) -> (tokens, parent) with tokens[0] == context[-1], parent[0] == -1.
    Returns (generated tokens, number of tokens emitted per round); each round emits
    1 + (accepted draft tokens) tokens.  With return_cache also the prefix K/V [L][P][Hkv][Dh] that
    the final context (minus its last token) implies."""
    context = [int(t) for t in prompt]
    out, per_round = [], []
    for r in range(n_rounds):
        prefix = context[:-1]
        if prefix:
            _, pk, pv = path_forward(cfg, w, None, None, prefix, return_kv=True)
        else:
            pk = pv = np.zeros((cfg.n_layers, 0, cfg.n_kv_heads, cfg.head_dim))
        tokens, parent = tree_fn(list(context), r)
        assert int(tokens[0]) == context[-1] and int(parent[0]) == -1
        logits = verify_tree(cfg, w, pk, pv, tokens, parent)["logits"]
        walk = accept_walk(logits, tokens, parent, temperature, top_p, seed, pos0=len(prefix))
        out += walk["tokens"]
        per_round.append(len(walk["tokens"]))
        context += walk["tokens"]
    if return_cache:
        _, pk, pv = path_forward(cfg, w, None, None, context[:-1], return_kv=True)
        return out, per_round, pk, pv
    return out, per_round
