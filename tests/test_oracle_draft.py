"""Pins for oracle/draft.py (Alg. 2, createDraftTree): brute-force enumeration of every continuation of a
tiny model, the invariants App. A states for the optimal tree, and the batch-size-one special case, which is
textbook best-first search."""
import itertools

import numpy as np
import pytest

import oracle
from workloads import ModelCfg, gen_weights, gen_tokens


@pytest.fixture(scope="module")
def tiny():
    cfg = ModelCfg(2, 32, 2, 2, 16, 48, 5, dtype="fp32")          # vocabulary of 5: all continuations can be listed
    w = gen_weights(cfg, seed=51)
    f = lambda t: t.double().numpy()
    w = dict(embed=f(w["embed"]) * 50, final_norm=f(w["final_norm"]), lm_head=f(w["lm_head"]) * 8,
             layers=[{k: (f(v) * (1 if k.endswith("norm") else 8)) for k, v in lw.items()} for lw in w["layers"]])
    prefix = gen_tokens(4, cfg.vocab, seed=52)
    _, pk, pv = oracle.path_forward(cfg, w, None, None, prefix, return_kv=True)
    return cfg, w, pk, pv


def _all_continuations(cfg, w, pk, pv, root, depth):
    """log-probability of every token sequence of length 1..depth after the root, by plain causal forwards."""
    from scipy.special import log_softmax
    out = {(): 0.0}
    frontier = [()]
    for _ in range(depth):
        nxt = []
        for path in frontier:
            lg = oracle.path_forward(cfg, w, pk, pv, [root] + list(path))
            lp = log_softmax(lg)
            for t in range(cfg.vocab):
                out[path + (t,)] = out[path] + float(lp[t])
                nxt.append(path + (t,))
        frontier = nxt
    return out


def _paths(tree):
    paths = []
    for i in range(len(tree["tokens"])):
        p, j = [], i
        while tree["parent"][j] >= 0:
            p.append(int(tree["tokens"][j]))
            j = int(tree["parent"][j])
        paths.append(tuple(reversed(p)))
    return paths


def test_batch_of_one_is_best_first_search_and_finds_the_most_probable_continuations(tiny):
    """B = 1, k = vocabulary, enough iterations: the tree is the root plus the K-1 most probable continuations
    among ALL sequences (App. A: the optimal tree), found here by listing every sequence up to depth 4."""
    cfg, w, pk, pv = tiny
    root, K = 3, 10
    tree = oracle.create_draft_tree(cfg, w, pk, pv, root, K=K, D=200, B=1, k=cfg.vocab)
    allp = _all_continuations(cfg, w, pk, pv, root, depth=5)
    best = sorted(allp.items(), key=lambda kv: -kv[1])[:K]
    assert max(len(p) for p, _ in best) < 5                       # the enumeration went deep enough to contain the optimum
    assert sorted(_paths(tree)) == sorted(p for p, _ in best)
    got = dict(zip(_paths(tree), tree["cum_logp"]))
    for p, lp in best:
        assert abs(got[p] - lp) <= 1e-5


@pytest.mark.parametrize("K,D,B,k", [(10, 6, 4, 3), (25, 8, 8, 5), (7, 3, 16, 2), (40, 5, 3, 4)])
def test_invariants_for_batched_construction(tiny, K, D, B, k):
    cfg, w, pk, pv = tiny
    tree = oracle.create_draft_tree(cfg, w, pk, pv, 1, K=K, D=D, B=B, k=k)
    tok, par, cum = tree["tokens"], tree["parent"], tree["cum_logp"]
    n = len(tok)
    assert 1 <= n <= K and n <= 1 + (D - 1) * B + 0 * k and tok[0] == 1 and par[0] == -1 and cum[0] == 0.0
    assert all(-1 <= par[i] < i for i in range(n)) and list(par).count(-1) == 1
    # a node's score is its path's log-probability under the model, and never above its parent's
    allp = _all_continuations(cfg, w, pk, pv, 1, depth=min(D - 1, 4))
    for p, c in zip(_paths(tree), cum):
        if len(p) <= 4:
            assert abs(allp[p] - c) <= 1e-4
    assert all(cum[i] <= cum[par[i]] + 1e-7 for i in range(1, n))
    # siblings carry different tokens; depth is bounded by the number of iterations
    assert len(set(zip(par.tolist(), tok.tolist()))) == n
    assert max(len(p) for p in _paths(tree)) <= D - 1 or D == 1


def test_large_batch_and_depth_contain_the_sequential_optimum(tiny):
    """With B and D large enough that nothing is cut early, batched construction must find the same K best
    continuations as one-at-a-time best-first search (the order of expansion does not matter then)."""
    cfg, w, pk, pv = tiny
    a = oracle.create_draft_tree(cfg, w, pk, pv, 2, K=9, D=200, B=1, k=cfg.vocab)
    b = oracle.create_draft_tree(cfg, w, pk, pv, 2, K=9, D=12, B=64, k=cfg.vocab)
    assert sorted(_paths(a)) == sorted(_paths(b))
