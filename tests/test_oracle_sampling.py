"""Pins for oracle/sampling.py: published RNG vectors, hand-worked nucleus cases, a chi-square
test against exact probabilities, and the paper's seed-exact equivalence with sequential
sampling (Sect. 4.1, Correctness)."""
import json
import os

import numpy as np
import pytest

import oracle
from workloads import ModelCfg, gen_weights, gen_tokens, gen_uniform_tree

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_uniform01_uses_published_splitmix64_outputs():
    g = json.load(open(os.path.join(GOLD, "splitmix64.json")))
    for pos, hx in enumerate(g["outputs_hex"]):
        assert oracle.uniform01(g["seed"], pos) == (int(hx, 16) >> 40) * 2.0 ** -24


def test_uniform01_range_and_uniformity():
    u = np.array([oracle.uniform01(123, p) for p in range(20000)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))
    hist = np.bincount((u * 20).astype(int), minlength=20)
    chi2 = ((hist - 1000.0) ** 2 / 1000.0).sum()
    assert chi2 < 50.0          # 19 dof, p ~ 1e-4


def test_nucleus_hand_cases():
    g = json.load(open(os.path.join(GOLD, "nucleus_cases.json")))
    for c in g["cases"]:
        tok, _ = oracle.sample_token(np.log(np.array(c["p"])), c["t"], c["top_p"], c["u"])
        assert tok == c["token"], c["work"]


def test_plain_categorical_chi_square():
    """t=1, top_p=1: the draw is the plain categorical distribution."""
    p = np.array([0.02, 0.4, 0.08, 0.25, 0.05, 0.2])
    n = 100000
    cnt = np.zeros(6)
    for s in range(n):
        tok, _ = oracle.sample_token(np.log(p), 1.0, 1.0, oracle.uniform01(s, 17))
        cnt[tok] += 1
    chi2 = ((cnt - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 25.7          # 5 dof, p ~ 1e-4


def test_top_p_zero_and_t_zero_are_greedy():
    r = np.random.default_rng(0)
    for _ in range(50):
        x = r.standard_normal(40)
        a, _ = oracle.sample_token(x, 0.0, 0.9, r.uniform())
        b, _ = oracle.sample_token(x, 0.7, 1e-9, r.uniform())
        assert a == b == int(np.argmax(x))


def test_nucleus_never_leaves_the_brute_force_set():
    """Brute force: enumerate the nucleus by repeated removal of the maximum."""
    r = np.random.default_rng(1)
    for trial in range(200):
        x = r.standard_normal(12) * 2
        t, top_p, u = 0.6, 0.9, r.uniform()
        p = np.exp(x / t)
        p /= p.sum()
        rest, nucleus, mass = list(range(12)), [], 0.0
        while mass < top_p:
            j = max(rest, key=lambda i: (p[i], -i))
            nucleus.append(j)
            rest.remove(j)
            mass += p[j]
        tok, m = oracle.sample_token(x, t, top_p, u)
        assert tok in nucleus
        # and the draw is the inverse CDF in id order
        acc = 0.0
        for j in sorted(nucleus):
            acc += p[j]
            if acc > u * mass:
                break
        if m["m_u"] > 1e-12 and m["m_p"] > 1e-12:
            assert tok == j


@pytest.fixture(scope="module")
def model():
    cfg = ModelCfg(2, 32, 2, 2, 16, 48, 12, dtype="fp32")
    w = gen_weights(cfg, seed=21)
    f = lambda t: t.double().numpy()
    w = dict(embed=f(w["embed"]) * 50, final_norm=f(w["final_norm"]), lm_head=f(w["lm_head"]) * 40,
             layers=[{k: (f(v) * (1 if k.endswith("norm") else 8)) for k, v in lw.items()} for lw in w["layers"]])
    prefix = gen_tokens(6, cfg.vocab, seed=22)
    _, pk, pv = oracle.path_forward(cfg, w, None, None, prefix, return_kv=True)
    return cfg, w, pk, pv


def test_walk_equals_sequential_sampling_for_every_seed(model):
    """Sect. 4.1: with the RNG fixed, walking the cache gives exactly the tokens that
    sequential sampling gives.  Trees: uniform random ones over a 12-token vocabulary, so
    that walks of several steps occur."""
    cfg, w, pk, pv = model
    P = pk.shape[1]
    lengths = []
    for s in range(30):
        tok, par = gen_uniform_tree(40, cfg.vocab, seed=100 + s)
        logits = oracle.verify_tree(cfg, w, pk, pv, tok, par)["logits"]
        res = oracle.accept_walk(logits, tok, par, 0.6, 0.9, seed=s, pos0=P)
        ref = oracle.sequential_sample(cfg, w, pk, pv, tok[0], len(res["tokens"]), 0.6, 0.9, seed=s, pos0=P)
        assert res["tokens"] == ref
        # the path is a root-to-node chain whose tokens are the sampled ones
        assert res["path"][0] == 0 and len(res["path"]) == len(res["tokens"])
        for a, b, x in zip(res["path"], res["path"][1:], res["tokens"]):
            assert par[b] == a and tok[b] == x
        lengths.append(len(res["tokens"]))
    assert max(lengths) >= 3            # the test did walk down the tree


def test_greedy_walk_follows_argmax(model):
    cfg, w, pk, pv = model
    tok, par = gen_uniform_tree(40, cfg.vocab, seed=7)
    logits = oracle.verify_tree(cfg, w, pk, pv, tok, par)["logits"]
    res = oracle.accept_walk(logits, tok, par, 0.0, 1.0, seed=0, pos0=pk.shape[1])
    for node, x in zip(res["path"], res["tokens"]):
        assert x == int(np.argmax(logits[node]))
    last = res["path"][-1]
    assert not np.any((par == last) & (tok == res["tokens"][-1]))


def test_duplicate_sibling_goes_to_lowest_index():
    tok = np.array([5, 3, 3, 9])
    par = np.array([-1, 0, 0, 1])
    logits = np.full((4, 10), -20.0)
    logits[0, 3] = 0.0
    logits[1, 9] = 0.0
    logits[2, 1] = 0.0
    logits[3, 2] = 0.0
    res = oracle.accept_walk(logits, tok, par, 0.0, 1.0, seed=1, pos0=0)
    assert res["path"] == [0, 1, 3] and res["tokens"] == [3, 9, 2]


def test_generation_over_many_rounds_equals_sequential_sampling(model):
    """Sect. 4.1 across rounds (Alg. 1's outer loop): whatever trees are offered each round -- here random
    ones over a 12-token vocabulary, so rounds accept 0 to several draft tokens -- the emitted stream is the
    token-by-token sample with the same seed, and the context grows by exactly the emitted tokens."""
    cfg, w, _, _ = model
    prompt = [int(t) for t in gen_tokens(5, cfg.vocab, seed=31)]
    for s in range(6):
        def tree_fn(context, r, s=s):
            tok, par = gen_uniform_tree(30, cfg.vocab, seed=1000 * s + r)
            tok = tok.copy()
            tok[0] = context[-1]
            return tok, par
        out, per_round = oracle.specexec_generate(cfg, w, prompt, 5, tree_fn, 0.6, 0.9, seed=s)
        assert len(per_round) == 5 and min(per_round) >= 1 and sum(per_round) == len(out)
        _, pk, pv = oracle.path_forward(cfg, w, None, None, prompt[:-1], return_kv=True)
        ref = oracle.sequential_sample(cfg, w, pk, pv, prompt[-1], len(out), 0.6, 0.9, seed=s, pos0=len(prompt) - 1)
        assert out == ref
    # trees that contain the next two tokens of the true stream (plus random siblings): such rounds must
    # accept exactly those two and emit a third
    _, pk, pv = oracle.path_forward(cfg, w, None, None, prompt[:-1], return_kv=True)
    truth = oracle.sequential_sample(cfg, w, pk, pv, prompt[-1], 12, 0.6, 0.9, seed=3, pos0=len(prompt) - 1)

    def informed(context, r):
        done = len(context) - len(prompt)
        tok, par = gen_uniform_tree(12, cfg.vocab, seed=77 + r)
        tok, par = list(tok), list(par)
        tok[0] = context[-1]
        tok += [truth[done], truth[done + 1]]
        par += [0, len(tok) - 2]
        # random siblings that happen to carry the true token would be walked first: rename them
        for i in range(1, len(tok) - 2):
            if par[i] == 0 and tok[i] == truth[done]:
                tok[i] = (tok[i] + 1) % cfg.vocab
        return np.array(tok, np.int32), np.array(par, np.int32)

    out, per_round = oracle.specexec_generate(cfg, w, prompt, 3, informed, 0.6, 0.9, seed=3)
    assert out == truth[:len(out)] and all(n >= 3 for n in per_round)
