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


# ------------------------------------------------------------------------------------------------
# specinfer_walk: acceptance with probability P_target / P_draft (Sect. 4.1, "Comparison to
# speculative decoding").  What fixes it: the emitted tokens must follow the target's (warped)
# distribution whatever the draft distribution is, and a single drafted token is accepted with
# probability sum_x min(p(x), q(x)) (the closed form of speculative sampling).
# ------------------------------------------------------------------------------------------------

_P6 = np.array([0.02, 0.4, 0.08, 0.25, 0.05, 0.2])
_Q6 = np.array([0.3, 0.1, 0.25, 0.05, 0.2, 0.1])


def _star_tree(child_tokens):
    """Root (token 0) with the given children."""
    tokens = np.array([0] + list(child_tokens), dtype=np.int32)
    parent = np.array([-1] + [0] * len(child_tokens), dtype=np.int32)
    return tokens, parent


def _rows(n, row):
    return np.tile(np.asarray(row, dtype=np.float64), (n, 1))


@pytest.mark.parametrize("k", [1, 3])
def test_specinfer_first_token_follows_the_target_distribution(k):
    """k children drawn independently from q by the test's own generator (equal tokens stay separate
    children); the first emitted token must be distributed as p.  chi-square, 5 dof."""
    r = np.random.default_rng(100 + k)
    n, cnt, accepted = 40000, np.zeros(6), 0
    for s in range(n):
        kids = r.choice(6, size=k, p=_Q6)
        tokens, parent = _star_tree(kids)
        w = oracle.specinfer_walk(_rows(k + 1, np.log(_P6)), _rows(k + 1, _Q6), tokens, parent, 1.0, 1.0, seed=s, pos0=5)
        cnt[w["tokens"][0]] += 1
        accepted += len(w["path"]) > 1
        assert len(w["tokens"]) == len(w["path"]) and all(tokens[c] == t for c, t in zip(w["path"][1:], w["tokens"]))
    chi2 = ((cnt - n * _P6) ** 2 / (n * _P6)).sum()
    assert chi2 < 25.7, (chi2, cnt / n)      # p ~ 1e-4
    if k == 1:   # one drafted token is accepted with probability sum min(p, q) = 0.47
        exp = np.minimum(_P6, _Q6).sum()
        assert abs(accepted / n - exp) < 4 * np.sqrt(exp * (1 - exp) / n), (accepted / n, exp)


def test_specinfer_warped_target_and_plain_sampling_agree_in_distribution():
    """With temperature and nucleus the target is the warped distribution; the draft one is used as given."""
    logits = np.log(_P6)
    p = oracle.warped_distribution(logits, 0.7, 0.9)
    assert abs(p.sum() - 1) < 1e-12 and (p == 0).sum() >= 1          # the nucleus drops the tail
    # the very distribution sample_token draws from: frequencies over a fine grid of uniforms
    grid = (np.arange(20000) + 0.5) / 20000
    freq = np.bincount([oracle.sample_token(logits, 0.7, 0.9, u)[0] for u in grid], minlength=6) / len(grid)
    assert np.abs(freq - p).max() < 1e-4
    r = np.random.default_rng(7)
    n, cnt = 40000, np.zeros(6)
    for s in range(n):
        tokens, parent = _star_tree(r.choice(6, size=2, p=_Q6))
        w = oracle.specinfer_walk(_rows(3, logits), _rows(3, _Q6), tokens, parent, 0.7, 0.9, seed=s, pos0=0)
        cnt[w["tokens"][0]] += 1
    keep = p > 0
    assert cnt[~keep].sum() == 0
    chi2 = ((cnt[keep] - n * p[keep]) ** 2 / (n * p[keep])).sum()
    assert chi2 < 27.9, (chi2, cnt / n, p)


def test_specinfer_two_levels_joint_distribution():
    """Depth 2: the pair of the first two emitted tokens must follow p1(x1) * p2(x2 | node of x1) -- the walk has
    to move to the accepted child and use that child's rows.  A second token exists only after an acceptance, so
    the comparison is made on the joint counts of accepted-first-token x second token, against p1-mass accepted."""
    V = 4
    p1, q1 = np.array([0.1, 0.2, 0.3, 0.4]), np.array([0.4, 0.3, 0.2, 0.1])
    p2 = [np.array([0.7, 0.1, 0.1, 0.1]), np.array([0.1, 0.7, 0.1, 0.1]), np.array([0.25, 0.25, 0.25, 0.25]),
          np.array([0.05, 0.05, 0.1, 0.8])]
    q2 = np.array([0.25, 0.25, 0.25, 0.25])
    r = np.random.default_rng(3)
    n = 60000
    second = np.zeros((V, V))
    first = np.zeros(V)
    for s in range(n):
        k1 = r.choice(V, size=2, p=q1)
        tokens, parent = [0], [-1]
        for t in k1:
            tokens.append(int(t)); parent.append(0)
        for ci in (1, 2):                                  # each first-level child gets one child drawn from q2
            tokens.append(int(r.choice(V, p=q2))); parent.append(ci)
        tokens, parent = np.array(tokens, dtype=np.int32), np.array(parent, dtype=np.int32)
        logits = np.stack([np.log(p1)] + [np.log(p2[t]) for t in tokens[1:3]] + [np.log(q2)] * 2)
        dq = np.stack([q1, q2, q2, q2, q2])
        w = oracle.specinfer_walk(logits, dq, tokens, parent, 1.0, 1.0, seed=s, pos0=9)
        first[w["tokens"][0]] += 1
        if len(w["path"]) > 1:
            second[w["tokens"][0], w["tokens"][1]] += 1
    assert ((first - n * p1) ** 2 / (n * p1)).sum() < 21.1            # 3 dof
    for a in range(V):                                                 # given the first token was an accepted a
        na = second[a].sum()
        assert na > 2000
        assert ((second[a] - na * p2[a]) ** 2 / (na * p2[a])).sum() < 21.1, (a, second[a] / na)


def test_specinfer_special_cases():
    # draft == target: the first child is always accepted (ratio one), down a whole chain
    tokens, parent = np.array([3, 1, 4, 1], dtype=np.int32), np.array([-1, 0, 1, 2], dtype=np.int32)
    for s in range(50):
        w = oracle.specinfer_walk(_rows(4, np.log(_P6)), _rows(4, _P6), tokens, parent, 1.0, 1.0, seed=s, pos0=2)
        assert w["path"] == [0, 1, 2, 3] and w["tokens"][:3] == [1, 4, 1] and len(w["tokens"]) == 4
    # a child whose token the target gives no mass is never accepted; greedy target: only the argmax is
    p = np.array([0.0, 0.5, 0.5, 0.0, 0.0, 0.0])
    with np.errstate(divide="ignore"):
        lg = np.log(p)
    tokens, parent = _star_tree([0, 3, 2])
    for s in range(200):
        w = oracle.specinfer_walk(_rows(4, lg), _rows(4, _Q6), tokens, parent, 1.0, 1.0, seed=s, pos0=0)
        assert w["tokens"][0] in (1, 2) and (len(w["path"]) == 1 or w["path"][1] == 3)
        g = oracle.specinfer_walk(_rows(4, np.log(_P6)), _rows(4, _Q6), *_star_tree([0, 1, 3]), 0.0, 1.0, seed=s, pos0=0)
        assert g["tokens"][0] == 1 and g["path"][:2] == [0, 2]
    # uniforms: a new one for every trial of a position, none shared with the plain walk's
    us = {oracle.trial_uniform(5, 10, j) for j in range(8)} | {oracle.uniform01(5, 10)}
    assert len(us) == 9
