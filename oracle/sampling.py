"""Oracle (test infrastructure): the acceptance walk of Alg. 1 and plain sequential sampling.

Alg. 1, main loop: generation is ordinary sequential sampling from the target model; the
tree only serves as a cache of target distributions.  While the sequence sampled so far
is a path of the tree, the next distribution is read from the cache (row of that node);
the walk ends at the first sampled token that no child of the current node carries.
Sect. 4.1 (Correctness): for any RNG seed the result equals sequential sampling with the
same seed -- ``sequential_sample`` below is that reference, with no tree anywhere.

Conventions the paper leaves open (they are this build's readings):
  * sampling warp: temperature first, then nucleus (top-p); the nucleus is the shortest
    prefix of tokens ordered by (probability descending, id ascending) whose mass reaches
    top_p, the token that crosses the threshold included (Sect. 5.1 quotes t=0.6, p=0.9);
  * draw: inverse CDF over the nucleus in token-id order at u * mass(nucleus), taking the
    first token whose running mass exceeds that target;
  * t == 0 is greedy: the lowest-id argmax;
  * RNG: one uniform per generated position, u = top 24 bits of a 64-bit mix of
    (seed, absolute position), so it does not depend on how the tree was built.
"""
from __future__ import annotations

import numpy as np

from .model import path_forward, tree_depths

_U64 = (1 << 64) - 1


def uniform01(seed: int, position: int) -> float:
    """u in [0,1) with 24 bits: SplitMix64's output function applied to
    seed + (position+1) * 0x9E3779B97F4A7C15, top 24 bits scaled by 2**-24."""
    z = (int(seed) + (int(position) + 1) * 0x9E3779B97F4A7C15) & _U64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _U64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _U64
    z = z ^ (z >> 31)
    return (z >> 40) * 2.0 ** -24


def sample_token(logits, temperature: float, top_p: float, u: float):
    """One draw from warp_{t,top_p}(softmax(logits)).  Returns (token, margins) where margins
    tells how far the decision was from flipping: 'm_p' (nucleus mass vs top_p at the
    boundary, in probability units), 'm_u' (distance of the draw to the nearest CDF edge),
    'm_top' (gap between the two largest logits; greedy only)."""
    x = np.asarray(logits, dtype=np.float64)
    V = len(x)
    if temperature == 0.0:
        tok = int(np.argmax(x))                       # first maximum = lowest id
        srt = np.sort(x)
        return tok, dict(m_top=float(srt[-1] - srt[-2]) if V > 1 else np.inf, m_p=np.inf, m_u=np.inf)
    z = x / temperature
    p = np.exp(z - z.max())
    p /= p.sum()
    order = np.argsort(-p, kind="stable")             # probability descending, id ascending
    csum = np.cumsum(p[order])
    n_keep = int(np.searchsorted(csum, top_p, side="left")) + 1   # first prefix with mass >= top_p
    n_keep = min(n_keep, V)
    keep = np.zeros(V, dtype=bool)
    keep[order[:n_keep]] = True
    mass = float(p[keep].sum())
    target = u * mass
    cdf = np.cumsum(np.where(keep, p, 0.0))           # token-id order
    hit = np.nonzero(keep & (cdf > target))[0]
    tok = int(hit[0]) if len(hit) else int(np.nonzero(keep)[0][-1])
    before = csum[n_keep - 2] if n_keep >= 2 else 0.0
    m_p = min(abs(csum[n_keep - 1] - top_p), abs(top_p - before)) if top_p < 1.0 else np.inf
    edges = cdf[keep]
    m_u = float(np.min(np.abs(edges - target)))
    if n_keep < V:  # also: a tie between the last kept and first dropped probability
        m_p = min(m_p, np.inf if p[order[n_keep - 1]] > p[order[n_keep]] else 0.0)
    return tok, dict(m_p=float(m_p), m_u=m_u, m_top=np.inf)


def accept_walk(logits, tokens, parent, temperature, top_p, seed, pos0):
    """Walk the cached tree (Alg. 1, loop body): start at node 0 (the first not-yet-verified
    token, at absolute position pos0), sample the next token from the current node's row,
    move to the lowest-index child carrying that token, stop when there is none.

    Returns dict(path=[node ids, starting with 0], tokens=[every sampled token; the last one
    is the token that left the tree, or extended past a leaf], margins=[per step])."""
    tokens = np.asarray(tokens)
    parent = np.asarray(parent)
    depth = tree_depths(parent)
    if parent[0] != -1:
        raise ValueError("node 0 must be the root")
    cur, path, out, margins = 0, [0], [], []
    while True:
        u = uniform01(seed, pos0 + int(depth[cur]) + 1)
        x, m = sample_token(logits[cur], temperature, top_p, u)
        out.append(x)
        margins.append(m)
        kids = np.nonzero((parent == cur) & (tokens == x))[0]
        if len(kids) == 0:
            break
        cur = int(kids[0])
        path.append(cur)
    return dict(path=path, tokens=out, margins=margins)


def sequential_sample(cfg, w, prefix_k, prefix_v, first_token, n_tokens, temperature, top_p,
                      seed, pos0):
    """Token-by-token sampling from the target model with no tree: the sequence starts as
    [first_token] at position pos0 and every new token re-runs a causal forward."""
    seq, out = [int(first_token)], []
    for _ in range(n_tokens):
        lg = path_forward(cfg, w, prefix_k, prefix_v, seq)
        x, _ = sample_token(lg, temperature, top_p, uniform01(seed, pos0 + len(seq)))
        out.append(x)
        seq.append(x)
    return out


# ------------------------------------------------------------------------------------------
# The comparison system of Sect. 4.1 ("Comparison to speculative decoding"): acceptance with
# probability P_target / P_draft instead of P_target.
# ------------------------------------------------------------------------------------------


def warped_distribution(logits, temperature: float, top_p: float) -> np.ndarray:
    """The distribution ``sample_token`` draws from, written out: softmax(logits / t) cut to its
    nucleus and renormalised (t == 0: all mass on the lowest-id argmax)."""
    x = np.asarray(logits, dtype=np.float64)
    V = len(x)
    p = np.zeros(V)
    if temperature == 0.0:
        p[int(np.argmax(x))] = 1.0
        return p
    z = x / temperature
    e = np.exp(z - z.max())
    e /= e.sum()
    order = np.argsort(-e, kind="stable")
    csum = np.cumsum(e[order])
    n_keep = min(int(np.searchsorted(csum, top_p, side="left")) + 1, V)
    p[order[:n_keep]] = e[order[:n_keep]]
    return p / p.sum()


def trial_uniform(seed: int, position: int, trial: int) -> float:
    """The uniform of the ``trial``-th decision taken at one position (this mode needs several per
    position): ``uniform01`` with the seed advanced by (trial + 1) * 0xD6E8FEB86659FD93 (mod 2^64)."""
    return uniform01((int(seed) + (int(trial) + 1) * 0xD6E8FEB86659FD93) & _U64, position)


def specinfer_walk(logits, draft_probs, tokens, parent, temperature, top_p, seed, pos0):
    """Tree acceptance the way speculative decoding does it (Sect. 4.1: a drafted token x is accepted
    with probability P_target(x) / P_draft(x), capped at one), for a tree whose children were *sampled*
    from the draft distribution -- the baseline the paper compares with, multi-step speculative sampling
    over a token tree.

    At the current node, p is the warped target distribution of its row and q = draft_probs[cur] the
    distribution its children were drawn from (independently; equal tokens may appear as separate
    children).  The children are tried in index order: child c with token x is accepted when
    r * q[x] < p[x], r = trial_uniform(seed, position, j) for the j-th child; the walk then moves to c.
    A rejection replaces p by the renormalised positive part of p - q (the part of the target's mass
    the draft did not cover) and goes on to the next child.  When every child is rejected (or there is
    none) the token is drawn from what p has become -- inverse CDF in id order at r * sum(p), r the
    next uniform of the position -- and the walk ends.  The emitted tokens then follow the target's
    warped distribution exactly, although no step samples from it directly.

    Returns dict(path, tokens, margins): as ``accept_walk``; margins[i] = how far each decision taken at
    step i was from flipping ('m_acc': min |r q[x] - p[x]| over the trials, 'm_u': distance of the
    final draw to the nearest CDF edge, inf when the step ended in an acceptance)."""
    tokens = np.asarray(tokens)
    parent = np.asarray(parent)
    depth = tree_depths(parent)
    if parent[0] != -1:
        raise ValueError("node 0 must be the root")
    cur, path, out, margins = 0, [0], [], []
    while True:
        pos = pos0 + int(depth[cur]) + 1
        p = warped_distribution(logits[cur], temperature, top_p)
        q = np.asarray(draft_probs[cur], dtype=np.float64)
        kids = np.nonzero(parent == cur)[0]
        m_acc, nxt = np.inf, None
        for j, c in enumerate(kids):
            x = int(tokens[c])
            r = trial_uniform(seed, pos, j)
            m_acc = min(m_acc, abs(r * q[x] - p[x]))
            if r * q[x] < p[x]:
                nxt = int(c)
                break
            rest = np.maximum(p - q, 0.0)
            if rest.sum() > 0.0:          # (zero only when p <= q everywhere, i.e. p == q: then x was accepted)
                p = rest / rest.sum()
        if nxt is not None:
            out.append(int(tokens[nxt]))
            margins.append(dict(m_acc=float(m_acc), m_u=np.inf))
            cur = nxt
            path.append(cur)
            continue
        target = trial_uniform(seed, pos, len(kids)) * p.sum()
        cdf = np.cumsum(p)
        hit = np.nonzero((p > 0) & (cdf > target))[0]
        x = int(hit[0]) if len(hit) else int(np.nonzero(p > 0)[0][-1])
        out.append(x)
        margins.append(dict(m_acc=float(m_acc), m_u=float(np.min(np.abs(cdf[p > 0] - target)))))
        return dict(path=path, tokens=out, margins=margins)
