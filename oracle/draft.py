"""Oracle (test infrastructure): Alg. 2, PARALLEL SSSP FOR DRAFTING -- createDraftTree -- with an
ordinary binary heap, one forward per batch by the tree oracle, nothing cached.

Reading of the listing (stated once here, the HIP path follows the same one):
  * the heap H holds candidate tokens (token, parent node, nll = -cumulative log-probability); the root x
    enters with nll 0;
  * one iteration pops up to B candidates in ascending nll; a popped candidate joins the tree only if
    its nll is below the threshold T (candidates at or above it are dropped: nothing later in the heap
    can be below it either, so the rest of the batch is empty);
  * once the tree holds at least K nodes, T = the K-th smallest nll in the tree;
  * the draft model scores the batch (each node sees the prefix and its tree ancestors), `selectBest`
    keeps, per node, its k most probable next tokens and, of those, the min(K, batch * k) best by
    cumulative log-probability; they enter the heap, which is then cut to its K best;
  * after D iterations (or when a batch comes up empty) the tree is cut to its K best nodes.
Node order of the result: order of insertion (iteration by iteration, ascending nll inside an iteration;
equal nll: the candidate that entered the heap first), which keeps parents before children.
"""
from __future__ import annotations

import heapq

import numpy as np

from .expand import expand_topk
from .model import verify_tree


def create_draft_tree(cfg, w, prefix_k, prefix_v, root_token, K, D, B, k, act_round=None):
    """Returns dict(tokens, parent, cum_logp (fp32, as the candidates' scores are), iterations).
    act_round="bf16" evaluates the draft model as a bf16 model (see model.verify_tree)."""
    tokens, parent, cum = [], [], []
    heap = [(0.0, 0, int(root_token), -1)]          # (nll, entry number, token, parent node)
    entered = 1
    T = np.inf
    iterations = 0
    for _ in range(D):
        batch = []
        for _ in range(B):
            if not heap:
                break
            nll, _, tok, par = heapq.heappop(heap)
            if nll < T:
                tokens.append(tok)
                parent.append(par)
                cum.append(np.float32(-nll))
                batch.append(len(tokens) - 1)
        if not batch:
            break
        iterations += 1
        if len(tokens) >= K:
            T = float(np.sort(-np.asarray(cum, dtype=np.float64))[K - 1])
        # the whole tree goes through the oracle's forward; only the batch's rows are used
        logits = verify_tree(cfg, w, prefix_k, prefix_v, np.asarray(tokens), np.asarray(parent),
                             act_round=act_round)["logits"]
        sel = expand_topk(logits[batch].astype(np.float32), np.asarray([cum[i] for i in batch], dtype=np.float32),
                          min(k, cfg.vocab), min(K, len(batch) * min(k, cfg.vocab)))
        for row, tok, score in zip(sel["row"], sel["token"], sel["score"]):
            heapq.heappush(heap, (-float(score), entered, int(tok), batch[int(row)]))
            entered += 1
        if len(heap) > K:
            heap = heapq.nsmallest(K, heap)
            heapq.heapify(heap)
    # trim(tau, K): the K best nodes, in insertion order, parents renumbered
    order = sorted(range(len(tokens)), key=lambda i: (-float(cum[i]), i))[:K]
    keep = sorted(order)
    new_index = {old: new for new, old in enumerate(keep)}
    return dict(tokens=np.asarray([tokens[i] for i in keep], dtype=np.int32),
                parent=np.asarray([new_index[parent[i]] if parent[i] >= 0 else -1 for i in keep], dtype=np.int32),
                cum_logp=np.asarray([cum[i] for i in keep], dtype=np.float32), iterations=iterations)
