"""Oracle (test infrastructure): one draft-expansion step of Alg. 2, fp64 numpy.

Alg. 2, inner part of the loop: the draft forward gives a B x vocab matrix of next-token
probabilities for the nodes just expanded; ``selectBest`` keeps the best continuations by
CUMULATIVE probability, each scored  nll = -log p_prefix - log p_i  (App. A: maximising
the product of probabilities along a path = minimising the sum of -log p).  Here that is
written as the plain definition: log-softmax, full sort of each row, full sort of all
candidates.

Readings where the paper is silent: a per-row top-k prefilter precedes the global select
(lossless whenever no row holds more than k winners); ties go to the lower token id and,
globally, to the lower flat candidate index row*k + rank; candidate scores are rounded to
fp32 before the global ordering (the precision the library decides in); no temperature
is applied to draft logits.
"""
from __future__ import annotations

import numpy as np


def log_softmax(x):
    """x - (max + log sum exp(x - max)) along the last axis, in fp64."""
    x = np.asarray(x, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    return x - (m + np.log(np.exp(x - m).sum(axis=-1, keepdims=True)))


def row_topk(x, k):
    """Indices of the k largest entries of each row, ordered by (value descending, index
    ascending), from a full stable sort.  Returns int64 [N, k]."""
    x = np.asarray(x)
    order = np.argsort(-x, axis=-1, kind="stable")
    return order[..., :k]


def expand_topk(logits, cum_logp, k, B):
    """Returns dict(row, token, score: the first min(B, N*k) candidates in global order;
    topk_idx [N,k], topk_logp [N,k]; margins m_k (smallest gap between the k-th and
    (k+1)-th raw logit over rows) and m_B (gap between the B-th and (B+1)-th score))."""
    logits = np.asarray(logits)
    N, V = logits.shape
    logp = log_softmax(logits)
    idx = row_topk(logits, k)                              # selection on raw logits = on logp
    val = np.take_along_axis(logp, idx, axis=-1)
    score = (np.asarray(cum_logp, dtype=np.float64)[:, None] + val).astype(np.float32)
    flat = score.reshape(-1)
    order = np.argsort(-flat, kind="stable")               # score descending, flat index ascending
    n_out = min(B, N * k)
    sel = order[:n_out]
    if k < V:
        srt = -np.sort(-logits.astype(np.float64), axis=-1)
        m_k = float(np.min(srt[:, k - 1] - srt[:, k]))
    else:
        m_k = np.inf
    m_B = float(flat[order[n_out - 1]] - flat[order[n_out]]) if n_out < N * k else np.inf
    return dict(row=(sel // k).astype(np.int32), token=idx.reshape(-1)[sel].astype(np.int32),
                score=flat[sel], topk_idx=idx.astype(np.int32), topk_logp=val,
                m_k=m_k, m_B=m_B, threshold=float(flat[order[n_out - 1]]))
