"""Oracle (test infrastructure): the target model's forward over a token tree, fp64 numpy.

What the paper fixes (Alg. 1, function PRECOMPUTE): one forward of the target model over
the K tree tokens returns a K x vocab matrix whose row i is the next-token distribution
after the sequence "path to node i, then node i".  App. D: the tree tokens are processed
in parallel under a merged attention mask, i.e. every tree token sees the cached prefix
and its own ancestors only.  The decoder itself is the standard pre-norm Llama block
(RMSNorm, rotary positions, grouped-query attention, SwiGLU), which the paper takes from
its model library; conventions the paper leaves open are listed beside each function.

Two independent formulations are given so that each pins the other:
  * ``verify_tree``  -- node-by-node attention over explicit ancestor lists;
  * ``path_forward`` -- an ordinary causal forward over one root-to-node token sequence,
                        dense lower-triangular mask, no notion of a tree at all.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(x):
    if hasattr(x, "detach"):  # torch tensor (possibly bf16)
        x = x.detach().to("cpu").double().numpy()
    return np.asarray(x, dtype=F64)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even) by way of fp32, as hardware that holds an
    fp32 value and stores a bf16 one does.  Used only when a bf16 model is evaluated with
    ``act_round='bf16'``: it marks the tensors such a model materialises in bf16."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).astype(F64)


def _rounder(act_round):
    if act_round is None:
        return lambda a: a
    if act_round == "bf16":
        return round_bf16
    raise ValueError(act_round)


# ------------------------------------------------------------------------------------
# tree bookkeeping (pi(x_i, tau): the path from the root to a node; Alg. 1, App. A)
# ------------------------------------------------------------------------------------


def tree_depths(parent) -> np.ndarray:
    """depth[i] = number of tree ancestors of node i; a parent of -1 means the node hangs
    directly off the last cached prefix token.  Requires parent[i] < i."""
    parent = np.asarray(parent)
    depth = np.zeros(len(parent), dtype=np.int64)
    for i, p in enumerate(parent):
        if p >= i or p < -1:
            raise ValueError(f"node {i}: parent {p} breaks the topological order")
        depth[i] = 0 if p < 0 else depth[p] + 1
    return depth


def ancestors(parent, i: int) -> list:
    """Indices on the path root -> ... -> i, inclusive, in root-first order."""
    out = []
    while i >= 0:
        out.append(int(i))
        i = int(parent[i])
    return out[::-1]


# ------------------------------------------------------------------------------------
# decoder pieces
# ------------------------------------------------------------------------------------


def rmsnorm(x, g, eps):
    """x * rsqrt(mean(x^2) + eps) * g over the last axis."""
    x = _f64(x)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * _f64(g)


def rope(x, pos, base):
    """Rotary embedding, half-split pairing: element i is paired with element i + Dh/2 and the
    pair is rotated by the angle pos * base**(-2i/Dh).  x: [n, H, Dh], pos: [n]."""
    x = _f64(x)
    n, H, Dh = x.shape
    half = Dh // 2
    inv = F64(base) ** (-np.arange(half, dtype=F64) * 2.0 / Dh)
    ang = np.asarray(pos, dtype=F64)[:, None] * inv[None, :]          # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def _silu(x):
    return x / (1.0 + np.exp(-x))


def tree_attention(q, k_tree, v_tree, k_prefix, v_prefix, parent):
    """Attention of every tree node over (all prefix keys) + (its ancestors and itself).

    q: [T,Hq,Dh]; k_tree, v_tree: [T,Hkv,Dh]; k_prefix, v_prefix: [P,Hkv,Dh].
    Query head h reads KV head h // (Hq/Hkv); scores are scaled by 1/sqrt(Dh).
    Returns [T, Hq, Dh]."""
    q, k_tree, v_tree = _f64(q), _f64(k_tree), _f64(v_tree)
    k_prefix, v_prefix = _f64(k_prefix), _f64(v_prefix)
    T, Hq, Dh = q.shape
    Hkv = k_tree.shape[1]
    G = Hq // Hkv
    out = np.zeros((T, Hq, Dh), dtype=F64)
    for i in range(T):
        anc = ancestors(parent, i)
        K = np.concatenate([k_prefix, k_tree[anc]], axis=0)          # [n, Hkv, Dh]
        V = np.concatenate([v_prefix, v_tree[anc]], axis=0)
        for h in range(Hq):
            kv = h // G
            s = K[:, kv, :] @ q[i, h] / np.sqrt(F64(Dh))
            p = np.exp(s - s.max())
            p /= p.sum()
            out[i, h] = p @ V[:, kv, :]
    return out


def verify_tree(cfg, w, prefix_k, prefix_v, tokens, parent, act_round=None, perturb=0.0):
    """FORWARD(tau, theta_target) of Alg. 1: logits [T, vocab], row i = distribution of the
    token that follows node i.  Also returns the tree's own K/V per layer.

    cfg: object with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
    rope_base, rms_eps.  w: dict(embed, layers[list of dict], final_norm, lm_head), linear
    weights row-major [out, in] (y = x W^T), no biases.  prefix_k/v: [L, P, Hkv, Dh], K
    already rotated at positions 0..P-1.  Node i sits at position P + depth(i).

    ``perturb`` (default 0) multiplies the embedded inputs by 1 + perturb * N(0,1): a knob for
    measuring how far two equally valid bf16 evaluations of the same model drift apart when
    their arithmetic differs in the last bits (the rounding-flip noise floor)."""
    R = _rounder(act_round)
    tokens = np.asarray(tokens)
    parent = np.asarray(parent)
    T = len(tokens)
    Hq, Hkv, Dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    prefix_k, prefix_v = _f64(prefix_k), _f64(prefix_v)
    P = prefix_k.shape[1]
    pos = P + tree_depths(parent)
    h = _f64(w["embed"])[tokens]                                      # [T, d]
    if perturb:
        h = h * (1.0 + perturb * np.random.default_rng(0).standard_normal(h.shape))
    tk, tv = [], []
    for l in range(cfg.n_layers):
        lw = w["layers"][l]
        x = R(rmsnorm(h, lw["attn_norm"], cfg.rms_eps))
        q = (x @ _f64(lw["wq"]).T).reshape(T, Hq, Dh)
        k = (x @ _f64(lw["wk"]).T).reshape(T, Hkv, Dh)
        v = (x @ _f64(lw["wv"]).T).reshape(T, Hkv, Dh)
        q, k, v = R(rope(q, pos, cfg.rope_base)), R(rope(k, pos, cfg.rope_base)), R(v)
        tk.append(k)
        tv.append(v)
        o = R(tree_attention(q, k, v, prefix_k[l], prefix_v[l], parent)).reshape(T, Hq * Dh)
        h = h + o @ _f64(lw["wo"]).T
        x = R(rmsnorm(h, lw["ffn_norm"], cfg.rms_eps))
        a = R(_silu(x @ _f64(lw["w_gate"]).T) * (x @ _f64(lw["w_up"]).T))
        h = h + a @ _f64(lw["w_down"]).T
    x = R(rmsnorm(h, w["final_norm"], cfg.rms_eps))
    logits = x @ _f64(w["lm_head"]).T
    return dict(logits=logits, tree_k=np.stack(tk), tree_v=np.stack(tv), hidden=h)


def path_forward(cfg, w, prefix_k, prefix_v, seq_tokens, act_round=None, return_all=False,
                 return_kv=False, perturb=0.0):
    """Ordinary causal decoding of ``seq_tokens`` placed after a cached prefix: token s sits at
    position P + s and attends to the whole prefix and to tokens 0..s of the sequence.
    Returns the logits after the last token (or after every token with ``return_all``).
    With an empty prefix (P = 0) and ``return_kv`` this doubles as the causal prefill that
    produces a prefix cache."""
    R = _rounder(act_round)
    seq = np.asarray(seq_tokens)
    n = len(seq)
    Hq, Hkv, Dh = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = Hq // Hkv
    if prefix_k is None:
        prefix_k = np.zeros((cfg.n_layers, 0, Hkv, Dh))
        prefix_v = np.zeros((cfg.n_layers, 0, Hkv, Dh))
    P = prefix_k.shape[1]                     # prefix_k/v may be any [L][P][Hkv][Dh] indexable (converted per layer)
    pos = P + np.arange(n)
    # dense mask over [prefix | sequence]: everything in the prefix, lower triangle after it
    allowed = np.concatenate([np.ones((n, P), dtype=bool), np.tril(np.ones((n, n), dtype=bool))], axis=1)
    h = _f64(w["embed"])[seq]
    if perturb:  # same knob as in verify_tree: a nudge of the inputs, to measure rounding-flip noise
        h = h * (1.0 + perturb * np.random.default_rng(0).standard_normal(h.shape))
    ks, vs = [], []
    for l in range(cfg.n_layers):
        lw = w["layers"][l]
        x = R(rmsnorm(h, lw["attn_norm"], cfg.rms_eps))
        q = R(rope((x @ _f64(lw["wq"]).T).reshape(n, Hq, Dh), pos, cfg.rope_base))
        k = R(rope((x @ _f64(lw["wk"]).T).reshape(n, Hkv, Dh), pos, cfg.rope_base))
        v = R((x @ _f64(lw["wv"]).T).reshape(n, Hkv, Dh))
        ks.append(k)
        vs.append(v)
        K = np.concatenate([_f64(prefix_k[l]), k], axis=0)            # [P+n, Hkv, Dh]
        V = np.concatenate([_f64(prefix_v[l]), v], axis=0)
        Kh = np.repeat(K, G, axis=1)                                  # [P+n, Hq, Dh]
        Vh = np.repeat(V, G, axis=1)
        s = np.einsum("ihd,jhd->hij", q, Kh) / np.sqrt(F64(Dh))       # [Hq, n, P+n]
        s = np.where(allowed[None], s, -np.inf)
        p = np.exp(s - s.max(axis=-1, keepdims=True))
        p = p / p.sum(axis=-1, keepdims=True)
        o = R(np.einsum("hij,jhd->ihd", p, Vh)).reshape(n, Hq * Dh)
        h = h + o @ _f64(lw["wo"]).T
        x = R(rmsnorm(h, lw["ffn_norm"], cfg.rms_eps))
        a = R(_silu(x @ _f64(lw["w_gate"]).T) * (x @ _f64(lw["w_up"]).T))
        h = h + a @ _f64(lw["w_down"]).T
    x = R(rmsnorm(h, w["final_norm"], cfg.rms_eps))
    if not return_all:
        x = x[-1:]
    logits = x @ _f64(w["lm_head"]).T
    logits = logits if return_all else logits[0]
    if return_kv:
        return logits, np.stack(ks), np.stack(vs)
    return logits
