"""Seeded generators for every synthetic input of the SpecExec verification hot path.

Two families:

* ``hash_normal`` -- a counter-based generator written with plain torch integer ops, so
  the same function yields bit-identical tensors on the CPU and on the GPU.  It is used
  for everything big (model weights, prefix KV): the 70B-shaped model is ~138 GB and is
  produced directly in HBM, while a CPU-side check can re-create any tensor (or pull the
  device copy back) and see the same bytes.  Element ``i`` of a tensor with key ``k`` is
  ``(sum of the 8 bytes of mix64(k + i*GOLDEN) - 1020) * std / 209.0239...``: an
  Irwin-Hall(8) variate, i.e. a bell-shaped approximation of N(0, std) with support
  +-4.88 std.  Only integer ops and one fp32 multiply are involved, so the result does
  not depend on any library's transcendental functions.
* numpy ``Philox`` streams for the small things (token ids, trees, draft logits).

The workloads these stand in for are the paper's Llama-2-7B/70B targets and draft trees
of 128-2048 tokens (Tables 1-3, Fig. 5); see the ``CONFIGS`` table below.
"""
from __future__ import annotations

import heapq
import math
from dataclasses import dataclass, replace

import numpy as np
import torch

# ----------------------------------------------------------------------------------
# model shapes
# ----------------------------------------------------------------------------------


@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "fp32"  # "fp32" | "bf16"

    def with_layers(self, n: int) -> "ModelCfg":
        return replace(self, n_layers=n)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16


CONFIGS = {
    # tiny fp32 decoder: full-tensor parity and every invariant
    "C1": dict(cfg=ModelCfg(2, 256, 4, 4, 64, 688, 1024, dtype="fp32"), P=128, T=64,
               temperature=0.6, top_p=0.9, k=4, B=16),
    # one Llama-2-7B-shaped layer, bf16
    "C2": dict(cfg=ModelCfg(1, 4096, 32, 32, 128, 11008, 32000, dtype="bf16"), P=512, T=256, k=8),
    # four Llama-2-70B-shaped layers (GQA 64/8), bf16
    "C3": dict(cfg=ModelCfg(4, 8192, 64, 8, 128, 28672, 32000, dtype="bf16"), P=1024, T=1024, k=16),
    # draft expansion step alone
    "C4": dict(N=2048, V=32000, k=32, B=2048, std=3.0, max_depth=32),
    # the full 80-layer 70B-shaped target, resident in HBM
    "C5": dict(cfg=ModelCfg(80, 8192, 64, 8, 128, 28672, 32000, dtype="bf16"), P=2048, T=2048, k=32,
               temperature=0.6, top_p=0.9),
}

# ----------------------------------------------------------------------------------
# counter-based bell-shaped generator (torch, device agnostic, bit-reproducible)
# ----------------------------------------------------------------------------------

_U64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    v &= _U64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)
_IH8_STD = math.sqrt(8.0 * (256.0 ** 2 - 1.0) / 12.0)  # std of a sum of 8 uniform bytes


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64_t(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _mix64_i(z: int) -> int:
    z &= _U64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _U64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _U64
    return z ^ (z >> 31)


def tensor_key(seed: int, *ids: int) -> int:
    """Derive a 64-bit stream key from a seed and a tuple of small integers."""
    k = _mix64_i(seed ^ 0xA5A5A5A5DEADBEEF)
    for i in ids:
        k = _mix64_i(k + 0x9E3779B97F4A7C15 * (int(i) + 1))
    return k


def hash_normal(key: int, shape, std: float = 1.0, mean: float = 0.0, dtype=torch.float32,
                device="cpu", chunk: int | None = None) -> torch.Tensor:
    """Bell-shaped (Irwin-Hall 8) pseudo-random tensor, identical on every device (and for every chunk size:
    the chunk only sets how much is computed at a time -- cache-sized pieces on a CPU, large ones on a GPU)."""
    n = int(np.prod(shape))
    if chunk is None:
        chunk = 1 << 18 if torch.device(device).type == "cpu" else 1 << 25
    out = torch.empty(n, dtype=dtype, device=device)
    scale = np.float32(std / _IH8_STD)
    k = _s64(key)
    m8 = 0x00FF00FF00FF00FF
    m16 = 0x0000FFFF0000FFFF
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        z = _mix64_t(idx * _GOLDEN + k)
        z = (z & m8) + (_lsr(z, 8) & m8)          # four 16-bit partial sums
        z = (z & m16) + (_lsr(z, 16) & m16)       # two 32-bit partial sums
        z = (z + _lsr(z, 32)) & 0xFFFF            # sum of the 8 bytes, 0..2040
        x = (z - 1020).to(torch.float32) * float(scale)
        if mean != 0.0:
            x = x + float(np.float32(mean))
        out[lo:hi] = x.to(dtype)
    return out.view(*shape)


# ----------------------------------------------------------------------------------
# weights / prefix KV
# ----------------------------------------------------------------------------------

_LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def layer_shapes(cfg: ModelCfg) -> dict:
    d, hq, hk, dh, f = cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn
    return dict(attn_norm=(d,), wq=(hq * dh, d), wk=(hk * dh, d), wv=(hk * dh, d), wo=(d, hq * dh),
                ffn_norm=(d,), w_gate=(f, d), w_up=(f, d), w_down=(d, f))


def gen_layer(cfg: ModelCfg, seed: int, layer: int, device="cpu") -> dict:
    """One decoder layer.  Linear weights are row-major [out, in] ~ N(0, 0.02); norm gains
    are 1 + N(0, 0.1) (not exactly one, so that a forgotten gain shows up in parity)."""
    out = {}
    for t, (name, shp) in enumerate(layer_shapes(cfg).items()):
        key = tensor_key(seed, 1, layer, t)
        if name.endswith("_norm"):
            out[name] = hash_normal(key, shp, std=0.1, mean=1.0, dtype=cfg.torch_dtype, device=device)
        else:
            out[name] = hash_normal(key, shp, std=0.02, dtype=cfg.torch_dtype, device=device)
    return out


def gen_model_ends(cfg: ModelCfg, seed: int, device="cpu") -> dict:
    """What a model holds besides its layers: embed [V,d], final_norm [d], lm_head [V,d] (untied)."""
    return dict(
        embed=hash_normal(tensor_key(seed, 0, 0), (cfg.vocab, cfg.d_model), std=0.02, dtype=cfg.torch_dtype, device=device),
        final_norm=hash_normal(tensor_key(seed, 0, 1), (cfg.d_model,), std=0.1, mean=1.0, dtype=cfg.torch_dtype,
                               device=device),
        lm_head=hash_normal(tensor_key(seed, 0, 2), (cfg.vocab, cfg.d_model), std=0.02, dtype=cfg.torch_dtype,
                            device=device))


def gen_weights(cfg: ModelCfg, seed: int, device="cpu", progress=None) -> dict:
    """Whole model: embed [V,d], layers[L], final_norm [d], lm_head [V,d] (untied)."""
    w = dict(cfg=cfg, layers=[])
    for l in range(cfg.n_layers):
        w["layers"].append(gen_layer(cfg, seed, l, device))
        if progress is not None:
            progress(l)
    w.update(gen_model_ends(cfg, seed, device))
    return w


def gen_prefix_kv(cfg: ModelCfg, P: int, seed: int, device="cpu"):
    """Synthetic prefix cache [L][P][Hkv][Dh] ~ N(0,1) in the model dtype.  K is taken to be
    already rotated at positions 0..P-1 (for the tiny config the tests instead build the
    cache with the oracle's own causal prefill)."""
    shp = (cfg.n_layers, P, cfg.n_kv_heads, cfg.head_dim)
    k = hash_normal(tensor_key(seed, 2, 0), shp, std=1.0, dtype=cfg.torch_dtype, device=device)
    v = hash_normal(tensor_key(seed, 2, 1), shp, std=1.0, dtype=cfg.torch_dtype, device=device)
    return k, v


# ----------------------------------------------------------------------------------
# tokens and trees (small: numpy Philox)
# ----------------------------------------------------------------------------------


def _rng(seed: int, *ids: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=tensor_key(seed, 7, *ids)))


def gen_tokens(n: int, vocab: int, seed: int) -> np.ndarray:
    return _rng(seed, 0).integers(0, vocab, size=n, dtype=np.int32)


def gen_uniform_tree(T: int, vocab: int, seed: int):
    """Tree of the tiny config: node 0 hangs off the last prefix token (parent -1), node i>0
    picks its parent uniformly among nodes 0..i-1, tokens are uniform over the vocabulary."""
    r = _rng(seed, 1)
    parent = np.full(T, -1, dtype=np.int32)
    for i in range(1, T):
        parent[i] = r.integers(0, i)
    tokens = r.integers(0, vocab, size=T, dtype=np.int32)
    return tokens, parent


def gen_chain_tree(T: int, vocab: int, seed: int):
    tokens = _rng(seed, 2).integers(0, vocab, size=T, dtype=np.int32)
    parent = np.arange(-1, T - 1, dtype=np.int32)
    return tokens, parent


def gen_best_first_tree(T: int, k: int, vocab: int, seed: int, max_depth: int = 32,
                        peaked: bool = True, std: float = 3.0):
    """Simulated best-first draft tree (stands in for the paper's draft-model search, Alg. 2).

    A fake draft model gives every expanded node a row of random logits (N(0,std); when
    ``peaked`` one random token is lifted so that it holds 30-95 % of the mass, like the
    sharp next-token distributions of Fig. 2).  Nodes are taken in order of cumulative
    log-probability (Dijkstra order), each contributing its k likeliest children to the
    frontier, until T nodes are chosen; nodes at ``max_depth`` are not expanded.  Nodes
    are numbered in the order chosen, so parent index < child index, the set is
    ancestor-closed (App. A) and sibling tokens are distinct.
    Returns (tokens i32[T], parent i32[T], cum_logp f32[T]).
    """
    root_tok = int(_rng(seed, 3).integers(0, vocab))
    tokens = np.zeros(T, dtype=np.int32)
    parent = np.full(T, -1, dtype=np.int32)
    cum = np.zeros(T, dtype=np.float64)
    depth = np.zeros(T, dtype=np.int32)
    heap = [(0.0, 0, -1, root_tok, 0)]  # (nll, tiebreak, parent, token, depth)
    serial = 1
    n = 0
    while n < T and heap:
        nll, _, par, tok, dep = heapq.heappop(heap)
        i = n
        n += 1
        tokens[i], parent[i], cum[i], depth[i] = tok, par, -nll, dep
        if dep >= max_depth:
            continue
        r = _rng(seed, 4, i)
        row = r.standard_normal(vocab) * std
        if peaked:
            j = int(r.integers(0, vocab))
            q = r.uniform(0.3, 0.95)
            row[j] = -np.inf
            m = row.max()
            rest = m + math.log(np.exp(row - m).sum())
            row[j] = rest + math.log(q / (1.0 - q))
        m = row.max()
        logp = row - (m + math.log(np.exp(row - m).sum()))
        top = np.argpartition(-logp, k - 1)[:k]
        for c in top:
            heapq.heappush(heap, (nll - float(logp[c]), serial, i, int(c), dep + 1))
            serial += 1
    if n < T:
        raise ValueError("tree generator ran out of frontier; raise k or max_depth")
    return tokens, parent, cum.astype(np.float32)


def tree_stats(parent: np.ndarray) -> dict:
    T = len(parent)
    depth = np.zeros(T, dtype=np.int64)
    for i in range(T):
        depth[i] = 0 if parent[i] < 0 else depth[parent[i]] + 1
    nchild = np.bincount(parent[parent >= 0], minlength=T)
    return dict(T=T, max_depth=int(depth.max()), mean_ancestors=float(depth.mean() + 1),
                leaves=int((nchild == 0).sum()), max_children=int(nchild.max()),
                depth_hist=np.bincount(depth).tolist())


# ----------------------------------------------------------------------------------
# draft-expansion inputs and crafted acceptance logits
# ----------------------------------------------------------------------------------


def gen_expand_inputs(N: int, V: int, seed: int, std: float = 3.0, max_depth: int = 32):
    """Draft logits fp32 [N,V] ~ N(0,std) and the expanded nodes' cumulative log-probs
    cum_logp[r] = -Exp(1) * depth_r with depth_r uniform in 1..max_depth."""
    r = _rng(seed, 5)
    logits = r.standard_normal((N, V), dtype=np.float32) * np.float32(std)
    depth = r.integers(1, max_depth + 1, size=N)
    cum = (-r.exponential(1.0, size=N) * depth).astype(np.float32)
    return logits, cum


def gen_crafted_logits(tokens: np.ndarray, parent: np.ndarray, V: int, seed: int,
                       boost: float = 8.0, sharp: bool = False) -> np.ndarray:
    """Target-logit stand-in that makes the acceptance walk traverse several tree levels on a
    random-init model: row i is N(0,1) noise plus ``boost`` on the token of one randomly
    chosen child of node i (leaves get pure noise).

    ``sharp`` mimics the peaked next-token distributions of trained LLMs (Fig. 2: the top 1-4
    tokens hold 90-98 % of the mass): the noise floor is pushed 12 units down and every row
    gets four more random tokens with logits uniform in [0, boost), so the nucleus holds a
    handful of well-separated tokens at every node, leaves included."""
    T = len(tokens)
    r = _rng(seed, 6)
    logits = r.standard_normal((T, V), dtype=np.float32)
    if sharp:
        logits -= np.float32(12.0)
        for i in range(T):
            alt = r.choice(V, size=min(4, V), replace=False)
            logits[i, alt] = r.uniform(0.0, boost, size=len(alt)).astype(np.float32)
    kids = [[] for _ in range(T)]
    for i in range(T):
        if parent[i] >= 0:
            kids[parent[i]].append(i)
    for i in range(T):
        if kids[i]:
            c = kids[i][int(r.integers(0, len(kids[i])))]
            logits[i, tokens[c]] = np.float32(boost) + (np.float32(0.0) if sharp else logits[i, tokens[c]])
    return logits


# ----------------------------------------------------------------------------------
# 4-bit group-quantised weights (storage only: random codes, scales and zero points)
# ----------------------------------------------------------------------------------


def gen_w4(N: int, K: int, group: int, seed: int):
    """Random quantised matrix: qweight uint32 [N][K/8] (eight 4-bit codes per word), scales bf16 [N][K/group]
    (0.002 .. 0.02), zeros uint8 [N][K/group] (0 .. 15).  numpy Philox; returns torch tensors on the CPU."""
    r = np.random.Generator(np.random.Philox(seed))
    qweight = r.integers(0, 2 ** 32, size=(N, K // 8), dtype=np.uint64).astype(np.uint32)
    scales = torch.from_numpy(r.uniform(0.002, 0.02, size=(N, K // group)).astype(np.float32)).to(torch.bfloat16)
    zeros = torch.from_numpy(r.integers(0, 16, size=(N, K // group), dtype=np.int64).astype(np.uint8))
    return torch.from_numpy(qweight.view(np.int32)), scales, zeros


def gen_w4_layers(cfg: ModelCfg, group: int, seed: int, device="cpu", scale: float = 0.3) -> list:
    """Random 4-bit decoder layers for a whole model, made on `device` with torch's generator (the 7B-shaped draft
    model holds 6.5 G codes: too many for the numpy stream of gen_w4 in reasonable time): per layer a dict name ->
    (qweight int32 [N][K/8], scales bf16 [N][K/group] in scale * (0.002 .. 0.02), zeros uint8 [N][K/group] in 0..15)."""
    g = torch.Generator(device=device).manual_seed(seed)
    shapes = layer_shapes(cfg)
    layers = []
    for _ in range(cfg.n_layers):
        lq = {}
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            N, K = shapes[name]
            qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (N, K // 8), dtype=torch.int32, device=device, generator=g)
            sc = ((torch.rand((N, K // group), device=device, generator=g) * 0.018 + 0.002) * scale).to(torch.bfloat16)
            zr = torch.randint(0, 16, (N, K // group), dtype=torch.uint8, device=device, generator=g)
            lq[name] = (qw, sc, zr)
        layers.append(lq)
    return layers
