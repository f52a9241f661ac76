#!/usr/bin/env python3
"""Writes tests/golden/bf16_noise_floor.json: how far the oracle's bf16-activation forward moves when its
inputs are nudged in the last bits -- the distance between two equally valid bf16 evaluations of one model.

Calls only oracle/ (the forward) and workloads/ (the seeded inputs); never the GPU library.  The GPU parity
tests at the benchmark sizes read the file: it tells them which nodes of the 80-layer configuration to
compare (several root-to-leaf paths spread over depth and node index, evaluated by the oracle as one
ancestor-closed sub-tree: by Alg. 1 a node's row depends on its own path only) and what error the oracle
shows against itself per layer, so that the kernel's error can be put beside it layer by layer.

Two oracle passes per configuration run side by side and share each layer's weights, which are generated
on the CPU one layer at a time.  Run time on 8 cores: C3 a few minutes, C5 about half an hour.

    python tests/golden/make_bf16_noise_floor.py [C3] [C5]
"""
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402
import workloads as wl  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "bf16_noise_floor.json")
PERTURB = 3e-6   # relative size of the nudge: what fp32 accumulation over K = 8192 terms differs from fp64 by
SEEDS = dict(weights=1, prefix=2, tree=3)     # the seeds the GPU tests use


def stats(d):
    d = np.abs(np.asarray(d, dtype=np.float64)).ravel()
    q = np.quantile(d, [0.5, 0.99, 0.9999])
    return dict(q50=float(q[0]), q99=float(q[1]), q9999=float(q[2]), max=float(d.max()),
                rms=float(np.sqrt(np.mean(d * d))), frac_within_2e_2=float((d <= 2e-2).mean()))


class SharedLayers:
    """w["layers"] for several oracle passes running side by side: layer l is generated once (on the CPU, a
    minute for a 70B-shaped layer) and handed to every pass that asks for it; two layers are kept."""

    def __init__(self, cfg, seed):
        self.cfg, self.seed = cfg, seed
        self.lock = threading.Lock()
        self.have = {}

    def __len__(self):
        return self.cfg.n_layers

    def __getitem__(self, l):
        with self.lock:
            if l not in self.have:
                t0 = time.time()
                self.have[l] = wl.gen_layer(self.cfg, self.seed, l)
                for old in [k for k in self.have if k < l - 1]:
                    del self.have[old]
                print(f"    layer {l + 1}/{self.cfg.n_layers} generated ({time.time() - t0:.0f}s)", flush=True)
            return self.have[l]


def two_passes(cfg, w, pk, pv, tok, par):
    """oracle.verify_tree with bf16 activations, plain and nudged, side by side."""
    res = {}

    def run(name, perturb):
        res[name] = oracle.verify_tree(cfg, w, pk, pv, tok, par, act_round="bf16", perturb=perturb)

    th = [threading.Thread(target=run, args=("a", 0.0)), threading.Thread(target=run, args=("b", PERTURB))]
    for t in th:
        t.start()
    for t in th:
        t.join()
    return res["a"], res["b"]


def model(name):
    c = wl.CONFIGS[name]
    cfg, P, T = c["cfg"], c["P"], c["T"]
    w = dict(wl.gen_model_ends(cfg, SEEDS["weights"]), layers=SharedLayers(cfg, SEEDS["weights"]))
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=SEEDS["prefix"])
    tok, par, _ = wl.gen_best_first_tree(T, c["k"], cfg.vocab, seed=SEEDS["tree"])
    return cfg, w, pk, pv, tok, par


def spread_leaves(par):
    """Leaves of >= 3 root-to-node paths spread over depth and over the node-index range (and so over the
    attention kernel's query tiles and the GEMMs' row tiles): the deepest node; the deepest node of the last
    quarter of the indices; a node of middling depth in the second quarter; the last node of depth <= 2."""
    depth = oracle.tree_depths(par)
    T = len(par)
    picks = [int(np.argmax(depth))]
    last_q = np.arange(3 * T // 4, T)
    picks.append(int(last_q[np.argmax(depth[last_q])]))
    second_q = np.arange(T // 4, T // 2)
    mid = int(np.median(depth))
    picks.append(int(second_q[np.argmin(np.abs(depth[second_q] - mid))]))
    shallow = np.nonzero(depth <= 2)[0]
    picks.append(int(shallow[-1]))
    return sorted(set(picks))


def subtree(par, leaves):
    """Sorted union of the paths to the leaves, and the parent array re-indexed to it."""
    nodes = sorted({a for leaf in leaves for a in oracle.ancestors(par, leaf)})
    pos = {n: i for i, n in enumerate(nodes)}
    sub_par = np.array([pos[int(par[n])] if par[n] >= 0 else -1 for n in nodes], dtype=np.int32)
    return np.array(nodes, dtype=np.int64), sub_par


def full_tensor(name):
    cfg, w, pk, pv, tok, par = model(name)
    a, b = two_passes(cfg, w, pk, pv, tok, par)
    return dict(perturb=PERTURB, seeds=SEEDS, logit_std=float(a["logits"].std()),
                logits=stats(b["logits"] - a["logits"]))


def sampled_paths(name):
    cfg, w, pk, pv, tok, par = model(name)
    leaves = spread_leaves(par)
    nodes, sub_par = subtree(par, leaves)
    depth = oracle.tree_depths(par)
    a, b = two_passes(cfg, w, pk, pv, tok[nodes], sub_par)
    per_layer = []
    for l in range(cfg.n_layers):
        dk, dv = b["tree_k"][l] - a["tree_k"][l], b["tree_v"][l] - a["tree_v"][l]
        per_layer.append(dict(k_max=float(np.abs(dk).max()), k_rms=float(np.sqrt(np.mean(dk * dk))),
                              v_max=float(np.abs(dv).max()), v_rms=float(np.sqrt(np.mean(dv * dv)))))
    return dict(perturb=PERTURB, seeds=SEEDS, leaves=leaves, leaf_depths=[int(depth[i]) for i in leaves],
                nodes=[int(n) for n in nodes], logit_std=float(a["logits"].std()),
                logits=stats(b["logits"] - a["logits"]), per_layer_kv=per_layer)


def main():
    which = sys.argv[1:] or ["C3", "C5"]
    out = json.load(open(OUT)) if os.path.exists(OUT) else {}
    for name in which:
        t0 = time.time()
        print(f"{name} ...", flush=True)
        out[name] = sampled_paths(name) if name == "C5" else full_tensor(name)
        print(f"{name}: logits floor {out[name]['logits']}  ({time.time() - t0:.0f}s)", flush=True)
        json.dump(out, open(OUT, "w"), indent=1)


if __name__ == "__main__":
    main()
