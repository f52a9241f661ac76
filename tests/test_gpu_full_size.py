"""GPU parity at the full benchmark sizes, on sampled outputs: the rows of whole root-to-leaf paths,
each recomputed by the oracle's plain causal forward over that path alone (Alg. 1: row i of the
tree forward is the target's next-token distribution after the path to node i)."""
import time

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import dev

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


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

    def __getitem__(self, l):
        if l % 10 == 9 and len(self.layers) > 10:
            self.say(f"    oracle: layer {l + 1}/{len(self.layers)}")   # a long run shows its steps
        return {k: v.cpu() for k, v in self.layers[l].items()}


def _run(sx, name, n_paths, with_floor, capsys):
    def say(msg):
        # progress lines reach the terminal even when pytest captures output: the 80-layer oracle pass takes two
        # minutes, and a run that prints nothing for that long looks hung to whoever watches it
        with capsys.disabled():
            print(msg, flush=True)

    c = wl.CONFIGS[name]
    cfg, P, T = c["cfg"], c["P"], c["T"]
    t0 = time.time()
    w = wl.gen_weights(cfg, seed=1, device=dev())
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=2, device=dev())
    tok, par, _ = wl.gen_best_first_tree(T, c["k"], cfg.vocab, seed=3)
    mw = sx.ModelWeights(cfg, w)
    logits, ws = sx.verify_tree(mw, pk, pv, torch.from_numpy(tok).to(dev()), torch.from_numpy(par).to(dev()))
    torch.cuda.synchronize()
    assert sx.check_status(ws) == 0
    say(f"\n[{name}] {cfg.n_layers} layers generated and verified on the GPU in {time.time() - t0:.1f}s")
    depth = oracle.tree_depths(par)
    leaves = np.argsort(-depth, kind="stable")[:n_paths]          # the deepest nodes: the longest paths
    wo = dict(embed=w["embed"].cpu(), final_norm=w["final_norm"].cpu(), lm_head=w["lm_head"].cpu(),
              layers=_LayersFromDevice(w["layers"], say))
    pkc, pvc = pk.cpu(), pv.cpu()
    worst, worst_floor, rows = 0.0, 0.0, 0
    for leaf in leaves:
        path = oracle.ancestors(par, int(leaf))
        t0 = time.time()
        ref = oracle.path_forward(cfg, wo, pkc, pvc, tok[path], act_round="bf16", return_all=True)
        got = logits[torch.as_tensor(path, device=dev())].cpu().double().numpy()
        err = float(np.abs(got - ref).max())
        worst, rows = max(worst, err), rows + len(path)
        msg = f"[{name}] path to node {leaf} ({len(path)} rows): max|gpu-oracle|={err:.3e}, logit std {ref.std():.2f}"
        if with_floor:
            ref2 = oracle.path_forward(cfg, wo, pkc, pvc, tok[path], act_round="bf16", return_all=True, perturb=3e-6)
            fl = float(np.abs(ref2 - ref).max())
            worst_floor = max(worst_floor, fl)
            msg += f", oracle self-noise floor {fl:.3e}"
        say(msg + f"  ({time.time() - t0:.0f}s)")
    return worst, worst_floor, rows


def test_c3_four_70b_layers_sampled_paths(sx, capsys):
    """1024-node tree, 1024 prefix tokens, 4 Llama-2-70B-shaped layers (GQA 64/8)."""
    err, floor, rows = _run(sx, "C3", n_paths=2, with_floor=True, capsys=capsys)
    assert rows >= 20
    assert err <= max(TOL_BF16, 2.0 * floor), (err, floor)


def test_c5_eighty_layer_model_sampled_path(sx, capsys):
    """The benchmark configuration: 2048-node tree, 2048 prefix tokens, all 80 layers (138 GB of
    weights resident).  One root-to-leaf path is re-evaluated by the oracle, streaming a layer at a
    time.  Measuring the oracle's self-noise floor here as well would double a two-minute test, so
    the bound is twice the floor measured once on this very path with the same knob (perturb 1e-7:
    max 0.345; 3e-6: max 0.451; the kernel itself: 0.326; a bf16-activation model against its own
    fp64-activation arithmetic: 0.79).  Indexing or masking mistakes produce errors of order 5."""
    err, _, rows = _run(sx, "C5", n_paths=1, with_floor=False, capsys=capsys)
    assert rows >= 10
    assert err <= 2 * 0.345, err
