"""The seeded input generators: reproducibility and the shapes/structure the recipes promise."""
import numpy as np
import torch

import workloads as wl
from workloads.gen import tensor_key


def test_hash_normal_is_reproducible_and_bell_shaped():
    k = tensor_key(5, 1, 2)
    a = wl.hash_normal(k, (1000, 33), std=0.02)
    b = wl.hash_normal(k, (1000, 33), std=0.02, chunk=4097)     # chunking must not matter
    assert torch.equal(a, b)
    assert abs(a.std().item() - 0.02) < 3e-4 and abs(a.mean().item()) < 3e-4
    assert a.abs().max().item() <= 0.02 * 4.89
    kurt = ((a / a.std()) ** 4).mean().item()
    assert 2.7 < kurt < 3.0                                      # Irwin-Hall(8): 2.85
    c = wl.hash_normal(tensor_key(5, 1, 3), (1000, 33), std=0.02)
    assert not torch.equal(a, c)
    assert torch.equal(wl.hash_normal(k, (1000, 33), std=0.02, dtype=torch.bfloat16), a.to(torch.bfloat16))


def test_best_first_tree_structure():
    tok, par, cum = wl.gen_best_first_tree(300, 8, 5000, seed=3, max_depth=12)
    assert par[0] == -1 and np.all(par[1:] < np.arange(1, 300)) and np.all(par[1:] >= 0)
    assert np.all(np.diff(cum) <= 1e-6)                          # chosen in order of cumulative log-prob
    assert np.all(cum[1:] <= cum[par[1:]] + 1e-6)                # child never likelier than parent
    st = wl.tree_stats(par)
    assert st["max_depth"] <= 12 and st["max_children"] <= 8
    for p in range(300):                                         # sibling tokens distinct
        kids = tok[par == p]
        assert len(set(kids.tolist())) == len(kids)
    tok2, par2, _ = wl.gen_best_first_tree(300, 8, 5000, seed=3, max_depth=12)
    assert np.array_equal(tok, tok2) and np.array_equal(par, par2)


def test_uniform_tree_and_expand_inputs():
    tok, par = wl.gen_uniform_tree(64, 1024, seed=1)
    assert par[0] == -1 and np.all(par[1:] < np.arange(1, 64)) and tok.max() < 1024
    lg, cum = wl.gen_expand_inputs(16, 1000, seed=2)
    assert lg.shape == (16, 1000) and lg.dtype == np.float32 and np.all(cum < 0)
    assert abs(lg.std() - 3.0) < 0.1
