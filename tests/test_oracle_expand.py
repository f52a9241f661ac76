"""Pins for oracle/expand.py: library log-softmax, torch.topk, brute force over all N*V
continuations, and a hand-worked case."""
import json
import os

import numpy as np
import scipy.special
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_log_softmax_vs_scipy_and_invariants():
    x = np.random.default_rng(0).standard_normal((6, 301)) * 5
    lp = oracle.log_softmax(x)
    np.testing.assert_allclose(lp, scipy.special.log_softmax(x, axis=-1), atol=1e-13)
    np.testing.assert_allclose(np.exp(lp).sum(-1), 1.0, atol=1e-12)
    np.testing.assert_allclose(oracle.log_softmax(x + 1234.5), lp, atol=1e-9)
    assert np.all(lp <= 0)


def test_row_topk_vs_torch_and_python_sort():
    r = np.random.default_rng(1)
    x = r.standard_normal((9, 200)).astype(np.float32)
    x[:, 50:60] = x[:, 10:20]           # plant ties
    idx = oracle.row_topk(x, 16)
    tv = torch.topk(torch.from_numpy(x), 16, dim=-1).values.numpy()
    np.testing.assert_array_equal(np.take_along_axis(x, idx, -1), tv)
    for row in range(9):
        ref = sorted(range(200), key=lambda j: (-x[row, j], j))[:16]
        assert idx[row].tolist() == ref
    full = oracle.row_topk(x, 200)
    assert all(sorted(full[row].tolist()) == list(range(200)) for row in range(9))


def test_hand_case():
    g = json.load(open(os.path.join(GOLD, "expand_case.json")))
    out = oracle.expand_topk(np.log(np.array(g["probs"])), np.log(np.array(g["cum_prob"])), g["k"], g["B"])
    assert out["topk_idx"].tolist() == g["topk_idx"]
    for j, e in enumerate(g["expect"]):
        assert (out["row"][j], out["token"][j]) == (e["row"], e["token"])
        assert abs(out["score"][j] - np.log(e["prob"])) < 1e-6


def test_equals_brute_force_over_all_continuations_when_k_ge_B():
    r = np.random.default_rng(2)
    N, V, k, B = 7, 40, 8, 8
    x = (r.standard_normal((N, V)) * 3).astype(np.float32)
    cum = (-r.exponential(1.0, N) * r.integers(1, 6, N)).astype(np.float32)
    out = oracle.expand_topk(x, cum, k, B)
    # brute force: every one of the N*V continuations, scored with scipy's log-softmax
    lp = scipy.special.log_softmax(x.astype(np.float64), axis=-1)
    allc = sorted(((np.float32(cum[rw] + lp[rw, t]), rw, t) for rw in range(N) for t in range(V)),
                  key=lambda c: (-c[0], c[1], c[2]))[:B]
    assert [(c[1], c[2]) for c in allc] == list(zip(out["row"].tolist(), out["token"].tolist()))
    np.testing.assert_allclose(out["score"], [c[0] for c in allc], atol=1e-6)
    # a child is never likelier than its parent (App. A)
    assert np.all(out["score"] <= cum[out["row"]] + 1e-6)
    assert np.all(np.diff(out["score"]) <= 0)


def test_B_larger_than_candidates_returns_all_sorted():
    r = np.random.default_rng(3)
    x = r.standard_normal((3, 10)).astype(np.float32)
    out = oracle.expand_topk(x, np.zeros(3, np.float32), 4, 100)
    assert len(out["row"]) == 12 and np.all(np.diff(out["score"]) <= 0)


def test_global_tie_goes_to_lower_flat_index():
    x = np.zeros((2, 4), dtype=np.float32)      # everything ties
    out = oracle.expand_topk(x, np.zeros(2, np.float32), 2, 3)
    assert out["row"].tolist() == [0, 0, 1] and out["token"].tolist() == [0, 1, 0]


def test_minus_inf_logits_sort_last():
    x = np.array([[0.0, -np.inf, 1.0, -np.inf]], dtype=np.float32)
    out = oracle.expand_topk(x, np.zeros(1, np.float32), 4, 4)
    assert out["token"].tolist() == [2, 0, 1, 3]
    assert np.isneginf(out["score"][2:]).all()
