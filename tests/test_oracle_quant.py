"""Pins for oracle/quant.py: a hand-worked fixture (nibble order, zero point, groups), the identity case, and
bf16 rounding of the dequantised weight against torch's conversion."""
import json
import os

import numpy as np
import torch

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_case():
    g = json.load(open(os.path.join(GOLD, "w4_case.json")))
    qw = np.array([[int(h, 16) for h in row] for row in g["qweight_hex"]], dtype=np.uint32)
    W = oracle.dequantize_w4(qw, np.array(g["scales"]), np.array(g["zeros"]), g["group"])
    assert W.tolist() == g["W"]
    X = np.eye(16)
    assert np.array_equal(oracle.gemm_w4a16(X, qw, np.array(g["scales"]), np.array(g["zeros"]), g["group"]), np.array(g["W"]).T)


def test_identity_scale_and_zero_return_the_codes():
    r = np.random.default_rng(0)
    codes = r.integers(0, 16, size=(5, 64), dtype=np.uint8)
    qw = np.zeros((5, 8), dtype=np.uint32)
    for k in range(64):                                              # packed by the definition, one code at a time
        qw[:, k // 8] |= codes[:, k].astype(np.uint32) << np.uint32(4 * (k % 8))
    assert np.array_equal(oracle.unpack_w4(qw), codes)
    W = oracle.dequantize_w4(qw, np.ones((5, 2)), np.zeros((5, 2)), 32)
    assert np.array_equal(W, codes.astype(np.float64))


def test_dequantised_weights_are_bf16_values_rounded_like_torch():
    r = np.random.default_rng(1)
    qw = r.integers(0, 2 ** 32, size=(7, 16), dtype=np.uint64).astype(np.uint32)
    s = torch.tensor(r.uniform(0.001, 0.05, size=(7, 4)), dtype=torch.float32).to(torch.bfloat16)
    z = r.integers(0, 16, size=(7, 4))
    W = oracle.dequantize_w4(qw, s.double().numpy(), z, 32)
    q = torch.from_numpy(oracle.unpack_w4(qw).astype(np.float32))
    ref = (s.float().repeat_interleave(32, dim=1) * (q - torch.from_numpy(np.repeat(z, 32, axis=1)).float())).to(torch.bfloat16)
    assert np.array_equal(W, ref.double().numpy())
