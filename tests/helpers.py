"""Shared helpers for the GPU parity tests: moving seeded inputs to the device and handing the
very same values to the oracle."""
import numpy as np
import torch


def dev():
    return torch.device("cuda:0")


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)) if isinstance(a, np.ndarray) else a
    if dtype is not None:
        t = t.to(dtype)
    return t.to(dev()).contiguous()


def weights_to(w, device):
    out = dict(cfg=w["cfg"], embed=w["embed"].to(device), final_norm=w["final_norm"].to(device),
               lm_head=w["lm_head"].to(device), layers=[{k: v.to(device) for k, v in lw.items()} for lw in w["layers"]])
    return out


def weights_np(w):
    f = lambda t: t.detach().cpu().double().numpy()
    return dict(embed=f(w["embed"]), final_norm=f(w["final_norm"]), lm_head=f(w["lm_head"]),
                layers=[{k: f(v) for k, v in lw.items()} for lw in w["layers"]])


def bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (numpy, elementwise)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)
