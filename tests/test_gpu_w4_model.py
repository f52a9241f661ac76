"""GPU parity of the forward with 4-bit decoder layers (Sect. 5: the paper's fastest setting runs its models quantised
to 4 bits) against the oracle evaluating the same model: the oracle dequantises every matrix by the stated formula
(oracle.dequantize_w4: w = bf16(scale * (code - zero))) and runs its ordinary bf16-activation forward on the result."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import dev, to_dev

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
GROUP = 128
W4_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


@pytest.fixture(scope="module")
def sx():
    import paper_2406_02532_amd as m
    return m


def _w4_model(cfg, seed):
    """bf16 embed / norms / lm_head from the usual generator, the seven matrices of every layer as random 4-bit codes
    with scales that give weights of the usual size (std ~ 0.02).  Returns (weights for the binding on the CPU,
    oracle weights: the same model with every matrix dequantised)."""
    w = wl.gen_weights(cfg, seed=seed)
    from workloads.gen import layer_shapes
    shapes = layer_shapes(cfg)
    layers_w4, layers_ref, layers_norm = [], [], []
    for l in range(cfg.n_layers):
        q4, ref = {}, {}
        for t, name in enumerate(W4_NAMES):
            N, K = shapes[name]
            qw, sc, zr = wl.gen_w4(N, K, GROUP, seed=1000 * seed + 10 * l + t)
            sc = (sc.float() * 0.3).to(torch.bfloat16)
            q4[name] = (qw, sc, zr)
            ref[name] = oracle.dequantize_w4(qw.numpy().view(np.uint32), sc.double().numpy(), zr.numpy(), GROUP)
        for name in ("attn_norm", "ffn_norm"):
            ref[name] = w["layers"][l][name]
        layers_w4.append(q4)
        layers_ref.append(ref)
        layers_norm.append({n: w["layers"][l][n] for n in ("attn_norm", "ffn_norm")})
    gpu = dict(cfg=cfg, embed=w["embed"], final_norm=w["final_norm"], lm_head=w["lm_head"], layers=layers_norm,
               layers_w4=layers_w4, w4_group=GROUP)
    ref = dict(embed=w["embed"], final_norm=w["final_norm"], lm_head=w["lm_head"], layers=layers_ref)
    return gpu, ref


def _to_device(gpu):
    out = dict(gpu)
    for k in ("embed", "final_norm", "lm_head"):
        out[k] = gpu[k].to(dev())
    out["layers"] = [{n: t.to(dev()) for n, t in lw.items()} for lw in gpu["layers"]]
    out["layers_w4"] = [{n: tuple(t.to(dev()) for t in m) for n, m in lq.items()} for lq in gpu["layers_w4"]]
    return out


def _bf16_twin(gpu, ref):
    """The same model as a plain bf16 one: every 4-bit matrix replaced by its dequantised bf16 values."""
    layers = []
    for lw, lr in zip(gpu["layers"], ref["layers"]):
        d = dict(lw)
        for n in W4_NAMES:
            d[n] = torch.from_numpy(lr[n]).to(torch.bfloat16)      # exact: the values are bf16 already
        layers.append({n: t.to(dev()) for n, t in d.items()})
    return dict(cfg=gpu["cfg"], embed=gpu["embed"].to(dev()), final_norm=gpu["final_norm"].to(dev()),
                lm_head=gpu["lm_head"].to(dev()), layers=layers)


@pytest.mark.parametrize("T", [100, 200])
def test_forward_with_4bit_layers_matches_oracle(sx, T):
    """T = 100: at most 128 query nodes, the linear layers read the 4-bit weights directly (dequantised in registers).
    T = 200: each layer is expanded to bf16 into the scratch and the wide kernels run on the copy -- which must give
    bit for bit what the plain bf16 model with those weights gives."""
    cfg = wl.ModelCfg(3, 1024, 8, 2, 128, 2816, 4000, dtype="bf16")
    P = 150
    gpu, ref_w = _w4_model(cfg, seed=91)
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=92)
    tok, par, _ = wl.gen_best_first_tree(T, 8, cfg.vocab, seed=93)
    ref = oracle.verify_tree(cfg, ref_w, pk, pv, tok, par, act_round="bf16")["logits"]
    floor = oracle.verify_tree(cfg, ref_w, pk, pv, tok, par, act_round="bf16", perturb=3e-6)["logits"]
    mw = sx.ModelWeights(cfg, _to_device(gpu))
    assert mw.workspace_bytes(P, T) >= sx.verify_tree_workspace(cfg, P, T)
    logits, ws = sx.verify_tree(mw, pk.to(dev()), pv.to(dev()), to_dev(tok), to_dev(par))
    torch.cuda.synchronize()
    assert sx.check_status(ws) == 0
    got = logits.cpu().double().numpy()
    err, floor_max = np.abs(got - ref), float(np.abs(floor - ref).max())
    q9999 = float(np.quantile(err, 0.9999))
    print(f"\n[4-bit layers, T={T}] max|gpu-oracle|={err.max():.2e} q99.99 {q9999:.2e} rms {np.sqrt((err ** 2).mean()):.2e}; "
          f"oracle self-noise max {floor_max:.2e}; logit std {ref.std():.2f}")
    assert ref.std() > 0.3
    assert q9999 <= TOL_BF16 and err.max() <= max(TOL_BF16, 2.0 * floor_max)
    if T > 128:
        twin = sx.ModelWeights(cfg, _bf16_twin(gpu, ref_w))
        logits2, _ = sx.verify_tree(twin, pk.to(dev()), pv.to(dev()), to_dev(tok), to_dev(par))
        torch.cuda.synchronize()
        assert torch.equal(logits, logits2)


def test_4bit_weight_errors_are_reported(sx):
    cfg = wl.ModelCfg(1, 1024, 8, 2, 128, 2816, 4000, dtype="bf16")
    gpu, _ = _w4_model(cfg, seed=94)
    g = _to_device(gpu)
    tok, par = to_dev(np.zeros(200, np.int32)), to_dev(np.arange(-1, 199, dtype=np.int32))
    mw = sx.ModelWeights(cfg, g)
    small = torch.empty(sx.verify_tree_workspace(cfg, 0, 200), dtype=torch.uint8, device=dev())
    with pytest.raises(sx.SxError) as e:      # more than 128 nodes need the scratch for the bf16 copy of a layer
        sx.verify_tree(mw, None, None, tok, par, workspace=small)
    assert e.value.code == -3
    bad = sx.ModelWeights(cfg, dict(g, w4_group=96))
    with pytest.raises(sx.SxError) as e:
        sx.verify_tree(bad, None, None, tok[:8], par[:8])
    assert e.value.code == -2
    with pytest.raises(sx.SxError) as e:      # a 4-bit draft model takes batches of at most 128 nodes
        sx.draft_tree(mw, None, None, 0, tok[:1], 64, 2, 256, 4)
    assert e.value.code == -2


def test_draft_tree_with_4bit_draft_model(sx):
    """Alg. 2 with a 4-bit draft model against the same loop on the plain bf16 model that holds the dequantised
    weights: the two differ only in the summation order of their GEMMs, which can swap candidates that nearly tie;
    at least 90% of the nodes coincide and their scores agree to 0.05."""
    cfg = wl.ModelCfg(2, 512, 4, 2, 128, 1408, 2000, dtype="bf16")
    gpu, ref_w = _w4_model(cfg, seed=95)
    gpu["lm_head"] = (gpu["lm_head"].float() * 12.0).to(torch.bfloat16)
    gpu["embed"] = (gpu["embed"].float() * 20.0).to(torch.bfloat16)
    P, K, D, B, k = 40, 60, 6, 32, 6
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=96)
    root = torch.tensor([11], dtype=torch.int32, device=dev())
    trees = []
    for weights in (_to_device(gpu), _bf16_twin(gpu, ref_w)):
        mw = sx.ModelWeights(cfg, weights)
        toks, par, cum, n, ws = sx.draft_tree(mw, pk.to(dev()), pv.to(dev()), P, root, K, D, B, k)
        torch.cuda.synchronize()
        assert sx.check_status(ws) == 0
        n = int(n.item())
        t = dict(tokens=toks[:n].cpu().numpy(), parent=par[:n].cpu().numpy(), cum_logp=cum[:n].cpu().numpy())
        paths = {}
        for i in range(n):
            p, j = [], i
            while j >= 0:
                p.append(int(t["tokens"][j]))
                j = int(t["parent"][j])
            paths[tuple(reversed(p))] = float(t["cum_logp"][i])
        trees.append(paths)
    a, b = trees
    common = set(a) & set(b)
    assert len(a) == len(b) == K and len(common) >= 0.9 * K, (len(a), len(b), len(common))
    assert max(abs(a[p] - b[p]) for p in common) <= 0.05
