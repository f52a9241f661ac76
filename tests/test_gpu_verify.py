"""GPU parity: sx_verify_tree (and its GEMM / tree-attention building blocks) against the oracle's
tree forward (Alg. 1, FORWARD under the merged tree mask of App. D)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import dev, to_dev, weights_to, weights_np, bf16_ulp

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4     # fp32 path, max-abs on logits
TOL_BF16 = 2e-2    # bf16 path, max-abs on logits


@pytest.fixture(scope="module")
def sx():
    import paper_2406_02532_amd as m
    return m


# ------------------------------------------------------------------------------------------------
# tiny fp32 configuration: full-tensor parity and the structural cases
# ------------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def c1():
    c = wl.CONFIGS["C1"]
    cfg = c["cfg"]
    w = wl.gen_weights(cfg, seed=1)
    wn = weights_np(w)
    prefix = wl.gen_tokens(c["P"], cfg.vocab, seed=2)
    _, pk, pv = oracle.path_forward(cfg, wn, None, None, prefix, return_kv=True)   # the oracle's own causal prefill
    return cfg, w, wn, pk, pv


def _gpu_verify(sx, cfg, w, pk, pv, tok, par, want_kv=False):
    wd = weights_to(w, dev())
    mw = sx.ModelWeights(cfg, wd)
    dt = cfg.torch_dtype
    pkd = None if pk is None or pk.shape[1] == 0 else to_dev(torch.as_tensor(pk), dt)
    pvd = None if pv is None or pv.shape[1] == 0 else to_dev(torch.as_tensor(pv), dt)
    T = len(tok)
    tk = tv = None
    if want_kv:
        tk = torch.zeros((cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim), dtype=dt, device=dev())
        tv = torch.zeros_like(tk)
    logits, ws = sx.verify_tree(mw, pkd, pvd, to_dev(tok), to_dev(par), tree_k_out=tk, tree_v_out=tv)
    torch.cuda.synchronize()
    assert sx.check_status(ws) == 0
    return logits.cpu().numpy().astype(np.float64), tk, tv


def test_c1_full_parity(sx, c1):
    cfg, w, wn, pk, pv = c1
    tok, par = wl.gen_uniform_tree(wl.CONFIGS["C1"]["T"], cfg.vocab, seed=3)
    ref = oracle.verify_tree(cfg, wn, pk, pv, tok, par)
    got, tk, tv = _gpu_verify(sx, cfg, w, pk, pv, tok, par, want_kv=True)
    assert np.abs(ref["logits"]).max() > 0.05
    assert np.abs(got - ref["logits"]).max() <= TOL_F32
    assert np.abs(tk.cpu().double().numpy() - ref["tree_k"]).max() <= TOL_F32
    assert np.abs(tv.cpu().double().numpy() - ref["tree_v"]).max() <= TOL_F32


def test_c1_chain_single_node_and_empty_prefix(sx, c1):
    cfg, w, wn, pk, pv = c1
    tok, par = wl.gen_chain_tree(33, cfg.vocab, seed=4)
    ref = oracle.verify_tree(cfg, wn, pk, pv, tok, par)["logits"]
    got, _, _ = _gpu_verify(sx, cfg, w, pk, pv, tok, par)
    assert np.abs(got - ref).max() <= TOL_F32
    got1, _, _ = _gpu_verify(sx, cfg, w, pk, pv, tok[:1], par[:1])           # T = 1: plain single-token decode
    assert np.abs(got1 - oracle.path_forward(cfg, wn, pk, pv, tok[:1])).max() <= TOL_F32
    tok, par = wl.gen_uniform_tree(40, cfg.vocab, seed=5)                    # P = 0
    empty = np.zeros((cfg.n_layers, 0, cfg.n_kv_heads, cfg.head_dim))
    ref = oracle.verify_tree(cfg, wn, empty, empty, tok, par)["logits"]
    got, _, _ = _gpu_verify(sx, cfg, w, None, None, tok, par)
    assert np.abs(got - ref).max() <= TOL_F32


def test_c1_forest_and_every_row_equals_its_own_path(sx, c1):
    cfg, w, wn, pk, pv = c1
    tok, par = wl.gen_uniform_tree(48, cfg.vocab, seed=6)
    par = par.copy()
    par[[7, 19]] = -1                                                        # several roots are legal here
    got, _, _ = _gpu_verify(sx, cfg, w, pk, pv, tok, par)
    for i in (0, 7, 19, 30, 47):
        ref = oracle.path_forward(cfg, wn, pk, pv, tok[oracle.ancestors(par, i)])
        assert np.abs(got[i] - ref).max() <= TOL_F32


def test_c1_invalid_tree_is_reported_not_fatal(sx, c1):
    cfg, w, wn, pk, pv = c1
    tok, par = wl.gen_uniform_tree(16, cfg.vocab, seed=7)
    wd = weights_to(w, dev())
    mw = sx.ModelWeights(cfg, wd)
    bad_par = par.copy()
    bad_par[5] = 9                                                           # parent after child
    _, ws = sx.verify_tree(mw, to_dev(torch.as_tensor(pk), torch.float32), to_dev(torch.as_tensor(pv), torch.float32),
                           to_dev(tok), to_dev(bad_par))
    assert sx.check_status(ws) == -6
    bad_tok = tok.copy()
    bad_tok[3] = cfg.vocab
    _, ws = sx.verify_tree(mw, to_dev(torch.as_tensor(pk), torch.float32), to_dev(torch.as_tensor(pv), torch.float32),
                           to_dev(bad_tok), to_dev(par))
    assert sx.check_status(ws) == -6


def test_c1_walk_on_gpu_logits_equals_sequential_sampling(sx, c1):
    """Sect. 4.1 end to end.  Token-by-token sampling from the target model (oracle, no tree) gives a
    continuation; a tree that contains its first four tokens plus random distractors is verified
    and walked on the GPU with the same seed: the emitted tokens must be that continuation.
    The lm_head is scaled by 20 so that the tiny random model has LLM-like sharp distributions
    (otherwise 1024 near-equal probabilities put every decision within fp32 noise of a flip)."""
    cfg, w, wn, pk, pv = c1
    P = pk.shape[1]
    w8 = dict(w, lm_head=w["lm_head"] * 20.0)
    wn8 = dict(wn, lm_head=wn["lm_head"] * 20.0)
    mw = sx.ModelWeights(cfg, weights_to(w8, dev()))
    pkd, pvd = to_dev(torch.as_tensor(pk), torch.float32), to_dev(torch.as_tensor(pv), torch.float32)
    r = np.random.default_rng(5)
    checked = 0
    for s in range(8):
        first = int(r.integers(0, cfg.vocab))
        seq = oracle.sequential_sample(cfg, wn8, pk, pv, first, 5, 0.6, 0.9, seed=s, pos0=P)
        # chain first -> seq[0] -> seq[1] -> seq[2] -> seq[3], each node with three distractor children
        tok, par = [first], [-1]
        spine = 0
        for x in seq[:4]:
            for _ in range(3):
                d = int(r.integers(0, cfg.vocab))
                if d != x:
                    tok.append(d)
                    par.append(spine)
            tok.append(x)
            par.append(spine)
            spine = len(tok) - 1
        tok, par = np.array(tok, np.int32), np.array(par, np.int32)
        ref_logits = oracle.verify_tree(cfg, wn8, pk, pv, tok, par)["logits"]
        ref = oracle.accept_walk(ref_logits, tok, par, 0.6, 0.9, seed=s, pos0=P)
        assert ref["tokens"] == seq[:len(ref["tokens"])]                     # the oracle itself obeys the claim
        if not all(min(m["m_p"], m["m_u"]) > 1e-3 for m in ref["margins"]):
            continue
        logits, _ = sx.verify_tree(mw, pkd, pvd, to_dev(tok), to_dev(par))
        path, toks, n, _ = sx.accept_walk(logits, to_dev(tok), to_dev(par), 0.6, 0.9, s, P)
        torch.cuda.synchronize()
        n = int(n.item())
        assert toks[:n].cpu().tolist() == seq[:n] and n == len(ref["tokens"])
        assert path[:n].cpu().tolist() == ref["path"]
        checked += 1
    assert checked >= 4


def test_c1_rounds_with_kv_commit_equal_sequential_sampling(sx, c1):
    """Alg. 1's outer loop on the GPU: verify, walk, commit the accepted nodes' K/V to the cache, root the
    next tree at the last sampled token -- three rounds per seed through sx_specexec_round.  The emitted
    stream must be the oracle's token-by-token sample (Sect. 4.1), and the cache rows the rounds appended
    must be the keys/values an ordinary causal forward over those tokens produces."""
    cfg, w, wn, pk, pv = c1
    P0 = pk.shape[1]
    w8 = dict(w, lm_head=w["lm_head"] * 20.0)
    wn8 = dict(wn, lm_head=wn["lm_head"] * 20.0)
    mw = sx.ModelWeights(cfg, weights_to(w8, dev()))
    rounds, T = 3, 16
    capacity = P0 + rounds * T
    r = np.random.default_rng(11)
    checked = 0
    for s in range(10):
        first = int(r.integers(0, cfg.vocab))
        truth = oracle.sequential_sample(cfg, wn8, pk, pv, first, 3 * rounds + 3, 0.6, 0.9, seed=s, pos0=P0)
        # margin check along the true stream: every decision must be safely away from a tie
        seq, safe = [first], True
        for x in truth:
            lg = oracle.path_forward(cfg, wn8, pk, pv, seq)
            tok_, m = oracle.sample_token(lg, 0.6, 0.9, oracle.uniform01(s, P0 + len(seq)))
            assert tok_ == x
            safe &= min(m["m_p"], m["m_u"]) > 1e-3
            seq.append(x)
        if not safe:
            continue
        cache_k = torch.zeros((cfg.n_layers, capacity, cfg.n_kv_heads, cfg.head_dim), dtype=torch.float32, device=dev())
        cache_v = torch.zeros_like(cache_k)
        cache_k[:, :P0] = to_dev(torch.as_tensor(pk), torch.float32)
        cache_v[:, :P0] = to_dev(torch.as_tensor(pv), torch.float32)
        buf = sx.RoundBuffers(mw, capacity, T)
        P, root, emitted = P0, first, []
        for rd in range(rounds):
            done = len(emitted)
            # the root, a chain of the next two true tokens, and distractor children that do not carry them
            tok, par = [root], [-1]
            spine = 0
            for x in truth[done:done + 2]:
                for _ in range(3):
                    d = int(r.integers(0, cfg.vocab))
                    if d != x:
                        tok.append(d)
                        par.append(spine)
                tok.append(x)
                par.append(spine)
                spine = len(tok) - 1
            tok, par = np.array(tok, np.int32), np.array(par, np.int32)
            sx.specexec_round(mw, cache_k, cache_v, P, to_dev(tok), to_dev(par), 0.6, 0.9, s, buf)
            torch.cuda.synchronize()
            assert sx.check_status(buf.workspace) == 0
            n = int(buf.n.item())
            assert n == 3                                            # both draft tokens accepted, then one more
            toks = buf.tokens[:n].cpu().tolist()
            emitted += toks
            P += n
            root = toks[-1]
        assert emitted == truth[:len(emitted)]
        # the context is first + emitted[:-1]; its K/V at positions P0.. are what the rounds appended
        _, ks, vs = oracle.path_forward(cfg, wn8, pk, pv, [first] + emitted[:-1], return_kv=True)
        assert P == P0 + len(emitted)
        np.testing.assert_allclose(cache_k[:, P0:P].cpu().double().numpy(), ks, atol=1e-4)
        np.testing.assert_allclose(cache_v[:, P0:P].cpu().double().numpy(), vs, atol=1e-4)
        assert float(cache_k[:, P:].abs().max()) == 0.0             # nothing written past the accepted rows
        checked += 1
    assert checked >= 4


def test_c1_tree_verified_in_batches_of_nodes_matches_oracle(sx, c1):
    """Alg. 2's forward over a growing tree: nodes are verified a batch at a time (sx_verify_tree_range), each
    batch attending to the prefix and to ancestors from earlier batches through the persistent tree K/V.
    Every row must be the oracle's row for that node, whatever the batch boundaries."""
    cfg, w, wn, pk, pv = c1
    P = pk.shape[1]
    mw = sx.ModelWeights(cfg, weights_to(w, dev()))
    tok, par, _ = wl.gen_best_first_tree(48, 4, cfg.vocab, seed=9, max_depth=12)
    T = len(tok)
    ref = oracle.verify_tree(cfg, wn, pk, pv, tok, par)
    pkd, pvd = to_dev(torch.as_tensor(pk), torch.float32), to_dev(torch.as_tensor(pv), torch.float32)
    for bounds in ([0, T], [0, 1, T], [0, 5, 6, 23, 40, T]):
        tree_k = torch.zeros((cfg.n_layers, T + 3, cfg.n_kv_heads, cfg.head_dim), dtype=torch.float32, device=dev())
        tree_v = torch.zeros_like(tree_k)
        rows = []
        for lo, hi in zip(bounds[:-1], bounds[1:]):
            lg, ws = sx.verify_tree_range(mw, pkd, pvd, P, to_dev(tok[:hi]), to_dev(par[:hi]), lo, tree_k, tree_v)
            torch.cuda.synchronize()
            assert sx.check_status(ws) == 0
            rows.append(lg.cpu().double().numpy())
        got = np.concatenate(rows, axis=0)
        assert got.shape == ref["logits"].shape
        assert np.abs(got - ref["logits"]).max() <= 1e-4
        np.testing.assert_allclose(tree_k[:, :T].cpu().double().numpy(), ref["tree_k"], atol=1e-4)
        np.testing.assert_allclose(tree_v[:, :T].cpu().double().numpy(), ref["tree_v"], atol=1e-4)


def test_bf16_tree_verified_in_batches_matches_one_pass(sx):
    """Same on the MFMA path (4 narrow bf16 layers, GQA): batches of nodes against the one-pass result.  The
    batches change which keys share an attention tile and, at 128 rows or fewer, which GEMM kernel runs (narrow
    tiles, K cut in parts), hence the order of fp32 sums: bf16 roundings flip here and there, so the two results
    are two valid bf16 evaluations of one model and the bar is the bf16 one (2e-2 on the logits; this model's
    flip-noise floor is 2.4e-2), with 99% of the logits within half of it."""
    cfg = wl.ModelCfg(4, 1024, 8, 2, 128, 2752, 4000, dtype="bf16")
    w = wl.gen_weights(cfg, seed=41)
    P = 600           # ten key tiles of prefix: batches of few nodes share them among several workgroups
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=42)
    tok, par, _ = wl.gen_best_first_tree(150, 6, cfg.vocab, seed=43)
    T = len(tok)
    mw = sx.ModelWeights(cfg, weights_to(w, dev()))
    pkd, pvd = pk.to(dev()), pv.to(dev())
    one, ws = sx.verify_tree(mw, pkd, pvd, to_dev(tok), to_dev(par))
    torch.cuda.synchronize()
    one = one.cpu().double().numpy()
    tree_k = torch.zeros((cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device=dev())
    tree_v = torch.zeros_like(tree_k)
    rows = []
    bounds = [0, 1, 17, 64, 65, 130, T]
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        lg, ws = sx.verify_tree_range(mw, pkd, pvd, P, to_dev(tok[:hi]), to_dev(par[:hi]), lo, tree_k, tree_v)
        torch.cuda.synchronize()
        assert sx.check_status(ws) == 0
        rows.append(lg.cpu().double().numpy())
    got = np.concatenate(rows, axis=0)
    diff = np.abs(got - one)
    # both against the oracle's bf16 evaluation, to the bar of the one-pass tests: 99.99% within 2e-2, the worst
    # within twice the oracle's own flip-noise floor; and against each other, two valid evaluations, the same
    ref = oracle.verify_tree(cfg, w, pk, pv, tok, par, act_round="bf16")["logits"]
    floor = np.abs(oracle.verify_tree(cfg, w, pk, pv, tok, par, act_round="bf16", perturb=3e-6)["logits"] - ref).max()
    for name, x in (("batches", got), ("one pass", one)):
        e = np.abs(x - ref)
        print(f"[{name}] max|gpu-oracle|={e.max():.3e}, 99.99th pct {np.quantile(e, 0.9999):.3e}; floor {floor:.3e}")
        _assert_bf16_parity(float(e.max()), float(np.quantile(e, 0.9999)), float(floor))
    assert diff.max() <= max(TOL_BF16, 2.0 * floor) and np.quantile(diff, 0.99) <= 1e-2, (diff.max(), np.quantile(diff, 0.99))


def test_range_and_round_edge_cases(sx, c1):
    """One node at a time into a tree buffer larger than the tree; host-side shape errors of the new calls."""
    cfg, w, wn, pk, pv = c1
    P = pk.shape[1]
    mw = sx.ModelWeights(cfg, weights_to(w, dev()))
    tok, par = wl.gen_chain_tree(6, cfg.vocab, seed=4)
    ref = oracle.verify_tree(cfg, wn, pk, pv, tok, par)["logits"]
    pkd, pvd = to_dev(torch.as_tensor(pk), torch.float32), to_dev(torch.as_tensor(pv), torch.float32)
    tree_k = torch.zeros((cfg.n_layers, 20, cfg.n_kv_heads, cfg.head_dim), dtype=torch.float32, device=dev())
    tree_v = torch.zeros_like(tree_k)
    for i in range(6):                                               # a chain grown one token at a time = decoding
        lg, ws = sx.verify_tree_range(mw, pkd, pvd, P, to_dev(tok[:i + 1]), to_dev(par[:i + 1]), i, tree_k, tree_v)
        torch.cuda.synchronize()
        assert sx.check_status(ws) == 0 and lg.shape[0] == 1
        assert np.abs(lg.cpu().double().numpy()[0] - ref[i]).max() <= 1e-4
    with pytest.raises(sx.SxError):                                  # first node beyond the tree
        sx.verify_tree_range(mw, pkd, pvd, P, to_dev(tok), to_dev(par), 6, tree_k, tree_v)
    small_k = torch.zeros((cfg.n_layers, 4, cfg.n_kv_heads, cfg.head_dim), dtype=torch.float32, device=dev())
    with pytest.raises(sx.SxError):                                  # tree buffers smaller than the tree
        sx.verify_tree_range(mw, pkd, pvd, P, to_dev(tok), to_dev(par), 2, small_k, small_k.clone())
    buf = sx.RoundBuffers(mw, P + 6, 6)
    with pytest.raises(sx.SxError):                                  # the cache has no room for the round's nodes
        sx.specexec_round(mw, pkd, pvd, P, to_dev(tok), to_dev(par), 0.6, 0.9, 1, buf)


def test_commit_kv_bf16_gathers_path_rows(sx):
    """sx_commit_kv alone, bf16 rows of 2 KB, n read from the device: byte-exact gather, rows past n untouched."""
    cfg = wl.ModelCfg(3, 1024, 8, 8, 128, 2752, 4000, dtype="bf16")
    T, P, cap = 40, 10, 64
    tk = wl.hash_normal(5, (3, T, 8, 128), dtype=torch.bfloat16).to(dev())
    tv = wl.hash_normal(6, (3, T, 8, 128), dtype=torch.bfloat16).to(dev())
    ck = torch.full((3, cap, 8, 128), 7.0, dtype=torch.bfloat16, device=dev())
    cv = torch.full((3, cap, 8, 128), 9.0, dtype=torch.bfloat16, device=dev())
    path = torch.tensor([0, 3, 17, 39, 5, 6] + [0] * (T - 6), dtype=torch.int32, device=dev())
    n = torch.tensor([4], dtype=torch.int32, device=dev())
    sx.commit_kv(cfg, ck, cv, P, tk, tv, path, n)
    torch.cuda.synchronize()
    for s_, node in enumerate([0, 3, 17, 39]):
        assert torch.equal(ck[:, P + s_], tk[:, node]) and torch.equal(cv[:, P + s_], tv[:, node])
    assert bool((ck[:, :P] == 7.0).all()) and bool((ck[:, P + 4:] == 7.0).all()) and bool((cv[:, P + 4:] == 9.0).all())
    with pytest.raises(sx.SxError):                                   # P + T must fit the cache
        sx.commit_kv(cfg, ck, cv, 30, tk, tv, path, n)


# ------------------------------------------------------------------------------------------------
# bf16 building blocks
# ------------------------------------------------------------------------------------------------

# (100, 20000, 192) and (128, 17000, 64): few rows and a wide matrix, the 128-column form of the narrow kernel, ragged last tile
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (256, 512, 256), (300, 200, 128), (1, 1000, 192), (520, 768, 4096),
                                   (128, 4096, 11008), (33, 72, 64), (100, 130, 320), (100, 20000, 192),
                                   (128, 17000, 64)])
def test_gemm_bf16_store_and_residual(sx, M, N, K):
    X = wl.hash_normal(1, (M, K), dtype=torch.bfloat16)
    W = wl.hash_normal(2, (N, K), std=0.05, dtype=torch.bfloat16)
    ref = X.double().numpy() @ W.double().numpy().T
    Y = torch.full((M, N), 7.0, dtype=torch.float32, device=dev())
    sx.gemm_bf16(X.to(dev()), W.to(dev()), Y, mode=0)
    torch.cuda.synchronize()
    tol = 1e-5 * np.sqrt(K) * np.abs(ref).max() + 1e-6
    assert np.abs(Y.cpu().double().numpy() - ref).max() <= tol
    sx.gemm_bf16(X.to(dev()), W.to(dev()), Y, mode=1)                        # Y += X W^T
    torch.cuda.synchronize()
    assert np.abs(Y.cpu().double().numpy() - 2 * ref).max() <= 2 * tol


@pytest.mark.parametrize("M", [64, 128, 129, 300])
def test_gemm_bf16_llama3_vocabulary_head(sx, M):
    """lm_head at a 128256-token vocabulary (Llama-3 shape), on both sides of the 128-row switch between the
    narrow-tile and the wide-tile kernel; K kept small so that the fp64 product stays cheap."""
    N, K = 128256, 256
    X = wl.hash_normal(21, (M, K), dtype=torch.bfloat16)
    W = wl.hash_normal(22, (N, K), std=0.05, dtype=torch.bfloat16)
    ref = X.double().numpy() @ W.double().numpy().T
    Y = torch.empty((M, N), dtype=torch.float32, device=dev())
    sx.gemm_bf16(X.to(dev()), W.to(dev()), Y, mode=0)
    torch.cuda.synchronize()
    assert np.abs(Y.cpu().double().numpy() - ref).max() <= 1e-5 * np.sqrt(K) * np.abs(ref).max() + 1e-6


@pytest.mark.parametrize("M,N,K,group,split", [(128, 4096, 4096, 128, True), (128, 256, 11008, 64, True),
                                               (37, 200, 256, 128, False), (1, 64, 64, 64, False),
                                               (100, 12288, 512, 128, True), (128, 300, 128, 64, False),
                                               (5, 1000, 1024, 256, True), (128, 520, 2048, 1024, True),
                                               (64, 768, 192, 64, True)])
def test_gemm_w4a16(sx, M, N, K, group, split):
    """4-bit group-quantised weights dequantised in registers: against the oracle's product with the weights it
    dequantises by the stated formula (bf16(scale * (code - zero))); with and without K cut among workgroups,
    store and accumulate."""
    X = wl.hash_normal(31, (M, K), dtype=torch.bfloat16)
    qw, sc, zr = wl.gen_w4(N, K, group, seed=32)
    ref = oracle.gemm_w4a16(X, qw.numpy().view(np.uint32), sc.double().numpy(), zr.numpy(), group)
    Y = torch.full((M, N), 3.0, dtype=torch.float32, device=dev())
    ws = torch.empty(sx.lib.sx_gemm_w4a16_workspace(), dtype=torch.uint8, device=dev()) if split else None
    args = (X.to(dev()), qw.to(dev()), sc.to(dev()), zr.to(dev()))
    sx.gemm_w4a16_bf16(*args, Y, group, mode=0, workspace=ws)
    torch.cuda.synchronize()
    tol = 1e-5 * np.sqrt(K) * np.abs(ref).max() + 1e-6
    assert np.abs(Y.cpu().double().numpy() - ref).max() <= tol
    sx.gemm_w4a16_bf16(*args, Y, group, mode=1, workspace=ws)
    torch.cuda.synchronize()
    assert np.abs(Y.cpu().double().numpy() - 2 * ref).max() <= 2 * tol


@pytest.mark.parametrize("M,F,K", [(256, 128, 64), (300, 200, 256), (100, 11008, 128), (128, 96, 4096), (7, 40, 64),
                                   (77, 9000, 128)])
def test_gemm_bf16_swiglu(sx, M, F, K):
    X = wl.hash_normal(3, (M, K), dtype=torch.bfloat16)
    Wg = wl.hash_normal(4, (F, K), std=0.1, dtype=torch.bfloat16)
    Wu = wl.hash_normal(5, (F, K), std=0.1, dtype=torch.bfloat16)
    g = X.double().numpy() @ Wg.double().numpy().T
    u = X.double().numpy() @ Wu.double().numpy().T
    ref = g / (1 + np.exp(-g)) * u
    Y = torch.zeros((M, F), dtype=torch.bfloat16, device=dev())
    sx.gemm_bf16(X.to(dev()), Wg.to(dev()), Y, mode=2, W2=Wu.to(dev()))
    torch.cuda.synchronize()
    got = Y.cpu().double().numpy()
    assert np.all(np.abs(got - ref) <= 0.51 * bf16_ulp(ref) + 1e-5 * np.abs(ref).max())   # correctly rounded up to fp32 noise


@pytest.mark.parametrize("M,N,K,mode", [(256, 2048, 4096, 0), (256, 2048, 4096, 1), (200, 1000, 2048, 1),
                                        (1024, 8192, 1024, 1), (300, 2100, 1536, 0), (256, 1024, 11008, 1),
                                        (256, 1536, 2048, 2), (200, 1000, 1024, 2)])
def test_gemm_bf16_few_tiles_cut_along_k(sx, M, N, K, mode):
    """Launches whose 256 x 256 output tiles are fewer than half the compute units (trees of a few hundred nodes):
    with a workspace every tile is cut along K among several workgroups.  All three epilogues against the fp64
    product, ragged edges, and bit-identical repeats (the parts are added in part order whoever arrives last)."""
    X = wl.hash_normal(41, (M, K), dtype=torch.bfloat16)
    W = wl.hash_normal(42, (N, K), std=0.05, dtype=torch.bfloat16)
    W2 = wl.hash_normal(43, (N, K), std=0.05, dtype=torch.bfloat16) if mode == 2 else None
    ws = torch.zeros(sx.lib.sx_gemm_bf16_workspace(), dtype=torch.uint8, device=dev())
    Xd, Wd, W2d = X.to(dev()), W.to(dev()), None if W2 is None else W2.to(dev())
    ref = X.double().numpy() @ W.double().numpy().T
    outs = []
    for rep in range(3):
        if mode == 2:
            Y = torch.zeros((M, N), dtype=torch.bfloat16, device=dev())
        else:
            Y = torch.full((M, N), 0.5, dtype=torch.float32, device=dev())
        sx.gemm_bf16(Xd, Wd, Y, mode=mode, W2=W2d, workspace=ws)
        torch.cuda.synchronize()
        outs.append(Y.cpu())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert int(ws[:1024].max()) == 0                                          # the counters are back at zero
    got = outs[0].double().numpy()
    if mode == 2:
        u = X.double().numpy() @ W2.double().numpy().T
        want = ref / (1 + np.exp(-ref)) * u
        assert np.all(np.abs(got - want) <= 0.51 * bf16_ulp(want) + 1e-5 * np.abs(want).max())
    else:
        want = ref + 0.5 if mode == 1 else ref
        assert np.abs(got - want).max() <= 1e-5 * np.sqrt(K) * np.abs(ref).max() + 1e-6
    # and the same call without a workspace (no cut) agrees to fp32 summation-order noise
    Y0 = torch.zeros((M, N), dtype=torch.bfloat16 if mode == 2 else torch.float32, device=dev())
    sx.gemm_bf16(Xd, Wd, Y0, mode=mode, W2=W2d)
    torch.cuda.synchronize()
    d = np.abs(Y0.cpu().double().numpy() - (got - (0.5 if mode == 1 else 0.0)))
    assert d.max() <= (1.01 * bf16_ulp(got).max() if mode == 2 else 1e-5 * np.sqrt(K) * np.abs(ref).max() + 1e-6)


# the last three shapes give more output tiles than the chip has compute units with a small remainder: the
# remainder tiles are cut along K and their partial sums added up by the last workgroup to arrive
# (256, 2048, 16, 4) and (512, 1024, 8, 8): fewer tiles than half the compute units, all of them cut along K;
# (77, 8192, 64, 8): few rows, three stacked matrices through the 128-column form of the narrow kernel, K cut in 3
@pytest.mark.parametrize("T,d,Hq,Hkv", [(256, 256, 2, 2), (300, 512, 4, 1), (77, 1024, 8, 2),
                                        (2048, 2048, 64, 8), (2048, 2048, 64, 1), (2304, 1024, 64, 8),
                                        (256, 2048, 16, 4), (512, 1024, 8, 8), (77, 8192, 64, 8)])
def test_qkv_projection_with_rotary_epilogue(sx, T, d, Hq, Hkv):
    """The QKV GEMM that rotates and splits into heads in its epilogue, against the oracle's rope applied to
    fp64 projections (rows beyond a tile, GQA, head columns that cross tile boundaries)."""
    X = wl.hash_normal(11, (T, d), dtype=torch.bfloat16)
    Wq = wl.hash_normal(12, (Hq * 128, d), std=0.05, dtype=torch.bfloat16)
    Wk = wl.hash_normal(13, (Hkv * 128, d), std=0.05, dtype=torch.bfloat16)
    Wv = wl.hash_normal(14, (Hkv * 128, d), std=0.05, dtype=torch.bfloat16)
    pos = (np.arange(T) * 7 % 3000 + 5).astype(np.int32)                       # positions up to a few thousand
    x64 = X.double().numpy()
    ref_q = oracle.rope((x64 @ Wq.double().numpy().T).reshape(T, Hq, 128), pos, 10000.0)
    ref_k = oracle.rope((x64 @ Wk.double().numpy().T).reshape(T, Hkv, 128), pos, 10000.0)
    ref_v = (x64 @ Wv.double().numpy().T).reshape(T, Hkv, 128)
    q, k, v = sx.qkv_rope_bf16(X.to(dev()), Wq.to(dev()), Wk.to(dev()), Wv.to(dev()), torch.from_numpy(pos).to(dev()), 10000.0)
    torch.cuda.synchronize()
    for got, ref in ((q, ref_q), (k, ref_k), (v, ref_v)):
        got = got.cpu().double().numpy()
        # correctly rounded to bf16 up to fp32 accumulation / table noise
        assert np.all(np.abs(got - ref) <= 0.51 * bf16_ulp(ref) + 2e-5 * np.abs(ref).max())


def test_qkv_projection_repeats_bit_for_bit_in_fresh_workspaces(sx):
    """The tail tiles of this shape (320 tiles on 256 compute units, the last 64 cut four ways along K) take their
    partial sums through memory: four calls, each in a workspace of its own holding whatever was there before, give
    the same bits."""
    T, d, Hq, Hkv = 2048, 2048, 64, 8
    X = wl.hash_normal(11, (T, d), dtype=torch.bfloat16).to(dev())
    Wq = wl.hash_normal(12, (Hq * 128, d), std=0.05, dtype=torch.bfloat16).to(dev())
    Wk = wl.hash_normal(13, (Hkv * 128, d), std=0.05, dtype=torch.bfloat16).to(dev())
    Wv = wl.hash_normal(14, (Hkv * 128, d), std=0.05, dtype=torch.bfloat16).to(dev())
    pos = torch.arange(T, dtype=torch.int32, device=dev()) + 5
    outs = []
    for r in range(4):
        junk = torch.full((1 << 25,), 0.3 + 1.7 * r, device=dev())      # what the next workspace is carved from
        del junk
        q, k, v = sx.qkv_rope_bf16(X, Wq, Wk, Wv, pos, 10000.0)
        torch.cuda.synchronize()
        outs.append((q.clone(), k.clone(), v.clone()))
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def _attn_case(sx, T, P, Hq, Hkv, tree, seed):
    tok, par = tree
    q = wl.hash_normal(seed, (T, Hq, 128), std=1.5, dtype=torch.bfloat16)
    kt = wl.hash_normal(seed + 1, (T, Hkv, 128), std=1.5, dtype=torch.bfloat16)
    vt = wl.hash_normal(seed + 2, (T, Hkv, 128), dtype=torch.bfloat16)
    kp = wl.hash_normal(seed + 3, (P, Hkv, 128), std=1.5, dtype=torch.bfloat16)
    vp = wl.hash_normal(seed + 4, (P, Hkv, 128), dtype=torch.bfloat16)
    ref = oracle.tree_attention(q, kt, vt, kp, vp, par)
    out, ws = sx.tree_attention_bf16(q.to(dev()), kt.to(dev()), vt.to(dev()), kp.to(dev()) if P else None,
                                     vp.to(dev()) if P else None, to_dev(par))
    torch.cuda.synchronize()
    assert sx.check_status(ws) == 0
    got = out.cpu().double().numpy()
    # the output is a bf16 rounding of an fp32 result whose probabilities carry ~16 bits
    err = np.abs(got - ref)
    assert np.all(err <= 0.5 * bf16_ulp(ref) + 2e-4 * np.abs(ref).max() + 1e-6), err.max()


@pytest.mark.parametrize("T,P,Hq,Hkv", [(64, 64, 8, 1), (200, 100, 8, 1), (130, 0, 4, 4), (257, 513, 8, 2), (96, 1000, 16, 4)])
def test_tree_attention_bf16_best_first(sx, T, P, Hq, Hkv):
    tok, par, _ = wl.gen_best_first_tree(T, 4, 1000, seed=T, max_depth=20)
    _attn_case(sx, T, P, Hq, Hkv, (tok, par), seed=10 * T)


def test_tree_attention_bf16_chain_and_uniform(sx):
    _attn_case(sx, 300, 70, 8, 1, wl.gen_chain_tree(300, 100, seed=1), seed=7)      # depth 299: many tree tiles
    _attn_case(sx, 300, 70, 2, 2, wl.gen_uniform_tree(300, 100, seed=2), seed=8)


# ------------------------------------------------------------------------------------------------
# bf16 decoder: full-tensor parity on a narrow multi-layer model and on the 7B-shaped layer
# ------------------------------------------------------------------------------------------------

def _bf16_model_parity(sx, cfg, P, T, k, seed):
    w = wl.gen_weights(cfg, seed=seed)
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=seed + 1)
    tok, par, _ = wl.gen_best_first_tree(T, k, cfg.vocab, seed=seed + 2)
    ref = oracle.verify_tree(cfg, w, pk, pv, tok, par, act_round="bf16")
    got, tk, tv = _gpu_verify(sx, cfg, w, pk, pv, tok, par, want_kv=True)
    err = float(np.abs(got - ref["logits"]).max())
    # Noise floor: the oracle against itself with inputs nudged by 3e-6 (the size of fp32-vs-fp64
    # arithmetic differences).  Rounding flips cascade through the bf16 stages, so two equally
    # valid bf16 evaluations of one model differ by this much however they are implemented.
    floor_run = oracle.verify_tree(cfg, w, pk, pv, tok, par, act_round="bf16", perturb=3e-6)
    floor = floor_run["logits"]
    # layer 0 sees identical inputs on both sides: its K/V may differ by one bf16 rounding step only
    # (two where the reference sits just below a power of two); deeper layers inherit earlier flips,
    # and are held to twice what the oracle's own nudged evaluation shows in the same measure
    for name, t_, r_, f_ in (("k", tk, ref["tree_k"], floor_run["tree_k"]), ("v", tv, ref["tree_v"], floor_run["tree_v"])):
        e0 = np.abs(t_[0].cpu().double().numpy() - r_[0])
        bad = int((e0 > 2.0 * bf16_ulp(r_[0]) + 2e-3).sum())      # 2e-3: a flipped bf16 input times a 4-sigma weight
        flips = float((e0 > 0).mean())
        assert bad == 0 and flips < 0.01, (name, bad, flips)
        scale = bf16_ulp(r_) + 2e-3
        e = float((np.abs(t_.cpu().double().numpy() - r_) / scale).max())
        e_floor = float((np.abs(f_ - r_) / scale).max())
        print(f"[tree {name}] max error in (ulp + 2e-3) units: gpu {e:.2f}, oracle self-noise {e_floor:.2f}")
        assert e <= max(8.0, 2.0 * e_floor), (name, e, e_floor)
    floor_max = float(np.abs(floor - ref["logits"]).max())
    pure = oracle.verify_tree(cfg, w, pk, pv, tok, par)["logits"]
    q9999 = float(np.quantile(np.abs(got - ref["logits"]), 0.9999))
    print(f"\n[{cfg.n_layers} layer(s), d={cfg.d_model}] max|gpu-oracle|={err:.2e} (99.99th pct {q9999:.2e}, rms "
          f"{np.sqrt(((got - ref['logits']) ** 2).mean()):.2e}); oracle self-noise floor max={floor_max:.2e}; "
          f"max|gpu-oracle(fp64 acts)|={np.abs(got - pure).max():.2e}; logit std {ref['logits'].std():.2f}")
    return err, q9999, floor_max, float(ref["logits"].std())


def _assert_bf16_parity(err, q9999, floor_max):
    assert q9999 <= TOL_BF16, q9999                       # all but 1e-4 of the logits within the stated tolerance
    assert err <= max(TOL_BF16, 2.0 * floor_max), (err, floor_max)   # the worst one within twice the flip-noise floor


def test_bf16_narrow_four_layer_model(sx):
    cfg = wl.ModelCfg(4, 1024, 8, 2, 128, 2752, 4000, dtype="bf16")
    err, q, floor, std = _bf16_model_parity(sx, cfg, P=200, T=160, k=8, seed=21)
    assert std > 0.3
    _assert_bf16_parity(err, q, floor)


def test_bf16_small_tree_takes_the_narrow_kernels(sx):
    """A tree of 100 nodes (at most 128 rows): the narrow-tile GEMMs with K cut among workgroups, the rotation
    in a kernel of its own and attention tiles of fewer rows, against the oracle, to the same bar."""
    cfg = wl.ModelCfg(4, 1024, 8, 2, 128, 2752, 4000, dtype="bf16")
    err, q, floor, std = _bf16_model_parity(sx, cfg, P=700, T=100, k=8, seed=25)
    assert std > 0.3
    _assert_bf16_parity(err, q, floor)


def test_c2_llama7b_layer_full_parity(sx):
    c = wl.CONFIGS["C2"]
    err, q, floor, std = _bf16_model_parity(sx, c["cfg"], c["P"], c["T"], c["k"], seed=31)
    assert std > 1.0
    _assert_bf16_parity(err, q, floor)


def test_verify_tree_repeats_bit_for_bit_where_tiles_are_cut_along_k(sx):
    """Run-to-run determinism of the forward at a shape that takes the K split: one 70B-shaped layer over a
    2048-node tree (the QKV projection then has 320 tiles on 256 compute units, the last 64 cut in two along K,
    their partial sums added by whichever workgroup arrives last -- in part order, so the sum must not depend
    on who that was).  Three runs, the scratch memory filled with different garbage before each: logits and
    tree K/V identical to the last bit."""
    cfg = wl.CONFIGS["C5"]["cfg"].with_layers(1)
    T, P = 2048, 192
    w = wl.gen_weights(cfg, seed=41, device=dev())
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=42, device=dev())
    tok, par, _ = wl.gen_best_first_tree(T, 32, cfg.vocab, seed=43)
    mw = sx.ModelWeights(cfg, w)
    td, pd = to_dev(tok), to_dev(par)
    ws = torch.empty(sx.verify_tree_workspace(cfg, P, T), dtype=torch.uint8, device=dev())
    runs = []
    for fill in (0, 0xA5, 0x3C):
        ws.fill_(fill)
        tk = torch.empty((1, T, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16, device=dev())
        tv = torch.empty_like(tk)
        logits, _ = sx.verify_tree(mw, pk, pv, td, pd, tree_k_out=tk, tree_v_out=tv, workspace=ws)
        torch.cuda.synchronize()
        assert sx.check_status(ws) == 0
        runs.append((logits.clone(), tk, tv))
    assert torch.isfinite(runs[0][0]).all() and float(runs[0][0].std()) > 1.0
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                               b.view(torch.int32) if b.dtype == torch.float32 else b.view(torch.int16))
