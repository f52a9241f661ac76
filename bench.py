#!/usr/bin/env python3
"""Benchmark of the SpecExec verification hot path on one MI355X.

One step = one pass of the whole path over resident synthetic inputs:
  sx_verify_tree (80-layer Llama-2-70B-shaped bf16 target, 2048 prefix tokens, a seeded best-first
  tree of 2048 tokens) -> sx_accept_walk (t=0.6, top-p 0.9) on the logits it produced ->
  sx_commit_kv (the accepted nodes' K/V join the prefix cache) ->
  sx_expand_topk (2048 x 32000 draft logits, k=32, best 2048 of 65536).
Prints one JSON line: verified tree tokens/s, the roofline of the dominant kernel (measured with
HIP events inside the timed steps) and the CPU oracle timed on a bounded sample of the same work.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0
CAL_COPY_BYTES = 1 << 30
# HBM bytes per launch of the dominant kernel, from hardware counters (two rocprofv3 --pmc runs of this
# file, scaled by the calibration copy); the text file states the commands and the arithmetic.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_gateup_swiglu_c5_hbm_traffic.txt")


KERNEL_SOURCES = {"gemm": os.path.join(ROOT, "paper_2406_02532_amd", "csrc", "gemm_bf16.hip"),
                  "attn": os.path.join(ROOT, "paper_2406_02532_amd", "csrc", "tree_attn_bf16.hip")}
# What the chip sustains, measured on the box with kernels that do nothing else (pure register loop of
# v_mfma_f32_16x16x32_bf16 on real operand data: the matrix pipe is power-limited; a plain streaming read of
# 262 MB): the second denominator beside the vendor's peak.
MEASURED_PEAK_BF16_TFLOPS = 1950.0
MEASURED_PEAK_HBM_READ_GBPS = 6200.0


def source_sha256(which):
    import hashlib
    return hashlib.sha256(open(KERNEL_SOURCES[which], "rb").read()).hexdigest()


def measured_traffic():
    """Counter figures recorded in TRAFFIC_FILE ('name = value' lines), each valid only while the kernel source
    it was measured on is unchanged: the file stores the sha256 of that source, and a figure whose source has
    changed since is reported as None (re-measure with the two commands the file states)."""
    vals = {}
    try:
        for line in open(TRAFFIC_FILE):
            if " = " in line and not line.startswith(" "):
                k, v = line.split(" = ", 1)
                vals[k.strip()] = v.split()[0]
    except OSError:
        return {}
    out = {}
    if vals.get("gemm_source_sha256") == source_sha256("gemm") and "traffic_bytes_per_launch" in vals:
        out["gemm_gateup"] = float(vals["traffic_bytes_per_launch"])
    if vals.get("attn_source_sha256") == source_sha256("attn") and "attn_fetch_bytes_per_launch" in vals:
        out["attn_fetch"] = float(vals["attn_fetch_bytes_per_launch"])
    return out


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C5", choices=["C2", "C3", "C5", "draft7b"],
                    help="C5 (default): the headline step.  draft7b: a side measurement, sx_draft_tree with a 32-layer "
                         "Llama-2-7B-shaped draft model (not the headline metric)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (development only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--w4", action="store_true", help="draft7b only: the draft model's decoder layers in 4 bits")
    ap.add_argument("--graph", action="store_true",
                    help="draft7b only: also time the tree construction recorded once into a HIP graph and replayed")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB -> 1 GiB device copy after the timed steps, so that a counter run "
                         "of this command holds a dispatch of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2406_02532_amd as sx
    import workloads as wl

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload == "draft7b":
        return bench_draft(args, sx, wl, torch, np, dev)
    c = wl.CONFIGS[args.workload]
    cfg = c["cfg"] if not args.layers else c["cfg"].with_layers(args.layers)
    P, T, k_tree = c["P"], c["T"], c["k"]
    c4 = wl.CONFIGS["C4"]
    temperature, top_p = c.get("temperature", 0.6), c.get("top_p", 0.9)

    # ---------------- resident inputs -------------------------------------------------------------
    t0 = time.time()
    w = wl.gen_weights(cfg, seed=1, device=dev, progress=lambda l: (l % 10 == 9 or cfg.n_layers < 10) and log(f"  weights: layer {l + 1}/{cfg.n_layers}"))
    torch.cuda.synchronize()
    nparam = sum(v.numel() for lw in w["layers"] for v in lw.values()) + w["embed"].numel() + w["lm_head"].numel()
    log(f"weights: {nparam / 1e9:.2f} G parameters ({nparam * 2 / 1e9:.1f} GB) generated on device in {time.time() - t0:.1f}s")
    pk0, pv0 = wl.gen_prefix_kv(cfg, P, seed=2, device=dev)
    # the prefix lives in a cache with room for one round's accepted tokens: [L][P + T][Hkv][Dh], rows [0, P) valid
    pk = torch.zeros((cfg.n_layers, P + T, cfg.n_kv_heads, cfg.head_dim), dtype=pk0.dtype, device=dev)
    pv = torch.zeros_like(pk)
    pk[:, :P] = pk0
    pv[:, :P] = pv0
    del pk0, pv0
    tree_k = torch.empty((cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim), dtype=pk.dtype, device=dev)
    tree_v = torch.empty_like(tree_k)
    tok, par, _ = wl.gen_best_first_tree(T, k_tree, cfg.vocab, seed=3)
    stats = wl.tree_stats(par)
    tok_d, par_d = torch.from_numpy(tok).to(dev), torch.from_numpy(par).to(dev)
    dl, dc = wl.gen_expand_inputs(c4["N"], c4["V"], seed=4, std=c4["std"], max_depth=c4["max_depth"])
    dl_d, dc_d = torch.from_numpy(dl).to(dev), torch.from_numpy(dc).to(dev)
    mw = sx.ModelWeights(cfg, w)

    logits = torch.empty((T, cfg.vocab), dtype=torch.float32, device=dev)
    ws_v = torch.empty(sx.verify_tree_workspace(cfg, P, T), dtype=torch.uint8, device=dev)
    ws_w = torch.empty(sx.lib.sx_accept_walk_workspace(T, cfg.vocab), dtype=torch.uint8, device=dev)
    ws_e = torch.empty(sx.lib.sx_expand_topk_workspace(c4["N"], c4["V"], c4["k"], c4["B"]), dtype=torch.uint8, device=dev)
    path_o = torch.empty(T, dtype=torch.int32, device=dev)
    toks_o = torch.empty(T, dtype=torch.int32, device=dev)
    n_o = torch.empty(1, dtype=torch.int32, device=dev)
    e_row = torch.empty(c4["B"], dtype=torch.int32, device=dev)
    e_tok = torch.empty(c4["B"], dtype=torch.int32, device=dev)
    e_sc = torch.empty(c4["B"], dtype=torch.float32, device=dev)
    e_n = torch.empty(1, dtype=torch.int32, device=dev)

    def step(seed):
        sx.verify_tree(mw, pk, pv, tok_d, par_d, logits_out=logits, tree_k_out=tree_k, tree_v_out=tree_v, workspace=ws_v, P=P)
        sx.accept_walk(logits, tok_d, par_d, temperature, top_p, seed, P, path_out=path_o, tokens_out=toks_o,
                       n_out=n_o, workspace=ws_w)
        sx.commit_kv(cfg, pk, pv, P, tree_k, tree_v, path_o, n_o)
        sx.expand_topk(dl_d, dc_d, c4["k"], c4["B"], out_row=e_row, out_token=e_tok, out_cum_logp=e_sc, n_out=e_n,
                       workspace=ws_e)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    assert sx.check_status(ws_v) == 0
    log(f"warmup: {args.warmup} step(s) done")

    # Inside the timed steps HIP events bracket the dominant kernel only (two event records per launch cost ~8 us of
    # stream time; around all ~500 launches of a step that would be 2% of it).  The table of all kernel classes
    # comes from one more, untimed, step afterwards.
    dom = "gemm_gateup_swiglu"
    launches_per_step = 12 * cfg.n_layers + 20
    sx.profile_select(dom)
    sx.profile_enable(launches_per_step * args.steps + 64)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(100 + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sx.profile_disable()
    dom_records = sx.profile_read(launches_per_step * args.steps + 64)
    sx.profile_select("")
    sx.profile_enable(launches_per_step + 64)
    step(99)
    torch.cuda.synchronize()
    sx.profile_disable()
    records = sx.profile_read(launches_per_step + 64)
    # ---------------- a walk that really walks (untimed by the headline) ------------------------------------
    # On a random-init target the walk leaves the tree at once.  Crafted logits (noise plus a large boost on the
    # token of the next node along the path to the deepest leaf) make accept_walk take one step per tree level
    # and commit_kv copy that many rows in every layer; both are timed with HIP events.
    walk = walk_block(sx, wl, torch, np, dev, cfg, tok, par, tok_d, par_d, pk, pv, tree_k, tree_v, P, temperature, top_p)
    sweep = t_sweep(sx, wl, torch, np, dev, cfg, mw, w, pk, pv, P, k_tree, T) if args.workload == "C5" else None
    if args.calibration_copy:
        src = torch.full((CAL_COPY_BYTES // 4,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)   # the one dispatch with a grid over 2^28 elements that reads and writes CAL_COPY_BYTES each
        torch.cuda.synchronize()
        del src, dst
    ms_per_step = elapsed / args.steps * 1e3
    log(f"timed: {args.steps} step(s) in {elapsed:.3f}s")
    value = T / (elapsed / args.steps)

    # ---------------- per-kernel figures -----------------------------------------------------------
    d, F, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    Nq, Nkv = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    depth = np.zeros(T, dtype=np.int64)
    for i in range(T):
        depth[i] = 0 if par[i] < 0 else depth[par[i]] + 1
    flops = {  # algorithmic FLOP per launch
        "gemm_qkv": 2.0 * T * d * (Nq + 2 * Nkv), "gemm_o": 2.0 * T * Nq * d, "gemm_gateup_swiglu": 4.0 * T * d * F,
        "gemm_down": 2.0 * T * F * d, "gemm_lmhead": 2.0 * T * d * V,
        "tree_attn": 4.0 * cfg.n_q_heads * cfg.head_dim * float((P + depth + 1).sum()),
    }
    nbytes = {"row_topk": 4.0 * c4["N"] * c4["V"]}   # algorithmic HBM bytes per launch
    agg = {}
    for name, ms in records:
        if name == dom:
            continue
        a = agg.setdefault(name, [0, 0.0, 1])
        a[0] += 1
        a[1] += ms
    agg[dom] = [len(dom_records), sum(ms for _, ms in dom_records), args.steps]   # the timed steps' own measurement
    kernels = {}
    for name, (n, tot, nsteps) in sorted(agg.items(), key=lambda kv: -kv[1][1] / kv[1][2]):
        e = dict(launches_per_step=n / nsteps, ms_avg=tot / n, ms_per_step=tot / nsteps)
        if name in flops:
            e["tflops"] = flops[name] / (tot / n * 1e-3) / 1e12
            e["frac_mfma_peak"] = e["tflops"] / PEAK_BF16_TFLOPS
        if name in nbytes:
            e["gbps"] = nbytes[name] / (tot / n * 1e-3) / 1e9
            e["frac_hbm_peak"] = e["gbps"] / PEAK_HBM_GBPS
        kernels[name] = {k: round(v, 6) for k, v in e.items()}
    total_flop = cfg.n_layers * (flops["gemm_qkv"] + flops["gemm_o"] + flops["gemm_gateup_swiglu"] + flops["gemm_down"]
                                 + flops["tree_attn"]) + flops["gemm_lmhead"]
    traffic = measured_traffic() if args.workload == "C5" else {}
    roofline = dict(bound="mfma", kernel="gemm_bf16_kernel<2, true> (gate|up GEMM + SwiGLU, M=%d N=%d K=%d)" % (T, 2 * F, d),
                    achieved=round(kernels[dom]["tflops"], 3), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(kernels[dom]["tflops"] / PEAK_BF16_TFLOPS, 5),
                    traffic=traffic.get("gemm_gateup"),
                    algorithmic_bytes_per_launch=2.0 * (T * d + 2 * F * d + T * F),
                    flop_per_launch=flops[dom], ms_avg=kernels[dom]["ms_avg"],
                    note="peak is the nominal dense bf16 figure; with real operand data the matrix pipe is power-limited: "
                         "a pure register loop of v_mfma_f32_16x16x32_bf16 sustains 1.93-1.97 PFLOP/s on this chip")
    roofline["frac_of_measured_peak"] = round(kernels[dom]["tflops"] / MEASURED_PEAK_BF16_TFLOPS, 5)
    roofline["measured_peak"] = MEASURED_PEAK_BF16_TFLOPS
    other = []
    for name, label in (("gemm_qkv", "gemm_bf16_kernel<3> (QKV + rotary)"), ("gemm_o", "gemm_bf16_kernel<1> (O + residual)"),
                        ("gemm_down", "gemm_bf16_kernel<1> (down + residual)"), ("tree_attn", "tree_attn_bf16_kernel")):
        if name in kernels:
            other.append(dict(kernel=label, bound="mfma", achieved=kernels[name]["tflops"], peak=PEAK_BF16_TFLOPS,
                              unit="TFLOP/s", frac=kernels[name]["frac_mfma_peak"],
                              frac_of_measured_peak=round(kernels[name]["tflops"] / MEASURED_PEAK_BF16_TFLOPS, 5)))
    kv_read_gbps = None
    if "tree_attn" in kernels:
        # K and V the attention has to read at least once per launch: prefix and tree rows of one layer
        kv_bytes = 2.0 * (P + T) * Nkv * 2
        kv_read_gbps = dict(algorithmic=round(kv_bytes / (kernels["tree_attn"]["ms_avg"] * 1e-3) / 1e9, 2),
                            algorithmic_bytes_per_launch=kv_bytes,
                            counter=(round(traffic["attn_fetch"] / (kernels["tree_attn"]["ms_avg"] * 1e-3) / 1e9, 2)
                                     if "attn_fetch" in traffic else None),
                            note="the kernel is bound by the matrix pipe, not by these reads: 16.8 MB per launch come from "
                                 "HBM once and are re-read by the query tiles from L2; 'counter' = FETCH_SIZE of the launch "
                                 "(q and K/V together) over its duration")
    if "row_topk" in kernels:
        other.append(dict(kernel="row_topk_kernel", bound="hbm", achieved=kernels["row_topk"]["gbps"], peak=PEAK_HBM_GBPS,
                          unit="GB/s", frac=kernels["row_topk"]["frac_hbm_peak"],
                          frac_of_measured_peak=round(kernels["row_topk"]["gbps"] / MEASURED_PEAK_HBM_READ_GBPS, 5)))

    out = dict(metric="verified tree tokens/s per target forward (T=%d)" % T, value=round(value, 2), unit="tokens/s",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 4), higher_is_better=True,
               scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload="%s: %d-layer Llama-2-70B-shaped target (d=%d, %d/%d heads x %d, FFN %d, vocab %d), "
                           "prefix %d, seeded best-first tree of %d tokens (k=%d), then accept_walk t=%.1f top-p %.1f, commit_kv and "
                           "expand_topk %dx%d k=%d B=%d" % (args.workload, cfg.n_layers, d, cfg.n_q_heads, cfg.n_kv_heads,
                                                              cfg.head_dim, F, V, P, T, k_tree, temperature, top_p,
                                                              c4["N"], c4["V"], c4["k"], c4["B"]),
                           tree=dict(max_depth=stats["max_depth"], mean_ancestors=round(stats["mean_ancestors"], 2)),
                           parameters_GB=round(nparam * 2 / 1e9, 1)),
               tflops=round(total_flop / (elapsed / args.steps) / 1e12, 2),
               frac_mfma_peak=round(total_flop / (elapsed / args.steps) / 1e12 / PEAK_BF16_TFLOPS, 5),
               topk_hbm_gbps=kernels.get("row_topk", {}).get("gbps"),
               kv_read_gbps=kv_read_gbps,
               measured_peaks=dict(mfma_bf16_tflops=MEASURED_PEAK_BF16_TFLOPS, hbm_read_gbps=MEASURED_PEAK_HBM_READ_GBPS,
                                   note="sustained on this chip by kernels that do nothing else: a register loop of "
                                        "v_mfma_f32_16x16x32_bf16 on real operand data (power-limited), a plain streaming read"),
               accepted_tokens_last_step=int(n_o.item()), walk=walk, t_sweep=sweep,
               roofline=roofline, other_rooflines=other, kernels=kernels)

    # ---------------- CPU oracle on a bounded sample ---------------------------------------------------
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, w, pk, pv, tok, par, dl, dc, c4, P, T, temperature, top_p)
    print(json.dumps(out), flush=True)


def walk_block(sx, wl, torch, np, dev, cfg, tok, par, tok_d, par_d, pk, pv, tree_k, tree_v, P, temperature, top_p):
    """accept_walk and commit_kv on crafted logits: the path to the deepest leaf is made overwhelmingly likely, so the
    walk takes one step per level.  Returns steps walked and microseconds per walk step / per commit."""
    T, V = len(tok), cfg.vocab
    depth = np.zeros(T, dtype=np.int64)
    for i in range(T):
        depth[i] = 0 if par[i] < 0 else depth[par[i]] + 1
    leaf, chain = int(np.argmax(depth)), []
    while leaf >= 0:
        chain.append(leaf)
        leaf = int(par[leaf])
    chain = chain[::-1]
    lg = torch.randn((T, V), dtype=torch.float32, device=dev, generator=torch.Generator(device=dev).manual_seed(5))
    for a, b in zip(chain[:-1], chain[1:]):
        lg[a, int(tok[b])] = 30.0          # the nucleus at node a is the token of its child on the chain
    path_o = torch.empty(T, dtype=torch.int32, device=dev)
    toks_o = torch.empty(T, dtype=torch.int32, device=dev)
    n_o = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(sx.lib.sx_accept_walk_workspace(T, V), dtype=torch.uint8, device=dev)
    reps, ev = 5, [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_walk = t_commit = 0.0
    for r in range(reps + 1):               # first repetition untimed
        ev[0].record()
        sx.accept_walk(lg, tok_d, par_d, temperature, top_p, 11 + r, P, path_out=path_o, tokens_out=toks_o, n_out=n_o,
                       workspace=ws)
        ev[1].record()
        sx.commit_kv(cfg, pk, pv, P, tree_k, tree_v, path_o, n_o)
        ev[2].record()
        torch.cuda.synchronize()
        if r:
            t_walk += ev[0].elapsed_time(ev[1])
            t_commit += ev[1].elapsed_time(ev[2])
    n = int(n_o.item())
    assert path_o[:n].cpu().tolist() == chain[:n] and n == len(chain), (n, len(chain))
    return dict(steps=n, accepted_draft_tokens=n - 1, us_per_walk=round(t_walk / reps * 1e3, 2),
                us_per_walk_step=round(t_walk / reps * 1e3 / n, 2), us_per_commit=round(t_commit / reps * 1e3, 2),
                rows_committed_per_layer=n, logits="crafted: N(0,1) plus 30 on the next token of the path to the deepest leaf")


def t_sweep(sx, wl, torch, np, dev, cfg, mw, w, pk, pv, P, k_tree, T_full):
    """Forward time against tree size (the paper's Fig. 1, right, asks how the target's forward time grows with the
    number of input tokens): sx_verify_tree alone on best-first trees of 128 to 2048 nodes, same model and prefix.
    Then the same target with its decoder layers in 4 bits (Sect. 5; random codes, group 128) at the two ends of the
    range: up to 128 nodes the 4-bit GEMM kernel runs, above it the layer is dequantised into a bf16 scratch copy."""
    def forward_ms(weights, T, reps=3):
        tok, par, _ = wl.gen_best_first_tree(T, k_tree, cfg.vocab, seed=3)
        tok_d, par_d = torch.from_numpy(tok).to(dev), torch.from_numpy(par).to(dev)
        logits = torch.empty((T, cfg.vocab), dtype=torch.float32, device=dev)
        ws = torch.empty(weights.workspace_bytes(P, T), dtype=torch.uint8, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for r in range(reps + 1):
            if r == 1:
                e0.record()
            sx.verify_tree(weights, pk, pv, tok_d, par_d, logits_out=logits, workspace=ws, P=P)
        e1.record()
        torch.cuda.synchronize()
        assert sx.check_status(ws) == 0
        return e0.elapsed_time(e1) / reps, par

    d, F, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    Nq, Nkv = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    out = []
    for T in (128, 256, 1024, T_full):
        ms, par = forward_ms(mw, T)
        depth = np.zeros(T, dtype=np.int64)
        for i in range(T):
            depth[i] = 0 if par[i] < 0 else depth[par[i]] + 1
        flop = cfg.n_layers * (2.0 * T * d * (Nq + 2 * Nkv) + 2.0 * T * Nq * d + 6.0 * T * d * F
                               + 4.0 * Nq * float((P + depth + 1).sum())) + 2.0 * T * d * V
        out.append(dict(T=T, weights="bf16", ms=round(ms, 3), tokens_per_s=round(T / ms * 1e3, 1), tflops=round(flop / ms / 1e9, 1)))
    free, _ = torch.cuda.mem_get_info()
    need = cfg.n_layers * (d * (Nq + 2 * Nkv) + Nq * d + 3 * d * F) * 0.53 + 8e9   # codes, scales, zero points, scratch
    if free > need:
        w4 = dict(embed=w["embed"], lm_head=w["lm_head"], final_norm=w["final_norm"],
                  layers=[{n: lw[n] for n in ("attn_norm", "ffn_norm")} for lw in w["layers"]],
                  layers_w4=wl.gen_w4_layers(cfg, 128, seed=7, device=dev), w4_group=128)
        mw4 = sx.ModelWeights(cfg, w4)
        for T in (128, T_full):
            ms, _ = forward_ms(mw4, T)
            out.append(dict(T=T, weights="4-bit decoder layers (group 128)", ms=round(ms, 3), tokens_per_s=round(T / ms * 1e3, 1)))
        del mw4, w4
        torch.cuda.empty_cache()
    return out


def bench_draft(args, sx, wl, torch, np, dev):
    """Side measurement: createDraftTree (Alg. 2) on the device with a Llama-2-7B-shaped 32-layer bf16 draft model,
    2048 cached prefix tokens, budget K=2048, D=24 iterations of B=128 nodes, k=32 children per node."""
    cfg = wl.CONFIGS["C2"]["cfg"].with_layers(args.layers or 32)
    K, D, B, k, P = 2048, 24, 128, 32, 2048
    w = wl.gen_weights(cfg, seed=5, device=dev)
    w["lm_head"] = (w["lm_head"].float() * 8).to(torch.bfloat16)      # sharper next-token distributions than N(0, 0.02)
    if args.w4:   # the same shape with 4-bit decoder layers (random codes, group 128); embed, norms and lm_head stay bf16
        w["layers_w4"] = wl.gen_w4_layers(cfg, 128, seed=7, device=dev)
        w["w4_group"] = 128
        w["layers"] = [{n: lw[n] for n in ("attn_norm", "ffn_norm")} for lw in w["layers"]]
        torch.cuda.empty_cache()
    mw = sx.ModelWeights(cfg, w)
    pk, pv = wl.gen_prefix_kv(cfg, P, seed=6, device=dev)
    root = torch.tensor([17], dtype=torch.int32, device=dev)
    toks, par, cum, n, ws = sx.draft_tree(mw, pk, pv, P, root, K, D, B, k)
    for _ in range(max(args.warmup - 1, 0)):
        sx.draft_tree(mw, pk, pv, P, root, K, D, B, k, workspace=ws)
    torch.cuda.synchronize()
    assert sx.check_status(ws) == 0
    launches = D * (12 * cfg.n_layers + 24) + 8
    graph_ms = capture_ms = None
    if args.graph:
        # the same call recorded once into a HIP graph (nothing in it allocates or synchronises) and replayed: what is
        # left of the gaps between ~8000 short launches when the host does not launch them one by one
        outs = (toks.clone(), par.clone(), cum.clone(), n.clone())
        eager = [t.clone() for t in (toks, par, cum, n)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            sx.draft_tree(mw, pk, pv, P, root, K, D, B, k, workspace=ws, out=outs)   # warm on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        t0 = time.perf_counter()
        with torch.cuda.graph(g, stream=side):
            sx.draft_tree(mw, pk, pv, P, root, K, D, B, k, workspace=ws, out=outs)
        capture_ms = (time.perf_counter() - t0) * 1e3   # recording ~8000 launches and instantiating the graph (host time)
        for rep in range(3):   # replays, with eager work and a synchronisation in between; every replay must give the eager tree
            g.replay()
            torch.cuda.synchronize()
            for a, b in zip(outs, eager):
                assert torch.equal(a, b), "graph replay differs from the eager call"
            outs[0].zero_()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / args.steps * 1e3
    sx.profile_enable(launches * args.steps + 64)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sx.draft_tree(mw, pk, pv, P, root, K, D, B, k, workspace=ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    sx.profile_disable()
    agg = {}
    for name, t in sx.profile_read(launches * args.steps + 64):
        a = agg.setdefault(name, [0, 0.0])
        a[0] += 1
        a[1] += t
    nn = int(n.item())
    par_h = par[:nn].cpu().numpy()
    depth = np.zeros(nn, dtype=np.int64)
    for i in range(1, nn):
        depth[i] = depth[par_h[i]] + 1
    nparam = sum(v.numel() for lw in w["layers"] for v in lw.values()) + w["embed"].numel() + w["lm_head"].numel()
    weight_bytes = nparam * 2
    if args.w4:
        weight_bytes += sum(t.numel() * t.element_size() for lq in w["layers_w4"] for m in lq.values() for t in m)
    print(json.dumps(dict(
        metric="draft tree construction time (side measurement, not the headline)", value=round(ms, 3), unit="ms",
        n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(ms, 3), higher_is_better=False, scaling="weak",
        vs_baseline=None, dtype="bf16", data="synthetic",
        config=dict(workload="draft7b: %d-layer Llama-2-7B-shaped draft (d=%d, %d heads x %d, FFN %d, vocab %d), prefix %d, "
                             "sx_draft_tree K=%d D=%d B=%d k=%d" % (cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.head_dim,
                                                                     cfg.d_ffn, cfg.vocab, P, K, D, B, k),
                    weights="4-bit decoder layers (group 128), bf16 embed / lm_head" if args.w4 else "bf16",
                    parameters_GB=round(weight_bytes / 1e9, 1)),
        ms_per_iteration=round(ms / D, 3), tree=dict(nodes=nn, max_depth=int(depth.max())),
        ms_per_tree_graph_replay=None if graph_ms is None else round(graph_ms, 3),
        graph_capture_ms=None if capture_ms is None else round(capture_ms, 1),
        weight_streaming_floor_ms_per_iteration=round(weight_bytes / 5.0e12 * 1e3, 3),
        kernels={k_: dict(launches_per_tree=v[0] / args.steps, ms_per_tree=round(v[1] / args.steps, 3))
                 for k_, v in sorted(agg.items(), key=lambda kv: -kv[1][1])})), flush=True)


def cpu_baseline(cfg, w, pk, pv, tok, par, dl, dc, c4, P, T, temperature, top_p):
    """The oracle as it stands, on this machine's host cores, on a bounded sample: the first 320 tree
    nodes (an ancestor-closed sub-tree) through 1 and through 2 layers (+ lm_head) to separate
    per-layer from per-call cost, 1024 rows of the draft expansion, one acceptance walk; scaled to
    the full step and expressed in the metric's unit."""
    import numpy as np
    import torch

    import oracle
    Ts, Ns = min(320, T), min(1024, c4["N"])
    cpu = lambda t: t.detach().to("cpu")
    log("cpu_baseline: copying 2 layers to the host ...")
    L2 = min(2, cfg.n_layers)
    wc = dict(embed=cpu(w["embed"]), final_norm=cpu(w["final_norm"]), lm_head=cpu(w["lm_head"]),
              layers=[{k: cpu(v) for k, v in w["layers"][l].items()} for l in range(L2)])
    pkc, pvc = cpu(pk[:L2, :P]), cpu(pv[:L2, :P])   # valid rows of the cache
    times = []
    for L in range(1, L2 + 1):
        t0 = time.perf_counter()
        oracle.verify_tree(cfg.with_layers(L), dict(wc, layers=wc["layers"][:L]), pkc[:L], pvc[:L], tok[:Ts], par[:Ts],
                           act_round="bf16")
        times.append(time.perf_counter() - t0)
        log(f"cpu_baseline: oracle verify_tree, {L} layer(s), {Ts} nodes: {times[-1]:.2f}s")
    t_layer = times[1] - times[0] if L2 == 2 else times[0]
    t_rest = max(times[0] - t_layer, 0.0)
    t0 = time.perf_counter()
    oracle.expand_topk(dl[:Ns], dc[:Ns], c4["k"], c4["B"])
    t_exp = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.accept_walk(dl[:T], tok, par, temperature, top_p, seed=1, pos0=P)   # draft logits stand in as rows to sample from
    t_walk = time.perf_counter() - t0
    step_s = (cfg.n_layers * t_layer + t_rest) * (T / Ts) + t_exp * (c4["N"] / Ns) + t_walk
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [torch.get_num_threads()])
    except Exception:
        cores = torch.get_num_threads()
    return dict(value=round(T / step_s, 4), unit="tokens/s", cores=int(cores), kind="oracle",
                sample=f"first {Ts} of {T} tree nodes through 1 and 2 of {cfg.n_layers} layers + lm_head "
                       f"({times[0]:.1f}s, {times[-1]:.1f}s), {Ns} of {c4['N']} expansion rows ({t_exp:.1f}s), one walk "
                       f"({t_walk:.2f}s); scaled linearly to the full step = {step_s:.0f}s",
                seconds_measured=round(sum(times) + t_exp + t_walk, 2))


if __name__ == "__main__":
    main()
