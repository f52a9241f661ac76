"""ctypes binding with the same names as the C ABI (include/specexec_mi.h): argument marshalling
only.  torch provides device memory and the stream; every step of the path runs in the HIP library."""
from __future__ import annotations

import ctypes as C
import os

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspecexec_mi.so")
EXPORTS = ["sx_verify_tree_workspace", "sx_verify_tree_w4_workspace", "sx_verify_tree", "sx_verify_tree_cached", "sx_verify_tree_range", "sx_commit_kv",
           "sx_specexec_round_workspace", "sx_specexec_round", "sx_draft_tree_workspace", "sx_draft_tree", "sx_accept_walk_workspace", "sx_accept_walk",
           "sx_expand_topk_workspace", "sx_expand_topk", "sx_expand_topk_static", "sx_check_status", "sx_status_string", "sx_version",
           "sx_row_logsoftmax_topk", "sx_gemm_bf16", "sx_gemm_bf16_workspace", "sx_gemm_bf16_ws", "sx_gemm_w4a16_workspace", "sx_gemm_w4a16_bf16", "sx_qkv_rope_workspace", "sx_qkv_rope_bf16", "sx_tree_attention_workspace", "sx_tree_attention_bf16",
           "sx_profile_enable", "sx_profile_select", "sx_profile_disable", "sx_profile_read"]

SX_F32, SX_BF16 = 0, 1


class SxError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32)]


_LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class _W4Matrix(C.Structure):
    _fields_ = [("qweight", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p)]


_W4_FIELDS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


class _LayerW4(C.Structure):
    _fields_ = [(n, _W4Matrix) for n in _W4_FIELDS]


class _Weights(C.Structure):
    _fields_ = [("cfg", _Cfg), ("embed", C.c_void_p), ("layers", C.POINTER(_Layer)), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p), ("layers_w4", C.POINTER(_LayerW4)), ("w4_group", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
                          "or python paper_2406_02532_amd/build.py). There is no fallback path.")
    L = C.CDLL(LIB_PATH)
    vp, i32, f32, u64, sz = C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_size_t
    L.sx_verify_tree_workspace.restype = sz
    L.sx_verify_tree_workspace.argtypes = [C.POINTER(_Cfg), i32, i32]
    L.sx_verify_tree_w4_workspace.restype = sz
    L.sx_verify_tree_w4_workspace.argtypes = [C.POINTER(_Cfg), i32, i32]
    L.sx_verify_tree.restype = C.c_int
    L.sx_verify_tree.argtypes = [C.POINTER(_Weights), vp, vp, i32, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.sx_accept_walk_workspace.restype = sz
    L.sx_verify_tree_cached.restype = C.c_int
    L.sx_verify_tree_cached.argtypes = [C.POINTER(_Weights), vp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.sx_verify_tree_range.restype = C.c_int
    L.sx_verify_tree_range.argtypes = [C.POINTER(_Weights), vp, vp, i32, i32, vp, vp, i32, i32, vp, vp, vp, i32, vp, sz, vp]
    L.sx_commit_kv.restype = C.c_int
    L.sx_commit_kv.argtypes = [C.POINTER(_Cfg), vp, vp, i32, i32, vp, vp, i32, vp, vp, vp]
    L.sx_specexec_round_workspace.restype = sz
    L.sx_specexec_round_workspace.argtypes = [C.POINTER(_Cfg), i32, i32]
    L.sx_specexec_round.restype = C.c_int
    L.sx_specexec_round.argtypes = [C.POINTER(_Weights), vp, vp, i32, i32, vp, vp, i32, f32, f32, u64, vp, vp, vp, vp, vp,
                                    vp, vp, sz, vp]
    L.sx_draft_tree_workspace.restype = sz
    L.sx_draft_tree_workspace.argtypes = [C.POINTER(_Cfg), i32, i32, i32, i32, i32]
    L.sx_draft_tree.restype = C.c_int
    L.sx_draft_tree.argtypes = [C.POINTER(_Weights), vp, vp, i32, i32, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.sx_accept_walk_workspace.argtypes = [i32, i32]
    L.sx_accept_walk.restype = C.c_int
    L.sx_accept_walk.argtypes = [vp, vp, vp, vp, i32, i32, f32, f32, u64, i32, vp, vp, vp, vp, sz, vp]
    L.sx_expand_topk_workspace.restype = sz
    L.sx_expand_topk_workspace.argtypes = [i32, i32, i32, i32]
    L.sx_expand_topk.restype = C.c_int
    L.sx_expand_topk.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    L.sx_expand_topk_static.restype = C.c_int
    L.sx_expand_topk_static.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
    L.sx_check_status.restype = C.c_int
    L.sx_check_status.argtypes = [vp, vp]
    L.sx_status_string.restype = C.c_char_p
    L.sx_status_string.argtypes = [C.c_int]
    L.sx_version.restype = C.c_int
    L.sx_row_logsoftmax_topk.restype = C.c_int
    L.sx_row_logsoftmax_topk.argtypes = [vp, i32, i32, i32, vp, vp, vp]
    L.sx_gemm_bf16.restype = C.c_int
    L.sx_gemm_bf16.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp]
    L.sx_gemm_bf16_workspace.restype = sz
    L.sx_gemm_bf16_workspace.argtypes = []
    L.sx_gemm_bf16_ws.restype = C.c_int
    L.sx_gemm_bf16_ws.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]
    L.sx_gemm_w4a16_workspace.restype = sz
    L.sx_gemm_w4a16_workspace.argtypes = []
    L.sx_gemm_w4a16_bf16.restype = C.c_int
    L.sx_gemm_w4a16_bf16.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, sz, vp]
    L.sx_qkv_rope_workspace.restype = sz
    L.sx_qkv_rope_workspace.argtypes = [i32, i32, i32]
    L.sx_qkv_rope_bf16.restype = C.c_int
    L.sx_qkv_rope_bf16.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, f32, vp, vp, vp, vp, sz, vp]
    L.sx_tree_attention_workspace.restype = sz
    L.sx_tree_attention_workspace.argtypes = [i32, i32, i32]
    L.sx_tree_attention_bf16.restype = C.c_int
    L.sx_tree_attention_bf16.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    L.sx_profile_enable.restype = C.c_int
    L.sx_profile_enable.argtypes = [i32]
    L.sx_profile_select.restype = C.c_int
    L.sx_profile_select.argtypes = [i32]
    L.sx_profile_disable.restype = C.c_int
    L.sx_profile_read.restype = C.c_int
    L.sx_profile_read.argtypes = [vp, vp, i32, vp]
    return L


lib = _load()

KERNEL_CLASSES = {1: "prep", 2: "embed", 3: "rmsnorm", 4: "gemm_qkv", 5: "rope", 6: "tree_attn", 7: "gemm_o",
                  8: "gemm_gateup_swiglu", 9: "gemm_down", 10: "gemm_lmhead", 11: "row_topk", 12: "global_select",
                  13: "accept_walk", 14: "f32_path", 15: "commit_kv"}


def status_string(code: int) -> str:
    return lib.sx_status_string(int(code)).decode()


def version() -> int:
    return lib.sx_version()


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise SxError(rc, where)


def _workspace(nbytes: int, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)  # torch allocations are 512-B aligned


def _make_cfg(cfg) -> _Cfg:
    return _Cfg(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                cfg.rope_base, cfg.rms_eps, SX_BF16 if cfg.dtype == "bf16" else SX_F32)


class ModelWeights:
    """sx_weights built from a dict of device tensors (embed, layers[list of dict], final_norm, lm_head).
    Holds references to the tensors so the pointers stay valid.  4-bit decoder layers: w["layers_w4"] = list of
    dicts name -> (qweight int32/uint32 [N][K/8], scales bf16 [N][K/group], zeros uint8 [N][K/group]) and
    w["w4_group"]; the bf16 matrices of `layers` may then be missing (the norm gains are still needed)."""

    def __init__(self, cfg, w: dict):
        self.cfg = cfg
        self._keep = w
        self.w4 = w.get("layers_w4") is not None
        self._layers = (_Layer * cfg.n_layers)()
        for l, lw in enumerate(w["layers"]):
            for n in _LAYER_FIELDS:
                t = lw.get(n)
                if t is None:
                    assert self.w4 and not n.endswith("_norm"), n
                    continue
                assert t.is_contiguous() and t.dtype == cfg.torch_dtype
                setattr(self._layers[l], n, t.data_ptr())
        self._layers_w4 = None
        if self.w4:
            self._layers_w4 = (_LayerW4 * cfg.n_layers)()
            for l, lq in enumerate(w["layers_w4"]):
                for n in _W4_FIELDS:
                    q, s, z = lq[n]
                    assert q.is_contiguous() and s.is_contiguous() and z.is_contiguous()
                    assert q.dtype in (torch.int32, torch.uint32) and s.dtype == torch.bfloat16 and z.dtype == torch.uint8
                    setattr(self._layers_w4[l], n, _W4Matrix(q.data_ptr(), s.data_ptr(), z.data_ptr()))
        self.c = _Weights(_make_cfg(cfg), w["embed"].data_ptr(), self._layers, w["final_norm"].data_ptr(),
                          w["lm_head"].data_ptr(), self._layers_w4, int(w.get("w4_group", 0)))
        self.device = w["embed"].device

    def workspace_bytes(self, P: int, T: int) -> int:
        c = _make_cfg(self.cfg)
        f = lib.sx_verify_tree_w4_workspace if self.w4 else lib.sx_verify_tree_workspace
        return f(C.byref(c), P, T)


def verify_tree_workspace(cfg, P: int, T: int) -> int:
    c = _make_cfg(cfg)
    return lib.sx_verify_tree_workspace(C.byref(c), P, T)


def verify_tree(weights: ModelWeights, prefix_k, prefix_v, tree_tokens, parent_idx, logits_out=None,
                tree_k_out=None, tree_v_out=None, workspace=None, stream=None, P=None):
    """sx_verify_tree.  Returns (logits_out, workspace); allocates them with torch when not given."""
    cfg = weights.cfg
    T = int(tree_tokens.numel())
    capacity = 0 if prefix_k is None else int(prefix_k.shape[1])
    P = capacity if P is None else int(P)          # P < capacity: the prefix is a cache with room to grow
    if logits_out is None:
        logits_out = torch.empty((T, cfg.vocab), dtype=torch.float32, device=weights.device)
    if workspace is None:
        workspace = _workspace(weights.workspace_bytes(P, T), weights.device)
    rc = lib.sx_verify_tree_cached(C.byref(weights.c), _ptr(prefix_k), _ptr(prefix_v), capacity, P, _ptr(tree_tokens),
                                   _ptr(parent_idx), T, _ptr(logits_out), _ptr(tree_k_out), _ptr(tree_v_out),
                                   _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "sx_verify_tree")
    return logits_out, workspace


def verify_tree_range(weights: ModelWeights, prefix_k, prefix_v, P: int, tree_tokens, parent_idx, first: int, tree_k,
                      tree_v, logits_out=None, workspace=None, stream=None):
    """sx_verify_tree_range: forward of nodes first .. T-1 of a tree whose earlier nodes' K/V are in tree_k/tree_v
    ([L][tree_capacity][Hkv][Dh], persistent).  Returns (logits [T - first][V], workspace)."""
    cfg = weights.cfg
    T = int(tree_tokens.numel())
    capacity = 0 if prefix_k is None else int(prefix_k.shape[1])
    if logits_out is None:
        logits_out = torch.empty((T - first, cfg.vocab), dtype=torch.float32, device=weights.device)
    if workspace is None:
        workspace = _workspace(weights.workspace_bytes(P, T), weights.device)
    rc = lib.sx_verify_tree_range(C.byref(weights.c), _ptr(prefix_k), _ptr(prefix_v), capacity, P, _ptr(tree_tokens),
                                  _ptr(parent_idx), T, first, _ptr(logits_out), _ptr(tree_k), _ptr(tree_v),
                                  int(tree_k.shape[1]), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "sx_verify_tree_range")
    return logits_out, workspace


def commit_kv(cfg, cache_k, cache_v, P: int, tree_k, tree_v, path, n, stream=None):
    """sx_commit_kv: cache[l][P + s] = tree[l][path[s]] for s < n (n a device int32 tensor)."""
    c = _make_cfg(cfg)
    capacity, T = int(cache_k.shape[1]), int(tree_k.shape[1])
    _check(lib.sx_commit_kv(C.byref(c), _ptr(cache_k), _ptr(cache_v), capacity, P, _ptr(tree_k), _ptr(tree_v), T, _ptr(path),
                            _ptr(n), _stream(stream)), "sx_commit_kv")


class RoundBuffers:
    """Device buffers of sx_specexec_round for trees of up to T nodes (allocated once, reused every round)."""

    def __init__(self, weights: ModelWeights, capacity: int, T: int):
        cfg, dev = weights.cfg, weights.device
        dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.T = T
        self.logits = torch.empty((T, cfg.vocab), dtype=torch.float32, device=dev)
        self.tree_k = torch.empty((cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim), dtype=dt, device=dev)
        self.tree_v = torch.empty_like(self.tree_k)
        self.path = torch.empty(T, dtype=torch.int32, device=dev)
        self.tokens = torch.empty(T, dtype=torch.int32, device=dev)
        self.n = torch.zeros(1, dtype=torch.int32, device=dev)
        c = _make_cfg(cfg)
        self.workspace = _workspace(lib.sx_specexec_round_workspace(C.byref(c), capacity, T), dev)


def specexec_round(weights: ModelWeights, cache_k, cache_v, P: int, tree_tokens, parent_idx, temperature: float,
                   top_p: float, seed: int, buf: RoundBuffers, stream=None):
    """sx_specexec_round: verify the tree against cache rows [0, P), walk it, append the accepted nodes' K/V to
    the cache.  Results are in buf (path, tokens, n, logits); nothing is synchronised."""
    T = int(tree_tokens.numel())
    capacity = int(cache_k.shape[1])
    rc = lib.sx_specexec_round(C.byref(weights.c), _ptr(cache_k), _ptr(cache_v), capacity, P, _ptr(tree_tokens),
                               _ptr(parent_idx), T, temperature, top_p, seed, _ptr(buf.logits), _ptr(buf.tree_k),
                               _ptr(buf.tree_v), _ptr(buf.path), _ptr(buf.tokens), _ptr(buf.n), _ptr(buf.workspace),
                               buf.workspace.numel(), _stream(stream))
    _check(rc, "sx_specexec_round")
    return buf


def draft_tree(weights: ModelWeights, prefix_k, prefix_v, P: int, root_token, K: int, D: int, B: int, k: int,
               workspace=None, stream=None, out=None):
    """sx_draft_tree: (tokens [K], parent [K], cum_logp [K], n [1], workspace) -- device tensors, nothing synchronised.
    out: the first four, preallocated (then the call allocates nothing, e.g. under stream capture)."""
    cfg, dev = weights.cfg, weights.device
    c = _make_cfg(cfg)
    capacity = 0 if prefix_k is None else int(prefix_k.shape[1])
    if out is not None:
        toks, par, cum, n = out
    else:
        toks = torch.zeros(K, dtype=torch.int32, device=dev)
        par = torch.zeros(K, dtype=torch.int32, device=dev)
        cum = torch.zeros(K, dtype=torch.float32, device=dev)
        n = torch.zeros(1, dtype=torch.int32, device=dev)
    if workspace is None:
        nbytes = lib.sx_draft_tree_workspace(C.byref(c), P, K, D, B, k)
        if nbytes == 0:
            raise SxError(-2, "sx_draft_tree_workspace")
        workspace = _workspace(nbytes, dev)
    _check(lib.sx_draft_tree(C.byref(weights.c), _ptr(prefix_k), _ptr(prefix_v), capacity, P, _ptr(root_token), K, D, B, k,
                             _ptr(toks), _ptr(par), _ptr(cum), _ptr(n), _ptr(workspace), workspace.numel(),
                             _stream(stream)), "sx_draft_tree")
    return toks, par, cum, n, workspace


def accept_walk(logits, tree_tokens, parent_idx, temperature: float, top_p: float, seed: int, pos0: int,
                path_out=None, tokens_out=None, n_out=None, workspace=None, stream=None, draft_probs=None):
    """sx_accept_walk.  Returns (path_out, tokens_out, n_out, workspace) -- device tensors."""
    T, V = logits.shape
    dev = logits.device
    if path_out is None:
        path_out = torch.empty(T, dtype=torch.int32, device=dev)
    if tokens_out is None:
        tokens_out = torch.empty(T, dtype=torch.int32, device=dev)
    if n_out is None:
        n_out = torch.empty(1, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = _workspace(lib.sx_accept_walk_workspace(T, V), dev)
    rc = lib.sx_accept_walk(_ptr(logits), _ptr(draft_probs), _ptr(tree_tokens), _ptr(parent_idx), T, V, temperature, top_p,
                            seed, pos0, _ptr(path_out), _ptr(tokens_out), _ptr(n_out), _ptr(workspace), workspace.numel(),
                            _stream(stream))
    _check(rc, "sx_accept_walk")
    return path_out, tokens_out, n_out, workspace


def expand_topk(logits, cum_logp, k: int, B: int, out_row=None, out_token=None, out_cum_logp=None, n_out=None,
                workspace=None, stream=None):
    """sx_expand_topk.  Returns (out_row, out_token, out_cum_logp, n_out, workspace)."""
    N, V = logits.shape
    dev = logits.device
    if out_row is None:
        out_row = torch.empty(B, dtype=torch.int32, device=dev)
    if out_token is None:
        out_token = torch.empty(B, dtype=torch.int32, device=dev)
    if out_cum_logp is None:
        out_cum_logp = torch.empty(B, dtype=torch.float32, device=dev)
    if n_out is None:
        n_out = torch.empty(1, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = _workspace(lib.sx_expand_topk_workspace(N, V, k, B), dev)
    rc = lib.sx_expand_topk(_ptr(logits), _ptr(cum_logp), N, V, k, B, _ptr(out_row), _ptr(out_token), _ptr(out_cum_logp),
                            _ptr(n_out), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc, "sx_expand_topk")
    return out_row, out_token, out_cum_logp, n_out, workspace


def expand_topk_static(logits, cum_logp, k: int, B: int, out_row, out_token, out_cum_logp, n_out, stream=None):
    """sx_expand_topk_static: the expansion step with the library's own fixed scratch; the caller brings every
    output (this wrapper allocates nothing either)."""
    N, V = logits.shape
    rc = lib.sx_expand_topk_static(_ptr(logits), _ptr(cum_logp), N, V, k, B, _ptr(out_row), _ptr(out_token),
                                   _ptr(out_cum_logp), _ptr(n_out), _stream(stream))
    _check(rc, "sx_expand_topk_static")
    return out_row, out_token, out_cum_logp, n_out


def row_logsoftmax_topk(logits, k: int, topk_logp=None, topk_idx=None, stream=None):
    N, V = logits.shape
    if topk_logp is None:
        topk_logp = torch.empty((N, k), dtype=torch.float32, device=logits.device)
    if topk_idx is None:
        topk_idx = torch.empty((N, k), dtype=torch.int32, device=logits.device)
    _check(lib.sx_row_logsoftmax_topk(_ptr(logits), N, V, k, _ptr(topk_logp), _ptr(topk_idx), _stream(stream)),
           "sx_row_logsoftmax_topk")
    return topk_logp, topk_idx


def gemm_bf16(X, W, Y, mode: int = 0, W2=None, workspace=None, stream=None):
    """sx_gemm_bf16 / sx_gemm_bf16_ws: Y = X W^T (mode 0), Y += X W^T (mode 1), Y = bf16(silu(X W^T) * (X W2^T))
    (mode 2).  workspace: a uint8 tensor of sx_gemm_bf16_workspace() bytes, zero before its first use."""
    M, K = X.shape
    N = W.shape[0]
    if workspace is None:
        _check(lib.sx_gemm_bf16(_ptr(X), _ptr(W), _ptr(W2), _ptr(Y), M, N, K, mode, _stream(stream)), "sx_gemm_bf16")
    else:
        _check(lib.sx_gemm_bf16_ws(_ptr(X), _ptr(W), _ptr(W2), _ptr(Y), M, N, K, mode, _ptr(workspace),
                                   workspace.numel(), _stream(stream)), "sx_gemm_bf16_ws")
    return Y


def gemm_w4a16_bf16(X, qweight, scales, zeros, Y, group: int, mode: int = 0, workspace=None, stream=None):
    """sx_gemm_w4a16_bf16: Y (+)= X dequant(qweight, scales, zeros)^T for M <= 128."""
    M, K = X.shape
    N = qweight.shape[0]
    _check(lib.sx_gemm_w4a16_bf16(_ptr(X), _ptr(qweight), _ptr(scales), _ptr(zeros), _ptr(Y), M, N, K, group, mode,
                                  _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)),
           "sx_gemm_w4a16_bf16")
    return Y


def qkv_rope_bf16(X, Wq, Wk, Wv, positions, rope_base: float, stream=None):
    """sx_qkv_rope_bf16: rotated q [T][Hq][128], rotated k and plain v [T][Hkv][128] from X [T][d]."""
    T, d = X.shape
    Hq, Hkv = Wq.shape[0] // 128, Wk.shape[0] // 128
    q = torch.empty((T, Hq, 128), dtype=torch.bfloat16, device=X.device)
    k = torch.empty((T, Hkv, 128), dtype=torch.bfloat16, device=X.device)
    v = torch.empty_like(k)
    ws = _workspace(lib.sx_qkv_rope_workspace(T, Hq, Hkv), X.device)
    _check(lib.sx_qkv_rope_bf16(_ptr(X), _ptr(Wq), _ptr(Wk), _ptr(Wv), T, d, Hq, Hkv, _ptr(positions), float(rope_base),
                                _ptr(q), _ptr(k), _ptr(v), _ptr(ws), ws.numel(), _stream(stream)), "sx_qkv_rope_bf16")
    return q, k, v


def tree_attention_bf16(q, k_tree, v_tree, k_prefix, v_prefix, parent_idx, out=None, workspace=None, stream=None):
    T, Hq, Dh = q.shape
    Hkv = k_tree.shape[1]
    P = 0 if k_prefix is None else int(k_prefix.shape[0])
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = _workspace(lib.sx_tree_attention_workspace(T, Hq, Hkv), q.device)
    _check(lib.sx_tree_attention_bf16(_ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(k_prefix), _ptr(v_prefix), _ptr(parent_idx),
                                      T, P, Hq, Hkv, _ptr(out), _ptr(workspace), workspace.numel(), _stream(stream)),
           "sx_tree_attention_bf16")
    return out, workspace


def check_status(workspace, stream=None) -> int:
    return lib.sx_check_status(_ptr(workspace), _stream(stream))


def profile_enable(max_records: int):
    _check(lib.sx_profile_enable(max_records), "sx_profile_enable")


def profile_select(kernel_class: str = ""):
    """Time only launches of the named kernel class (a value of KERNEL_CLASSES; "" = all)."""
    code = 0 if not kernel_class else {v: k for k, v in KERNEL_CLASSES.items()}[kernel_class]
    _check(lib.sx_profile_select(code), "sx_profile_select")


def profile_disable():
    lib.sx_profile_disable()


def profile_read(capacity: int = 1 << 16):
    """Returns a list of (kernel class name, milliseconds) and clears the log."""
    tags = (C.c_int32 * capacity)()
    ms = (C.c_float * capacity)()
    n = C.c_int32(0)
    _check(lib.sx_profile_read(tags, ms, capacity, C.byref(n)), "sx_profile_read")
    return [(KERNEL_CLASSES.get(tags[i], str(tags[i])), ms[i]) for i in range(n.value)]
