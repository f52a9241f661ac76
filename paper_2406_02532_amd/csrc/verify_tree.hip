// sx_verify_tree: host-side orchestration of the target forward over a token tree (Alg. 1,
// PRECOMPUTE: next_probs := FORWARD(tau, theta_target); App. D: one pass under the merged tree mask).
// Everything is enqueued on the caller's stream; there is no host synchronisation and no allocation.
#include <string.h>

#include "kernels.h"

namespace {

// Hands out 256-byte aligned slices of the workspace; with a null base it only measures.
struct Layout {
  int32_t *tok_s, *par_s, *depth, *klist, *kcnt;
  float2* rope_cs;
  unsigned long long* rowmask;
  float *h, *qkv, *gate, *up, *gu;
  void *x, *q, *o, *act, *tk, *tv;
  void* split_ws;
  size_t split_bytes;
  void* attn_split_ws;
  size_t attn_split_bytes;
  size_t bytes;
};

// One function lays the workspace out, for the size query (base == nullptr) and for the run.
Layout carve(const sx_model_cfg& c, int P, int T, void* ws) {
  (void)P;
  SxCarver cv(ws, SX_WS_HEADER);
  Layout L;
  const size_t es = c.dtype == SX_BF16 ? 2 : 4;
  const size_t Nq = (size_t)c.n_q_heads * c.head_dim, Nkv = (size_t)c.n_kv_heads * c.head_dim;
  L.tok_s = cv.take<int32_t>(T);
  L.par_s = cv.take<int32_t>(T);
  L.depth = cv.take<int32_t>(T);
  L.rope_cs = cv.take<float2>((size_t)T * (c.head_dim / 2));
  L.h = cv.take<float>((size_t)T * c.d_model);
  L.x = cv.take<char>((size_t)T * c.d_model * es);
  L.qkv = cv.take<float>((size_t)T * (Nq + 2 * Nkv));  // fp32 QKV of the paths that rotate in a kernel of their own
  L.split_bytes = c.dtype == SX_BF16 ? sx_gemm_split_workspace() : 0;  // K-split counters and partial sums of the GEMMs
  L.split_ws = L.split_bytes ? cv.take<char>(L.split_bytes) : nullptr;
  // partial attention results of small batches (at most 128 query nodes) that share the key tiles among workgroups
  L.attn_split_bytes = c.dtype == SX_BF16 ? sx_tree_attn_split_workspace(T < 128 ? T : 128, c.n_q_heads) : 0;
  L.attn_split_ws = L.attn_split_bytes ? cv.take<char>(L.attn_split_bytes) : nullptr;
  L.q = cv.take<char>((size_t)T * Nq * es);
  L.tk = cv.take<char>((size_t)T * Nkv * es);
  L.tv = cv.take<char>((size_t)T * Nkv * es);
  L.o = cv.take<char>((size_t)T * Nq * es);
  L.act = cv.take<char>((size_t)T * c.d_ffn * es);
  if (c.dtype == SX_BF16) {
    const int npt = sx_attn_min_nodes_per_tile(c.n_q_heads, c.n_kv_heads);
    const size_t tiles = (T + npt - 1) / npt;
    L.klist = cv.take<int32_t>(tiles * (size_t)T);
    L.kcnt = cv.take<int32_t>(tiles);
    L.rowmask = cv.take<unsigned long long>((size_t)T * ((T + 63) / 64));
    L.gate = L.up = nullptr;
    // gate|up product in fp32 of a batch of at most 128 nodes: the 4-bit kernels leave the SwiGLU to a kernel of its own
    L.gu = cv.take<float>((size_t)(T < 128 ? T : 128) * 2 * c.d_ffn);
  } else {
    L.klist = L.kcnt = nullptr;
    L.rowmask = nullptr;
    L.gu = nullptr;
    L.gate = cv.take<float>((size_t)T * c.d_ffn);
    L.up = cv.take<float>((size_t)T * c.d_ffn);
  }
  L.bytes = cv.off;
  return L;
}

int check_cfg(const sx_model_cfg& c, int P, int T) {
  if (c.dtype != SX_F32 && c.dtype != SX_BF16) return SX_ERR_DTYPE;
  if (c.n_layers < 1 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.head_dim < 2 || c.d_ffn < 1 ||
      c.vocab < 1 || T < 1 || T > 16384 || P < 0)
    return SX_ERR_SHAPE;
  if (c.n_q_heads % c.n_kv_heads != 0 || c.head_dim % 2 != 0) return SX_ERR_SHAPE;
  if (c.dtype == SX_BF16) {
    const int G = c.n_q_heads / c.n_kv_heads;
    if (c.head_dim != 128 || !(G == 1 || G == 2 || G == 4 || G == 8)) return SX_ERR_SHAPE;
    if (c.d_model % 64 != 0 || (c.n_q_heads * c.head_dim) % 64 != 0 || c.d_ffn % 64 != 0) return SX_ERR_SHAPE;
  } else {
    if (c.head_dim > 256 || (size_t)P + 2 * (size_t)T > 15360) return SX_ERR_SHAPE;
  }
  return SX_OK;
}

// bf16 copy of one decoder layer's seven matrices (4-bit weights, more than 128 query nodes: the wide GEMM is bound by
// the matrix cores, so the weights are expanded once per layer into this scratch and the bf16 kernels run unchanged)
size_t w4_layer_scratch_bytes(const sx_model_cfg& c) {
  const size_t Nq = (size_t)c.n_q_heads * c.head_dim, Nkv = (size_t)c.n_kv_heads * c.head_dim, d = c.d_model, F = c.d_ffn;
  return sx_align_up((Nq * d + 2 * Nkv * d + d * Nq + 3 * F * d) * 2, 256);
}

int check_w4(const sx_weights& w) {
  const sx_model_cfg& c = w.cfg;
  if (c.dtype != SX_BF16) return SX_ERR_DTYPE;
  const int g = w.w4_group, Nq = c.n_q_heads * c.head_dim;
  if (g < 64 || (g & (g - 1)) != 0 || c.d_model % g != 0 || Nq % g != 0 || c.d_ffn % g != 0) return SX_ERR_SHAPE;
  if (c.d_model % 128 != 0 || Nq % 128 != 0 || c.d_ffn % 128 != 0) return SX_ERR_SHAPE;
  for (int l = 0; l < c.n_layers; ++l) {
    const sx_layer_weights_w4& q = w.layers_w4[l];
    const sx_w4_matrix* m[7] = {&q.wq, &q.wk, &q.wv, &q.wo, &q.w_gate, &q.w_up, &q.w_down};
    for (int i = 0; i < 7; ++i)
      if (!m[i]->qweight || !m[i]->scales || !m[i]->zeros) return SX_ERR_NULL;
  }
  return SX_OK;
}

// same, bracketed by the optional event timer
#define SX_TIMED(tag, expr)   \
  do {                        \
    sx_prof_begin(tag, st);   \
    const int rc_ = (expr);   \
    sx_prof_end(st);          \
    if (rc_ != SX_OK) return rc_; \
  } while (0)

}  // namespace

extern "C" size_t sx_verify_tree_workspace(const sx_model_cfg* cfg, int32_t P, int32_t T) {
  if (!cfg || check_cfg(*cfg, P, T) != SX_OK) return 0;
  return carve(*cfg, P, T, nullptr).bytes;
}

extern "C" size_t sx_verify_tree_w4_workspace(const sx_model_cfg* cfg, int32_t P, int32_t T) {
  const size_t base = sx_verify_tree_workspace(cfg, P, T);
  if (base == 0 || cfg->dtype != SX_BF16) return 0;
  return sx_align_up(base, 256) + (T > 128 ? w4_layer_scratch_bytes(*cfg) : 0);
}

extern "C" int sx_verify_tree(const sx_weights* w, const void* prefix_k, const void* prefix_v, int32_t P,
                              const int32_t* tree_tokens, const int32_t* parent_idx, int32_t T, float* logits_out,
                              void* tree_k_out, void* tree_v_out, void* workspace, size_t workspace_bytes,
                              void* stream) {
  return sx_verify_tree_cached(w, prefix_k, prefix_v, P, P, tree_tokens, parent_idx, T, logits_out, tree_k_out,
                               tree_v_out, workspace, workspace_bytes, stream);
}

extern "C" int sx_verify_tree_cached(const sx_weights* w, const void* prefix_k, const void* prefix_v, int32_t capacity,
                                     int32_t P, const int32_t* tree_tokens, const int32_t* parent_idx, int32_t T,
                                     float* logits_out, void* tree_k_out, void* tree_v_out, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  return sx_verify_tree_range(w, prefix_k, prefix_v, capacity, P, tree_tokens, parent_idx, T, 0, logits_out, tree_k_out,
                              tree_v_out, T, workspace, workspace_bytes, stream);
}

extern "C" int sx_verify_tree_range(const sx_weights* w, const void* prefix_k, const void* prefix_v, int32_t capacity,
                                    int32_t P, const int32_t* tree_tokens, const int32_t* parent_idx, int32_t T,
                                    int32_t first, float* logits_out, void* tree_k_out, void* tree_v_out,
                                    int32_t tree_capacity, void* workspace, size_t workspace_bytes, void* stream) {
  return sx_verify_tree_range_impl(w, prefix_k, prefix_v, capacity, P, tree_tokens, parent_idx, T, first, logits_out,
                                   tree_k_out, tree_v_out, tree_capacity, workspace, workspace_bytes, false, stream);
}

int sx_verify_tree_range_impl(const sx_weights* w, const void* prefix_k, const void* prefix_v, int32_t capacity,
                              int32_t P, const int32_t* tree_tokens, const int32_t* parent_idx, int32_t T, int32_t first,
                              float* logits_out, void* tree_k_out, void* tree_v_out, int32_t tree_capacity,
                              void* workspace, size_t workspace_bytes, bool keep_status, void* stream) {
  if (capacity < P || first < 0 || first >= T || tree_capacity < T) return SX_ERR_SHAPE;
  if (first > 0 && (!tree_k_out || !tree_v_out)) return SX_ERR_NULL;  // the earlier nodes' K/V live there
  const int n = T - first;  // rows of this call: nodes first .. T-1
  if (!w || !tree_tokens || !parent_idx || !logits_out || !w->embed || !w->layers || !w->final_norm || !w->lm_head)
    return SX_ERR_NULL;
  const sx_model_cfg& c = w->cfg;
  SX_TRY(check_cfg(c, P, T));
  if (P > 0 && (!prefix_k || !prefix_v)) return SX_ERR_NULL;
  if ((tree_k_out == nullptr) != (tree_v_out == nullptr)) return SX_ERR_NULL;
  const bool w4 = w->layers_w4 != nullptr;
  if (w4) SX_TRY(check_w4(*w));
  for (int l = 0; l < c.n_layers; ++l) {
    const sx_layer_weights& lw = w->layers[l];
    if (!lw.attn_norm || !lw.ffn_norm) return SX_ERR_NULL;
    if (!w4 && (!lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.w_gate || !lw.w_up || !lw.w_down)) return SX_ERR_NULL;
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return SX_ERR_WORKSPACE;
  const Layout L = carve(c, P, T, workspace);
  if (workspace_bytes < L.bytes) return SX_ERR_WORKSPACE;
  // 4-bit weights and a wide batch: room for one layer's bf16 copy behind the ordinary workspace
  char* w4_scratch = nullptr;
  if (w4 && n > 128) {
    const size_t at = sx_align_up(L.bytes, 256);
    if (workspace_bytes < at + w4_layer_scratch_bytes(c)) return SX_ERR_WORKSPACE;
    w4_scratch = static_cast<char*>(workspace) + at;
  }

  hipStream_t st = (hipStream_t)stream;
  const bool bf = c.dtype == SX_BF16;
  const size_t es = bf ? 2 : 4;
  const int d = c.d_model, Hq = c.n_q_heads, Hkv = c.n_kv_heads, Dh = c.head_dim, F = c.d_ffn, V = c.vocab;
  const int Nq = Hq * Dh, Nkv = Hkv * Dh;
  int32_t* status = static_cast<int32_t*>(workspace);

  SX_TIMED(SX_K_PREP, sx_launch_tree_prep(tree_tokens, parent_idx, T, V, P, Dh, c.rope_base, L.tok_s, L.par_s, L.depth,
                                          L.rope_cs, status, !keep_status, st));
  if (bf)
    SX_TIMED(SX_K_PREP, sx_launch_qtile_prep(L.par_s, T, sx_attn_nodes_per_tile(Hq, Hkv, n), first, L.klist, L.kcnt,
                                             L.rowmask, st));
  SX_TIMED(SX_K_EMBED, sx_launch_embed(w->embed, c.dtype, L.tok_s + first, n, d, L.h, st));
  const float2* rope_cs = L.rope_cs + (size_t)first * (Dh / 2);  // rows of this call's nodes
  void* split_ws = L.split_ws;
  const size_t split_bytes = L.split_bytes;
  if (split_ws) SX_TRY(sx_launch_zero_i32(reinterpret_cast<int32_t*>(split_ws), 256, st));  // K-split counters

  for (int l = 0; l < c.n_layers; ++l) {
    sx_layer_weights lw = w->layers[l];
    const sx_layer_weights_w4* q4 = w4 ? &w->layers_w4[l] : nullptr;
    if (w4_scratch) {  // expand this layer's matrices; from here on the layer looks like a bf16 one
      char* at = w4_scratch;
      auto expand = [&](const sx_w4_matrix& m, int N, int K, const void** slot) -> int {
        SX_TRY(sx_launch_dequant_w4(&m, N, K, w->w4_group, at, st));
        *slot = at;
        at += (size_t)N * K * 2;
        return SX_OK;
      };
      sx_prof_begin(SX_K_NORM, st);  // (timed with the other bandwidth-bound kernels of the layer)
      SX_TRY(expand(q4->wq, Nq, d, &lw.wq));
      SX_TRY(expand(q4->wk, Nkv, d, &lw.wk));
      SX_TRY(expand(q4->wv, Nkv, d, &lw.wv));
      SX_TRY(expand(q4->wo, d, Nq, &lw.wo));
      SX_TRY(expand(q4->w_gate, F, d, &lw.w_gate));
      SX_TRY(expand(q4->w_up, F, d, &lw.w_up));
      SX_TRY(expand(q4->w_down, d, F, &lw.w_down));
      sx_prof_end(st);
      q4 = nullptr;
    }
    const size_t kv_layer = (size_t)l * tree_capacity * Nkv * es, pre_layer = (size_t)l * capacity * Nkv * es;
    // this layer's K/V of all tree nodes (keys of the attention) and where this call's nodes go in them
    char* tkb = tree_k_out ? static_cast<char*>(tree_k_out) + kv_layer : static_cast<char*>(L.tk);
    char* tvb = tree_v_out ? static_cast<char*>(tree_v_out) + kv_layer : static_cast<char*>(L.tv);
    void* tk = tkb + (size_t)first * Nkv * es;
    void* tv = tvb + (size_t)first * Nkv * es;
    const void* pk = P > 0 ? static_cast<const char*>(prefix_k) + pre_layer : nullptr;
    const void* pv = P > 0 ? static_cast<const char*>(prefix_v) + pre_layer : nullptr;

    SX_TIMED(SX_K_NORM, sx_launch_rmsnorm(L.h, lw.attn_norm, c.dtype, n, d, c.rms_eps, L.x, st));
    // the wide GEMM's epilogue rotates and splits into heads; small batches (the draft model's) take the narrow
    // GEMM, whose 64-column tiles do not hold a whole head, and rotate in a kernel of their own
    const bool fused_rope = bf && Dh == 128 && n > 128;
    if (q4) {  // at most 128 rows: the three 4-bit projections stacked in one launch, rotation in its own kernel
      const sx_w4_matrix mats[3] = {q4->wq, q4->wk, q4->wv};
      const int ns[3] = {Nq, Nkv, Nkv};
      SX_TIMED(SX_K_GEMM_QKV, sx_launch_gemm_w4_regs(L.x, mats, ns, 3, w->w4_group, L.qkv, Nq + 2 * Nkv, n, d,
                                                     SX_GEMM_STORE, split_ws, split_bytes, st));
    } else if (fused_rope) {
      SX_TIMED(SX_K_GEMM_QKV,
               sx_launch_gemm_qkv_rope_bf16(L.x, lw.wq, lw.wk, lw.wv, Hq, Hkv, rope_cs, L.q, tk, tv, n, d, split_ws,
                                            split_bytes, st));
    } else if (bf) {
      SX_TIMED(SX_K_GEMM_QKV,
               sx_launch_gemm_bf16(L.x, lw.wq, lw.wk, lw.wv, Nq, Nkv, Nkv, L.qkv, n, d, SX_GEMM_STORE, split_ws, split_bytes, st));
    } else {
      const int ld = Nq + 2 * Nkv;
      const float* x = static_cast<const float*>(L.x);
      SX_TRY(sx_launch_gemm_f32(x, (const float*)lw.wq, L.qkv, n, Nq, d, ld, false, st));
      SX_TRY(sx_launch_gemm_f32(x, (const float*)lw.wk, L.qkv + Nq, n, Nkv, d, ld, false, st));
      SX_TRY(sx_launch_gemm_f32(x, (const float*)lw.wv, L.qkv + Nq + Nkv, n, Nkv, d, ld, false, st));
    }
    if (!fused_rope)
      SX_TIMED(SX_K_ROPE, sx_launch_rope_split(L.qkv, rope_cs, n, Hq, Hkv, Dh, c.dtype, L.q, tk, tv, st));
    if (bf) {
      SX_TIMED(SX_K_ATTN, sx_launch_tree_attn_bf16(L.q, tkb, tvb, pk, pv, L.klist, L.kcnt, L.rowmask, T, n, P, Hq, Hkv,
                                                   L.o, n <= 128 ? L.attn_split_ws : nullptr, L.attn_split_bytes, st));
      if (q4) {
        const int one_d[1] = {d}, two_f[2] = {F, F};
        const sx_w4_matrix gu[2] = {q4->w_gate, q4->w_up};
        SX_TIMED(SX_K_GEMM_O, sx_launch_gemm_w4_regs(L.o, &q4->wo, one_d, 1, w->w4_group, L.h, d, n, Nq, SX_GEMM_RESIDUAL,
                                                     split_ws, split_bytes, st));
        SX_TIMED(SX_K_NORM, sx_launch_rmsnorm(L.h, lw.ffn_norm, c.dtype, n, d, c.rms_eps, L.x, st));
        SX_TIMED(SX_K_GEMM_GATEUP, sx_launch_gemm_w4_regs(L.x, gu, two_f, 2, w->w4_group, L.gu, 2 * F, n, d, SX_GEMM_STORE,
                                                          split_ws, split_bytes, st));
        SX_TIMED(SX_K_GEMM_GATEUP, sx_launch_swiglu_pair_bf16(L.gu, n, F, L.act, st));
        SX_TIMED(SX_K_GEMM_DOWN, sx_launch_gemm_w4_regs(L.act, &q4->w_down, one_d, 1, w->w4_group, L.h, d, n, F,
                                                        SX_GEMM_RESIDUAL, split_ws, split_bytes, st));
      } else {
      SX_TIMED(SX_K_GEMM_O,
               sx_launch_gemm_bf16(L.o, lw.wo, nullptr, nullptr, d, 0, 0, L.h, n, Nq, SX_GEMM_RESIDUAL, split_ws, split_bytes, st));
      SX_TIMED(SX_K_NORM, sx_launch_rmsnorm(L.h, lw.ffn_norm, c.dtype, n, d, c.rms_eps, L.x, st));
      SX_TIMED(SX_K_GEMM_GATEUP,
               sx_launch_gemm_bf16(L.x, lw.w_gate, lw.w_up, nullptr, F, F, 0, L.act, n, d, SX_GEMM_SWIGLU, split_ws, split_bytes, st));
      SX_TIMED(SX_K_GEMM_DOWN,
               sx_launch_gemm_bf16(L.act, lw.w_down, nullptr, nullptr, d, 0, 0, L.h, n, F, SX_GEMM_RESIDUAL, split_ws, split_bytes, st));
      }
    } else {
      SX_TRY(sx_launch_tree_attn_f32((const float*)L.q, (const float*)tkb, (const float*)tvb, (const float*)pk,
                                     (const float*)pv, L.par_s, L.depth, T, first, P, Hq, Hkv, Dh, (float*)L.o, st));
      SX_TRY(sx_launch_gemm_f32((const float*)L.o, (const float*)lw.wo, L.h, n, d, Nq, d, true, st));
      SX_TRY(sx_launch_rmsnorm(L.h, lw.ffn_norm, c.dtype, n, d, c.rms_eps, L.x, st));
      SX_TRY(sx_launch_gemm_f32((const float*)L.x, (const float*)lw.w_gate, L.gate, n, F, d, F, false, st));
      SX_TRY(sx_launch_gemm_f32((const float*)L.x, (const float*)lw.w_up, L.up, n, F, d, F, false, st));
      SX_TRY(sx_launch_swiglu_f32(L.gate, L.up, (float*)L.act, (size_t)n * F, st));
      SX_TRY(sx_launch_gemm_f32((const float*)L.act, (const float*)lw.w_down, L.h, n, d, F, d, true, st));
    }
  }
  SX_TIMED(SX_K_NORM, sx_launch_rmsnorm(L.h, w->final_norm, c.dtype, n, d, c.rms_eps, L.x, st));
  if (bf)
    SX_TIMED(SX_K_GEMM_LMHEAD,
             sx_launch_gemm_bf16(L.x, w->lm_head, nullptr, nullptr, V, 0, 0, logits_out, n, d, SX_GEMM_STORE, split_ws, split_bytes, st));
  else
    SX_TRY(sx_launch_gemm_f32((const float*)L.x, (const float*)w->lm_head, logits_out, n, V, d, V, false, st));
  return SX_OK;
}

// ---- KV commit and one whole round (Alg. 1, loop body) ----------------------------------------------
namespace {
// cache[l][P + s][:] = tree[l][path[s]][:] for s < *n; one workgroup per (layer, s mod gridDim.y), 16 bytes per lane
__global__ __launch_bounds__(256) void commit_kv_kernel(char* __restrict__ cache_k, char* __restrict__ cache_v,
                                                        const char* __restrict__ tree_k, const char* __restrict__ tree_v,
                                                        const int* __restrict__ path, const int* __restrict__ n_dev,
                                                        int capacity, int P, int T, int row_bytes) {
  const int l = blockIdx.x;
  int n = *n_dev;
  n = n < 0 ? 0 : (n > T ? T : n);
  if (P + n > capacity) n = capacity - P;  // the host checked P + T <= capacity; never write past the cache
  for (int s = blockIdx.y; s < n; s += gridDim.y) {
    int node = path[s];
    node = node < 0 ? 0 : (node >= T ? T - 1 : node);
    const size_t src = ((size_t)l * T + node) * row_bytes, dst = ((size_t)l * capacity + P + s) * row_bytes;
    for (int b = threadIdx.x * 16; b < row_bytes; b += 256 * 16) {
      *reinterpret_cast<u32x4*>(cache_k + dst + b) = *reinterpret_cast<const u32x4*>(tree_k + src + b);
      *reinterpret_cast<u32x4*>(cache_v + dst + b) = *reinterpret_cast<const u32x4*>(tree_v + src + b);
    }
  }
}
}  // namespace

extern "C" int sx_commit_kv(const sx_model_cfg* cfg, void* cache_k, void* cache_v, int32_t capacity, int32_t P,
                            const void* tree_k, const void* tree_v, int32_t T, const int32_t* path, const int32_t* n,
                            void* stream) {
  if (!cfg || !cache_k || !cache_v || !tree_k || !tree_v || !path || !n) return SX_ERR_NULL;
  if (cfg->dtype != SX_F32 && cfg->dtype != SX_BF16) return SX_ERR_DTYPE;
  const size_t es = cfg->dtype == SX_BF16 ? 2 : 4;
  const size_t row_bytes = (size_t)cfg->n_kv_heads * cfg->head_dim * es;
  if (cfg->n_layers < 1 || T < 1 || P < 0 || (long long)P + T > capacity || row_bytes == 0 || row_bytes % 16 != 0)
    return SX_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  sx_prof_begin(SX_K_COMMIT, st);
  commit_kv_kernel<<<dim3(cfg->n_layers, 8), 256, 0, st>>>(static_cast<char*>(cache_k), static_cast<char*>(cache_v),
                                                           static_cast<const char*>(tree_k), static_cast<const char*>(tree_v),
                                                           path, n, capacity, P, T, (int)row_bytes);
  sx_prof_end(st);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

extern "C" size_t sx_specexec_round_workspace(const sx_model_cfg* cfg, int32_t P, int32_t T) {
  const size_t v = sx_verify_tree_workspace(cfg, P, T);
  if (v == 0) return 0;
  const size_t a = sx_accept_walk_workspace(T, cfg->vocab);
  return ((v + 255) & ~(size_t)255) + a;
}

extern "C" int sx_specexec_round(const sx_weights* w, void* cache_k, void* cache_v, int32_t capacity, int32_t P,
                                 const int32_t* tree_tokens, const int32_t* parent_idx, int32_t T, float temperature,
                                 float top_p, uint64_t seed, float* logits, void* tree_k, void* tree_v,
                                 int32_t* path_out, int32_t* tokens_out, int32_t* n_out, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!w || !logits || !tree_k || !tree_v || !path_out || !tokens_out || !n_out || !workspace) return SX_ERR_NULL;
  if ((long long)P + T > capacity) return SX_ERR_SHAPE;
  const size_t v = sx_verify_tree_workspace(&w->cfg, P, T);
  if (v == 0) return SX_ERR_SHAPE;
  const size_t v_al = (v + 255) & ~(size_t)255;
  if (workspace_bytes < v_al + sx_accept_walk_workspace(T, w->cfg.vocab)) return SX_ERR_WORKSPACE;
  SX_TRY(sx_verify_tree_cached(w, cache_k, cache_v, capacity, P, tree_tokens, parent_idx, T, logits, tree_k, tree_v,
                               workspace, v, stream));
  SX_TRY(sx_accept_walk(logits, nullptr, tree_tokens, parent_idx, T, w->cfg.vocab, temperature, top_p, seed, P, path_out,
                        tokens_out, n_out, static_cast<char*>(workspace) + v_al, workspace_bytes - v_al, stream));
  return sx_commit_kv(&w->cfg, cache_k, cache_v, capacity, P, tree_k, tree_v, T, path_out, n_out, stream);
}

// Attention alone: lays out only what it needs at the head of the workspace.
namespace {
struct AttnLayout {
  int32_t *tok_s, *par_s, *depth, *klist, *kcnt;
  float2* cs;
  unsigned long long* rowmask;
  size_t bytes;
};
AttnLayout carve_attn(int T, int npt, void* ws) {
  SxCarver cv(ws, SX_WS_HEADER);
  AttnLayout L;
  const size_t tiles = (T + npt - 1) / npt;
  L.tok_s = cv.take<int32_t>(T);
  L.par_s = cv.take<int32_t>(T);
  L.depth = cv.take<int32_t>(T);
  L.cs = cv.take<float2>((size_t)T * 64);
  L.klist = cv.take<int32_t>(tiles * (size_t)T);
  L.kcnt = cv.take<int32_t>(tiles);
  L.rowmask = cv.take<unsigned long long>((size_t)T * ((T + 63) / 64));
  L.bytes = cv.off;
  return L;
}
bool attn_shape_ok(int T, int Hq, int Hkv) {
  if (T < 1 || T > 16384 || Hkv < 1 || Hq < 1 || Hq % Hkv != 0) return false;
  const int G = Hq / Hkv;
  return G == 1 || G == 2 || G == 4 || G == 8;
}
}  // namespace

extern "C" size_t sx_tree_attention_workspace(int32_t T, int32_t n_q_heads, int32_t n_kv_heads) {
  if (!attn_shape_ok(T, n_q_heads, n_kv_heads)) return 0;
  return carve_attn(T, sx_attn_min_nodes_per_tile(n_q_heads, n_kv_heads), nullptr).bytes;
}

extern "C" int sx_tree_attention_bf16(const void* q, const void* k_tree, const void* v_tree, const void* k_prefix,
                                      const void* v_prefix, const int32_t* parent_idx, int32_t T, int32_t P,
                                      int32_t n_q_heads, int32_t n_kv_heads, void* out, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  if (!q || !k_tree || !v_tree || !parent_idx || !out) return SX_ERR_NULL;
  if (P > 0 && (!k_prefix || !v_prefix)) return SX_ERR_NULL;
  if (P < 0 || !attn_shape_ok(T, n_q_heads, n_kv_heads)) return SX_ERR_SHAPE;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return SX_ERR_WORKSPACE;
  const int npt = sx_attn_nodes_per_tile(n_q_heads, n_kv_heads, T);
  const AttnLayout L = carve_attn(T, sx_attn_min_nodes_per_tile(n_q_heads, n_kv_heads), workspace);
  if (workspace_bytes < L.bytes) return SX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  SX_TRY(sx_launch_tree_prep(nullptr, parent_idx, T, 1, P, 128, 10000.f, L.tok_s, L.par_s, L.depth, L.cs,
                             static_cast<int32_t*>(workspace), true, st));
  SX_TRY(sx_launch_qtile_prep(L.par_s, T, npt, 0, L.klist, L.kcnt, L.rowmask, st));
  return sx_launch_tree_attn_bf16(q, k_tree, v_tree, k_prefix, v_prefix, L.klist, L.kcnt, L.rowmask, T, T, P, n_q_heads,
                                  n_kv_heads, out, nullptr, 0, st);
}

// cos/sin table, then (256-byte aligned) the K-split counters and partial sums of the GEMM
static size_t qkv_rope_table_bytes(int32_t T) { return (((size_t)T * 64 * sizeof(float2)) + 255) & ~(size_t)255; }
extern "C" size_t sx_qkv_rope_workspace(int32_t T, int32_t n_q_heads, int32_t n_kv_heads) {
  if (T < 1 || n_q_heads < 1 || n_kv_heads < 1) return 0;
  return qkv_rope_table_bytes(T) + sx_gemm_split_workspace();
}

extern "C" int sx_qkv_rope_bf16(const void* X, const void* Wq, const void* Wk, const void* Wv, int32_t T, int32_t d_model,
                                int32_t n_q_heads, int32_t n_kv_heads, const int32_t* positions, float rope_base,
                                void* q_out, void* k_out, void* v_out, void* workspace, size_t workspace_bytes,
                                void* stream) {
  if (!X || !Wq || !Wk || !Wv || !positions || !q_out || !k_out || !v_out || !workspace) return SX_ERR_NULL;
  if (T < 1 || d_model < 64 || d_model % 64 != 0 || n_q_heads < 1 || n_kv_heads < 1) return SX_ERR_SHAPE;
  if (workspace_bytes < sx_qkv_rope_workspace(T, n_q_heads, n_kv_heads) || (reinterpret_cast<uintptr_t>(workspace) & 255))
    return SX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  float2* cs = static_cast<float2*>(workspace);
  char* split_ws = static_cast<char*>(workspace) + qkv_rope_table_bytes(T);
  SX_TRY(sx_launch_rope_table(positions, T, 0, 128, rope_base, cs, st));
  SX_TRY(sx_launch_zero_i32(reinterpret_cast<int32_t*>(split_ws), 256, st));
  return sx_launch_gemm_qkv_rope_bf16(X, Wq, Wk, Wv, n_q_heads, n_kv_heads, cs, q_out, k_out, v_out, T, d_model, split_ws,
                                      workspace_bytes - qkv_rope_table_bytes(T), st);
}

extern "C" int sx_check_status(const void* workspace, void* stream) {
  if (!workspace) return SX_ERR_NULL;
  int32_t v = 0;
  hipStream_t st = (hipStream_t)stream;
  SX_HIP_TRY(hipMemcpyAsync(&v, workspace, sizeof(v), hipMemcpyDeviceToHost, st));
  SX_HIP_TRY(hipStreamSynchronize(st));
  return v == SX_OK ? SX_OK : (v == SX_ERR_TREE ? SX_ERR_TREE : SX_ERR_HIP);
}

extern "C" const char* sx_status_string(int s) {
  switch (s) {
    case SX_OK: return "ok";
    case SX_ERR_NULL: return "a required pointer is NULL";
    case SX_ERR_SHAPE: return "a size is outside the supported range";
    case SX_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SX_ERR_DTYPE: return "unsupported dtype";
    case SX_ERR_HIP: return "a HIP call or kernel launch failed";
    case SX_ERR_TREE: return "tree data invalid: parent index out of order or token outside the vocabulary";
  }
  return "unknown status";
}

extern "C" int sx_version(void) { return 1; }
