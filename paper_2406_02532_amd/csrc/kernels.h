// Host-side launchers shared between the translation units of the library.  Each returns an
// sx_status and only enqueues work on the given stream.
#pragma once
#include "common.h"

// ---- tree bookkeeping (tree_prep.hip) -------------------------------------------------------------
// Checks parent/token ranges (status word <- SX_ERR_TREE on violation), writes sanitised copies,
// the depth of every node and the rotary table cs[T][Dh/2] = (cos, sin) of (P+depth)*base^(-2j/Dh).
// reset_status: the status word starts at SX_OK (false: an error recorded by an earlier call on the same
// workspace stays, so a forward that grows a tree call by call reports the first bad batch at the end).
int sx_launch_tree_prep(const int32_t* tokens, const int32_t* parent, int T, int V, int P, int head_dim,
                        float rope_base, int32_t* tok_s, int32_t* par_s, int32_t* depth, float2* rope_cs,
                        int32_t* status, bool reset_status, hipStream_t st);
// cs[T][head_dim/2] = (cos, sin) of (P + pos[i]) * base^(-2j/head_dim), evaluated in fp64.
int sx_launch_rope_table(const int32_t* pos, int T, int P, int head_dim, float rope_base, float2* rope_cs, hipStream_t st);
// Per query tile of `nodes_per_tile` consecutive nodes: the sorted union of their ancestors
// (klist[tile][0..kcnt[tile])) and, per node, a bitmask over positions of that list
// (rowmask[node][w], bit b of word w <=> list position 64w+b is an ancestor-or-self of node).
// The tiles cover the query nodes first .. T-1 (rowmask rows indexed by node - first); list entries are node ids.
int sx_launch_qtile_prep(const int32_t* par_s, int T, int nodes_per_tile, int first, int32_t* klist, int32_t* kcnt,
                         unsigned long long* rowmask, hipStream_t st);

// ---- elementwise (elementwise.hip) -----------------------------------------------------------------
int sx_launch_embed(const void* embed, int dtype, const int32_t* tok_s, int T, int d, float* h, hipStream_t st);
int sx_launch_rmsnorm(const float* h, const void* gain, int dtype, int T, int d, float eps, void* x_out,
                      hipStream_t st);
// qkv fp32 [T][Nq+2Nkv] -> q (dtype) [T][Hq][Dh] rotated, k (dtype) [T][Hkv][Dh] rotated, v (dtype)
int sx_launch_rope_split(const float* qkv, const float2* rope_cs, int T, int Hq, int Hkv, int Dh, int dtype,
                         void* q, void* k, void* v, hipStream_t st);
int sx_launch_swiglu_f32(const float* g, const float* u, float* a, size_t n, hipStream_t st);

// ---- fp32 reference-precision path (path_f32.hip) ---------------------------------------------------
// Y[M][N] (+)= X[M][K] W[N][K]^T, all fp32, ldy = row stride of Y.
int sx_launch_gemm_f32(const float* X, const float* W, float* Y, int M, int N, int K, int ldy, bool accumulate,
                       hipStream_t st);
// q and out hold the query nodes first .. T-1 (row = node - first); k_tree / v_tree hold all T nodes.
int sx_launch_tree_attn_f32(const float* q, const float* k_tree, const float* v_tree, const float* k_prefix,
                            const float* v_prefix, const int32_t* par_s, const int32_t* depth, int T, int first, int P,
                            int Hq, int Hkv, int Dh, float* out, hipStream_t st);

// The GEMM kernels address their operands with 32-bit byte offsets from the start of each matrix: every
// operand (X, and each stacked weight matrix on its own) must stay below 4 GiB.
static inline bool sx_operand_fits_u32(long long rows, long long row_bytes) {
  return rows >= 0 && row_bytes >= 0 && (unsigned long long)rows * (unsigned long long)row_bytes < (1ull << 32);
}

// ---- bf16 MFMA path -------------------------------------------------------------------------------
enum { SX_GEMM_STORE = 0, SX_GEMM_RESIDUAL = 1, SX_GEMM_SWIGLU = 2, SX_GEMM_QKV_ROPE = 3 };
// Y = X [W0;W1;W2]^T with n0/n1/n2 rows per segment (modes 0/1, Y fp32 [M][n0+n1+n2]), or
// Y bf16 [M][n0] = silu(X W0^T) * (X W1^T) (mode 2, n1 == n0, n2 == 0).
// Same contract for M <= 128 (narrow tiles; modes store, residual, SwiGLU); sx_launch_gemm_bf16 forwards to it.
int sx_launch_gemm_skinny_bf16(const void* X, const void* W0, const void* W1, const void* W2, int n0, int n1, int n2,
                               void* Y, int M, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st);
// split_ws: see sx_gemm_split_workspace (may be null).
int sx_launch_gemm_bf16(const void* X, const void* W0, const void* W1, const void* W2, int n0, int n1, int n2,
                        void* Y, int M, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st);
// q, k, v (bf16 [M][hq][128], [M][hkv][128], [M][hkv][128]) = rotary(X [Wq;Wk;Wv]^T): the QKV projection with
// the split into heads and the rotation by rope_cs[M][64] = (cos, sin) done in the GEMM's epilogue (v unrotated).
// split_ws (may be null: then no split): sx_gemm_split_workspace() bytes whose first 1 KB is zero before the first
// launch (the kernel leaves it zero); lets the tiles of a launch that fills the chip unevenly, or hardly at all, be
// cut along K and summed by the last workgroup to arrive.
size_t sx_gemm_split_workspace();
int sx_launch_gemm_qkv_rope_bf16(const void* X, const void* Wq, const void* Wk, const void* Wv, int hq, int hkv,
                                 const float2* rope_cs, void* q, void* k, void* v, int M, int K, void* split_ws,
                                 size_t split_ws_bytes, hipStream_t st);
// 4-bit weights (gemm_w4_regs.hip, gemm_skinny_w4.hip, elementwise.hip) -----------------------------------------------
// Stacked 4-bit matrices (n_mats <= 3, every non-final one a multiple of 64 rows), M <= 128, K % 128 == 0: weights
// dequantised in registers on the way to the matrix cores.  Y fp32 [M][ldy].  SX_ERR_SHAPE for other shapes.
int sx_launch_gemm_w4_regs(const void* X, const sx_w4_matrix* mats, const int* ns, int n_mats, int group, float* Y, int ldy,
                           int M, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st);
// The older form (weights dequantised into LDS; M <= 128, K % 64 == 0, one matrix, Y fp32 [M][N] contiguous).
int sx_launch_gemm_skinny_w4(const void* X, const void* qweight, const void* scales, const void* zeros, int group,
                             void* Y, int M, int N, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st);
// W bf16 [N][K] = the dequantised matrix (for the wide GEMM, which is bound by the matrix cores and gains nothing
// from reading fewer bytes).
int sx_launch_dequant_w4(const sx_w4_matrix* m, int N, int K, int group, void* W_bf16, hipStream_t st);
// act bf16 [n][F] = silu(gu[:, :F]) * gu[:, F:], gu fp32 [n][2F]
int sx_launch_swiglu_pair_bf16(const float* gu, int n, int F, void* act, hipStream_t st);
// n int32 zeros (a fill kernel: safe to capture in a graph, unlike a memset node)
int sx_launch_zero_i32(int32_t* p, int n, hipStream_t st);
// q and out hold Tq query nodes; k_tree / v_tree hold all T nodes of the tree; klist rows have stride T.
int sx_launch_tree_attn_bf16(const void* q, const void* k_tree, const void* v_tree, const void* k_prefix,
                             const void* v_prefix, const int32_t* klist, const int32_t* kcnt,
                             const unsigned long long* rowmask, int T, int Tq, int P, int Hq, int Hkv, void* out,
                             void* split_ws, size_t split_ws_bytes, hipStream_t st);
// memory for the partial results when few query rows make the launch share the key tiles among workgroups
// (used only for Tq <= Tq_max; split_ws may be null: no sharing)
size_t sx_tree_attn_split_workspace(int Tq_max, int Hq);
// Query nodes per attention workgroup: 128 rows / G, fewer (down to one wave's 32 rows) when there are so few
// query nodes that the grid would leave most of the chip idle -- the draft model's small batches.  The
// workspace is sized for the smallest value.
static inline int sx_attn_min_nodes_per_tile(int Hq, int Hkv) {
  const int G = Hq / Hkv;
  return G >= 32 ? 1 : 32 / G;
}
static inline int sx_attn_nodes_per_tile(int Hq, int Hkv, int Tq) {
  int npt = 128 / (Hq / Hkv);
  const int lo = sx_attn_min_nodes_per_tile(Hq, Hkv);
  while (npt > lo && ((Tq + npt - 1) / npt) * Hkv < 256) npt /= 2;
  return npt;
}

// ---- the forward itself (verify_tree.hip) -----------------------------------------------------------------
// sx_verify_tree_range with one more knob: keep_status leaves an error that an earlier call recorded in the
// workspace's status word in place (the draft loop's later iterations), instead of starting from SX_OK.
int sx_verify_tree_range_impl(const sx_weights* w, const void* prefix_k, const void* prefix_v, int32_t capacity,
                              int32_t P, const int32_t* tree_tokens, const int32_t* parent_idx, int32_t T, int32_t first,
                              float* logits_out, void* tree_k_out, void* tree_v_out, int32_t tree_capacity,
                              void* workspace, size_t workspace_bytes, bool keep_status, void* stream);

// ---- optional event timing around single launches (prof.hip) -----------------------------------------
enum {
  SX_K_PREP = 1, SX_K_EMBED, SX_K_NORM, SX_K_GEMM_QKV, SX_K_ROPE, SX_K_ATTN, SX_K_GEMM_O, SX_K_GEMM_GATEUP,
  SX_K_GEMM_DOWN, SX_K_GEMM_LMHEAD, SX_K_ROW_TOPK, SX_K_SELECT, SX_K_WALK, SX_K_F32_PATH, SX_K_COMMIT
};
void sx_prof_begin(int tag, hipStream_t st);
void sx_prof_end(hipStream_t st);
