/*
 * specexec_mi.h -- C ABI of the MI355X (gfx950) SpecExec verification hot path.
 *
 * The three main calls follow the paper's problem statement:
 *   sx_verify_tree  = FORWARD(tau, theta_target) of Alg. 1 (function PRECOMPUTE): one target
 *                     forward over the K tree tokens under the merged tree mask of App. D,
 *                     giving the K x vocab matrix "next_probs" (as logits, pre-softmax);
 *   sx_accept_walk  = the loop body of Alg. 1: sample from the cached row of the current
 *                     node, follow the child that carries the sampled token, stop on a miss;
 *   sx_expand_topk  = the selectBest step of Alg. 2 with the nll score of its last lines
 *                     (cumulative log-probability of parent plus log-probability of child,
 *                     App. A Eq. 4-5).
 * A few building blocks (GEMM, tree attention, row top-k) are exported as well so that they
 * can be tested and profiled one by one.
 *
 * General rules
 *   - Every pointer named "device" is GPU global memory owned by the caller; the library
 *     never allocates, frees or keeps a pointer after the call returns.  Scratch memory is
 *     passed in as `workspace`, sized by the matching *_workspace() query, 256-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; nothing synchronises with the host.  Outputs are valid once the
 *     caller has synchronised the stream.
 *   - Return value: SX_OK or a negative sx_status.  Errors that can be seen from the host
 *     (null pointers, bad shapes, short workspace) are returned before anything is
 *     launched.  Errors that live in device data (a parent index out of order, a token id
 *     outside the vocabulary) are recorded by the kernels in the first word of the
 *     workspace; sx_check_status() reads it back (this one call does synchronise).  After
 *     such an error the outputs are unspecified, but no kernel reads or writes out of
 *     bounds because of it.
 *   - Nothing throws or aborts across this boundary.
 */
#ifndef SPECEXEC_MI_H
#define SPECEXEC_MI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sx_status {
  SX_OK = 0,
  SX_ERR_NULL = -1,       /* a required pointer is NULL */
  SX_ERR_SHAPE = -2,      /* a size is out of the supported range (see each call) */
  SX_ERR_WORKSPACE = -3,  /* workspace missing, misaligned or smaller than the query says */
  SX_ERR_DTYPE = -4,      /* cfg.dtype is neither SX_F32 nor SX_BF16 */
  SX_ERR_HIP = -5,        /* a HIP call or kernel launch failed */
  SX_ERR_TREE = -6        /* device data: parent_idx not in {-1} U [0,i), or token outside [0,V) */
} sx_status;

typedef enum sx_dtype { SX_F32 = 0, SX_BF16 = 1 } sx_dtype;

/* Llama-style decoder shape.  Linear layers have no bias; embed and lm_head are untied. */
typedef struct sx_model_cfg {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base; /* 10000 for Llama-2 */
  float rms_eps;   /* 1e-5 */
  int32_t dtype;   /* sx_dtype of weights, prefix KV and tree KV */
} sx_model_cfg;

/* One decoder layer, device pointers, model dtype, row-major [out][in] (y = x W^T). */
typedef struct sx_layer_weights {
  const void *attn_norm; /* [d] */
  const void *wq;        /* [Hq*Dh][d] */
  const void *wk;        /* [Hkv*Dh][d] */
  const void *wv;        /* [Hkv*Dh][d] */
  const void *wo;        /* [d][Hq*Dh] */
  const void *ffn_norm;  /* [d] */
  const void *w_gate;    /* [F][d] */
  const void *w_up;      /* [F][d] */
  const void *w_down;    /* [d][F] */
} sx_layer_weights;

/* A weight matrix W [N][K] stored in 4 bits (Sect. 5: the paper's fastest setting runs its models quantised to
 * 4 bits; it names the quantiser and leaves the storage open -- this is the common group-wise one): codes 0..15,
 * eight per 32-bit word (code j of word i of a row is k = 8 i + j, bits 4j..4j+3); per row and group of `group`
 * consecutive k one bf16 scale and one zero point 0..15 (a byte); w = bf16(scale * (code - zero)), the product exact
 * in fp32 and rounded once.  All device pointers. */
typedef struct sx_w4_matrix {
  const void *qweight; /* uint32 [N][K/8] */
  const void *scales;  /* bf16   [N][K/group] */
  const void *zeros;   /* uint8  [N][K/group] */
} sx_w4_matrix;

/* The seven linear layers of one decoder layer in 4 bits (shapes as in sx_layer_weights). */
typedef struct sx_layer_weights_w4 {
  sx_w4_matrix wq, wk, wv, wo, w_gate, w_up, w_down;
} sx_layer_weights_w4;

typedef struct sx_weights {
  sx_model_cfg cfg;
  const void *embed;              /* device [V][d] */
  const sx_layer_weights *layers; /* HOST array of n_layers structs holding device pointers */
  const void *final_norm;         /* device [d] */
  const void *lm_head;            /* device [V][d] */
  /* Optional 4-bit decoder layers (cfg.dtype must be SX_BF16).  NULL: the bf16 matrices of `layers` are used.
   * Not NULL: HOST array of n_layers structs; every linear layer of the decoder then takes its weights from here
   * (the matrix pointers in `layers` may be NULL; the norm gains still come from there), embed and lm_head stay
   * bf16, activations and all arithmetic are as in the bf16 model with w in place of the bf16 weight.  w4_group:
   * the group size, a power of two >= 64 that divides d_model, Hq*Dh and d_ffn; d_model, Hq*Dh and d_ffn must
   * then be multiples of 128 (64 for calls with at most 128 query nodes). */
  const sx_layer_weights_w4 *layers_w4;
  int32_t w4_group;
} sx_weights;

/* ------------------------------------------------------------------------------------------
 * sx_verify_tree -- Alg. 1, PRECOMPUTE: next_probs := FORWARD(tau, theta_target); App. D:
 * all tree tokens in one pass under a merged attention mask.
 *
 * Node i (0 <= i < T) carries token tree_tokens[i] and hangs under node parent_idx[i]
 * (-1: directly under the last cached prefix token).  Nodes are in topological order,
 * parent_idx[i] < i.  Node i sits at position P + depth(i) for the rotary embedding and
 * attends to all P prefix keys, its tree ancestors and itself.  Query head h reads KV head
 * h / (n_q_heads / n_kv_heads); scores are scaled by 1/sqrt(head_dim).
 *
 *   prefix_k, prefix_v  device [L][P][Hkv][Dh], model dtype; K already rotated at 0..P-1.
 *                       May be NULL when P == 0.
 *   tree_tokens, parent_idx   device int32 [T]
 *   logits_out          device float [T][V]; row i = logits of the token after node i
 *   tree_k_out, tree_v_out    device [L][T][Hkv][Dh], model dtype: the tree's own (rotated) K
 *                       and V, for a later KV commit.  Both NULL = not wanted.
 *
 * Supported shapes.  SX_F32: head_dim even and <= 256, P + 2T <= 15360 (the scores of one node live in LDS).  SX_BF16: head_dim
 * == 128, n_q_heads/n_kv_heads in {1,2,4,8}, d_model, Hq*Dh and d_ffn multiples of 64.
 * T >= 1, P >= 0, T <= 16384.  The bf16 GEMM kernels address each operand with 32-bit byte offsets, so
 * every matrix on its own must be smaller than 4 GiB: T*d_model*2, T*d_ffn*2, vocab*d_model*2 (embed is
 * exempt), d_ffn*d_model*2 and Hq*Dh*d_model*2 bytes all < 2^32, else SX_ERR_SHAPE.  In SX_BF16 the tensors a bf16 model materialises (normed
 * activations, q, k, v, attention output, SwiGLU output) are rounded to bf16; the residual
 * stream, softmax and norm statistics, and all accumulation are fp32.
 * ---------------------------------------------------------------------------------------- */
size_t sx_verify_tree_workspace(const sx_model_cfg *cfg, int32_t P, int32_t T);
/* Workspace of the same calls when w->layers_w4 is set (4-bit decoder layers, Sect. 5).  With at most 128 query
 * nodes per call (the draft model's batches) the linear layers read the 4-bit weights directly -- dequantised in
 * registers on the way to the matrix cores, the regime where fewer weight bytes mean less time -- and this equals
 * sx_verify_tree_workspace.  With more query nodes the product is bound by the matrix cores, not by weight bytes:
 * each layer's seven matrices are then expanded to bf16 once per call into a scratch behind the ordinary
 * workspace (one layer's worth: 1.7 GB for a 70B-shaped layer) and the bf16 kernels run on that copy. */
size_t sx_verify_tree_w4_workspace(const sx_model_cfg *cfg, int32_t P, int32_t T);
int sx_verify_tree(const sx_weights *w, const void *prefix_k, const void *prefix_v, int32_t P,
                   const int32_t *tree_tokens, const int32_t *parent_idx, int32_t T,
                   float *logits_out, void *tree_k_out, void *tree_v_out, void *workspace,
                   size_t workspace_bytes, void *stream);

/* Same as sx_verify_tree with the prefix held in a cache that has room to grow: prefix_k and
 * prefix_v are device [L][capacity][Hkv][Dh] of which rows [0, P) of every layer are valid
 * (capacity >= P).  sx_verify_tree is this call with capacity == P. */
int sx_verify_tree_cached(const sx_weights *w, const void *prefix_k, const void *prefix_v,
                          int32_t capacity, int32_t P, const int32_t *tree_tokens,
                          const int32_t *parent_idx, int32_t T, float *logits_out, void *tree_k_out,
                          void *tree_v_out, void *workspace, size_t workspace_bytes, void *stream);

/* The same forward for the nodes first .. T-1 only, of a tree whose nodes 0 .. first-1 went through an
 * earlier call (Alg. 2: "forward(batch, theta_draft) ... attend to past tokens": a tree that grows
 * by a batch of nodes per step).  tree_k_out / tree_v_out are device [L][tree_capacity][Hkv][Dh]
 * (tree_capacity >= T) and persistent across calls: rows [0, first) of every layer are read as keys and
 * values, rows [first, T) are written.  They are required when first > 0.  tree_tokens and parent_idx
 * describe all T nodes (indices are global); logits_out is device float [T - first][V], row i for node
 * first + i.  Workspace as for sx_verify_tree(P, T).  sx_verify_tree_cached is this call with first = 0
 * and tree_capacity = T.  Every call starts the workspace's status word afresh: check it after each
 * call of a sequence that grows one tree. */
int sx_verify_tree_range(const sx_weights *w, const void *prefix_k, const void *prefix_v,
                         int32_t capacity, int32_t P, const int32_t *tree_tokens,
                         const int32_t *parent_idx, int32_t T, int32_t first, float *logits_out,
                         void *tree_k_out, void *tree_v_out, int32_t tree_capacity, void *workspace,
                         size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * sx_accept_walk -- Alg. 1, main loop: p_target := cache[x]; x_next ~ sample(p_target).
 *
 * Starts at node 0 (which must be the only root), and repeats: draw a token from
 * warp(softmax(logits[cur] / temperature), top_p) with the uniform u(seed, pos0 +
 * depth(cur) + 1); emit it; move to the lowest-index child of cur that carries it; stop
 * when there is none.  temperature == 0 means greedy (lowest-id argmax).  The nucleus is
 * the shortest prefix, in (probability descending, id ascending) order, whose mass reaches
 * top_p; the draw is the inverse CDF over the nucleus in id order at u * mass(nucleus).
 * u(seed, pos) = top 24 bits of SplitMix64's mixer applied to seed + (pos+1)*0x9E3779B97F4A7C15.
 * pos0 is the absolute position of node 0 (= P), so the stream of uniforms is the one
 * sequential decoding would use (Sect. 4.1, seed-exact equivalence).
 *
 *   logits        device float [T][V]
 *   draft_probs   NULL: the walk above (SpecExec accepts with the target probability alone).
 *                 Not NULL: device float [T][V], row i = the distribution the children of node i were
 *                 drawn from (independent draws; equal tokens may be separate children).  The call then
 *                 runs the comparison system of Sect. 4.1, speculative decoding's acceptance with
 *                 probability P_target(x) / P_draft(x) capped at one, over the tree: with p the warped
 *                 target distribution of the current node (nucleus renormalised) and q its draft row,
 *                 the children are tried in index order, the j-th accepted when r_j q[x] < p[x]; a
 *                 rejection replaces p by the renormalised positive part of p - q; after the last
 *                 rejection the token is drawn from what p has become (inverse CDF in id order) and the
 *                 walk ends.  r_j = u(seed + (j+1)*0xD6E8FEB86659FD93, position): one uniform per
 *                 decision.  The emitted tokens follow the target's warped distribution; they are not
 *                 seed-for-seed those of sequential sampling (the paper says as much of this baseline).
 *   path_out      device int32 [T]: visited nodes, path_out[0] == 0
 *   tokens_out    device int32 [T]: tokens_out[s] = token sampled at path_out[s]
 *   n_out         device int32 [1]: number of entries written to both (>= 1); the number of
 *                 accepted draft tokens is n_out - 1, the last token is the one that left the tree
 * Supported: 1 <= V <= 131072, T >= 1, 0 < top_p <= 1, temperature >= 0.
 * ---------------------------------------------------------------------------------------- */
size_t sx_accept_walk_workspace(int32_t T, int32_t V);
int sx_accept_walk(const float *logits, const float *draft_probs, const int32_t *tree_tokens,
                   const int32_t *parent_idx, int32_t T, int32_t V, float temperature, float top_p,
                   uint64_t seed, int32_t pos0, int32_t *path_out, int32_t *tokens_out,
                   int32_t *n_out, void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * sx_expand_topk -- Alg. 2: topk := selectBest(batch, probs, tau, K), scored by
 * nll := -log p_prefix - log p_i.
 *
 * For each of N expanded nodes: log-softmax of its V draft logits and its k best tokens
 * (value descending, token id ascending on ties).  Then the B best of the N*k candidates by
 * cum_logp[row] + logp (fp32), ties to the lower flat index row*k + rank.  Outputs are in
 * that order.
 *
 *   logits     device float [N][V];  cum_logp  device float [N]
 *   out_row, out_token   device int32 [B];  out_cum_logp  device float [B]
 *   n_out      device int32 [1] = min(B, N*k)
 * Supported: 1 <= k <= min(V, 256), V <= 131072, 1 <= B <= 8192, N >= 1, N*k < 2^31.
 * ---------------------------------------------------------------------------------------- */
size_t sx_expand_topk_workspace(int32_t N, int32_t V, int32_t k, int32_t B);
int sx_expand_topk(const float *logits, const float *cum_logp, int32_t N, int32_t V, int32_t k,
                   int32_t B, int32_t *out_row, int32_t *out_token, float *out_cum_logp,
                   int32_t *n_out, void *workspace, size_t workspace_bytes, void *stream);

/* sx_expand_topk for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, results and kernels as
 * sx_expand_topk, but the N*k candidates are staged in a fixed device array that is part of the library
 * (3 x 4 bytes per candidate, 768 KB in all, held by every GPU the library runs on until the process ends).
 * Limit: N * k <= SX_EXPAND_STATIC_MAX_CANDIDATES (the paper-sized expansion step, 2048 nodes x 32
 * tokens, just fits); larger calls return SX_ERR_SHAPE and belong to sx_expand_topk.  The call allocates
 * and frees nothing and uses no allocating library routine; the first call on a device looks up that
 * device's copy of the array (make the device current before calling).  All calls on one GPU share the
 * array: calls that overlap on one GPU (two streams, two threads) race; calls on one stream are ordered
 * and need no clearing between them, since every entry a call reads it has written itself. */
#define SX_EXPAND_STATIC_MAX_CANDIDATES 65536
int sx_expand_topk_static(const float *logits, const float *cum_logp, int32_t N, int32_t V, int32_t k,
                          int32_t B, int32_t *out_row, int32_t *out_token, float *out_cum_logp,
                          int32_t *n_out, void *stream);

/* ------------------------------------------------------------------------------------------
 * sx_commit_kv -- Alg. 1, end of the loop body: the tokens the walk accepted join the
 * context.  Copies the keys and values of the visited nodes into the prefix cache:
 * cache[l][P + s] = tree[l][path[s]] for every layer l and s < *n.  The node visited at step s
 * has depth s, so the key it carries was rotated at position P + s, the position it now takes
 * in the prefix.  The token sampled last (tokens_out[*n - 1] of the walk) is not in the cache:
 * it is the root of the next round's tree, to be verified at position P + *n.
 *
 *   cache_k, cache_v  device [L][capacity][Hkv][Dh], model dtype; rows [0, P) valid before,
 *                     [0, P + *n) after.  Requires P + T <= capacity (checked on the host).
 *   tree_k, tree_v    device [L][T][Hkv][Dh], as written by sx_verify_tree
 *   path, n           device int32 [T] and [1]: path_out and n_out of sx_accept_walk (read on
 *                     the device: no host round trip between the walk and the commit)
 * ---------------------------------------------------------------------------------------- */
int sx_commit_kv(const sx_model_cfg *cfg, void *cache_k, void *cache_v, int32_t capacity, int32_t P,
                 const void *tree_k, const void *tree_v, int32_t T, const int32_t *path,
                 const int32_t *n, void *stream);

/* One round of Alg. 1's loop on a stream, without host synchronisation: sx_verify_tree_cached,
 * sx_accept_walk (uniforms keyed by absolute position, pos0 = P) and sx_commit_kv.  Arguments as
 * in those calls; tree_k and tree_v are required (device [L][T][Hkv][Dh] scratch or output).
 * After the stream has run: *n_out accepted nodes were appended to the cache, the new prefix
 * length is P + *n_out and the next tree is rooted at tokens_out[*n_out - 1].  workspace: at
 * least sx_specexec_round_workspace(cfg, P, T) bytes, 256-byte aligned. */
size_t sx_specexec_round_workspace(const sx_model_cfg *cfg, int32_t P, int32_t T);
int sx_specexec_round(const sx_weights *w, void *cache_k, void *cache_v, int32_t capacity, int32_t P,
                      const int32_t *tree_tokens, const int32_t *parent_idx, int32_t T,
                      float temperature, float top_p, uint64_t seed, float *logits, void *tree_k,
                      void *tree_v, int32_t *path_out, int32_t *tokens_out, int32_t *n_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * sx_draft_tree -- Alg. 2, PARALLEL SSSP FOR DRAFTING: createDraftTree(x, theta_draft, K, D, B).
 *
 * Builds the tree of likely continuations of the root token with the draft model `w`, entirely on
 * the stream (no host synchronisation between iterations).  Each of the D iterations pops the up
 * to B best candidates from the priority queue (ordered by cumulative log-probability, ties to the
 * candidate that entered first; the queue is first cut to its K best), makes those above the
 * threshold tree nodes (threshold: the K-th best score in the tree once it holds K nodes), runs the
 * draft model over them (they attend to the prefix and to their tree ancestors), keeps per node its k
 * most probable next tokens and of those the min(K, B k) best by cumulative log-probability, and
 * inserts them into the queue.  Finally the tree is cut to its K best nodes.
 *
 *   prefix_k, prefix_v  the DRAFT model's cache, device [L][capacity][Hkv][Dh], rows [0, P) valid
 *   root_token          device int32 [1]: the last accepted token (e.g. tokens_out[n-1] of the walk)
 *   tree_tokens_out, parent_out   device int32 [K]; cum_logp_out device float [K]; n_out device
 *                       int32 [1] (1 <= n <= K).  Nodes in order of insertion (parents before
 *                       children, node 0 = root with parent -1): the input sx_verify_tree expects.
 * Supported: D * B <= 16384, k <= 256 (k is clamped to the vocabulary), min(K, B k) <= 8192,
 * K + min(K, B k) <= 16384, and the model shapes of sx_verify_tree with T = D * B.  A draft model with 4-bit
 * layers (w->layers_w4) needs B <= 128 (its batches then read the 4-bit weights directly; no scratch copy).
 * workspace: sx_draft_tree_workspace bytes, 256-byte aligned; sx_check_status on it reports an error of
 * any of the D forward passes (the first pass resets the status word, the later ones leave an error in place).
 * ---------------------------------------------------------------------------------------- */
size_t sx_draft_tree_workspace(const sx_model_cfg *cfg, int32_t P, int32_t K, int32_t D, int32_t B,
                               int32_t k);
int sx_draft_tree(const sx_weights *w, const void *prefix_k, const void *prefix_v, int32_t capacity,
                  int32_t P, const int32_t *root_token, int32_t K, int32_t D, int32_t B, int32_t k,
                  int32_t *tree_tokens_out, int32_t *parent_out, float *cum_logp_out, int32_t *n_out,
                  void *workspace, size_t workspace_bytes, void *stream);

/* Reads the device-side status word of a workspace used by one of the calls above.
 * Synchronises `stream`.  Returns SX_OK, SX_ERR_TREE, or SX_ERR_HIP. */
int sx_check_status(const void *workspace, void *stream);

const char *sx_status_string(int status);
int sx_version(void);

/* ------------------------------------------------------------------------------------------
 * Building blocks (the kernels the three calls are made of), exported for tests/profiling.
 * ---------------------------------------------------------------------------------------- */

/* First half of sx_expand_topk (Alg. 2, probs -> per-row best tokens): row-wise
 * log-softmax + top-k.  topk_logp device float [N][k], topk_idx device int32 [N][k]. */
int sx_row_logsoftmax_topk(const float *logits, int32_t N, int32_t V, int32_t k,
                           float *topk_logp, int32_t *topk_idx, void *stream);

/* Y = X W^T with bf16 operands and fp32 accumulation on the matrix cores; the linear layers
 * of the decoder forward (Alg. 1, FORWARD).  X device bf16 [M][K] row-major, W device bf16
 * [N][K] row-major, K % 64 == 0; M*K*2 and N*K*2 bytes each below 4 GiB (SX_ERR_SHAPE otherwise).  mode 0: Y float [M][N] = acc;  mode 1: Y float [M][N] += acc
 * (residual add);  mode 2: W2 is a second [N][K] matrix and Y bf16 [M][N] =
 * bf16(silu(X W^T) * (X W2^T)) (SwiGLU).  W2 is ignored in modes 0 and 1. */
int sx_gemm_bf16(const void *X, const void *W, const void *W2, void *Y, int32_t M, int32_t N,
                 int32_t K, int32_t mode, void *stream);
/* The same product with memory for partial sums, as the forward calls it: where the output tiles (256 x 256)
 * are fewer than half the compute units, or their last round would fill at most half of them, those tiles
 * are cut along K among several workgroups; the parts are added in a fixed order, so results repeat bit for
 * bit.  workspace: NULL (then exactly sx_gemm_bf16), or device memory of sx_gemm_bf16_workspace() bytes,
 * 256-byte aligned (SX_ERR_WORKSPACE otherwise), whose first 1024 bytes are zero before the first call (every call
 * leaves them zero); caller-owned; calls that share a workspace must not overlap. */
size_t sx_gemm_bf16_workspace(void);
int sx_gemm_bf16_ws(const void *X, const void *W, const void *W2, void *Y, int32_t M, int32_t N,
                    int32_t K, int32_t mode, void *workspace, size_t workspace_bytes, void *stream);

/* QKV projection of the decoder layer (Alg. 1, FORWARD) with the rotary embedding applied in the
 * GEMM's epilogue, head_dim 128: q_out device bf16 [T][n_q_heads][128], k_out and v_out device
 * bf16 [T][n_kv_heads][128]; q and k are rotated by the angle of positions[i] (device int32 [T]:
 * prefix length + tree depth of node i), half-split pairing (element j with j + 64), v is not.
 * X device bf16 [T][d_model], Wq bf16 [n_q_heads*128][d_model], Wk, Wv bf16
 * [n_kv_heads*128][d_model], d_model % 64 == 0.  workspace: device, 256-byte aligned, at least
 * sx_qkv_rope_workspace(T, n_q_heads, n_kv_heads) bytes (the cos/sin table and, where the output
 * tiles fill the chip unevenly, partial sums of the tiles that are cut along K); caller-owned,
 * contents need not be initialised. */
size_t sx_qkv_rope_workspace(int32_t T, int32_t n_q_heads, int32_t n_kv_heads);
int sx_qkv_rope_bf16(const void *X, const void *Wq, const void *Wk, const void *Wv, int32_t T,
                     int32_t d_model, int32_t n_q_heads, int32_t n_kv_heads,
                     const int32_t *positions, float rope_base, void *q_out, void *k_out,
                     void *v_out, void *workspace, size_t workspace_bytes, void *stream);

/* Y = X W^T for a small batch (M <= 128) with 4-bit group-quantised weights (Sect. 5: the paper's fastest
 * setting runs the models quantised to 4 bits): dequantisation in registers on the way to the matrix cores.
 * X device bf16 [M][K]; qweight device uint32 [N][K/8], eight 4-bit codes per word, code j of word i of a
 * row being k = 8 i + j in bits 4j..4j+3; scales device bf16 [N][K/group]; zeros device uint8 [N][K/group],
 * values 0..15; w = bf16(scale * (code - zero)).  group a power of two >= 64, K % group == 0.  mode 0: Y float
 * [M][N] = X W^T; mode 1: Y += X W^T.  workspace: NULL, or device memory of sx_gemm_w4a16_workspace()
 * bytes, 256-byte aligned (lets launches with few column tiles cut K among workgroups); caller-owned. */
size_t sx_gemm_w4a16_workspace(void);
int sx_gemm_w4a16_bf16(const void *X, const void *qweight, const void *scales, const void *zeros, void *Y,
                       int32_t M, int32_t N, int32_t K, int32_t group, int32_t mode, void *workspace,
                       size_t workspace_bytes, void *stream);

/* Tree attention alone (App. D merged mask), bf16: q device bf16 [T][Hq][128], tree K/V
 * [T][Hkv][128], prefix K/V [P][Hkv][128], out device bf16 [T][Hq][128]; n_q_heads/n_kv_heads in {1,2,4,8}.  workspace sized by
 * sx_tree_attention_workspace. */
size_t sx_tree_attention_workspace(int32_t T, int32_t n_q_heads, int32_t n_kv_heads);
int sx_tree_attention_bf16(const void *q, const void *k_tree, const void *v_tree,
                           const void *k_prefix, const void *v_prefix, const int32_t *parent_idx,
                           int32_t T, int32_t P, int32_t n_q_heads, int32_t n_kv_heads, void *out,
                           void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------
 * Optional kernel timing for callers that measure (not part of the method).  Between
 * sx_profile_enable and sx_profile_disable the three calls above record a pair of HIP events
 * on the caller's stream around each kernel launch, up to max_records pairs (events are
 * created here, once).  sx_profile_read waits for the recorded events, returns for each pair
 * its kernel class (sx_kernel_class) and elapsed milliseconds, and clears the log.
 * One process-wide log; not thread-safe.
 * ---------------------------------------------------------------------------------------- */
typedef enum sx_kernel_class {
  SX_KC_PREP = 1, SX_KC_EMBED, SX_KC_NORM, SX_KC_GEMM_QKV, SX_KC_ROPE, SX_KC_ATTN, SX_KC_GEMM_O,
  SX_KC_GEMM_GATEUP, SX_KC_GEMM_DOWN, SX_KC_GEMM_LMHEAD, SX_KC_ROW_TOPK, SX_KC_SELECT, SX_KC_WALK,
  SX_KC_F32_PATH, SX_KC_COMMIT
} sx_kernel_class;
int sx_profile_enable(int32_t max_records);
/* Restricts the timing to launches of one kernel class (0: all classes, the default): two event records per
 * launch cost about 8 us of stream time, which adds up over the ~500 launches of a 80-layer forward. */
int sx_profile_select(int32_t kernel_class);
int sx_profile_disable(void);
int sx_profile_read(int32_t *classes, float *milliseconds, int32_t capacity, int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* SPECEXEC_MI_H */
