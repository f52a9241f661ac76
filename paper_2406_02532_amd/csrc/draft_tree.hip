// Draft-side tree construction (Alg. 2, PARALLEL SSSP FOR DRAFTING: createDraftTree) on the device, without a
// host round trip between iterations.
//
// The priority queue H is a list of candidate ids; the candidates themselves (token, parent node, cumulative
// log-probability) live in an append-only log, and a candidate's id is the order in which it entered, which
// is also the tie-break among equal scores.  One iteration is four launches on the stream:
//   take    (one workgroup)  sort H by (score descending, id ascending), cut it to its K best (trim), pop up
//                            to B of them: those above the threshold become tree nodes in slots
//                            [base, base + B), the others are dropped; update the threshold (once the tree
//                            has K nodes: the K-th best score in it);
//   forward (sx_verify_tree_range) the draft model over the B new slots, which attend to the prefix and to
//                            their ancestors through the persistent tree K/V;
//   expand  (sx_expand_topk) per node its k best next tokens, of those the min(K, B k) best by cumulative score;
//   merge   (one workgroup)  append them to the log and to H.
// Shapes are fixed: an iteration always carries B slots; slots it does not fill are dead (score -inf, token 0,
// hung under node 0) and cost a wasted row of the forward, nothing else.  After D iterations `finish` cuts the
// tree to its K best nodes and renumbers parents (trim(tau, K)).
#include "kernels.h"
#include "../../include/specexec_mi.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kSortCap = 16384;  // candidates the take kernel can order (LDS: 128 KB of 64-bit keys)

struct DraftState {  // device scalars
  int hn[2];         // size of H (ping-pong)
  int logn;          // candidates logged so far
  int n_alive;       // tree nodes so far
  float thr;         // a candidate joins the tree only if its score is above this (-T of Alg. 2)
};

struct DraftBufs {
  int32_t *tok, *par, *alive;  // tree slots [S]
  float* cum;                  // [S] cumulative log-probability of the slot's node (-inf: dead)
  int32_t *cand_tok, *cand_par;
  float* cand_score;           // candidate log [logcap]
  uint32_t* H[2];              // candidate ids [hcap]
  DraftState* state;
};

__global__ void draft_init_kernel(DraftBufs b, const int32_t* root_token) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    b.cand_tok[0] = root_token[0];
    b.cand_par[0] = -1;
    b.cand_score[0] = 0.f;
    b.H[0][0] = 0u;
    b.state->hn[0] = 1;
    b.state->hn[1] = 0;
    b.state->logn = 1;
    b.state->n_alive = 0;
    b.state->thr = -__builtin_huge_valf();
  }
}

// K-th largest of the order keys key(i), i < n (n >= K >= 1), by bitwise search; every lane gets the result.
template <typename KeyFn>
__device__ unsigned kth_largest_key(int n, int K, KeyFn key, int* red) {
  unsigned T = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const unsigned trial = T | (1u << bit);
    int c = 0;
    for (int i = threadIdx.x; i < n; i += kThreads) c += key(i) >= trial ? 1 : 0;
    if (block_sum_i<kThreads / 64>(c, red) >= K) T = trial;
  }
  return T;
}

__global__ __launch_bounds__(kThreads) void draft_take_kernel(DraftBufs b, int cur, int base, int B, int K) {
  __shared__ unsigned long long keys[kSortCap];
  __shared__ int red[16];
  __shared__ int s_b;
  const int tid = threadIdx.x;
  const uint32_t* Hin = b.H[cur];
  uint32_t* Hout = b.H[cur ^ 1];
  const int n = min(b.state->hn[cur], kSortCap);
  const float thr = b.state->thr;
  // read here, ahead of every barrier: lane 0 overwrites the state at the end of the kernel, and a wave that
  // read it only then could see the new value and take the other side of the (barrier-holding) branch below
  const int alive_before = b.state->n_alive;
  const int np2 = next_pow2(n < 2 ? 2 : n);
  for (int i = tid; i < np2; i += kThreads) {
    unsigned long long k = ~0ull;
    if (i < n) {
      const uint32_t id = Hin[i];
      k = ((unsigned long long)(~f32_order_key(b.cand_score[id])) << 32) | id;
    }
    keys[i] = k;
  }
  if (tid == 0) s_b = 0;
  __syncthreads();
  block_bitonic_sort_u64<kThreads>(keys, np2);
  const int heap = min(n, K);        // trim(H, K)
  const int pops = min(B, heap);     // extractMin, B times
  // popped candidates above the threshold are a prefix of the order
  for (int i = tid; i < pops; i += kThreads) {
    const uint32_t id = (uint32_t)(keys[i] & 0xFFFFFFFFull);
    if (b.cand_score[id] > thr) atomicAdd(&s_b, 1);
  }
  __syncthreads();
  const int nb = s_b;
  for (int i = tid; i < B; i += kThreads) {
    const int slot = base + i;
    if (i < nb) {
      const uint32_t id = (uint32_t)(keys[i] & 0xFFFFFFFFull);
      b.tok[slot] = b.cand_tok[id];
      b.par[slot] = b.cand_par[id];
      b.cum[slot] = b.cand_score[id];
      b.alive[slot] = 1;
    } else {
      b.tok[slot] = 0;
      b.par[slot] = slot == 0 ? -1 : 0;
      b.cum[slot] = -__builtin_huge_valf();
      b.alive[slot] = 0;
    }
  }
  for (int i = pops + tid; i < heap; i += kThreads) Hout[i - pops] = (uint32_t)(keys[i] & 0xFFFFFFFFull);
  __syncthreads();  // the slots just written are read below
  const int alive_now = alive_before + nb;
  float new_thr = thr;
  if (alive_now >= K) {  // T := K-th best cumulative log-probability in the tree
    const float* cum = b.cum;
    const unsigned kk = kth_largest_key(base + B, K, [&](int i) { return f32_order_key(cum[i]); }, red);
    new_thr = f32_from_order_key(kk);
  }
  if (tid == 0) {
    b.state->hn[cur ^ 1] = heap - pops;
    b.state->n_alive = alive_now;
    b.state->thr = new_thr;
  }
}

// appends the finite-score picks of sx_expand_topk (sorted by score, so they are a prefix) to the log and to H
__global__ __launch_bounds__(kThreads) void draft_merge_kernel(DraftBufs b, int cur, int base, const int32_t* sel_row,
                                                               const int32_t* sel_tok, const float* sel_score,
                                                               const int32_t* sel_n, int logcap, int hcap) {
  __shared__ int red[16];
  const int tid = threadIdx.x;
  const int n = sel_n[0];
  int c = 0;
  for (int j = tid; j < n; j += kThreads) c += sel_score[j] > -__builtin_huge_valf() ? 1 : 0;
  int nfin = block_sum_i<kThreads / 64>(c, red);
  const int logn = b.state->logn, hn = b.state->hn[cur];
  nfin = min(nfin, min(logcap - logn, hcap - hn));  // cannot happen with the sizes the host checked
  for (int j = tid; j < nfin; j += kThreads) {
    const int id = logn + j;
    b.cand_tok[id] = sel_tok[j];
    b.cand_par[id] = base + sel_row[j];
    b.cand_score[id] = sel_score[j];
    b.H[cur][hn + j] = (uint32_t)id;
  }
  __syncthreads();
  if (tid == 0) {
    b.state->logn = logn + nfin;
    b.state->hn[cur] = hn + nfin;
  }
}

// trim(tau, K): the K best alive slots by (score descending, slot ascending), in slot order, parents renumbered
__global__ __launch_bounds__(kThreads) void draft_finish_kernel(DraftBufs b, int S, int K, int32_t* out_tok,
                                                                int32_t* out_par, float* out_cum, int32_t* out_n,
                                                                int32_t* newidx) {
  __shared__ int red[16];
  __shared__ int s_wave[kThreads / 64];
  __shared__ int s_carry;
  const int tid = threadIdx.x;
  const float* cum = b.cum;
  const int alive = b.state->n_alive;
  const int keep = min(alive, K);
  unsigned kk = 0;
  int ties_to_take = 0;
  if (alive > K) {
    kk = kth_largest_key(S, K, [&](int i) { return b.alive[i] ? f32_order_key(cum[i]) : 0u; }, red);
    int c = 0;
    for (int i = tid; i < S; i += kThreads) c += (b.alive[i] && f32_order_key(cum[i]) > kk) ? 1 : 0;
    ties_to_take = K - block_sum_i<kThreads / 64>(c, red);  // of the slots equal to the K-th score, the first ones
  }
  if (tid == 0) s_carry = 0;
  __syncthreads();
  // one sweep in slot order, a chunk of kThreads slots at a time: running counts of kept slots and of ties seen
  int ties_seen_total = 0;  // identical in all lanes
  for (int c0 = 0; c0 < S; c0 += kThreads) {
    const int i = c0 + tid;
    bool is_tie = false, sel = false;
    if (i < S && b.alive[i]) {
      if (alive <= K) sel = true;
      else {
        const unsigned k = f32_order_key(cum[i]);
        sel = k > kk;
        is_tie = k == kk;
      }
    }
    // rank of this lane's tie among the ties of the chunk
    const unsigned long long tb = __builtin_amdgcn_ballot_w64(is_tie);
    const int lane = tid & 63, wv = tid >> 6;
    int tie_rank = __builtin_popcountll(tb & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wv] = __builtin_popcountll(tb);
    __syncthreads();
    int chunk_ties = 0;
    for (int w = 0; w < kThreads / 64; ++w) {
      if (w < wv) tie_rank += s_wave[w];
      chunk_ties += s_wave[w];
    }
    __syncthreads();
    if (is_tie && ties_seen_total + tie_rank < ties_to_take) sel = true;
    ties_seen_total += chunk_ties;
    // position of the kept slots
    const unsigned long long sb = __builtin_amdgcn_ballot_w64(sel);
    int pos = __builtin_popcountll(sb & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wv] = __builtin_popcountll(sb);
    __syncthreads();
    int chunk_sel = 0;
    for (int w = 0; w < kThreads / 64; ++w) {
      if (w < wv) pos += s_wave[w];
      chunk_sel += s_wave[w];
    }
    const int carry = s_carry;
    __syncthreads();
    if (i < S) newidx[i] = sel ? carry + pos : -1;
    if (tid == 0) s_carry = carry + chunk_sel;
    __syncthreads();
  }
  // parents come before their children in slot order, and a kept node's parent is kept (its score is not lower)
  for (int i = tid; i < S; i += kThreads) {
    const int ni = newidx[i];
    if (ni >= 0) {
      out_tok[ni] = b.tok[i];
      out_cum[ni] = cum[i];
      const int p = b.par[i];
      out_par[ni] = p < 0 ? -1 : newidx[p];
    }
  }
  if (tid == 0) out_n[0] = keep;
}

struct DraftLayout {
  DraftBufs b;
  float* logits;
  int32_t *sel_row, *sel_tok, *sel_n, *newidx;
  float* sel_score;
  void *expand_ws, *tree_k, *tree_v, *verify_ws;
  size_t expand_ws_bytes, verify_ws_bytes, bytes;
  int S, logcap, hcap, ksel, bsel;
};

bool draft_shape_ok(const sx_model_cfg& c, int P, int K, int D, int B, int k) {
  if (K < 1 || D < 1 || B < 1 || k < 1) return false;
  const long long S = (long long)D * B;
  if (S > 16384) return false;
  const int ksel = k < c.vocab ? k : c.vocab;
  if (ksel > 256) return false;
  const long long bsel = (long long)B * ksel < K ? (long long)B * ksel : K;
  if (bsel > 8192 || (long long)K + bsel > kSortCap) return false;
  return sx_verify_tree_workspace(&c, P, (int)S) != 0;
}

DraftLayout draft_carve(const sx_model_cfg& c, int P, int K, int D, int B, int k, void* ws) {
  SxCarver cv(ws, 0);
  DraftLayout L;
  L.S = D * B;
  L.ksel = k < c.vocab ? k : c.vocab;
  L.bsel = (long long)B * L.ksel < K ? B * L.ksel : K;
  L.logcap = 1 + D * L.bsel;
  L.hcap = K + L.bsel;
  const size_t es = c.dtype == SX_BF16 ? 2 : 4;
  // the forward's workspace comes first: its status word is then the one sx_check_status reads
  L.verify_ws_bytes = sx_verify_tree_workspace(&c, P, L.S);
  L.verify_ws = cv.take<char>(L.verify_ws_bytes);
  L.b.tok = cv.take<int32_t>(L.S);
  L.b.par = cv.take<int32_t>(L.S);
  L.b.alive = cv.take<int32_t>(L.S);
  L.b.cum = cv.take<float>(L.S);
  L.b.cand_tok = cv.take<int32_t>(L.logcap);
  L.b.cand_par = cv.take<int32_t>(L.logcap);
  L.b.cand_score = cv.take<float>(L.logcap);
  L.b.H[0] = cv.take<uint32_t>(L.hcap);
  L.b.H[1] = cv.take<uint32_t>(L.hcap);
  L.b.state = cv.take<DraftState>(1);
  L.newidx = cv.take<int32_t>(L.S);
  L.logits = cv.take<float>((size_t)B * c.vocab);
  L.sel_row = cv.take<int32_t>(L.bsel);
  L.sel_tok = cv.take<int32_t>(L.bsel);
  L.sel_score = cv.take<float>(L.bsel);
  L.sel_n = cv.take<int32_t>(1);
  L.expand_ws_bytes = sx_expand_topk_workspace(B, c.vocab, L.ksel, L.bsel);
  L.expand_ws = cv.take<char>(L.expand_ws_bytes);
  const size_t kv = (size_t)c.n_layers * L.S * c.n_kv_heads * c.head_dim * es;
  L.tree_k = cv.take<char>(kv);
  L.tree_v = cv.take<char>(kv);
  L.bytes = cv.off;
  return L;
}

}  // namespace

extern "C" size_t sx_draft_tree_workspace(const sx_model_cfg* cfg, int32_t P, int32_t K, int32_t D, int32_t B,
                                          int32_t k) {
  if (!cfg || !draft_shape_ok(*cfg, P, K, D, B, k)) return 0;
  return draft_carve(*cfg, P, K, D, B, k, nullptr).bytes;
}

extern "C" int sx_draft_tree(const sx_weights* w, const void* prefix_k, const void* prefix_v, int32_t capacity, int32_t P,
                             const int32_t* root_token, int32_t K, int32_t D, int32_t B, int32_t k,
                             int32_t* tree_tokens_out, int32_t* parent_out, float* cum_logp_out, int32_t* n_out,
                             void* workspace, size_t workspace_bytes, void* stream) {
  if (!w || !root_token || !tree_tokens_out || !parent_out || !cum_logp_out || !n_out) return SX_ERR_NULL;
  const sx_model_cfg& c = w->cfg;
  if (!draft_shape_ok(c, P, K, D, B, k) || capacity < P) return SX_ERR_SHAPE;
  if (w->layers_w4 && B > 128) return SX_ERR_SHAPE;  // wider batches of a 4-bit model would need the bf16 scratch copy
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return SX_ERR_WORKSPACE;
  const DraftLayout L = draft_carve(c, P, K, D, B, k, workspace);
  if (workspace_bytes < L.bytes) return SX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;

  draft_init_kernel<<<1, 64, 0, st>>>(L.b, root_token);
  SX_LAUNCH_CHECK();
  int cur = 0;
  for (int d = 0; d < D; ++d) {
    const int base = d * B;
    draft_take_kernel<<<1, kThreads, 0, st>>>(L.b, cur, base, B, K);
    SX_LAUNCH_CHECK();
    cur ^= 1;
    // the first iteration resets the status word, the later ones keep what an earlier one recorded
    SX_TRY(sx_verify_tree_range_impl(w, prefix_k, prefix_v, capacity, P, L.b.tok, L.b.par, base + B, base, L.logits,
                                     L.tree_k, L.tree_v, L.S, L.verify_ws, L.verify_ws_bytes, d > 0, st));
    SX_TRY(sx_expand_topk(L.logits, L.b.cum + base, B, c.vocab, L.ksel, L.bsel, L.sel_row, L.sel_tok, L.sel_score,
                          L.sel_n, L.expand_ws, L.expand_ws_bytes, st));
    draft_merge_kernel<<<1, kThreads, 0, st>>>(L.b, cur, base, L.sel_row, L.sel_tok, L.sel_score, L.sel_n, L.logcap,
                                               L.hcap);
    SX_LAUNCH_CHECK();
  }
  draft_finish_kernel<<<1, kThreads, 0, st>>>(L.b, L.S, K, tree_tokens_out, parent_out, cum_logp_out, n_out, L.newidx);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
