// Acceptance walk (Alg. 1, main loop): sequential sampling from the target model, served from the
// tree of precomputed distributions for as long as the sampled tokens stay on a tree path.
//
// One workgroup walks the tree; every step is data-parallel over the V logits of the current
// node.  The row is read once per step and kept as exp((x - max)/t) in registers (V <= 32768) or
// in a caller-provided scratch row (larger V).  Nucleus and draw are found with bitwise searches
// whose probes are block reductions in a fixed order, so a given input always gives the same path:
//   * nucleus threshold: the largest float bit pattern K with  sum{e >= K} >= top_p * Z;
//   * draw: the largest id Y with  sum{nucleus, id < Y} <= u * mass  (inverse CDF in id order).
//
// With draft probabilities (SI = true) the same kernel runs the comparison system of Sect. 4.1 instead:
// a drafted child with token x is accepted with probability P_target(x) / P_draft(x), capped at one.  The
// warped target distribution p of the current node is then a normalised vector in the scratch row; the
// children are tried in index order, child j of the position accepted when r_j q[x] < p[x]; a rejection
// replaces p by the renormalised positive part of p - q; after the last rejection the token is drawn
// from what p has become and the walk ends.
#include "kernels.h"

namespace {

__device__ __forceinline__ float uniform01(unsigned long long seed, long long position) {
  unsigned long long z = seed + (unsigned long long)(position + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  return (float)(z >> 40) * 5.9604644775390625e-08f;  // 2^-24
}

// the uniform of the trial-th decision at one position (the ratio test needs several per position)
__device__ __forceinline__ float trial_uniform(unsigned long long seed, long long position, int trial) {
  return uniform01(seed + (unsigned long long)(trial + 1) * 0xD6E8FEB86659FD93ull, position);
}

// ITEMS > 0: lane holds elements j*NT + tid, j < ITEMS, in registers.  ITEMS == 0: elements live in ebuf.
// SI (only with ITEMS == 0): acceptance by the ratio of target and draft probability, see the header.
template <int NT, int ITEMS, bool SI>
__global__ __launch_bounds__(NT) void accept_walk_kernel(const float* __restrict__ logits,
                                                         const float* __restrict__ draft_probs,
                                                         const int* __restrict__ tokens,
                                                         const int* __restrict__ parent, int T, int V,
                                                         float temperature, float top_p, unsigned long long seed,
                                                         int pos0, int* __restrict__ path_out,
                                                         int* __restrict__ tokens_out, int* __restrict__ n_out,
                                                         float* __restrict__ ebuf, int* __restrict__ status) {
  static_assert(!SI || ITEMS == 0, "the ratio test keeps its distribution in the scratch row");
  constexpr int NW = NT / 64;
  constexpr int R = ITEMS > 0 ? ITEMS : 1;
  __shared__ float redf[16];
  __shared__ int redi[16];
  const int tid = threadIdx.x;
  const float NEG_INF = -__builtin_huge_valf();

  if (tid == 0) status[0] = (parent[0] != -1) ? SX_ERR_TREE : SX_OK;  // node 0 must be the root

  float ev[R];
  // sum of e over elements selected by pred(bits(e), id)
  auto sum_if = [&](auto pred) -> float {
    float a = 0.f;
    if constexpr (ITEMS > 0) {
#pragma unroll
      for (int j = 0; j < ITEMS; ++j) {
        const int id = j * NT + tid;
        a += pred(__float_as_uint(ev[j]), id) ? ev[j] : 0.f;  // padding holds e = 0
      }
    } else {
      for (int id = tid; id < V; id += NT) {
        const float e = ebuf[id];
        a += pred(__float_as_uint(e), id) ? e : 0.f;
      }
    }
    return block_sum<NW>(a, redf);
  };
  auto count_if = [&](auto pred) -> int {
    int c = 0;
    if constexpr (ITEMS > 0) {
#pragma unroll
      for (int j = 0; j < ITEMS; ++j) {
        const int id = j * NT + tid;
        c += (id < V && pred(__float_as_uint(ev[j]), id)) ? 1 : 0;
      }
    } else {
      for (int id = tid; id < V; id += NT) c += pred(__float_as_uint(ebuf[id]), id) ? 1 : 0;
    }
    return block_sum_i<NW>(c, redi);
  };

  int cur = 0, depth = 0, n = 0;
  for (int step = 0; step < T; ++step) {
    const float* x = logits + (size_t)cur * (size_t)V;
    // ---- row maximum (and the greedy answer) ------------------------------------------------------
    float tm = NEG_INF;
    if constexpr (ITEMS > 0) {
#pragma unroll
      for (int j = 0; j < ITEMS; ++j) {
        const int id = j * NT + tid;
        ev[j] = id < V ? x[id] : NEG_INF;
        tm = fmaxf(tm, ev[j]);
      }
    } else {
      for (int id = tid; id < V; id += NT) tm = fmaxf(tm, x[id]);
    }
    const float M = block_max<NW>(tm, redf);
    int token;
    if (temperature == 0.f) {
      int best = 0x7FFFFFFF;
      if constexpr (ITEMS > 0) {
#pragma unroll
        for (int j = ITEMS - 1; j >= 0; --j) {
          const int id = j * NT + tid;
          if (id < V && ev[j] == M) best = id;
        }
      } else {
        for (int id = tid; id < V; id += NT)
          if (x[id] == M) best = min(best, id);
      }
      token = block_min_i<NW>(best, redi);
      if constexpr (SI) {  // p = all mass on the argmax
        __syncthreads();
        for (int id = tid; id < V; id += NT) ebuf[id] = id == token ? 1.0f : 0.f;
        __syncthreads();
      }
    } else {
      // ---- e = exp((x - max)/t), Z ------------------------------------------------------------
      const float inv_t = 1.0f / temperature;
      float zs = 0.f;
      if constexpr (ITEMS > 0) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
          const int id = j * NT + tid;
          ev[j] = id < V ? expf((ev[j] - M) * inv_t) : 0.f;
          zs += ev[j];
        }
      } else {
        for (int id = tid; id < V; id += NT) {
          const float e = expf((x[id] - M) * inv_t);
          ebuf[id] = e;
          zs += e;
        }
        __syncthreads();
      }
      const float Z = block_sum<NW>(zs, redf);
      const float thr = top_p * Z;
      // ---- nucleus: largest bit pattern K with sum{e >= K} >= thr --------------------------------
      unsigned K = 0;
      for (int bit = 30; bit >= 0; --bit) {
        const unsigned trial = K | (1u << bit);
        const float S = sum_if([&](unsigned b, int) { return b >= trial; });
        if (S >= thr) K = trial;
      }
      const float S_gt = sum_if([&](unsigned b, int) { return b > K; });
      const int n_tie = count_if([&](unsigned b, int) { return b == K; });
      const float eK = __uint_as_float(K);
      int m = 1;  // ties (equal probabilities) enter in id order until the mass reaches thr
      while (m < n_tie && S_gt + (float)m * eK < thr) ++m;
      unsigned Ytie = 0xFFFFFFFFu;
      if (m < n_tie) {  // largest Y with #(tie, id < Y) <= m
        Ytie = 0;
        for (int bit = 17; bit >= 0; --bit) {
          const unsigned trial = Ytie | (1u << bit);
          const int c = count_if([&](unsigned b, int id) { return b == K && (unsigned)id < trial; });
          if (c <= m) Ytie = trial;
        }
      }
      auto member = [&](unsigned b, int id) { return b > K || (b == K && (unsigned)id < Ytie); };
      const float mass = sum_if(member);
      if constexpr (SI) {  // p = the nucleus, normalised; the draw below is not taken in this mode
        const float inv_mass = 1.0f / mass;
        __syncthreads();
        for (int id = tid; id < V; id += NT) {
          const float e = ebuf[id];
          ebuf[id] = member(__float_as_uint(e), id) ? e * inv_mass : 0.f;
        }
        __syncthreads();
      }
      token = 0;
      if constexpr (!SI) {
        const float u = uniform01(seed, (long long)pos0 + depth + 1);
        const float target = u * mass;
        // ---- inverse CDF in id order: largest Y <= V with sum{member, id < Y} <= target ---------
        unsigned Y = 0;
        for (int bit = 17; bit >= 0; --bit) {
          const unsigned trial = Y | (1u << bit);
          if (trial > (unsigned)V) continue;  // uniform across the block
          const float G = sum_if([&](unsigned b, int id) { return (unsigned)id < trial && member(b, id); });
          if (G <= target) Y = trial;
        }
        token = (int)Y;
        if (Y >= (unsigned)V) {  // only by rounding: fall back to the last nucleus token
          int last = -1;
          if constexpr (ITEMS > 0) {
#pragma unroll
            for (int j = 0; j < ITEMS; ++j) {
              const int id = j * NT + tid;
              if (id < V && member(__float_as_uint(ev[j]), id)) last = id;
            }
          } else {
            for (int id = tid; id < V; id += NT)
              if (member(__float_as_uint(ebuf[id]), id)) last = id;
          }
          token = -block_min_i<NW>(-last, redi);
        }
      }
    }
    if constexpr (SI) {
      // ---- ratio test over the children of cur, in index order ------------------------------------------
      const float* q = draft_probs + (size_t)cur * (size_t)V;
      const long long pos = (long long)pos0 + depth + 1;
      int after = cur, trial = 0, accepted = -1;
      while (true) {
        int c = 0x7FFFFFFF;
        for (int j = after + 1 + tid; j < T; j += NT)
          if (parent[j] == cur) c = min(c, j);
        c = block_min_i<NW>(c, redi);
        if (c == 0x7FFFFFFF) break;
        const int x = tokens[c];
        after = c;
        if (x < 0 || x >= V) {  // not a token: nothing to accept, nothing the draft could have covered
          if (tid == 0) status[0] = SX_ERR_TREE;
          ++trial;
          continue;
        }
        if (trial_uniform(seed, pos, trial) * q[x] < ebuf[x]) {
          accepted = c;
          break;
        }
        ++trial;
        float z = 0.f;
        for (int id = tid; id < V; id += NT) z += fmaxf(ebuf[id] - q[id], 0.f);
        const float Zr = block_sum<NW>(z, redf);  // its barriers also order the reads of ebuf[x] above before the writes
        if (Zr > 0.f) {
          const float inv = 1.0f / Zr;
          for (int id = tid; id < V; id += NT) ebuf[id] = fmaxf(ebuf[id] - q[id], 0.f) * inv;
        }
        __syncthreads();
      }
      if (accepted >= 0) {
        if (tid == 0) {
          path_out[n] = cur;
          tokens_out[n] = tokens[accepted];
        }
        ++n;
        cur = accepted;
        ++depth;
        continue;
      }
      // ---- every child rejected: draw from what p has become, then stop ----------------------------------
      const float S = sum_if([&](unsigned, int) { return true; });
      const float target = trial_uniform(seed, pos, trial) * S;
      unsigned Y = 0;
      for (int bit = 17; bit >= 0; --bit) {
        const unsigned t2 = Y | (1u << bit);
        if (t2 > (unsigned)V) continue;
        const float G = sum_if([&](unsigned, int id) { return (unsigned)id < t2; });
        if (G <= target) Y = t2;
      }
      token = (int)Y;
      if (Y >= (unsigned)V) {  // only by rounding: the last token with mass
        int last = -1;
        for (int id = tid; id < V; id += NT)
          if (ebuf[id] > 0.f) last = id;
        token = -block_min_i<NW>(-last, redi);
      }
      if (tid == 0) {
        path_out[n] = cur;
        tokens_out[n] = token;
      }
      ++n;
      break;
    }
    if (tid == 0) {
      path_out[n] = cur;
      tokens_out[n] = token;
    }
    ++n;
    // ---- cache lookup: lowest-index child of cur carrying the sampled token -------------------------
    int child = 0x7FFFFFFF;
    for (int j = cur + 1 + tid; j < T; j += NT)
      if (parent[j] == cur && tokens[j] == token) child = min(child, j);
    child = block_min_i<NW>(child, redi);
    if (child == 0x7FFFFFFF) break;
    cur = child;
    ++depth;
  }
  if (tid == 0) n_out[0] = n;
}

}  // namespace

extern "C" size_t sx_accept_walk_workspace(int32_t T, int32_t V) {
  (void)T;
  if (V < 1) return 0;
  return SX_WS_HEADER + sx_align_up((size_t)V * 4, 256);
}

extern "C" int sx_accept_walk(const float* logits, const float* draft_probs, const int32_t* tree_tokens,
                              const int32_t* parent_idx, int32_t T, int32_t V, float temperature, float top_p,
                              uint64_t seed, int32_t pos0, int32_t* path_out, int32_t* tokens_out, int32_t* n_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!logits || !tree_tokens || !parent_idx || !path_out || !tokens_out || !n_out) return SX_ERR_NULL;
  if (T < 1 || V < 1 || V > 131072 || !(top_p > 0.f) || top_p > 1.f || !(temperature >= 0.f)) return SX_ERR_SHAPE;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < sx_accept_walk_workspace(T, V))
    return SX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  int* status = reinterpret_cast<int*>(workspace);
  float* ebuf = reinterpret_cast<float*>(static_cast<char*>(workspace) + SX_WS_HEADER);
#define SX_WALK(NT, ITEMS, SI)                                                                                        \
  accept_walk_kernel<NT, ITEMS, SI><<<1, NT, 0, st>>>(logits, draft_probs, tree_tokens, parent_idx, T, V, temperature, \
                                                      top_p, (unsigned long long)seed, pos0, path_out, tokens_out,    \
                                                      n_out, ebuf, status)
  sx_prof_begin(SX_K_WALK, st);
  if (draft_probs) SX_WALK(1024, 0, true);
  else if (V <= 1024) SX_WALK(512, 2, false);
  else if (V <= 8192) SX_WALK(512, 16, false);
  else if (V <= 32768) SX_WALK(512, 64, false);
  else SX_WALK(1024, 0, false);
#undef SX_WALK
  sx_prof_end(st);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
