// Draft-side expansion step (Alg. 2: probs -> selectBest by cumulative log-probability).
//
// Kernel 1, row_topk_kernel: one workgroup per expanded node.  The row of V fp32 logits is read
// from HBM exactly once into registers (float4 per lane, fully coalesced), and everything else
// -- max, sum of exponentials, the k best entries -- is computed from those registers.  This is
// the HBM-bound part: 4*V bytes per row in, 8*k bytes out.
// Selection: the k-th largest of the per-thread maxima is a lower bound t0 of the k-th largest
// entry of the row (k distinct threads hold a value >= t0), so only entries >= t0 can be among
// the k best.  For k << V that leaves a few dozen candidates, which are sorted in LDS by
// (value descending, index ascending).  Rows where the bound is useless (massive ties) fall back
// to an exact bitwise threshold search over the same registers.
//
// Vocabularies above 32768 do not fit the registers of such a workgroup; row_topk_stream_kernel
// streams the row instead (running maximum and rescaled sum per lane) and takes the candidates
// from a second sweep that L2 serves.
//
// Kernel 2, global_select_kernel: one workgroup picks the B best of the N*k candidates by
// score = cum_logp[row] + logp, ties to the lower flat index, and writes them in that order.
#include "kernels.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kCandCap = 1024;  // LDS slots for row candidates before the exact fallback is taken

template <int THREADS>
__device__ __forceinline__ int block_count(bool pred, int* red) {
  return block_sum_i<THREADS / 64>(pred ? 1 : 0, red);
}

// Exact selection for rows the cheap bound cannot handle.  Bitwise search for the k-th largest
// order key, then for the index below which ties are taken, each probe being one pass over the
// row (served by L2: the row was just read).  Leaves exactly k entries in cand[], returns k.
template <int THREADS>
__device__ __noinline__ int exact_topk_from_memory(const float* __restrict__ x, int V, int k, int* redi, int* s_cnt,
                                                   unsigned long long* cand) {
  constexpr int NW = THREADS / 64;
  const int tid = threadIdx.x;
  unsigned K = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const unsigned trial = K | (1u << bit);
    int c = 0;
    for (int i = tid; i < V; i += THREADS) c += (f32_order_key(x[i]) >= trial) ? 1 : 0;
    if (block_sum_i<NW>(c, redi) >= k) K = trial;
  }
  int cg = 0;
  for (int i = tid; i < V; i += THREADS) cg += (f32_order_key(x[i]) > K) ? 1 : 0;
  const int need = k - block_sum_i<NW>(cg, redi);  // ties to take, >= 1
  unsigned Y = 0;                                 // largest Y with #(tie, idx < Y) <= need
  for (int bit = 17; bit >= 0; --bit) {
    const unsigned trial = Y | (1u << bit);
    int c = 0;
    for (int i = tid; i < V && (unsigned)i < trial; i += THREADS) c += (f32_order_key(x[i]) == K) ? 1 : 0;
    if (block_sum_i<NW>(c, redi) <= need) Y = trial;
  }
  if (tid == 0) *s_cnt = 0;
  __syncthreads();
  for (int i = tid; i < V; i += THREADS) {
    const unsigned key = f32_order_key(x[i]);
    if (key > K || (key == K && (unsigned)i < Y)) {
      const int pos = atomicAdd(s_cnt, 1);
      if (pos < kCandCap) cand[pos] = ((unsigned long long)(~key) << 32) | (unsigned)i;
    }
  }
  __syncthreads();
  const int C = min(*s_cnt, kCandCap);
  __syncthreads();
  return C;
}

// THREADS lanes, each holding IPT4 float4 of the row.  Element (j, c) of a lane is index
// (j*THREADS + tid)*4 + c.
template <int THREADS, int IPT4, bool VEC>
__global__ __launch_bounds__(THREADS) void row_topk_kernel(const float* __restrict__ logits,
                                                           const float* __restrict__ cum_logp, int V, int k,
                                                           float* __restrict__ topk_logp,
                                                           int* __restrict__ topk_idx,
                                                           float* __restrict__ score) {
  constexpr int NW = THREADS / 64;
  __shared__ float smax[THREADS];
  __shared__ float redf[32];
  __shared__ float s_gmax[64];
  __shared__ int redi[16];
  __shared__ float s_t0;
  __shared__ int s_cnt;
  __shared__ int s_part[NW][64];  // partial ranks / places, one row per wave
  __shared__ unsigned long long cand[kCandCap];

  const int tid = threadIdx.x;
  const size_t row = blockIdx.x;
  const float* x = logits + row * (size_t)V;
  const float NEG_INF = -__builtin_huge_valf();

  float v[IPT4 * 4];
#pragma unroll
  for (int j = 0; j < IPT4; ++j) {
    const int base = (j * THREADS + tid) * 4;
    if (VEC) {
      if (base < V) {
        const float4 t = *reinterpret_cast<const float4*>(x + base);
        v[4 * j + 0] = t.x; v[4 * j + 1] = t.y; v[4 * j + 2] = t.z; v[4 * j + 3] = t.w;
      } else {
        v[4 * j + 0] = v[4 * j + 1] = v[4 * j + 2] = v[4 * j + 3] = NEG_INF;
      }
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) v[4 * j + c] = (base + c < V) ? x[base + c] : NEG_INF;
    }
  }

  // ---- maxima: per lane, per group of GS lanes (64 groups), per wave -----------------------------
  constexpr int GS = THREADS / 64;
  float tm = NEG_INF;
#pragma unroll
  for (int e = 0; e < IPT4 * 4; ++e) tm = fmaxf(tm, v[e]);
  float gm = tm;
#pragma unroll
  for (int o = 1; o < GS; o <<= 1) gm = fmaxf(gm, __shfl_xor(gm, o, 64));
  const float wmx = wave_max(gm);
  const bool small_k = k <= 64;  // uniform
  if ((tid & 63) == 0) redf[tid >> 6] = wmx;
  if ((tid & (GS - 1)) == 0) s_gmax[tid / GS] = gm;
  if (!small_k) smax[tid] = tm;
  if (tid == 0) s_cnt = 0;
  __syncthreads();  // (1)
  float M = redf[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) M = fmaxf(M, redf[w]);

  // ---- sum of exponentials, and the ranks of the group maxima ------------------------------------------
  // t0 = k-th largest of a set of group maxima (rank by value, then group id) is a lower bound of
  // the k-th largest entry.  k <= 64: 64 groups (hardly looser than per-lane maxima and far cheaper),
  // ranked with lane broadcasts by all waves together, each comparing the 64 maxima with its share of
  // 64 / NW of them (all 64 broadcasts on one wave were the longest single-wave stretch of the kernel);
  // the partial ranks meet in LDS at the next barrier.  Larger k: every lane is a group.
  const int lane = tid & 63, wave = tid >> 6;
  float gmine = 0.f;
  if (small_k) {
    gmine = s_gmax[lane];
    int prank = 0;
#pragma unroll
    for (int jj = 0; jj < 64 / NW; ++jj) {
      const int j = __builtin_amdgcn_readfirstlane(wave) * (64 / NW) + jj;
      const float o = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(gmine), j));
      prank += (o > gmine || (o == gmine && j < lane)) ? 1 : 0;
    }
    s_part[wave][lane] = prank;
  }
  float se = 0.f;
  const float mshift = -M * kLog2e;
#pragma unroll
  for (int e = 0; e < IPT4 * 4; ++e) se += __builtin_amdgcn_exp2f(fmaf(v[e], kLog2e, mshift));
  se = wave_sum(se);
  if ((tid & 63) == 0) redf[NW + (tid >> 6)] = se;
  if (!small_k) {
    int rank = 0;
    for (int j = 0; j < THREADS; ++j) {
      const float o = smax[j];
      rank += (o > tm || (o == tm && j < tid)) ? 1 : 0;
    }
    if (rank == k - 1) s_t0 = tm;
  }
  __syncthreads();  // (2)
  float S = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) S += redf[NW + w];
  const float lse = M + logf(S);
  float t0;
  if (small_k) {  // exactly one group has rank k - 1 (ranks are a permutation of 0..63)
    int rank = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) rank += s_part[w][lane];
    const unsigned long long who = __builtin_amdgcn_ballot_w64(rank == k - 1);
    t0 = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(gmine), __builtin_ctzll(who)));
  } else {
    t0 = s_t0;
  }

  // ---- gather candidates >= t0 ---------------------------------------------------------------
  // Hits are rare (a few dozen per row): the four values of a register quad are looked at only where the
  // quad's maximum of some lane of the wave reaches t0 -- two instructions and one scalar branch per quad.
#pragma unroll
  for (int j = 0; j < IPT4; ++j) {
    const float m4 = fmaxf(fmaxf(v[4 * j + 0], v[4 * j + 1]), fmaxf(v[4 * j + 2], v[4 * j + 3]));
    if (__builtin_amdgcn_ballot_w64(m4 >= t0) != 0ull) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int idx = (j * THREADS + tid) * 4 + c;
        if (v[4 * j + c] >= t0 && idx < V) {
          const int pos = atomicAdd(&s_cnt, 1);
          if (pos < kCandCap)
            cand[pos] = ((unsigned long long)(~f32_order_key(v[4 * j + c])) << 32) | (unsigned)idx;
        }
      }
    }
  }
  __syncthreads();  // (3)
  int C = s_cnt;
  const float cl = cum_logp ? cum_logp[row] : 0.f;

  if (small_k && C <= 64) {
    // ---- the usual case: a few dozen candidates, ordered in registers ------------------------------------
    // Keys are distinct (the index is part of them), so a candidate's place is the number of smaller keys:
    // scalar broadcasts and compares, no sorting network and no cross-lane latency chain.  Every wave holds
    // all candidates (lane = candidate) and counts against its share of 64 / NW of them.
    const unsigned long long x64 = lane < C ? cand[lane] : ~0ull;
    const unsigned xlo = (unsigned)x64, xhi = (unsigned)(x64 >> 32);
    int pplace = 0;
#pragma unroll
    for (int jj = 0; jj < 64 / NW; ++jj) {
      const int j = __builtin_amdgcn_readfirstlane(wave) * (64 / NW) + jj;
      const unsigned olo = __builtin_amdgcn_readlane(xlo, j), ohi = __builtin_amdgcn_readlane(xhi, j);
      pplace += (ohi < xhi || (ohi == xhi && olo < xlo)) ? 1 : 0;
    }
    s_part[wave][lane] = pplace;  // (the ranks in there were read before barrier (3))
    __syncthreads();  // (4)
    if (tid >= 64) return;
    int place = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) place += s_part[w][lane];
    if (tid < C && place < k) {
      const float val = f32_from_order_key(~xhi);
      const float lp = val - lse;
      const size_t o = row * (size_t)k + place;
      topk_idx[o] = (int)xlo;
      topk_logp[o] = lp;
      if (score) score[o] = cl + lp;
    }
    return;
  }
  __syncthreads();
  if (C > kCandCap) {  // the bound was useless (massive ties): exact search, re-reading the row from L2
    C = exact_topk_from_memory<THREADS>(x, V, k, redi, &s_cnt, cand);
  }

  // ---- general case: order the candidates in LDS and emit the first k --------------------------------
  const int n = next_pow2(C < 2 ? 2 : C);
  for (int i = C + tid; i < n; i += THREADS) cand[i] = ~0ull;
  block_bitonic_sort_u64<THREADS>(cand, n);
  for (int c = tid; c < k; c += THREADS) {
    const unsigned long long e = cand[c];
    const float val = f32_from_order_key(~(unsigned)(e >> 32));
    const float lp = val - lse;
    const size_t o = row * (size_t)k + c;
    topk_idx[o] = (int)(unsigned)(e & 0xFFFFFFFFull);
    topk_logp[o] = lp;
    if (score) score[o] = cl + lp;
  }
}

// Lane `tid` owns the float4 slots tid, tid + THREADS, ... of the row (element index 4 * slot + c).
// Pass 1 streams the row from HBM four slots at a time, keeping only a running maximum and a sum of
// exponentials relative to it; pass 2 streams it again, now from L2, and keeps the few entries >= t0.
// Few registers whatever V is: used for vocabularies too large for the register-resident kernel above.
template <int THREADS, bool VEC>
__global__ __launch_bounds__(THREADS) void row_topk_stream_kernel(const float* __restrict__ logits,
                                                           const float* __restrict__ cum_logp, int V, int k,
                                                           float* __restrict__ topk_logp,
                                                           int* __restrict__ topk_idx,
                                                           float* __restrict__ score) {
  constexpr int NW = THREADS / 64;
  constexpr int U = 4;  // float4 slots in flight per lane
  __shared__ float smax[THREADS];
  __shared__ float redf[32];
  __shared__ float s_gmax[64];
  __shared__ int redi[16];
  __shared__ float s_t0;
  __shared__ int s_cnt;
  __shared__ unsigned long long cand[kCandCap];

  const int tid = threadIdx.x;
  const size_t row = blockIdx.x;
  const float* x = logits + row * (size_t)V;
  const float NEG_INF = -__builtin_huge_valf();
  const int nslot = (V + 3) / 4;

  // slots [s0, s0 + U * THREADS) of the row into c[U * 4]; out-of-range elements read as -inf
  auto load_chunk = [&](int s0, float (&c)[U * 4]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int slot = s0 + u * THREADS + tid;
      if (VEC) {
        if (slot < nslot) {
          const float4 t = *reinterpret_cast<const float4*>(x + 4 * (size_t)slot);
          c[4 * u + 0] = t.x; c[4 * u + 1] = t.y; c[4 * u + 2] = t.z; c[4 * u + 3] = t.w;
        } else {
          c[4 * u + 0] = c[4 * u + 1] = c[4 * u + 2] = c[4 * u + 3] = NEG_INF;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) c[4 * u + e] = (4 * slot + e < V) ? x[4 * (size_t)slot + e] : NEG_INF;
      }
    }
  };

  // ---- pass 1: lane maximum tm and lane sum se of exp(x - tm), rescaled whenever tm rises ----------------
  float tm = NEG_INF, se = 0.f;
  for (int s0 = 0; s0 < nslot; s0 += U * THREADS) {
    float c[U * 4];
    load_chunk(s0, c);
    float cm = c[0];
#pragma unroll
    for (int e = 1; e < U * 4; ++e) cm = fmaxf(cm, c[e]);
    if (cm > tm) {  // also the first finite chunk: exp2(-inf) = 0 clears the (empty) sum
      se *= __builtin_amdgcn_exp2f((tm - cm) * kLog2e);
      tm = cm;
    }
    if (tm > NEG_INF) {
#pragma unroll
      for (int e = 0; e < U * 4; ++e) se += __builtin_amdgcn_exp2f((c[e] - tm) * kLog2e);
    }
  }

  // ---- maxima: per group of GS lanes (64 groups), per wave ---------------------------------------------
  constexpr int GS = THREADS / 64;
  float gm = tm;
#pragma unroll
  for (int o = 1; o < GS; o <<= 1) gm = fmaxf(gm, __shfl_xor(gm, o, 64));
  const float wmx = wave_max(gm);
  const bool small_k = k <= 64;  // uniform
  if ((tid & 63) == 0) redf[tid >> 6] = wmx;
  if ((tid & (GS - 1)) == 0) s_gmax[tid / GS] = gm;
  if (!small_k) smax[tid] = tm;
  if (tid == 0) s_cnt = 0;
  __syncthreads();  // (1)
  float M = redf[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) M = fmaxf(M, redf[w]);

  // ---- lane sums brought to the row maximum; meanwhile wave 0 ranks the group maxima -----------------------
  // t0 = k-th largest of a set of group maxima (rank by value, then group id) is a lower bound of
  // the k-th largest entry.  k <= 64: 64 groups ranked by one wave with lane broadcasts (hardly
  // looser than per-lane maxima and far cheaper); else every lane is a group.
  se = tm > NEG_INF ? se * __builtin_amdgcn_exp2f((tm - M) * kLog2e) : 0.f;
  se = wave_sum(se);
  if ((tid & 63) == 0) redf[NW + (tid >> 6)] = se;
  if (small_k) {
    if (tid < 64) {
      const float g = s_gmax[tid];
      int rank = 0;
#pragma unroll
      for (int j = 0; j < 64; ++j) {
        const float o = __shfl(g, j, 64);
        rank += (o > g || (o == g && j < tid)) ? 1 : 0;
      }
      if (rank == k - 1) s_t0 = g;
    }
  } else {
    int rank = 0;
    for (int j = 0; j < THREADS; ++j) {
      const float o = smax[j];
      rank += (o > tm || (o == tm && j < tid)) ? 1 : 0;
    }
    if (rank == k - 1) s_t0 = tm;
  }
  __syncthreads();  // (2)
  float S = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) S += redf[NW + w];
  const float lse = M + logf(S);
  const float t0 = s_t0;

  // ---- pass 2: gather candidates >= t0 (the row comes from L2 this time) -------------------------------
  // Hits are rare (a few dozen per row): one compare and one scalar branch per value, and the divergent
  // code only where some lane of the wave has one.  A lane whose maximum is below t0 holds none, and a
  // wave of such lanes skips its share of the row altogether.
  if (__builtin_amdgcn_ballot_w64(tm >= t0) != 0ull) {
    for (int s0 = 0; s0 < nslot; s0 += U * THREADS) {
      float c[U * 4];
      load_chunk(s0, c);
#pragma unroll
      for (int e = 0; e < U * 4; ++e) {
        const bool hit = c[e] >= t0;
        if (__builtin_amdgcn_ballot_w64(hit) != 0ull) {
          const int idx = 4 * (s0 + (e >> 2) * THREADS + tid) + (e & 3);
          if (hit && idx < V) {
            const int pos = atomicAdd(&s_cnt, 1);
            if (pos < kCandCap) cand[pos] = ((unsigned long long)(~f32_order_key(c[e])) << 32) | (unsigned)idx;
          }
        }
      }
    }
  }
  __syncthreads();  // (3)
  int C = s_cnt;
  const float cl = cum_logp ? cum_logp[row] : 0.f;

  if (small_k && C <= 64) {
    // ---- the usual case: a few dozen candidates, placed by one wave in registers --------------------
    // keys are distinct (the index is part of them), so a candidate's place is the number of smaller
    // keys: 64 scalar broadcasts and compares, no sorting network and no cross-lane latency chain
    if (tid >= 64) return;
    const unsigned long long x64 = tid < C ? cand[tid] : ~0ull;
    const unsigned xlo = (unsigned)x64, xhi = (unsigned)(x64 >> 32);
    int place = 0;
#pragma unroll
    for (int j = 0; j < 64; ++j) {
      const unsigned olo = __builtin_amdgcn_readlane(xlo, j), ohi = __builtin_amdgcn_readlane(xhi, j);
      place += (ohi < xhi || (ohi == xhi && olo < xlo)) ? 1 : 0;
    }
    if (tid < C && place < k) {
      const float val = f32_from_order_key(~xhi);
      const float lp = val - lse;
      const size_t o = row * (size_t)k + place;
      topk_idx[o] = (int)xlo;
      topk_logp[o] = lp;
      if (score) score[o] = cl + lp;
    }
    return;
  }
  __syncthreads();
  if (C > kCandCap) {  // the bound was useless (massive ties): exact search, re-reading the row from L2
    C = exact_topk_from_memory<THREADS>(x, V, k, redi, &s_cnt, cand);
  }

  // ---- general case: order the candidates in LDS and emit the first k --------------------------------
  const int n = next_pow2(C < 2 ? 2 : C);
  for (int i = C + tid; i < n; i += THREADS) cand[i] = ~0ull;
  block_bitonic_sort_u64<THREADS>(cand, n);
  for (int c = tid; c < k; c += THREADS) {
    const unsigned long long e = cand[c];
    const float val = f32_from_order_key(~(unsigned)(e >> 32));
    const float lp = val - lse;
    const size_t o = row * (size_t)k + c;
    topk_idx[o] = (int)(unsigned)(e & 0xFFFFFFFFull);
    topk_logp[o] = lp;
    if (score) score[o] = cl + lp;
  }
}

// One workgroup of 1024 lanes; lane t owns the flat candidates [t*per, (t+1)*per).
// REG = true keeps the (<= 64) keys of a lane in registers.
constexpr int kSelThreads = 1024;

template <bool REG>
__global__ __launch_bounds__(kSelThreads) void global_select_kernel(const float* __restrict__ score,
                                                                    const int* __restrict__ topk_idx, int n, int k,
                                                                    int B, int per, int* __restrict__ out_row,
                                                                    int* __restrict__ out_token,
                                                                    float* __restrict__ out_score,
                                                                    int* __restrict__ n_out) {
  constexpr int NW = kSelThreads / 64;
  constexpr int RK = 64;  // keys a lane can hold in registers
  extern __shared__ unsigned long long sbuf[];
  __shared__ int redi[16];
  __shared__ int s_wave_ties[NW];
  __shared__ int s_probe[2][NW];
  __shared__ int s_pos;

  const int tid = threadIdx.x;
  const int Bsel = min(B, n);

  // ---- threshold: K = largest order key with #(key >= K) >= Bsel, by bitwise search --------------------
  // For the search a lane holds the keys tid, tid + 1024, ... (coalesced); slots past n hold key 0,
  // below every real key.
  unsigned key[REG ? RK : 1];
  if (REG) {
#pragma unroll
    for (int e = 0; e < RK; ++e) {
      const int i = e * kSelThreads + tid;
      key[e] = i < n ? f32_order_key(score[i]) : 0u;
    }
  }
  unsigned K = 0;
  if (n > Bsel) {
    // One barrier per probe: the per-wave counts alternate between two LDS rows, so the next probe's
    // writers can never overtake this probe's readers.
    for (int bit = 31; bit >= 0; --bit) {
      const unsigned trial = K | (1u << bit);
      int c = 0;
      if (REG) {
#pragma unroll
        for (int e = 0; e < RK; ++e) c += (key[e] >= trial) ? 1 : 0;
      } else {
        for (int i = tid; i < n; i += kSelThreads) c += (f32_order_key(score[i]) >= trial) ? 1 : 0;
      }
      c = wave_sum_i(c);
      int* row = s_probe[bit & 1];
      if ((tid & 63) == 0) row[tid >> 6] = c;
      __syncthreads();
      int total = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) total += row[w];
      if (total >= Bsel) K = trial;
    }
  }

  // ---- winners: every key > K, and of the keys == K the `need` lowest flat indices -----------------------
  int gt = 0, eq = 0;
  if (REG) {
#pragma unroll
    for (int e = 0; e < RK; ++e) {
      gt += (key[e] > K) ? 1 : 0;
      eq += (key[e] == K) ? 1 : 0;
    }
  } else {
    for (int i = tid; i < n; i += kSelThreads) {
      const unsigned kk = f32_order_key(score[i]);
      gt += kk > K;
      eq += kk == K;
    }
  }
  if (tid == 0) s_pos = 0;
  const int need = Bsel - block_sum_i<NW>(gt, redi);
  const int ties = block_sum_i<NW>(eq, redi);
  auto push = [&](unsigned kk, int flat) {
    const int pos = atomicAdd(&s_pos, 1);
    sbuf[pos] = ((unsigned long long)(~kk) << 32) | (unsigned)flat;
  };
  const bool all_ties = (ties == need);  // the usual case (a single key equals K): no ranking needed
  // (re-read from L2 in a rolled, coalesced loop: pushing from the register copy would unroll 64
  // conditional atomics and spill)
#pragma unroll 4
  for (int i = tid; i < n; i += kSelThreads) {
    const unsigned kk = f32_order_key(score[i]);
    if (kk > K || (all_ties && kk == K)) push(kk, i);
  }
  if (!all_ties) {
    // Rare: more keys equal K than fit.  Lanes walk contiguous ranges so that an exclusive scan of
    // their tie counts ranks the ties in flat-index order; the `need` first ones are taken.
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    int mine = 0;
    for (int i = lo; i < hi; ++i) mine += f32_order_key(score[i]) == K;
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o, 64);
      if ((tid & 63) >= o) incl += t;
    }
    if ((tid & 63) == 63) s_wave_ties[tid >> 6] = incl;
    __syncthreads();
    int tie_rank = incl - mine;
    for (int w = 0; w < (tid >> 6); ++w) tie_rank += s_wave_ties[w];
    for (int i = lo; i < hi && tie_rank < need; ++i)
      if (f32_order_key(score[i]) == K) {
        push(K, i);
        ++tie_rank;
      }
  }
  __syncthreads();
  const int nsort = next_pow2(Bsel < 2 ? 2 : Bsel);
  for (int i = Bsel + tid; i < nsort; i += kSelThreads) sbuf[i] = ~0ull;
  block_bitonic_sort_u64<kSelThreads>(sbuf, nsort);
  for (int i = tid; i < Bsel; i += kSelThreads) {
    const unsigned flat = (unsigned)(sbuf[i] & 0xFFFFFFFFull);
    out_row[i] = (int)(flat / (unsigned)k);
    out_token[i] = topk_idx[flat];
    out_score[i] = score[flat];
  }
  if (tid == 0) n_out[0] = Bsel;
}

template <int THREADS, int IPT4>
void launch_row(const float* logits, const float* cum, int N, int V, int k, float* lp, int* idx, float* score,
                hipStream_t st) {
  const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(logits) & 15) == 0);
  if (vec)
    row_topk_kernel<THREADS, IPT4, true><<<N, THREADS, 0, st>>>(logits, cum, V, k, lp, idx, score);
  else
    row_topk_kernel<THREADS, IPT4, false><<<N, THREADS, 0, st>>>(logits, cum, V, k, lp, idx, score);
}

int row_topk_dispatch(const float* logits, const float* cum, int N, int V, int k, float* lp, int* idx, float* score,
                      hipStream_t st) {
  // lanes x float4-per-lane sized so that a row fits in registers with >= 2 workgroups per CU
  if (V <= 1024) launch_row<256, 1>(logits, cum, N, V, k, lp, idx, score, st);
  else if (V <= 4096) launch_row<256, 4>(logits, cum, N, V, k, lp, idx, score, st);
  else if (V <= 16384) launch_row<256, 16>(logits, cum, N, V, k, lp, idx, score, st);
  else if (V <= 32768) launch_row<512, 16>(logits, cum, N, V, k, lp, idx, score, st);
  else {  // the row no longer fits the registers of a workgroup that leaves room for a second one
    const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(logits) & 15) == 0);
    if (vec) row_topk_stream_kernel<512, true><<<N, 512, 0, st>>>(logits, cum, V, k, lp, idx, score);
    else row_topk_stream_kernel<512, false><<<N, 512, 0, st>>>(logits, cum, V, k, lp, idx, score);
  }
  SX_LAUNCH_CHECK();
  return SX_OK;
}

bool row_shape_ok(int N, int V, int k) {
  return N >= 1 && V >= 1 && V <= 131072 && k >= 1 && k <= 256 && k <= V && (long long)N * k < (1ll << 31);
}

}  // namespace

extern "C" int sx_row_logsoftmax_topk(const float* logits, int32_t N, int32_t V, int32_t k, float* topk_logp,
                                      int32_t* topk_idx, void* stream) {
  if (!logits || !topk_logp || !topk_idx) return SX_ERR_NULL;
  if (!row_shape_ok(N, V, k)) return SX_ERR_SHAPE;
  return row_topk_dispatch(logits, nullptr, N, V, k, topk_logp, topk_idx, nullptr, (hipStream_t)stream);
}

// workspace: header | score f32[N*k] | topk_logp f32[N*k] | topk_idx i32[N*k]
extern "C" size_t sx_expand_topk_workspace(int32_t N, int32_t V, int32_t k, int32_t B) {
  (void)V;
  (void)B;
  if (N < 1 || k < 1) return 0;
  const size_t nk = sx_align_up((size_t)N * (size_t)k * 4, 256);
  return SX_WS_HEADER + 3 * nk;
}

namespace {

// B = 8192 needs the full 64 KB of dynamic LDS next to the static arrays; set once per device
int configure_select_once() {
  static bool configured[64] = {};
  int dev = 0;
  SX_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return SX_ERR_HIP;
  if (configured[dev]) return SX_OK;
  SX_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&global_select_kernel<true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 8));
  SX_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&global_select_kernel<false>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 8));
  configured[dev] = true;
  return SX_OK;
}

// both kernels of the expansion step on `st`; score / lp / idx hold N*k entries each (every one of them is
// written by the first kernel before the second reads it: nothing has to be cleared)
int expand_topk_run(const float* logits, const float* cum_logp, int N, int V, int k, int B, int* out_row,
                    int* out_token, float* out_cum_logp, int* n_out, float* score, float* lp, int* idx,
                    hipStream_t st) {
  SX_TRY(configure_select_once());
  sx_prof_begin(SX_K_ROW_TOPK, st);
  const int rc = row_topk_dispatch(logits, cum_logp, N, V, k, lp, idx, score, st);
  sx_prof_end(st);
  if (rc != SX_OK) return rc;
  const int n = N * k;
  const int per = (n + kSelThreads - 1) / kSelThreads;
  const int Bsel = B < n ? B : n;
  int nsort = 2;
  while (nsort < Bsel) nsort <<= 1;
  const size_t shmem = (size_t)nsort * sizeof(unsigned long long);
  sx_prof_begin(SX_K_SELECT, st);
  if (per <= 64)
    global_select_kernel<true><<<1, kSelThreads, shmem, st>>>(score, idx, n, k, B, per, out_row, out_token,
                                                               out_cum_logp, n_out);
  else
    global_select_kernel<false><<<1, kSelThreads, shmem, st>>>(score, idx, n, k, B, per, out_row, out_token,
                                                                out_cum_logp, n_out);
  sx_prof_end(st);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

}  // namespace

extern "C" int sx_expand_topk(const float* logits, const float* cum_logp, int32_t N, int32_t V, int32_t k, int32_t B,
                              int32_t* out_row, int32_t* out_token, float* out_cum_logp, int32_t* n_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!logits || !cum_logp || !out_row || !out_token || !out_cum_logp || !n_out) return SX_ERR_NULL;
  if (!row_shape_ok(N, V, k) || B < 1 || B > 8192) return SX_ERR_SHAPE;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) ||
      workspace_bytes < sx_expand_topk_workspace(N, V, k, B))
    return SX_ERR_WORKSPACE;
  const size_t nk = sx_align_up((size_t)N * (size_t)k * 4, 256);
  char* ws = static_cast<char*>(workspace);
  return expand_topk_run(logits, cum_logp, N, V, k, B, out_row, out_token, out_cum_logp, n_out,
                         reinterpret_cast<float*>(ws + SX_WS_HEADER), reinterpret_cast<float*>(ws + SX_WS_HEADER + nk),
                         reinterpret_cast<int*>(ws + SX_WS_HEADER + 2 * nk), (hipStream_t)stream);
}

// ---- the same step for callers that cannot allocate ----------------------------------------------------
// The three candidate arrays (score, log-probability, token id; N*k entries each) live in a file-scope
// device array instead of a caller's workspace.  Every GPU holds its own copy of the array at its own
// address; the name below is only a host-side handle for hipGetSymbolAddress, never a kernel argument.
namespace {
constexpr int kStaticMaxCand = SX_EXPAND_STATIC_MAX_CANDIDATES;
static __device__ __align__(256) unsigned char scratch[3 * (size_t)kStaticMaxCand * 4];
void* g_scratch_ptr[64] = {};  // per device: address of that device's copy of `scratch`
}  // namespace

extern "C" int sx_expand_topk_static(const float* logits, const float* cum_logp, int32_t N, int32_t V, int32_t k,
                                     int32_t B, int32_t* out_row, int32_t* out_token, float* out_cum_logp,
                                     int32_t* n_out, void* stream) {
  if (!logits || !cum_logp || !out_row || !out_token || !out_cum_logp || !n_out) return SX_ERR_NULL;
  if (!row_shape_ok(N, V, k) || B < 1 || B > 8192) return SX_ERR_SHAPE;
  if ((long long)N * k > kStaticMaxCand) return SX_ERR_SHAPE;  // beyond the fixed scratch: use sx_expand_topk
  int dev = 0;
  SX_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return SX_ERR_HIP;
  if (!g_scratch_ptr[dev]) {  // first call on this device (with it current): look its copy of the array up
    void* p = nullptr;
    SX_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SX_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  char* base = static_cast<char*>(g_scratch_ptr[dev]);
  const size_t nk = (size_t)kStaticMaxCand * 4;
  return expand_topk_run(logits, cum_logp, N, V, k, B, out_row, out_token, out_cum_logp, n_out,
                         reinterpret_cast<float*>(base), reinterpret_cast<float*>(base + nk),
                         reinterpret_cast<int*>(base + 2 * nk), (hipStream_t)stream);
}
