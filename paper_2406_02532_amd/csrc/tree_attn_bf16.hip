// Tree attention on the gfx950 matrix cores (App. D: all tree tokens in one pass under a merged mask;
// every node sees the cached prefix, its ancestors and itself).  bf16 q/k/v, fp32 softmax statistics
// and accumulation, GQA.
//
// Work split.  grid = (query tiles, KV heads).  A workgroup (4 waves) owns 128 query rows of one KV
// head: 128/G consecutive nodes x the G query heads that share the KV head; a wave owns 32 rows.
// Keys come in tiles of 64: first the dense prefix (no mask), then the tile's tree keys -- not all
// T tree tokens, only the sorted union of the ancestors of the tile's nodes (a few dozen for
// best-first trees), gathered by index, with a 64-bit per-node mask saying which of them are that
// node's own ancestors.  Work on the tree part is therefore proportional to what is attended.
//
// Data flow per key tile (flash-style online softmax):
//   K rows  -> LDS [key][d], 16-byte chunks XOR-swizzled by key & 15 (16 lanes x 16 B per LDS cycle);
//   V rows  -> LDS transposed [d][key slot], packed on the fly from 4-byte column pairs;
//   S^T = K Q^T   (MFMA 32x32x16: A = K from LDS, B = Q held in registers for the whole kernel).
//         Computing the transpose puts a query row in ONE lane pair (l, l^32): max and sum need a
//         single cross-lane exchange, and the probabilities already sit in the B-operand layout.
//   O^T += V^T P^T (A = V^T from LDS, B = P).  P is split into a bf16 head and a bf16 remainder
//         (two MFMAs) so that the probabilities carry ~16 mantissa bits instead of 8; running
//         max / sum / rescale factors of a row live in the same lane as its accumulators.
#include "kernels.h"

namespace {

constexpr int DH = 128;
constexpr int QROWS = 128;
constexpr int KTILE = 64;
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

struct AttnArgs {
  const unsigned short* q;         // [T][Hq][128]
  const unsigned short* k_tree;    // [T][Hkv][128]
  const unsigned short* v_tree;
  const unsigned short* k_prefix;  // [P][Hkv][128]
  const unsigned short* v_prefix;
  const int* klist;                // [tiles][T]
  const int* kcnt;                 // [tiles]
  const unsigned long long* rowmask;  // [T][W64]
  unsigned short* out;             // [T][Hq][128]
  int T, P, Hq, Hkv, G, npt, W64;
};

__device__ __forceinline__ int ks_off(int key, int chunk) { return key * (DH * 2) + ((chunk ^ (key & 15)) << 4); }
__device__ __forceinline__ int vt_off(int d, int chunk) { return d * (KTILE * 2) + ((chunk ^ ((d ^ (d >> 3)) & 7)) << 4); }

typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned cvt_pk_bf16(float lo, float hi) {  // one v_cvt_pk_bf16_f32
  f32x2 t = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2));
}

__global__ __launch_bounds__(kThreads, 2) void tree_attn_bf16_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) char Ks[KTILE * DH * 2];
  __shared__ __attribute__((aligned(16))) char Vt[DH * KTILE * 2];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int tile = blockIdx.x, kvh = blockIdx.y;
  const int n0 = tile * a.npt;

  // ---- this lane's query row -----------------------------------------------------------------------
  const int r = wave * 32 + l32;
  const int node = n0 + r / a.G;
  const int head = kvh * a.G + r % a.G;
  const bool row_ok = node < a.T;
  bf16x8 qf[8];
  {
    const unsigned short* qp = a.q + ((size_t)(row_ok ? node : 0) * a.Hq + head) * DH + lh * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 t = {0u, 0u, 0u, 0u};
      if (row_ok) t = *reinterpret_cast<const u32x4*>(qp + ks * 16);
      qf[ks] = __builtin_bit_cast(bf16x8, t);
    }
  }
  const int cnt = a.kcnt[tile];
  const int nPre = (a.P + KTILE - 1) / KTILE;
  const int nTree = (cnt + KTILE - 1) / KTILE;
  const int* kl = a.klist + (size_t)tile * a.T;
  const unsigned long long* rm = a.rowmask + (size_t)(row_ok ? node : 0) * a.W64;
  const unsigned rowB = (unsigned)a.Hkv * DH * 2;  // bytes between consecutive key rows

  // ---- staging registers for the next tile ------------------------------------------------------------
  // K: lane fetches the 16-byte chunk (tid & 15) of keys (tid >> 4) + 16 i.  V: wave w fetches, for
  // the 16 key slots it transposes, the 4-byte column pair `lane` of each.  Slots past the end of
  // the key list re-read the last valid key (finite data); the mask keeps them out of the softmax.
  u32x4 rk[4];
  unsigned rv[2][8];
  unsigned long long rmask = 0ull;
  const unsigned kcol = (unsigned)kvh * DH * 2 + (tid & 15) * 16;
  const unsigned vcol = (unsigned)kvh * DH * 2 + lane * 4;
  auto fetch_prefix = [&](int t) {
    const int base = t * KTILE;
    const int last = a.P - 1;
    const char* kb = reinterpret_cast<const char*>(a.k_prefix);
    const char* vb = reinterpret_cast<const char*>(a.v_prefix);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = min(base + (tid >> 4) + 16 * i, last);
      rk[i] = *reinterpret_cast<const u32x4*>(kb + (size_t)((unsigned)row * rowB + kcol));
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = min(base + 16 * wave + (j >> 2) * 8 + 4 * h + (j & 3), last);
        rv[h][j] = *reinterpret_cast<const unsigned*>(vb + (size_t)((unsigned)row * rowB + vcol));
      }
    const int count = min(KTILE, a.P - base);
    rmask = count == KTILE ? ~0ull : ((1ull << count) - 1ull);
  };
  auto fetch_tree = [&](int t) {
    const int base = t * KTILE;
    const int last = cnt - 1;
    const char* kb = reinterpret_cast<const char*>(a.k_tree);
    const char* vb = reinterpret_cast<const char*>(a.v_tree);
    int krow[4], vrow[2][8];
#pragma unroll
    for (int i = 0; i < 4; ++i) krow[i] = kl[min(base + (tid >> 4) + 16 * i, last)];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 8; ++j) vrow[h][j] = kl[min(base + 16 * wave + (j >> 2) * 8 + 4 * h + (j & 3), last)];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      rk[i] = *reinterpret_cast<const u32x4*>(kb + (size_t)((unsigned)krow[i] * rowB + kcol));
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        rv[h][j] = *reinterpret_cast<const unsigned*>(vb + (size_t)((unsigned)vrow[h][j] * rowB + vcol));
    rmask = row_ok ? rm[t] : 0ull;
  };
  auto fetch = [&](int t) {
    if (t < nPre) fetch_prefix(t);
    else fetch_tree(t - nPre);
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(Ks + ks_off((tid >> 4) + 16 * i, tid & 15)) = rk[i];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u32x4 ev, od;  // d = 2*lane (low halves) and d = 2*lane+1 (high halves), 8 key slots each
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const unsigned w0 = rv[h][2 * p], w1 = rv[h][2 * p + 1];
        ev[p] = (w0 & 0xFFFFu) | (w1 << 16);
        od[p] = (w0 >> 16) | (w1 & 0xFFFF0000u);
      }
      *reinterpret_cast<u32x4*>(Vt + vt_off(2 * lane, 2 * wave + h)) = ev;
      *reinterpret_cast<u32x4*>(Vt + vt_off(2 * lane + 1, 2 * wave + h)) = od;
    }
  };

  // ---- running state of this lane's row ----------------------------------------------------------
  // m_ref is the reference the exponentials are taken against.  It follows the running maximum
  // lazily: only when a tile's maximum exceeds it by more than kSlack (in exponent bits) are the
  // accumulators rescaled, so probabilities stay below 2^kSlack and most tiles skip the rescale.
  const float NEG_INF = -__builtin_huge_valf();
  const float c2 = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)
  constexpr float kSlack = 8.0f;
  const float slack_raw = kSlack / c2;
  float m_ref = NEG_INF, l_run = 0.f;
  f32x16 oacc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;

  const int nTiles = nPre + nTree;
  if (nTiles > 0) fetch(0);
  for (int t = 0; t < nTiles; ++t) {
    __syncthreads();  // everyone is done reading the previous tile
    stash();
    const unsigned long long mask = rmask >> (4 * lh);
    __syncthreads();
    if (t + 1 < nTiles) fetch(t + 1);

    // ---- S^T = K Q^T : st[kb][e] = score(key 32kb + 8(e/4) + 4lh + e%4, this lane's row) --------------
    f32x16 st[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) st[kb][e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(Ks + ks_off(32 * kb + l32, 2 * ks + lh));
        st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], st[kb], 0, 0, 0);
      }
    }
    // ---- online softmax for this row ------------------------------------------------------------
    float mx = NEG_INF;
    if (mask != (~0ull >> (4 * lh))) {  // some key slots are not this row's: only tail and tree tiles
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int bit = 32 * kb + 8 * (e >> 2) + (e & 3);  // + 4*lh, already shifted out of `mask`
          st[kb][e] = ((mask >> bit) & 1ull) ? st[kb][e] : NEG_INF;
        }
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[kb][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    float alpha = 1.0f;
    if (mx > m_ref + slack_raw) {  // also taken on the first tile (m_ref = -inf)
      alpha = __builtin_amdgcn_exp2f((m_ref - mx) * c2);
      m_ref = mx;
    }
    const float m_use = (m_ref == NEG_INF) ? 0.f : m_ref;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
    }
    float psum = 0.f;
    bf16x8 phi[4], plo[4];
    const float mc = m_use * c2;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      u32x4 hi4, lo4;
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) {
        const float p0 = __builtin_amdgcn_exp2f(st[s4 >> 1][8 * (s4 & 1) + 2 * jp] * c2 - mc);
        const float p1 = __builtin_amdgcn_exp2f(st[s4 >> 1][8 * (s4 & 1) + 2 * jp + 1] * c2 - mc);
        psum += p0 + p1;
        const unsigned h2 = cvt_pk_bf16(p0, p1);
        hi4[jp] = h2;
        lo4[jp] = cvt_pk_bf16(p0 - __uint_as_float(h2 << 16), p1 - __uint_as_float(h2 & 0xFFFF0000u));
      }
      phi[s4] = __builtin_bit_cast(bf16x8, hi4);
      plo[s4] = __builtin_bit_cast(bf16x8, lo4);
    }
    l_run += psum;
    // ---- O^T += V^T P^T : oacc[db][e] = out(d = 32db + 8(e/4) + 4lh + e%4, this lane's row) ------------
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x8 vf = *reinterpret_cast<const bf16x8*>(Vt + vt_off(32 * db + l32, 2 * s4 + lh));
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, phi[s4], oacc[db], 0, 0, 0);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, plo[s4], oacc[db], 0, 0, 0);
      }
  }

  // ---- normalise and store -------------------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (row_ok && l_tot > 0.f) {
    const float inv = 1.0f / l_tot;
    unsigned short* op = a.out + ((size_t)node * a.Hq + head) * DH;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d = 32 * db + 8 * g + 4 * lh;
        u32x2 w;
        w[0] = cvt_pk_bf16(oacc[db][4 * g + 0] * inv, oacc[db][4 * g + 1] * inv);
        w[1] = cvt_pk_bf16(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
        *reinterpret_cast<u32x2*>(op + d) = w;
      }
  }
}

}  // namespace

int sx_launch_tree_attn_bf16(const void* q, const void* k_tree, const void* v_tree, const void* k_prefix,
                             const void* v_prefix, const int32_t* klist, const int32_t* kcnt,
                             const unsigned long long* rowmask, int T, int P, int Hq, int Hkv, void* out,
                             hipStream_t st) {
  const int G = Hq / Hkv;
  if (Hq % Hkv != 0 || !(G == 1 || G == 2 || G == 4 || G == 8)) return SX_ERR_SHAPE;
  AttnArgs a;
  a.q = static_cast<const unsigned short*>(q);
  a.k_tree = static_cast<const unsigned short*>(k_tree);
  a.v_tree = static_cast<const unsigned short*>(v_tree);
  a.k_prefix = static_cast<const unsigned short*>(k_prefix ? k_prefix : k_tree);
  a.v_prefix = static_cast<const unsigned short*>(v_prefix ? v_prefix : v_tree);
  a.klist = klist;
  a.kcnt = kcnt;
  a.rowmask = rowmask;
  a.out = static_cast<unsigned short*>(out);
  a.T = T;
  a.P = P;
  a.Hq = Hq;
  a.Hkv = Hkv;
  a.G = G;
  a.npt = QROWS / G;
  a.W64 = (T + 63) / 64;
  dim3 grid((T + a.npt - 1) / a.npt, Hkv);
  tree_attn_bf16_kernel<<<grid, kThreads, 0, st>>>(a);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
