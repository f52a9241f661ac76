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
//   K and V rows -> LDS by buffer loads that write LDS directly (no staging registers, no LDS-write
//         instructions, nothing to transpose by hand: staging through registers and packing V^T
//         with bit operations was 46% of the kernel's time).  Both tiles are [key][128 d] rows of
//         256 bytes, two stages each, one barrier per tile.  16-byte chunks are XOR-swizzled, K by
//         key & 15 and V by (key & 3) << 2, each conflict-free for the way it is read; the
//         swizzle is applied on the global side (a wave's 1 KB of LDS per instruction is contiguous).
//   S^T = K Q^T   (MFMA 32x32x16: A = K from LDS, B = Q held in registers for the whole kernel).
//         Computing the transpose puts a query row in ONE lane pair (l, l^32): max and sum need a
//         single cross-lane exchange, and the probabilities already sit in the B-operand layout.
//   O^T += V^T P^T (A = V^T, B = P).  V^T fragments come out of the row-major V tile through the
//         LDS transpose read (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i % 4 of
//         the 8 bytes addressed by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4): lane s of a
//         group points at V[key0 + s / 4][d0 + 4 (s % 4) ..], lane i receives V[key0 .. key0 + 3][d0 + i].
//         P is split into a bf16 head and a bf16 remainder (two MFMAs) so that the probabilities
//         carry ~16 mantissa bits instead of 8: an error of 1e-4 relative before the output's bf16
//         rounding flips ~7% of those roundings against a correctly rounded reference.  Running
//         max / sum / rescale factors of a row live in the same lane as its accumulators.
#include "kernels.h"

namespace {

constexpr int DH = 128;
constexpr int QROWS = 128;
constexpr int KTILE = 64;
constexpr int kThreads = 256;
constexpr int kTileBytes = KTILE * DH * 2;  // 16 KB: one K or V tile
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
  int T, Tq, P, Hq, Hkv, G, npt, W64;  // T: nodes of the tree (klist stride); Tq: query nodes in q/out
  // splits > 1: blockIdx.z takes a contiguous share of the key tiles and leaves, per query row, its
  // unnormalised output, reference maximum and sum for attn_combine_kernel
  int splits;
  float *part_o, *part_m, *part_l;  // [splits][Tq * Hq][128], [splits][Tq * Hq] x 2
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, -1, 0x00020000);
}
__device__ __forceinline__ int ks_off(int key, int chunk) { return key * (DH * 2) + ((chunk ^ (key & 15)) << 4); }

typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned cvt_pk_bf16(float lo, float hi) {  // one v_cvt_pk_bf16_f32
  f32x2 t = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2));
}

// nothing is scheduled across this point (keeps the fragment reads of a tile ahead of its first MFMA)
#define SX_ATT_SCHED_BARRIER __builtin_amdgcn_sched_barrier(0);
// maximum of a value over the lane pair (l, l ^ 32): one lane-half swap inside the vector unit, no LDS round trip
__device__ __forceinline__ float pair_max(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
#define SX_ATT_XMAX(x) pair_max(x)
// s_waitcnt: all vector-memory operations (the copies) and all LDS reads of this wave done
constexpr int kWaitAll = 0x0070;
// The barrier intrinsic does not order memory operations for the compiler, and a workgroup fence would be
// heavier than needed; empty asm statements that claim to touch memory pin LDS reads and copies to their side.
#define SX_WAIT_BARRIER()                  \
  asm volatile("" ::: "memory");           \
  __builtin_amdgcn_s_waitcnt(kWaitAll);    \
  __builtin_amdgcn_s_barrier();            \
  asm volatile("" ::: "memory");

__global__ __launch_bounds__(kThreads, 2) void tree_attn_bf16_kernel(AttnArgs a) {
  // one array per stage and operand: the compiler tracks loads-to-LDS per array, so reads of the stage in
  // use do not wait for the copies in flight to the other
  __shared__ __attribute__((aligned(1024))) char K0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char K1[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char V0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char V1[kTileBytes];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  With a multiple of 8 KV heads
  // every XCD takes the heads congruent to its number, one after the other, all query tiles of a head
  // before the next: the K/V rows of a head are then fetched into one L2 only, and the workgroups that
  // run there side by side all read them.
  int tile = blockIdx.x, kvh = blockIdx.y;
  if ((gridDim.y & 7) == 0) {
    const int lin = blockIdx.x + gridDim.x * blockIdx.y, j = lin >> 3;
    tile = j % gridDim.x;
    kvh = ((j / gridDim.x) << 3) + (lin & 7);
  }
  const int n0 = tile * a.npt;

  // ---- this lane's query row -----------------------------------------------------------------------
  const int r = wave * 32 + l32;
  const int node = n0 + r / a.G;
  const int head = kvh * a.G + r % a.G;
  const bool row_ok = node < a.Tq && r / a.G < a.npt;  // tiles of fewer than 128 rows leave waves without rows
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

  // ---- copies: global -> LDS ---------------------------------------------------------------------------
  // Copy instruction t (0..3) of wave w fills tile rows 16 w + 4 t .. + 3 (1 KB of LDS): lane l supplies
  // row 16 w + 4 t + l / 16, LDS chunk position l % 16, i.e. the chunk that the swizzle puts there.
  // Slots past the end of the key list re-read the last valid key (finite data); the mask keeps them
  // out of the softmax.
  const __amdgpu_buffer_rsrc_t kpre = make_rsrc(a.k_prefix), vpre = make_rsrc(a.v_prefix);
  const __amdgpu_buffer_rsrc_t ktre = make_rsrc(a.k_tree), vtre = make_rsrc(a.v_tree);
  const int crow = 16 * wave + (lane >> 4);               // + 4 t
  const unsigned colB = (unsigned)kvh * DH * 2;
  unsigned kcol[4];                                        // byte offset of the K chunk inside the row, per t
#pragma unroll
  for (int t = 0; t < 4; ++t) kcol[t] = colB + ((((unsigned)lane & 15u) ^ ((4u * t + ((unsigned)lane >> 4)) & 15u)) << 4);
  const unsigned vcol = colB + ((((unsigned)lane & 15u) ^ ((((unsigned)lane >> 4) & 3u) << 2)) << 4);
  const int cdst = wave * 4096;
  unsigned long long rmask = 0ull;

#define SX_COPY_TILE(KS_, VS_, KRES_, VRES_, ROWOFF_)                                                              \
  _Pragma("unroll") for (int t = 0; t < 4; ++t) {                                                                  \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(KRES_, (lds_void_ptr)(KS_ + cdst + t * 1024), 16, ROWOFF_[t] + kcol[t], 0, 0, \
                                             0);                                                                   \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(VRES_, (lds_void_ptr)(VS_ + cdst + t * 1024), 16, ROWOFF_[t] + vcol, 0, 0, 0); \
  }
// starts the copies of tile T_ (prefix tiles first, then tree tiles) into stage (KS_, VS_) and sets rmask
#define SX_FETCH(T_, KS_, VS_)                                                                                     \
  if ((T_) < nPre) {                                                                                               \
    const int base = (T_) * KTILE, last = a.P - 1;                                                                 \
    unsigned roff[4];                                                                                              \
    _Pragma("unroll") for (int t = 0; t < 4; ++t) roff[t] = (unsigned)min(base + crow + 4 * t, last) * rowB;       \
    SX_COPY_TILE(KS_, VS_, kpre, vpre, roff)                                                                       \
    const int count = min(KTILE, a.P - base);                                                                      \
    rmask = count == KTILE ? ~0ull : ((1ull << count) - 1ull);                                                     \
  } else {                                                                                                         \
    const int base = ((T_) - nPre) * KTILE, last = cnt - 1;                                                        \
    unsigned roff[4];                                                                                              \
    _Pragma("unroll") for (int t = 0; t < 4; ++t) roff[t] = (unsigned)kl[min(base + crow + 4 * t, last)] * rowB;   \
    SX_COPY_TILE(KS_, VS_, ktre, vtre, roff)                                                                       \
    rmask = row_ok ? rm[(T_) - nPre] : 0ull;                                                                       \
  }

  // ---- V^T fragment addresses (transpose read) -----------------------------------------------------------
  // Fragment (db, s4) for lane l: d = 32 db + l32, the 8 keys 16 s4 + 4 lh + {0..3} and + 8 (the order
  // in which this lane's probabilities sit in the P operand).  Lane s = l % 16 of the 16-lane group
  // q = l / 16 addresses key 16 s4 + 8 r + 4 lh + s / 4, d = 32 db + 16 (q % 2) + 4 (s % 4) .. + 3.
  const int vs = lane & 15, vq = lane >> 4;
  const int vkey = 4 * lh + (vs >> 2);                             // + 16 s4 + 8 r
  const int vbase = vkey * (DH * 2) + 8 * (vs & 1);                // row and the 8-byte half of the chunk
  const int vchunk = 2 * (vq & 1) + ((vs & 3) >> 1);               // + 4 db
  const int vswz = (vkey & 3) << 2;
  int vpc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) vpc[db] = vbase + (((4 * db + vchunk) ^ vswz) << 4);

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

// one key tile out of stage (KS_, VS_); `mask` = which of its 64 slots belong to this lane's row (bits of
// the lane half already shifted out)
#define SX_TILE(KS_, VS_)                                                                                          \
  {                                                                                                                \
    /* ---- S^T = K Q^T : st[kb][e] = score(key 32kb + 8(e/4) + 4lh + e%4, this lane's row) ---- */               \
    f32x16 st[2];                                                                                                  \
    {                                                                                                              \
      /* all 16 fragment reads go out before the first MFMA: one LDS latency per tile instead of one per MFMA */   \
      bf16x8 kfa[8], kfb[8];                                                                                       \
      _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)                                                             \
          kfa[ks] = *reinterpret_cast<const bf16x8*>(KS_ + ks_off(l32, 2 * ks + lh));                              \
      _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)                                                             \
          kfb[ks] = *reinterpret_cast<const bf16x8*>(KS_ + ks_off(32 + l32, 2 * ks + lh));                         \
      SX_ATT_SCHED_BARRIER                                                                                         \
      _Pragma("unroll") for (int e = 0; e < 16; ++e) st[0][e] = st[1][e] = 0.f;                                    \
      _Pragma("unroll") for (int ks = 0; ks < 8; ++ks) {                                                           \
        st[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfa[ks], qf[ks], st[0], 0, 0, 0);                          \
        st[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfb[ks], qf[ks], st[1], 0, 0, 0);                          \
      }                                                                                                            \
    }                                                                                                              \
    /* ---- online softmax for this row ---- */                                                                    \
    float mx = NEG_INF;                                                                                            \
    if (mask != (~0ull >> (4 * lh))) { /* some key slots are not this row's: only tail and tree tiles */           \
      _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int e = 0; e < 16; ++e) {            \
        const int bit = 32 * kb + 8 * (e >> 2) + (e & 3); /* + 4*lh, already shifted out of `mask` */              \
        st[kb][e] = ((mask >> bit) & 1ull) ? st[kb][e] : NEG_INF;                                                  \
      }                                                                                                            \
    }                                                                                                              \
    _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int e = 0; e < 16; ++e)                \
        mx = fmaxf(mx, st[kb][e]);                                                                                 \
    mx = SX_ATT_XMAX(mx);                                                                                          \
    float alpha = 1.0f;                                                                                            \
    if (mx > m_ref + slack_raw) { /* also taken on the first tile (m_ref = -inf) */                                \
      alpha = __builtin_amdgcn_exp2f((m_ref - mx) * c2);                                                           \
      m_ref = mx;                                                                                                  \
    }                                                                                                              \
    const float m_use = (m_ref == NEG_INF) ? 0.f : m_ref;                                                          \
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {                                                      \
      l_run *= alpha;                                                                                              \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) _Pragma("unroll") for (int e = 0; e < 16; ++e)                 \
          oacc[i][e] *= alpha;                                                                                     \
    }                                                                                                              \
    float psum = 0.f;                                                                                              \
    bf16x8 phi[4], plo[4];                                                                                         \
    const float mc = m_use * c2;                                                                                   \
    _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) {                                                             \
      u32x4 hi4, lo4;                                                                                              \
      _Pragma("unroll") for (int jp = 0; jp < 4; ++jp) {                                                           \
        const float p0 = __builtin_amdgcn_exp2f(st[s4 >> 1][8 * (s4 & 1) + 2 * jp] * c2 - mc);                     \
        const float p1 = __builtin_amdgcn_exp2f(st[s4 >> 1][8 * (s4 & 1) + 2 * jp + 1] * c2 - mc);                 \
        psum += p0 + p1;                                                                                           \
        const unsigned h2 = cvt_pk_bf16(p0, p1);                                                                   \
        hi4[jp] = h2;                                                                                              \
        lo4[jp] = cvt_pk_bf16(p0 - __uint_as_float(h2 << 16), p1 - __uint_as_float(h2 & 0xFFFF0000u));             \
      }                                                                                                            \
      phi[s4] = __builtin_bit_cast(bf16x8, hi4);                                                                   \
      plo[s4] = __builtin_bit_cast(bf16x8, lo4);                                                                   \
    }                                                                                                              \
    l_run += psum;                                                                                                 \
    /* ---- O^T += V^T P^T : oacc[db][e] = out(d = 32db + 8(e/4) + 4lh + e%4, this lane's row) ---- */             \
    _Pragma("unroll") for (int s4 = 0; s4 < 4; ++s4) _Pragma("unroll") for (int db = 0; db < 4; ++db) {            \
      const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(VS_ + s4 * 4096 + vpc[db]));        \
      const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(VS_ + s4 * 4096 + 2048 + vpc[db])); \
      const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));       \
      oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, phi[s4], oacc[db], 0, 0, 0);                          \
      oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, plo[s4], oacc[db], 0, 0, 0);                          \
    }                                                                                                              \
  }

  // Tile t lives in stage t % 2.  Top of an iteration: wait for this wave's copies of tile t, barrier
  // (everybody's are in, and everybody is done with tile t-1, whose stage the copies of tile t+1 go to).
  const int nAll = nPre + nTree;
  const int tBeg = (int)((long long)blockIdx.z * nAll / a.splits);   // this workgroup's share of the key tiles
  const int nTiles = (int)((long long)(blockIdx.z + 1) * nAll / a.splits);
  if (tBeg < nTiles) { SX_FETCH(tBeg, K0, V0) }
  for (int t = tBeg; t < nTiles; t += 2) {
    {
      SX_WAIT_BARRIER()
      const unsigned long long mask = rmask >> (4 * lh);
      if (t + 1 < nTiles) { SX_FETCH(t + 1, K1, V1) }
      SX_TILE(K0, V0)
    }
    if (t + 1 < nTiles) {
      SX_WAIT_BARRIER()
      const unsigned long long mask = rmask >> (4 * lh);
      if (t + 2 < nTiles) { SX_FETCH(t + 2, K0, V0) }
      SX_TILE(K1, V1)
    }
  }
#undef SX_TILE
#undef SX_FETCH
#undef SX_COPY_TILE
#undef SX_WAIT_BARRIER

  // ---- normalise and store -------------------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (a.splits > 1) {
    if (row_ok) {
      const size_t qrow = (size_t)node * a.Hq + head, nrow = (size_t)a.Tq * a.Hq;
      float* po = a.part_o + ((size_t)blockIdx.z * nrow + qrow) * DH;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 w = {oacc[db][4 * g + 0], oacc[db][4 * g + 1], oacc[db][4 * g + 2], oacc[db][4 * g + 3]};
          *reinterpret_cast<f32x4*>(po + 32 * db + 8 * g + 4 * lh) = w;
        }
      if (lh == 0) {
        a.part_m[(size_t)blockIdx.z * nrow + qrow] = m_ref;
        a.part_l[(size_t)blockIdx.z * nrow + qrow] = l_tot;
      }
    }
    return;
  }
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

// out[row][d] = sum_z O_z[row][d] 2^((m_z - M) c) / sum_z l_z 2^((m_z - M) c), M = max_z m_z: the softmax over all
// keys put together from the shares of the key tiles (m_z = -inf, l_z = 0 for a share without keys of the row)
__global__ __launch_bounds__(128) void attn_combine_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_m,
                                                           const float* __restrict__ part_l, int splits, int nrow,
                                                           unsigned short* __restrict__ out) {
  const int row = blockIdx.x, d = threadIdx.x;
  const float c2 = kLog2e * 0.08838834764831845f;
  float M = -__builtin_huge_valf();
  for (int z = 0; z < splits; ++z) M = fmaxf(M, part_m[(size_t)z * nrow + row]);
  float num = 0.f, den = 0.f;
  for (int z = 0; z < splits; ++z) {
    const float m = part_m[(size_t)z * nrow + row];
    if (m == -__builtin_huge_valf()) continue;
    const float wgt = __builtin_amdgcn_exp2f((m - M) * c2);
    num += part_o[((size_t)z * nrow + row) * DH + d] * wgt;
    den += part_l[(size_t)z * nrow + row] * wgt;
  }
  out[(size_t)row * DH + d] = den > 0.f ? (unsigned short)f32_to_bf16_bits(num / den) : (unsigned short)0;
}

}  // namespace

size_t sx_tree_attn_split_workspace(int Tq_max, int Hq) {
  return (size_t)8 * Tq_max * Hq * (DH + 2) * sizeof(float);
}

int sx_launch_tree_attn_bf16(const void* q, const void* k_tree, const void* v_tree, const void* k_prefix,
                             const void* v_prefix, const int32_t* klist, const int32_t* kcnt,
                             const unsigned long long* rowmask, int T, int Tq, int P, int Hq, int Hkv, void* out,
                             void* split_ws, size_t split_ws_bytes, hipStream_t st) {
  const int G = Hq / Hkv;
  if (Hq % Hkv != 0 || !(G == 1 || G == 2 || G == 4 || G == 8)) return SX_ERR_SHAPE;
  // the copies address rows with 32-bit byte offsets from the start of each K/V array
  if ((unsigned long long)(P > T ? P : T) * Hkv * DH * 2 >= (1ull << 32)) return SX_ERR_SHAPE;
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
  a.Tq = Tq;
  a.P = P;
  a.Hq = Hq;
  a.Hkv = Hkv;
  a.G = G;
  a.npt = sx_attn_nodes_per_tile(Hq, Hkv, Tq);  // the same value the tile lists were built with
  a.W64 = (T + 63) / 64;
  dim3 grid((Tq + a.npt - 1) / a.npt, Hkv);
  // few query rows (a batch of the draft model): the grid leaves most of the chip idle while each workgroup
  // walks all key tiles one after the other; give shares of the key tiles to up to 8 workgroups instead
  a.splits = 1;
  a.part_o = a.part_m = a.part_l = nullptr;
  const int wgs = (int)(grid.x * grid.y), npre = (P + KTILE - 1) / KTILE;
  if (split_ws && wgs < 256 && npre >= 4) {
    int s = 512 / wgs;
    if (s > 8) s = 8;
    if (s > npre / 2) s = npre / 2;
    const size_t nrow = (size_t)Tq * Hq;
    if (s > 1 && split_ws_bytes >= (size_t)s * nrow * (DH + 2) * sizeof(float)) {
      a.splits = s;
      a.part_o = static_cast<float*>(split_ws);
      a.part_m = a.part_o + (size_t)s * nrow * DH;
      a.part_l = a.part_m + (size_t)s * nrow;
    }
  }
  grid.z = a.splits;
  tree_attn_bf16_kernel<<<grid, kThreads, 0, st>>>(a);
  SX_LAUNCH_CHECK();
  if (a.splits > 1) {
    attn_combine_kernel<<<Tq * Hq, 128, 0, st>>>(a.part_o, a.part_m, a.part_l, a.splits, Tq * Hq, a.out);
    SX_LAUNCH_CHECK();
  }
  return SX_OK;
}
