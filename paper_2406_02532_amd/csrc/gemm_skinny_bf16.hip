// Y = X W^T for few rows (M <= 128): the linear layers of the draft model's forward over one batch of tree
// nodes (Alg. 2, forward(batch, theta_draft)).  At this M the product is bound by streaming the weights once
// from HBM, so the tile is narrow in N (128 x 64 per workgroup: many workgroups, each a different slice of W)
// and, where even that leaves compute units idle, K is cut as well and the partial sums are added up by the
// last workgroup to arrive, in a fixed order.  Same building blocks as the wide kernel: operands go global ->
// LDS by buffer loads that write LDS (whole 128-byte lines, chunk swizzle applied on the global side), three
// stages of K = 64, one barrier per stage, v_mfma_f32_16x16x32_bf16 with the product formed transposed so that
// a lane holds 4 consecutive output columns.
//
// What bounds it (7B shapes, 128 rows): 2.0-2.4 TB/s of weights from HBM, 3-6 TB/s out of the Infinity Cache.
// A plain load kernel walking the same 64 rows x 128 bytes per step streams the same matrix from HBM at 5 TB/s,
// and a fifth wave touching the weight lines 3 to 12 slabs ahead of the copies made every shape slower: HBM is
// not what the copies wait for.  With the copies of W taken out the kernel still takes 29 us of 54 (gate|up,
// warm), with those of X taken out 48: a 64-column tile copies all 128 rows of X again (16 KB per slab next to
// 8 KB of weights), so the L2 -> LDS stream carries three times the weight bytes with two slabs of lookahead.
// Hence the 128-column form below for wide matrices: 31 us for the same product.
#include "kernels.h"

namespace {

// A workgroup is NH groups of 4 waves; group h owns output columns 64 h .. 64 h + 63 of a 128 x 64 NH tile and all
// groups share the tile's X slab.  NH = 1: three stages of 24 KB, two workgroups per compute unit.  NH = 2: four
// stages of 32 KB, one workgroup of 8 waves: X is copied once for 128 columns instead of twice and the copies run
// three slabs ahead instead of two -- for wide matrices (many column tiles); narrow ones keep NH = 1, which gives
// twice as many workgroups to cut K among.
constexpr int BM = 128, BK = 64;
constexpr int kXBytes = BM * BK * 2;   // 16 KB
constexpr int kWBytes = 64 * BK * 2;   // 8 KB per group of 64 columns
constexpr int kWideMinSlabs = 40;

struct SkinnyArgs {
  const unsigned short* X;
  const unsigned short* W0;
  const unsigned short* W1;
  const unsigned short* W2;
  int n0, n1, n2;
  void* Y;
  int M, N, K;
  int tilesN, split;
  float* part;
  int* part_cnt;
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, -1, 0x00020000);
}

constexpr int kWaitVm0 = 0x0070, kWaitVm6 = 0x0076, kWaitVm8 = 0x0078;
#define SX_WAIT_BARRIER(IMM)              \
  asm volatile("" ::: "memory");          \
  __builtin_amdgcn_s_waitcnt(IMM);        \
  __builtin_amdgcn_s_barrier();           \
  asm volatile("" ::: "memory");

template <int MODE, int NH>
__global__ __launch_bounds__(256 * NH, 3 - NH) void gemm_skinny_bf16_kernel(SkinnyArgs a) {
  constexpr int BN = 64 * NH;
  constexpr int kStageBytes = kXBytes + NH * kWBytes;
  constexpr int kPartFloats = BM * BN;   // partial sums of one K part of one tile
  constexpr int kXCopies = 4 / NH;       // copy instructions (1 KB each) per wave and slab: X, then 2 for W
  // one array per stage: X rows then W rows, 128 bytes each, 16-byte chunk c of row r at position c ^ ((r >> 1) & 7)
  __shared__ __attribute__((aligned(1024))) unsigned char st0[kStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char st1[kStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char st2[kStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char st3[NH == 2 ? kStageBytes : 1024];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wh = wave >> 2, wm = (wave >> 1) & 1, wn = wave & 1;
  const int l16 = lane & 15, lq = lane >> 4;
  const int tile_n = blockIdx.x / a.split, kpart = blockIdx.x % a.split;

  // ---- copies: instruction t of wave w fills X rows 8 (kXCopies w + t) .. + 7 or W rows 16 w + 8 t .. + 7 (t < 2)
  const __amdgpu_buffer_rsrc_t xres = make_rsrc(a.X);
  const __amdgpu_buffer_rsrc_t wres0 = make_rsrc(a.W0), wres1 = make_rsrc(a.W1), wres2 = make_rsrc(a.W2);
  __amdgpu_buffer_rsrc_t wres[2];
  int xoff[4], woff[2];
#pragma unroll
  for (int t = 0; t < kXCopies; ++t) {
    const int cchunk = (lane & 7) ^ ((4 * (t & 1) + (lane >> 4)) & 7);
    int m = 8 * (kXCopies * wave + t) + (lane >> 3);
    m = m < a.M ? m : a.M - 1;
    xoff[t] = (int)(((unsigned)m * (unsigned)a.K + cchunk * 8) * 2u);
  }
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int cchunk = (lane & 7) ^ ((4 * (t & 1) + (lane >> 4)) & 7);
    if (MODE == SX_GEMM_SWIGLU) {
      // slab rows in 16-row groups, even = gate, odd = up: wave w copies group w
      int f = tile_n * (BN / 2) + (wave >> 1) * 16 + 8 * t + (lane >> 3);
      f = f < a.N ? f : a.N - 1;
      wres[t] = (wave & 1) ? wres1 : wres0;
      woff[t] = (int)(((unsigned)f * (unsigned)a.K + cchunk * 8) * 2u);
    } else {
      const int r0 = tile_n * BN + 16 * wave + 8 * t;
      const int g0 = min(r0, a.N - 1);  // first row of the 8-row group decides the matrix
      int n = min(r0 + (lane >> 3), a.N - 1);
      int first = 0;
      wres[t] = wres0;
      if (g0 >= a.n0 + a.n1) {
        wres[t] = wres2;
        first = a.n0 + a.n1;
      } else if (g0 >= a.n0) {
        wres[t] = wres1;
        first = a.n0;
      }
      woff[t] = (int)(((unsigned)(n - first) * (unsigned)a.K + cchunk * 8) * 2u);
    }
  }
#define SX_COPY(STG_, SLAB_)                                                                                     \
  {                                                                                                              \
    const int so = (SLAB_) * (BK * 2);                                                                           \
    _Pragma("unroll") for (int t = 0; t < kXCopies; ++t) __builtin_amdgcn_raw_ptr_buffer_load_lds(               \
        xres, (lds_void_ptr)(STG_ + (kXCopies * wave + t) * 1024), 16, xoff[t], so, 0, 0);                       \
    _Pragma("unroll") for (int t = 0; t < 2; ++t) __builtin_amdgcn_raw_ptr_buffer_load_lds(                      \
        wres[t], (lds_void_ptr)(STG_ + kXBytes + wave * 2048 + t * 1024), 16, woff[t], so, 0, 0);                \
  }

  // acc[i][j]: W rows (output columns) 64 wh + 32 wn + 16 i .. + 15, X rows (output rows) 64 wm + 16 j .. + 15
  f32x4 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  const int fsw = (l16 >> 1) & 7;
  const int xrow = (wm * 64 + l16) * (BK * 2);
  const int wrow = kXBytes + (wh * 64 + wn * 32 + l16) * (BK * 2);
  const int kc[2] = {(lq ^ fsw) << 4, ((4 + lq) ^ fsw) << 4};

// "+v": the accumulators stay where they are (see the wide kernel); statements are volatile, order as written
#define SX_MFMA(ACC, A, B) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(ACC) : "v"(A), "v"(B));
#define SX_SLAB(STG_, STG_F, SLAB_F)                                                                             \
  SX_WAIT_BARRIER(NH == 1 ? kWaitVm6 : kWaitVm8)                                                                 \
  SX_COPY(STG_F, SLAB_F)                                                                                         \
  _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                             \
    bf16x8 fx[4], fw[2];                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                                \
        fw[i] = *reinterpret_cast<const bf16x8*>(STG_ + wrow + i * (16 * BK * 2) + kc[ks]);                      \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                                \
        fx[j] = *reinterpret_cast<const bf16x8*>(STG_ + xrow + j * (16 * BK * 2) + kc[ks]);                      \
    _Pragma("unroll") for (int i = 0; i < 2; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)                  \
        SX_MFMA(acc[i][j], fw[i], fx[j])                                                                         \
  }

  // slabs [first, first + NB) of K; slab s sits in stage (s - first) % 3.  Iteration: wait for this wave's
  // copies of the current slab (those of the next may stay in flight), barrier (everybody's are in, everybody
  // is done with the previous slab), start the copies of the slab after next into the stage just freed.
  const int nb_all = a.K / BK;
  const int first = kpart * nb_all / a.split;
  const int NB = (kpart + 1) * nb_all / a.split - first, last = first + NB - 1;
  // (NH = 2: four stages, the copies of the next two slabs may stay in flight, those of the third go out)
  SX_COPY(st0, first)
  SX_COPY(st1, min(first + 1, last))
  int s = 0;
  if (NH == 1) {
    for (; s + 3 <= NB; s += 3) {
      SX_SLAB(st0, st2, min(first + s + 2, last))
      SX_SLAB(st1, st0, min(first + s + 3, last))
      SX_SLAB(st2, st1, min(first + s + 4, last))
    }
    if (s < NB) {
      SX_SLAB(st0, st2, last)
      if (s + 1 < NB) { SX_SLAB(st1, st0, last) }
    }
  } else {
    SX_COPY(st2, min(first + 2, last))
    for (; s + 4 <= NB; s += 4) {
      SX_SLAB(st0, st3, min(first + s + 3, last))
      SX_SLAB(st1, st0, min(first + s + 4, last))
      SX_SLAB(st2, st1, min(first + s + 5, last))
      SX_SLAB(st3, st2, min(first + s + 6, last))
    }
    if (s < NB) {
      SX_SLAB(st0, st3, last)
      if (s + 1 < NB) { SX_SLAB(st1, st0, last) }
      if (s + 2 < NB) { SX_SLAB(st2, st1, last) }
    }
  }
  __builtin_amdgcn_s_waitcnt(kWaitVm0);  // copies past the end of K must land before the LDS is released
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");  // the matrix pipe's last results (hand-written MFMAs)
#undef SX_SLAB
#undef SX_MFMA
#undef SX_COPY

  // ---- K split: partial sums meet in memory, the last workgroup to arrive adds them in part order -------------
  // (device-scope stores and loads, stores complete before the counter's atomic: see the wide kernel)
  if (a.split > 1) {
    constexpr int kScopeDevice = 16;
    __shared__ int s_last;
    const __amdgpu_buffer_rsrc_t pres = make_rsrc(a.part);
    const unsigned mine = (unsigned)((tile_n * a.split + kpart) * kPartFloats + wave * (8 * 256) + lane * 4) * 4u;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[i][j]), pres, mine + (i * 4 + j) * 1024, 0,
                                               kScopeDevice);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __syncthreads();
    if (tid == 0) {
      const int before = atomicAdd(a.part_cnt + tile_n, 1);
      s_last = before == a.split - 1;
      if (s_last) a.part_cnt[tile_n] = 0;
    }
    __syncthreads();
    if (!s_last) return;
    // all 8 blocks of a part are requested together (one memory round trip per part, not one per block); the
    // workgroup's own part comes from its registers (the same bits it stored); parts are added in part order
    const unsigned all = (unsigned)(tile_n * a.split * kPartFloats + wave * (8 * 256) + lane * 4) * 4u;
    f32x4 sum[8];
    for (int p = 0; p < a.split; ++p) {
      f32x4 t[8];
      if (p == kpart) {
#pragma unroll
        for (int b = 0; b < 8; ++b) t[b] = acc[b >> 2][b & 3];
      } else {
#pragma unroll
        for (int b = 0; b < 8; ++b)
          t[b] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                               pres, all + (unsigned)p * (kPartFloats * 4u) + b * 1024, 0, kScopeDevice));
      }
#pragma unroll
      for (int b = 0; b < 8; ++b) sum[b] = p == 0 ? t[b] : sum[b] + t[b];
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[b >> 2][b & 3] = sum[b];
  }

  // ---- epilogue.  acc[i][j][e]: output row 64 wm + 16 j + l16, W row 32 wn + 16 i + 4 lq + e ------------------
  const bool vec = (a.N & 3) == 0;
  if (MODE == SX_GEMM_SWIGLU) {
    unsigned short* Y = static_cast<unsigned short*>(a.Y);
    const int f = tile_n * (BN / 2) + (2 * wh + wn) * 16 + 4 * lq;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = wm * 64 + 16 * j + l16;
      if (m >= a.M || f >= a.N) continue;
      unsigned short h[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float g = acc[0][j][e], u = acc[1][j][e];
        h[e] = (unsigned short)f32_to_bf16_bits(silu_mul_bf16_bound(g, u));
      }
      unsigned short* y = Y + (size_t)m * a.N + f;
      if (vec) {
        u32x2 v;
        v[0] = h[0] | ((uint32_t)h[1] << 16);
        v[1] = h[2] | ((uint32_t)h[3] << 16);
        *reinterpret_cast<u32x2*>(y) = v;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (f + e < a.N) y[e] = h[e];
      }
    }
  } else if (vec && tile_n * BN + BN <= a.N) {
    // whole column tile: the residual of all 8 blocks is requested before the first add (rows past M read row M - 1
    // and store nothing); block by block the epilogue was 8 memory round trips long
    float* Yb = static_cast<float*>(a.Y) + (tile_n * BN + wh * 64 + wn * 32 + 4 * lq);
    f32x4 r[4][2];
    if (MODE == SX_GEMM_RESIDUAL) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i)
          r[j][i] = *reinterpret_cast<const f32x4*>(Yb + (size_t)min(wm * 64 + 16 * j + l16, a.M - 1) * a.N + 16 * i);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = wm * 64 + 16 * j + l16;
      if (m >= a.M) continue;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        f32x4 v = acc[i][j];
        if (MODE == SX_GEMM_RESIDUAL) v += r[j][i];
        *reinterpret_cast<f32x4*>(Yb + (size_t)m * a.N + 16 * i) = v;
      }
    }
  } else {
    float* Y = static_cast<float*>(a.Y);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = wm * 64 + 16 * j + l16;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int n = tile_n * BN + wh * 64 + wn * 32 + 16 * i + 4 * lq;
        if (m >= a.M || n >= a.N) continue;
        float* y = Y + (size_t)m * a.N + n;
        if (vec) {
          f32x4 v = acc[i][j];
          if (MODE == SX_GEMM_RESIDUAL) v += *reinterpret_cast<const f32x4*>(y);
          *reinterpret_cast<f32x4*>(y) = v;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < a.N) {
              if (MODE == SX_GEMM_RESIDUAL) y[e] += acc[i][j][e];
              else y[e] = acc[i][j][e];
            }
        }
      }
    }
  }
}
#undef SX_WAIT_BARRIER


}  // namespace

// M <= 128.  Arguments as sx_launch_gemm_bf16 (modes store, residual, SwiGLU).
int sx_launch_gemm_skinny_bf16(const void* X, const void* W0, const void* W1, const void* W2, int n0, int n1, int n2,
                               void* Y, int M, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st) {
  if (M < 1 || M > BM || K < BK || K % BK != 0 || n0 < 1 || n1 < 0 || n2 < 0) return SX_ERR_SHAPE;
  if (!sx_operand_fits_u32(M, 2ll * K) || !sx_operand_fits_u32(n0, 2ll * K) || !sx_operand_fits_u32(n1, 2ll * K) ||
      !sx_operand_fits_u32(n2, 2ll * K))
    return SX_ERR_SHAPE;
  if (mode != SX_GEMM_SWIGLU && ((n1 > 0 && n0 % 8 != 0) || (n2 > 0 && n1 % 8 != 0))) return SX_ERR_SHAPE;
  SkinnyArgs a;
  a.X = static_cast<const unsigned short*>(X);
  a.W0 = static_cast<const unsigned short*>(W0);
  a.W1 = static_cast<const unsigned short*>(W1 ? W1 : W0);
  a.W2 = static_cast<const unsigned short*>(W2 ? W2 : W0);
  a.n0 = n0;
  a.n1 = n1;
  a.n2 = n2;
  a.Y = Y;
  a.M = M;
  a.K = K;
  int cols;  // rows of W that a launch walks (gate and up both count)
  if (mode == SX_GEMM_SWIGLU) {
    if (n1 != n0 || n2 != 0 || !W1) return SX_ERR_SHAPE;
    a.N = n0;
    cols = 2 * n0;
  } else {
    a.N = n0 + n1 + n2;
    cols = a.N;
  }
  // Cut K only while there are fewer tiles than compute units (measured: with a tile per unit or more the extra
  // parts cost more in partial sums and short K loops than they gain), parts of at least 4 slabs, and only as
  // far as the caller's memory for partial sums (and its 256 counters) goes.
  // 128-column tiles (8 waves) where they need no cut or the parts of the cut stay long (40 slabs: the 7B QKV
  // projection, cut in two parts of 32, is better off with 192 uncut 64-column tiles; the 70B one, three parts of
  // 42, is not); otherwise twice as many 64-column tiles.
  const int slots = sx_compute_units(), nb = K / BK;
  auto plan = [&](int bn, int& tiles, int& split) {
    tiles = (cols + bn - 1) / bn;
    split = 1;
    if (split_ws && tiles <= 256 && 2 * tiles <= slots) {
      split = slots / tiles;
      if (split > 8) split = 8;
      while (split > 1 && nb / split < 4) --split;
      if (split_ws_bytes < 1024 + (size_t)tiles * split * BM * bn * sizeof(float)) split = 1;
    }
  };
  int nh = 1, tiles = 0, split = 1;
  if (cols >= 128) {
    plan(128, tiles, split);
    if (split == 1 ? 2 * tiles > slots : nb / split >= kWideMinSlabs) nh = 2;
  }
  if (nh == 1) plan(64, tiles, split);
  a.tilesN = tiles;
  a.split = split;
  a.part = nullptr;
  a.part_cnt = nullptr;
  if (split > 1) {
    a.part_cnt = static_cast<int*>(split_ws);
    a.part = reinterpret_cast<float*>(static_cast<char*>(split_ws) + 1024);
  }
  const int grid = a.tilesN * a.split;
#define SX_GO(MODE_)                                                                    \
  if (nh == 2) gemm_skinny_bf16_kernel<MODE_, 2><<<grid, 512, 0, st>>>(a);              \
  else gemm_skinny_bf16_kernel<MODE_, 1><<<grid, 256, 0, st>>>(a);
  switch (mode) {
    case SX_GEMM_STORE: SX_GO(SX_GEMM_STORE) break;
    case SX_GEMM_RESIDUAL: SX_GO(SX_GEMM_RESIDUAL) break;
    case SX_GEMM_SWIGLU: SX_GO(SX_GEMM_SWIGLU) break;
    default: return SX_ERR_SHAPE;
  }
#undef SX_GO
  SX_LAUNCH_CHECK();
  return SX_OK;
}
