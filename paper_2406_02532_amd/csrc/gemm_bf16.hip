// Y = X W^T on the gfx950 matrix cores: the linear layers of the decoder forward (Alg. 1, FORWARD) at
// M = number of tree tokens.  bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16).
//
// Tiling.  A workgroup of 4 waves (2 x 2) owns a 256 x 256 output tile; each wave a 128 x 128
// quadrant = 4 x 4 MFMA blocks, 256 fp32 accumulators per lane.  K is walked in slabs of 32 (two
// k-steps of 16 = 32 MFMAs per wave), held in a ring of 4 LDS stages (4 x 32 KB).  Global memory is
// read 64 K-elements at a time (whole 128-byte lines) into one of two register sets, three slab
// pairs ahead of use, and written to LDS one pair ahead.  Because a slab's data is complete in LDS
// a full slab before it is needed, the fragments of its first k-step are read before the barrier
// that precedes it, so no LDS latency is exposed at slab boundaries.  Both operands are
// K-contiguous in memory, which is exactly the per-lane layout the MFMA wants (8 consecutive k per
// lane), so LDS rows are plain 64-byte row segments with an XOR swizzle of the 16-byte chunk index
// that is conflict-free for the 64-bank LDS (measured ~220 B/clk per CU against ~140 for a naive one).
//
// XCD-aware tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.
// Tile index = xcd * chunk + id / 8 with tiles ordered M-fastest, so the workgroups resident on
// one XCD at a time share the same few W column tiles (fetched from HBM once per XCD) and sweep
// all of X's row tiles.
//
// Epilogues: store fp32, add into an fp32 residual, or SwiGLU.  For SwiGLU the W slab interleaves
// 32-row groups of W_gate and W_up, so gate and up of one output column sit in the same lane and
// register of neighbouring accumulator blocks and silu(g)*u needs no data movement.
#include "kernels.h"

namespace {

constexpr int BM = 256, BN = 256;
constexpr int BK = 64;                    // K elements fetched from global memory at a time (full 128-byte lines)
constexpr int SK = 32;                    // K elements per LDS stage ("slab"): two k-steps of 16
constexpr int kThreads = 256;
constexpr int kOperandBytes = BM * SK * 2;            // 16 KB: one operand of one slab
constexpr int kStageStride = 2 * kOperandBytes + 128; // X slab, W slab, and a 128-byte skew (see stash)
constexpr int kStages = 4;
constexpr int kLdsBytes = kStages * kStageStride;

struct GemmArgs {
  const unsigned short* X;
  const unsigned short* W0;
  const unsigned short* W1;
  const unsigned short* W2;
  int n0, n1, n2;
  void* Y;
  int M, N, K;  // N = logical output columns
  int tilesM, tilesN, chunk;
};

// Byte offset of 16-byte chunk `c4` (0..3) of row `row` inside one operand of a slab.  Rows are 64 bytes;
// the chunk index is XORed with (row >> 2) & 3.  The LDS serves 16 lanes x 16 bytes per cycle (64 banks):
// 16 consecutive rows reading the same k chunk then fall on 16 different bank groups
// ((row & 3) * 4 + (c4 ^ (row >> 2) & 3) takes 16 distinct values).
// Raw buffer resource over a whole matrix (no bounds: rows are clamped by the caller; < 4 GB).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, -1, 0x00020000);
}
__device__ __forceinline__ int lds_off(int row, int c4) { return row * (SK * 2) + ((c4 ^ ((row >> 2) & 3)) << 4); }

template <int MODE>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;

  // ---- which tile ----------------------------------------------------------------------------
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int lin = xcd * a.chunk + slot;
  if (slot >= a.chunk || lin >= a.tilesM * a.tilesN) return;
  const int tile_m = lin % a.tilesM, tile_n = lin / a.tilesM;

  // ---- global source rows of this lane: 8 rows of X and 8 rows of W, one 16-byte chunk each -------
  // Row r0 + 32 i of the slab.  All lanes of the block share the 32-row group i, and a group never
  // straddles two weight matrices (segment sizes are multiples of 32), so the matrix base pointer is
  // uniform per i (scalar registers) and only a 32-bit byte offset is kept per lane.
  const int kc = tid & 7;         // chunk within the 64-wide slab
  const int r0 = tid >> 3;        // rows r0 + 32*i
  // Loads go through buffer resources (scalar base + 32-bit lane offset + scalar slab offset), so the
  // K loop spends no vector instructions or registers on 64-bit addresses.
  const __amdgpu_buffer_rsrc_t xres = make_rsrc(a.X);
  const __amdgpu_buffer_rsrc_t wres0 = make_rsrc(a.W0), wres1 = make_rsrc(a.W1), wres2 = make_rsrc(a.W2);
  __amdgpu_buffer_rsrc_t wres[8];
  unsigned xoff[8], woff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = r0 + 32 * i;
    int m = tile_m * BM + r;
    m = m < a.M ? m : a.M - 1;
    xoff[i] = ((unsigned)m * (unsigned)a.K + kc * 8) * 2u;
    if (MODE == SX_GEMM_SWIGLU) {
      int f = tile_n * (BN / 2) + (i >> 1) * 32 + (r & 31);  // group i: even = gate, odd = up
      f = f < a.N ? f : a.N - 1;
      wres[i] = (i & 1) ? wres1 : wres0;
      woff[i] = ((unsigned)f * (unsigned)a.K + kc * 8) * 2u;
    } else {
      const int g0 = min(tile_n * BN + 32 * i, a.N - 1);     // first row of the group decides the matrix
      int n = tile_n * BN + r;
      n = n < a.N ? n : a.N - 1;
      int first = 0;
      wres[i] = wres0;
      if (g0 >= a.n0 + a.n1) {
        wres[i] = wres2;
        first = a.n0 + a.n1;
      } else if (g0 >= a.n0) {
        wres[i] = wres1;
        first = a.n0;
      }
      woff[i] = ((unsigned)(n - first) * (unsigned)a.K + kc * 8) * 2u;
    }
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Two register sets stage the global -> LDS traffic two K slabs ahead: the slab fetched during
  // iteration kt is written to LDS at the end of iteration kt+1 and consumed in iteration kt+2, so
  // a fetch has two slabs' worth of MFMA time (~1.7 us) to come back from HBM.
  u32x4 rx0[8], rw0[8], rx1[8], rw1[8];
  // byte offsets of this lane's fragment rows inside a stage (chunk 0; the chunk index is XORed in).
  // Every fragment row of a lane has the same (row >> 2) & 3 = (lane >> 2) & 3.
  int aoff[4], boff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    aoff[i] = (wm * 128 + i * 32 + l32) * (SK * 2);
    boff[i] = kOperandBytes + (wn * 128 + i * 32 + l32) * (SK * 2);
  }
  const int sw = (lane >> 2) & 3;
  // where this lane's fetched chunk goes: the 64-wide fetch covers two slabs; chunk kc < 4 belongs to the
  // first, kc >= 4 to the second (one stage further).  Odd stages are skewed by 128 bytes
  // (kStageStride) so that the two halves of a 16-lane write land on different banks.
  const int st_sub = (kc >> 2) * kStageStride;
  bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];

#define SX_FETCH(RX, RW, PAIR_, I0)                                                                \
  _Pragma("unroll") for (int i = I0; i < I0 + 4; ++i) {                                           \
    RX[i] = __builtin_amdgcn_raw_buffer_load_b128(xres, xoff[i], (PAIR_) * (BK * 2), 0);           \
    RW[i] = __builtin_amdgcn_raw_buffer_load_b128(wres[i], woff[i], (PAIR_) * (BK * 2), 0);        \
  }
// write a fetched pair of slabs into stages STG_ and STG_ + 1
#define SX_STASH(RX, RW, STG_, I0)                                                                 \
  _Pragma("unroll") for (int i = I0; i < I0 + 4; ++i) {                                           \
    const int off = (STG_) * kStageStride + st_sub + lds_off(r0 + 32 * i, kc & 3);                \
    *reinterpret_cast<u32x4*>(lds + off) = RX[i];                                                 \
    *reinterpret_cast<u32x4*>(lds + kOperandBytes + off) = RW[i];                                 \
  }
#define SX_READ(STG_, A, B, ks)                                                                    \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
    const int c = (STG_) * kStageStride + (((2 * (ks) + lh) ^ sw) << 4);                          \
    A[i] = *reinterpret_cast<const bf16x8*>(lds + aoff[i] + c);                                   \
    B[i] = *reinterpret_cast<const bf16x8*>(lds + boff[i] + c);                                   \
  }
#define SX_MMA(A, B)                                                                               \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)      \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[i], B[j], acc[i][j], 0, 0, 0);
// Issue order.  sched_barrier(0) fences keep three phases of a slab apart: (1) the 8 fragment reads of
// k-step 1, issued a full k-step (16 MFMAs, ~500 cycles) before they are needed; (2) the MFMAs of
// k-step 0 with half of the slab's side instructions (LDS writes or global reads) dealt out between
// them; (3) the MFMAs of k-step 1 with the other half and with the fragment reads of the NEXT
// slab's k-step 0, which therefore cross the barrier already in registers.
// Masks: 0x008 MFMA, 0x100 LDS read, 0x200 LDS write, 0x020 global read.
#define SX_FENCE __builtin_amdgcn_sched_barrier(0);
#define SX_DEAL(SIDE_MASK, WITH_READS)                                                             \
  _Pragma("unroll") for (int r_ = 0; r_ < 8; ++r_) {                                              \
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                             \
    __builtin_amdgcn_sched_group_barrier(SIDE_MASK, 1, 0);                                         \
    if (WITH_READS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                             \
  }
// A pair of slabs p = stages (S0, S0+1).  Register set (SRX, SRW) holds pair p+1: it is written to
// stages (S2, S2+1) during the first slab, and refilled with pair p+3 during the second.  On entry
// fa0/fb0 hold k-step 0 of the first slab.  The stages written here were last read a whole pair
// ago, and are first read (k-step 0 of the next pair) after the barrier that ends the first slab.
#define SX_PAIR(S0, S2, SRX, SRW, NEXT_PAIR)                                                       \
  SX_READ(S0, fa1, fb1, 1)                                                                         \
  SX_FENCE                                                                                         \
  SX_STASH(SRX, SRW, S2, 0)                                                                        \
  SX_MMA(fa0, fb0)                                                                                 \
  SX_DEAL(0x200, false)                                                                            \
  SX_FENCE                                                                                         \
  SX_STASH(SRX, SRW, S2, 4)                                                                        \
  SX_READ(S0 + 1, fa0, fb0, 0)                                                                     \
  SX_MMA(fa1, fb1)                                                                                 \
  SX_DEAL(0x200, true)                                                                             \
  SX_FENCE                                                                                         \
  __syncthreads();                                                                                 \
  SX_READ(S0 + 1, fa1, fb1, 1)                                                                     \
  SX_FENCE                                                                                         \
  SX_FETCH(SRX, SRW, NEXT_PAIR, 0)                                                                 \
  SX_MMA(fa0, fb0)                                                                                 \
  SX_DEAL(0x020, false)                                                                            \
  SX_FENCE                                                                                         \
  SX_FETCH(SRX, SRW, NEXT_PAIR, 4)                                                                 \
  SX_READ(S2, fa0, fb0, 0)                                                                         \
  SX_MMA(fa1, fb1)                                                                                 \
  SX_DEAL(0x020, true)                                                                             \
  SX_FENCE                                                                                         \
  __syncthreads();

  // The loop body is branch-free: past the end of K it re-fetches the last pair and writes it to
  // stages nobody reads again, which costs nothing and keeps each slab one schedulable block.
  const int NP = a.K / BK;  // pairs of slabs
  const int last = NP - 1;
  SX_FETCH(rx1, rw1, 0, 0)
  SX_FETCH(rx1, rw1, 0, 4)
  SX_STASH(rx1, rw1, 0, 0)
  SX_STASH(rx1, rw1, 0, 4)
  SX_FETCH(rx0, rw0, min(1, last), 0)
  SX_FETCH(rx0, rw0, min(1, last), 4)
  SX_FETCH(rx1, rw1, min(2, last), 0)
  SX_FETCH(rx1, rw1, min(2, last), 4)
  __syncthreads();
  SX_READ(0, fa0, fb0, 0)
  int p = 0;
  for (; p + 1 < NP; p += 2) {
    SX_PAIR(0, 2, rx0, rw0, min(p + 3, last))  // even pair: stages 0,1; set 0 holds pair p+1 -> stages 2,3
    SX_PAIR(2, 0, rx1, rw1, min(p + 4, last))  // odd pair: stages 2,3; set 1 holds pair p+2 -> stages 0,1
  }
  if (p < NP) {  // odd number of pairs: the last one sits in stages 0,1 and fa0/fb0 hold its first k-step
    SX_READ(0, fa1, fb1, 1)
    SX_MMA(fa0, fb0)
    SX_READ(1, fa0, fb0, 0)
    SX_MMA(fa1, fb1)
    SX_READ(1, fa1, fb1, 1)
    SX_MMA(fa0, fb0)
    SX_MMA(fa1, fb1)
  }
#undef SX_FETCH
#undef SX_STASH
#undef SX_READ
#undef SX_MMA
#undef SX_PAIR
#undef SX_DEAL
#undef SX_FENCE

  // ---- epilogue.  acc[i][j][e]: row = 32i + 8(e/4) + 4*lh + e%4, col = 32j + l32 within the quadrant --
  const int mbase = tile_m * BM + wm * 128;
  if (MODE == SX_GEMM_SWIGLU) {
    unsigned short* Y = static_cast<unsigned short*>(a.Y);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int f = tile_n * (BN / 2) + wn * 64 + jj * 32 + l32;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = mbase + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
          if (m < a.M && f < a.N) {
            const float g = acc[i][2 * jj][e], u = acc[i][2 * jj + 1][e];
            Y[(size_t)m * a.N + f] = (unsigned short)f32_to_bf16_bits(g / (1.0f + expf(-g)) * u);
          }
        }
      }
  } else {
    float* Y = static_cast<float*>(a.Y);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int n = tile_n * BN + wn * 128 + j * 32 + l32;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = mbase + i * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
          if (m < a.M && n < a.N) {
            float* y = Y + (size_t)m * a.N + n;
            if (MODE == SX_GEMM_RESIDUAL) *y += acc[i][j][e];
            else *y = acc[i][j][e];
          }
        }
      }
  }
}

template <int MODE>
int launch(const GemmArgs& a, hipStream_t st) {
  static bool configured = false;  // raising the dynamic-LDS cap is a per-kernel, per-process setting
  if (!configured) {
    SX_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<MODE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
    configured = true;
  }
  gemm_bf16_kernel<MODE><<<8 * a.chunk, kThreads, kLdsBytes, st>>>(a);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

}  // namespace

int sx_launch_gemm_bf16(const void* X, const void* W0, const void* W1, const void* W2, int n0, int n1, int n2,
                        void* Y, int M, int K, int mode, hipStream_t st) {
  if (M < 1 || K < BK || K % BK != 0 || n0 < 1) return SX_ERR_SHAPE;
  GemmArgs a;
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
  a.tilesM = (M + BM - 1) / BM;
  if (mode == SX_GEMM_SWIGLU) {
    if (n1 != n0 || n2 != 0 || !W1) return SX_ERR_SHAPE;
    a.N = n0;
    a.tilesN = (n0 + BN / 2 - 1) / (BN / 2);
  } else {
    a.N = n0 + n1 + n2;
    a.tilesN = (a.N + BN - 1) / BN;
  }
  a.chunk = (a.tilesM * a.tilesN + 7) / 8;
  switch (mode) {
    case SX_GEMM_STORE: return launch<SX_GEMM_STORE>(a, st);
    case SX_GEMM_RESIDUAL: return launch<SX_GEMM_RESIDUAL>(a, st);
    case SX_GEMM_SWIGLU: return launch<SX_GEMM_SWIGLU>(a, st);
  }
  return SX_ERR_SHAPE;
}

extern "C" int sx_gemm_bf16(const void* X, const void* W, const void* W2, void* Y, int32_t M, int32_t N, int32_t K,
                            int32_t mode, void* stream) {
  if (!X || !W || !Y || (mode == SX_GEMM_SWIGLU && !W2)) return SX_ERR_NULL;
  if (mode < 0 || mode > 2 || N < 1) return SX_ERR_SHAPE;
  if (mode == SX_GEMM_SWIGLU) return sx_launch_gemm_bf16(X, W, W2, nullptr, N, N, 0, Y, M, K, mode, (hipStream_t)stream);
  return sx_launch_gemm_bf16(X, W, nullptr, nullptr, N, 0, 0, Y, M, K, mode, (hipStream_t)stream);
}
