// Y = X W^T on the gfx950 matrix cores: the linear layers of the decoder forward (Alg. 1, FORWARD) at
// M = number of tree tokens.  bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16).
//
// Tiling.  A workgroup of 4 waves (2 x 2) owns a 256 x 256 output tile; each wave a 128 x 128
// quadrant = 4 x 4 MFMA blocks, 256 fp32 accumulators per lane.  K is walked in slabs of 64:
// the 256x64 X slab and the 256x64 W slab (32 KB each) are double-buffered in LDS (128 KB of the
// 160 KB), fetched global -> registers two slabs ahead (two register sets) and written to LDS after
// the current slab's MFMAs.  Both operands are K-contiguous in memory, which is exactly the per-lane layout the MFMA
// wants (8 consecutive k per lane), so LDS rows are plain 128-byte row segments; the 16-byte
// chunk index is XOR-swizzled with (row >> 1) & 7: the LDS serves 16 lanes x 16 bytes per cycle
// (64 banks), and with this swizzle 16 consecutive rows reading the same k chunk -- and 16
// consecutive lanes writing two rows -- touch 16 different bank groups (measured: ~220 B/clk per
// CU against ~140 B/clk for a swizzle by row & 7).
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

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kSlabBytes = BM * BK * 2;  // 32 KB per operand per stage
constexpr int kLdsBytes = 4 * kSlabBytes;

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

__device__ __forceinline__ int lds_off(int row, int kchunk) { return row * (BK * 2) + ((kchunk ^ ((row >> 1) & 7)) << 4); }

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
  const char* xbase = reinterpret_cast<const char*>(a.X);
  const char* wbase[8];
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
      wbase[i] = reinterpret_cast<const char*>((i & 1) ? a.W1 : a.W0);
      woff[i] = ((unsigned)f * (unsigned)a.K + kc * 8) * 2u;
    } else {
      const int g0 = min(tile_n * BN + 32 * i, a.N - 1);     // first row of the group decides the matrix
      int n = tile_n * BN + r;
      n = n < a.N ? n : a.N - 1;
      const unsigned short* base = a.W0;
      int first = 0;
      if (g0 >= a.n0 + a.n1) {
        base = a.W2;
        first = a.n0 + a.n1;
      } else if (g0 >= a.n0) {
        base = a.W1;
        first = a.n0;
      }
      wbase[i] = reinterpret_cast<const char*>(base);
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
  // Every fragment row of a lane has the same (row >> 1) & 7 = (lane >> 1) & 7.
  int aoff[4], boff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    aoff[i] = (wm * 128 + i * 32 + l32) * (BK * 2);
    boff[i] = kSlabBytes + (wn * 128 + i * 32 + l32) * (BK * 2);
  }
  const int sw = (lane >> 1) & 7;
  bf16x8 fa0[4], fb0[4], fa1[4], fb1[4];

#define SX_FETCH(RX, RW, KT_, I0)                                                                  \
  _Pragma("unroll") for (int i = I0; i < I0 + 4; ++i) {                                           \
    RX[i] = *reinterpret_cast<const u32x4*>(xbase + (size_t)(KT_) * (BK * 2) + xoff[i]);          \
    RW[i] = *reinterpret_cast<const u32x4*>(wbase[i] + (size_t)(KT_) * (BK * 2) + woff[i]);       \
  }
#define SX_STASH(RX, RW, BUF_, I0)                                                                 \
  _Pragma("unroll") for (int i = I0; i < I0 + 4; ++i) {                                           \
    const int off = lds_off(r0 + 32 * i, kc);                                                     \
    *reinterpret_cast<u32x4*>(lds + (BUF_) * 2 * kSlabBytes + off) = RX[i];                       \
    *reinterpret_cast<u32x4*>(lds + (BUF_) * 2 * kSlabBytes + kSlabBytes + off) = RW[i];          \
  }
#define SX_READ(STAGE, A, B, ks)                                                                   \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                 \
    const int c = ((2 * (ks) + lh) ^ sw) << 4;                                                    \
    A[i] = *reinterpret_cast<const bf16x8*>((STAGE) + aoff[i] + c);                               \
    B[i] = *reinterpret_cast<const bf16x8*>((STAGE) + boff[i] + c);                               \
  }
#define SX_MMA(A, B)                                                                               \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)      \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[i], B[j], acc[i][j], 0, 0, 0);
// One K slab: 4 k-steps of 16 MFMAs.  Fragments of step ks+1 are read while step ks multiplies; the
// global fetch of the slab two ahead and the LDS write of the slab one ahead are dealt out between
// the MFMA groups so that their issue slots hide under matrix-core time.
// Issue order requested from the scheduler for one slab (masks: 0x008 MFMA, 0x100 LDS read, 0x200 LDS
// write, 0x020 global read): both leading fragment sets, then 16 rounds of 4 MFMAs each carrying
// one LDS write and one global read; rounds 4-11 also carry the two fragment reads that refill the
// set the preceding k-step has just finished with.
#define SX_SCHED                                                                                   \
  __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);                                              \
  _Pragma("unroll") for (int r_ = 0; r_ < 16; ++r_) {                                             \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);                                             \
    if (r_ >= 4 && r_ < 12) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                     \
    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                             \
    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                             \
  }
#define SX_SLAB(STAGE, FRX, FRW, FKT, SRX, SRW, SBUF)                                              \
  SX_READ(STAGE, fa0, fb0, 0)                                                                      \
  SX_READ(STAGE, fa1, fb1, 1)                                                                      \
  SX_FETCH(FRX, FRW, FKT, 0)                                                                       \
  SX_MMA(fa0, fb0)                                                                                 \
  SX_READ(STAGE, fa0, fb0, 2)                                                                      \
  SX_STASH(SRX, SRW, SBUF, 0)                                                                      \
  SX_MMA(fa1, fb1)                                                                                 \
  SX_READ(STAGE, fa1, fb1, 3)                                                                      \
  SX_FETCH(FRX, FRW, FKT, 4)                                                                       \
  SX_MMA(fa0, fb0)                                                                                 \
  SX_STASH(SRX, SRW, SBUF, 4)                                                                      \
  SX_MMA(fa1, fb1)                                                                                 \
  SX_SCHED

  // The loop body is branch-free: past the end of K it re-fetches the last slab and writes it to a
  // stage nobody reads again, which costs nothing and keeps each slab one schedulable block.
  const int KT = a.K / BK;
  const int last = KT - 1;
  SX_FETCH(rx0, rw0, 0, 0)
  SX_FETCH(rx0, rw0, 0, 4)
  SX_STASH(rx0, rw0, 0, 0)
  SX_STASH(rx0, rw0, 0, 4)
  SX_FETCH(rx1, rw1, min(1, last), 0)
  SX_FETCH(rx1, rw1, min(1, last), 4)
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    // even slab: in LDS stage 0; set 0 is free (fetch slab kt+2 into it), set 1 holds slab kt+1 (-> stage 1)
    SX_SLAB(lds, rx0, rw0, min(kt + 2, last), rx1, rw1, 1)
    __syncthreads();
    // odd slab: in LDS stage 1; set 1 is free (fetch slab kt+3), set 0 holds slab kt+2 (-> stage 0)
    SX_SLAB(lds + 2 * kSlabBytes, rx1, rw1, min(kt + 3, last), rx0, rw0, 0)
    __syncthreads();
  }
  if (kt < KT) {  // odd slab count: the last one sits in stage 0
    SX_READ(lds, fa0, fb0, 0)
    SX_MMA(fa0, fb0)
    SX_READ(lds, fa0, fb0, 1)
    SX_MMA(fa0, fb0)
    SX_READ(lds, fa0, fb0, 2)
    SX_MMA(fa0, fb0)
    SX_READ(lds, fa0, fb0, 3)
    SX_MMA(fa0, fb0)
  }
#undef SX_FETCH
#undef SX_STASH
#undef SX_READ
#undef SX_MMA
#undef SX_SLAB
#undef SX_SCHED

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
