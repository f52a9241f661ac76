// Y = X W^T on the gfx950 matrix cores: the linear layers of the decoder forward (Alg. 1, FORWARD) at
// M = number of tree tokens.  bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16).
//
// Tiling.  A workgroup of 4 waves (2 x 2) owns a 256 x 256 output tile; each wave a 128 x 128
// quadrant = 4 x 4 MFMA blocks, 256 fp32 accumulators per lane.  K is walked in slabs of 64:
// the 256x64 X slab and the 256x64 W slab (32 KB each) are double-buffered in LDS (128 KB of the
// 160 KB), fetched global -> registers one slab ahead and written to LDS after the current slab's
// MFMAs.  Both operands are K-contiguous in memory, which is exactly the per-lane layout the MFMA
// wants (8 consecutive k per lane), so LDS rows are plain 128-byte row segments; the 16-byte
// chunk index is XOR-swizzled with (row & 7) so that the 8 lanes served per LDS cycle hit 8
// different bank groups on both the write and the read side.
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

__device__ __forceinline__ int lds_off(int row, int kchunk) { return row * (BK * 2) + ((kchunk ^ (row & 7)) << 4); }

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
  const int kc = tid & 7;         // chunk within the 64-wide slab
  const int r0 = tid >> 3;        // rows r0 + 32*i
  const unsigned short* xrow[8];
  const unsigned short* wrow[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = r0 + 32 * i;
    int m = tile_m * BM + r;
    m = m < a.M ? m : a.M - 1;
    xrow[i] = a.X + (size_t)m * a.K + kc * 8;
    const unsigned short* w;
    if (MODE == SX_GEMM_SWIGLU) {
      const int g = r >> 5;                                  // 32-row group: even = gate, odd = up
      int f = tile_n * (BN / 2) + (g >> 1) * 32 + (r & 31);
      f = f < a.N ? f : a.N - 1;
      w = ((g & 1) ? a.W1 : a.W0) + (size_t)f * a.K;
    } else {
      int n = tile_n * BN + r;
      n = n < a.N ? n : a.N - 1;
      if (n < a.n0) w = a.W0 + (size_t)n * a.K;
      else if (n < a.n0 + a.n1) w = a.W1 + (size_t)(n - a.n0) * a.K;
      else w = a.W2 + (size_t)(n - a.n0 - a.n1) * a.K;
    }
    wrow[i] = w + kc * 8;
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 rx[8], rw[8];
  auto fetch = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      rx[i] = *reinterpret_cast<const u32x4*>(xrow[i] + (size_t)kt * BK);
      rw[i] = *reinterpret_cast<const u32x4*>(wrow[i] + (size_t)kt * BK);
    }
  };
  auto stash = [&](int buf) {
    char* xs = lds + buf * 2 * kSlabBytes;
    char* ws = xs + kSlabBytes;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int off = lds_off(r0 + 32 * i, kc);
      *reinterpret_cast<u32x4*>(xs + off) = rx[i];
      *reinterpret_cast<u32x4*>(ws + off) = rw[i];
    }
  };

  const int KT = a.K / BK;
  fetch(0);
  stash(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    if (kt + 1 < KT) fetch(kt + 1);
    const char* xs = lds + (kt & 1) * 2 * kSlabBytes;
    const char* ws = xs + kSlabBytes;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[4], bf[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(xs + lds_off(wm * 128 + i * 32 + l32, 2 * ks + lh));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        bf[j] = *reinterpret_cast<const bf16x8*>(ws + lds_off(wn * 128 + j * 32 + l32, 2 * ks + lh));
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) stash((kt + 1) & 1);
    __syncthreads();
  }

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
