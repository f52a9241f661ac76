// Y = X W^T for few rows (M <= 128) with 4-bit group-quantised weights (the paper's fastest setting runs the
// models quantised to 4 bits, Sect. 5): at this M the product is bound by streaming the weights, and the
// weights are a quarter of the bytes.  Storage: eight 4-bit codes per 32-bit word (code j of word i of a row is
// k = 8 i + j, bits 4j..4j+3), one bf16 scale and one zero point (0..15, a byte) per row and group of `group`
// consecutive k; w = bf16(scale * (code - zero)).
// Same tile and pipeline as the bf16 narrow kernel (128 x 64, three K = 64 stages, X copied straight into LDS),
// except that W goes global -> registers (8 bytes = 16 codes per lane and stage, one stage ahead) ->
// dequantised to bf16 -> LDS, in the swizzled layout the fragment reads expect.
#include "kernels.h"

namespace {

constexpr int BM = 128, BN = 64, BK = 64;
constexpr int kThreads = 256;
constexpr int kXBytes = BM * BK * 2;   // 16 KB
constexpr int kWBytes = BN * BK * 2;   // 8 KB
constexpr int kStageBytes = kXBytes + kWBytes;
constexpr int kPartFloats = BM * BN;   // partial sums of one K part of one tile

struct W4Args {
  const unsigned short* X;
  const uint32_t* qweight;        // [N][K/8]
  const unsigned short* scales;   // bf16 [N][K/group]
  const unsigned char* zeros;     // [N][K/group]
  int group, group_log2;
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

typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned cvt_pk_bf16(float lo, float hi) {  // one v_cvt_pk_bf16_f32
  f32x2 t = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2));
}

constexpr int kWaitVm0 = 0x0070, kWaitVm7 = 0x0077;
#define SX_WAIT_BARRIER(IMM)              \
  asm volatile("" ::: "memory");          \
  __builtin_amdgcn_s_waitcnt(IMM);        \
  __builtin_amdgcn_s_barrier();           \
  asm volatile("" ::: "memory");

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void gemm_skinny_w4_kernel(W4Args a) {
  // one array per stage: X rows then W rows, 128 bytes each, 16-byte chunk c of row r at position c ^ ((r >> 1) & 7)
  // X and W of a stage are separate arrays: W is written by ordinary LDS stores, and in one array with X the
  // compiler would make those stores wait for the copies in flight to the same stage
  __shared__ __attribute__((aligned(1024))) unsigned char sx0[kXBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sx1[kXBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sx2[kXBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sw0[kWBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sw1[kWBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sw2[kWBytes];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lq = lane >> 4;
  const int tile_n = blockIdx.x / a.split, kpart = blockIdx.x % a.split;

  // ---- X copies: instruction t of wave w fills X rows 32 w + 8 t .. + 7 --------------------------------------
  const __amdgpu_buffer_rsrc_t xres = make_rsrc(a.X);
  int xoff[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int cchunk = (lane & 7) ^ ((4 * (t & 1) + (lane >> 4)) & 7);
    int m = 32 * wave + 8 * t + (lane >> 3);
    m = m < a.M ? m : a.M - 1;
    xoff[t] = (int)(((unsigned)m * (unsigned)a.K + cchunk * 8) * 2u);
  }
#define SX_COPY(STG_, SLAB_)                                                                                     \
  {                                                                                                              \
    const int so = (SLAB_) * (BK * 2);                                                                           \
    _Pragma("unroll") for (int t = 0; t < 4; ++t) __builtin_amdgcn_raw_ptr_buffer_load_lds(                      \
        xres, (lds_void_ptr)(STG_ + wave * 4096 + t * 1024), 16, xoff[t], so, 0, 0);                             \
  }
  // ---- W: lane handles row tid / 4 of the tile's 64, codes 16 (tid % 4) .. + 15 of a stage's 64 ------------------
  const int wr = tid >> 2, wq = tid & 3;
  const int wn_row = min(tile_n * BN + wr, a.N - 1);
  // 32-bit offsets from the start of each array (buffer loads: scalar base + lane offset + scalar slab offset)
  const __amdgpu_buffer_rsrc_t qres = make_rsrc(a.qweight), sres = make_rsrc(a.scales), zres = make_rsrc(a.zeros);
  const int qoff = (int)(((unsigned)wn_row * (unsigned)(a.K / 8) + 2u * wq) * 4u);   // + 32 bytes per slab
  const int goff = (int)((unsigned)wn_row * (unsigned)(a.K >> a.group_log2));        // + group index
  // where the 16 dequantised values (two 16-byte chunks 2 wq, 2 wq + 1 of row wr) go in a stage
  const int wdst0 = wr * (BK * 2) + (((2 * wq) ^ ((wr >> 1) & 7)) << 4);
  const int wdst1 = wr * (BK * 2) + (((2 * wq + 1) ^ ((wr >> 1) & 7)) << 4);
  struct Packed {
    u32x2 q;
    float s;
    int z;
  };
  auto load_w = [&](int slab) {
    Packed p;
    p.q = __builtin_amdgcn_raw_buffer_load_b64(qres, qoff, slab * 32, 0);
    const int g = (slab * BK) >> a.group_log2;
    p.s = bf16_bits_to_f32((unsigned short)__builtin_amdgcn_raw_buffer_load_b16(sres, goff * 2, g * 2, 0));
    p.z = (unsigned char)__builtin_amdgcn_raw_buffer_load_b8(zres, goff, g, 0);
    return p;
  };
#define SX_DEQUANT(STG_, P_)                                                                                     \
  {                                                                                                              \
    u32x4 c0, c1;                                                                                                \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                              \
      const float a0 = (float)((int)((P_.q[0] >> (8 * j)) & 15u) - P_.z) * P_.s;                                 \
      const float a1 = (float)((int)((P_.q[0] >> (8 * j + 4)) & 15u) - P_.z) * P_.s;                             \
      const float b0 = (float)((int)((P_.q[1] >> (8 * j)) & 15u) - P_.z) * P_.s;                                 \
      const float b1 = (float)((int)((P_.q[1] >> (8 * j + 4)) & 15u) - P_.z) * P_.s;                             \
      c0[j] = cvt_pk_bf16(a0, a1);                                                                               \
      c1[j] = cvt_pk_bf16(b0, b1);                                                                               \
    }                                                                                                            \
    *reinterpret_cast<u32x4*>(STG_ + wdst0) = c0;                                                                \
    *reinterpret_cast<u32x4*>(STG_ + wdst1) = c1;                                                                \
  }

  // acc[i][j]: W rows (output columns) 32 wn + 16 i .. + 15, X rows (output rows) 64 wm + 16 j .. + 15
  f32x4 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
  const int fsw = (l16 >> 1) & 7;
  const int xrow = (wm * 64 + l16) * (BK * 2);
  const int wrow = (wn * 32 + l16) * (BK * 2);
  const int kc[2] = {(lq ^ fsw) << 4, ((4 + lq) ^ fsw) << 4};

// "+v": the accumulators stay where they are (see the wide kernel); statements are volatile, order as written
#define SX_MFMA(ACC, A, B) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(ACC) : "v"(A), "v"(B));
// Iteration for the slab in stage (XS_, WS_): barrier; start the X copies of the slab after next (stage XF_) and
// the W loads of the slab three ahead (registers; older in the queue than anything the next two barriers wait
// for, so waiting for them costs nothing); dequantise the W registers of the next slab into its stage WN_; multiply.
#define SX_SLAB(XS_, WS_, WN_, XF_, SLAB_F, SLAB_W)                                                              \
  SX_WAIT_BARRIER(kWaitVm7)                                                                                      \
  SX_COPY(XF_, SLAB_F)                                                                                           \
  {                                                                                                              \
    const Packed nw = load_w(SLAB_W);                                                                            \
    SX_DEQUANT(WN_, pw0)                                                                                         \
    pw0 = pw1;                                                                                                   \
    pw1 = nw;                                                                                                    \
  }                                                                                                              \
  _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                             \
    bf16x8 fx[4], fw[2];                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 2; ++i)                                                                \
        fw[i] = *reinterpret_cast<const bf16x8*>(WS_ + wrow + i * (16 * BK * 2) + kc[ks]);                       \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                                \
        fx[j] = *reinterpret_cast<const bf16x8*>(XS_ + xrow + j * (16 * BK * 2) + kc[ks]);                       \
    _Pragma("unroll") for (int i = 0; i < 2; ++i) _Pragma("unroll") for (int j = 0; j < 4; ++j)                  \
        SX_MFMA(acc[i][j], fw[i], fx[j])                                                                         \
  }

  // slabs [first, first + NB) of K; slab s sits in stage (s - first) % 3
  const int nb_all = a.K / BK;
  const int first = kpart * nb_all / a.split;
  const int NB = (kpart + 1) * nb_all / a.split - first, last = first + NB - 1;
  Packed pw0 = load_w(first);
  SX_COPY(sx0, first)
  SX_COPY(sx1, min(first + 1, last))
  SX_DEQUANT(sw0, pw0)
  pw0 = load_w(min(first + 1, last));
  Packed pw1 = load_w(min(first + 2, last));
  int s = 0;
  for (; s + 3 <= NB; s += 3) {
    SX_SLAB(sx0, sw0, sw1, sx2, min(first + s + 2, last), min(first + s + 3, last))
    SX_SLAB(sx1, sw1, sw2, sx0, min(first + s + 3, last), min(first + s + 4, last))
    SX_SLAB(sx2, sw2, sw0, sx1, min(first + s + 4, last), min(first + s + 5, last))
  }
  if (s < NB) {
    SX_SLAB(sx0, sw0, sw1, sx2, last, last)
    if (s + 1 < NB) { SX_SLAB(sx1, sw1, sw2, sx0, last, last) }
  }
  __builtin_amdgcn_s_waitcnt(kWaitVm0);  // copies past the end of K must land before the LDS is released
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");  // the matrix pipe's last results (hand-written MFMAs)
#undef SX_SLAB
#undef SX_MFMA
#undef SX_COPY
#undef SX_DEQUANT

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
    const unsigned all = (unsigned)(tile_n * a.split * kPartFloats + wave * (8 * 256) + lane * 4) * 4u;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        f32x4 sum = __builtin_bit_cast(
            f32x4, __builtin_amdgcn_raw_buffer_load_b128(pres, all + (i * 4 + j) * 1024, 0, kScopeDevice));
        for (int p = 1; p < a.split; ++p)
          sum += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                               pres, all + (unsigned)p * (kPartFloats * 4u) + (i * 4 + j) * 1024, 0,
                                               kScopeDevice));
        acc[i][j] = sum;
      }
  }

  // ---- epilogue.  acc[i][j][e]: output row 64 wm + 16 j + l16, W row 32 wn + 16 i + 4 lq + e ------------------
  const bool vec = (a.N & 3) == 0;
  {
    float* Y = static_cast<float*>(a.Y);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = wm * 64 + 16 * j + l16;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int n = tile_n * BN + wn * 32 + 16 * i + 4 * lq;
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

int sx_launch_gemm_skinny_w4(const void* X, const void* qweight, const void* scales, const void* zeros, int group,
                             void* Y, int M, int N, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st) {
  if (M < 1 || M > BM || K < BK || K % BK != 0 || N < 1 || group < BK || (group & (group - 1)) != 0 || K % group != 0)
    return SX_ERR_SHAPE;
  if (!sx_operand_fits_u32(N, K / 2) || !sx_operand_fits_u32(M, 2ll * K)) return SX_ERR_SHAPE;  // 32-bit byte offsets
  if (mode != SX_GEMM_STORE && mode != SX_GEMM_RESIDUAL) return SX_ERR_SHAPE;
  W4Args a;
  a.X = static_cast<const unsigned short*>(X);
  a.qweight = static_cast<const uint32_t*>(qweight);
  a.scales = static_cast<const unsigned short*>(scales);
  a.zeros = static_cast<const unsigned char*>(zeros);
  a.group = group;
  a.group_log2 = __builtin_ctz((unsigned)group);
  a.Y = Y;
  a.M = M;
  a.N = N;
  a.K = K;
  a.tilesN = (N + BN - 1) / BN;
  a.split = 1;
  a.part = nullptr;
  a.part_cnt = nullptr;
  const int slots = sx_compute_units(), nb = K / BK;
  if (split_ws && a.tilesN <= 256 && 2 * a.tilesN <= slots) {
    int split = slots / a.tilesN;
    if (split > 8) split = 8;
    while (split > 1 && nb / split < 4) --split;
    if (split > 1 && split_ws_bytes >= 1024 + (size_t)a.tilesN * split * kPartFloats * sizeof(float)) {
      a.split = split;
      a.part_cnt = static_cast<int*>(split_ws);
      a.part = reinterpret_cast<float*>(static_cast<char*>(split_ws) + 1024);
    }
  }
  const int grid = a.tilesN * a.split;
  if (mode == SX_GEMM_STORE) gemm_skinny_w4_kernel<SX_GEMM_STORE><<<grid, kThreads, 0, st>>>(a);
  else gemm_skinny_w4_kernel<SX_GEMM_RESIDUAL><<<grid, kThreads, 0, st>>>(a);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

extern "C" size_t sx_gemm_w4a16_workspace(void) { return sx_gemm_split_workspace(); }

extern "C" int sx_gemm_w4a16_bf16(const void* X, const void* qweight, const void* scales, const void* zeros, void* Y,
                                  int32_t M, int32_t N, int32_t K, int32_t group, int32_t mode, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  if (!X || !qweight || !scales || !zeros || !Y) return SX_ERR_NULL;
  hipStream_t st = (hipStream_t)stream;
  if (workspace) {
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) || workspace_bytes < 1024) return SX_ERR_WORKSPACE;
    SX_TRY(sx_launch_zero_i32(static_cast<int32_t*>(workspace), 256, st));  // the K-split counters
  }
  // K a multiple of 128: weights dequantised in registers; otherwise through LDS
  if (M >= 1 && M <= 128 && K >= 128 && K % 128 == 0 && N >= 1) {
    const sx_w4_matrix m = {qweight, scales, zeros};
    const int n = N;
    return sx_launch_gemm_w4_regs(X, &m, &n, 1, group, static_cast<float*>(Y), N, M, K, mode, workspace, workspace_bytes, st);
  }
  return sx_launch_gemm_skinny_w4(X, qweight, scales, zeros, group, Y, M, N, K, mode, workspace, workspace_bytes, st);
}
