// Y = X W^T for few rows (M <= 128) with 4-bit group-quantised weights, second form (Sect. 5: the paper's fastest
// setting runs its models quantised to 4 bits; for the draft model's small batches the product is bound by
// streaming the weights, and these are a quarter of the bytes).
//
// The weights never pass through LDS.  The A operand of v_mfma_f32_16x16x32_bf16 wants, per lane, eight
// consecutive k of one W row -- exactly one 32-bit word of eight 4-bit codes.  So a lane fetches the words of
// its own fragments straight from global memory (16 bytes = four fragments per load), dequantises them in
// registers (w = bf16(scale * (code - zero)): one byte-to-float conversion and one fma per weight, exact in
// fp32, rounded once) and feeds the matrix core.  Only X goes through LDS (copied by buffer loads that write
// LDS), where the 128 rows are shared by the four waves.
//
// Tiling: a workgroup owns all M <= 128 rows x 128 columns; wave w the columns 32 w .. + 31 (2 blocks of 16 W
// rows) x 8 blocks of 16 X rows: 16 MFMAs per k-step against 8 KB of X fragments.  K is walked in slabs of 128
// (four k-steps).  The contraction index may be permuted as long as both operands agree: in k-step s of a slab a
// lane of quarter lq takes the 16-byte chunk 4 lq + s of its row, so its four fragments of the slab are one
// contiguous 16-byte load (64 contiguous bytes per W row and wave).
// With at most a few dozen column tiles the K range is cut among workgroups (grid.y); partial sums meet in
// memory and the last workgroup to arrive adds them in part order (deterministic, nobody waits).
//
// Up to three weight matrices may be stacked along N (the QKV projections, or gate and up) as long as each
// holds a multiple of 64 rows: a wave's 64 columns then belong to one matrix.
#include "kernels.h"

namespace {

constexpr int BM = 128, BK = 128;   // columns per workgroup: 4 waves x WB blocks of 16 (template parameter)
constexpr int kThreads = 256;
constexpr int kXBytes = BM * BK * 2;   // 32 KB: one slab of X

struct W4Mat {
  const uint32_t* q;          // [n][K/8]
  const unsigned short* s;    // bf16 [n][K/group]
  const unsigned char* z;     // [n][K/group]
};

struct W4RegArgs {
  const unsigned short* X;
  W4Mat m[3];
  int n0, n1, n2;
  int group_log2;
  float* Y;
  int ldy;
  int M, N, K;
  int split;
  float* part;
  int* part_cnt;
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, -1, 0x00020000);
}
__device__ __forceinline__ unsigned cvt_pk_bf16(float lo, float hi) {  // one v_cvt_pk_bf16_f32
  f32x2 t = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(t, bf16x2));
}

// eight codes of one word -> eight bf16 in k order; sc = scale, nzs = -zero * scale (both exact in fp32, and so is
// code * sc + nzs = sc * (code - zero): 8 significant bits times at most 4)
__device__ __forceinline__ bf16x8 dequant8(uint32_t q, float sc, float nzs) {
  const uint32_t lo = q & 0x0F0F0F0Fu, hi = (q >> 4) & 0x0F0F0F0Fu;  // codes 0,2,4,6 and 1,3,5,7, one per byte
  u32x4 o;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const float e = fmaf((float)((lo >> (8 * b)) & 0xFFu), sc, nzs);
    const float f = fmaf((float)((hi >> (8 * b)) & 0xFFu), sc, nzs);
    o[b] = cvt_pk_bf16(e, f);
  }
  return __builtin_bit_cast(bf16x8, o);
}

constexpr int kWaitVm0 = 0x0070;
// all LDS reads of this wave done, all its vector-memory operations done, then meet the other waves
#define SX_WAIT_BARRIER()                  \
  asm volatile("" ::: "memory");           \
  __builtin_amdgcn_s_waitcnt(kWaitVm0);    \
  __builtin_amdgcn_s_barrier();            \
  asm volatile("" ::: "memory");

template <int MODE, int WB>
__global__ __launch_bounds__(kThreads, 2) void gemm_w4_regs_kernel(W4RegArgs a) {
  constexpr int BN = 64 * WB;             // columns of the workgroup
  constexpr int kPartFloats = BM * BN;    // partial sums of one K part of one tile
  // X slab: row r is 256 bytes at r * 256, its 16-byte chunk c at position c ^ (r & 15): the 16 rows a fragment
  // read touches for one chunk index fall on 16 different bank groups.  Two stages.
  __shared__ __attribute__((aligned(1024))) unsigned char sx0[kXBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char sx1[kXBytes];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, lq = lane >> 4;
  const int tile_n = blockIdx.x, kpart = blockIdx.y;

  // ---- X copies: instruction t (0..7) of wave w fills rows 32 w + 4 t .. + 3 (1 KB of LDS): lane l supplies row
  // + l / 16, position l % 16, i.e. chunk (l % 16) ^ (row & 15) of that row's 256 bytes of the slab
  const __amdgpu_buffer_rsrc_t xres = make_rsrc(a.X);
  int xoff[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int r = 32 * wave + 4 * t + (lane >> 4);
    const int c = (lane & 15) ^ (r & 15);
    const int m = r < a.M ? r : a.M - 1;
    xoff[t] = (int)(((unsigned)m * (unsigned)a.K + c * 8) * 2u);
  }
#define SX_COPY(STG_, SLAB_)                                                                                     \
  {                                                                                                              \
    const int so = (SLAB_) * (BK * 2);                                                                           \
    _Pragma("unroll") for (int t = 0; t < 8; ++t) __builtin_amdgcn_raw_ptr_buffer_load_lds(                      \
        xres, (lds_void_ptr)(STG_ + wave * 8192 + t * 1024), 16, xoff[t], so, 0, 0);                             \
  }

  // ---- W: this wave's columns belong to one of the stacked matrices -------------------------------------------
  const int c0 = tile_n * BN + 16 * WB * wave;  // first column of the wave (uniform)
  int first = 0, rows = a.n0, which = 0;
  if (c0 >= a.n0 + a.n1) {
    first = a.n0 + a.n1;
    rows = a.n2;
    which = 2;
  } else if (c0 >= a.n0) {
    first = a.n0;
    rows = a.n1;
    which = 1;
  }
  const bool wave_has_cols = c0 < a.N;
  const __amdgpu_buffer_rsrc_t qres = make_rsrc(a.m[which].q), sres = make_rsrc(a.m[which].s),
                               zres = make_rsrc(a.m[which].z);
  const int ngroups = a.K >> a.group_log2;
  int qoff[WB], goff[WB];
#pragma unroll
  for (int i = 0; i < WB; ++i) {
    int n = c0 - first + 16 * i + l16;          // row of the matrix; columns past the end re-read the last row
    n = n < rows ? n : rows - 1;
    n = n < 0 ? 0 : n;
    qoff[i] = (int)(((unsigned)n * (unsigned)(a.K / 8) + 4u * lq) * 4u);   // + 64 bytes per slab
    goff[i] = (int)((unsigned)n * (unsigned)ngroups);
  }
  // group of this lane's k range of a slab: k = 128 slab + 32 lq + 8 s + (0..7), the same for all four k-steps s
  // whenever the group holds at least 32 values (groups are powers of two >= 64)
  auto group_of = [&](int slab) { return (slab * BK + 32 * lq) >> a.group_log2; };

  struct WRaw {
    u32x4 q[WB];
    float sc[WB], nzs[WB];
  };
  auto load_w = [&](int slab) {
    WRaw w;
    const int g = group_of(slab);
#pragma unroll
    for (int i = 0; i < WB; ++i) {
      w.q[i] = __builtin_amdgcn_raw_buffer_load_b128(qres, qoff[i], slab * 64, 0);
      const float sc = bf16_bits_to_f32((unsigned short)__builtin_amdgcn_raw_buffer_load_b16(sres, (goff[i] + g) * 2, 0, 0));
      const float z = (float)(unsigned char)__builtin_amdgcn_raw_buffer_load_b8(zres, goff[i] + g, 0, 0);
      w.sc[i] = sc;
      w.nzs[i] = -z * sc;
    }
    return w;
  };

  // acc[i][j]: W rows (output columns) c0 + 16 i .. + 15, X rows (output rows) 16 j .. + 15
  f32x4 acc[WB][8];
#pragma unroll
  for (int i = 0; i < WB; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // X fragment of block j in k-step s: row 16 j + l16, chunk 4 lq + s, at position chunk ^ (row & 15) = chunk ^ l16
  const int xrow = l16 * (BK * 2);
#define SX_SLAB(XS_, W_)                                                                                         \
  _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                                                \
    bf16x8 fw[WB], fx[8];                                                                                        \
    _Pragma("unroll") for (int i = 0; i < WB; ++i) fw[i] = dequant8(W_.q[i][s], W_.sc[i], W_.nzs[i]);            \
    const int xc = xrow + (((4 * lq + s) ^ l16) << 4);                                                           \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                                                \
        fx[j] = *reinterpret_cast<const bf16x8*>(XS_ + j * (16 * BK * 2) + xc);                                  \
    _Pragma("unroll") for (int i = 0; i < WB; ++i) _Pragma("unroll") for (int j = 0; j < 8; ++j)                 \
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[i], fx[j], acc[i][j], 0, 0, 0);                   \
  }

  // Slabs [first_slab, first_slab + NB) of K; slab t sits in stage t % 2.  Per slab: wait for its X copies and W
  // words and for everybody to be done with the other stage, start the copies of the next slab into that stage and
  // the W loads of the next slab into registers, then multiply.  (Fetching two slabs ahead was measured in two forms
  // -- a hand-counted wait that leaves the youngest loads in flight, which the compiler's own reordering of loads and
  // copies defeats, and X through registers so that the compiler counts everything itself -- and gained nothing:
  // the loop is not waiting for memory.)
  const int nb_all = a.K / BK;
  const int first_slab = kpart * nb_all / a.split;
  const int NB = (kpart + 1) * nb_all / a.split - first_slab;
  SX_COPY(sx0, first_slab)
  WRaw w0 = load_w(first_slab);
  for (int t = 0; t < NB; t += 2) {
    {
      SX_WAIT_BARRIER()
      WRaw w1 = w0;
      if (t + 1 < NB) {
        SX_COPY(sx1, first_slab + t + 1)
        w1 = load_w(first_slab + t + 1);
      }
      SX_SLAB(sx0, w0)
      w0 = w1;
    }
    if (t + 1 < NB) {
      SX_WAIT_BARRIER()
      WRaw w1 = w0;
      if (t + 2 < NB) {
        SX_COPY(sx0, first_slab + t + 2)
        w1 = load_w(first_slab + t + 2);
      }
      SX_SLAB(sx1, w0)
      w0 = w1;
    }
  }
#undef SX_SLAB
#undef SX_COPY

  // ---- K split: partial sums meet in memory, the last workgroup to arrive adds them in part order -------------
  // (device-scope stores and loads, stores complete before the counter's device-scope atomic is issued)
  if (a.split > 1) {
    constexpr int kScopeDevice = 16;
    __shared__ int s_last;
    const __amdgpu_buffer_rsrc_t pres = make_rsrc(a.part);
    const unsigned mine =
        (unsigned)((tile_n * a.split + kpart) * kPartFloats + wave * (8 * WB * 256) + lane * 4) * 4u;  // bytes
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[i][j]), pres, mine + (i * 8 + j) * 1024, 0,
                                               kScopeDevice);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __syncthreads();
    if (tid == 0) {
      const int before = atomicAdd(a.part_cnt + tile_n, 1);
      s_last = before == a.split - 1;
      if (s_last) a.part_cnt[tile_n] = 0;  // ready for the next launch
    }
    __syncthreads();
    if (!s_last) return;
    // batches of 16 blocks per part, all loads of a batch in flight together (one memory round trip per batch
    // and part, not one per block); parts are added in part order
    const unsigned all = (unsigned)(tile_n * a.split * kPartFloats + wave * (8 * WB * 256) + lane * 4) * 4u;
#pragma unroll
    for (int b0 = 0; b0 < 8 * WB; b0 += 16) {
      f32x4 sum[16];
#pragma unroll
      for (int b = 0; b < 16; ++b)
        sum[b] = __builtin_bit_cast(
            f32x4, __builtin_amdgcn_raw_buffer_load_b128(pres, all + (b0 + b) * 1024, 0, kScopeDevice));
      for (int p = 1; p < a.split; ++p) {
        f32x4 t[16];
#pragma unroll
        for (int b = 0; b < 16; ++b)
          t[b] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                               pres, all + (unsigned)p * (kPartFloats * 4u) + (b0 + b) * 1024, 0,
                                               kScopeDevice));
#pragma unroll
        for (int b = 0; b < 16; ++b) sum[b] += t[b];
      }
#pragma unroll
      for (int b = 0; b < 16; ++b) acc[(b0 + b) >> 3][(b0 + b) & 7] = sum[b];
    }
  }

  // ---- epilogue.  acc[i][j][e]: output row 16 j + l16, column c0 + 16 i + 4 lq + e --------------------------------
  if (!wave_has_cols) return;
  const bool vec = (a.N & 3) == 0 && (a.ldy & 3) == 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int m = 16 * j + l16;
#pragma unroll
    for (int i = 0; i < WB; ++i) {
      const int n = c0 + 16 * i + 4 * lq;
      if (m >= a.M || n >= a.N) continue;
      float* y = a.Y + (size_t)m * a.ldy + n;
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
#undef SX_WAIT_BARRIER

}  // namespace

// Stacked 4-bit matrices (n1, n2 may be 0; every non-final segment a multiple of 64 rows), M <= 128, K a multiple of 128,
// group a power of two >= 64 dividing K.  Y fp32 [M][ldy] (ldy >= n0 + n1 + n2), mode store or residual.
// split_ws: 1 KB of counters (zero before the first launch; the kernel leaves them zero) followed by room for the
// partial sums; null = no K split.  Returns SX_ERR_SHAPE for shapes outside this form (the caller then takes the
// LDS-dequantising kernel).
int sx_launch_gemm_w4_regs(const void* X, const sx_w4_matrix* mats, const int* ns, int n_mats, int group, float* Y, int ldy,
                           int M, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st) {
  if (M < 1 || M > BM || K < BK || K % BK != 0 || n_mats < 1 || n_mats > 3) return SX_ERR_SHAPE;
  if (group < 64 || (group & (group - 1)) != 0 || K % group != 0) return SX_ERR_SHAPE;
  if (mode != SX_GEMM_STORE && mode != SX_GEMM_RESIDUAL) return SX_ERR_SHAPE;
  W4RegArgs a;
  int N = 0;
  for (int i = 0; i < 3; ++i) {
    const int n = i < n_mats ? ns[i] : 0;
    if (i < n_mats && (n < 1 || !mats[i].qweight || !mats[i].scales || !mats[i].zeros)) return SX_ERR_SHAPE;
    if (i + 1 < n_mats && n % 64 != 0) return SX_ERR_SHAPE;
    if (!sx_operand_fits_u32(n, K / 2)) return SX_ERR_SHAPE;
    const sx_w4_matrix& src = mats[i < n_mats ? i : 0];
    a.m[i].q = static_cast<const uint32_t*>(src.qweight);
    a.m[i].s = static_cast<const unsigned short*>(src.scales);
    a.m[i].z = static_cast<const unsigned char*>(src.zeros);
    N += n;
  }
  if (!sx_operand_fits_u32(M, 2ll * K) || ldy < N) return SX_ERR_SHAPE;
  a.X = static_cast<const unsigned short*>(X);
  a.n0 = ns[0];
  a.n1 = n_mats > 1 ? ns[1] : 0;
  a.n2 = n_mats > 2 ? ns[2] : 0;
  a.group_log2 = __builtin_ctz((unsigned)group);
  a.Y = Y;
  a.ldy = ldy;
  a.M = M;
  a.N = N;
  a.K = K;
  // Columns per workgroup: 128 (two blocks of 16 per wave).  256 was measured too (32 MFMAs per k-step against the
  // same 8 KB of X fragments): slower at every 7B and 70B layer shape but one, where it ties -- half the tiles,
  // K cut into twice the parts, twice the partial sums per part.
  constexpr int WB = 2;
  const int BN = 64 * WB;
  const int tilesN = (N + BN - 1) / BN;
  a.split = 1;
  a.part = nullptr;
  a.part_cnt = nullptr;
  // two workgroups fit a compute unit; cut K until the launch has about that many, parts of at least 4 slabs
  const int min_slabs = 4;
  const int slots = 2 * sx_compute_units(), nb = K / BK;
  if (split_ws && tilesN <= 256) {
    int split = slots / tilesN;
    if (split > 16) split = 16;
    while (split > 1 && nb / split < min_slabs) --split;
    if (split > 1 && split_ws_bytes >= 1024 + (size_t)tilesN * split * BM * BN * sizeof(float)) {
      a.split = split;
      a.part_cnt = static_cast<int*>(split_ws);
      a.part = reinterpret_cast<float*>(static_cast<char*>(split_ws) + 1024);
    }
  }
  const dim3 grid(tilesN, a.split);
  if (mode == SX_GEMM_STORE) gemm_w4_regs_kernel<SX_GEMM_STORE, WB><<<grid, kThreads, 0, st>>>(a);
  else gemm_w4_regs_kernel<SX_GEMM_RESIDUAL, WB><<<grid, kThreads, 0, st>>>(a);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
