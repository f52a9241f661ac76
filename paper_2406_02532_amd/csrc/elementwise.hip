// The small memory-bound pieces of the decoder forward (Alg. 1, FORWARD): embedding gather,
// RMSNorm, rotary embedding at position P + tree depth, SwiGLU (fp32 path only; the bf16 path
// fuses it into the gate/up GEMM).
#include "kernels.h"

namespace {

template <typename T>
__device__ __forceinline__ float ld(const T* p, size_t i);
template <>
__device__ __forceinline__ float ld<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ld<unsigned short>(const unsigned short* p, size_t i) {
  return bf16_bits_to_f32(p[i]);
}
template <typename T>
__device__ __forceinline__ void st(T* p, size_t i, float v);
template <>
__device__ __forceinline__ void st<float>(float* p, size_t i, float v) { p[i] = v; }
template <>
__device__ __forceinline__ void st<unsigned short>(unsigned short* p, size_t i, float v) {
  p[i] = (unsigned short)f32_to_bf16_bits(v);
}

template <typename W>
__global__ void embed_kernel(const W* __restrict__ embed, const int* __restrict__ tok, int d, float* __restrict__ h) {
  const int i = blockIdx.x;
  const size_t src = (size_t)tok[i] * d, dst = (size_t)i * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) h[dst + c] = ld<W>(embed, src + c);
}

// One workgroup (256 lanes) per row: x = h * rsqrt(mean(h^2) + eps) * g.
template <typename W>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h, const W* __restrict__ g, int d,
                                                      float eps, W* __restrict__ x) {
  __shared__ float red[4];
  const size_t row = (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) {
    const float v = h[row + c];
    ss += v * v;
  }
  ss = block_sum<4>(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += 256) st<W>(x, row + c, h[row + c] * r * ld<W>(g, c));
}

// Same for d = 1024 * VPT and bf16 output: the row is read once, 16 bytes per lane and instruction, and
// stays in registers between the two passes.
template <int VPT>
__global__ __launch_bounds__(256) void rmsnorm_row_in_regs_kernel(const float* __restrict__ h,
                                                                  const unsigned short* __restrict__ g, float eps,
                                                                  unsigned short* __restrict__ x) {
  __shared__ float red[4];
  constexpr int d = 1024 * VPT;
  const f32x4* hr = reinterpret_cast<const f32x4*>(h + (size_t)blockIdx.x * d);
  f32x4 v[VPT];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    v[i] = hr[i * 256 + threadIdx.x];
    ss += v[i][0] * v[i][0] + v[i][1] * v[i][1] + v[i][2] * v[i][2] + v[i][3] * v[i][3];
  }
  ss = block_sum<4>(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)d + eps);
  const u32x2* gr = reinterpret_cast<const u32x2*>(g);
  u32x2* xr = reinterpret_cast<u32x2*>(x + (size_t)blockIdx.x * d);
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const u32x2 gg = gr[i * 256 + threadIdx.x];
    const float g0 = bf16_bits_to_f32(gg[0] & 0xffffu), g1 = bf16_bits_to_f32(gg[0] >> 16);
    const float g2 = bf16_bits_to_f32(gg[1] & 0xffffu), g3 = bf16_bits_to_f32(gg[1] >> 16);
    u32x2 o;
    o[0] = f32_to_bf16_bits(v[i][0] * r * g0) | (f32_to_bf16_bits(v[i][1] * r * g1) << 16);
    o[1] = f32_to_bf16_bits(v[i][2] * r * g2) | (f32_to_bf16_bits(v[i][3] * r * g3) << 16);
    xr[i * 256 + threadIdx.x] = o;
  }
}

// Pair (j, j + Dh/2) of every q and k head is rotated by the node's angle; v is copied.
template <typename W>
__global__ void rope_split_kernel(const float* __restrict__ qkv, const float2* __restrict__ cs, int T, int Hq, int Hkv,
                                  int Dh, W* __restrict__ q, W* __restrict__ k, W* __restrict__ v) {
  const int half = Dh / 2;
  const int heads = Hq + 2 * Hkv;
  const size_t total = (size_t)T * heads * half;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int j = (int)(idx % half);
  const int hd = (int)((idx / half) % heads);
  const int i = (int)(idx / ((size_t)half * heads));
  const float* src = qkv + ((size_t)i * heads + hd) * Dh;
  const float a = src[j], b = src[j + half];
  if (hd < Hq + Hkv) {
    const float2 t = cs[(size_t)i * half + j];
    const float ra = a * t.x - b * t.y, rb = a * t.y + b * t.x;
    if (hd < Hq) {
      const size_t o = ((size_t)i * Hq + hd) * Dh;
      st<W>(q, o + j, ra);
      st<W>(q, o + j + half, rb);
    } else {
      const size_t o = ((size_t)i * Hkv + (hd - Hq)) * Dh;
      st<W>(k, o + j, ra);
      st<W>(k, o + j + half, rb);
    }
  } else {
    const size_t o = ((size_t)i * Hkv + (hd - Hq - Hkv)) * Dh;
    st<W>(v, o + j, a);
    st<W>(v, o + j + half, b);
  }
}

__global__ void swiglu_f32_kernel(const float* __restrict__ g, const float* __restrict__ u, float* __restrict__ a,
                                  size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const float x = g[i];
    a[i] = x / (1.0f + expf(-x)) * u[i];
  }
}

// act[i][f] = bf16(silu(gu[i][f]) * gu[i][F + f]): the SwiGLU of a gate|up product kept in fp32 (4-bit path)
__global__ void swiglu_pair_bf16_kernel(const float* __restrict__ gu, int n, int F, unsigned short* __restrict__ act) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * F) return;
  const size_t i = idx / F, f = idx % F;
  const float g = gu[i * 2 * F + f], u = gu[i * 2 * F + F + f];
  act[idx] = (unsigned short)f32_to_bf16_bits(silu_mul_bf16_bound(g, u));
}

// One 32-bit word of eight 4-bit codes per thread -> eight bf16 weights w = bf16(scale * (code - zero)) (16 bytes).
__global__ void dequant_w4_kernel(const uint32_t* __restrict__ q, const unsigned short* __restrict__ sc,
                                  const unsigned char* __restrict__ zr, size_t words, int words_per_row, int group_log2,
                                  int groups_per_row, unsigned short* __restrict__ W) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= words) return;
  const size_t row = idx / words_per_row;
  const int wi = (int)(idx % words_per_row);
  const size_t g = row * groups_per_row + ((wi * 8) >> group_log2);
  const float s = bf16_bits_to_f32(sc[g]);
  const float z = (float)zr[g];
  const uint32_t v = q[idx];
  u32x4 o;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const float e = (float)((int)((v >> (8 * b)) & 15u)) - z, f = (float)((int)((v >> (8 * b + 4)) & 15u)) - z;
    o[b] = pack_bf16x2(e * s, f * s);  // exact products (8 significant bits times at most 5), rounded once
  }
  *reinterpret_cast<u32x4*>(W + idx * 8) = o;
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace

int sx_launch_embed(const void* embed, int dtype, const int32_t* tok_s, int T, int d, float* h, hipStream_t s) {
  if (dtype == SX_F32)
    embed_kernel<float><<<T, 256, 0, s>>>((const float*)embed, tok_s, d, h);
  else
    embed_kernel<unsigned short><<<T, 256, 0, s>>>((const unsigned short*)embed, tok_s, d, h);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_rmsnorm(const float* h, const void* gain, int dtype, int T, int d, float eps, void* x_out,
                      hipStream_t s) {
  if (dtype == SX_F32)
    rmsnorm_kernel<float><<<T, 256, 0, s>>>(h, (const float*)gain, d, eps, (float*)x_out);
  else if (d == 8192)
    rmsnorm_row_in_regs_kernel<8><<<T, 256, 0, s>>>(h, (const unsigned short*)gain, eps, (unsigned short*)x_out);
  else if (d == 4096)
    rmsnorm_row_in_regs_kernel<4><<<T, 256, 0, s>>>(h, (const unsigned short*)gain, eps, (unsigned short*)x_out);
  else
    rmsnorm_kernel<unsigned short><<<T, 256, 0, s>>>(h, (const unsigned short*)gain, d, eps, (unsigned short*)x_out);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_rope_split(const float* qkv, const float2* rope_cs, int T, int Hq, int Hkv, int Dh, int dtype, void* q,
                         void* k, void* v, hipStream_t s) {
  const size_t total = (size_t)T * (Hq + 2 * Hkv) * (Dh / 2);
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (dtype == SX_F32)
    rope_split_kernel<float><<<blocks, 256, 0, s>>>(qkv, rope_cs, T, Hq, Hkv, Dh, (float*)q, (float*)k, (float*)v);
  else
    rope_split_kernel<unsigned short><<<blocks, 256, 0, s>>>(qkv, rope_cs, T, Hq, Hkv, Dh, (unsigned short*)q,
                                                             (unsigned short*)k, (unsigned short*)v);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_zero_i32(int32_t* p, int n, hipStream_t s) {
  zero_i32_kernel<<<(n + 255) / 256, 256, 0, s>>>(p, n);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_swiglu_pair_bf16(const float* gu, int n, int F, void* act, hipStream_t s) {
  const size_t total = (size_t)n * F;
  swiglu_pair_bf16_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(gu, n, F, (unsigned short*)act);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_dequant_w4(const sx_w4_matrix* m, int N, int K, int group, void* W_bf16, hipStream_t s) {
  if (!m || !m->qweight || !m->scales || !m->zeros || !W_bf16) return SX_ERR_NULL;
  if (N < 1 || K < 8 || K % 8 != 0 || group < 8 || (group & (group - 1)) != 0 || K % group != 0) return SX_ERR_SHAPE;
  const size_t words = (size_t)N * (K / 8);
  dequant_w4_kernel<<<(unsigned)((words + 255) / 256), 256, 0, s>>>(
      (const uint32_t*)m->qweight, (const unsigned short*)m->scales, (const unsigned char*)m->zeros, words, K / 8,
      __builtin_ctz((unsigned)group), K / group, (unsigned short*)W_bf16);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_swiglu_f32(const float* g, const float* u, float* a, size_t n, hipStream_t s) {
  swiglu_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(g, u, a, n);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
