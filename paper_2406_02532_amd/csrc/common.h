// Shared device/host helpers for the gfx950 kernels.  No arithmetic of the method lives here:
// only type aliases, bf16 bit helpers, wave/block reductions and launch-error plumbing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/specexec_mi.h"

#define SX_WAVE 64

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Offsets into a workspace: word 0 is the device-side status (0 = ok, else an sx_status).
#define SX_WS_HEADER 256

static inline size_t sx_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

#define SX_HIP_TRY(expr)                     \
  do {                                       \
    if ((expr) != hipSuccess) {              \
      (void)hipGetLastError();               \
      return SX_ERR_HIP;                     \
    }                                        \
  } while (0)

#define SX_LAUNCH_CHECK()                    \
  do {                                       \
    if (hipGetLastError() != hipSuccess) return SX_ERR_HIP; \
  } while (0)

// returns the callee's status from the caller unless it is SX_OK
#define SX_TRY(expr)                         \
  do {                                       \
    const int rc_ = (expr);                  \
    if (rc_ != SX_OK) return rc_;            \
  } while (0)

// Hands out 256-byte aligned pieces of a workspace; with a null base it only adds up sizes.
struct SxCarver {
  uintptr_t base;
  size_t off;
  SxCarver(void* p, size_t first) : base(reinterpret_cast<uintptr_t>(p)), off(first) {}
  template <typename T>
  T* take(size_t n) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += sx_align_up(n * sizeof(T), 256);
    return p;
  }
};

// compute units of the current device (256 if the runtime cannot tell)
static inline int sx_compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      n = 256;
  }
  return n;
}

// ---- bf16 <-> fp32 bit helpers ------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {  // round to nearest even (hardware cvt)
  __bf16 h = (__bf16)f;
  return (uint32_t)__builtin_bit_cast(unsigned short, h);
}
typedef float sx_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {  // both roundings in one v_cvt_pk_bf16_f32
  const sx_f32x2 t = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(t, bf16x2));
}

// silu(g) * u where the product is rounded to bf16 right after (the SwiGLU epilogues of the bf16 paths): the
// hardware's exp2 and reciprocal, one ulp each, instead of expf and an IEEE division -- 6 instructions for 30.
// The relative error, a few 1e-7, is four orders below the bf16 rounding step.  g -> -inf gives -0 as it should
// (exp2 overflows to +inf, whose reciprocal is 0).
__device__ __forceinline__ float silu_mul_bf16_bound(float g, float u) {
  return g * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f)) * u;
}

// ---- order-preserving float <-> uint map (larger float <=> larger key) ------------------------
__device__ __forceinline__ uint32_t f32_order_key(float f) {
  uint32_t b = __float_as_uint(f + 0.0f);  // -0 -> +0 so that the two compare equal
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float f32_from_order_key(uint32_t k) {
  uint32_t b = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
  return __uint_as_float(b);
}

// ---- wave reductions (64 lanes) ---------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ int wave_min_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  return v;
}

// Block reductions over NW waves through a small LDS array (at least NW entries).  Every thread
// gets the result.  Two barriers per call; the summation order is fixed, so results are
// reproducible run to run.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) s += red[w];
  return s;
}
template <int NW>
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) s = fmaxf(s, red[w]);
  return s;
}
template <int NW>
__device__ __forceinline__ int block_sum_i(int v, int* red) {
  v = wave_sum_i(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) s += red[w];
  return s;
}
template <int NW>
__device__ __forceinline__ int block_min_i(int v, int* red) {
  v = wave_min_i(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  int s = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) s = min(s, red[w]);
  return s;
}

// Ascending bitonic sort of n (a power of two) 64-bit keys held in LDS, by all NT threads of the
// block.  Ends with a barrier.
template <int NT>
__device__ __forceinline__ void block_bitonic_sort_u64(unsigned long long* a, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int i = threadIdx.x; i < (n >> 1); i += NT) {
        int lo = ((i / stride) * (stride << 1)) + (i % stride);
        int hi = lo + stride;
        bool up = ((lo & size) == 0);
        unsigned long long x = a[lo], y = a[hi];
        if ((x > y) == up) {
          a[lo] = y;
          a[hi] = x;
        }
      }
    }
  }
  __syncthreads();
}

__device__ __forceinline__ int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}
