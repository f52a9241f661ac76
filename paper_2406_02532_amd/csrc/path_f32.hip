// fp32 variants of the two heavy pieces of the forward (Alg. 1, FORWARD; App. D tree mask), used when
// the model dtype is fp32 (the tiny configuration that is compared with the oracle to 1e-4).  Plain
// FMA, no matrix cores: clarity and exact fp32 semantics matter here, not speed.
#include "kernels.h"

namespace {

// 64x64 output tile, 16-deep K slabs staged in LDS, 256 lanes x (4x4) outputs.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ X, const float* __restrict__ W,
                                                       float* __restrict__ Y, int M, int N, int K, int ldy,
                                                       int accumulate) {
  __shared__ float xs[16][64 + 1];
  __shared__ float ws[16][64 + 1];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int e = tid; e < 64 * 16; e += 256) {
      const int r = e / 16, c = e % 16;
      const int m = m0 + r, n = n0 + r, kk = k0 + c;
      xs[c][r] = (m < M && kk < K) ? X[(size_t)m * K + kk] : 0.f;
      ws[c][r] = (n < N && kk < K) ? W[(size_t)n * K + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = xs[c][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = ws[c][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float* y = Y + (size_t)m * ldy + n;
      *y = accumulate ? (*y + acc[i][j]) : acc[i][j];
    }
  }
}

// One workgroup per (node, query head).  Keys = the P prefix rows, then the node's ancestors and
// itself (found by walking parent pointers).  LDS: scores for all keys, then the ancestor list.
constexpr int kAttnThreads = 128;
__global__ __launch_bounds__(kAttnThreads) void tree_attn_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k_tree, const float* __restrict__ v_tree,
    const float* __restrict__ k_prefix, const float* __restrict__ v_prefix, const int* __restrict__ par_s,
    const int* __restrict__ depth, int first, int P, int Hq, int Hkv, int Dh, float* __restrict__ out) {
  extern __shared__ float lds[];
  __shared__ float red[2];
  const int node = first + blockIdx.x, h = blockIdx.y;
  const int kv = h / (Hq / Hkv);
  const int na = depth[node] + 1;
  const int nk = P + na;
  float* sc = lds;                                 // [nk]
  int* anc = reinterpret_cast<int*>(lds + nk);     // [na]
  const int tid = threadIdx.x;
  if (tid == 0) {
    int j = node;
    for (int s = na - 1; s >= 0; --s) {
      anc[s] = j;
      j = par_s[j];
    }
  }
  __syncthreads();
  const float* qv = q + ((size_t)blockIdx.x * Hq + h) * Dh;
  const float scale = 1.0f / sqrtf((float)Dh);
  float mx = -__builtin_huge_valf();
  for (int j = tid; j < nk; j += kAttnThreads) {
    const float* kr = (j < P) ? k_prefix + ((size_t)j * Hkv + kv) * Dh : k_tree + ((size_t)anc[j - P] * Hkv + kv) * Dh;
    float s = 0.f;
    for (int c = 0; c < Dh; ++c) s += qv[c] * kr[c];
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = block_max<2>(mx, red);
  float sum = 0.f;
  for (int j = tid; j < nk; j += kAttnThreads) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = block_sum<2>(sum, red);  // includes the barrier that publishes sc[]
  const float inv = 1.0f / sum;
  for (int c = tid; c < Dh; c += kAttnThreads) {
    float o = 0.f;
    for (int j = 0; j < nk; ++j) {
      const float* vr = (j < P) ? v_prefix + ((size_t)j * Hkv + kv) * Dh : v_tree + ((size_t)anc[j - P] * Hkv + kv) * Dh;
      o += sc[j] * vr[c];
    }
    out[((size_t)blockIdx.x * Hq + h) * Dh + c] = o * inv;
  }
}

}  // namespace

int sx_launch_gemm_f32(const float* X, const float* W, float* Y, int M, int N, int K, int ldy, bool accumulate,
                       hipStream_t st) {
  dim3 grid((N + 63) / 64, (M + 63) / 64);
  gemm_f32_kernel<<<grid, 256, 0, st>>>(X, W, Y, M, N, K, ldy, accumulate ? 1 : 0);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_tree_attn_f32(const float* q, const float* k_tree, const float* v_tree, const float* k_prefix,
                            const float* v_prefix, const int32_t* par_s, const int32_t* depth, int T, int first, int P,
                            int Hq, int Hkv, int Dh, float* out, hipStream_t st) {
  // worst case: a chain, depth T-1
  const size_t shmem = (size_t)(P + 2 * T) * sizeof(float);
  if (shmem > 60 * 1024) return SX_ERR_SHAPE;
  dim3 grid(T - first, Hq);
  tree_attn_f32_kernel<<<grid, kAttnThreads, shmem, st>>>(q, k_tree, v_tree, k_prefix, v_prefix, par_s, depth, first, P,
                                                          Hq, Hkv, Dh, out);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
