// Tree bookkeeping for the verification forward: what the paper calls the path pi(x_i, tau) of a
// node (Alg. 1, App. A) turned into the data the kernels need -- depth (= rotary position offset),
// and, for the tensor-core attention kernel, the "merged attention mask" of App. D in a compact
// form: per tile of query nodes the sorted union of their ancestors, per node a bitmask over it.
#include "kernels.h"

namespace {

constexpr int kPrepThreads = 1024;

// One workgroup.  Validates, sanitises (bad parent -> -1, bad token -> 0) and computes depths by
// walking the sanitised parent array held in LDS.
__global__ __launch_bounds__(kPrepThreads) void tree_prep_kernel(const int* __restrict__ tokens,
                                                                 const int* __restrict__ parent, int T, int V,
                                                                 int* __restrict__ tok_s, int* __restrict__ par_s,
                                                                 int* __restrict__ depth, int* __restrict__ status, int reset) {
  extern __shared__ int sp[];
  const int tid = threadIdx.x;
  int bad = 0;
  for (int i = tid; i < T; i += kPrepThreads) {
    int p = parent[i];
    int t = tokens ? tokens[i] : 0;  // tokens may be absent (attention-only entry point)
    if (p < -1 || p >= i) {
      bad = 1;
      p = -1;
    }
    if (t < 0 || t >= V) {
      bad = 1;
      t = 0;
    }
    sp[i] = p;
    par_s[i] = p;
    tok_s[i] = t;
  }
  if (tid == 0 && reset) status[0] = SX_OK;  // a call that continues a tree (reset == 0) keeps an earlier call's error
  __syncthreads();
  if (bad) status[0] = SX_ERR_TREE;
  for (int i = tid; i < T; i += kPrepThreads) {
    int d = 0;
    for (int j = sp[i]; j >= 0; j = sp[j]) ++d;  // sp[j] < j: the walk ends after at most i steps
    depth[i] = d;
  }
}

// cos/sin of (P + depth) * base^(-2j/Dh), angle and functions in fp64, stored as fp32.
__global__ void rope_table_kernel(const int* __restrict__ depth, int T, int P, int half, double log_base,
                                  float2* __restrict__ cs) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= T * half) return;
  const int i = idx / half, j = idx % half;
  const double inv = exp(-log_base * (double)j / (double)half);  // base^(-2j/Dh), Dh = 2*half
  const double ang = (double)(P + depth[i]) * inv;
  cs[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

// One workgroup per query tile.
constexpr int kQtThreads = 256;
// Tiles cover the query nodes first, first + 1, ..., T - 1 (first > 0: the earlier nodes were processed by
// a previous call and only serve as keys); rowmask rows are indexed by node - first.
__global__ __launch_bounds__(kQtThreads) void qtile_prep_kernel(const int* __restrict__ par_s, int T, int npt, int first,
                                                                int* __restrict__ klist, int* __restrict__ kcnt,
                                                                unsigned long long* __restrict__ rowmask) {
  extern __shared__ unsigned int lds[];
  const int W = (T + 31) / 32;      // words of the ancestor bitmap
  const int W64 = (T + 63) / 64;    // row stride of rowmask
  unsigned int* bm = lds;           // [W]   union of ancestors-or-self over the tile's nodes
  unsigned int* pre = lds + W;      // [W+1] exclusive prefix of popcounts
  const int tid = threadIdx.x;
  const int tile = blockIdx.x;
  const int n0 = first + tile * npt;
  for (int w = tid; w < W; w += kQtThreads) bm[w] = 0u;
  __syncthreads();
  if (tid < npt && n0 + tid < T) {
    for (int j = n0 + tid; j >= 0; j = par_s[j]) atomicOr(&bm[j >> 5], 1u << (j & 31));
  }
  __syncthreads();
  for (int w = tid; w <= W; w += kQtThreads) {
    int s = 0;
    for (int x = 0; x < w; ++x) s += __popc(bm[x]);
    pre[w] = (unsigned)s;
  }
  __syncthreads();
  const int cnt = (int)pre[W];
  if (tid == 0) kcnt[tile] = cnt;
  int* kl = klist + (size_t)tile * (size_t)T;
  for (int w = tid; w < W; w += kQtThreads) {
    unsigned int bits = bm[w];
    int o = (int)pre[w];
    while (bits) {
      const int b = __ffs(bits) - 1;
      kl[o++] = w * 32 + b;
      bits &= bits - 1;
    }
  }
  // per-node masks over list positions; each row is touched by its own lane only
  const int nw = (cnt + 63) / 64;
  if (tid < npt && n0 + tid < T) {
    unsigned long long* rm = rowmask + (size_t)(n0 + tid - first) * (size_t)W64;
    for (int w = 0; w < nw; ++w) rm[w] = 0ull;
    for (int j = n0 + tid; j >= 0; j = par_s[j]) {
      const int pos = (int)pre[j >> 5] + __popc(bm[j >> 5] & ((1u << (j & 31)) - 1u));
      rm[pos >> 6] |= 1ull << (pos & 63);
    }
  }
}

}  // namespace

int sx_launch_tree_prep(const int32_t* tokens, const int32_t* parent, int T, int V, int P, int head_dim,
                        float rope_base, int32_t* tok_s, int32_t* par_s, int32_t* depth, float2* rope_cs,
                        int32_t* status, bool reset_status, hipStream_t st) {
  tree_prep_kernel<<<1, kPrepThreads, (size_t)T * sizeof(int), st>>>(tokens, parent, T, V, tok_s, par_s, depth, status,
                                                                     reset_status ? 1 : 0);
  SX_LAUNCH_CHECK();
  return sx_launch_rope_table(depth, T, P, head_dim, rope_base, rope_cs, st);
}

int sx_launch_rope_table(const int32_t* pos, int T, int P, int head_dim, float rope_base, float2* rope_cs, hipStream_t st) {
  const int half = head_dim / 2;
  const int n = T * half;
  rope_table_kernel<<<(n + 255) / 256, 256, 0, st>>>(pos, T, P, half, log((double)rope_base), rope_cs);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

int sx_launch_qtile_prep(const int32_t* par_s, int T, int nodes_per_tile, int first, int32_t* klist, int32_t* kcnt,
                         unsigned long long* rowmask, hipStream_t st) {
  const int tiles = (T - first + nodes_per_tile - 1) / nodes_per_tile;
  const int W = (T + 31) / 32;
  qtile_prep_kernel<<<tiles, kQtThreads, (size_t)(2 * W + 1) * sizeof(unsigned int), st>>>(par_s, T, nodes_per_tile,
                                                                                           first, klist, kcnt, rowmask);
  SX_LAUNCH_CHECK();
  return SX_OK;
}
