// Y = X W^T on the gfx950 matrix cores: the linear layers of the decoder forward (Alg. 1, FORWARD) at
// M = number of tree tokens.  bf16 operands, fp32 accumulation.
//
// Tiling.  A workgroup of 4 waves (2 x 2) owns a 256 x 256 output tile; each wave a 128 x 128
// quadrant = 8 x 8 blocks of v_mfma_f32_16x16x32_bf16, 256 fp32 accumulators per lane.  With real
// operand data the chip is power-limited long before the MFMA issue rate is: in a pure register loop
// the 16x16x32 shape sustains ~1.95 PFLOP/s against ~1.75 for 32x32x16 (it holds a ~10% higher
// clock), which is why the smaller block is used.  The product is formed transposed (W rows feed
// the A operand, X rows the B operand), so a lane ends up with 4 consecutive output columns of one
// row: 16-byte stores.
//
// K is walked in slabs of 64 (two MFMA k-steps, 128 MFMAs per wave) held in two LDS stages of 64 KB.
//
// Global -> LDS without registers.  Operand slabs are copied by buffer loads that write LDS
// directly (16 bytes per lane, a wave fills 1 KB of consecutive LDS per instruction), so the K loop
// spends no vector registers and no LDS-write instructions on staging.  Both operands are
// K-contiguous in memory, which is the per-lane layout the MFMA wants (8 consecutive k per lane),
// so an LDS row is a plain 128-byte row segment; the XOR swizzle of its 16-byte chunks that makes
// fragment reads conflict-free on the 64-bank LDS is applied on the global side (each lane picks
// the chunk whose swizzled position is the lane's slot in the wave's 1 KB).  Eight lanes fetch
// one whole 128-byte line.  That matters: the copy stream of this kernel alone (no math) runs at
// 17 TB/s L2 -> LDS with whole-line requests and at 11.5 TB/s with half-line ones, which would make
// the copies, not the MFMAs, the bound.  Whole lines are why a stage holds 64 K-elements and why
// there are only two of them.
// Each stage is its own __shared__ array: the compiler tracks outstanding loads-to-LDS per array,
// so a fragment read of one stage does not wait for the copies in flight to the other.
//
// Schedule of a slab (stage S, other stage S'): phase 1 runs the MFMAs of k-step 0 and reads the
// fragments of k-step 1; then one barrier, before which every wave waits for its own copies of the
// next slab (now S' is complete and S is read out); phase 2 runs the MFMAs of k-step 1, starts the
// copies of the slab after next into S and reads the next slab's k-step 0 from S'.  One barrier
// per 128 MFMAs; a copy has about a slab's worth of MFMAs to arrive.  Copies and fragment reads
// are dealt out evenly between the MFMAs: bursts of copies fill the memory pipeline's queues and
// stall the wave that issues them.
//
// XCD-aware tile order.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.
// Tile index = xcd * chunk + id / 8 with tiles ordered M-fastest, so the workgroups resident on
// one XCD at a time share the same few W column tiles (fetched from HBM once per XCD) and sweep
// all of X's row tiles.
//
// Epilogues: store fp32, add into an fp32 residual, or SwiGLU.  For SwiGLU the W slab interleaves
// 16-row groups of W_gate and W_up, so gate and up of one output column sit in the same lane and
// register of neighbouring accumulator blocks and silu(g)*u needs no data movement.
#include "kernels.h"

namespace {

constexpr int BM = 256, BN = 256;
constexpr int BK = 64;                    // K elements per LDS stage ("slab"): two MFMA k-steps, whole 128-byte lines
constexpr int kThreads = 256;
constexpr int kOperandBytes = BM * BK * 2;            // 32 KB: one operand of one slab
constexpr int kStageBytes = 2 * kOperandBytes;        // X slab then W slab
constexpr int kPfDist = 3;                            // slabs between an L2 prefetch and the copy of the same lines

struct GemmArgs {
  const unsigned short* X;
  const unsigned short* W0;
  const unsigned short* W1;
  const unsigned short* W2;
  int n0, n1, n2;
  void* Y;
  int M, N, K;  // N = logical output columns
  int tilesM, tilesN, chunk;
  // SX_GEMM_QKV_ROPE only: rotary table [M][64] (cos, sin), outputs bf16 [M][hq][128], [M][hkv][128] x 2
  const float2* cs;
  unsigned short *q, *k, *v;
  int hq, hkv;
  // K split of the tail tiles (split > 1): partial sums [tail tile][split][wave][block][lane] f32x4, counters
  float* part;
  int* part_cnt;
  int split, full_tiles, tail_items, full_per_xcd, tail_per_xcd;
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;

// Raw buffer resource over a whole matrix (no bounds: rows are clamped by the caller; < 4 GB).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, -1, 0x00020000);
}

// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]):
// all LDS reads done, at most N vector-memory operations outstanding.
constexpr int kWaitVm0 = 0x0070, kWaitVm2 = 0x0072, kWaitVm16 = 0x4070, kWaitVm18 = 0x4072;

// Wait until this wave's LDS reads are done and at most the given number of copies are in flight, then
// meet the other waves.  The barrier intrinsic alone does not order memory operations for the compiler,
// and a workgroup fence makes it wait for every copy in flight, so empty asm statements that claim to
// touch memory pin the LDS reads and the copies to their side of the barrier instead.
#define SX_WAIT_BARRIER(IMM)              \
  asm volatile("" ::: "memory");          \
  __builtin_amdgcn_s_waitcnt(IMM);        \
  __builtin_amdgcn_s_barrier();           \
  asm volatile("" ::: "memory");

template <int MODE, bool PF>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(GemmArgs a) {
  // One array per stage (see the header).  Row r of an operand's slab is 128 bytes at r * 128; 16-byte
  // chunk c of the row sits at position c ^ ((r >> 1) & 7).  The LDS serves 16 lanes x 16 bytes per
  // cycle (64 banks): 16 consecutive rows reading the same k chunk fall on 16 different bank groups.
  __shared__ __attribute__((aligned(1024))) unsigned char stA[kStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char stB[kStageBytes];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l16 = lane & 15, lq = lane >> 4;

  // ---- which tile ----------------------------------------------------------------------------
  // Without a K split: tile lin = xcd * chunk + slot.  With one (a.split > 1) the first full_per_xcd
  // slots of an XCD are whole tiles and the rest are the tail: the last few tiles, which would
  // otherwise occupy a fraction of the chip for a whole round, each cut into a.split K ranges.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int lin, kpart = 0, ksplit = 1;
  if (a.split > 1) {
    if (slot < a.full_per_xcd) {
      lin = xcd * a.full_per_xcd + slot;
      if (lin >= a.full_tiles) return;
    } else {
      const int idx = xcd * a.tail_per_xcd + (slot - a.full_per_xcd);
      if (slot - a.full_per_xcd >= a.tail_per_xcd || idx >= a.tail_items) return;
      lin = a.full_tiles + idx / a.split;
      kpart = idx % a.split;
      ksplit = a.split;
    }
  } else {
    lin = xcd * a.chunk + slot;
    if (slot >= a.chunk || lin >= a.tilesM * a.tilesN) return;
  }
  const int tile_m = lin % a.tilesM, tile_n = lin / a.tilesM;

  // ---- global sources of this lane's copies ---------------------------------------------------------
  // Copy instruction t (0..7) of wave w fills rows 64 w + 8 t .. + 7 of an operand's slab (1 KB of LDS):
  // lane l supplies row 64 w + 8 t + l / 8, LDS chunk position l % 8, i.e. k chunk
  // (l % 8) ^ ((row >> 1) & 7) with (row >> 1) & 7 = (4 t + l / 16) & 7.  Eight lanes read one whole
  // 128-byte line: the L2 serves whole-line requests half again as fast as half-line ones.  An 8-row
  // group never straddles two weight matrices (segment sizes are multiples of 16).
  const int crow = 64 * wave + (lane >> 3);
  const __amdgpu_buffer_rsrc_t xres = make_rsrc(a.X);
  const __amdgpu_buffer_rsrc_t wres0 = make_rsrc(a.W0), wres1 = make_rsrc(a.W1), wres2 = make_rsrc(a.W2);
  __amdgpu_buffer_rsrc_t wres[8];
  int xoff[8], woff[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int r = crow + 8 * t;
    const int cchunk = (lane & 7) ^ ((4 * (t & 1) + (lane >> 4)) & 7);
    int m = tile_m * BM + r;
    m = m < a.M ? m : a.M - 1;
    xoff[t] = (int)(((unsigned)m * (unsigned)a.K + cchunk * 8) * 2u);
    if (MODE == SX_GEMM_SWIGLU) {
      // slab rows in 16-row groups: even group = gate, odd = up; rows 64 w + 8 t are in group 4 w + t / 2
      int f = tile_n * (BN / 2) + (2 * wave + (t >> 2)) * 16 + (t & 1) * 8 + (lane >> 3);
      f = f < a.N ? f : a.N - 1;
      wres[t] = (t & 2) ? wres1 : wres0;
      woff[t] = (int)(((unsigned)f * (unsigned)a.K + cchunk * 8) * 2u);
    } else {
      const int g0 = min(tile_n * BN + 64 * wave + 8 * t, a.N - 1);  // first row of the group decides the matrix
      int n = tile_n * BN + r;
      n = n < a.N ? n : a.N - 1;
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
  const int cdst = wave * 8192;  // this wave's 8 KB of an operand's slab

  // ---- L2 prefetch (PF kernels: 8 row tiles, column tiles a multiple of 4) ---------------------------
  // The 32 workgroups that run side by side on an XCD are then 8 row tiles x 4 column tiles: an X tile
  // is read by 4 of them and a W tile by 8, at about the same time, so all of them wait for the one
  // fabric access.  Instead each touches its share of the lines (X: 64 rows = 16 per wave; W: 32 rows
  // = 8 per wave; one dword per 128-byte line) kPfDist slabs ahead, and the copies of all of them find
  // the lines in L2.  Measured at the 70B shapes: QKV +12%, gate/up +4%, down +6%, O -3%.  (Where nobody shares --
  // other tile counts -- a workgroup touching all of its own lines ahead of its copies was measured too: 5 to 20%
  // slower at every shape and distance; the copies are not waiting for HBM latency there.)
  int pfx = 0, pfw = 0, pfxoff = 0, pfwoff = 0;
  __amdgpu_buffer_rsrc_t pfwres = wres0;
  if (PF) {
    int m = tile_m * BM + 64 * (tile_n & 3) + 16 * wave + (lane & 15);
    m = m < a.M ? m : a.M - 1;
    pfxoff = (int)((unsigned)m * (unsigned)a.K * 2u);
    const int r = 32 * tile_m + 8 * wave;  // slab row of this wave's 8 W rows (uniform)
    if (MODE == SX_GEMM_SWIGLU) {
      int f = tile_n * (BN / 2) + (r >> 5) * 16 + (r & 15) + (lane & 7);
      f = f < a.N ? f : a.N - 1;
      pfwres = ((r >> 4) & 1) ? wres1 : wres0;
      pfwoff = (int)((unsigned)f * (unsigned)a.K * 2u);
    } else {
      const int g0 = min(tile_n * BN + r, a.N - 1);
      int n = min(tile_n * BN + r + (lane & 7), a.N - 1);
      int first = 0;
      if (g0 >= a.n0 + a.n1) {
        pfwres = wres2;
        first = a.n0 + a.n1;
      } else if (g0 >= a.n0) {
        pfwres = wres1;
        first = a.n0;
      }
      pfwoff = (int)((unsigned)(n - first) * (unsigned)a.K * 2u);
    }
  }

  // acc[i][j]: W rows (output columns) 16 i .. + 15 of the quadrant, X rows (output rows) 16 j .. + 15
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // fragment addresses: row (quadrant base + 16 i + l16), k chunk 4 ks + lq at position ^ ((row >> 1) & 7)
  const int fsw = (l16 >> 1) & 7;
  const int xrow = (wm * 128 + l16) * (BK * 2);
  const int wrow = kOperandBytes + (wn * 128 + l16) * (BK * 2);
  const int kc0 = ((lq ^ fsw) << 4), kc1 = (((4 + lq) ^ fsw) << 4);
  bf16x8 fx0[8], fw0[8], fx1[8], fw1[8];   // k-step 0 and k-step 1 of a slab

// One copy instruction: rows 8 t .. + 7 of this wave's share of X (OP_ 0) or W (OP_ 1) at byte offset SO_
// along K into stage STG_.  The K offset travels in the scalar offset: the instruction's immediate
// offset would be added to the LDS address as well.
#define SX_COPY1(STG_, SO_, OP_, t)                                                                            \
  if (OP_)                                                                                                     \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(wres[t], (lds_void_ptr)(STG_ + kOperandBytes + cdst + (t) * 1024), 16,   \
                                             woff[t], SO_, 0, 0);                                              \
  else                                                                                                         \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_void_ptr)(STG_ + cdst + (t) * 1024), 16, xoff[t], SO_, 0, 0);
#define SX_COPY(STG_, SLAB_)                                                                                   \
  _Pragma("unroll") for (int t = 0; t < 8; ++t) {                                                             \
    SX_COPY1(STG_, (SLAB_) * (BK * 2), 0, t)                                                                   \
    SX_COPY1(STG_, (SLAB_) * (BK * 2), 1, t)                                                                   \
  }
#define SX_READW(STG_, FW, i, KC) FW[i] = *reinterpret_cast<const bf16x8*>(STG_ + wrow + (i) * (16 * BK * 2) + KC);
#define SX_READX(STG_, FX, i, KC) FX[i] = *reinterpret_cast<const bf16x8*>(STG_ + xrow + (i) * (16 * BK * 2) + KC);
// The MFMA is written out: left to itself the compiler gives an accumulator that is updated more than
// once per loop body a new destination register each time and shuffles hundreds of registers per
// iteration to undo it.  "+a" keeps every accumulator in place in the accumulation registers.  The
// statements are volatile, so the issue order below is the one written here.
#define SX_MFMA(ACC, A, B) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(A), "v"(B));
#define SX_MMA(FX, FW)                                                                                         \
  _Pragma("unroll") for (int i = 0; i < 8; ++i) _Pragma("unroll") for (int j = 0; j < 8; ++j)                  \
      SX_MFMA(acc[i][j], FW[i], FX[j])
// The 16 fragment reads of a k-step, dealt over the 8 row blocks of the phase before it in the order
// the next phase needs them: W block 0 and all X blocks first, then W blocks 1..7.
#define SX_READS_A(STG_, FX, FW, KC, r)                                                                        \
  if (r == 0) { SX_READW(STG_, FW, 0, KC) SX_READX(STG_, FX, 0, KC) }                                          \
  if (r == 1) { SX_READX(STG_, FX, 2, KC) SX_READX(STG_, FX, 3, KC) }                                          \
  if (r == 2) { SX_READX(STG_, FX, 5, KC) SX_READX(STG_, FX, 6, KC) }                                          \
  if (r == 3) { SX_READW(STG_, FW, 1, KC) }                                                                    \
  if (r == 4) { SX_READW(STG_, FW, 3, KC) }                                                                    \
  if (r == 5) { SX_READW(STG_, FW, 5, KC) }                                                                    \
  if (r == 6) { SX_READW(STG_, FW, 7, KC) }
#define SX_READS_B(STG_, FX, FW, KC, r)                                                                        \
  if (r == 0) { SX_READX(STG_, FX, 1, KC) }                                                                    \
  if (r == 1) { SX_READX(STG_, FX, 4, KC) }                                                                    \
  if (r == 2) { SX_READX(STG_, FX, 7, KC) }                                                                    \
  if (r == 3) { SX_READW(STG_, FW, 2, KC) }                                                                    \
  if (r == 4) { SX_READW(STG_, FW, 4, KC) }                                                                    \
  if (r == 5) { SX_READW(STG_, FW, 6, KC) }
// One slab from stage STG_ (its k-step 0 already in fx0/fw0):
//   phase 1: the 64 MFMAs of k-step 0, with the fragment reads of k-step 1 between them;
//   barrier: everybody has read all of STG_, and everybody's copies of the next slab (stage STG_N) are in;
//   phase 2: the 64 MFMAs of k-step 1, with the copies of the slab after next (K offset SO_) into STG_
//   and the reads of the next slab's k-step 0 between them.  The copies go out early in the phase
//   (kCopyRows row blocks): they have until the next barrier, a slab's worth of MFMAs away.
#define SX_SLAB(STG_, STG_N, SO_)                                                                              \
  _Pragma("unroll") for (int r = 0; r < 8; ++r) {                                                             \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) SX_MFMA(acc[r][j], fw0[r], fx0[j])                           \
    SX_READS_A(STG_, fx1, fw1, kc1, r)                                                                         \
    _Pragma("unroll") for (int j = 4; j < 8; ++j) SX_MFMA(acc[r][j], fw0[r], fx0[j])                           \
    SX_READS_B(STG_, fx1, fw1, kc1, r)                                                                         \
  }                                                                                                            \
  SX_WAIT_BARRIER(PF ? kWaitVm2 : kWaitVm0)                                                                      \
  _Pragma("unroll") for (int r = 0; r < 8; ++r) {                                                             \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) SX_MFMA(acc[r][j], fw1[r], fx1[j])                           \
    if (r < kCopyRows) {                                                                                       \
      _Pragma("unroll") for (int c = 0; c < 8 / kCopyRows; ++c) SX_COPY1(STG_, SO_, 0, r * (8 / kCopyRows) + c) \
    }                                                                                                          \
    SX_READS_A(STG_N, fx0, fw0, kc0, r)                                                                        \
    _Pragma("unroll") for (int j = 4; j < 8; ++j) SX_MFMA(acc[r][j], fw1[r], fx1[j])                           \
    if (r < kCopyRows) {                                                                                       \
      _Pragma("unroll") for (int c = 0; c < 8 / kCopyRows; ++c) SX_COPY1(STG_, SO_, 1, r * (8 / kCopyRows) + c) \
    }                                                                                                          \
    SX_READS_B(STG_N, fx0, fw0, kc0, r)                                                                        \
  }                                                                                                            \
  if (PF) { /* youngest in the queue: the barrier's wait lets these two loads stay in flight */                \
    asm volatile("" ::"v"(pfx), "v"(pfw) : "memory"); /* and they stay behind the copies issued above */       \
    const int pso = min((SO_) + kPfDist * (BK * 2), last * (BK * 2));                 \
    pfx = __builtin_amdgcn_raw_buffer_load_b32(xres, pfxoff, pso, 0);                                          \
    pfw = __builtin_amdgcn_raw_buffer_load_b32(pfwres, pfwoff, pso, 0);                                        \
  }
  constexpr int kCopyRows = 8;

  // The loop body is branch-free: past the end of K it copies the last slab again, into a stage nobody
  // reads any more, and reads fragments nobody uses.
  const int nb_all = a.K / BK;
  const int first = kpart * nb_all / ksplit;                      // slabs of this workgroup: [first, first + NB)
  const int NB = (kpart + 1) * nb_all / ksplit - first, last = first + NB - 1;
  SX_COPY(stA, first)
  SX_COPY(stB, min(first + 1, last))
  if (PF) {
    // The in-loop barriers let the two youngest operations stay in flight, taking them to be a slab's two
    // prefetch loads.  Before the first slab has issued any, the two youngest would be the last copies into the
    // second stage (X and W rows 56..63 of each wave's share), read by the first slab's second phase: so the
    // prologue issues a pair of prefetch loads of its own.  (Without them those rows were occasionally stale.)
    asm volatile("" ::: "memory");
    const int pso = min(first + 2, last) * (BK * 2);
    pfx = __builtin_amdgcn_raw_buffer_load_b32(xres, pfxoff, pso, 0);
    pfw = __builtin_amdgcn_raw_buffer_load_b32(pfwres, pfwoff, pso, 0);
  }
  SX_WAIT_BARRIER(PF ? kWaitVm18 : kWaitVm16)
  _Pragma("unroll") for (int i = 0; i < 8; ++i) { SX_READW(stA, fw0, i, kc0) SX_READX(stA, fx0, i, kc0) }
  int s = 0;
  for (; s + 2 <= NB; s += 2) {
    SX_SLAB(stA, stB, min(first + s + 2, last) * (BK * 2))
    SX_SLAB(stB, stA, min(first + s + 3, last) * (BK * 2))
  }
  if (s < NB) {  // one slab left, in stage A
    SX_SLAB(stA, stB, last * (BK * 2))
  }
  // Copies past the end of K may still be in flight: they must land before this workgroup's LDS is released.
  __builtin_amdgcn_s_waitcnt(kWaitVm0);
  asm volatile("" ::"v"(pfx), "v"(pfw));
  // the matrix pipe's last results must be written back before ordinary instructions read them; the
  // compiler cannot see the hand-written MFMAs, so the wait states are spelled out
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#undef SX_COPY1
#undef SX_COPY
#undef SX_READW
#undef SX_READX
#undef SX_MFMA
#undef SX_MMA
#undef SX_SLAB
#undef SX_READS_A
#undef SX_READS_B

  // ---- K-split tail: the partial sums meet in memory, the last workgroup to arrive adds them up ---------
  // Every part writes its accumulators (register layout, 1 KB per wave and block: coalesced) and
  // bumps the tile's counter; whoever finds the others' bumps already there reads all parts back in
  // part order, so the sum does not depend on who came last.  Nobody waits for anybody.
  // Coherence without flushing caches: the partial sums are stored and loaded with device scope
  // (sc1: the stores write through the XCD's L2, the loads do not trust it), the stores are
  // complete (vmcnt 0) before the counter's device-scope atomic is issued, and the loads are issued
  // after it has returned.  A release/acquire fence pair would do the same by writing back and
  // invalidating the whole L2 under the feet of the workgroups still computing (measured: +40 us).
  if (ksplit > 1) {
    constexpr int kScopeDevice = 16;  // cache-policy bit sc1
    __shared__ int s_last;
    const int tail_tile = lin - a.full_tiles;
    const __amdgpu_buffer_rsrc_t pres = make_rsrc(a.part);
    const unsigned mine = (unsigned)(((tail_tile * ksplit + kpart) * 4 + wave) * (64 * 256) + lane * 4) * 4u;  // bytes
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[i][j]), pres, mine + (i * 8 + j) * 1024, 0,
                                               kScopeDevice);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __syncthreads();
    if (tid == 0) {
      const int before = atomicAdd(a.part_cnt + tail_tile, 1);
      s_last = before == ksplit - 1;
      if (s_last) a.part_cnt[tail_tile] = 0;  // ready for the next launch
    }
    __syncthreads();
    if (!s_last) return;
    constexpr int kBatch = 16;
    // Read back in batches of kBatch blocks per part, all loads of a batch in flight together: one memory round
    // trip per batch and part instead of one per block (a block at a time, the 64 dependent round trips were
    // most of what the split cost).  Parts are added in part order whatever the batch size.
    const unsigned all = (unsigned)((tail_tile * ksplit * 4 + wave) * (64 * 256) + lane * 4) * 4u;
#pragma unroll
    for (int b0 = 0; b0 < 64; b0 += kBatch) {
      f32x4 sum[kBatch];
      for (int p = 0; p < ksplit; ++p) {
        f32x4 t[kBatch];
        if (p == kpart) {  // this workgroup's own part is still in its registers (the same bits it stored)
#pragma unroll
          for (int b = 0; b < kBatch; ++b) t[b] = acc[(b0 + b) >> 3][(b0 + b) & 7];
        } else {
#pragma unroll
          for (int b = 0; b < kBatch; ++b)
            t[b] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                                                 pres, all + (unsigned)p * (4u * 64 * 256 * 4) + (b0 + b) * 1024, 0,
                                                 kScopeDevice));
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b) sum[b] = p == 0 ? t[b] : sum[b] + t[b];
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b) acc[(b0 + b) >> 3][(b0 + b) & 7] = sum[b];
    }
  }

  // ---- epilogue.  acc[i][j][e]: output row 16 j + l16 of the quadrant, W row 16 i + 4 lq + e ---------
  const int mbase = tile_m * BM + wm * 128;
  const bool vec = (a.N & 3) == 0;  // then every group of 4 columns is whole and 16-byte (8-byte) aligned
  if (MODE == SX_GEMM_QKV_ROPE) {
    // The quadrant's 128 columns are one head (head_dim 128): query head, key head or value head,
    // the same for the whole wave.  Column 16 i + 4 lq + e and column + 64 (block i + 4, same lane and
    // register) are the pair the rotary embedding turns by the row's angle (Alg. 1: node at position
    // P + depth); the values are rounded to bf16 once, after the rotation.
    // The tile's 256 rows of the cos/sin table (512 bytes each) are first copied into the LDS the K loop has
    // left free -- rows 0..127 into the first stage's array, 128..255 into the second's -- and read from there:
    // loaded from memory row block by row block, every load waited behind the stores of the block before (one
    // counter covers both on this chip), 32 memory round trips per tile.  16-byte chunk c of table row r sits at
    // chunk position (c & 16) | ((c ^ r) & 15) of its 512 bytes: the 16 rows a read instruction covers fall on 16
    // bank groups.
    const int head = tile_n * 2 + wn;
    const bool is_v = head >= a.hq + a.hkv;
    unsigned short* dst = head < a.hq ? a.q : is_v ? a.v : a.k;
    const int hh = head < a.hq ? head : is_v ? head - a.hq - a.hkv : head - a.hq;
    const int nh = head < a.hq ? a.hq : a.hkv;
    if (tile_n * 2 < a.hq + a.hkv) {  // the tile holds a query or key head (same answer in all four waves)
      __syncthreads();  // every wave is past its last fragment reads of the stages
      const __amdgpu_buffer_rsrc_t cres = make_rsrc(a.cs);
#pragma unroll
      for (int t = 0; t < 32; ++t) {  // copy t of wave w: table rows 2 (16 w + t % 16) and + 1 of half t / 16
        const int r = 2 * (16 * wave + (t & 15)) + (lane >> 5);
        int m = tile_m * BM + (t >> 4) * 128 + r;
        m = m < a.M ? m : a.M - 1;
        const int pch = lane & 31, c = (pch & 16) | ((pch ^ r) & 15);
        unsigned char* stg = (t >> 4) ? stB : stA;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(cres, (lds_void_ptr)(stg + (16 * wave + (t & 15)) * 1024), 16,
                                                 (int)((unsigned)m * 512u + (unsigned)c * 16u), 0, 0, 0);
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(kWaitVm0);
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }
    if (head < a.hq + 2 * a.hkv) {
      const unsigned char* tb = wm ? stB : stA;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int m = mbase + 16 * j + l16;
        if (m >= a.M) continue;
        unsigned short* y = dst + ((size_t)m * nh + hh) * 128 + 4 * lq;
        if (is_v) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            u32x2 o;
            o[0] = pack_bf16x2(acc[i][j][0], acc[i][j][1]);
            o[1] = pack_bf16x2(acc[i][j][2], acc[i][j][3]);
            *reinterpret_cast<u32x2*>(y + 16 * i) = o;
          }
        } else {
          const int r = 16 * j + l16;
          const unsigned char* trow = tb + r * 512;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            // (cos, sin) of pairs 16 i + 4 lq + 0..3: chunks 8 i + 2 lq and + 1 of the row
            const int c0 = 8 * i + 2 * lq;
            const f32x4 c01 = *reinterpret_cast<const f32x4*>(trow + (((c0 & 16) | ((c0 ^ r) & 15)) << 4));
            const f32x4 c23 = *reinterpret_cast<const f32x4*>(trow + ((((c0 + 1) & 16) | (((c0 + 1) ^ r) & 15)) << 4));
            const float cs_[4] = {c01[0], c01[2], c23[0], c23[2]}, sn_[4] = {c01[1], c01[3], c23[1], c23[3]};
            float lo[4], hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float x0 = acc[i][j][e], x1 = acc[i + 4][j][e];
              lo[e] = x0 * cs_[e] - x1 * sn_[e];
              hi[e] = x0 * sn_[e] + x1 * cs_[e];
            }
            u32x2 o;
            o[0] = pack_bf16x2(lo[0], lo[1]);
            o[1] = pack_bf16x2(lo[2], lo[3]);
            *reinterpret_cast<u32x2*>(y + 16 * i) = o;
            o[0] = pack_bf16x2(hi[0], hi[1]);
            o[1] = pack_bf16x2(hi[2], hi[3]);
            *reinterpret_cast<u32x2*>(y + 64 + 16 * i) = o;
          }
        }
      }
    }
  } else if (MODE == SX_GEMM_SWIGLU && vec && tile_m * BM + BM <= a.M && tile_n * (BN / 2) + BN / 2 <= a.N) {
    // a whole tile: no edge tests between the stores
    unsigned short* Yb = static_cast<unsigned short*>(a.Y) + (size_t)(mbase + l16) * a.N + (tile_n * (BN / 2) + wn * 64 + 4 * lq);
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int ii = 0; ii < 4; ++ii) {
        float h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = silu_mul_bf16_bound(acc[2 * ii][j][e], acc[2 * ii + 1][j][e]);
        u32x2 v;
        v[0] = pack_bf16x2(h[0], h[1]);
        v[1] = pack_bf16x2(h[2], h[3]);
        *reinterpret_cast<u32x2*>(Yb + (size_t)(16 * j) * a.N + 16 * ii) = v;
      }
  } else if (MODE == SX_GEMM_SWIGLU) {
    unsigned short* Y = static_cast<unsigned short*>(a.Y);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int m = mbase + 16 * j + l16;
#pragma unroll
      for (int ii = 0; ii < 4; ++ii) {
        const int f = tile_n * (BN / 2) + wn * 64 + ii * 16 + 4 * lq;
        if (m >= a.M || f >= a.N) continue;
        unsigned short h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float g = acc[2 * ii][j][e], u = acc[2 * ii + 1][j][e];
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
    }
  } else if (vec && tile_m * BM + BM <= a.M && tile_n * BN + BN <= a.N) {
    // A whole tile: no edge tests, and the residual comes in 16 loads at a time (two row blocks) before the first
    // add -- a load, an add and a store per block, each waiting for its own load, made the epilogue 64 memory
    // round trips long.
    float* Yb = static_cast<float*>(a.Y) + (size_t)(mbase + l16) * a.N + (tile_n * BN + wn * 128 + 4 * lq);
#pragma unroll
    for (int j0 = 0; j0 < 8; j0 += 2) {
      f32x4 r[2][8];
      if (MODE == SX_GEMM_RESIDUAL) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int i = 0; i < 8; ++i)
            r[jj][i] = *reinterpret_cast<const f32x4*>(Yb + (size_t)(16 * (j0 + jj)) * a.N + 16 * i);
      }
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          f32x4 v = acc[i][j0 + jj];
          if (MODE == SX_GEMM_RESIDUAL) v += r[jj][i];
          *reinterpret_cast<f32x4*>(Yb + (size_t)(16 * (j0 + jj)) * a.N + 16 * i) = v;
        }
    }
  } else {
    float* Y = static_cast<float*>(a.Y);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int m = mbase + 16 * j + l16;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int n = tile_n * BN + wn * 128 + 16 * i + 4 * lq;
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


// Decides which tiles are cut along K, given memory for the partial sums.  More tiles than compute units with a
// remainder that would fill at most half of the chip for a whole round: the remainder tiles, up to 4 ways (as many
// as it takes to give every compute unit a part).  Fewer tiles than half the compute units: all of them.  Parts
// are at least 8 slabs long.  (Batches of at most 128 rows never come here: for them a partial tile of 256 KB
// outweighs the weights a part streams, and they take the narrow-tile kernel instead.)
constexpr float kSplitPerPartSlabs = 4.5f;
constexpr int kSplitMaxWays = 16;
void plan_split(GemmArgs& a, void* split_ws, size_t split_ws_bytes) {
  a.split = 1;
  a.part = nullptr;
  a.part_cnt = nullptr;
  a.full_tiles = a.tail_items = a.full_per_xcd = a.tail_per_xcd = 0;
  const int cus = sx_compute_units(), tiles = a.tilesM * a.tilesN, nb = a.K / BK;
  if (!split_ws) return;
  if (2 * tiles <= cus) {
    // Fewer tiles than half the compute units (trees of a few hundred nodes, narrow models): every tile is cut, as
    // many ways as keeps all parts in one round and pays.  Cost of a cut in slab times: each part walks nb / s
    // slabs, and every further way costs about 4.5 (a partial tile written, and read back by the last arriver) --
    // fitted to sweeps at the 70B and 7B layer shapes for 256 to 1024 rows, where it picks the fastest or
    // second-fastest cut (e.g. 8192 x 8192 at 256 rows: 152 us uncut, 74 us cut 5 ways, 82 us cut 8 ways).
    int best = 1;
    float best_cost = (float)nb + kSplitPerPartSlabs;
    for (int s2 = 2; s2 * tiles <= cus && s2 <= kSplitMaxWays && nb / s2 >= 8; ++s2) {
      const float cost = (float)nb / s2 + kSplitPerPartSlabs * s2;
      if (cost < best_cost) {
        best_cost = cost;
        best = s2;
      }
    }
    if (best < 2 || tiles > 256) return;
    if (split_ws_bytes < 1024 + (size_t)tiles * best * BM * BN * sizeof(float)) return;
    a.split = best;
    a.full_tiles = 0;
    a.tail_items = tiles * best;
    a.full_per_xcd = 0;
    a.tail_per_xcd = (a.tail_items + 7) / 8;
    a.part_cnt = static_cast<int*>(split_ws);
    a.part = reinterpret_cast<float*>(static_cast<char*>(split_ws) + 1024);
    return;
  }
  if (tiles <= cus) return;
  const int rest = tiles % cus;
  if (rest == 0 || 2 * rest > cus) return;
  int split = cus / rest;
  if (split > 4) split = 4;  // measured at the 70B QKV shape: 4 ways 289 us, 3 ways 295, 2 ways 313 (uncut: 372)
  while (split > 1 && nb / split < 8) --split;
  if (split < 2 || rest > 256) return;
  if (split_ws_bytes < 1024 + (size_t)rest * split * BM * BN * sizeof(float)) return;
  a.split = split;
  a.full_tiles = tiles - rest;
  a.tail_items = rest * split;
  a.full_per_xcd = (a.full_tiles + 7) / 8;
  a.tail_per_xcd = (a.tail_items + 7) / 8;
  a.part_cnt = static_cast<int*>(split_ws);
  a.part = reinterpret_cast<float*>(static_cast<char*>(split_ws) + 1024);
}

template <int MODE>
int launch(const GemmArgs& a, hipStream_t st) {
  const int grid = a.split > 1 ? 8 * (a.full_per_xcd + a.tail_per_xcd) : 8 * a.chunk;
  if (a.tilesM == 8 && a.tilesN % 4 == 0)
    gemm_bf16_kernel<MODE, true><<<grid, kThreads, 0, st>>>(a);
  else
    gemm_bf16_kernel<MODE, false><<<grid, kThreads, 0, st>>>(a);
  SX_LAUNCH_CHECK();
  return SX_OK;
}

}  // namespace

int sx_launch_gemm_bf16(const void* X, const void* W0, const void* W1, const void* W2, int n0, int n1, int n2,
                        void* Y, int M, int K, int mode, void* split_ws, size_t split_ws_bytes, hipStream_t st) {
  if (M < 1 || K < BK || K % BK != 0 || n0 < 1 || n1 < 0 || n2 < 0) return SX_ERR_SHAPE;
  if (!sx_operand_fits_u32(M, 2ll * K) || !sx_operand_fits_u32(n0, 2ll * K) || !sx_operand_fits_u32(n1, 2ll * K) ||
      !sx_operand_fits_u32(n2, 2ll * K))
    return SX_ERR_SHAPE;
  if (M <= 128)  // weight-streaming regime: narrow tiles
    return sx_launch_gemm_skinny_bf16(X, W0, W1, W2, n0, n1, n2, Y, M, K, mode, split_ws, split_ws_bytes, st);
  // a 16-row copy group must not straddle two stacked weight matrices
  if (mode != SX_GEMM_SWIGLU && ((n1 > 0 && n0 % 16 != 0) || (n2 > 0 && n1 % 16 != 0))) return SX_ERR_SHAPE;
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
  plan_split(a, split_ws, split_ws_bytes);
  switch (mode) {
    case SX_GEMM_STORE: return launch<SX_GEMM_STORE>(a, st);
    case SX_GEMM_RESIDUAL: return launch<SX_GEMM_RESIDUAL>(a, st);
    case SX_GEMM_SWIGLU: return launch<SX_GEMM_SWIGLU>(a, st);
  }
  return SX_ERR_SHAPE;
}

// 1 KB of counters (at most 256 split tiles, zero before the first launch) and one partial tile per compute unit
size_t sx_gemm_split_workspace() { return 1024 + (size_t)sx_compute_units() * BM * BN * sizeof(float); }

int sx_launch_gemm_qkv_rope_bf16(const void* X, const void* Wq, const void* Wk, const void* Wv, int hq, int hkv,
                                 const float2* rope_cs, void* q, void* k, void* v, int M, int K, void* split_ws,
                                 size_t split_ws_bytes, hipStream_t st) {
  if (M < 1 || K < BK || K % BK != 0 || hq < 1 || hkv < 1) return SX_ERR_SHAPE;
  if (!sx_operand_fits_u32(M, 2ll * K) || !sx_operand_fits_u32(128ll * hq, 2ll * K) ||
      !sx_operand_fits_u32(128ll * hkv, 2ll * K) || !sx_operand_fits_u32(M, 512))  // the table: 512 bytes per row
    return SX_ERR_SHAPE;
  GemmArgs a;
  a.X = static_cast<const unsigned short*>(X);
  a.W0 = static_cast<const unsigned short*>(Wq);
  a.W1 = static_cast<const unsigned short*>(Wk);
  a.W2 = static_cast<const unsigned short*>(Wv);
  a.n0 = hq * 128;
  a.n1 = a.n2 = hkv * 128;
  a.Y = nullptr;
  a.M = M;
  a.K = K;
  a.N = a.n0 + a.n1 + a.n2;
  a.tilesM = (M + BM - 1) / BM;
  a.tilesN = (a.N + BN - 1) / BN;
  a.chunk = (a.tilesM * a.tilesN + 7) / 8;
  a.cs = rope_cs;
  a.q = static_cast<unsigned short*>(q);
  a.k = static_cast<unsigned short*>(k);
  a.v = static_cast<unsigned short*>(v);
  a.hq = hq;
  a.hkv = hkv;
  plan_split(a, split_ws, split_ws_bytes);
  return launch<SX_GEMM_QKV_ROPE>(a, st);
}

extern "C" size_t sx_gemm_bf16_workspace(void) { return sx_gemm_split_workspace(); }

extern "C" int sx_gemm_bf16_ws(const void* X, const void* W, const void* W2, void* Y, int32_t M, int32_t N, int32_t K,
                               int32_t mode, void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !W || !Y || (mode == SX_GEMM_SWIGLU && !W2)) return SX_ERR_NULL;
  if (mode < 0 || mode > 2 || N < 1) return SX_ERR_SHAPE;
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255)) return SX_ERR_WORKSPACE;
  if (mode == SX_GEMM_SWIGLU)
    return sx_launch_gemm_bf16(X, W, W2, nullptr, N, N, 0, Y, M, K, mode, workspace, workspace_bytes, (hipStream_t)stream);
  return sx_launch_gemm_bf16(X, W, nullptr, nullptr, N, 0, 0, Y, M, K, mode, workspace, workspace_bytes,
                             (hipStream_t)stream);
}

extern "C" int sx_gemm_bf16(const void* X, const void* W, const void* W2, void* Y, int32_t M, int32_t N, int32_t K,
                            int32_t mode, void* stream) {
  return sx_gemm_bf16_ws(X, W, W2, Y, M, N, K, mode, nullptr, 0, stream);
}
