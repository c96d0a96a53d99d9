// bf16 LM head fused with the vocabulary arg-max, large-tile (MFMA-bound) variant for gfx950.
//
// logits^T[v, r] = sum_k W[v, k] * hidden[r, k]  (Eq. (2): next-token scores of every block row)
// for R = B*T in the hundreds (batched verification): arithmetic intensity ~R flop/byte
// exceeds the machine balance, so the product is bound by the matrix cores and organised as
// a classic LDS-tiled GEMM:
//
//   * workgroup tile 256 vocabulary rows x 256 hidden rows, k-tiles of 64; 4 waves in a 2x2 grid, one per
//     SIMD, each owning 128 x 128 = 4x4 accumulator tiles of v_mfma_f32_32x32x16_bf16 (all 256 accumulator
//     registers of the lane), so that 8 operand fragments feed 16 MFMAs per 16-wide k step;
//   * with one wave per SIMD nothing else hides latency, so the loop is software-pipelined by hand and the
//     order is pinned with scheduling barriers: the fragments of k step s+1 are read from LDS between the
//     MFMAs of step s (two fragment register sets), and the staging work (registers -> the LDS buffer that
//     is not being read, each staging register re-armed at once from global memory) is spread evenly over
//     the four k steps of a k-tile, four registers each; one barrier per k-tile, before step 3 prefetches
//     the first fragments of the next k-tile;
//   * LDS tiles have 128-byte rows with XOR-swizzled 16-byte chunks (conflict-free fragment reads and
//     staging writes);
//   * epilogue: arg-max lane -> wave -> workgroup with the total order (larger value, then
//     smaller id); one (value, id) pair per (vocabulary slab, row) goes to the workspace and
//     the cross-slab kernel finishes.  The logits never reach memory.
//   * workgroup ids are arranged so that the workgroups that stream the same W slab (the
//     R/256 row tiles) are congruent modulo 8, i.e. run on one XCD and share its L2: W comes
//     from HBM once.
#include <math.h>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kTileBytes = 256 * 128;                    // one operand tile: 256 rows x 64 bf16
constexpr int kBufBytes = 2 * kTileBytes;                // W tile + hidden tile
constexpr int kThreads = 256;
constexpr int kMT = 4, kNT = 4;                          // accumulator tiles per wave
constexpr int kLdsBytes = 2 * kBufBytes;                 // 128 KB; the arg-max exchange reuses buffer 0

struct TileArgs {
  const __bf16* hidden;
  const __bf16* w;
  float2* part;     // [nslab][R]
  int R, Hd, V;
  int nslab, nrtile;
  int tiled;        // W given as contiguous [V/128][k-tile][128][64] tiles
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ __launch_bounds__(kThreads) void lmhead_bf16_tile_kernel(TileArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int col = lane & 31, half = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;             // wave's 128 x 128 block: vocabulary rows 128*wm.., hidden rows 128*wn..

  // workgroup id -> (slab, row tile): the row tiles of one slab sit 8 ids apart
  const int per = 8 * a.nrtile;
  const int blk = blockIdx.x / per, rem = blockIdx.x - blk * per;
  const int rt = rem >> 3;
  const int slab = blk * 8 + (rem & 7);
  if (slab >= a.nslab) return;
  const int v0 = slab * kBM, r0 = rt * kBN;
  const int R = a.R, Hd = a.Hd, V = a.V;

  // ---- staging: thread (lr = tid/8, lc = tid%8) moves 16-byte chunk lc of rows 32*p + lr, p = 0..7, of both
  // tiles.  Addresses = workgroup-uniform base + per-thread 32-bit byte offset + uniform k-tile step.
  const int lr = tid >> 3, lc = tid & 7;
  const unsigned char* wbase;
  const unsigned char* hbase = reinterpret_cast<const unsigned char*>(a.hidden);
  unsigned woff[8], hoff[8];
  unsigned wstep, w_second = 0;
  if (a.tiled) {
    const int n128 = (V + 127) / 128;
    const size_t slab_bytes = static_cast<size_t>(Hd / 64) * 128 * 128;       // one 128-row slab, all k-tiles
    wbase = reinterpret_cast<const unsigned char*>(a.w) + static_cast<size_t>(2 * slab) * slab_bytes;
    w_second = (2 * slab + 1 < n128) ? static_cast<unsigned>(slab_bytes) : 0u;   // no second slab: duplicate, masked later
#pragma unroll
    for (int p = 0; p < 8; ++p) woff[p] = (p >= 4 ? w_second : 0u) + static_cast<unsigned>(((32 * p + lr) & 127) * 128 + 16 * lc);
    wstep = 128 * 128;
  } else {
    wbase = reinterpret_cast<const unsigned char*>(a.w) + static_cast<size_t>(v0) * Hd * 2;
#pragma unroll
    for (int p = 0; p < 8; ++p)                        // rows past V: duplicate of the last row, masked later
      woff[p] = static_cast<unsigned>(min(32 * p + lr, V - 1 - v0)) * static_cast<unsigned>(Hd * 2) + 16 * lc;
    wstep = kBK * 2;
  }
  hbase += static_cast<size_t>(r0) * Hd * 2;
#pragma unroll
  for (int p = 0; p < 8; ++p) hoff[p] = static_cast<unsigned>(min(32 * p + lr, R - 1 - r0)) * static_cast<unsigned>(Hd * 2) + 16 * lc;

  // LDS tiles: 128-byte rows, the 16-byte chunk index XORed with (row/2)%8 (conflict-free fragment reads
  // and staging writes).  Writer slot of (row 32p + lr, chunk lc); reader slot of (row 32t + col, chunk 2s + half).
  const unsigned wr0 = static_cast<unsigned>(lr * 128 + ((lc ^ ((lr >> 1) & 7)) * 16));
  unsigned rd[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) rd[s] = static_cast<unsigned>(col * 128 + (((2 * s + half) ^ ((col >> 1) & 7)) * 16));
  const unsigned wave_w = static_cast<unsigned>(wm * 128 * 128);
  const unsigned wave_h = static_cast<unsigned>(kTileBytes + wn * 128 * 128);

  u32x4 wreg[8], hreg[8];
  bf16x8 fa[2][kMT], fb[2][kNT];
  f32x16 acc[kMT][kNT];
#pragma unroll
  for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;

// (W with the non-temporal hint: the two row tiles that share a W line run side by side on one XCD, so the hint costs this
// kernel nothing, and the 262 MB it would otherwise leave in L2 and in the memory-side cache cost the kernel after it
// 8 us: the batched attention runs 186 us behind this kernel with the hint, 194 us without)
#define OURO_GLOAD_W(P, KT) wreg[P] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wbase + static_cast<size_t>(KT) * wstep + woff[P]));
#define OURO_GLOAD_H(P, KT) hreg[P] = *reinterpret_cast<const u32x4*>(hbase + static_cast<size_t>(KT) * (kBK * 2) + hoff[P]);
#define OURO_STORE_W(P, BUF) *reinterpret_cast<u32x4*>(lds + (BUF) * kBufBytes + (P) * 4096 + wr0) = wreg[P];
#define OURO_STORE_H(P, BUF) *reinterpret_cast<u32x4*>(lds + (BUF) * kBufBytes + kTileBytes + (P) * 4096 + wr0) = hreg[P];
// fragment Q (0..3: W rows 32Q.., 4..7: hidden rows 32(Q-4)..) of k step S from buffer BUF into register set SET
#define OURO_FRAG(Q, S, BUF, SET)                                                                              \
  if ((Q) < 4)                                                                                                 \
    fa[SET][(Q) & 3] = *reinterpret_cast<const bf16x8*>(lds + (BUF) * kBufBytes + wave_w + ((Q) & 3) * 4096 + rd[S]); \
  else                                                                                                         \
    fb[SET][(Q) & 3] = *reinterpret_cast<const bf16x8*>(lds + (BUF) * kBufBytes + wave_h + ((Q) & 3) * 4096 + rd[S]);
// One 16-wide k step: 16 MFMAs on register set SET; between the first eight, the 8 fragment reads of the next k step
// (step NS of buffer NBUF, into the other register set); between the last eight, a quarter of the staging work: four
// staging registers go to LDS and each is re-armed at once from global memory.  The scheduling barriers pin this
// interleaving: one wave per SIMD, so all latency hiding is in this order.
//   STAGE 1: W rows 128.. (registers 4-7) of k-tile kt+1 -> the other buffer, re-armed with k-tile kt+2
//   STAGE 2, 3: hidden rows (registers 0-3, 4-7) of k-tile kt+1 -> the other buffer, re-armed with k-tile kt+2
//   STAGE 4 (the step after the barrier): W rows 0..127 (registers 0-3) of k-tile kt+2 -> the buffer just read out,
//            re-armed with k-tile kt+3
// so that every k step carries the same 4 LDS stores and 4 global loads: all four waves run in lock step, and with the
// staging bunched into two of the four steps their 64 loads met in the address unit in one burst that held the
// matrix instructions behind them back.
#define OURO_KSTEP(SET, NS, NBUF, STAGE)                                                                       \
  _Pragma("unroll") for (int j = 0; j < 16; ++j) {                                                             \
    acc[j >> 2][j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[SET][j >> 2], fb[SET][j & 3], acc[j >> 2][j & 3], 0, 0, 0); \
    if (j < 8) {                                                                                               \
      const int q_ = j == 0 ? 0 : j < 5 ? j + 3 : j - 4;   /* order: W0, H0..H3, W1..W3 */                     \
      OURO_FRAG(q_, NS, NBUF, (SET) ^ 1)                                                                       \
    } else if ((j & 1) == 0) {                                                                                 \
      const int p_ = (j - 8) >> 1;                                                                             \
      if ((STAGE) == 1) { OURO_STORE_W(4 + p_, cur ^ 1) OURO_GLOAD_W(4 + p_, ktl) }                            \
      if ((STAGE) == 2) { OURO_STORE_H(p_, cur ^ 1) OURO_GLOAD_H(p_, ktl) }                                    \
      if ((STAGE) == 3) { OURO_STORE_H(4 + p_, cur ^ 1) OURO_GLOAD_H(4 + p_, ktl) }                            \
      if ((STAGE) == 4) { OURO_STORE_W(p_, cur) OURO_GLOAD_W(p_, ktl3) }                                       \
    }                                                                                                          \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
  }

  const int nkt = Hd / kBK;
  // prologue: k-tile 0 -> LDS buffer 0; W rows 0..127 of k-tile 1 -> buffer 1; registers: W 0-3 <- k-tile 2, W 4-7 and
  // the hidden rows <- k-tile 1; first fragments -> register set 0.  (The last loads are issued in the order in which
  // the loop re-arms them, so that its counted waits are exact from the first iteration.)
  {
    const int kt1 = min(1, nkt - 1), kt2 = min(2, nkt - 1);
    u32x4 w1[4];
#pragma unroll
    for (int p = 0; p < 8; ++p) { OURO_GLOAD_W(p, 0) }
#pragma unroll
    for (int p = 0; p < 8; ++p) { OURO_GLOAD_H(p, 0) }
#pragma unroll
    for (int p = 0; p < 4; ++p) w1[p] = *reinterpret_cast<const u32x4*>(wbase + static_cast<size_t>(kt1) * wstep + woff[p]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < 8; ++p) { OURO_STORE_W(p, 0) }
#pragma unroll
    for (int p = 0; p < 8; ++p) { OURO_STORE_H(p, 0) }
#pragma unroll
    for (int p = 4; p < 8; ++p) { OURO_GLOAD_W(p, kt1) }
#pragma unroll
    for (int p = 0; p < 8; ++p) { OURO_GLOAD_H(p, kt1) }
#pragma unroll
    for (int p = 0; p < 4; ++p) { OURO_GLOAD_W(p, kt2) }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < 4; ++p) *reinterpret_cast<u32x4*>(lds + kBufBytes + p * 4096 + wr0) = w1[p];
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 8; ++q) { OURO_FRAG(q, 0, 0, 0) }

  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    const int ktl = min(kt + 2, nkt - 1);     // past the end: a harmless reload of the last k-tile
    const int ktl3 = min(kt + 3, nkt - 1);
    OURO_KSTEP(0, 1, cur, 1)
    OURO_KSTEP(1, 2, cur, 2)
    OURO_KSTEP(0, 3, cur, 3)
    // Every wave has read the last fragments of buffer cur before this barrier (they are in its registers), and has
    // written its share of k-tile kt+1 to buffer cur^1: after it, cur^1 is complete and cur may be overwritten.
    __syncthreads();
    OURO_KSTEP(1, 0, cur ^ 1, 4)
  }
#undef OURO_GLOAD_W
#undef OURO_GLOAD_H
#undef OURO_STORE_W
#undef OURO_STORE_H
#undef OURO_FRAG
#undef OURO_KSTEP

  // ---- arg-max epilogue.  Lane (col, half) of wave (wm, wn) holds, for hidden row r0 + 128*wn + 32*nt + col,
  // the logits of vocabulary rows v0 + 128*wm + 32*mt + 8*(i/4) + 4*half + i%4.
  __syncthreads();                                          // all fragment reads done: buffer 0 is free
  const bool full_slab = v0 + kBM <= V;                     // workgroup-uniform: no row to mask
  float* bestv = reinterpret_cast<float*>(lds);             // [2 wave rows][256]
  int* besti = reinterpret_cast<int*>(lds + 2 * kBN * 4);
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int v = v0 + 128 * wm + 32 * mt + 8 * (i >> 2) + 4 * half + (i & 3);
        const float x = (full_slab || v < V) ? acc[mt][nt][i] : -INFINITY;
        if (x > bv) { bv = x; bi = v; }                    // v ascending within the lane
      }
    const float ov = __shfl_xor(bv, 32);
    const int oi = __shfl_xor(bi, 32);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    if (half == 0) {
      bestv[wm * kBN + 128 * wn + 32 * nt + col] = bv;
      besti[wm * kBN + 128 * wn + 32 * nt + col] = bi;
    }
  }
  __syncthreads();
  if (tid < kBN && r0 + tid < R) {
    const int rl = tid;
    float bv = bestv[rl];
    int bi = besti[rl];
    const float v2 = bestv[kBN + rl];                       // the second wave row: larger vocabulary ids
    const int i2 = besti[kBN + rl];
    if (better(v2, i2, bv, bi)) { bv = v2; bi = i2; }
    a.part[static_cast<size_t>(slab) * R + r0 + rl] = make_float2(bv, __int_as_float(bi));
  }
}

}  // namespace

int launch_lmhead_bf16_tile(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream) {
  TileArgs a{};
  a.hidden = static_cast<const __bf16*>(d.hidden);
  a.w = static_cast<const __bf16*>(d.w);
  a.part = static_cast<float2*>(d.workspace);
  a.R = d.R;
  a.Hd = d.Hd;
  a.V = d.V;
  a.nslab = plan.nslab;
  a.nrtile = plan.nrtile;
  a.tiled = d.w_layout == OURO_W_TILED;
  static DeviceOnce once;
  const int ready = device_once(once, [] {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_bf16_tile_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    return e == hipSuccess ? static_cast<int>(OURO_OK) : hip_failed(e);
  });
  if (ready != OURO_OK) return ready;
  const unsigned grid = static_cast<unsigned>((plan.nslab + 7) / 8) * 8u * plan.nrtile;
  hipLaunchKernelGGL(lmhead_bf16_tile_kernel, dim3(grid), dim3(kThreads), kLdsBytes, stream, a);
  return check_launch();
}

}  // namespace ouro
