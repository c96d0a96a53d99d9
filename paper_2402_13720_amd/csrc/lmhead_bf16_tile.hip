// bf16 LM head fused with the vocabulary arg-max, large-tile (MFMA-bound) variant for gfx950.
//
// logits^T[v, r] = sum_k W[v, k] * hidden[r, k]  (Eq. (2): next-token scores of every block row)
// for R = B*T in the hundreds (batched verification): arithmetic intensity ~R flop/byte
// exceeds the machine balance, so the product is bound by the matrix cores and organised as
// a classic LDS-tiled GEMM:
//
//   * workgroup tile 256 vocabulary rows x 256 hidden rows, k-tiles of 64; 8 waves in a 4x2
//     grid, each owning 64 x 128 = 2x4 accumulator tiles of v_mfma_f32_32x32x16_bf16 (128
//     accumulator registers per lane), so that two waves share a SIMD and one wave's LDS
//     reads and waits hide behind the other's MFMAs; 6 operand fragments feed 8 MFMAs per
//     16-wide k step;
//   * global -> registers -> LDS (XOR-swizzled 128-byte rows, conflict-free fragment reads),
//     two LDS buffers: the k-tile after next is in flight in registers while the next one is
//     already in LDS; one barrier per k-tile;
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
constexpr int kThreads = 512;
constexpr int kMT = 2, kNT = 4;                          // accumulator tiles per wave
constexpr int kBestOff = 2 * kBufBytes;                  // [4 wave rows][256] (value, id)
constexpr int kLdsBytes = kBestOff + 4 * kBN * 8;

struct TileArgs {
  const __bf16* hidden;
  const __bf16* w;
  float2* part;     // [nslab][R]
  int R, Hd, V;
  int nslab, nrtile;
  int tiled;        // W given as contiguous [V/128][k-tile][128][64] tiles
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// 16-byte slot of chunk c (0..7) of row `row` in a tile with 128-byte rows (see lmhead_bf16.hip).
__device__ __forceinline__ int tile_slot(int row, int c) { return row * 8 + (c ^ ((row >> 1) & 7)); }

__global__ __launch_bounds__(kThreads) void lmhead_bf16_tile_kernel(TileArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int col = lane & 31, half = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;             // wave's 64 x 128 block: vocabulary rows 64*wm.., hidden rows 128*wn..

  // workgroup id -> (slab, row tile): the row tiles of one slab sit 8 ids apart
  const int per = 8 * a.nrtile;
  const int blk = blockIdx.x / per, rem = blockIdx.x - blk * per;
  const int rt = rem >> 3;
  const int slab = blk * 8 + (rem & 7);
  if (slab >= a.nslab) return;
  const int v0 = slab * kBM, r0 = rt * kBN;
  const int R = a.R, Hd = a.Hd, V = a.V;

  // staging: thread (lr = tid/8, lc = tid%8) moves chunk lc of rows 64*p + lr, p = 0..3, of both tiles
  const int lr = tid >> 3, lc = tid & 7;
  const __bf16* wp[4];
  const __bf16* hp[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int row = 64 * p + lr;                       // row of the 256-row tile = two 128-row tiled slabs
    const int slab128 = min(2 * slab + (row >> 7), (V + 127) / 128 - 1);
    wp[p] = a.tiled ? a.w + (static_cast<size_t>(slab128) * (Hd / 64) * 128 + (row & 127)) * 64 + 8 * lc
                    : a.w + static_cast<size_t>(min(v0 + row, V - 1)) * Hd + 8 * lc;   // rows past V: duplicate, masked later
    hp[p] = a.hidden + static_cast<size_t>(min(r0 + 64 * p + lr, R - 1)) * Hd + 8 * lc;
  }
  const size_t wstep = a.tiled ? 128 * 64 : kBK;
  u32x4 wreg[4], hreg[4];
#define OURO_TILE_GLOAD(KT)                                                                                    \
  {                                                                                                            \
    const size_t koff = static_cast<size_t>(KT) * kBK;                                                         \
    _Pragma("unroll") for (int p = 0; p < 4; ++p)                                                              \
        wreg[p] = *reinterpret_cast<const u32x4*>(wp[p] + static_cast<size_t>(KT) * wstep);                    \
    _Pragma("unroll") for (int p = 0; p < 4; ++p) hreg[p] = *reinterpret_cast<const u32x4*>(hp[p] + koff);     \
  }
#define OURO_TILE_LDS_STORE(BUF)                                                                               \
  {                                                                                                            \
    unsigned char* wl_ = lds + (BUF) * kBufBytes;                                                              \
    unsigned char* hl_ = wl_ + kTileBytes;                                                                     \
    _Pragma("unroll") for (int p = 0; p < 4; ++p)                                                              \
        *reinterpret_cast<u32x4*>(wl_ + tile_slot(64 * p + lr, lc) * 16) = wreg[p];                            \
    _Pragma("unroll") for (int p = 0; p < 4; ++p)                                                              \
        *reinterpret_cast<u32x4*>(hl_ + tile_slot(64 * p + lr, lc) * 16) = hreg[p];                            \
  }

  f32x16 acc[kMT][kNT];
#pragma unroll
  for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;

  const int nkt = Hd / kBK;
  OURO_TILE_GLOAD(0)
  OURO_TILE_LDS_STORE(0)
  if (nkt > 1) OURO_TILE_GLOAD(1)
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    // k-tile kt+1 (in registers since the previous iteration) -> the other LDS buffer, whose readers
    // all passed the barrier that ended the previous iteration; then put k-tile kt+2 in flight.
    // (Spreading this staging work over the four k steps was measured slower.)
    if (kt + 1 < nkt) OURO_TILE_LDS_STORE(cur ^ 1)
    if (kt + 2 < nkt) OURO_TILE_GLOAD(kt + 2)

    const unsigned char* wl = lds + cur * kBufBytes + (wm * 64) * 128;
    const unsigned char* hl = lds + cur * kBufBytes + kTileBytes + (wn * 128) * 128;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 af[kMT], bf[kNT];
#pragma unroll
      for (int mt = 0; mt < kMT; ++mt)
        af[mt] = *reinterpret_cast<const bf16x8*>(wl + tile_slot(32 * mt + col, 2 * s + half) * 16);
#pragma unroll
      for (int nt = 0; nt < kNT; ++nt)
        bf[nt] = *reinterpret_cast<const bf16x8*>(hl + tile_slot(32 * nt + col, 2 * s + half) * 16);
#pragma unroll
      for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bf[nt], acc[mt][nt], 0, 0, 0);
    }
    __syncthreads();
  }
#undef OURO_TILE_GLOAD
#undef OURO_TILE_LDS_STORE

  // ---- arg-max epilogue.  Lane (col, half) of wave (wm, wn) holds, for hidden row r0 + 128*wn + 32*nt + col,
  // the logits of vocabulary rows v0 + 64*wm + 32*mt + 8*(i/4) + 4*half + i%4.
  float* bestv = reinterpret_cast<float*>(lds + kBestOff);
  int* besti = reinterpret_cast<int*>(lds + kBestOff + 4 * kBN * 4);
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int v = v0 + 64 * wm + 32 * mt + 8 * (i >> 2) + 4 * half + (i & 3);
        const float x = v < V ? acc[mt][nt][i] : -INFINITY;
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
#pragma unroll
    for (int q = 1; q < 4; ++q) {                           // the four wave rows, ascending vocabulary
      const float v2 = bestv[q * kBN + rl];
      const int i2 = besti[q * kBN + rl];
      if (better(v2, i2, bv, bi)) { bv = v2; bi = i2; }
    }
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
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_bf16_tile_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return hip_failed(e);
    attr_set = true;
  }
  const unsigned grid = static_cast<unsigned>((plan.nslab + 7) / 8) * 8u * plan.nrtile;
  hipLaunchKernelGGL(lmhead_bf16_tile_kernel, dim3(grid), dim3(kThreads), kLdsBytes, stream, a);
  return check_launch();
}

}  // namespace ouro
