// bf16 LM head fused with the vocabulary arg-max, weight-streaming variant for gfx950.
//
// logits^T[v, r] = sum_k W[v, k] * hidden[r, k]   (Eq. (2): next-token scores of every block
// row), then arg max over v per row r, lowest id on ties.  With R = B*T <= 128 rows the
// product is bound by streaming W from HBM exactly once, so the kernel is organised around
// keeping many bytes in flight per compute unit rather than around MFMA occupancy:
//
//   * a workgroup (4 waves) owns a slab of MT*32 vocabulary rows and NT*32 hidden rows;
//   * the hidden dimension is cut into 64-wide k-tiles dealt round-robin to the 4 waves
//     (split-K inside the workgroup), so the waves never synchronise in the main loop and
//     together read 512 contiguous bytes of every W row per round;
//   * per k-tile a wave moves its W tile (MT*32 x 64) and hidden tile (NT*32 x 64) with
//     coalesced 16-byte loads into registers, then into its private XOR-swizzled LDS
//     region, and issues MT*NT v_mfma_f32_32x32x16_bf16 per 16-wide k step; the loads of
//     the wave's next k-tile are issued before the math of the current one;
//   * after the loop the 4 partial accumulator sets are summed through LDS (fixed order),
//     and the arg-max epilogue reduces lane -> wave -> workgroup; one (value, index) pair
//     per (slab, row) goes to the workspace, the logits never leave the chip;
//   * a second tiny kernel reduces the pairs over the slabs (no float atomics; the result is
//     order-independent because (larger value, then smaller index) is a total order).  A
//     single-launch variant in which the last workgroup did this reduction was measured
//     slower: store acknowledgement, ticket and reload are three device-scope round trips
//     that every workgroup pays at the very end, when nothing is left to overlap them with.
#include <math.h>
#include <stdlib.h>

#include <algorithm>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;   // 16-byte staging register
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

struct LmArgs {
  const __bf16* hidden;
  const __bf16* w;
  float2* part;        // [nslab][R]
  int R, Hd, V;
  int nslab, nrtile;
  int tiled;        // W given as contiguous [slab][k-tile][128][64] tiles
  // plain-projection mode (kStore): out[r, v] = product (+ residual[r, v]), bf16, row stride V
  __bf16* out;
  const __bf16* residual;
  // ... with the k range split over ksplit workgroups per (slab, row tile) when the grid would otherwise leave most
  // compute units idle: fp32 partial sums go to part_f32[ks][R][V] and linear_reduce_kernel finishes
  float* part_f32;
  int ksplit;
};

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// 16-byte slot of chunk c (0..7) of row `row` in a tile with 128-byte rows.  The XOR term
// makes 16 lanes that read one chunk column of 16 consecutive rows hit 16 distinct banks.
__device__ __forceinline__ int tile_slot(int row, int c) { return row * 8 + (c ^ ((row >> 1) & 7)); }

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int MT, int NT>
struct LmCfg {
  static constexpr int kWRows = MT * 32, kHRows = NT * 32;
  static constexpr int kWaveLds = (kWRows + kHRows) * 128;        // main-loop tiles of one wave
  static constexpr int kTiles = MT * NT;
  static constexpr int kRedBytes = 4 * 4 * 4096;                  // reduction round: 4 waves x 4 tiles x 4 KB
  static constexpr int kMainBytes = 4 * kWaveLds > kRedBytes ? 4 * kWaveLds : kRedBytes;
  static constexpr int kBestOff = kMainBytes;                     // [MT][kHRows] (value, index)
  static constexpr int kLdsBytes = kBestOff + MT * kHRows * 8;
};

// kStore = false: LM head, the epilogue reduces to one (value, id) pair per (slab, row).
// kStore = true: the same streaming product as a plain projection x . W^T, the epilogue writes the bf16 outputs
// (optionally adding a residual): the other weight matrices of the verifying layer are streamed the same way.
template <int MT, int NT, bool kStore>
__global__ __launch_bounds__(256) void lmhead_bf16_kernel(LmArgs a) {
  using C = LmCfg<MT, NT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, half = lane >> 5;
  // workgroup id -> (slab, row tile): the row tiles of one slab sit 8 ids apart, i.e. run at the same time on the
  // same XCD and share its L2, so that W still comes from HBM once when R needs several row tiles
  const int inner = kStore ? a.nrtile * a.ksplit : a.nrtile;   // workgroups per slab (they share the slab's W rows)
  const int per = 8 * inner;
  const int blk = blockIdx.x / per, rem = blockIdx.x - blk * per;
  const int slab = blk * 8 + (rem & 7);
  if (slab >= a.nslab) return;
  const int slab0 = slab * C::kWRows;
  const int sub = rem >> 3;
  const int ks = kStore ? sub / a.nrtile : 0;
  const int r0 = (sub - ks * a.nrtile) * C::kHRows;
  const int R = a.R, Hd = a.Hd, V = a.V;
  unsigned char* wl = lds + wave * C::kWaveLds;
  unsigned char* hl = wl + C::kWRows * 128;

  // lane (lr = lane/8, lc = lane%8) moves chunk lc of rows 8*p + lr
  const int lr = lane >> 3, lc = lane & 7;
  u32x4 wreg[MT * 4], hreg[NT * 4];
  // Row pointers of this lane are fixed for the whole kernel; only the k offset moves.
  const __bf16* wrow[MT * 4];
  const __bf16* hrow[NT * 4];
  // Row-major W: row pointers, k-tile kt at +64*kt.  Tiled W: the slab's tiles are contiguous 16 KB blocks,
  // row r of k-tile kt at (kt*128 + r)*64, so one load instruction of the wave reads 1 KB contiguous.
  const size_t wstep = a.tiled ? 128 * 64 : 64;
#pragma unroll
  for (int p = 0; p < MT * 4; ++p)
    wrow[p] = a.tiled ? a.w + (static_cast<size_t>(slab) * (Hd / 64) * 128 + 8 * p + lr) * 64 + 8 * lc
                      : a.w + static_cast<size_t>(min(slab0 + 8 * p + lr, V - 1)) * Hd + 8 * lc;   // rows past V: duplicate, masked later
#pragma unroll
  for (int p = 0; p < NT * 4; ++p)
    hrow[p] = a.hidden + static_cast<size_t>(min(r0 + 8 * p + lr, R - 1)) * Hd + 8 * lc;
#define OURO_LM_ISSUE_LOADS(KT)                                                            \
  {                                                                                        \
    const size_t koff = static_cast<size_t>(KT) * 64;                                      \
    _Pragma("unroll") for (int p = 0; p < MT * 4; ++p)                                     \
        wreg[p] = *reinterpret_cast<const u32x4*>(wrow[p] + static_cast<size_t>(KT) * wstep); \
    _Pragma("unroll") for (int p = 0; p < NT * 4; ++p)                                     \
        hreg[p] = *reinterpret_cast<const u32x4*>(hrow[p] + koff);                         \
  }

  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;

  // this workgroup's k-tiles: all of them, or its share of an even split
  const int nkt_all = Hd / 64;
  const int kt_per = kStore ? (nkt_all + a.ksplit - 1) / a.ksplit : nkt_all;
  const int kt0 = ks * kt_per;
  const int nkt = min(nkt_all, kt0 + kt_per);
  int kt = kt0 + wave;
  if (kt < nkt) OURO_LM_ISSUE_LOADS(kt)
  for (; kt < nkt; kt += 4) {
    // Each staging register is copied to LDS and immediately re-armed with its load of the wave's next
    // k-tile, so the memory queue of the wave is never empty while the tile is being written (the last
    // iteration harmlessly re-reads its own tile).
    const size_t ktn = static_cast<size_t>(kt + 4 < nkt ? kt + 4 : kt);
    const size_t knext = ktn * 64, wnext = ktn * wstep;
#pragma unroll
    for (int p = 0; p < MT * 4; ++p) {
      *reinterpret_cast<u32x4*>(wl + tile_slot(8 * p + lr, lc) * 16) = wreg[p];
      wreg[p] = *reinterpret_cast<const u32x4*>(wrow[p] + wnext);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int p = 0; p < NT * 4; ++p) {
      *reinterpret_cast<u32x4*>(hl + tile_slot(8 * p + lr, lc) * 16) = hreg[p];
      hreg[p] = *reinterpret_cast<const u32x4*>(hrow[p] + knext);
      __builtin_amdgcn_sched_barrier(0);
    }
    wave_lds_fence();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 af[MT], bf[NT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        af[mt] = *reinterpret_cast<const bf16x8*>(wl + tile_slot(32 * mt + col, 2 * s + half) * 16);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        bf[nt] = *reinterpret_cast<const bf16x8*>(hl + tile_slot(32 * nt + col, 2 * s + half) * 16);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bf[nt], acc[mt][nt], 0, 0, 0);
    }
    wave_lds_fence();
  }

#undef OURO_LM_ISSUE_LOADS

  // ---- sum the 4 waves' accumulators, 4 tiles per round; wave w reduces tile 4*round + w ----
  float* bestv = reinterpret_cast<float*>(lds + C::kBestOff);
  int* besti = reinterpret_cast<int*>(lds + C::kBestOff + MT * C::kHRows * 4);
  constexpr int kRounds = C::kTiles / 4;
  static_assert(C::kTiles % 4 == 0, "tiles per wave must be a multiple of 4");
#pragma unroll
  for (int rd = 0; rd < kRounds; ++rd) {
    __syncthreads();                                          // main-loop LDS (or previous round) no longer read
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      const int tile = rd * 4 + tt;
      const int mt = tile / NT, nt = tile % NT;
      f32x4* dst = reinterpret_cast<f32x4*>(lds) + ((wave * 4 + tt) * 4) * 64 + lane;
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 v4 = {acc[mt][nt][4 * ig + 0], acc[mt][nt][4 * ig + 1], acc[mt][nt][4 * ig + 2], acc[mt][nt][4 * ig + 3]};
        dst[ig * 64] = v4;
      }
    }
    __syncthreads();
    const int tile = rd * 4 + wave;
    const int mt = tile / NT, nt = tile % NT;
    if constexpr (kStore) {
      // lane (col, half) holds, for row r0 + 32*nt + col, the outputs of columns slab0 + 32*mt + 8*ig + 4*half + 0..3
      const int r = r0 + 32 * nt + col;
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) sum += reinterpret_cast<const f32x4*>(lds)[((wv * 4 + wave) * 4 + ig) * 64 + lane];
        const int v = slab0 + 32 * mt + 8 * ig + 4 * half;
        if (r < R && v < V) {                                    // V is a multiple of 8 in this mode: whole groups
          const size_t o = static_cast<size_t>(r) * V + v;
          if (a.ksplit > 1) {
            *reinterpret_cast<f32x4*>(a.part_f32 + static_cast<size_t>(ks) * R * V + o) = sum;
            continue;
          }
          if (a.residual) {
            const bf16x4 res = *reinterpret_cast<const bf16x4*>(a.residual + o);
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[e] += static_cast<float>(res[e]);
          }
          *reinterpret_cast<bf16x4*>(a.out + o) = __builtin_convertvector(sum, bf16x4);
        }
      }
      continue;
    }
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int ig = 0; ig < 4; ++ig) {
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) sum += reinterpret_cast<const f32x4*>(lds)[((wv * 4 + wave) * 4 + ig) * 64 + lane];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = slab0 + 32 * mt + 8 * ig + 4 * half + e;   // accumulator register 4*ig+e of this lane
        const float x = v < V ? sum[e] : -INFINITY;
        if (x > bv) { bv = x; bi = v; }                          // v ascending within the lane
      }
    }
    const float ov = __shfl_xor(bv, 32);
    const int oi = __shfl_xor(bi, 32);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    if (half == 0) {
      bestv[mt * C::kHRows + 32 * nt + col] = bv;
      besti[mt * C::kHRows + 32 * nt + col] = bi;
    }
  }
  if constexpr (kStore) return;
  __syncthreads();
  for (int rl = threadIdx.x; rl < C::kHRows; rl += 256) {
    if (r0 + rl >= R) continue;
    float bv = bestv[rl];
    int bi = besti[rl];
#pragma unroll
    for (int mt = 1; mt < MT; ++mt) {
      const float v2 = bestv[mt * C::kHRows + rl];
      const int i2 = besti[mt * C::kHRows + rl];
      if (better(v2, i2, bv, bi)) { bv = v2; bi = i2; }
    }
    a.part[static_cast<size_t>(slab) * R + r0 + rl] = make_float2(bv, __int_as_float(bi));
  }
}

// out = bf16(sum over the k splits in ascending order (+ residual)); 4 outputs per thread
__global__ __launch_bounds__(256) void linear_reduce_kernel(const float* __restrict__ part, const __bf16* residual,
                                                            __bf16* out, size_t n, int ksplit) {
  const size_t i = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  f32x4 sum = *reinterpret_cast<const f32x4*>(part + i);
  for (int ks = 1; ks < ksplit; ++ks) sum += *reinterpret_cast<const f32x4*>(part + static_cast<size_t>(ks) * n + i);
  if (residual) {
    const bf16x4 res = *reinterpret_cast<const bf16x4*>(residual + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) sum[e] += static_cast<float>(res[e]);
  }
  *reinterpret_cast<bf16x4*>(out + i) = __builtin_convertvector(sum, bf16x4);
}

// Row-major bf16 [V, Hd] -> [ceil(V/128)][Hd/64][128][64] tiles, 16 bytes per thread; rows past V become zero.
__global__ __launch_bounds__(256) void pack_w_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int V, int Hd,
                                                     size_t n16) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n16) return;
  const int c = static_cast<int>(i & 7);                 // 16-byte chunk within a 64-column row
  const int r = static_cast<int>((i >> 3) & 127);        // row within the tile
  const size_t tile = i >> 10;
  const int nkt = Hd / 64;
  const int kt = static_cast<int>(tile % nkt);
  const size_t slab = tile / nkt;
  const size_t v = slab * 128 + r;
  u32x4 x = {0u, 0u, 0u, 0u};
  if (v < static_cast<size_t>(V)) x = src[(v * Hd + static_cast<size_t>(kt) * 64) / 8 + c];
  dst[i] = x;
}

template <int MT, int NT, bool kStore>
int launch_variant(const LmArgs& a, const LmPlan& plan, hipStream_t stream) {
  using C = LmCfg<MT, NT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_bf16_kernel<MT, NT, kStore>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
    if (e != hipSuccess) return hip_failed(e);
    attr_set = true;
  }
  const unsigned grid = static_cast<unsigned>((plan.nslab + 7) / 8) * 8u * plan.nrtile * (kStore ? a.ksplit : 1);
  hipLaunchKernelGGL((lmhead_bf16_kernel<MT, NT, kStore>), dim3(grid), dim3(256), C::kLdsBytes, stream, a);
  return check_launch();
}

}  // namespace

int launch_pack_w(const void* src, void* dst, int V, int Hd, hipStream_t stream) {
  const size_t n16 = static_cast<size_t>((V + 127) / 128) * 128 * static_cast<size_t>(Hd) / 8;
  hipLaunchKernelGGL(pack_w_kernel, dim3(static_cast<unsigned>((n16 + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), V, Hd, n16);
  return check_launch();
}

int launch_lmhead_bf16(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream) {
  LmArgs a{};
  a.hidden = static_cast<const __bf16*>(d.hidden);
  a.w = static_cast<const __bf16*>(d.w);
  a.part = static_cast<float2*>(d.workspace);
  a.R = d.R;
  a.Hd = d.Hd;
  a.V = d.V;
  a.tiled = d.w_layout == OURO_W_TILED;
  a.nslab = plan.nslab;
  a.nrtile = plan.nrtile;
  if (plan.variant == 3) return launch_lmhead_bf16_tile(d, plan, stream);
  if (plan.variant == 1) return launch_variant<4, 2, false>(a, plan, stream);
  return launch_variant<4, 4, false>(a, plan, stream);
}

// Split of the k range of a projection over workgroups: enough of them to occupy the chip, at least 8 k-tiles each.
int linear_ksplit(int R, int K, int N) {
  const int nrtile = R <= 64 ? 1 : (R + 127) / 128;
  const long wgs = static_cast<long>((N + 127) / 128) * nrtile;
  long ks = std::max<long>(1, 256 / std::max<long>(wgs, 1));
  ks = std::min<long>(ks, std::max(1, K / 64 / 8));
  const char* env = std::getenv("OURO_LINEAR_KSPLIT");
  if (env && *env) ks = std::max(1L, std::min<long>(std::atol(env), K / 64));
  return static_cast<int>(ks);
}

size_t linear_workspace_bytes(int R, int K, int N) {
  const int ks = linear_ksplit(R, K, N);
  return ks > 1 ? static_cast<size_t>(ks) * R * N * sizeof(float) : 0;
}

int launch_linear_bf16(const ouro_linear_desc& d, hipStream_t stream) {
  LmArgs a{};
  a.hidden = static_cast<const __bf16*>(d.x);
  a.w = static_cast<const __bf16*>(d.w);
  a.R = d.R;
  a.Hd = d.K;
  a.V = d.N;
  a.tiled = d.w_layout == OURO_W_TILED;
  a.out = static_cast<__bf16*>(d.out);
  a.residual = static_cast<const __bf16*>(d.residual);
  a.ksplit = linear_ksplit(d.R, d.K, d.N);
  a.part_f32 = static_cast<float*>(d.workspace);
  LmPlan plan{};
  plan.slab = 128;
  plan.nslab = (d.N + 127) / 128;
  a.nslab = plan.nslab;
  int st;
  if (d.R <= 64) {
    plan.rtile = 64;
    a.nrtile = plan.nrtile = 1;
    st = launch_variant<4, 2, true>(a, plan, stream);
  } else {
    plan.rtile = 128;                             // more rows: 128-row tiles; the tiles of a slab share an XCD's L2
    a.nrtile = plan.nrtile = (d.R + 127) / 128;
    st = launch_variant<4, 4, true>(a, plan, stream);
  }
  if (st != OURO_OK || a.ksplit == 1) return st;
  const size_t n = static_cast<size_t>(d.R) * d.N;
  hipLaunchKernelGGL(linear_reduce_kernel, dim3(static_cast<unsigned>((n / 4 + 255) / 256)), dim3(256), 0, stream,
                     a.part_f32, a.residual, a.out, n, a.ksplit);
  return check_launch();
}

}  // namespace ouro
