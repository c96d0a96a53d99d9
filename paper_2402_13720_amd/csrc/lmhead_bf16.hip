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
//     coalesced 16-byte buffer loads into registers, then into its private XOR-swizzled LDS
//     region, and issues MT*NT v_mfma_f32_32x32x16_bf16 per 16-wide k step; every staging
//     register is re-armed with its next load right after its LDS write (W two k-tiles
//     ahead where the registers allow, the L2-resident hidden rows one).  Within a k-tile the
//     hidden rows are re-armed before W: loads complete in issue order, and the hidden tile
//     is needed one k-tile from now, W two, so with W first the wait for the hidden tile
//     would also wait for the W loads issued in front of it and empty the pipeline;
//   * after the loop the 4 partial accumulator sets are summed through LDS (fixed order),
//     and the arg-max epilogue reduces lane -> wave -> workgroup; one (value, index) pair
//     per (slab, row) goes to the workspace, the logits never leave the chip;
//   * a second tiny kernel reduces the pairs over the slabs (no float atomics; the result is
//     order-independent because (larger value, then smaller index) is a total order).  A
//     single-launch variant in which the last workgroup did this reduction was measured
//     slower: store acknowledgement, ticket and reload are three device-scope round trips
//     that every workgroup pays at the very end, when nothing is left to overlap them with.
#include <math.h>

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
  int swiglu;       // kStore: columns 2j, 2j+1 are gate and up of feature j; out[r, j] = silu(gate) * up, row stride V/2
  // kStore, rms_eps > 0: every output row is scaled by 1 / sqrt(mean_k hidden[r, k]^2 + rms_eps) (RMSNorm of the input
  // with its gain folded into W).  The sums of squares come from the hidden tiles the workgroup stages anyway; with
  // the k range split, the slab-0 workgroups leave their share in part_ss[ks][R] and the reduction kernel finishes.
  float rms_eps;
  float* part_ss;
};

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + expf(-g)) * u; }
// sum of the squares of 8 packed bf16 values (a bf16 is the upper half of an fp32)
__device__ __forceinline__ float sumsq_bf16x8(u32x4 v) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(v[i] << 16), hi = __uint_as_float(v[i] & 0xffff0000u);
    s = fmaf(lo, lo, s);
    s = fmaf(hi, hi, s);
  }
  return s;
}

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
// kTiled: W is in the tiled layout (every slab padded to 128 rows), else row-major.
template <int MT, int NT, bool kStore, bool kTiled>
__global__ __launch_bounds__(256) void lmhead_bf16_kernel(LmArgs a) {
  using C = LmCfg<MT, NT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
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

  // lane (lr = lane/8, lc = lane%8) moves chunk lc of rows 8*p + lr.  Addresses = one uniform base per operand +
  // a per-lane 32-bit element offset per row (fixed for the whole kernel) + the k-tile step.
  const int lr = lane >> 3, lc = lane & 7;
  // Row-major W: k-tile kt at +64*kt.  Tiled W: the slab's tiles are contiguous 16 KB blocks, row r of k-tile kt at
  // (kt*128 + r)*64, so one load instruction of the wave reads 1 KB contiguous.
  // Loads go through raw buffer descriptors (one per operand, covering exactly the rows this workgroup reads):
  // address = descriptor base + 32-bit per-lane byte offset (fixed for the whole kernel) + wave-uniform offset
  // (k-tile, and for the padded tiled layout also the row group), so no 64-bit address arithmetic or pointer
  // registers live in the loop.  Row-major W and the hidden rows need a per-row clamp (rows past V or R: duplicate
  // of the last one, masked or unused later) and keep one offset register per row group.
  const unsigned wstep = kTiled ? 128 * 64 * 2 : 64 * 2;
  const __bf16* wptr = kTiled ? a.w + static_cast<size_t>(slab) * (Hd / 64) * 128 * 64 : a.w + static_cast<size_t>(slab0) * Hd;
  const unsigned wbytes = static_cast<unsigned>(kTiled ? 128 : min(C::kWRows, V - slab0)) * static_cast<unsigned>(Hd) * 2u;
  const unsigned hbytes = static_cast<unsigned>(min(C::kHRows, R - r0)) * static_cast<unsigned>(Hd) * 2u;
  const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(wptr), 0, wbytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t hbuf =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(a.hidden + static_cast<size_t>(r0) * Hd), 0, hbytes, 0x00020000);
  unsigned woff[kTiled ? 1 : MT * 4], hoff[NT * 4];
  if constexpr (kTiled) {
    woff[0] = static_cast<unsigned>(lr * 128 + 16 * lc);
  } else {
#pragma unroll
    for (int p = 0; p < MT * 4; ++p)
      woff[p] = static_cast<unsigned>(min(8 * p + lr, V - 1 - slab0)) * static_cast<unsigned>(Hd * 2) + 16 * lc;
  }
#pragma unroll
  for (int p = 0; p < NT * 4; ++p)
    hoff[p] = static_cast<unsigned>(min(8 * p + lr, R - 1 - r0)) * static_cast<unsigned>(Hd * 2) + 16 * lc;
// (cache policy 2 = non-temporal: every W byte is read once, so its lines are not kept in L2, which they would otherwise
// fill at the expense of the hidden rows every workgroup re-reads and of whatever the next kernel needs; measured on the
// 64-row workloads: 92.4 -> 85.1 us at hidden size 8192, 50.8 -> 49.3 us at 4096, and 2 us off the attention that follows)
#define OURO_LM_WLOAD(P, KT) \
  __builtin_amdgcn_raw_buffer_load_b128(wbuf, woff[kTiled ? 0 : (P)], (KT) * wstep + (kTiled ? (P) * 1024 : 0), 2)
  // LDS slot of (row 8p + lr, chunk lc): the swizzle term depends on p only through its parity
  const unsigned lds_even = static_cast<unsigned>(lr * 128 + ((lc ^ ((lr >> 1) & 7)) * 16));
  const unsigned lds_odd = static_cast<unsigned>(lr * 128 + ((lc ^ (((lr >> 1) + 4) & 7)) * 16));
#define OURO_LM_LDS_SLOT(P) ((((P) & 1) ? lds_odd : lds_even) + (P) * 1024)

  // W is the stream that comes from HBM: two k-tiles of it are in flight per wave (two staging sets, if the
  // registers allow: kWSets), one k-tile of the hidden rows (they come from L2).
  constexpr int kWSets = (C::kTiles <= 8 && kTiled) ? 2 : 1;
  u32x4 wreg[kWSets][MT * 4], hreg[NT * 4];
#define OURO_LM_LOAD_W(SET, KT)                                                                       \
  _Pragma("unroll") for (int p = 0; p < MT * 4; ++p)                                                  \
      wreg[SET][p] = OURO_LM_WLOAD(p, KT);
#define OURO_LM_LOAD_H(KT)                                                                            \
  _Pragma("unroll") for (int p = 0; p < NT * 4; ++p)                                                  \
      hreg[p] = __builtin_amdgcn_raw_buffer_load_b128(hbuf, hoff[p], (KT) * 128, 0);

  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;
  // Sums of squares of the hidden rows (rms): lane (col, half) squares the 8 values of row 32nt + col it holds as an MFMA
  // operand fragment in every k step; the vector ALU does that between the MFMAs, which it would otherwise sit out.
  const bool rms = kStore && a.rms_eps > 0.f;
  float ss[kStore ? NT : 1];
#pragma unroll
  for (int nt = 0; nt < (kStore ? NT : 1); ++nt) ss[nt] = 0.f;

  // this workgroup's k-tiles: all of them, or its share of an even split; this wave's: first + 4*j, j = 0..nj-1
  const int nkt_all = Hd / 64;
  const int kt_per = kStore ? (nkt_all + a.ksplit - 1) / a.ksplit : nkt_all;
  const int kt0 = ks * kt_per;
  const int nkt = min(nkt_all, kt0 + kt_per);
  const int first = kt0 + wave;
  const int nj = first < nkt ? (nkt - first + 3) / 4 : 0;
  const int last = first + 4 * max(nj - 1, 0);            // loads past the wave's share re-read this tile (harmless)
  const int kt_safe = min(last, nkt_all - 1);

// One k-tile: staging registers (hidden rows, then W set SET) -> this wave's LDS tiles, each register re-armed at once with
// its next load (W: KT_W, the tile kWSets steps ahead; hidden: KT_H, the next tile), then the MFMAs.  Loads and stores
// are unconditional so that the compiler's counted waits stay exact; only the MFMAs of a step past the end are skipped.
#define OURO_LM_KTILE(SET, KT_W, KT_H, VALID)                                                         \
  {                                                                                                   \
    _Pragma("unroll") for (int p = 0; p < NT * 4; ++p) {                                              \
      *reinterpret_cast<u32x4*>(hl + OURO_LM_LDS_SLOT(p)) = hreg[p];                                  \
      hreg[p] = __builtin_amdgcn_raw_buffer_load_b128(hbuf, hoff[p], (KT_H) * 128, 0);                \
      __builtin_amdgcn_sched_barrier(0);                                                              \
    }                                                                                                 \
    _Pragma("unroll") for (int p = 0; p < MT * 4; ++p) {                                              \
      *reinterpret_cast<u32x4*>(wl + OURO_LM_LDS_SLOT(p)) = wreg[SET][p];                             \
      wreg[SET][p] = OURO_LM_WLOAD(p, KT_W);                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                              \
    }                                                                                                 \
    wave_lds_fence();                                                                                 \
    if (VALID) {                                                                                      \
      _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                                 \
        bf16x8 af[MT], bf[NT];                                                                        \
        _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                             \
            af[mt] = *reinterpret_cast<const bf16x8*>(wl + tile_slot(32 * mt + col, 2 * s + half) * 16); \
        _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                             \
            bf[nt] = *reinterpret_cast<const bf16x8*>(hl + tile_slot(32 * nt + col, 2 * s + half) * 16); \
        _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                             \
            _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                         \
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], bf[nt], acc[mt][nt], 0, 0, 0); \
        if constexpr (kStore) {                                                                       \
          if (rms) {                                                                                  \
            _Pragma("unroll") for (int nt = 0; nt < NT; ++nt)                                         \
                ss[nt] += sumsq_bf16x8(__builtin_bit_cast(u32x4, bf[nt]));                            \
          }                                                                                           \
        }                                                                                             \
      }                                                                                               \
    }                                                                                                 \
    wave_lds_fence();                                                                                 \
  }

  if (nj > 0) {
    OURO_LM_LOAD_W(0, first)
    OURO_LM_LOAD_H(first)
    if (kWSets == 2) { OURO_LM_LOAD_W(kWSets - 1, min(first + 4, kt_safe)) }
    if (kWSets == 2) {
      for (int j = 0; j < nj; j += 2) {
        const int t0 = first + 4 * j;
        OURO_LM_KTILE(0, min(t0 + 8, kt_safe), min(t0 + 4, kt_safe), true)
        OURO_LM_KTILE(kWSets - 1, min(t0 + 12, kt_safe), min(t0 + 8, kt_safe), j + 1 < nj)
      }
    } else {
      for (int j = 0; j < nj; ++j) {
        const int t0 = first + 4 * j;
        OURO_LM_KTILE(0, min(t0 + 4, kt_safe), min(t0 + 4, kt_safe), true)
      }
    }
  }
#undef OURO_LM_KTILE
#undef OURO_LM_LOAD_W
#undef OURO_LM_LOAD_H
#undef OURO_LM_WLOAD
#undef OURO_LM_LDS_SLOT


  // ---- sum the 4 waves' accumulators, 4 tiles per round; wave w reduces tile 4*round + w ----
  float* bestv = reinterpret_cast<float*>(lds + C::kBestOff);
  int* besti = reinterpret_cast<int*>(lds + C::kBestOff + MT * C::kHRows * 4);
  float* rowss = bestv;                                       // kStore: [4 waves][kHRows] sums of squares
  if constexpr (kStore) {
    if (rms) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const float t = ss[nt] + __shfl_xor(ss[nt], 32);      // the two k halves of row 32nt + col
        if (half == 0) rowss[wave * C::kHRows + 32 * nt + col] = t;
      }
    }
  }
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
      float rinv = 1.0f;
      if (rms && a.ksplit == 1) {                               // (the first barrier of the round ordered the rowss writes)
        const int rl = 32 * nt + col;
        const float tot = (rowss[rl] + rowss[C::kHRows + rl]) + (rowss[2 * C::kHRows + rl] + rowss[3 * C::kHRows + rl]);
        rinv = 1.0f / sqrtf(tot / static_cast<float>(Hd) + a.rms_eps);
      }
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
          sum *= rinv;
          if (a.swiglu) {
            const bf16x2 act = {static_cast<__bf16>(silu_mul(sum[0], sum[1])), static_cast<__bf16>(silu_mul(sum[2], sum[3]))};
            *reinterpret_cast<bf16x2*>(a.out + o / 2) = act;         // o = r*V + v with V and v even: r*(V/2) + v/2
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
  if constexpr (kStore) {
    if (rms && a.ksplit > 1 && slab == 0) {
      for (int rl = threadIdx.x; rl < C::kHRows; rl += 256)
        if (r0 + rl < R)
          a.part_ss[static_cast<size_t>(ks) * R + r0 + rl] =
              (rowss[rl] + rowss[C::kHRows + rl]) + (rowss[2 * C::kHRows + rl] + rowss[3 * C::kHRows + rl]);
    }
    return;
  }
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
// (part_ss: the k-split shares of the rows' sums of squares, or null; N, K: columns of the product, input features)
__global__ __launch_bounds__(256) void linear_reduce_kernel(const float* __restrict__ part, const __bf16* residual,
                                                            __bf16* out, size_t n, int ksplit, int swiglu,
                                                            const float* __restrict__ part_ss, int N, int K, float rms_eps) {
  const size_t i = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  f32x4 sum = *reinterpret_cast<const f32x4*>(part + i);
  for (int ks = 1; ks < ksplit; ++ks) sum += *reinterpret_cast<const f32x4*>(part + static_cast<size_t>(ks) * n + i);
  if (part_ss) {
    const size_t r = i / N, R = n / N;
    float tot = part_ss[r];
    for (int ks = 1; ks < ksplit; ++ks) tot += part_ss[static_cast<size_t>(ks) * R + r];
    sum *= 1.0f / sqrtf(tot / static_cast<float>(K) + rms_eps);
  }
  if (swiglu) {                                                        // (gate, up) pairs -> [R, N/2]
    const bf16x2 act = {static_cast<__bf16>(silu_mul(sum[0], sum[1])), static_cast<__bf16>(silu_mul(sum[2], sum[3]))};
    *reinterpret_cast<bf16x2*>(out + i / 2) = act;
    return;
  }
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

template <int MT, int NT, bool kStore, bool kTiled>
int launch_instance(const LmArgs& a, const LmPlan& plan, hipStream_t stream) {
  using C = LmCfg<MT, NT>;
  static DeviceOnce once;                                   // one per kernel instance
  const int ready = device_once(once, [] {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_bf16_kernel<MT, NT, kStore, kTiled>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
    return e == hipSuccess ? static_cast<int>(OURO_OK) : hip_failed(e);
  });
  if (ready != OURO_OK) return ready;
  const unsigned grid = static_cast<unsigned>((plan.nslab + 7) / 8) * 8u * plan.nrtile * (kStore ? a.ksplit : 1);
  hipLaunchKernelGGL((lmhead_bf16_kernel<MT, NT, kStore, kTiled>), dim3(grid), dim3(256), C::kLdsBytes, stream, a);
  return check_launch();
}

template <int MT, int NT, bool kStore>
int launch_variant(const LmArgs& a, const LmPlan& plan, hipStream_t stream) {
  return a.tiled ? launch_instance<MT, NT, kStore, true>(a, plan, stream)
                 : launch_instance<MT, NT, kStore, false>(a, plan, stream);
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
// (`forced` > 0: a count given by the caller for tests and tuning runs.)
int linear_ksplit(int R, int K, int N, int forced) {
  const int nrtile = R <= 64 ? 1 : (R + 127) / 128;
  const long wgs = static_cast<long>((N + 127) / 128) * nrtile;
  long ks = std::max<long>(1, 256 / std::max<long>(wgs, 1));
  ks = std::min<long>(ks, std::max(1, K / 64 / 8));
  if (forced > 0) ks = std::max(1L, std::min<long>(forced, K / 64));
  return static_cast<int>(ks);
}

size_t linear_workspace_bytes(int R, int K, int N, int ksplit_override) {
  const int ks = linear_ksplit(R, K, N, ksplit_override);
  return ks > 1 ? static_cast<size_t>(ks) * R * (static_cast<size_t>(N) + 1) * sizeof(float) : 0;   // partial sums + row shares
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
  a.ksplit = linear_ksplit(d.R, d.K, d.N, d.ksplit_override);
  a.part_f32 = static_cast<float*>(d.workspace);
  a.swiglu = d.epilogue == OURO_EPI_SWIGLU_PAIRS;
  a.rms_eps = d.rms_eps > 0.f ? d.rms_eps : 0.f;
  a.part_ss = a.part_f32 ? a.part_f32 + static_cast<size_t>(a.ksplit) * d.R * d.N : nullptr;
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
                     a.part_f32, a.residual, a.out, n, a.ksplit, a.swiglu, a.rms_eps > 0.f ? a.part_ss : nullptr, d.N, d.K,
                     a.rms_eps);
  return check_launch();
}

}  // namespace ouro
