// bf16 draft-block attention for gfx950: split-KV with in-workgroup key splitting.
//
// What is computed (Sec. 3.2, Eq. (8)): every block row attends to the whole cached prefix
// of its sequence plus the block tokens of its own lengthened draft.  The block part of the
// mask is evaluated from per-token (phrase_id, branch_off) pairs in registers; only the
// key tiles that overlap the block (the last T keys) pay for it, cache tiles are mask-free.
//
// Work decomposition.  Query rows of one (sequence, KV head) are the T*G rows of the G query
// heads sharing that KV head (row = t*G + head_in_group), cut into row blocks of 32 rows.
// The key axis [cache | block] is cut into chunks.  One workgroup (4 waves) owns one
// (sequence, KV head, chunk, row block); its waves take the chunk's 32-key tiles round-robin,
// so together they stream one contiguous window of K and V.  Each wave runs a flash-style
// loop on its own tiles without ever synchronising with the other waves:
//
//   global --coalesced 16B loads--> registers --> wave-private LDS (K row-major swizzled,
//   V transposed with in-register byte-permutes) --> MFMA operands
//
//   S^T[key, q]  = K . Q^T          v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q rows from a
//                                    workgroup-shared LDS tile (keeps the kernel under 256 registers:
//                                    two waves per SIMD, no spills between a prefetch and its use)
//   online softmax in the exp2 domain, one query per lane column, keys along registers
//   O^T[d, q]   += V^T . P^T        A = V^T from LDS, B = P^T = the S^T accumulator registers
//                                    rounded to bf16 (no shuffle: the accumulator layout of
//                                    S^T already is a valid B-operand layout, with the key
//                                    order of V^T permuted to match when V is transposed)
//
// The next tile's global loads are issued before the current tile's math.  After the loop
// the 4 wave states (O, running max, running sum) are merged pairwise through LDS, staged
// row-major in LDS and written with coalesced 16-byte stores.  A sequence that spans several
// chunks leaves one fp32 partial per workgroup, and a second small kernel merges the partials
// of a row in ascending chunk order (deterministic) and writes bf16.  (A single-launch variant
// in which the last workgroup of a row block merged the partials was measured slower: the
// device-scope store/ticket/load round trips stall every workgroup for several microseconds.)
//
// Workgroup ids are mapped so that workgroups reading the same K/V window (different row
// blocks) are congruent modulo 8, i.e. land on the same XCD and share its L2.
#include <math.h>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;   // 16-byte staging register

constexpr int kD = 128;
constexpr int kKBytes = 32 * 256;             // K tile, 16-byte slots XOR-swizzled by row (no padding)
constexpr int kVtBytes = 128 * 32 * 2;        // V^T tile, swizzled 16-byte slots
constexpr int kWaveLds = kKBytes + kVtBytes;  // 16 KB per wave, 64 KB per workgroup
constexpr int kStageRow = 132;                // floats per staged output row (128 + 4 pad: conflict-free 16B column writes)
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const __bf16* q;
  const __bf16* k_cache;
  const __bf16* v_cache;
  const __bf16* k_blk;
  const __bf16* v_blk;
  const int64_t* cu;
  const ouro_tok_meta* meta;
  __bf16* out;
  float* lse;
  float* part_ml;      // [group][chunk][rows_wg][2]
  float* part_o;       // [group][chunk][rows_wg][128]
  int n_x;             // B * Hkv * nch
  int T, Hq, Hkv, G, M;
  int nrb, nch, chunk;
  float scale_log2;
};

constexpr int cmax(int x, int y) { return x > y ? x : y; }

constexpr int kRows = 32;                                  // query rows per workgroup
constexpr int kQBytes = kRows * 256;                       // Q tile shared by the 4 waves, same swizzle as the K tile
constexpr int kStateBytes = 16 * 64 * 16;                  // O accumulators of one wave, lane-major
constexpr int kMergeBytes = 2 * kStateBytes + 2 * 64 * 8;  // two slots + their (max, sum) pairs
constexpr int kStageBytes = kRows * kStageRow * 4 + kRows * 8;
constexpr int kLdsBytes = kQBytes + cmax(cmax(4 * kWaveLds, kMergeBytes), kStageBytes);   // 72 KB: two workgroups per CU

// Slot (16 bytes = 8 keys of one head-dim element d) of the transposed V tile.
// d = 8*a + j, c = key group (0..3).  Writers (fixed j, c; a = 0..15) and readers
// (fixed c; 16 consecutive d) both touch 16 distinct slots modulo 16, i.e. distinct banks.
__device__ __forceinline__ int vt_slot(int a, int j, int c) { return 16 * (8 * c + j) + ((a + 2 * j) & 15); }

// Slot of 16-byte chunk c (0..15) of key row `row` (0..31) in the K tile: a row-major tile
// whose chunk index is XORed with the row, so that 16 lanes reading one chunk column of 16
// consecutive rows (MFMA A operand) and 16 lanes writing one row both hit 16 distinct banks.
__device__ __forceinline__ int k_slot(int row, int c) { return row * 16 + (c ^ (row & 15)); }

__device__ __forceinline__ unsigned dword_of(const u32x4& v, int w) { return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w; }

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;

  // ---- workgroup id -> (x = (sequence, KV head, chunk), row block); same x => same id modulo 8 ----
  const int per = 8 * a.nrb;
  const int blk = blockIdx.x / per, rem = blockIdx.x - blk * per;
  const int rb = rem >> 3;
  const int x = blk * 8 + (rem & 7);
  if (x >= a.n_x) return;
  const int chunk = x % a.nch;
  const int bg = x / a.nch;
  const int b = bg / a.Hkv, g = bg - b * a.Hkv;
  const long cu0 = a.cu[b];
  const int L = static_cast<int>(a.cu[b + 1] - cu0);
  const int T = a.T;
  const int n = L + T;
  const int k_begin = chunk * a.chunk;
  if (k_begin >= n) return;                       // chunk slot beyond this sequence (uniform for the workgroup)
  const int k_end = min(n, k_begin + a.chunk);
  const int nchb = (n + a.chunk - 1) / a.chunk;   // chunks this sequence really has

  unsigned char* ql = lds;                        // Q tile, shared
  unsigned char* kl = lds + kQBytes + wave * kWaveLds;
  unsigned char* vl = kl + kKBytes;
  const int col = lane & 31, half = lane >> 5;
  const int G = a.G, M = a.M, Hq = a.Hq, Hkv = a.Hkv;
  const int row0 = rb * kRows;

  // ---- Q tile -> LDS (coalesced: 16 lanes per 256-byte row), read back as the B operand of S^T = K . Q^T ----
  for (int p = tid; p < kRows * 16; p += 256) {
    const int row = p >> 4, c = p & 15;
    const int rr = min(row0 + row, M - 1);        // rows past M are computed on a duplicate and never stored
    const int t = rr / G, hh = rr - t * G;
    const __bf16* qp = a.q + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
    *reinterpret_cast<u32x4*>(ql + k_slot(row, c) * 16) = *reinterpret_cast<const u32x4*>(qp + 8 * c);
  }
  // this lane's query row (its column of S^T) and that row's metadata
  const int rq = min(row0 + col, M - 1);
  const int tq = rq / G;
  const ouro_tok_meta mq = a.meta[static_cast<size_t>(b) * T + tq];
  const int pidq = mq.phrase_id, boffq = mq.branch_off;

  // ---- staging: lane (kq = lane/16, c16 = lane%16) loads 16 B of 8 key rows per tile ----
  // Load i of a lane fetches key 4*i + kq of the tile, so one load instruction covers 4 adjacent
  // key rows.  The 8 keys of a lane must be one key group of the P.V contraction, and the S^T
  // accumulator fixes which accumulator rows form a group (rows 16*(kq/2) + 8*jj + 4*(kq%2) + r,
  // i = 4*jj + r); so key 4*i + kq is simply stored in that row of the K tile: the rows of S^T are a
  // permutation of the tile's keys, which only the mask has to know about (key_of_reg below).
  const int kq = lane >> 4, c16 = lane & 15;
  const int row_base = 16 * (kq >> 1) + 4 * (kq & 1);
  u32x4 kr[8], vr[8];
  // Element offset of this lane's first row from the first row of a tile; its other rows follow at
  // fixed multiples of the key stride (tile wholly inside the cache: one wave-uniform base pointer
  // plus these, no per-row address arithmetic in the loop).
  const unsigned kstride = static_cast<unsigned>(Hkv) * kD;
  const unsigned loff0 = static_cast<unsigned>(kq) * kstride + 8 * c16;
#define OURO_ATTN_ISSUE_LOADS(TILE)                                                                                \
  if ((TILE) + 32 <= L) {                                                                                          \
    const size_t base = (static_cast<size_t>(cu0 + (TILE)) * Hkv + g) * kD;                                        \
    const __bf16* kt = a.k_cache + base;                                                                           \
    const __bf16* vt = a.v_cache + base;                                                                           \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                \
      const unsigned off = loff0 + static_cast<unsigned>(4 * i) * kstride;                                         \
      kr[i] = *reinterpret_cast<const u32x4*>(kt + off);                                                           \
      vr[i] = *reinterpret_cast<const u32x4*>(vt + off);                                                           \
    }                                                                                                              \
  } else {                                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                \
      const int kidx = min((TILE) + 4 * i + kq, n - 1); /* clamp: finite data, masked later */                     \
      const bool in_cache = kidx < L;                                                                              \
      const size_t row = in_cache ? static_cast<size_t>(cu0 + kidx) : static_cast<size_t>(b) * T + (kidx - L);     \
      const size_t off = (row * Hkv + g) * kD + 8 * c16;                                                           \
      kr[i] = *reinterpret_cast<const u32x4*>((in_cache ? a.k_cache : a.k_blk) + off);                             \
      vr[i] = *reinterpret_cast<const u32x4*>((in_cache ? a.v_cache : a.v_blk) + off);                             \
    }                                                                                                              \
  }

  f32x16 o[4];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;

  // this wave's tiles: k_begin + 32*(wave + 4*i)
  int tile = k_begin + 32 * wave;
  if (tile < k_end) { OURO_ATTN_ISSUE_LOADS(tile) }
  __syncthreads();                                // Q tile complete
  for (; tile < k_end; tile += 128) {
    // ---- registers -> LDS ----
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4*>(kl + k_slot(row_base + 8 * (i >> 2) + (i & 3), c16) * 16) = kr[i];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      // 8 keys of head-dim element 8*c16 + j: dword j/2 of each row, low or high half
      const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;
      u32x4 t4;
      t4.x = __builtin_amdgcn_perm(dword_of(vr[1], j >> 1), dword_of(vr[0], j >> 1), sel);
      t4.y = __builtin_amdgcn_perm(dword_of(vr[3], j >> 1), dword_of(vr[2], j >> 1), sel);
      t4.z = __builtin_amdgcn_perm(dword_of(vr[5], j >> 1), dword_of(vr[4], j >> 1), sel);
      t4.w = __builtin_amdgcn_perm(dword_of(vr[7], j >> 1), dword_of(vr[6], j >> 1), sel);
      *reinterpret_cast<u32x4*>(vl + vt_slot(c16, j, kq) * 16) = t4;
    }
    if (tile + 128 < k_end) { OURO_ATTN_ISSUE_LOADS(tile + 128) }
    wave_lds_fence();

    // ---- S^T = K . Q^T ----
    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kl + k_slot(col, 2 * s + half) * 16);
      const bf16x8 qf = *reinterpret_cast<const bf16x8*>(ql + k_slot(col, 2 * s + half) * 16);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf, sacc, 0, 0, 0);
    }

    // ---- mask (only tiles that touch block keys or run past n; wave-uniform branch) ----
    // Accumulator register i of a lane (half h) is S^T row 8*(i/4) + 4*h + i%4, which holds
    // key 16*((i/4)%2) + 4*(i%4) + 2*(i/8) + h of the tile.
    if (tile + 32 > L) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kb = tile + 16 * ((i >> 2) & 1) + 4 * (i & 3) + 2 * (i >> 3) + half - L;
        bool vis = kb < 0;
        if (kb >= 0 && kb < T) {
          const int pidk = a.meta[static_cast<size_t>(b) * T + kb].phrase_id;
          vis = pidk == 0 ? kb <= boffq : (pidk == pidq && kb <= tq);
        }
        sacc[i] = vis ? sacc[i] : -INFINITY;
      }
    }

    // ---- online softmax (log2 domain) ----
    // The running reference m_run is only raised when a score exceeds it by more than 8 (a factor
    // 256, harmless in fp32 and for the bf16 rounding of P, which is relative); O and the sum stay
    // consistent with whatever reference is in use, so the result is unchanged, and the 64-register
    // rescale of O is skipped on almost every tile.
    float tmax = sacc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sacc[i]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32)) * a.scale_log2;
    if (__any(tmax > m_run + 8.0f)) {
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
    }
    const float neg_m = m_run == -INFINITY ? 0.f : -m_run;
    float psum = 0.f;
    f32x8 p0, p1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      p0[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], a.scale_log2, neg_m));
      p1[i] = __builtin_amdgcn_exp2f(fmaf(sacc[8 + i], a.scale_log2, neg_m));
      psum += p0[i] + p1[i];
    }
    l_run += psum;                                  // per-half partial sum; halves are added at the end
    const bf16x8 pf0 = __builtin_convertvector(p0, bf16x8);
    const bf16x8 pf1 = __builtin_convertvector(p1, bf16x8);

    // ---- O^T += V^T . P^T ----
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const bf16x8 vf0 = *reinterpret_cast<const bf16x8*>(vl + vt_slot(4 * dt + (col >> 3), col & 7, half) * 16);
      const bf16x8 vf1 = *reinterpret_cast<const bf16x8*>(vl + vt_slot(4 * dt + (col >> 3), col & 7, 2 + half) * 16);
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf0, pf0, o[dt], 0, 0, 0);
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf1, pf1, o[dt], 0, 0, 0);
    }
    wave_lds_fence();                               // reads of this tile precede the next tile's LDS writes
  }
#undef OURO_ATTN_ISSUE_LOADS

  // ---- merge the 4 wave states pairwise through LDS: (2,3) -> (0,1), then 1 -> 0 ----
  unsigned char* scratch = lds + kQBytes;
  f32x4* slot_o = reinterpret_cast<f32x4*>(scratch);
  float* slot_ml = reinterpret_cast<float*>(scratch + 2 * kStateBytes);
#pragma unroll
  for (int sft = 2; sft >= 1; sft >>= 1) {
    __syncthreads();
    if (wave >= sft && wave < 2 * sft) {
      const int slot = wave - sft;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int ig = 0; ig < 4; ++ig) {
          f32x4 v4 = {o[dt][4 * ig + 0], o[dt][4 * ig + 1], o[dt][4 * ig + 2], o[dt][4 * ig + 3]};
          slot_o[(slot * 16 + dt * 4 + ig) * 64 + lane] = v4;
        }
      slot_ml[(slot * 64 + lane) * 2 + 0] = m_run;
      slot_ml[(slot * 64 + lane) * 2 + 1] = l_run;
    }
    __syncthreads();
    if (wave < sft) {
      const int slot = wave;
      const float m_b = slot_ml[(slot * 64 + lane) * 2 + 0];
      const float l_b = slot_ml[(slot * 64 + lane) * 2 + 1];
      const float m_new = fmaxf(m_run, m_b);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float fa = exp2f(m_run - m_safe), fb = exp2f(m_b - m_safe);
      m_run = m_new;
      l_run = l_run * fa + l_b * fb;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int ig = 0; ig < 4; ++ig) {
          const f32x4 ob = slot_o[(slot * 16 + dt * 4 + ig) * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[dt][4 * ig + e] = o[dt][4 * ig + e] * fa + ob[e] * fb;
        }
    }
  }
  __syncthreads();

  // ---- wave 0 stages the workgroup's state row-major: stage_o[row][132], stage_ml[row][2] ----
  float* stage_o = reinterpret_cast<float*>(scratch);
  float* stage_ml = stage_o + kRows * kStageRow;
  if (wave == 0) {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 v4 = {o[dt][4 * ig + 0], o[dt][4 * ig + 1], o[dt][4 * ig + 2], o[dt][4 * ig + 3]};
        *reinterpret_cast<f32x4*>(stage_o + col * kStageRow + 32 * dt + 8 * ig + 4 * half) = v4;
      }
    if (half == 0) {
      stage_ml[col * 2 + 0] = m_run;
      stage_ml[col * 2 + 1] = l_tot;
    }
  }
  __syncthreads();

  const int group = bg * a.nrb + rb;
  if (nchb == 1) {
    // ---- the workgroup saw every key of the sequence: normalise and write bf16, 16 B per thread ----
    for (int p = tid; p < kRows * 16; p += 256) {
      const int row = p >> 4, c = p & 15;
      const int r = row0 + row;
      if (r >= M) continue;
      const float inv = 1.0f / stage_ml[row * 2 + 1];
      const f32x4 x0 = *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 8 * c);
      const f32x4 x1 = *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 8 * c + 4);
      f32x8 v8 = {x0[0] * inv, x0[1] * inv, x0[2] * inv, x0[3] * inv, x1[0] * inv, x1[1] * inv, x1[2] * inv, x1[3] * inv};
      const int t = r / G, hh = r - t * G;
      __bf16* op = a.out + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
      *reinterpret_cast<bf16x8*>(op + 8 * c) = __builtin_convertvector(v8, bf16x8);
      if (a.lse && c == 0)
        a.lse[(static_cast<size_t>(b) * Hq + g * G + hh) * T + t] =
            (stage_ml[row * 2] + log2f(stage_ml[row * 2 + 1])) * kLn2;
    }
    return;
  }

  // ---- several chunks: leave a partial for the combine kernel (plain coalesced stores, no waiting) ----
  const size_t pbase = (static_cast<size_t>(group) * a.nch + chunk) * kRows;
  for (int p = tid; p < kRows * 32; p += 256) {
    const int row = p >> 5, c = p & 31;
    *reinterpret_cast<f32x4*>(a.part_o + (pbase + row) * kD + 4 * c) =
        *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 4 * c);
  }
  for (int p = tid; p < kRows * 2; p += 256) a.part_ml[pbase * 2 + p] = stage_ml[p];
}

// Merge the chunk partials of every query row of the sequences that span several chunks:
// out = sum_c 2^(m_c - m*) O_c / sum_c 2^(m_c - m*) l_c, chunks folded in ascending order
// (deterministic).  One thread per (row, 8 head-dim elements); loads are issued four chunks
// at a time so that their latencies overlap.
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
  constexpr int rows_wg = kRows;
  const long p = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
  const int c = static_cast<int>(p & 15);
  const long rowg = p >> 4;
  const int row = static_cast<int>(rowg % rows_wg);
  const long group = rowg / rows_wg;
  if (group >= static_cast<long>(a.n_x / a.nch) * a.nrb) return;
  const int rb = static_cast<int>(group % a.nrb);
  const int bg = static_cast<int>(group / a.nrb);
  const int b = bg / a.Hkv, g = bg - b * a.Hkv;
  const int r = rb * rows_wg + row;
  if (r >= a.M) return;
  const int n = static_cast<int>(a.cu[b + 1] - a.cu[b]) + a.T;
  const int nchb = (n + a.chunk - 1) / a.chunk;
  if (nchb == 1) return;                            // written directly by the main kernel
  const size_t gbase = static_cast<size_t>(group) * a.nch * rows_wg;
  float m_star = -INFINITY, lsum = 0.f;
  f32x8 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int ch0 = 0; ch0 < nchb; ch0 += 4) {
    float m_c[4], l_c[4];
    f32x4 x0[4], x1[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int ch = min(ch0 + u, nchb - 1);          // clamped duplicates are skipped below
      const size_t prow = gbase + static_cast<size_t>(ch) * rows_wg + row;
      m_c[u] = a.part_ml[prow * 2];
      l_c[u] = a.part_ml[prow * 2 + 1];
      x0[u] = *reinterpret_cast<const f32x4*>(a.part_o + prow * kD + 8 * c);
      x1[u] = *reinterpret_cast<const f32x4*>(a.part_o + prow * kD + 8 * c + 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (ch0 + u >= nchb) continue;
      const float m_new = fmaxf(m_star, m_c[u]);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float fa = exp2f(m_star - m_safe), fb = exp2f(m_c[u] - m_safe);
      m_star = m_new;
      lsum = lsum * fa + l_c[u] * fb;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[e] = acc[e] * fa + x0[u][e] * fb;
        acc[4 + e] = acc[4 + e] * fa + x1[u][e] * fb;
      }
    }
  }
  const float inv = 1.0f / lsum;
  const int t = r / a.G, hh = r - t * a.G;
  __bf16* op = a.out + ((static_cast<size_t>(b) * a.T + t) * a.Hq + g * a.G + hh) * kD;
  *reinterpret_cast<bf16x8*>(op + 8 * c) = __builtin_convertvector(acc * inv, bf16x8);
  if (a.lse && c == 0)
    a.lse[(static_cast<size_t>(b) * a.Hq + g * a.G + hh) * a.T + t] = (m_star + log2f(lsum)) * kLn2;
}

}  // namespace

int launch_attn_bf16(const ouro_attn_desc& d, const AttnPlan& plan, float scale, hipStream_t stream) {
  AttnArgs a{};
  a.q = static_cast<const __bf16*>(d.q);
  a.k_cache = static_cast<const __bf16*>(d.k_cache);
  a.v_cache = static_cast<const __bf16*>(d.v_cache);
  a.k_blk = static_cast<const __bf16*>(d.k_blk);
  a.v_blk = static_cast<const __bf16*>(d.v_blk);
  a.cu = d.cu_seqlens;
  a.meta = d.meta;
  a.out = static_cast<__bf16*>(d.out);
  a.lse = d.lse;
  unsigned char* ws = static_cast<unsigned char*>(d.workspace);
  a.part_ml = reinterpret_cast<float*>(ws);
  a.part_o = reinterpret_cast<float*>(ws + plan.part_ml_bytes);
  a.T = d.T;
  a.Hq = d.Hq;
  a.Hkv = d.Hkv;
  a.G = d.Hq / d.Hkv;
  a.M = d.T * a.G;
  a.nrb = plan.nrb;
  a.nch = plan.nch;
  a.chunk = plan.chunk;
  a.n_x = d.B * d.Hkv * plan.nch;
  a.scale_log2 = scale * 1.4426950408889634f;
  const unsigned grid = static_cast<unsigned>((a.n_x + 7) / 8) * 8u * plan.nrb;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return hip_failed(e);
    attr_set = true;
  }
  if (d.ev_start && hipEventRecord(static_cast<hipEvent_t>(d.ev_start), stream) != hipSuccess) return hip_failed(hipGetLastError());
  hipLaunchKernelGGL(attn_bf16_kernel, dim3(grid), dim3(256), kLdsBytes, stream, a);
  int st = check_launch();
  if (st == OURO_OK && d.ev_stop && hipEventRecord(static_cast<hipEvent_t>(d.ev_stop), stream) != hipSuccess)
    return hip_failed(hipGetLastError());
  if (st != OURO_OK || plan.nch == 1) return st;
  const long threads = static_cast<long>(d.B) * d.Hkv * plan.nrb * kRows * 16;
  hipLaunchKernelGGL(attn_combine_kernel, dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0, stream, a);
  return check_launch();
}

}  // namespace ouro
