// bf16 draft-block attention for gfx950: split-KV, one independent wave per work item.
//
// What is computed (Sec. 3.2, Eq. (8)): every block row attends to the whole cached prefix
// of its sequence plus the block tokens of its own lengthened draft.  The block part of the
// mask is evaluated from per-token (phrase_id, branch_off) pairs in registers; only the
// key tiles that overlap the block (the last T keys) pay for it, cache tiles are mask-free.
//
// Work decomposition.  Query rows of one (sequence, KV head) are the T*G rows of the G query
// heads sharing that KV head (row = t*G + head_in_group), cut into row blocks of 32*QT rows.
// The key axis [cache | block] is cut into chunks.  One 64-lane wave owns one
// (sequence, KV head, chunk, row block) item and runs a flash-style loop over 32-key tiles:
//
//   global --coalesced 16B loads--> registers --> wave-private LDS (K row-major swizzled,
//   V transposed with in-register byte-permutes) --> MFMA operands
//
//   S^T[key, q]  = K . Q^T          v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q (registers)
//   online softmax in the exp2 domain, one query per lane column, keys along registers
//   O^T[d, q]   += V^T . P^T        A = V^T from LDS, B = P^T = the S^T accumulator registers
//                                    rounded to bf16 (no shuffle: the accumulator layout of
//                                    S^T already is a valid B-operand layout, with the key
//                                    order of V^T permuted to match when V is transposed)
//
// Waves never synchronise with each other (no s_barrier): each wave has its own LDS region
// and LDS operations of one wave execute in order.  The next tile's global loads are issued
// before the current tile's math, so a wave keeps 16 KB in flight.
// If a sequence spans several chunks every item leaves an un-normalised fp32 partial
// (O, running max, running sum); a second kernel merges the partials of a row in fixed
// chunk order (deterministic) and writes bf16.
#include <math.h>
#include <stdlib.h>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;   // 16-byte staging register

constexpr int kD = 128;
constexpr int kKBytes = 32 * 256;             // K tile, 16-byte slots XOR-swizzled by row (no padding)
constexpr int kVtBytes = 128 * 32 * 2;        // V^T tile, swizzled 16-byte slots
constexpr int kWaveLds = kKBytes + kVtBytes;  // 16 KB per wave, 64 KB per workgroup

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
  float* part_o;   // [group][chunk][rows_wave][128]
  float* part_ml;  // [group][chunk][rows_wave][2]
  long n_items;
  int T, Hq, Hkv, G, M;
  int nrb, nch, chunk;
  float scale_log2;
};

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

template <int QT>
__global__ __launch_bounds__(256) void attn_bf16_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[4 * kWaveLds];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long item = static_cast<long>(blockIdx.x) * 4 + wave;
  if (item >= a.n_items) return;
  const int rb = static_cast<int>(item % a.nrb);
  const long tmp = item / a.nrb;
  const int chunk = static_cast<int>(tmp % a.nch);
  const int bg = static_cast<int>(tmp / a.nch);
  const int b = bg / a.Hkv, g = bg - b * a.Hkv;
  const long cu0 = a.cu[b];
  const int L = static_cast<int>(a.cu[b + 1] - cu0);
  const int T = a.T;
  const int n = L + T;
  const int k_begin = chunk * a.chunk;
  if (k_begin >= n) return;                       // chunk slot beyond this sequence
  const int k_end = min(n, k_begin + a.chunk);

  unsigned char* kl = lds + wave * kWaveLds;
  unsigned char* vl = kl + kKBytes;
  const int col = lane & 31, half = lane >> 5;
  const int G = a.G, M = a.M, Hq = a.Hq, Hkv = a.Hkv;

  // ---- query fragments (B operand of S^T = K . Q^T) and the row's metadata ----
  bf16x8 qf[QT][8];
  int tq[QT], pidq[QT], boffq[QT], rowq[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = rb * (32 * QT) + qt * 32 + col;
    rowq[qt] = r;
    const int rr = min(r, M - 1);                 // rows past M are computed on a duplicate and never stored
    const int t = rr / G, hh = rr - t * G;
    const __bf16* qp = a.q + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[qt][s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s + 8 * half);
    const ouro_tok_meta mq = a.meta[static_cast<size_t>(b) * T + t];
    tq[qt] = t;
    pidq[qt] = mq.phrase_id;
    boffq[qt] = mq.branch_off;
  }

  // ---- staging: lane (kq = lane/16, c16 = lane%16) loads 16 B of 8 key rows per tile ----
  // Row order inside the tile is chosen so that the 8 rows of a lane are exactly one key
  // group of the P.V contraction: rows 16*(kq/2) + 8*jj + 4*(kq%2) + r, i = 4*jj + r.
  const int kq = lane >> 4, c16 = lane & 15;
  const int row_base = 16 * (kq >> 1) + 4 * (kq & 1);
  u32x4 kr[8], vr[8];
#define OURO_ATTN_ISSUE_LOADS(TILE)                                                                              \
  {                                                                                                              \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                              \
      const int kidx = min((TILE) + row_base + 8 * (i >> 2) + (i & 3), n - 1); /* clamp: finite data, masked */  \
      const bool in_cache = kidx < L;                                                                            \
      const size_t row = in_cache ? static_cast<size_t>(cu0 + kidx) : static_cast<size_t>(b) * T + (kidx - L);   \
      const size_t off = (row * Hkv + g) * kD + 8 * c16;                                                         \
      kr[i] = *reinterpret_cast<const u32x4*>((in_cache ? a.k_cache : a.k_blk) + off);                           \
      vr[i] = *reinterpret_cast<const u32x4*>((in_cache ? a.v_cache : a.v_blk) + off);                           \
    }                                                                                                            \
  }

  f32x16 o[QT][4];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qt][dt][i] = 0.f;
  }

  OURO_ATTN_ISSUE_LOADS(k_begin)
  for (int tile = k_begin; tile < k_end; tile += 32) {
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
    if (tile + 32 < k_end) OURO_ATTN_ISSUE_LOADS(tile + 32)
    wave_lds_fence();

    // ---- S^T = K . Q^T ----
    f32x16 sacc[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[qt][i] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kl + k_slot(col, 2 * s + half) * 16);
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) sacc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qt][s], sacc[qt], 0, 0, 0);
    }

    // ---- mask + online softmax (log2 domain).  Register i of a lane is key 8*(i/4) + 4*half + i%4 ----
    const bool need_mask = tile + 32 > L;          // tile touches block keys or runs past n (wave-uniform)
    int pidk[16];
    if (need_mask) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int kb = tile + 8 * (i >> 2) + 4 * half + (i & 3) - L;
        pidk[i] = (kb >= 0 && kb < T) ? a.meta[static_cast<size_t>(b) * T + kb].phrase_id : 0;
      }
    }
    bf16x8 pf[QT][2];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float tmax = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float s = sacc[qt][i] * a.scale_log2;
        if (need_mask) {
          const int kb = tile + 8 * (i >> 2) + 4 * half + (i & 3) - L;
          const bool vis = kb < 0 || (kb < T && (pidk[i] == 0 ? kb <= boffq[qt] : (pidk[i] == pidq[qt] && kb <= tq[qt])));
          s = vis ? s : -INFINITY;
        }
        sacc[qt][i] = s;
        tmax = fmaxf(tmax, s);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m_run[qt], tmax);
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = exp2f(m_run[qt] - m_safe);
      m_run[qt] = m_new;
      float psum = 0.f;
      f32x8 p0, p1;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        p0[i] = exp2f(sacc[qt][i] - m_safe);
        p1[i] = exp2f(sacc[qt][8 + i] - m_safe);
        psum += p0[i] + p1[i];
      }
      l_run[qt] = l_run[qt] * alpha + psum;         // per-half partial sum; halves are added at the end
      pf[qt][0] = __builtin_convertvector(p0, bf16x8);
      pf[qt][1] = __builtin_convertvector(p1, bf16x8);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[qt][dt][i] *= alpha;
    }

    // ---- O^T += V^T . P^T ----
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        const bf16x8 vf =
            *reinterpret_cast<const bf16x8*>(vl + vt_slot(4 * dt + (col >> 3), col & 7, 2 * s + half) * 16);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][s], o[qt][dt], 0, 0, 0);
      }
    }
    wave_lds_fence();                               // reads of this tile precede the next tile's LDS writes
  }

#undef OURO_ATTN_ISSUE_LOADS

  // ---- epilogue ----
  const int group = bg * a.nrb + rb;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float l_tot = l_run[qt] + __shfl_xor(l_run[qt], 32);
    const int r = rowq[qt];
    if (r >= M) continue;
    const int t = tq[qt], hh = r - t * G;
    if (a.nch == 1) {
      const float inv = 1.0f / l_tot;
      __bf16* op = a.out + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int ig = 0; ig < 4; ++ig) {
          f32x4 v4 = {o[qt][dt][4 * ig + 0] * inv, o[qt][dt][4 * ig + 1] * inv, o[qt][dt][4 * ig + 2] * inv,
                      o[qt][dt][4 * ig + 3] * inv};
          *reinterpret_cast<bf16x4*>(op + 32 * dt + 8 * ig + 4 * half) = __builtin_convertvector(v4, bf16x4);
        }
      if (a.lse && half == 0)
        a.lse[(static_cast<size_t>(b) * Hq + g * G + hh) * T + t] = (m_run[qt] + log2f(l_tot)) * 0.6931471805599453f;
    } else {
      const size_t prow = (static_cast<size_t>(group) * a.nch + chunk) * (32 * QT) + qt * 32 + col;
      float* po = a.part_o + prow * kD;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int ig = 0; ig < 4; ++ig) {
          f32x4 v4 = {o[qt][dt][4 * ig + 0], o[qt][dt][4 * ig + 1], o[qt][dt][4 * ig + 2], o[qt][dt][4 * ig + 3]};
          *reinterpret_cast<f32x4*>(po + 32 * dt + 8 * ig + 4 * half) = v4;
        }
      if (half == 0) {
        f32x2 ml = {m_run[qt], l_tot};
        *reinterpret_cast<f32x2*>(a.part_ml + prow * 2) = ml;
      }
    }
  }
}

// Merge the chunk partials of one query row: out = sum_c 2^(m_c - m*) O_c / sum_c 2^(m_c - m*) l_c,
// chunks visited in ascending order.  One wave per row, lane <-> two head-dim elements.
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a, int rows_wave) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long w = static_cast<long>(blockIdx.x) * 4 + wave;
  const long n_rows = static_cast<long>(a.n_items / a.nch) * rows_wave;   // groups * rows_wave
  if (w >= n_rows) return;
  const int row = static_cast<int>(w % rows_wave);
  const int group = static_cast<int>(w / rows_wave);
  const int rb = group % a.nrb, bg = group / a.nrb;
  const int b = bg / a.Hkv, g = bg - b * a.Hkv;
  const int r = rb * rows_wave + row;
  if (r >= a.M) return;
  const int n = static_cast<int>(a.cu[b + 1] - a.cu[b]) + a.T;
  const int nchb = (n + a.chunk - 1) / a.chunk;
  const size_t base = static_cast<size_t>(group) * a.nch * rows_wave + row;
  float m_star = -INFINITY;
  for (int c = 0; c < nchb; ++c) m_star = fmaxf(m_star, a.part_ml[(base + static_cast<size_t>(c) * rows_wave) * 2]);
  float lsum = 0.f;
  f32x2 acc = {0.f, 0.f};
  for (int c = 0; c < nchb; ++c) {
    const size_t prow = base + static_cast<size_t>(c) * rows_wave;
    const f32x2 ml = *reinterpret_cast<const f32x2*>(a.part_ml + prow * 2);
    const float wgt = exp2f(ml[0] - m_star);
    lsum += wgt * ml[1];
    const f32x2 po = *reinterpret_cast<const f32x2*>(a.part_o + prow * kD + 2 * lane);
    acc[0] += wgt * po[0];
    acc[1] += wgt * po[1];
  }
  const int t = r / a.G, hh = r - t * a.G;
  const float inv = 1.0f / lsum;
  f32x2 res = {acc[0] * inv, acc[1] * inv};
  __bf16* op = a.out + ((static_cast<size_t>(b) * a.T + t) * a.Hq + g * a.G + hh) * kD;
  *reinterpret_cast<bf16x2*>(op + 2 * lane) = __builtin_convertvector(res, bf16x2);
  if (a.lse && lane == 0)
    a.lse[(static_cast<size_t>(b) * a.Hq + g * a.G + hh) * a.T + t] = (m_star + log2f(lsum)) * 0.6931471805599453f;
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
  a.part_o = static_cast<float*>(d.workspace);
  a.part_ml = reinterpret_cast<float*>(static_cast<unsigned char*>(d.workspace) + plan.part_o_bytes);
  a.T = d.T;
  a.Hq = d.Hq;
  a.Hkv = d.Hkv;
  a.G = d.Hq / d.Hkv;
  a.M = d.T * a.G;
  a.nrb = plan.nrb;
  a.nch = plan.nch;
  a.chunk = plan.chunk;
  a.n_items = static_cast<long>(d.B) * d.Hkv * plan.nrb * plan.nch;
  a.scale_log2 = scale * 1.4426950408889634f;
  const unsigned grid = static_cast<unsigned>((a.n_items + 3) / 4);
  if (plan.qt == 2) hipLaunchKernelGGL(attn_bf16_kernel<2>, dim3(grid), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(attn_bf16_kernel<1>, dim3(grid), dim3(256), 0, stream, a);
  int st = check_launch();
  if (st != OURO_OK || plan.nch == 1) return st;
  const long n_rows = static_cast<long>(d.B) * d.Hkv * plan.nrb * plan.rows_wave;
  hipLaunchKernelGGL(attn_combine_kernel, dim3(static_cast<unsigned>((n_rows + 3) / 4)), dim3(256), 0, stream, a,
                     plan.rows_wave);
  return check_launch();
}

}  // namespace ouro
