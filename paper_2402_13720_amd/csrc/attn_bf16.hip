// bf16 draft-block attention for gfx950: split-KV flash-style kernels.
//
// What is computed (Sec. 3.2, Eq. (8)): every block row attends to the whole cached prefix
// of its sequence plus the block tokens of its own lengthened draft.  The block part of the
// mask is evaluated from per-token (phrase_id, branch_off) pairs (per query row a 128-bit set of
// the block keys it sees, formed once from a small LDS table of key classes); only the key tiles
// that overlap the block (the last T keys) pay for it, cache tiles are mask-free.
//
// Three kernels share the tile building blocks below: attn_bf16_kernel (the waves of a workgroup
// split the keys; described next), attn_bf16_rows8_kernel (eight waves, 128 query rows: the waves
// split rows and keys and share the staged tiles) and its four-wave predecessor
// attn_bf16_rows_kernel (each described where it is defined).  Workgroups take sequences by
// length rank (sequence_at), and K/V that only one workgroup reads is loaded with the
// non-temporal hint (kStreamKV).
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
// the 4 wave states (O, running max, running sum) go row-major to LDS once; every thread then
// folds the four states of its 4 output floats and writes them with a coalesced 16-byte (fp32
// partial) or 8-byte (bf16 output) store.  A sequence that spans several
// chunks leaves one fp32 partial per workgroup, and a second small kernel merges the partials
// of a row in ascending chunk order (deterministic) and writes bf16.  (A single-launch variant
// in which the last workgroup of a row block merged the partials was measured slower: the
// device-scope store/ticket/load round trips stall every workgroup for several microseconds.)
//
// Workgroup ids are mapped so that workgroups reading the same K/V window (different row
// blocks) are congruent modulo 8, i.e. land on the same XCD and share its L2.
#include <math.h>

#include <algorithm>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
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
  const int32_t* len;  // cached tokens per sequence, or null: the regions given by cu are packed
  unsigned kv_row_stride;   // cache addressing, in elements: row r of KV head g starts at r * kv_row_stride +
  size_t kv_head_stride;    // g * kv_head_stride ([rows, Hkv, D]: Hkv*D and D; [Hkv, rows, D]: D and rows*D)
  const ouro_tok_meta* meta;
  __bf16* out;
  float* lse;
  float* part_ml;      // [group][chunk][rows_wg][2]
  float* part_o;       // [group][chunk][rows_wg][128]
  int n_x;             // B * Hkv * nch
  int T, Hq, Hkv, G, M;
  int nrb, nch, chunk;
  int rows_wg;         // query rows per workgroup (32 x row blocks per workgroup)
  int nbg;             // B * Hkv
  FastDiv div_per, div_nbg, div_hkv, div_g, div_nrb, div_chunk;   // by 8 * nrb, B * Hkv, Hkv, G, nrb, chunk
  int B;               // sequences
  int round_seqs;      // sequences whose workgroups of one chunk index fill the chip once (>= 1): see sequence_at
  int max_seqlen;      // the host's bound on every length: grid, chunk slots and workspace were sized from it, so a
                       // longer device-side length is cut to it (a stale bound must not reach past any of them)
  float scale_log2;
};

constexpr int cmax(int x, int y) { return x > y ? x : y; }

constexpr int kRows = 32;                                  // query rows per workgroup
constexpr int kQBytes = kRows * 256;                       // Q tile shared by the 4 waves, same swizzle as the K tile
constexpr int kStateBytes = 16 * 64 * 16;                  // O accumulators of one wave, lane-major
constexpr int kMergeBytes = 4 * kRows * (kStageRow * 4 + 8);   // the four wave states, row-major, + their (max, sum) pairs
constexpr int kClassBytes = 128 * 16;                      // per phrase id 0..127: 128-bit set of the block keys that carry it
constexpr int kMainLds = cmax(kQBytes + 4 * kWaveLds, kMergeBytes);   // the merge reuses the tiles' space
constexpr int kLdsBytes = kMainLds + kClassBytes;          // 74 KB: two workgroups per CU

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

// Maximum over the two 32-lane halves of the wave (lanes l and l ^ 32), returned in both: one register swap between the
// halves on the vector ALU (v_permlane32_swap) instead of a round trip through the LDS crossbar, which sat in the
// dependent chain of every tile (scores -> maximum -> exponentials).
__device__ __forceinline__ float max_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// ---- which sequence a workgroup takes ---------------------------------------------------------------------------------
// Workgroups are handed to compute units in id order, and a compute unit's share of the memory system is bounded, so
// with sequences of unequal length the launch ends with the compute units that happened to draw the long ones while the
// rest idle (batched workload: 238 us in batch order against 216-220 us in any length-sorted order).  So position p
// of the dispatch order is not sequence p but the sequence whose length has a given rank (longest first; ties by index):
// ranks in descending order, except that the second chip-filling round runs backwards when two rounds are resident at
// once (kSnake: the key-split kernel has two workgroups per compute unit, and the unit that drew the longest of the
// first round then gets the shortest of the second).  Every wave ranks the lengths for itself, one sequence per lane
// (four per lane from 65 to 256 sequences; beyond that, and for a single sequence, positions are sequences).  The result
// is uniform.
template <bool kSnake>
__device__ __forceinline__ int sequence_at(const AttnArgs& a, int pos, int lane) {
  const int B = a.B;
  if (B < 2 || B > 256) return pos;
  const int rs = a.round_seqs;
  const int round = pos / rs, j = pos - round * rs;
  const int m = min(rs, B - round * rs);          // sequences of this round
  const int want = round * rs + ((kSnake && round == 1) ? m - 1 - j : j);
  auto length = [&](int i) {
    return i < B ? min(a.len ? a.len[i] : static_cast<int>(a.cu[i + 1] - a.cu[i]), a.max_seqlen) : -1;
  };
  if (B <= 64) {
    const int li = length(lane);
    int rank = 0;                                 // sequences ahead of this lane's: longer, or as long with a lower index
    for (int k = 0; k < B; ++k) {
      const int v = __builtin_amdgcn_readlane(li, k);
      rank += (v > li || (v == li && k < lane)) ? 1 : 0;
    }
    const unsigned long long hit = __ballot(lane < B && rank == want);
    return hit ? __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(hit)) - 1) : pos;
  }
  // 65 .. 256 sequences: four per lane (sequence lane + 64 q), the same count against every other length
  int li[4], rank[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    li[q] = length(lane + 64 * q);
    rank[q] = 0;
  }
#pragma unroll
  for (int qq = 0; qq < 4; ++qq) {
    const int nk = min(64, B - 64 * qq);
    for (int kk = 0; kk < nk; ++kk) {
      const int v = __builtin_amdgcn_readlane(li[qq], kk);
      const int k = 64 * qq + kk;
#pragma unroll
      for (int q = 0; q < 4; ++q) rank[q] += (v > li[q] || (v == li[q] && k < lane + 64 * q)) ? 1 : 0;
    }
  }
  int b = pos;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const unsigned long long hit = __ballot(lane + 64 * q < B && rank[q] == want);
    if (hit) b = 64 * q + __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(hit)) - 1);
  }
  return b;
}

// ---- the block part of the mask as bit sets ----------------------------------------------------------------------
// Row q sees block key k iff  pid[k] == 0 ? k <= boff[q] : (pid[k] == pid[q] && k <= q)  (Eq. (2) / Eq. (8)).  Per
// workgroup, a small LDS table holds for every phrase id the 128-bit set of block keys that carry it (built with one
// LDS atomic per key); a lane then forms the set its own query row sees with a few word operations,
//   vis = class[0] & low(boff_q + 1)  |  (pid_q != 0 ? class[pid_q] & low(q + 1) : 0),
// once, and a tile step that touches block keys masks its 16 scores with bit tests on a 32-bit window of that set:
// no memory access and no data-dependent branch per score.
__device__ __forceinline__ u32x4 low_bits(int n) {        // the n lowest of 128 bits (n <= 0: none; n >= 128: all)
  u32x4 r;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int m = n - 32 * w;
    r[w] = m >= 32 ? ~0u : m <= 0 ? 0u : ((1u << m) - 1u);
  }
  return r;
}
__device__ __forceinline__ u32x4 row_visibility(const u32x4* cls, int pidq, int boffq, int tq) {
  u32x4 vis = cls[0] & low_bits(boffq + 1);
  const u32x4 own = cls[pidq & 127] & low_bits(tq + 1);
  if (pidq != 0) vis |= own;
  return vis;
}
// Scores S (accumulator layout: register i of a lane of half h holds key 16*((i/4)%2) + 4*(i%4) + 2*(i/8) + h of the
// tile) of the tile at key TILE: keys before the block are cached tokens, visible to every row; block key kb is bit kb
// of vis; keys past the block are not there.  [32 ones | vis | zeros] shifted to the tile's first key is the window.
#define OURO_ATTN_MASK_TILE(TILE, S)                                                                               \
  if ((TILE) + 32 > L) {                                                                                           \
    const int e_ = (TILE) - L + 32;               /* >= 1; wave-uniform */                                         \
    const int wi_ = e_ >> 5;                                                                                       \
    const unsigned lo_ = wi_ == 0 ? ~0u : wi_ == 1 ? vis.x : wi_ == 2 ? vis.y : wi_ == 3 ? vis.z : wi_ == 4 ? vis.w : 0u; \
    const unsigned hi_ = wi_ == 0 ? vis.x : wi_ == 1 ? vis.y : wi_ == 2 ? vis.z : wi_ == 3 ? vis.w : 0u;           \
    const unsigned win_ = __builtin_amdgcn_alignbit(hi_, lo_, static_cast<unsigned>(e_ & 31)) >> half;             \
    _Pragma("unroll") for (int i = 0; i < 16; ++i)                                                                 \
        S[i] = (win_ & (1u << (16 * ((i >> 2) & 1) + 4 * (i & 3) + 2 * (i >> 3)))) ? S[i] : -INFINITY;             \
  }

// ---- building blocks shared by the two kernels (macros rather than functions: the register arrays they
// ---- work on must stay in registers) ---------------------------------------------------------------------
// Names they expect in scope: a, b, g, T, L, k_end, fast_end, cu0, Hkv, kq, c16, row_base, loff0, kstride (staging);
// col, half, o, m_run, l_run (the wave's flash state); vis (the block keys this lane's query row sees, one bit per key).

// Issue the global loads of the 32-key tile that starts at key TILE of the sequence's [cache | block] axis into
// the staging registers (8 K loads, then 8 V loads: always, so that counted waits stay exact); a tile wholly
// inside the cache part of the workgroup's window takes the fast path, any other has its keys clamped into the window.
// kStreamKV (a compile-time flag of the kernel): the cache is read with the non-temporal hint.  When every K/V byte is
// read by exactly one workgroup (one row-block group per KV head) nothing is gained by keeping it in L2, and
// lines that are not retained leave the cache to what is re-read (batched workload: 216 -> 192 us); when several row
// blocks read the same window the second reader must find it in L2, and the hint costs 2-3 us.
#define OURO_ATTN_ISSUE_HALF(TILE, REG, CACHE, BLK)                                                                 \
  if ((TILE) + 32 <= fast_end) {                                                                                   \
    const __bf16* src = (CACHE) + static_cast<size_t>(cu0 + (TILE)) * kstride + g * a.kv_head_stride;              \
    _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                                  \
        REG[i] = kStreamKV ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + loff0 + static_cast<unsigned>(4 * i) * kstride)) \
                           : *reinterpret_cast<const u32x4*>(src + loff0 + static_cast<unsigned>(4 * i) * kstride); \
  } else {                                                                                                         \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                \
      const int kidx = min((TILE) + 4 * i + kq, k_end - 1); /* clamp: finite data, masked or unused later */       \
      const bool in_cache = kidx < L;                                                                              \
      const size_t off = in_cache ? static_cast<size_t>(cu0 + kidx) * kstride + g * a.kv_head_stride               \
                                  : ((static_cast<size_t>(b) * T + (kidx - L)) * Hkv + g) * kD;                    \
      REG[i] = *reinterpret_cast<const u32x4*>((in_cache ? (CACHE) : (BLK)) + off + 8 * c16);                      \
    }                                                                                                              \
  }
#define OURO_ATTN_ISSUE_K(TILE, KR) OURO_ATTN_ISSUE_HALF(TILE, KR, a.k_cache, a.k_blk)
#define OURO_ATTN_ISSUE_V(TILE, VR) OURO_ATTN_ISSUE_HALF(TILE, VR, a.v_cache, a.v_blk)
#define OURO_ATTN_ISSUE_LOADS(TILE, KR, VR) OURO_ATTN_ISSUE_K(TILE, KR) OURO_ATTN_ISSUE_V(TILE, VR)

// Staging registers -> one K tile (row-major, swizzled) and one V^T tile (transposed with byte permutes;
// head-dim elements 8*c16 + j, j = J0..J1-1: 8 keys of one element are dword j/2, low or high half, of each row).
#define OURO_ATTN_STORE_K(KL, KR)                                                                                  \
  _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                                    \
      *reinterpret_cast<u32x4*>((KL) + k_slot(row_base + 8 * (i >> 2) + (i & 3), c16) * 16) = KR[i];
#define OURO_ATTN_STORE_V(VL, VR, J0, J1)                                                                          \
  _Pragma("unroll") for (int j = (J0); j < (J1); ++j) {                                                            \
    const unsigned sel = (j & 1) ? 0x07060302u : 0x05040100u;                                                      \
    u32x4 t4;                                                                                                      \
    t4.x = __builtin_amdgcn_perm(dword_of(VR[1], j >> 1), dword_of(VR[0], j >> 1), sel);                           \
    t4.y = __builtin_amdgcn_perm(dword_of(VR[3], j >> 1), dword_of(VR[2], j >> 1), sel);                           \
    t4.z = __builtin_amdgcn_perm(dword_of(VR[5], j >> 1), dword_of(VR[4], j >> 1), sel);                           \
    t4.w = __builtin_amdgcn_perm(dword_of(VR[7], j >> 1), dword_of(VR[6], j >> 1), sel);                           \
    *reinterpret_cast<u32x4*>((VL) + vt_slot(c16, j, kq) * 16) = t4;                                               \
  }
#define OURO_ATTN_STORE_TILE(KL, VL, KR, VR) { OURO_ATTN_STORE_K(KL, KR) OURO_ATTN_STORE_V(VL, VR, 0, 8) }

// One 32-row x 32-key step of the flash loop on the tile in (KL, VL) with the query tile in QL.
//
// S^T = K . Q^T; then the mask, only on tiles that touch block keys or run past n (wave-uniform branch):
// accumulator register i of a lane (half h) is S^T row 8*(i/4) + 4*h + i%4, which holds key
// 16*((i/4)%2) + 4*(i%4) + 2*(i/8) + h of the tile.  The rule is Eq. (8) on (phrase id, branch offset) pairs:
// cache keys are visible to every row; a main-draft key up to the row's branch point; a phrase key only to
// later rows of the same phrase.  The phrase ids of the block keys come from a small LDS table.
//
// Online softmax in the log2 domain.  The running reference m_run is only raised when a score exceeds it by
// more than 8 (a factor 256, harmless in fp32 and for the bf16 rounding of P, which is relative); O and the
// sum stay consistent with whatever reference is in use, so the result is unchanged, and the 64-register
// rescale of O is skipped on almost every tile.  l_run is a per-half partial sum; halves are added at the end.
//
// O^T += V^T . P^T with P^T = the S^T accumulator registers rounded to bf16.
#define OURO_ATTN_KFRAG(KL, S) *reinterpret_cast<const bf16x8*>((KL) + k_slot(col, 2 * (S) + half) * 16)
#define OURO_ATTN_VFRAG(VL, DT, C) *reinterpret_cast<const bf16x8*>((VL) + vt_slot(4 * (DT) + (col >> 3), col & 7, (C)) * 16)
// Order of a tile step (two waves per SIMD and 256 registers each, so the fragment registers are few and the order in
// which LDS reads are issued decides how much of their latency the wave sits out): the (K, Q) fragment pairs of
// S^T = K . Q^T are read four k steps ahead of the MFMA that uses them (a rolling set of 8 fragment registers; read
// one pair at a time right before its MFMA, every MFMA of the chain waited for a full LDS round trip); the 8 V^T
// fragments are then read into the same registers before the softmax arithmetic, which hides their latency, so
// that the O^T += V^T . P^T MFMAs find their operands waiting.
#define OURO_ATTN_COMPUTE_TILE(TILE, KL, VL, QL)                                                                   \
  {                                                                                                                \
    f32x16 sacc;                                                                                                   \
    bf16x8 fr[8];                                                                                                  \
    _Pragma("unroll") for (int s = 0; s < 4; ++s) {                                                                \
      fr[2 * s] = OURO_ATTN_KFRAG(KL, s);                                                                          \
      fr[2 * s + 1] = OURO_ATTN_KFRAG(QL, s);                                                                      \
    }                                                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                                             \
    {                                                                                                              \
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};      \
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[0], fr[1], zero16, 0, 0, 0);                               \
    }                                                                                                              \
    _Pragma("unroll") for (int s = 1; s < 8; ++s) {                                                                \
      if (s + 3 < 8) {                                                                                             \
        fr[2 * ((s + 3) & 3)] = OURO_ATTN_KFRAG(KL, s + 3);                                                        \
        fr[2 * ((s + 3) & 3) + 1] = OURO_ATTN_KFRAG(QL, s + 3);                                                    \
      }                                                                                                            \
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[2 * (s & 3)], fr[2 * (s & 3) + 1], sacc, 0, 0, 0);         \
      __builtin_amdgcn_sched_barrier(0);                                                                           \
    }                                                                                                              \
    _Pragma("unroll") for (int dt = 0; dt < 4; ++dt) {                                                             \
      fr[2 * dt] = OURO_ATTN_VFRAG(VL, dt, half);                                                                  \
      fr[2 * dt + 1] = OURO_ATTN_VFRAG(VL, dt, 2 + half);                                                          \
    }                                                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                                             \
    OURO_ATTN_MASK_TILE(TILE, sacc)                                                                                \
    float tmax = sacc[0];                                                                                          \
    _Pragma("unroll") for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sacc[i]);                                    \
    tmax = max_across_halves(tmax) * a.scale_log2;                                                                 \
    if (__any(tmax > m_run + 8.0f)) {                                                                              \
      const float m_new = fmaxf(m_run, tmax);                                                                      \
      const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));                      \
      m_run = m_new;                                                                                               \
      l_run *= alpha;                                                                                              \
      _Pragma("unroll") for (int dt = 0; dt < 4; ++dt)                                                             \
          _Pragma("unroll") for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;                                        \
    }                                                                                                              \
    const float neg_m = m_run == -INFINITY ? 0.f : -m_run;                                                         \
    float psum = 0.f;                                                                                              \
    f32x8 p0, p1;                                                                                                  \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                \
      p0[i] = __builtin_amdgcn_exp2f(fmaf(sacc[i], a.scale_log2, neg_m));                                          \
      p1[i] = __builtin_amdgcn_exp2f(fmaf(sacc[8 + i], a.scale_log2, neg_m));                                      \
      psum += p0[i] + p1[i];                                                                                       \
    }                                                                                                              \
    l_run += psum;                                                                                                 \
    const bf16x8 pf0 = __builtin_convertvector(p0, bf16x8);                                                        \
    const bf16x8 pf1 = __builtin_convertvector(p1, bf16x8);                                                        \
    _Pragma("unroll") for (int dt = 0; dt < 4; ++dt) {                                                             \
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[2 * dt], pf0, o[dt], 0, 0, 0);                            \
      o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[2 * dt + 1], pf1, o[dt], 0, 0, 0);                        \
    }                                                                                                              \
  }


template <bool kStreamKV>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(AttnArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;

  // ---- workgroup id -> (x = (sequence, KV head, chunk), row block); same x => same id modulo 8 ----
  const int per = 8 * a.nrb;
  const int blk = fdiv(blockIdx.x, a.div_per), rem = blockIdx.x - blk * per;
  const int rb = rem >> 3;
  const int x = blk * 8 + (rem & 7);
  if (x >= a.n_x) return;
  // chunk-major: the (sequence, KV head) pairs of one chunk index are consecutive, so every XCD (id modulo 8)
  // sees all chunk indices; pair-major order would give the rarely populated late chunks to a few XCDs
  const int nbg = a.nbg;
  const int chunk = fdiv(x, a.div_nbg);
  const int bgpos = x - chunk * nbg;
  const int bpos = fdiv(bgpos, a.div_hkv), g = bgpos - bpos * a.Hkv;
  const int b = sequence_at<true>(a, bpos, threadIdx.x & 63);   // by length rank, not batch order
  const int bg = b * a.Hkv + g;
  const int T = a.T;
  const int col = lane & 31, half = lane >> 5;
  const int G = a.G, M = a.M, Hq = a.Hq, Hkv = a.Hkv;
  const int row0 = rb * kRows;

  // ---- prologue loads: all of them are issued before anything waits, so that the workgroup pays one memory
  // round trip, not one per item.  First the ones that need nothing but the workgroup's indices (the sequence's
  // offset and length, the phrase ids of the block keys, the Q tile, this lane's metadata): they are in flight
  // while the offset and length arrive, which the first tile's addresses then need.  (A workgroup whose chunk slot
  // lies beyond its sequence leaves right after; its few loads are in bounds and unused.)
  // (offset and length are fetched with vector loads, through an index the compiler cannot see is uniform: a scalar
  // load's result would have to be waited for at once, because the scalar registers it lands in are spilled)
  int vzero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
  const long cu0_v = a.cu[b + vzero];
  const int cu1_v = *reinterpret_cast<const int*>(a.cu + b + 1 + vzero);    // low word: a length fits 32 bits
  int len_v = 0;
  if (a.len) len_v = a.len[b + vzero];
  const short my_kpid = tid < T ? a.meta[static_cast<size_t>(b) * T + tid].phrase_id : static_cast<short>(0);
  u32x4 qreg[kRows * 16 / 256];                   // Q tile: 16 lanes per 256-byte row, 2 pieces per thread
#pragma unroll
  for (int u = 0; u < kRows * 16 / 256; ++u) {
    const int p = tid + 256 * u;
    const int row = p >> 4, c = p & 15;
    const int rr = min(row0 + row, M - 1);        // rows past M are computed on a duplicate and never stored
    const int t = fdiv(rr, a.div_g), hh = rr - t * G;
    qreg[u] = *reinterpret_cast<const u32x4*>(a.q + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD + 8 * c);
  }
  // this lane's query row (its column of S^T) and that row's metadata
  const int rq = min(row0 + col, M - 1);
  const int tq = fdiv(rq, a.div_g);
  const ouro_tok_meta mq = a.meta[static_cast<size_t>(b) * T + tq];
  __builtin_amdgcn_sched_barrier(0);              // keep the loads above ahead of the wait for the length below
  int c0lo = static_cast<int>(cu0_v), c0hi = static_cast<int>(cu0_v >> 32), c1lo = cu1_v;
  asm volatile("" : "+v"(c0lo), "+v"(c0hi), "+v"(c1lo), "+v"(len_v));   // first use of the loaded values: here, not earlier
  const long cu0 = (static_cast<long>(__builtin_amdgcn_readfirstlane(c0hi)) << 32) |
                   static_cast<unsigned>(__builtin_amdgcn_readfirstlane(c0lo));
  const int L = min(__builtin_amdgcn_readfirstlane(a.len ? len_v : c1lo - c0lo), a.max_seqlen);   // a length fits 32 bits

  const int n = L + T;
  const int k_begin = chunk * a.chunk;
  if (k_begin >= n) return;                       // chunk slot beyond this sequence (uniform for the workgroup)
  const int k_end = min(n, k_begin + a.chunk);
  const bool whole = n <= a.chunk;                // the sequence has one chunk: this workgroup sees every key
  const int fast_end = min(L, k_end);             // tiles that end by here lie wholly in the cache part of the window

  unsigned char* ql = lds;                        // Q tile, shared
  unsigned char* kl = lds + kQBytes + wave * kWaveLds;
  unsigned char* vl = kl + kKBytes;
  u32x4* cls = reinterpret_cast<u32x4*>(lds + kMainLds);      // per phrase id: the set of block keys that carry it
  if (tid < 128) cls[tid] = u32x4{0u, 0u, 0u, 0u};

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
  const unsigned kstride = a.kv_row_stride;        // elements between consecutive cache rows of one head
  const unsigned loff0 = static_cast<unsigned>(kq) * kstride + 8 * c16;
  // this wave's tiles: k_begin + 32*(wave + 4*i)
  int tile = k_begin + 32 * wave;
  if (tile < k_end) { OURO_ATTN_ISSUE_LOADS(tile, kr, vr) }
  // ---- Q tile and phrase-id table -> LDS (the Q tile is read back as the B operand of S^T = K . Q^T) ----
  __builtin_amdgcn_sched_barrier(0);              // keep the stores (and their waits) behind every load above
  f32x16 o[4];                                    // (cleared here: nothing that can wait stands before the first loads)
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  __syncthreads();                                // the class table is cleared
  if (tid < T) atomicOr(reinterpret_cast<unsigned*>(cls + (my_kpid & 127)) + (tid >> 5), 1u << (tid & 31));
#pragma unroll
  for (int u = 0; u < kRows * 16 / 256; ++u) {
    const int p = tid + 256 * u;
    *reinterpret_cast<u32x4*>(ql + k_slot(p >> 4, p & 15) * 16) = qreg[u];
  }
  __syncthreads();                                // Q tile and class table complete
  u32x4 vis = {0u, 0u, 0u, 0u};
  if (k_end > L) vis = row_visibility(cls, mq.phrase_id, mq.branch_off, tq);   // the window reaches block keys
  for (; tile < k_end; tile += 128) {
    OURO_ATTN_STORE_TILE(kl, vl, kr, vr)
    if (tile + 128 < k_end) { OURO_ATTN_ISSUE_LOADS(tile + 128, kr, vr) }
    wave_lds_fence();
    OURO_ATTN_COMPUTE_TILE(tile, kl, vl, ql)
    wave_lds_fence();                               // reads of this tile precede the next tile's LDS writes
  }

  // ---- merge of the 4 wave states.  Every wave leaves its state row-major in LDS (O rows of kStageRow floats,
  // one (max, sum) pair per row; the Q and K/V tiles are dead by now), then thread (row, c) folds the four
  // states of its 4 output floats in wave order, O = sum_w 2^(m_w - m*) O_w, and writes them straight to memory:
  // the normalised bf16 output when the workgroup saw every key of the sequence, else its fp32 partial.
  __syncthreads();                                // all waves are done with the tiles
  float* st_o = reinterpret_cast<float*>(lds);                                  // [4][kRows][kStageRow]
  float* st_ml = st_o + 4 * kRows * kStageRow;                                  // [4][kRows][2]
  {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    float* mine = st_o + (wave * kRows + col) * kStageRow;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 v4 = {o[dt][4 * ig + 0], o[dt][4 * ig + 1], o[dt][4 * ig + 2], o[dt][4 * ig + 3]};
        *reinterpret_cast<f32x4*>(mine + 32 * dt + 8 * ig + 4 * half) = v4;
      }
    if (half == 0) {
      st_ml[(wave * kRows + col) * 2 + 0] = m_run;
      st_ml[(wave * kRows + col) * 2 + 1] = l_tot;
    }
  }
  __syncthreads();

  const int group = bg * a.nrb + rb;
  const size_t pbase = (static_cast<size_t>(group) * a.nch + chunk) * kRows;
#pragma unroll
  for (int u = 0; u < kRows * 32 / 256; ++u) {
    const int p = tid + 256 * u;
    const int row = p >> 5, c = p & 31;
    float m_w[4], l_w[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      m_w[w] = st_ml[(w * kRows + row) * 2 + 0];
      l_w[w] = st_ml[(w * kRows + row) * 2 + 1];
    }
    const float m_star = fmaxf(fmaxf(m_w[0], m_w[1]), fmaxf(m_w[2], m_w[3]));
    const float m_safe = m_star == -INFINITY ? 0.f : m_star;
    float lsum = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = exp2f(m_w[w] - m_safe);       // a wave without keys has m = -inf, O = 0: factor 0
      lsum += f * l_w[w];
      acc += f * *reinterpret_cast<const f32x4*>(st_o + (w * kRows + row) * kStageRow + 4 * c);
    }
    if (whole) {
      // the workgroup saw every key of the sequence: normalise and write bf16
      const int r = row0 + row;
      if (r >= M) continue;
      const int t = fdiv(r, a.div_g), hh = r - t * G;
      __bf16* op = a.out + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
      *reinterpret_cast<bf16x4*>(op + 4 * c) = __builtin_convertvector(acc * (1.0f / lsum), bf16x4);
      if (a.lse && c == 0)
        a.lse[(static_cast<size_t>(b) * Hq + g * G + hh) * T + t] = (m_star + log2f(lsum)) * kLn2;
    } else {
      // several chunks: leave a partial for the combine kernel (plain coalesced stores, no waiting)
      *reinterpret_cast<f32x4*>(a.part_o + (pbase + row) * kD + 4 * c) = acc;
      if (c == 0) *reinterpret_cast<float2*>(a.part_ml + (pbase + row) * 2) = make_float2(m_star, lsum);
    }
  }
}

// ---- row-split variant: more than 32 query rows per (sequence, KV head) -------------------------------------
// With T*G > 32 rows (long drafts, grouped-query heads) the K/V window of a chunk is needed by several
// 32-row blocks.  Here the workgroup keeps RW of them (RW = 2 or 4) and its waves share the staged tiles:
// a stage is 128 keys = four 32-key tiles, one staged by each wave exactly as above, and wave (rw, kw) runs
// its row block rw over the tiles kw, kw + KW, ... of the stage (KW = 4 / RW key groups).  Staging work, K/V
// global loads and LDS writes per query row drop by RW.
//
// One wave per SIMD (the whole register file: Q fragments, K and V fragments, two score accumulators stay in
// registers), so nothing but the instruction order hides latency; it is pipelined by hand and pinned with
// scheduling barriers.  Two LDS stage buffers; while the waves compute on stage s,
//   * the staging registers (stage s+1, loaded during stage s-1) go to the other buffer, a piece per tile slot,
//   * each staging register is re-armed with stage s+2 as soon as it has been stored (the 64 KB of loads of a
//     stage would otherwise block every wave for the ~1000 cycles they need to pass the address pipeline),
// and one barrier ends the stage.  Inside a stage, per tile u:
//
//   staging piece | read V fragments(u) | mask, running maximum(u) | the S^T MFMAs of tile u+1 interleaved
//                 with the exponentials of tile u | read K fragments(u+2) | P.V MFMAs(u)
//
// Every wave issues its 16 loads per stage whether or not its tile exists (clamped addresses), so that the
// counted waits never drain the prefetch.  At the end the KW states of a row block are merged through LDS and
// the workgroup writes 32*RW rows.
#define OURO_ATTN_READ_KF(TK)                                                                                      \
  _Pragma("unroll") for (int s = 0; s < 8; ++s)                                                                    \
      kf[s] = *reinterpret_cast<const bf16x8*>((TK) + k_slot(col, 2 * s + half) * 16);
#define OURO_ATTN_READ_VF(TV)                                                                                      \
  _Pragma("unroll") for (int dt = 0; dt < 4; ++dt) {                                                               \
    vf[2 * dt] = *reinterpret_cast<const bf16x8*>((TV) + vt_slot(4 * dt + (col >> 3), col & 7, half) * 16);        \
    vf[2 * dt + 1] = *reinterpret_cast<const bf16x8*>((TV) + vt_slot(4 * dt + (col >> 3), col & 7, 2 + half) * 16); \
  }
#define OURO_ATTN_QK(S)                                                                                            \
  {                                                                                                                \
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};        \
    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[0], zero16, 0, 0, 0);                                    \
    _Pragma("unroll") for (int s = 1; s < 8; ++s) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], S, 0, 0, 0); \
  }
// mask + running-maximum update for the scores S of the tile at key TILE (see OURO_ATTN_COMPUTE_TILE) ...
#define OURO_ATTN_SOFTMAX_MAX(TILE, S)                                                                             \
  {                                                                                                                \
    OURO_ATTN_MASK_TILE(TILE, S)                                                                                   \
    float tmax = S[0];                                                                                             \
    _Pragma("unroll") for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, S[i]);                                       \
    tmax = max_across_halves(tmax) * a.scale_log2;                                                             \
    if (__any(tmax > m_run + 8.0f)) {                                                                              \
      const float m_new = fmaxf(m_run, tmax);                                                                      \
      const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));                      \
      m_run = m_new;                                                                                               \
      l_run *= alpha;                                                                                              \
      _Pragma("unroll") for (int dt = 0; dt < 4; ++dt)                                                             \
          _Pragma("unroll") for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;                                        \
    }                                                                                                              \
  }
// ... and the exponentials: leaves P^T (bf16) in pf0, pf1 and adds the row sums to l_run
#define OURO_ATTN_SOFTMAX_EXP(S)                                                                                   \
  {                                                                                                                \
    const float neg_m = m_run == -INFINITY ? 0.f : -m_run;                                                         \
    float psum = 0.f;                                                                                              \
    f32x8 p0, p1;                                                                                                  \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) {                                                                \
      p0[i] = __builtin_amdgcn_exp2f(fmaf(S[i], a.scale_log2, neg_m));                                             \
      p1[i] = __builtin_amdgcn_exp2f(fmaf(S[8 + i], a.scale_log2, neg_m));                                         \
      psum += p0[i] + p1[i];                                                                                       \
    }                                                                                                              \
    l_run += psum;                                                                                                 \
    pf0 = __builtin_convertvector(p0, bf16x8);                                                                     \
    pf1 = __builtin_convertvector(p1, bf16x8);                                                                     \
  }
#define OURO_ATTN_PV()                                                                                             \
  _Pragma("unroll") for (int dt = 0; dt < 4; ++dt) {                                                               \
    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * dt], pf0, o[dt], 0, 0, 0);                              \
    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * dt + 1], pf1, o[dt], 0, 0, 0);                          \
  }

template <int RW>
constexpr int rows_main_lds() {
  // two stage buffers; the merge slots and the staged output reuse the same memory from its start
  return cmax(2 * 4 * kWaveLds, cmax((4 / RW / 2) * RW * (kStateBytes + 64 * 8), 32 * RW * kStageRow * 4 + 32 * RW * 8));
}
template <int RW>
constexpr int rows_lds_bytes() { return rows_main_lds<RW>() + kClassBytes; }

template <int RW>
__global__ __launch_bounds__(256) void attn_bf16_rows_kernel(AttnArgs a) {
  constexpr bool kStreamKV = false;
  constexpr int KW = 4 / RW;                      // key groups
  constexpr int NT = 4 / KW;                      // tiles of a stage per wave
  constexpr int kRowsWg = 32 * RW;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int rw = wave % RW, kw = wave / RW;

  // ---- workgroup id -> (x = (sequence, KV head, chunk), row block); same x => same id modulo 8 ----
  const int per = 8 * a.nrb;
  const int blk = fdiv(blockIdx.x, a.div_per), rem = blockIdx.x - blk * per;
  const int rb = rem >> 3;
  const int x = blk * 8 + (rem & 7);
  if (x >= a.n_x) return;
  // chunk-major: the (sequence, KV head) pairs of one chunk index are consecutive, so every XCD (id modulo 8)
  // sees all chunk indices; pair-major order would give the rarely populated late chunks to a few XCDs
  const int nbg = a.nbg;
  const int chunk = fdiv(x, a.div_nbg);
  const int bgpos = x - chunk * nbg;
  const int bpos = fdiv(bgpos, a.div_hkv), g = bgpos - bpos * a.Hkv;
  const int b = sequence_at<false>(a, bpos, threadIdx.x & 63);   // by length rank, not batch order
  const int bg = b * a.Hkv + g;
  const int T = a.T;
  const int col = lane & 31, half = lane >> 5;
  const int G = a.G, M = a.M, Hq = a.Hq, Hkv = a.Hkv;
  const int row0 = rb * kRowsWg + 32 * rw;        // first row of this wave's block (may lie past M: duplicates)

  // ---- prologue loads that need nothing but the workgroup's indices, as in the kernel above: the sequence's offset
  // and length (vector loads; first use pinned below), the phrase ids of the block keys, this lane's metadata and its
  // Q fragments straight into registers.  They are in flight while the offset and length arrive.
  int vzero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
  const long cu0_v = a.cu[b + vzero];
  const int cu1_v = *reinterpret_cast<const int*>(a.cu + b + 1 + vzero);    // low word: a length fits 32 bits
  int len_v = 0;
  if (a.len) len_v = a.len[b + vzero];
  const short my_kpid = tid < T ? a.meta[static_cast<size_t>(b) * T + tid].phrase_id : static_cast<short>(0);
  const int rq = min(row0 + col, M - 1);          // rows past M are computed on a duplicate and never stored
  const int tq = fdiv(rq, a.div_g);
  const ouro_tok_meta mq = a.meta[static_cast<size_t>(b) * T + tq];
  bf16x8 qf[8], kf[8], vf[8], pf0, pf1;
  {
    const __bf16* qp = a.q + ((static_cast<size_t>(b) * T + tq) * Hq + g * G + (rq - tq * G)) * kD + 8 * half;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
  }
  __builtin_amdgcn_sched_barrier(0);              // keep the loads above ahead of the wait for the length below
  int c0lo = static_cast<int>(cu0_v), c0hi = static_cast<int>(cu0_v >> 32), c1lo = cu1_v;
  asm volatile("" : "+v"(c0lo), "+v"(c0hi), "+v"(c1lo), "+v"(len_v));   // first use of the loaded values: here, not earlier
  const long cu0 = (static_cast<long>(__builtin_amdgcn_readfirstlane(c0hi)) << 32) |
                   static_cast<unsigned>(__builtin_amdgcn_readfirstlane(c0lo));
  const int L = min(__builtin_amdgcn_readfirstlane(a.len ? len_v : c1lo - c0lo), a.max_seqlen);

  const int n = L + T;
  const int k_begin = chunk * a.chunk;
  if (k_begin >= n) return;                       // chunk slot beyond this sequence (uniform for the workgroup)
  const int k_end = min(n, k_begin + a.chunk);
  const bool whole = n <= a.chunk;                // the sequence has one chunk: this workgroup sees every key
  const int fast_end = min(L, k_end);             // tiles that end by here lie wholly in the cache part of the window

  constexpr int kStageBytes4 = 4 * kWaveLds;      // one stage: 4 x (K tile, V^T tile)
  u32x4* cls = reinterpret_cast<u32x4*>(lds + rows_main_lds<RW>());   // per phrase id: the set of block keys that carry it
  if (tid < 128) cls[tid] = u32x4{0u, 0u, 0u, 0u};

  const int kq = lane >> 4, c16 = lane & 15;      // staging roles, as in the kernel above
  const int row_base = 16 * (kq >> 1) + 4 * (kq & 1);
  u32x4 kr[8], vr[8];
  const unsigned kstride = a.kv_row_stride;        // elements between consecutive cache rows of one head
  const unsigned loff0 = static_cast<unsigned>(kq) * kstride + 8 * c16;

  f32x16 o[4], sacc[2];
  float m_run = -INFINITY, l_run = 0.f;

  // staging piece PH (0..3) of a stage: registers -> this wave's tile in the buffer at NB, re-armed with tile NEXT
#define OURO_ATTN_STAGING(PH, NB, NEXT)                                                                            \
  {                                                                                                                \
    unsigned char* nk_ = (NB) + wave * kWaveLds;                                                                   \
    if ((PH) == 0) { OURO_ATTN_STORE_K(nk_, kr) OURO_ATTN_ISSUE_K(NEXT, kr) }                                      \
    if ((PH) == 1) { OURO_ATTN_STORE_V(nk_ + kKBytes, vr, 0, 4) }                                                  \
    if ((PH) == 2) { OURO_ATTN_STORE_V(nk_ + kKBytes, vr, 4, 8) OURO_ATTN_ISSUE_V(NEXT, vr) }                      \
  }

  // prologue: stage 0 -> buffer 0, stage 1 in flight (every prologue load is issued before anything waits)
  OURO_ATTN_ISSUE_LOADS(k_begin + 32 * wave, kr, vr)
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)                  // (cleared here: nothing that can wait stands before the first loads)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  __syncthreads();                                // the class table is cleared
  if (tid < T) atomicOr(reinterpret_cast<unsigned*>(cls + (my_kpid & 127)) + (tid >> 5), 1u << (tid & 31));
  {
    unsigned char* kl = lds + wave * kWaveLds;
    OURO_ATTN_STORE_K(kl, kr)
    OURO_ATTN_ISSUE_K(k_begin + 128 + 32 * wave, kr)
    OURO_ATTN_STORE_V(kl + kKBytes, vr, 0, 8)
    OURO_ATTN_ISSUE_V(k_begin + 128 + 32 * wave, vr)
  }
  __syncthreads();
  u32x4 vis = {0u, 0u, 0u, 0u};
  if (k_end > L) vis = row_visibility(cls, mq.phrase_id, mq.branch_off, tq);   // the window reaches block keys

  int cur = 0;
  for (int sb = k_begin; sb < k_end; sb += 128, cur ^= 1) {
    const unsigned char* kv = lds + cur * kStageBytes4;         // the stage being computed
    unsigned char* nb = lds + (cur ^ 1) * kStageBytes4;         // the stage being filled
    const int next = sb + 256 + 32 * wave;                      // the tile this wave's registers are re-armed with
    const int t0 = sb + 32 * kw;                  // this wave's tiles of the stage: t0 + 32*KW*u, u = 0..NT-1
    if (t0 < k_end) {
      OURO_ATTN_READ_KF(kv + kw * kWaveLds)
      OURO_ATTN_QK(sacc[0])
      if (NT > 1 && t0 + 32 * KW < k_end) { OURO_ATTN_READ_KF(kv + (kw + KW) * kWaveLds) }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      const int tile = t0 + 32 * KW * u;
#pragma unroll
      for (int ph = u * (4 / NT); ph < (u + 1) * (4 / NT); ++ph) { OURO_ATTN_STAGING(ph, nb, next) }
      __builtin_amdgcn_sched_barrier(0);
      if (tile < k_end) {
        OURO_ATTN_READ_VF(kv + (kw + KW * u) * kWaveLds + kKBytes)
        OURO_ATTN_SOFTMAX_MAX(tile, sacc[u & 1])
        __builtin_amdgcn_sched_barrier(0);
        // The S^T MFMAs of the next tile form a dependent chain; the exponentials of this tile are issued
        // between them (one MFMA, then a group of vector-ALU instructions), or the wave would sit through the
        // chain.  (Past the end of the chunk the fragments are stale and the scores unused.)
        if (u + 1 < NT) { OURO_ATTN_QK(sacc[(u + 1) & 1]) }
        OURO_ATTN_SOFTMAX_EXP(sacc[u & 1])
        if (u + 1 < NT) {
#pragma unroll
          for (int r = 0; r < 8; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);   // eight VALU
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (u + 2 < NT) { OURO_ATTN_READ_KF(kv + (kw + KW * (u + 2)) * kWaveLds) }
        OURO_ATTN_PV()
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();                              // stage sb fully read, stage sb+128 fully written
  }
#undef OURO_ATTN_STAGING

  // ---- merge the KW states of every row block through LDS ----
  unsigned char* scratch = lds;
  f32x4* slot_o = reinterpret_cast<f32x4*>(scratch);
  float* slot_ml = reinterpret_cast<float*>(scratch + (KW / 2) * RW * kStateBytes);
#pragma unroll
  for (int sft = KW / 2; sft >= 1; sft >>= 1) {
    if (kw >= sft && kw < 2 * sft) {
      const int slot = (kw - sft) * RW + rw;
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
    if (kw < sft) {
      const int slot = kw * RW + rw;
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
    __syncthreads();
  }

  // ---- the kw = 0 wave of every row block stages its state row-major: stage_o[row][132], stage_ml[row][2] ----
  float* stage_o = reinterpret_cast<float*>(scratch);
  float* stage_ml = stage_o + kRowsWg * kStageRow;
  if (kw == 0) {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const int lrow = 32 * rw + col;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 v4 = {o[dt][4 * ig + 0], o[dt][4 * ig + 1], o[dt][4 * ig + 2], o[dt][4 * ig + 3]};
        *reinterpret_cast<f32x4*>(stage_o + lrow * kStageRow + 32 * dt + 8 * ig + 4 * half) = v4;
      }
    if (half == 0) {
      stage_ml[lrow * 2 + 0] = m_run;
      stage_ml[lrow * 2 + 1] = l_tot;
    }
  }
  __syncthreads();

  const int group = bg * a.nrb + rb;
  if (whole) {
    // ---- the workgroup saw every key of the sequence: normalise and write bf16, 16 B per thread ----
    for (int p = tid; p < kRowsWg * 16; p += 256) {
      const int row = p >> 4, c = p & 15;
      const int r = rb * kRowsWg + row;
      if (r >= M) continue;
      const float inv = 1.0f / stage_ml[row * 2 + 1];
      const f32x4 x0 = *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 8 * c);
      const f32x4 x1 = *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 8 * c + 4);
      f32x8 v8 = {x0[0] * inv, x0[1] * inv, x0[2] * inv, x0[3] * inv, x1[0] * inv, x1[1] * inv, x1[2] * inv, x1[3] * inv};
      const int t = fdiv(r, a.div_g), hh = r - t * G;
      __bf16* op = a.out + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
      *reinterpret_cast<bf16x8*>(op + 8 * c) = __builtin_convertvector(v8, bf16x8);
      if (a.lse && c == 0)
        a.lse[(static_cast<size_t>(b) * Hq + g * G + hh) * T + t] =
            (stage_ml[row * 2] + log2f(stage_ml[row * 2 + 1])) * kLn2;
    }
    return;
  }

  // ---- several chunks: leave a partial for the combine kernel (coalesced streaming stores, no waiting: the 128-row
  // partials of a launch add up to many megabytes, and written as ordinary stores they sit dirty in L2 until the
  // kernels that follow evict them; measured 31.4 -> 28.6 us for this kernel at 128 rows x 40 heads x 6 chunks) ----
  const size_t pbase = (static_cast<size_t>(group) * a.nch + chunk) * kRowsWg;
  for (int p = tid; p < kRowsWg * 32; p += 256) {
    const int row = p >> 5, c = p & 31;
    __builtin_nontemporal_store(*reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 4 * c),
                                reinterpret_cast<f32x4*>(a.part_o + (pbase + row) * kD + 4 * c));
  }
  for (int p = tid; p < kRowsWg * 2; p += 256) a.part_ml[pbase * 2 + p] = stage_ml[p];
}

// ---- row-split variant with eight waves: 128 query rows per workgroup, two waves per SIMD ---------------------------
// The four-wave kernel above has one wave per SIMD, and a single wave runs its scores -> softmax -> P.V chain one link
// at a time: while it is on the vector ALU the matrix pipe idles, and the other way round (a stage of 128 keys costs it
// about 4 x (512 MFMA + 900 vector-ALU + LDS) cycles).  Here the workgroup has eight waves under 256 registers each:
// wave (rw = wave % 4, kw = wave / 4) runs row block rw over tiles kw and kw + 2 of every four-tile stage, so each
// SIMD holds the two key groups of one row block and one wave's MFMAs overlap the other's softmax with no hand-made
// interleave.  To fit the registers the tile step is the key-split kernel's (Q tile in LDS, one rolling fragment
// set) and a wave stages half a tile: waves 0..3 the K part of tile `wave` of the next stage, waves 4..7 the V part
// of tile `wave - 4` (transposed), each re-armed at once with the stage after.  LDS: four Q tiles + two stage buffers =
// 160 KB; the class table of the mask lives in the second stage buffer until the first stage is written over it.
constexpr int kRows8Lds = 4 * kQBytes + 2 * 4 * kWaveLds;

template <bool kStreamKV>
__global__ __launch_bounds__(512, 1) void attn_bf16_rows8_kernel(AttnArgs a) {
  constexpr int RW = 4, KW = 2, kRowsWg = 32 * RW;
  constexpr int kStageBytes4 = 4 * kWaveLds;      // one stage: 4 x (K tile, V^T tile)
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int rw = wave & 3, kw = wave >> 2;
  const int st_tile = wave & 3;                   // staging role: part (K or V) of this tile of a stage
  const bool st_v = wave >= 4;

  // ---- workgroup id -> (x = (sequence, KV head, chunk), row block); same x => same id modulo 8 ----
  const int per = 8 * a.nrb;
  const int blk = fdiv(blockIdx.x, a.div_per), rem = blockIdx.x - blk * per;
  const int rb = rem >> 3;
  const int x = blk * 8 + (rem & 7);
  if (x >= a.n_x) return;
  const int nbg = a.nbg;
  const int chunk = fdiv(x, a.div_nbg);           // chunk-major, as in the kernels above
  const int bgpos = x - chunk * nbg;
  const int bpos = fdiv(bgpos, a.div_hkv), g = bgpos - bpos * a.Hkv;
  const int b = sequence_at<false>(a, bpos, threadIdx.x & 63);   // by length rank, not batch order
  const int bg = b * a.Hkv + g;
  const int T = a.T;
  const int col = lane & 31, half = lane >> 5;
  const int G = a.G, M = a.M, Hq = a.Hq, Hkv = a.Hkv;
  const int row0 = rb * kRowsWg + 32 * rw;        // first row of this wave's block (may lie past M: duplicates)

  // ---- prologue loads that need nothing but the workgroup's indices (see the key-split kernel) ----
  int vzero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
  const long cu0_v = a.cu[b + vzero];
  const int cu1_v = *reinterpret_cast<const int*>(a.cu + b + 1 + vzero);    // low word: a length fits 32 bits
  int len_v = 0;
  if (a.len) len_v = a.len[b + vzero];
  const short my_kpid = tid < T ? a.meta[static_cast<size_t>(b) * T + tid].phrase_id : static_cast<short>(0);
  u32x4 qreg[kRowsWg * 16 / 512];                 // the four Q tiles: 16 lanes per 256-byte row, 4 pieces per thread
#pragma unroll
  for (int u = 0; u < kRowsWg * 16 / 512; ++u) {
    const int p = tid + 512 * u;
    const int row = p >> 4, c = p & 15;
    const int rr = min(rb * kRowsWg + row, M - 1); // rows past M are computed on a duplicate and never stored
    const int t = fdiv(rr, a.div_g), hh = rr - t * G;
    qreg[u] = *reinterpret_cast<const u32x4*>(a.q + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD + 8 * c);
  }
  const int rq = min(row0 + col, M - 1);          // this lane's query row (its column of S^T) and that row's metadata
  const int tq = fdiv(rq, a.div_g);
  const ouro_tok_meta mq = a.meta[static_cast<size_t>(b) * T + tq];
  __builtin_amdgcn_sched_barrier(0);              // keep the loads above ahead of the wait for the length below
  int c0lo = static_cast<int>(cu0_v), c0hi = static_cast<int>(cu0_v >> 32), c1lo = cu1_v;
  asm volatile("" : "+v"(c0lo), "+v"(c0hi), "+v"(c1lo), "+v"(len_v));   // first use of the loaded values: here, not earlier
  const long cu0 = (static_cast<long>(__builtin_amdgcn_readfirstlane(c0hi)) << 32) |
                   static_cast<unsigned>(__builtin_amdgcn_readfirstlane(c0lo));
  const int L = min(__builtin_amdgcn_readfirstlane(a.len ? len_v : c1lo - c0lo), a.max_seqlen);

  const int n = L + T;
  const int k_begin = chunk * a.chunk;
  if (k_begin >= n) return;                       // chunk slot beyond this sequence (uniform for the workgroup)
  const int k_end = min(n, k_begin + a.chunk);
  const bool whole = n <= a.chunk;                // the sequence has one chunk: this workgroup sees every key
  const int fast_end = min(L, k_end);             // tiles that end by here lie wholly in the cache part of the window

  unsigned char* ql = lds + rw * kQBytes;         // this wave's Q tile
  unsigned char* stage0 = lds + 4 * kQBytes;      // two stage buffers
  u32x4* cls = reinterpret_cast<u32x4*>(stage0 + kStageBytes4);   // (in the second one, which the prologue leaves alone)
  if (tid < 128) cls[tid] = u32x4{0u, 0u, 0u, 0u};

  const int kq = lane >> 4, c16 = lane & 15;      // staging roles of the lanes, as in the kernels above
  const int row_base = 16 * (kq >> 1) + 4 * (kq & 1);
  u32x4 sr[8];
  const unsigned kstride = a.kv_row_stride;        // elements between consecutive cache rows of one head
  const unsigned loff0 = static_cast<unsigned>(kq) * kstride + 8 * c16;
  const __bf16* const s_cache = st_v ? a.v_cache : a.k_cache;
  const __bf16* const s_blk = st_v ? a.v_blk : a.k_blk;
  // this wave's half tile: registers -> the stage buffer at NB, re-armed with the tile at key NEXT
#define OURO_ATTN_STAGE_HALF(NB, NEXT)                                                                             \
  {                                                                                                                \
    unsigned char* nk_ = (NB) + st_tile * kWaveLds;                                                                \
    if (st_v) { OURO_ATTN_STORE_V(nk_ + kKBytes, sr, 0, 8) } else { OURO_ATTN_STORE_K(nk_, sr) }                   \
    OURO_ATTN_ISSUE_HALF(NEXT, sr, s_cache, s_blk)                                                                 \
  }

  OURO_ATTN_ISSUE_HALF(k_begin + 32 * st_tile, sr, s_cache, s_blk)
  __builtin_amdgcn_sched_barrier(0);
  f32x16 o[4];
  float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)                  // (cleared here: nothing that can wait stands before the first loads)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  __syncthreads();                                // the class table is cleared
  if (tid < T) atomicOr(reinterpret_cast<unsigned*>(cls + (my_kpid & 127)) + (tid >> 5), 1u << (tid & 31));
#pragma unroll
  for (int u = 0; u < kRowsWg * 16 / 512; ++u) {
    const int p = tid + 512 * u;
    *reinterpret_cast<u32x4*>(lds + (p >> 9) * kQBytes + k_slot((p >> 4) & 31, p & 15) * 16) = qreg[u];
  }
  OURO_ATTN_STAGE_HALF(stage0, k_begin + 128 + 32 * st_tile)   // stage 0 -> buffer 0, stage 1 in flight
  __syncthreads();                                // Q tiles, class table and stage 0 complete
  u32x4 vis = {0u, 0u, 0u, 0u};
  if (k_end > L) vis = row_visibility(cls, mq.phrase_id, mq.branch_off, tq);   // the window reaches block keys
  __syncthreads();                                // every lane has its set: the second buffer may be written

  int cur = 0;
  for (int sb = k_begin; sb < k_end; sb += 128, cur ^= 1) {
    const unsigned char* kv = stage0 + cur * kStageBytes4;      // the stage being computed
    unsigned char* nb = stage0 + (cur ^ 1) * kStageBytes4;      // the stage being filled
    OURO_ATTN_STAGE_HALF(nb, sb + 256 + 32 * st_tile)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int tile = sb + 32 * (kw + KW * u);
      if (tile < k_end) {
        const unsigned char* kl = kv + (kw + KW * u) * kWaveLds;
        OURO_ATTN_COMPUTE_TILE(tile, kl, kl + kKBytes, ql)
      }
    }
    __syncthreads();                              // stage sb fully read, stage sb+128 fully written
  }
#undef OURO_ATTN_STAGE_HALF

  // ---- merge the two key groups of every row block through LDS ----
  f32x4* slot_o = reinterpret_cast<f32x4*>(lds);
  float* slot_ml = reinterpret_cast<float*>(lds + RW * kStateBytes);
  if (kw == 1) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 v4 = {o[dt][4 * ig + 0], o[dt][4 * ig + 1], o[dt][4 * ig + 2], o[dt][4 * ig + 3]};
        slot_o[(rw * 16 + dt * 4 + ig) * 64 + lane] = v4;
      }
    slot_ml[(rw * 64 + lane) * 2 + 0] = m_run;
    slot_ml[(rw * 64 + lane) * 2 + 1] = l_run;
  }
  __syncthreads();
  if (kw == 0) {
    const float m_b = slot_ml[(rw * 64 + lane) * 2 + 0];
    const float l_b = slot_ml[(rw * 64 + lane) * 2 + 1];
    const float m_new = fmaxf(m_run, m_b);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float fa = exp2f(m_run - m_safe), fb = exp2f(m_b - m_safe);
    m_run = m_new;
    l_run = l_run * fa + l_b * fb;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        const f32x4 ob = slot_o[(rw * 16 + dt * 4 + ig) * 64 + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[dt][4 * ig + e] = o[dt][4 * ig + e] * fa + ob[e] * fb;
      }
  }
  __syncthreads();

  // ---- the kw = 0 wave of every row block stages its state row-major: stage_o[row][132], stage_ml[row][2] ----
  float* stage_o = reinterpret_cast<float*>(lds);
  float* stage_ml = stage_o + kRowsWg * kStageRow;
  if (kw == 0) {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const int lrow = 32 * rw + col;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int ig = 0; ig < 4; ++ig) {
        f32x4 v4 = {o[dt][4 * ig + 0], o[dt][4 * ig + 1], o[dt][4 * ig + 2], o[dt][4 * ig + 3]};
        *reinterpret_cast<f32x4*>(stage_o + lrow * kStageRow + 32 * dt + 8 * ig + 4 * half) = v4;
      }
    if (half == 0) {
      stage_ml[lrow * 2 + 0] = m_run;
      stage_ml[lrow * 2 + 1] = l_tot;
    }
  }
  __syncthreads();

  const int group = bg * a.nrb + rb;
  if (whole) {
    // ---- the workgroup saw every key of the sequence: normalise and write bf16, 16 B per thread ----
    for (int p = tid; p < kRowsWg * 16; p += 512) {
      const int row = p >> 4, c = p & 15;
      const int r = rb * kRowsWg + row;
      if (r >= M) continue;
      const float inv = 1.0f / stage_ml[row * 2 + 1];
      const f32x4 x0 = *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 8 * c);
      const f32x4 x1 = *reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 8 * c + 4);
      f32x8 v8 = {x0[0] * inv, x0[1] * inv, x0[2] * inv, x0[3] * inv, x1[0] * inv, x1[1] * inv, x1[2] * inv, x1[3] * inv};
      const int t = fdiv(r, a.div_g), hh = r - t * G;
      __bf16* op = a.out + ((static_cast<size_t>(b) * T + t) * Hq + g * G + hh) * kD;
      *reinterpret_cast<bf16x8*>(op + 8 * c) = __builtin_convertvector(v8, bf16x8);
      if (a.lse && c == 0)
        a.lse[(static_cast<size_t>(b) * Hq + g * G + hh) * T + t] =
            (stage_ml[row * 2] + log2f(stage_ml[row * 2 + 1])) * kLn2;
    }
    return;
  }

  // ---- several chunks: leave a partial for the combine kernel (coalesced streaming stores, no waiting: the 128-row
  // partials of a launch add up to many megabytes, and written as ordinary stores they sit dirty in L2 until the
  // kernels that follow evict them; measured 31.4 -> 28.6 us for this kernel at 128 rows x 40 heads x 6 chunks) ----
  const size_t pbase = (static_cast<size_t>(group) * a.nch + chunk) * kRowsWg;
  for (int p = tid; p < kRowsWg * 32; p += 512) {
    const int row = p >> 5, c = p & 31;
    __builtin_nontemporal_store(*reinterpret_cast<const f32x4*>(stage_o + row * kStageRow + 4 * c),
                                reinterpret_cast<f32x4*>(a.part_o + (pbase + row) * kD + 4 * c));
  }
  for (int p = tid; p < kRowsWg * 2; p += 512) a.part_ml[pbase * 2 + p] = stage_ml[p];
}

// Merge the chunk partials of every query row of the sequences that span several chunks:
// out = sum_c 2^(m_c - m*) O_c / sum_c 2^(m_c - m*) l_c, chunks folded in ascending order
// (deterministic).  One thread per (row, 8 head-dim elements); loads are issued four chunks
// at a time so that their latencies overlap.
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
  const int rows_wg = a.rows_wg;
  const long p = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
  const int c = static_cast<int>(p & 15);
  const long rowg = p >> 4;
  const int row = static_cast<int>(rowg & (rows_wg - 1));      // rows_wg is 32, 64 or 128
  const long group = rowg >> (rows_wg == 32 ? 5 : rows_wg == 64 ? 6 : 7);
  if (group >= static_cast<long>(a.nbg) * a.nrb) return;
  const int bg = fdiv(static_cast<int>(group), a.div_nrb);
  const int rb = static_cast<int>(group) - bg * a.nrb;
  const int b = fdiv(bg, a.div_hkv), g = bg - b * a.Hkv;
  const int r = rb * rows_wg + row;
  if (r >= a.M) return;
  const size_t gbase = static_cast<size_t>(group) * a.nch * rows_wg;
  float m_star = -INFINITY, lsum = 0.f;
  f32x8 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float m_c[4], l_c[4];
  f32x4 x0[4], x1[4];
  // `last` bounds the chunk index of a batch of four partial loads
  auto load4 = [&](int ch0, int last) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int ch = min(ch0 + u, last);
      const size_t prow = gbase + static_cast<size_t>(ch) * rows_wg + row;
      m_c[u] = a.part_ml[prow * 2];
      l_c[u] = a.part_ml[prow * 2 + 1];
      x0[u] = *reinterpret_cast<const f32x4*>(a.part_o + prow * kD + 8 * c);
      x1[u] = *reinterpret_cast<const f32x4*>(a.part_o + prow * kD + 8 * c + 4);
    }
  };
  auto merge4 = [&](int ch0, int nchb) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (ch0 + u >= nchb) continue;                  // slots past the sequence's chunks hold nothing
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
  };
  // The first batch is addressed without the sequence length (the workspace holds a.nch slots per
  // group, so every slot is readable), which puts its loads in flight together with the length's.
  load4(0, a.nch - 1);
  const int n = min(a.len ? a.len[b] : static_cast<int>(a.cu[b + 1] - a.cu[b]), a.max_seqlen) + a.T;
  const int nchb = fdiv(n + a.chunk - 1, a.div_chunk);   // <= a.nch: the length is cut to the bound a.nch was sized from
  if (nchb == 1) return;                            // written directly by the main kernel
  merge4(0, nchb);
  for (int ch0 = 4; ch0 < nchb; ch0 += 4) {
    load4(ch0, nchb - 1);
    merge4(ch0, nchb);
  }
  const float inv = 1.0f / lsum;
  const int t = fdiv(r, a.div_g), hh = r - t * a.G;
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
  a.len = d.seq_len;
  a.kv_row_stride = d.kv_layout == OURO_KV_HEAD_MAJOR ? kD : static_cast<unsigned>(d.Hkv) * kD;
  a.kv_head_stride = d.kv_layout == OURO_KV_HEAD_MAJOR ? static_cast<size_t>(d.cache_rows) * kD : kD;
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
  a.nbg = d.B * d.Hkv;
  a.div_per = make_fastdiv(8u * plan.nrb);
  a.div_nbg = make_fastdiv(static_cast<unsigned>(a.nbg));
  a.div_hkv = make_fastdiv(static_cast<unsigned>(d.Hkv));
  a.div_g = make_fastdiv(static_cast<unsigned>(a.G));
  a.div_nrb = make_fastdiv(static_cast<unsigned>(plan.nrb));
  a.div_chunk = make_fastdiv(static_cast<unsigned>(plan.chunk));
  a.scale_log2 = scale * 1.4426950408889634f;
  a.rows_wg = plan.rows_wg;
  a.max_seqlen = d.max_seqlen;
  a.B = d.B;
  a.round_seqs = std::max(1, 256 / (d.Hkv * plan.nrb));
  const unsigned grid = static_cast<unsigned>((a.n_x + 7) / 8) * 8u * plan.nrb;
  static DeviceOnce once;
  const int ready = device_once(once, [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_rows_kernel<2>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, rows_lds_bytes<2>());
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_rows_kernel<4>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, rows_lds_bytes<4>());
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_rows8_kernel<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kRows8Lds);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_rows8_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kRows8Lds);
    return e == hipSuccess ? static_cast<int>(OURO_OK) : hip_failed(e);
  });
  if (ready != OURO_OK) return ready;
  if (d.ev_start && hipEventRecord(static_cast<hipEvent_t>(d.ev_start), stream) != hipSuccess) return hip_failed(hipGetLastError());
  const bool stream_kv = plan.nrb == 1;            // every K/V byte is read by one workgroup only
  if (plan.rw == 4 && plan.waves == 8 && stream_kv)
    hipLaunchKernelGGL(attn_bf16_rows8_kernel<true>, dim3(grid), dim3(512), kRows8Lds, stream, a);
  else if (plan.rw == 4 && plan.waves == 8)
    hipLaunchKernelGGL(attn_bf16_rows8_kernel<false>, dim3(grid), dim3(512), kRows8Lds, stream, a);
  else if (plan.rw == 4)
    hipLaunchKernelGGL(attn_bf16_rows_kernel<4>, dim3(grid), dim3(256), rows_lds_bytes<4>(), stream, a);
  else if (plan.rw == 2)
    hipLaunchKernelGGL(attn_bf16_rows_kernel<2>, dim3(grid), dim3(256), rows_lds_bytes<2>(), stream, a);
  else if (stream_kv)
    hipLaunchKernelGGL(attn_bf16_kernel<true>, dim3(grid), dim3(256), kLdsBytes, stream, a);
  else
    hipLaunchKernelGGL(attn_bf16_kernel<false>, dim3(grid), dim3(256), kLdsBytes, stream, a);
  int st = check_launch();
  if (st == OURO_OK && d.ev_stop && hipEventRecord(static_cast<hipEvent_t>(d.ev_stop), stream) != hipSuccess)
    return hip_failed(hipGetLastError());
  if (st != OURO_OK || plan.nch == 1) return st;
  const long threads = static_cast<long>(d.B) * d.Hkv * plan.nrb * plan.rows_wg * 16;
  hipLaunchKernelGGL(attn_combine_kernel, dim3(static_cast<unsigned>((threads + 255) / 256)), dim3(256), 0, stream, a);
  return check_launch();
}

}  // namespace ouro
