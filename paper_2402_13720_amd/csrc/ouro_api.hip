// Host side of the C ABI: descriptor validation, launch planning, dispatch.
// Every check here runs before the first HIP call so that it works without a GPU.
#include <algorithm>
#include <cmath>
#include <cstdlib>

#include "ouro_internal.hpp"

namespace ouro {

static thread_local int g_last_hip_error = 0;

int hip_failed(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return OURO_E_HIP;
}

// Launch plan of the bf16 attention.  A workgroup streams `chunk` keys of one (sequence,
// KV head) for its query rows and, when the sequence spans several chunks, leaves one fp32
// partial.  Small chunks fill the 256 compute units; large chunks keep the partial traffic
// (rows * 512 bytes per workgroup) small against the K/V bytes of a chunk (chunk * 512 bytes).
//
// Up to 64 query rows per (sequence, KV head): one 32-row block per workgroup, the four waves split the
// keys ("key-split" kernel); the default aims at about 1.25 workgroups per compute unit (two are resident at a
// time; measured best where per-workgroup prologue/epilogue latency dominates).
// More rows (long drafts, grouped-query heads), two ways, chosen by a cost estimate fitted to measurements:
//  * the "row-split" kernel: the workgroup keeps 4 row blocks and its waves share the staged tiles; one workgroup
//    per compute unit, the chunk count the largest that still lets every workgroup be resident at once.  K/V crosses
//    from L2 to a compute unit once per 128 rows, but a workgroup has only ~64 KB in flight, and the many chunk
//    slots it needs to fill the chip leave several times the fp32 partials of the other plan for the merge launch
//    to read back: about 10 + 3.6 * stages microseconds (eight-wave kernel, merge included in the constant);
//  * the key-split kernel with one workgroup per 32-row block: every row block stages the K/V window again, so K/V
//    crosses L2 -> compute unit once per 32 rows (measured ~11 TB/s in aggregate), but two workgroups per compute
//    unit keep twice the bytes in flight and hide each other's latencies: about 6 + 0.095 us per MB of (row blocks x
//    K/V bytes).  It wins where the K/V of the launch is small and the row blocks few (a short cache, a few hundred
//    rows at most); at 64 query / 8 KV heads x 64 block tokens over 4096 cached tokens (16 row blocks) the two are
//    within 4 us of each other and the row-split kernel gives the shorter step (119.9 us against 121.0 us).
// The descriptor's plan_override (row blocks per workgroup, keys per chunk) replaces the estimate in tests and tuning.
AttnPlan plan_attn_bf16(const ouro_attn_desc& d) {
  AttnPlan p{};
  const int G = d.Hq / d.Hkv;
  const int M = d.T * G;
  const long maxn = static_cast<long>(d.max_seqlen) + d.T;
  const long tiles = (maxn + 31) / 32;
  const long stages = (tiles + 3) / 4;
  const long pairs = std::max<long>(1, static_cast<long>(d.B) * d.Hkv);       // (sequence, KV head) pairs
  // the row-split plan: workgroups, stages per workgroup
  const long groups4 = pairs * ((M + 127) / 128);
  const long want4 = std::max<long>(1, std::min(256 / groups4, stages));
  const long stages_wg4 = (stages + want4 - 1) / want4;
  p.rw = 1;
  if (M > 64) {
    const double kv_mb = 2.0 * static_cast<double>(maxn) * static_cast<double>(pairs) * 256.0 / 1.0e6;   // upper bound
    const double rounds4 = static_cast<double>((groups4 + 255) / 256);
    const double t_rows = 10.0 + 3.6 * static_cast<double>(stages_wg4) * rounds4;
    const double t_keys = 6.0 + 0.095 * kv_mb * static_cast<double>((M + 31) / 32);
    p.rw = t_keys < t_rows ? 1 : 4;                  // (2 is built as well; measured no faster than 1 at 64 rows)
  }
  const int rw_forced = d.plan_override & 0x7f;
  if (rw_forced == 1 || rw_forced == 2 || rw_forced == 4) p.rw = rw_forced;
  // four row blocks: the eight-wave kernel (two key groups per row block, two waves per SIMD) unless the four-wave one
  // (one wave per SIMD, pipelined by hand; kept for comparison) is asked for
  p.waves = (p.rw == 4 && !(d.plan_override & 0x80)) ? 8 : 4;
  p.rows_wg = 32 * p.rw;
  p.nrb = (M + p.rows_wg - 1) / p.rows_wg;
  const long groups = pairs * p.nrb;
  long tiles_per_chunk;
  if (p.rw == 1) {
    long want = ((M <= 64 ? 320 : 256) + groups - 1) / groups;   // chunk slots per sequence
    want = std::max<long>(1, std::min(want, (tiles + 3) / 4));
    tiles_per_chunk = ((tiles + want - 1) / want + 3) / 4 * 4;
  } else {
    const long resident = 256;                         // workgroups the chip holds at once (one per compute unit)
    const long want = std::max<long>(1, std::min(resident / groups, stages));
    tiles_per_chunk = (stages + want - 1) / want * 4;
  }
  const long chunk_forced = static_cast<long>(static_cast<unsigned>(d.plan_override) >> 8);   // in units of 128 keys
  if (chunk_forced >= 1) tiles_per_chunk = chunk_forced * 4;
  p.chunk = static_cast<int>(tiles_per_chunk * 32);
  p.nch = static_cast<int>((maxn + p.chunk - 1) / p.chunk);
  if (p.nch > 1) {
    const size_t slots = static_cast<size_t>(groups) * p.nch;
    p.part_ml_bytes = round_up(slots * p.rows_wg * 2 * sizeof(float), 256);
    p.part_o_bytes = round_up(slots * p.rows_wg * d.D * sizeof(float), 256);
  }
  return p;
}

LmPlan plan_lmhead(const ouro_lmhead_desc& d) {
  LmPlan p{};
  if (d.dtype == OURO_F32) {
    p.variant = 0;
    p.slab = 8;                                      // two vocabulary rows per wave: many short workgroups (the path is latency-bound)
    p.rtile = 1024;
  } else if (d.R <= 64) {
    p.variant = 1;
    p.slab = 128;
    p.rtile = 64;
  } else if (d.R <= 128) {
    p.variant = 2;
    p.slab = 128;
    p.rtile = 128;
  } else {
    p.variant = 3;                                   // MFMA-bound: 256 x 256 workgroup tiles
    p.slab = 256;
    p.rtile = 256;
  }
  p.nslab = (d.V + p.slab - 1) / p.slab;
  p.nrtile = (d.R + p.rtile - 1) / p.rtile;
  p.part_bytes = round_up(static_cast<size_t>(p.nslab) * std::max(d.R, 1) * 8, 256);
  return p;
}

static int validate_attn(const ouro_attn_desc* d, bool need_pointers) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_attn_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_F32 && d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->B < 0 || d->B > 65535 || d->T < 1 || d->T > 128 || d->Hq < 1 || d->Hkv < 1 || d->Hq % d->Hkv != 0) return OURO_E_BAD_SHAPE;
  if (d->max_seqlen < 0) return OURO_E_BAD_SHAPE;
  if (d->dtype == OURO_BF16 ? d->D != 128 : (d->D != 64 && d->D != 128)) return OURO_E_BAD_SHAPE;
  if (static_cast<long>(d->T) * (d->Hq / d->Hkv) > 32768) return OURO_E_BAD_SHAPE;
  if (d->kv_layout != OURO_KV_ROW_MAJOR && d->kv_layout != OURO_KV_HEAD_MAJOR) return OURO_E_BAD_SHAPE;
  if (d->kv_layout == OURO_KV_HEAD_MAJOR && (d->cache_rows < 0 || d->cache_rows > (1LL << 40))) return OURO_E_BAD_SHAPE;
  if (d->plan_override < 0) return OURO_E_BAD_SHAPE;
  if (!need_pointers || d->B == 0) return OURO_OK;
  if (!d->q || !d->cu_seqlens || !d->k_blk || !d->v_blk || !d->meta || !d->out) return OURO_E_NULLPTR;
  if (d->max_seqlen > 0 && (!d->k_cache || !d->v_cache)) return OURO_E_NULLPTR;
  if (!aligned16(d->q) || !aligned16(d->k_cache) || !aligned16(d->v_cache) || !aligned16(d->k_blk) ||
      !aligned16(d->v_blk) || !aligned16(d->out) || !aligned16(d->workspace))
    return OURO_E_MISALIGNED;
  return OURO_OK;
}

int validate_lmhead(const ouro_lmhead_desc* d, bool need_pointers) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_lmhead_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_F32 && d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->R < 0 || d->V < 1 || d->Hd < 1) return OURO_E_BAD_SHAPE;
  if (d->Hd % (d->dtype == OURO_BF16 ? 64 : 4) != 0) return OURO_E_BAD_SHAPE;
  if (d->w_layout != OURO_W_ROW_MAJOR && !(d->w_layout == OURO_W_TILED && d->dtype == OURO_BF16)) return OURO_E_BAD_SHAPE;
  if (!need_pointers || d->R == 0) return OURO_OK;
  if (!d->hidden || !d->w || !d->argmax_out) return OURO_E_NULLPTR;
  if (!aligned16(d->hidden) || !aligned16(d->w) || !aligned16(d->workspace)) return OURO_E_MISALIGNED;
  return OURO_OK;
}

static int validate_accept(const ouro_accept_desc* d) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_accept_desc)) return OURO_E_BAD_STRUCT;
  if (d->B < 0 || d->gamma < 1 || d->K < 0 || d->K > 63 || d->beta < 0 || d->T < 1 || d->T > 128) return OURO_E_BAD_SHAPE;
  if (static_cast<long>(d->gamma) + static_cast<long>(d->K) * d->beta != d->T) return OURO_E_BAD_SHAPE;
  if (d->K > 0 && d->beta < 1) return OURO_E_BAD_SHAPE;
  if (d->B == 0) return OURO_OK;
  if (!d->draft_tok || !d->argmax || !d->meta || !d->n_accept || !d->path || !d->bonus || !d->accept_idx)
    return OURO_E_NULLPTR;
  const int nseg_ptrs = (d->n_seg != nullptr) + (d->seg_start != nullptr) + (d->seg_len != nullptr);
  if (nseg_ptrs != 0 && nseg_ptrs != 3) return OURO_E_NULLPTR;
  return OURO_OK;
}

static int validate_kv_commit(const ouro_kv_commit_desc* d) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_kv_commit_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_F32 && d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->B < 0 || d->B > 65535 || d->T < 1 || d->T > 128 || d->Hkv < 1 || d->D < 1) return OURO_E_BAD_SHAPE;
  if (d->max_accept < 1 || d->max_accept > d->T) return OURO_E_BAD_SHAPE;
  const long row_bytes = static_cast<long>(d->Hkv) * d->D * (d->dtype == OURO_BF16 ? 2 : 4);
  if (row_bytes % 16 != 0 || row_bytes > (1L << 30)) return OURO_E_BAD_SHAPE;
  if (d->kv_layout != OURO_KV_ROW_MAJOR && d->kv_layout != OURO_KV_HEAD_MAJOR) return OURO_E_BAD_SHAPE;
  if (d->kv_layout == OURO_KV_HEAD_MAJOR &&
      (d->cache_rows < 1 || d->cache_rows > (1LL << 40) || (static_cast<long>(d->D) * (d->dtype == OURO_BF16 ? 2 : 4)) % 16 != 0))
    return OURO_E_BAD_SHAPE;
  if (d->B == 0) return OURO_OK;
  if (!d->k_blk || !d->v_blk || !d->accept_idx || !d->n_accept || !d->k_cache || !d->v_cache || !d->cu_seqlens ||
      !d->seq_len || !d->overflow)
    return OURO_E_NULLPTR;
  if (!aligned16(d->k_blk) || !aligned16(d->v_blk) || !aligned16(d->k_cache) || !aligned16(d->v_cache))
    return OURO_E_MISALIGNED;
  return OURO_OK;
}

// The two launches of the LM head (main kernel, cross-slab arg-max) on a validated descriptor whose workspace holds
// at least plan.total() bytes.
int enqueue_lmhead(const ouro_lmhead_desc& d, const LmPlan& p, hipStream_t stream) {
  if (d.ev_start && hipEventRecord(static_cast<hipEvent_t>(d.ev_start), stream) != hipSuccess)
    return hip_failed(hipGetLastError());
  const int st = d.dtype == OURO_BF16 ? launch_lmhead_bf16(d, p, stream) : launch_lmhead_f32(d, p, stream);
  if (st != OURO_OK) return st;
  if (d.ev_stop && hipEventRecord(static_cast<hipEvent_t>(d.ev_stop), stream) != hipSuccess)
    return hip_failed(hipGetLastError());
  return launch_lmhead_final(d, p, stream);
}

}  // namespace ouro

using namespace ouro;

extern "C" {

size_t ouro_verify_attn_workspace(const ouro_attn_desc* desc) {
  if (validate_attn(desc, false) != OURO_OK || desc->dtype != OURO_BF16 || desc->B == 0) return 0;
  return plan_attn_bf16(*desc).total();
}

int ouro_verify_attn_plan(const ouro_attn_desc* desc, int32_t plan[5]) {
  if (!plan) return OURO_E_NULLPTR;
  const int st = validate_attn(desc, false);
  if (st != OURO_OK) return st;
  plan[0] = plan[1] = plan[2] = plan[3] = plan[4] = 0;
  if (desc->dtype != OURO_BF16) {
    plan[1] = desc->max_seqlen + desc->T;
    plan[2] = 1;
    plan[3] = desc->B * desc->Hq * desc->T;
    return OURO_OK;
  }
  const AttnPlan p = plan_attn_bf16(*desc);
  plan[0] = p.rw;
  plan[4] = p.waves;
  plan[1] = p.chunk;
  plan[2] = p.nch;
  plan[3] = static_cast<int32_t>((static_cast<long>(desc->B) * desc->Hkv * p.nch + 7) / 8 * 8 * p.nrb);
  return OURO_OK;
}

int ouro_verify_attn(const ouro_attn_desc* desc, void* hip_stream) {
  int st = validate_attn(desc, true);
  if (st != OURO_OK) return st;
  if (desc->B == 0) return OURO_OK;
  const float scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / std::sqrt(static_cast<float>(desc->D));
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (desc->dtype == OURO_F32) return launch_attn_f32(*desc, scale, stream);
  AttnPlan p = plan_attn_bf16(*desc);
  if (static_cast<long>(desc->B) * desc->Hkv * p.nch * p.nrb + 8L * p.nrb >= (1L << 31)) return OURO_E_BAD_SHAPE;   // grid size
  const size_t need = p.total();
  if (need > 0) {
    if (!desc->workspace) return OURO_E_NULLPTR;
    if (desc->workspace_bytes < need) return OURO_E_WORKSPACE_TOO_SMALL;
  }
  return launch_attn_bf16(*desc, p, scale, stream);
}

size_t ouro_lmhead_argmax_workspace(const ouro_lmhead_desc* desc) {
  if (validate_lmhead(desc, false) != OURO_OK || desc->R == 0) return 0;
  return plan_lmhead(*desc).total();
}

int ouro_lmhead_argmax(const ouro_lmhead_desc* desc, void* hip_stream) {
  int st = validate_lmhead(desc, true);
  if (st != OURO_OK) return st;
  if (desc->R == 0) return OURO_OK;
  LmPlan p = plan_lmhead(*desc);
  if (!desc->workspace) return OURO_E_NULLPTR;
  if (desc->workspace_bytes < p.total()) return OURO_E_WORKSPACE_TOO_SMALL;
  return enqueue_lmhead(*desc, p, static_cast<hipStream_t>(hip_stream));
}

size_t ouro_lmhead_packed_w_bytes(int32_t V, int32_t Hd) {
  if (V < 1 || Hd < 64 || Hd % 64 != 0) return 0;
  return static_cast<size_t>((V + 127) / 128) * 128 * static_cast<size_t>(Hd) * 2;
}

int ouro_lmhead_pack_w(const void* w_row_major, void* w_tiled, int32_t V, int32_t Hd, void* hip_stream) {
  if (!w_row_major || !w_tiled) return OURO_E_NULLPTR;
  if (ouro_lmhead_packed_w_bytes(V, Hd) == 0) return OURO_E_BAD_SHAPE;
  if (!aligned16(w_row_major) || !aligned16(w_tiled)) return OURO_E_MISALIGNED;
  return launch_pack_w(w_row_major, w_tiled, V, Hd, static_cast<hipStream_t>(hip_stream));
}

int ouro_accept(const ouro_accept_desc* desc, void* hip_stream) {
  int st = validate_accept(desc);
  if (st != OURO_OK) return st;
  if (desc->B == 0) return OURO_OK;
  return launch_accept(*desc, static_cast<hipStream_t>(hip_stream));
}

int ouro_kv_commit(const ouro_kv_commit_desc* desc, void* hip_stream) {
  int st = validate_kv_commit(desc);
  if (st != OURO_OK) return st;
  if (desc->B == 0) return OURO_OK;
  return launch_kv_commit(*desc, static_cast<hipStream_t>(hip_stream));
}

int ouro_rope_block(const ouro_rope_desc* d, void* hip_stream) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_rope_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_F32 && d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->B < 0 || d->B > 65535 || d->T < 1 || d->T > 128 || d->Hq < 1 || d->Hkv < 1 || d->D < 2 || d->D % 2 != 0 || d->D > 1024)
    return OURO_E_BAD_SHAPE;
  if (d->B == 0) return OURO_OK;
  if (!d->q || !d->k_blk || !d->meta || !d->cu_seqlens) return OURO_E_NULLPTR;
  if (d->qkv && !d->v_blk) return OURO_E_NULLPTR;
  return launch_rope_block(*d, static_cast<hipStream_t>(hip_stream));
}

int ouro_rmsnorm(const ouro_rmsnorm_desc* d, void* hip_stream) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_rmsnorm_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_F32 && d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->R < 0 || d->Hd < 1 || !(d->eps >= 0.f)) return OURO_E_BAD_SHAPE;
  if (d->R == 0) return OURO_OK;
  if (!d->x || !d->gain || !d->out) return OURO_E_NULLPTR;
  return launch_rmsnorm(*d, static_cast<hipStream_t>(hip_stream));
}

static int validate_linear(const ouro_linear_desc* d) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_linear_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->R < 0 || d->K < 64 || d->K % 64 != 0 || d->N < 8 || d->N % 8 != 0) return OURO_E_BAD_SHAPE;
  if (d->w_layout != OURO_W_ROW_MAJOR && d->w_layout != OURO_W_TILED) return OURO_E_BAD_SHAPE;
  if (d->epilogue != OURO_EPI_NONE && d->epilogue != OURO_EPI_SWIGLU_PAIRS) return OURO_E_BAD_SHAPE;
  if (d->epilogue == OURO_EPI_SWIGLU_PAIRS && (d->N % 16 != 0 || d->residual)) return OURO_E_BAD_SHAPE;
  if (d->ksplit_override < 0) return OURO_E_BAD_SHAPE;
  return OURO_OK;
}

size_t ouro_linear_workspace(const ouro_linear_desc* d) {
  if (validate_linear(d) != OURO_OK || d->R == 0) return 0;
  return linear_workspace_bytes(d->R, d->K, d->N, d->ksplit_override);
}

int ouro_linear(const ouro_linear_desc* d, void* hip_stream) {
  int st = validate_linear(d);
  if (st != OURO_OK) return st;
  if (d->R == 0) return OURO_OK;
  if (!d->x || !d->w || !d->out) return OURO_E_NULLPTR;
  if (!aligned16(d->x) || !aligned16(d->w) || !aligned16(d->out) || !aligned16(d->residual) || !aligned16(d->workspace))
    return OURO_E_MISALIGNED;
  const size_t need = linear_workspace_bytes(d->R, d->K, d->N, d->ksplit_override);
  if (need > 0) {
    if (!d->workspace) return OURO_E_NULLPTR;
    if (d->workspace_bytes < need) return OURO_E_WORKSPACE_TOO_SMALL;
  }
  return launch_linear_bf16(*d, static_cast<hipStream_t>(hip_stream));
}

static int validate_weight_relayout(const void* a, const void* b, const void* out, int32_t rows, int32_t K) {
  if (!a || !b || !out) return OURO_E_NULLPTR;
  if (rows < 1 || K < 8 || K % 8 != 0) return OURO_E_BAD_SHAPE;
  if (!aligned16(a) || !aligned16(b) || !aligned16(out)) return OURO_E_MISALIGNED;
  return OURO_OK;
}

int ouro_fold_rmsnorm_gain(const void* w, const void* gain, void* out, int32_t N, int32_t K, void* hip_stream) {
  const int st = validate_weight_relayout(w, gain, out, N, K);
  if (st != OURO_OK) return st;
  return launch_fold_rmsnorm_gain(w, gain, out, N, K, static_cast<hipStream_t>(hip_stream));
}

int ouro_interleave_gate_up(const void* w_gate, const void* w_up, void* out, int32_t F, int32_t K, void* hip_stream) {
  const int st = validate_weight_relayout(w_gate, w_up, out, F, K);
  if (st != OURO_OK) return st;
  return launch_interleave_gate_up(w_gate, w_up, out, F, K, static_cast<hipStream_t>(hip_stream));
}

int ouro_silu_mul(const ouro_silu_mul_desc* d, void* hip_stream) {
  if (!d) return OURO_E_NULLPTR;
  if (d->struct_size != sizeof(ouro_silu_mul_desc)) return OURO_E_BAD_STRUCT;
  if (d->dtype != OURO_F32 && d->dtype != OURO_BF16) return OURO_E_UNSUPPORTED_DTYPE;
  if (d->R < 0 || d->F < 1) return OURO_E_BAD_SHAPE;
  if (d->R == 0) return OURO_OK;
  if (!d->gate_up || !d->out) return OURO_E_NULLPTR;
  return launch_silu_mul(*d, static_cast<hipStream_t>(hip_stream));
}

int ouro_validate_meta_host(const ouro_tok_meta* m, int32_t T, int32_t gamma, int32_t K, int32_t beta) {
  if (!m) return OURO_E_NULLPTR;
  if (T < 1 || gamma < 1 || K < 0 || beta < 0 || static_cast<long>(gamma) + static_cast<long>(K) * beta != T)
    return OURO_E_BAD_SHAPE;
  for (int i = 0; i < gamma; ++i)
    if (m[i].phrase_id != 0 || m[i].branch_off != i) return OURO_E_BAD_META;
  for (int j = 1; j <= K; ++j) {
    const int lo = gamma + (j - 1) * beta;
    const int bj = m[lo].branch_off;
    if (bj < -1 || bj >= gamma) return OURO_E_BAD_META;
    for (int i = 0; i < beta; ++i)
      if (m[lo + i].phrase_id != j || m[lo + i].branch_off != bj) return OURO_E_BAD_META;
  }
  return OURO_OK;
}

const char* ouro_status_string(int status) {
  switch (status) {
    case OURO_OK: return "ok";
    case OURO_E_NULLPTR: return "a required pointer is NULL";
    case OURO_E_BAD_SHAPE: return "a size is out of range or inconsistent";
    case OURO_E_UNSUPPORTED_DTYPE: return "unsupported dtype";
    case OURO_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case OURO_E_MISALIGNED: return "a pointer is not 16-byte aligned";
    case OURO_E_HIP: return "a HIP call failed";
    case OURO_E_BAD_STRUCT: return "struct_size does not match the header";
    case OURO_E_BAD_META: return "block metadata violates the layout rules";
    case OURO_E_STATIC_SCRATCH_TOO_SMALL: return "the size needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
  }
}

int ouro_last_hip_error(void) { return g_last_hip_error; }
int ouro_version(void) { return OURO_VERSION; }

}  // extern "C"
