/*
 * ouro.h -- C ABI of the MI355X (gfx950) verification-step library.
 *
 * One verification pass of Ouroboros speculative decoding (Sec. 2, Eq. (2)-(3);
 * Sec. 3.2, Eq. (7)-(9)): the target model scores a whole draft block -- a main
 * draft d_1..gamma followed by K candidate phrase suffixes -- in one parallel
 * pass against the KV cache, under an attention mask that gives every block row
 * exactly the context its own lengthened draft would have; the greedy token of
 * every row is taken, and the longest accepted prefix is selected.
 *
 * Three stages, three entry points:
 *   ouro_verify_attn     masked draft-block attention against the KV cache
 *   ouro_lmhead_argmax   LM-head product fused with the arg-max over the vocabulary
 *   ouro_accept          accepted-prefix decision over main draft + phrases
 * and the step that closes the loop:
 *   ouro_kv_commit       keeps the keys/values of the accepted tokens in the cache
 *
 * General contract
 *   - Every data pointer in a descriptor is DEVICE memory owned by the caller and
 *     must stay valid until the work enqueued on the stream has finished.
 *     Descriptors themselves are HOST memory, read during the call only.
 *   - Calls only enqueue work on the given HIP stream (a hipStream_t passed as
 *     void*; NULL = the default stream).  They never allocate, free or
 *     synchronise, and may be called from several threads on different streams
 *     with disjoint outputs and workspaces.  The library keeps nothing between
 *     calls except, per device, the fact that the kernels' shared-memory limits
 *     have been raised (done once, thread-safe, on the first launch on a device);
 *     nothing is read from the process environment.
 *   - Return value: OURO_OK (0) or a negative OURO_E_* code.  On an error nothing
 *     has been enqueued, except OURO_E_HIP which reports a failed launch (the
 *     hipError_t is kept per thread for ouro_last_hip_error()).
 *   - All shape/pointer/alignment/workspace checks run on the host before any
 *     HIP call, so they can be exercised on a machine without a GPU.
 *   - Inputs must be finite; NaN handling is unspecified.
 */
#ifndef OURO_H
#define OURO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OURO_VERSION 211 /* major*10000 + minor*100 + patch */

/* Exported from libouro.so (everything else in the library has hidden visibility). */
#define OURO_API __attribute__((visibility("default")))

enum {
  OURO_OK = 0,
  OURO_E_NULLPTR = -1,             /* a required pointer is NULL */
  OURO_E_BAD_SHAPE = -2,           /* a size is out of range or inconsistent */
  OURO_E_UNSUPPORTED_DTYPE = -3,
  OURO_E_WORKSPACE_TOO_SMALL = -4,
  OURO_E_MISALIGNED = -5,          /* a pointer is not 16-byte aligned */
  OURO_E_HIP = -6,                 /* a HIP call failed; see ouro_last_hip_error() */
  OURO_E_BAD_STRUCT = -7,          /* struct_size does not match this header */
  OURO_E_BAD_META = -8,            /* ouro_validate_meta_host only */
  OURO_E_STATIC_SCRATCH_TOO_SMALL = -9   /* ouro_lmhead_argmax_static only: the size needs more than the built-in buffer */
};

typedef enum { OURO_F32 = 0, OURO_BF16 = 1 } ouro_dtype;

/*
 * Per-token block metadata, 4 bytes.  The block of T tokens is laid out as the main
 * draft (block indices 0..gamma-1) followed by the phrases (Eq. (7)); a phrase
 * occupies a contiguous ascending index range.
 *   main token i      : phrase_id = 0, branch_off = i
 *   token of phrase j : phrase_id = j (1..K), branch_off = b_j, the 0-based main-draft
 *                       index the phrase hangs off.  The paper's layout (every phrase
 *                       starts with d_gamma, Sec. 3.2) is b_j = gamma-1.  b_j = -1: the
 *                       phrase hangs off the last cached token and sees no main token.
 * The attention mask is computed from these pairs inside the kernel; no dense mask is
 * ever read from memory.  Row q sees block key k iff
 *   phrase_id[k] == 0 ? k <= branch_off[q] : (phrase_id[k] == phrase_id[q] && k <= q),
 * which is the conditioning set of Eq. (2) for main rows and of Eq. (8) for phrase rows.
 */
typedef struct {
  int16_t phrase_id;
  int16_t branch_off;
} ouro_tok_meta;

/* ------------------------------------------------------------------------------------ */
/* Draft-block attention (the attention of the single verifying forward, Sec. 3.2).      */
/*                                                                                       */
/* For sequence b, query head h and block row t:                                         */
/*   out = softmax(scale * q . K_vis^T) . V_vis                                          */
/* over the L_b cached keys of the sequence (all visible) followed by the block keys      */
/* visible to row t.  Query head h reads KV head h / (Hq / Hkv).  Q and K arrive with     */
/* positional rotation already applied.  bf16: products on bf16 MFMA, fp32 accumulation,  */
/* probabilities rounded to bf16 before the value product, bf16 output.  f32: fp32        */
/* arithmetic throughout.                                                                */
/* ------------------------------------------------------------------------------------ */
typedef struct {
  uint32_t struct_size;        /* sizeof(ouro_attn_desc) */
  int32_t dtype;               /* ouro_dtype of q, k_*, v_*, out */
  int32_t B;                   /* sequences, >= 0 (0: nothing to do) */
  int32_t T;                   /* block tokens per sequence, 1..128 */
  int32_t Hq;                  /* query heads */
  int32_t Hkv;                 /* key/value heads, divides Hq */
  int32_t D;                   /* head dim: 128 (bf16) ; 64 or 128 (f32) */
  int32_t max_seqlen;          /* host-side upper bound on every L_b (sizes the launch; no device read-back).  A
                                  sequence whose device-side length exceeds it is attended over its first
                                  max_seqlen cached tokens only: a stale bound gives a contained result, never an
                                  access outside the workspace or the sequence's region */
  const void* q;               /* [B, T, Hq, D] */
  const void* k_cache;         /* [rows, Hkv, D] (or head-major, see kv_layout); sequence b in the region of rows
                                  cu_seqlens[b] .. cu_seqlens[b+1]-1 */
  const void* v_cache;         /* same layout; may be NULL only if max_seqlen == 0 */
  const int64_t* cu_seqlens;   /* [B+1], cu[0] = 0, non-decreasing region offsets.  Without seq_len the regions are
                                  packed: L_b = cu[b+1] - cu[b].  0 <= L_b <= max_seqlen */
  const void* k_blk;           /* [B, T, Hkv, D] keys of the block tokens (not yet in the cache) */
  const void* v_blk;           /* [B, T, Hkv, D] */
  const ouro_tok_meta* meta;   /* [B, T] */
  float softmax_scale;         /* <= 0: 1/sqrt(D) */
  void* out;                   /* [B, T, Hq, D], same dtype as q */
  float* lse;                  /* optional [B, Hq, T]: natural-log softmax denominator; NULL to skip */
  void* workspace;             /* >= ouro_verify_attn_workspace() bytes, 16-byte aligned; contents arbitrary */
  size_t workspace_bytes;
  void* ev_start;              /* optional hipEvent_t pair (NULL to skip), recorded on the stream right before and */
  void* ev_stop;               /* right after the call's main kernel, so that a profiler can time that kernel alone */
  const int32_t* seq_len;      /* optional [B]: L_b, the cached tokens at the start of region b; the rest of the region
                                  is room for tokens accepted later (ouro_kv_commit).  NULL: packed regions */
  int32_t kv_layout;           /* OURO_KV_ROW_MAJOR: caches are [rows, Hkv, D].  OURO_KV_HEAD_MAJOR: [Hkv, cache_rows, D],
                                  every (sequence, KV head) stream contiguous in memory, which HBM delivers fastest */
  int32_t plan_override;       /* 0: the library chooses the launch shape.  Tests and tuning runs may force it (bf16
                                  only): bits 0..6 = 32-row query blocks per workgroup (1, 2 or 4; 0 = library's
                                  choice), bit 7 = with 4 row blocks, the four-wave kernel instead of the eight-wave
                                  one, bits 8..31 = keys per workgroup / 128 (0 = library's choice).  The same
                                  value must be given to the workspace query */
  int64_t cache_rows;          /* OURO_KV_HEAD_MAJOR: rows per KV head of the cache allocation (>= cu_seqlens[B]) */
} ouro_attn_desc;

enum { OURO_KV_ROW_MAJOR = 0, OURO_KV_HEAD_MAJOR = 1 };

/* Host-only: bytes of workspace the call will need for this descriptor (data pointers are
 * not read).  Returns 0 if the descriptor is invalid or no workspace is needed. */
OURO_API size_t ouro_verify_attn_workspace(const ouro_attn_desc* desc);
OURO_API int ouro_verify_attn(const ouro_attn_desc* desc, void* hip_stream);
/* Host-only: the launch shape the call will use for this descriptor (data pointers are not read), for logs, benchmarks
 * and tuning: plan[0] = 32-row query blocks per workgroup (1: the kernel whose waves split the keys; 2, 4: the kernel
 * whose waves split the rows and share staged K/V tiles; 0: the fp32 kernel), plan[1] = keys per workgroup,
 * plan[2] = chunk slots per sequence (> 1: partial results are merged by a second launch), plan[3] = workgroups of the
 * main kernel, plan[4] = waves per workgroup (4; 8 for the four-row-block kernel in its eight-wave form; 0: the fp32
 * kernel).  Returns OURO_OK or the descriptor's validation error. */
OURO_API int ouro_verify_attn_plan(const ouro_attn_desc* desc, int32_t plan[5]);

/* ------------------------------------------------------------------------------------ */
/* LM head fused with the greedy pick (Eq. (2) under greedy decoding).                   */
/*   logits[r, v] = sum_k hidden[r, k] * w[v, k]   ;   argmax_out[r] = arg max_v logits   */
/* Ties go to the smallest v.  The logits are never written to memory.  bf16: bf16 MFMA   */
/* with fp32 accumulation; f32: fp32 arithmetic.                                          */
/* ------------------------------------------------------------------------------------ */
typedef struct {
  uint32_t struct_size;        /* sizeof(ouro_lmhead_desc) */
  int32_t dtype;               /* ouro_dtype of hidden and w */
  int32_t R;                   /* rows (B*T block tokens), >= 0 */
  int32_t Hd;                  /* hidden size, multiple of 64 (bf16) / 4 (f32) */
  int32_t V;                   /* vocabulary, >= 1 */
  int32_t w_layout;            /* OURO_W_ROW_MAJOR or OURO_W_TILED (bf16 only) */
  const void* hidden;          /* [R, Hd] row-major (the attention output viewed as [B*T, Hq*D]) */
  const void* w;               /* OURO_W_ROW_MAJOR: [V, Hd], row v is the output embedding of token v.
                                  OURO_W_TILED: the same matrix re-blocked once by ouro_lmhead_pack_w into
                                  contiguous 16 KB tiles [ceil(V/128)][Hd/64][128 rows][64 columns] (rows past V
                                  zero): every wave then streams whole contiguous tiles, which is what HBM
                                  delivers fastest.  Weights are static, so the packing is a load-time step. */
  int32_t* argmax_out;         /* [R] */
  float* max_out;              /* optional [R]: the winning logit (fp32); NULL to skip */
  void* workspace;             /* >= ouro_lmhead_argmax_workspace() bytes, 16-byte aligned; contents arbitrary */
  size_t workspace_bytes;
  void* ev_start;              /* optional hipEvent_t pair around the main (weight-streaming) kernel, as above */
  void* ev_stop;
} ouro_lmhead_desc;

enum { OURO_W_ROW_MAJOR = 0, OURO_W_TILED = 1 };

OURO_API size_t ouro_lmhead_argmax_workspace(const ouro_lmhead_desc* desc);
OURO_API int ouro_lmhead_argmax(const ouro_lmhead_desc* desc, void* hip_stream);

/* For callers that cannot allocate device memory or hand a workspace over (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): ouro_lmhead_argmax with the cross-slab partials kept in a buffer that is
 * part of the library's own device image (OURO_LMHEAD_STATIC_SCRATCH_BYTES per GPU, held until the process ends).
 * Same descriptor, same kernels, same results; desc->workspace and workspace_bytes are ignored.  The call allocates
 * nothing and calls no allocating routine.  A size whose partials (ouro_lmhead_argmax_workspace bytes) exceed the
 * buffer is rejected with OURO_E_STATIC_SCRATCH_TOO_SMALL before anything is enqueued (with V = 32000 the limit is
 * 2097 rows).  All calls on one GPU share that GPU's buffer:
 * calls that may overlap on one GPU (different streams, several threads) race on it and must be serialised by the
 * caller; calls on different GPUs are independent.  Nothing in the buffer has to be cleared between calls: every
 * partial a call reads it has written before. */
#define OURO_LMHEAD_STATIC_SCRATCH_BYTES (2u << 20)
OURO_API int ouro_lmhead_argmax_static(const ouro_lmhead_desc* desc, void* hip_stream);

/* Bytes of the OURO_W_TILED form of a bf16 [V, Hd] weight (Hd a multiple of 64); 0 if the shape is invalid. */
OURO_API size_t ouro_lmhead_packed_w_bytes(int32_t V, int32_t Hd);
/* Enqueue the re-blocking of a bf16 row-major DEVICE weight [V, Hd] into w_tiled (DEVICE, 16-byte aligned,
 * >= ouro_lmhead_packed_w_bytes bytes, not overlapping w_row_major). */
OURO_API int ouro_lmhead_pack_w(const void* w_row_major, void* w_tiled, int32_t V, int32_t Hd, void* hip_stream);

/* ------------------------------------------------------------------------------------ */
/* Acceptance (Eq. (3) for the main draft, Eq. (9) for each phrase, and the rule after    */
/* Eq. (9): extend the accepted draft by the phrase with the longest accepted run).       */
/*                                                                                       */
/* Block position t is compared with the greedy token predicted by the row of the token   */
/* that precedes it in its own lengthened draft (root_pred for a position that follows     */
/* the cached prefix directly).  A = leading matches of the main draft; Ahat'_j = leading  */
/* matches inside phrase j's beta block tokens; phrase j is usable iff A >= b_j + 1 and    */
/* then yields b_j + 1 + Ahat'_j accepted tokens; the longest candidate wins, the main      */
/* draft first and then the lowest phrase id on ties.  bonus = the prediction of the last   */
/* accepted row (root_pred if nothing is accepted, -1 if root_pred is NULL as well).        */
/* Every accepted token must equal a prediction of the target (the lossless property,       */
/* Eq. (4)).  The one exception is declared by the caller: with root_pred NULL, main token   */
/* 0 is the sequence's last, already accepted token and counts as accepted unchecked.  A     */
/* phrase that hangs off the cached prefix (b_j = -1) then has nothing its first token       */
/* could be checked against: that token counts as a mismatch and the phrase is never used.   */
/* ------------------------------------------------------------------------------------ */
typedef struct {
  uint32_t struct_size;        /* sizeof(ouro_accept_desc) */
  int32_t B;                   /* sequences, >= 0 */
  int32_t T;                   /* == gamma + K * beta, 1..128 */
  int32_t gamma;               /* main draft length, >= 1 */
  int32_t K;                   /* phrases, 0..63 */
  int32_t beta;                /* block tokens per phrase (the paper's beta - 1) */
  const int32_t* draft_tok;    /* [B, T] */
  const int32_t* argmax;       /* [B, T] greedy token of every block row */
  const ouro_tok_meta* meta;   /* [B, T] */
  const int32_t* root_pred;    /* [B] target's prediction after the cached prefix; NULL: main token 0 counts as
                                  accepted without a check (see above) */
  int32_t* n_accept;           /* [B] number of accepted block tokens */
  int32_t* path;               /* [B] 0 = main draft only, j = main draft up to b_j then phrase j */
  int32_t* bonus;              /* [B] */
  int32_t* accept_idx;         /* [B, gamma + beta] accepted block indices in order, -1 padded */
  int32_t* main_A;             /* optional [B] */
  int32_t* phrase_A;           /* optional [B, K] */
  int32_t* n_match;            /* optional [B]: number of main-draft positions equal to the target's
                                  prediction, accepted or not (#Match, Eq. (10)) */
  /* Optional by-products for the phrase pool (Sec. 3.3, the two paragraphs after Eq. (10)); NULL to skip. */
  uint8_t* match_out;          /* [B, T]: 1 where the block token equals the target's greedy token at its position
                                  (the indicator summed by Eq. (10)); main token 0 without root_pred counts as 1 */
  int32_t* n_seg;              /* [B]: number of matching sub-segments of the discarded draft: maximal runs of
                                  matches among main positions > A.  n_seg, seg_start, seg_len: all or none */
  int32_t* seg_start;          /* [B, max(1, (gamma+1)/2)]: first main index of each run, ascending, -1 padded */
  int32_t* seg_len;            /* [B, max(1, (gamma+1)/2)]: run lengths, 0 padded */
  int32_t* repaired;           /* [B, K, beta+1]: for every phrase o, its first token (the main-draft token at its
                                  branch point; -1 if it hangs off the prefix) followed by the target's greedy
                                  token at each of its beta block positions: the phrase (p^o_1, v^o_2..) that
                                  replaces p^o in the pool when o was not the phrase used */
} ouro_accept_desc;

OURO_API int ouro_accept(const ouro_accept_desc* desc, void* hip_stream);

/* ------------------------------------------------------------------------------------ */
/* Keeping the accepted tokens (the sentence after Eq. (3): d_1..A are accepted, the rest  */
/* of the draft is discarded; after Eq. (9): d_1..gamma and p^j_2..Ahat^j are accepted).   */
/*                                                                                       */
/* For every sequence b the keys/values of the accepted block tokens                      */
/* accept_idx[b, 0 .. n_accept[b]-1] (block indices in accepted order, as written by        */
/* ouro_accept) are copied from k_blk/v_blk to the cache rows                              */
/* cu_seqlens[b] + seq_len[b] + i, and seq_len[b] grows by n_accept[b]; the other block      */
/* tokens are dropped.  The cache is the layout ouro_verify_attn reads with its seq_len      */
/* field: region offsets in cu_seqlens, cached tokens at the start of each region.  A        */
/* sequence whose region cannot take its accepted tokens is left untouched (rows and         */
/* length) and overflow[b] is set to 1, else to 0.  Copies are bit-exact.  The work is       */
/* enqueued as two small kernels (copy, then lengths), so seq_len is updated in place.       */
/* ------------------------------------------------------------------------------------ */
typedef struct {
  uint32_t struct_size;        /* sizeof(ouro_kv_commit_desc) */
  int32_t dtype;               /* ouro_dtype of the caches and of k_blk, v_blk */
  int32_t B;                   /* sequences, >= 0 */
  int32_t T;                   /* block tokens per sequence, 1..128 */
  int32_t Hkv;                 /* key/value heads */
  int32_t D;                   /* head dim; Hkv * D * element size must be a multiple of 16 bytes */
  int32_t max_accept;          /* row length of accept_idx (gamma + beta for ouro_accept), 1..T */
  const void* k_blk;           /* [B, T, Hkv, D] */
  const void* v_blk;           /* [B, T, Hkv, D] */
  const int32_t* accept_idx;   /* [B, max_accept], entries 0 .. n_accept[b]-1 in [0, T) */
  const int32_t* n_accept;     /* [B], 0 .. max_accept */
  void* k_cache;               /* [rows, Hkv, D] or [Hkv, cache_rows, D], see kv_layout */
  void* v_cache;
  const int64_t* cu_seqlens;   /* [B+1] region offsets */
  int32_t* seq_len;            /* [B] in/out */
  int32_t* overflow;           /* [B] out */
  int32_t kv_layout;           /* layout of k_cache / v_cache, as in ouro_attn_desc */
  int32_t reserved0;           /* 0 */
  int64_t cache_rows;          /* OURO_KV_HEAD_MAJOR: rows per KV head of the cache allocation */
} ouro_kv_commit_desc;

OURO_API int ouro_kv_commit(const ouro_kv_commit_desc* desc, void* hip_stream);

/* ------------------------------------------------------------------------------------ */
/* The rest of the verifying layer around the attention.  The paper verifies the block with */
/* one forward of the target model (Sec. 3.2) and fixes one thing about that forward beyond  */
/* the mask: since every lengthened draft of Eq. (7) is an ordinary linear sequence, a block   */
/* token's position is the number of tokens before it in its own draft,                      */
/*   pos = L_b + i                 for main token i,                                        */
/*   pos = L_b + b_j + 1 + i       for the i-th block token of a phrase hanging off main b_j. */
/* The operations themselves are the target model's (Llama-2: RMSNorm, rotate-half rotary     */
/* embedding, SwiGLU); all inner arithmetic in fp32.                                         */
/* ------------------------------------------------------------------------------------ */

/* Rotary embedding of the block's queries and keys at the positions above: the pair           */
/* (x[i], x[i + D/2]) of every head is rotated by the angle pos * base^(-2i/D).                */
/* Two forms.  In place (qkv NULL): q and k_blk are rotated where they are.  From a fused       */
/* projection (qkv non-NULL): row b*T + t of qkv holds [Hq heads | Hkv key heads | Hkv value    */
/* heads], each of D elements; the rotated queries and keys are written to q and k_blk and the   */
/* values are copied to v_blk, so that one launch turns the projection's output into the three   */
/* operands ouro_verify_attn takes.  qkv must not overlap q, k_blk or v_blk.                     */
typedef struct {
  uint32_t struct_size;        /* sizeof(ouro_rope_desc) */
  int32_t dtype;
  int32_t B, T, Hq, Hkv, D;    /* D even */
  float base;                  /* <= 0: 10000 */
  void* q;                     /* [B, T, Hq, D] in/out (out only with qkv) */
  void* k_blk;                 /* [B, T, Hkv, D] in/out (out only with qkv) */
  const ouro_tok_meta* meta;   /* [B, T] */
  const int64_t* cu_seqlens;   /* [B+1], as in ouro_attn_desc */
  const int32_t* seq_len;      /* optional [B], as in ouro_attn_desc */
  int32_t* positions;          /* optional out [B, T] */
  const void* qkv;             /* optional [B*T, (Hq + 2*Hkv) * D]: source of the second form */
  void* v_blk;                 /* [B, T, Hkv, D] out; required with qkv, ignored without */
} ouro_rope_desc;
OURO_API int ouro_rope_block(const ouro_rope_desc* desc, void* hip_stream);

/* out[r, :] = x[r, :] / sqrt(mean(x[r, :]^2) + eps) * gain */
typedef struct {
  uint32_t struct_size;
  int32_t dtype;
  int32_t R, Hd;
  float eps;
  const void* x;               /* [R, Hd] */
  const void* gain;            /* [Hd] */
  void* out;                   /* [R, Hd]; may alias x */
} ouro_rmsnorm_desc;
OURO_API int ouro_rmsnorm(const ouro_rmsnorm_desc* desc, void* hip_stream);

/* out[r, n] = sum_k x[r, k] * w[n, k] (+ residual[r, n]): every projection of the layer.  bf16 only (bf16 MFMA,  */
/* fp32 accumulation, one rounding at the end).  The weight is streamed from HBM once, like the LM head's, and may   */
/* be given in the same tiled form (ouro_lmhead_pack_w with V = N, Hd = K).                                        */
/* Epilogue OURO_EPI_SWIGLU_PAIRS (the MLP's first projection and its gate in one launch): rows 2j and 2j+1 of w    */
/* are the gate and the up projection of feature j, and out[r, j] = silu(y[r, 2j]) * y[r, 2j+1] with y the fp32     */
/* product, silu(a) = a / (1 + exp(-a)); out is then [R, N/2], N a multiple of 16, residual NULL.                    */
enum { OURO_EPI_NONE = 0, OURO_EPI_SWIGLU_PAIRS = 1 };
typedef struct {
  uint32_t struct_size;
  int32_t dtype;               /* OURO_BF16 */
  int32_t R;                   /* rows, >= 0 */
  int32_t K;                   /* input features, multiple of 64 */
  int32_t N;                   /* output features (rows of w), multiple of 8 */
  int32_t w_layout;            /* OURO_W_ROW_MAJOR or OURO_W_TILED */
  int32_t epilogue;            /* OURO_EPI_NONE or OURO_EPI_SWIGLU_PAIRS */
  float rms_eps;               /* > 0: the product's row r is scaled by 1 / sqrt(mean_k x[r, k]^2 + rms_eps) before the
                                  epilogue and the residual: RMSNorm of the input with its gain folded into w
                                  (w[n, k] * gain[k]: ouro_fold_rmsnorm_gain, at load time), in the same launch; <= 0: off */
  int32_t ksplit_override;     /* 0: the library chooses over how many workgroups the k range is split.  Tests and
                                  tuning runs may force a count (clamped to K / 64); the same value must be given to
                                  the workspace query */
  int32_t reserved0;           /* 0 */
  const void* x;               /* [R, K] */
  const void* w;               /* [N, K] or tiled */
  const void* residual;        /* optional [R, N]; may alias out */
  void* out;                   /* [R, N]  ([R, N/2] with OURO_EPI_SWIGLU_PAIRS) */
  void* workspace;             /* >= ouro_linear_workspace() bytes, 16-byte aligned; contents arbitrary.  Needed when
                                  N is small: the k range is then split over several workgroups whose fp32 partial
                                  sums are added in a fixed order by a second small kernel */
  size_t workspace_bytes;
} ouro_linear_desc;
OURO_API size_t ouro_linear_workspace(const ouro_linear_desc* desc);   /* host-only; 0 if invalid or none needed */
OURO_API int ouro_linear(const ouro_linear_desc* desc, void* hip_stream);

/* Load-time re-layouts of projection weights (bf16, DEVICE pointers, 16-byte aligned, K a multiple of 8; out must  */
/* not overlap the inputs).  Both are one pass over the weight and are meant to run once per weight, like            */
/* ouro_lmhead_pack_w; the result may then be packed into the tiled form.                                            */
/*   ouro_fold_rmsnorm_gain:   out[n, k] = bf16(w[n, k] * gain[k]) (fp32 product, one rounding): the weight that      */
/*                             ouro_linear with rms_eps > 0 expects.                                                 */
/*   ouro_interleave_gate_up:  out[2j, :] = w_gate[j, :], out[2j+1, :] = w_up[j, :] (j < F): the row order that       */
/*                             OURO_EPI_SWIGLU_PAIRS expects.                                                        */
OURO_API int ouro_fold_rmsnorm_gain(const void* w, const void* gain, void* out, int32_t N, int32_t K, void* hip_stream);
OURO_API int ouro_interleave_gate_up(const void* w_gate, const void* w_up, void* out, int32_t F, int32_t K, void* hip_stream);

/* out[r, f] = silu(gate_up[r, f]) * gate_up[r, F + f], silu(z) = z / (1 + exp(-z)) */
typedef struct {
  uint32_t struct_size;
  int32_t dtype;
  int32_t R, F;
  const void* gate_up;         /* [R, 2F]: gate columns then up columns (one fused projection) */
  void* out;                   /* [R, F] */
} ouro_silu_mul_desc;
OURO_API int ouro_silu_mul(const ouro_silu_mul_desc* desc, void* hip_stream);

/* ------------------------------------------------------------------------------------ */
/* Measurement aids (not part of the verification path; used by the benchmark to state    */
/* every kernel's rate against what the machine at hand delivers, next to the datasheet).  */
/* ------------------------------------------------------------------------------------ */
/* One streaming read of `bytes` (>= 1 MiB; whole 16 KB blocks are read, 16-byte non-temporal loads, 2048 workgroups) of the DEVICE
 * buffer buf; sink: 4 writable DEVICE bytes (never written for ordinary data).  HBM rate = bytes / kernel time when
 * the buffer exceeds the last-level cache. */
OURO_API int ouro_probe_stream_read(const void* buf, size_t bytes, void* sink, void* hip_stream);
/* A bare loop of bf16 32x32x16 matrix-core instructions on register operands: `workgroups` x 4 waves x `rounds` x 16
 * instructions of 32768 flop each; sink as above. */
OURO_API int ouro_probe_mfma_bf16(int32_t workgroups, int32_t rounds, void* sink, void* hip_stream);

/* ------------------------------------------------------------------------------------ */
/* Host-side helpers                                                                     */
/* ------------------------------------------------------------------------------------ */
/* Debug check of a HOST copy of one sequence's metadata against the layout rules above
 * (main tokens first with branch_off = index, phrases contiguous and ascending with ids
 * 1..K, -1 <= b_j < gamma).  Returns OURO_OK or OURO_E_BAD_META / OURO_E_NULLPTR /
 * OURO_E_BAD_SHAPE.  Not called on the hot path. */
OURO_API int ouro_validate_meta_host(const ouro_tok_meta* meta_host, int32_t T, int32_t gamma, int32_t K, int32_t beta);

OURO_API const char* ouro_status_string(int status);
OURO_API int ouro_last_hip_error(void);   /* hipError_t of the calling thread's last OURO_E_HIP, else 0 */
OURO_API int ouro_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OURO_H */
