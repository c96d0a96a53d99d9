// fp32 draft-block attention (correctness-grade path, used by the fp32 workload).
//
// One 64-lane wave per (sequence, query head, block row).  Keys are visited 64 at a time
// (lane <-> key) for the scores, with an online softmax carried across chunks; the value
// product then runs lane <-> head-dim element.  All arithmetic is fp32 on the vector ALU:
// no matrix-core instruction is used, so the result stays within fp32 rounding of the
// exact softmax.  The block part of the mask comes from the per-token metadata:
// row q sees block key k iff  pid[k]==0 ? k <= boff[q] : (pid[k]==pid[q] && k <= q)
// (conditioning sets of Eq. (2) and Eq. (8)); cached keys are always visible.
#include <math.h>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

template <int D>
__global__ __launch_bounds__(64) void attn_f32_kernel(ouro_attn_desc d, float scale) {
  constexpr int DPL = D / 64;  // head-dim elements per lane in the value product
  __shared__ float q_s[D];
  __shared__ float p_s[64];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  const int T = d.T, Hq = d.Hq, Hkv = d.Hkv;
  const int g = h / (Hq / Hkv);
  const long cu0 = d.cu_seqlens[b];
  // (cut to the host's bound like the bf16 kernels, so that both precisions treat a stale bound alike)
  const int L = min(d.seq_len ? d.seq_len[b] : static_cast<int>(d.cu_seqlens[b + 1] - cu0), d.max_seqlen);
  const int n = L + T;
  const float* q = static_cast<const float*>(d.q) + ((static_cast<size_t>(b) * T + t) * Hq + h) * D;
  // cache addressing: [rows, Hkv, D] or [Hkv, rows, D]
  const size_t row_stride = d.kv_layout == OURO_KV_HEAD_MAJOR ? D : static_cast<size_t>(Hkv) * D;
  const size_t head_stride = d.kv_layout == OURO_KV_HEAD_MAJOR ? static_cast<size_t>(d.cache_rows) * D : D;
  const float* kc = static_cast<const float*>(d.k_cache);
  const float* vc = static_cast<const float*>(d.v_cache);
  const float* kb = static_cast<const float*>(d.k_blk) + static_cast<size_t>(b) * T * Hkv * D;
  const float* vb = static_cast<const float*>(d.v_blk) + static_cast<size_t>(b) * T * Hkv * D;
  const ouro_tok_meta* meta = d.meta + static_cast<size_t>(b) * T;
  const int pid_q = meta[t].phrase_id, boff_q = meta[t].branch_off;

  for (int i = lane; i < D; i += 64) q_s[i] = q[i];
  __syncthreads();

  float m = -INFINITY, l = 0.f;
  float acc[DPL];
#pragma unroll
  for (int i = 0; i < DPL; ++i) acc[i] = 0.f;

  for (int base = 0; base < n; base += 64) {
    const int kidx = base + lane;
    bool vis = kidx < n;
    const float* krow = nullptr;
    if (vis) {
      if (kidx < L) {
        krow = kc + static_cast<size_t>(cu0 + kidx) * row_stride + g * head_stride;
      } else {
        const int kk = kidx - L;
        const int pid_k = meta[kk].phrase_id;
        vis = pid_k == 0 ? (kk <= boff_q) : (pid_k == pid_q && kk <= t);
        krow = kb + (static_cast<size_t>(kk) * Hkv + g) * D;
      }
    }
    float s = -INFINITY;
    if (vis) {
      float dot = 0.f;
      const float4* k4 = reinterpret_cast<const float4*>(krow);
#pragma unroll 16
      for (int i = 0; i < D / 4; ++i) {
        const float4 kv = k4[i];
        dot = fmaf(q_s[4 * i + 0], kv.x, dot);
        dot = fmaf(q_s[4 * i + 1], kv.y, dot);
        dot = fmaf(q_s[4 * i + 2], kv.z, dot);
        dot = fmaf(q_s[4 * i + 3], kv.w, dot);
      }
      s = dot * scale;
    }
    float cmax = s;
    for (int off = 32; off >= 1; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off));
    const float m_new = fmaxf(m, cmax);
    if (m_new == -INFINITY) continue;            // nothing visible so far (wave-uniform)
    const float alpha = expf(m - m_new);         // m = -inf -> 0
    const float p = vis ? expf(s - m_new) : 0.f;
    float psum = p;
    for (int off = 32; off >= 1; off >>= 1) psum += __shfl_xor(psum, off);
    l = l * alpha + psum;
    m = m_new;
    __syncthreads();
    p_s[lane] = p;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < DPL; ++i) acc[i] *= alpha;
    // sixteen value rows per round, loaded before any is used (a hidden key has p = 0 and adds nothing; its row is in
    // bounds, the values are finite); keys in ascending order, as a one-by-one loop would take them
    const int cnt = min(64, n - base);
    for (int j0 = 0; j0 < cnt; j0 += 16) {
      float vv[16][DPL], pj[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int j = min(j0 + u, cnt - 1);
        const int kj = base + j;
        const float* vrow = kj < L ? vc + static_cast<size_t>(cu0 + kj) * row_stride + g * head_stride
                                   : vb + (static_cast<size_t>(kj - L) * Hkv + g) * D;
        pj[u] = j0 + u < cnt ? p_s[j] : 0.f;
#pragma unroll
        for (int i = 0; i < DPL; ++i) vv[u][i] = vrow[lane + 64 * i];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u)
#pragma unroll
        for (int i = 0; i < DPL; ++i) acc[i] = fmaf(pj[u], vv[u][i], acc[i]);
    }
  }
  float* out = static_cast<float*>(d.out) + ((static_cast<size_t>(b) * T + t) * Hq + h) * D;
  const float inv = 1.0f / l;
#pragma unroll
  for (int i = 0; i < DPL; ++i) out[lane + 64 * i] = acc[i] * inv;
  if (d.lse && lane == 0) d.lse[(static_cast<size_t>(b) * Hq + h) * T + t] = m + logf(l);
}

}  // namespace

int launch_attn_f32(const ouro_attn_desc& d, float scale, hipStream_t stream) {
  dim3 grid(d.T, d.Hq, d.B);
  if (d.ev_start && hipEventRecord(static_cast<hipEvent_t>(d.ev_start), stream) != hipSuccess) return hip_failed(hipGetLastError());
  if (d.D == 64) hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(64), 0, stream, d, scale);
  else hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(64), 0, stream, d, scale);
  const int st = check_launch();
  if (st == OURO_OK && d.ev_stop && hipEventRecord(static_cast<hipEvent_t>(d.ev_stop), stream) != hipSuccess)
    return hip_failed(hipGetLastError());
  return st;
}

}  // namespace ouro
