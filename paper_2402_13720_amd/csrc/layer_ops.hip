// Small element-wise pieces of the verifying layer around the draft-block attention: positions of the block
// tokens and the rotary embedding that uses them, RMSNorm, and the SwiGLU gate.
//
// Positions are the part the method fixes: every lengthened draft of Eq. (7) is an ordinary linear sequence, so a
// block token sits at (cached tokens of its sequence) + (tokens before it in its own draft): main token i at L + i,
// the i-th block token of a phrase that hangs off main index b at L + b + 1 + i (Sec. 3.2).  The rest is the target
// model's published formulation (rotate-half rotary embedding, RMSNorm, SiLU gate), fp32 arithmetic inside.
//
// All three are bandwidth-trivial (a few MB at most) next to the weight-streaming projections; they are written for
// coalesced 16-byte accesses and nothing else.
#include <math.h>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ float load(const float* p) { return *p; }
  static __device__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<__bf16> {
  static __device__ float load(const __bf16* p) { return static_cast<float>(*p); }
  static __device__ void store(__bf16* p, float v) { *p = static_cast<__bf16>(v); }
};

// Tokens of the block before t in t's own draft.  Phrases are contiguous ascending index ranges of equal ids.
__device__ int depth_of(const ouro_tok_meta* meta, int t) {
  const int pid = meta[t].phrase_id;
  if (pid == 0) return t;
  int within = 0;
  while (t - within - 1 >= 0 && meta[t - within - 1].phrase_id == pid) ++within;
  return meta[t].branch_off + 1 + within;
}

// One workgroup per (sequence, block token); threads sweep (head, rotation pair) of q and then of k.
template <typename T>
__global__ __launch_bounds__(256) void rope_block_kernel(ouro_rope_desc d, float log2_base) {
  const int b = blockIdx.x / d.T, t = blockIdx.x - b * d.T;
  const int L = d.seq_len ? d.seq_len[b] : static_cast<int>(d.cu_seqlens[b + 1] - d.cu_seqlens[b]);
  const int pos = L + depth_of(d.meta + static_cast<size_t>(b) * d.T, t);
  if (d.positions && threadIdx.x == 0) d.positions[blockIdx.x] = pos;
  const int half = d.D / 2;
  T* q = static_cast<T*>(d.q) + static_cast<size_t>(blockIdx.x) * d.Hq * d.D;
  T* k = static_cast<T*>(d.k_blk) + static_cast<size_t>(blockIdx.x) * d.Hkv * d.D;
  const int nq = d.Hq * half, nk = d.Hkv * half;
  for (int p = threadIdx.x; p < nq + nk; p += 256) {
    const bool is_q = p < nq;
    const int pp = is_q ? p : p - nq;
    const int h = pp / half, i = pp - h * half;
    T* x = (is_q ? q : k) + static_cast<size_t>(h) * d.D;
    // angle = pos * base^(-2i/D); the argument can be thousands of radians: full-range sincosf
    const float inv = exp2f(-2.0f * static_cast<float>(i) / static_cast<float>(d.D) * log2_base);
    float s, c;
    sincosf(static_cast<float>(pos) * inv, &s, &c);
    const float x0 = Elem<T>::load(x + i), x1 = Elem<T>::load(x + i + half);
    Elem<T>::store(x + i, x0 * c - x1 * s);
    Elem<T>::store(x + i + half, x1 * c + x0 * s);
  }
}

// One workgroup per row: sum of squares (fp32, fixed reduction order), then scale by the gain.
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(ouro_rmsnorm_desc d) {
  __shared__ float part[4];
  const int r = blockIdx.x;
  const T* x = static_cast<const T*>(d.x) + static_cast<size_t>(r) * d.Hd;
  const T* g = static_cast<const T*>(d.gain);
  T* y = static_cast<T*>(d.out) + static_cast<size_t>(r) * d.Hd;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d.Hd; i += 256) {
    const float v = Elem<T>::load(x + i);
    ss += v * v;
  }
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (part[0] + part[1]) + (part[2] + part[3]);
  const float scale = 1.0f / sqrtf(tot / static_cast<float>(d.Hd) + d.eps);
  for (int i = threadIdx.x; i < d.Hd; i += 256) Elem<T>::store(y + i, Elem<T>::load(x + i) * scale * Elem<T>::load(g + i));
}

// out[r, f] = silu(gate_up[r, f]) * gate_up[r, F + f]
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_kernel(ouro_silu_mul_desc d) {
  const size_t n = static_cast<size_t>(d.R) * d.F;
  const T* gu = static_cast<const T*>(d.gate_up);
  T* out = static_cast<T*>(d.out);
  for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<size_t>(gridDim.x) * 256) {
    const size_t r = i / d.F, f = i - r * d.F;
    const float g = Elem<T>::load(gu + r * 2 * d.F + f), u = Elem<T>::load(gu + r * 2 * d.F + d.F + f);
    Elem<T>::store(out + i, g / (1.0f + expf(-g)) * u);
  }
}

}  // namespace

int launch_rope_block(const ouro_rope_desc& d, hipStream_t stream) {
  const float log2_base = log2f(d.base > 0.f ? d.base : 10000.0f);
  const unsigned grid = static_cast<unsigned>(d.B) * d.T;
  if (d.dtype == OURO_BF16) hipLaunchKernelGGL(rope_block_kernel<__bf16>, dim3(grid), dim3(256), 0, stream, d, log2_base);
  else hipLaunchKernelGGL(rope_block_kernel<float>, dim3(grid), dim3(256), 0, stream, d, log2_base);
  return check_launch();
}

int launch_rmsnorm(const ouro_rmsnorm_desc& d, hipStream_t stream) {
  if (d.dtype == OURO_BF16) hipLaunchKernelGGL(rmsnorm_kernel<__bf16>, dim3(d.R), dim3(256), 0, stream, d);
  else hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(d.R), dim3(256), 0, stream, d);
  return check_launch();
}

int launch_silu_mul(const ouro_silu_mul_desc& d, hipStream_t stream) {
  const size_t n = static_cast<size_t>(d.R) * d.F;
  const unsigned grid = static_cast<unsigned>(std::min<size_t>((n + 255) / 256, 4096));
  if (d.dtype == OURO_BF16) hipLaunchKernelGGL(silu_mul_kernel<__bf16>, dim3(grid), dim3(256), 0, stream, d);
  else hipLaunchKernelGGL(silu_mul_kernel<float>, dim3(grid), dim3(256), 0, stream, d);
  return check_launch();
}

}  // namespace ouro
