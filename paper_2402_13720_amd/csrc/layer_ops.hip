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
  __shared__ ouro_tok_meta smeta[128];                  // the sequence's block metadata: the walk below stays in LDS
  const int b = blockIdx.x / d.T, t = blockIdx.x - b * d.T;
  for (int i = threadIdx.x; i <= t; i += 256) smeta[i] = d.meta[static_cast<size_t>(b) * d.T + i];
  const int L = d.seq_len ? d.seq_len[b] : static_cast<int>(d.cu_seqlens[b + 1] - d.cu_seqlens[b]);
  __syncthreads();
  const int pos = L + depth_of(smeta, t);
  if (d.positions && threadIdx.x == 0) d.positions[blockIdx.x] = pos;
  const int half = d.D / 2;
  T* q = static_cast<T*>(d.q) + static_cast<size_t>(blockIdx.x) * d.Hq * d.D;
  T* k = static_cast<T*>(d.k_blk) + static_cast<size_t>(blockIdx.x) * d.Hkv * d.D;
  // sources: the operands themselves (in place), or this token's row of a fused projection [q heads | k heads | v heads]
  const T* row = d.qkv ? static_cast<const T*>(d.qkv) + static_cast<size_t>(blockIdx.x) * (d.Hq + 2 * d.Hkv) * d.D : nullptr;
  const T* qs = row ? row : q;
  const T* ks = row ? row + static_cast<size_t>(d.Hq) * d.D : k;
  // angle = pos * base^(-2i/D) can be thousands of radians: it is formed and reduced to [-pi, pi] in fp64
  // (a handful of fp64 operations per pair), after which the fast fp32 sine/cosine are accurate to ~1e-6
#define OURO_ROPE_SINCOS(I, S, C)                                                                              \
  {                                                                                                            \
    const float inv_ = exp2f(-2.0f * static_cast<float>(I) / static_cast<float>(d.D) * log2_base);             \
    const double ang_ = static_cast<double>(pos) * static_cast<double>(inv_);                                  \
    const float red_ = static_cast<float>(ang_ - 6.283185307179586 * rint(ang_ * 0.15915494309189535));        \
    S = __sinf(red_);                                                                                          \
    C = __cosf(red_);                                                                                          \
  }
  typedef T vec8 __attribute__((ext_vector_type(8)));
  const bool vec = half % 8 == 0 && ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) |
                                      reinterpret_cast<uintptr_t>(qs) | reinterpret_cast<uintptr_t>(ks)) & 15) == 0;
  if (vec) {
    // work item = 8 consecutive rotation pairs of one head: two 16-byte (bf16) vectors in, two out
    const int per_head = half / 8;
    const int nq = d.Hq * per_head, nk = d.Hkv * per_head;
    for (int p = threadIdx.x; p < nq + nk; p += 256) {
      const bool is_q = p < nq;
      const int pp = is_q ? p : p - nq;
      const int h = pp / per_head, i0 = (pp - h * per_head) * 8;
      T* x = (is_q ? q : k) + static_cast<size_t>(h) * d.D + i0;
      const T* xs = (is_q ? qs : ks) + static_cast<size_t>(h) * d.D + i0;
      const vec8 a = *reinterpret_cast<const vec8*>(xs), bb = *reinterpret_cast<const vec8*>(xs + half);
      vec8 oa, ob;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float sn, cs;
        OURO_ROPE_SINCOS(i0 + e, sn, cs)
        const float x0 = static_cast<float>(a[e]), x1 = static_cast<float>(bb[e]);
        oa[e] = static_cast<T>(x0 * cs - x1 * sn);
        ob[e] = static_cast<T>(x1 * cs + x0 * sn);
      }
      *reinterpret_cast<vec8*>(x) = oa;
      *reinterpret_cast<vec8*>(x + half) = ob;
    }
  } else {
    const int nq = d.Hq * half, nk = d.Hkv * half;
    for (int p = threadIdx.x; p < nq + nk; p += 256) {
      const bool is_q = p < nq;
      const int pp = is_q ? p : p - nq;
      const int h = pp / half, i = pp - h * half;
      T* x = (is_q ? q : k) + static_cast<size_t>(h) * d.D;
      const T* xs = (is_q ? qs : ks) + static_cast<size_t>(h) * d.D;
      float sn, cs;
      OURO_ROPE_SINCOS(i, sn, cs)
      const float x0 = Elem<T>::load(xs + i), x1 = Elem<T>::load(xs + i + half);
      Elem<T>::store(x + i, x0 * cs - x1 * sn);
      Elem<T>::store(x + i + half, x1 * cs + x0 * sn);
    }
  }
#undef OURO_ROPE_SINCOS
  if (row) {
    // the value heads of the fused row are copied as they are
    const T* vs = row + static_cast<size_t>(d.Hq + d.Hkv) * d.D;
    T* v = static_cast<T*>(d.v_blk) + static_cast<size_t>(blockIdx.x) * d.Hkv * d.D;
    const int n = d.Hkv * d.D;
    if (n % 8 == 0 && ((reinterpret_cast<uintptr_t>(vs) | reinterpret_cast<uintptr_t>(v)) & 15) == 0) {
      for (int i = threadIdx.x * 8; i < n; i += 256 * 8) *reinterpret_cast<vec8*>(v + i) = *reinterpret_cast<const vec8*>(vs + i);
    } else {
      for (int i = threadIdx.x; i < n; i += 256) v[i] = vs[i];
    }
  }
}

// One workgroup per row: sum of squares (fp32, fixed reduction order), then scale by the gain.  The row is read
// once, 8 elements (16 or 32 bytes) per thread and step, and kept in registers when it fits (Hd <= 8192).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(ouro_rmsnorm_desc d) {
  __shared__ float part[4];
  constexpr int kKeep = 4;                                // steps of 2048 elements held in registers
  const int r = blockIdx.x;
  const T* x = static_cast<const T*>(d.x) + static_cast<size_t>(r) * d.Hd;
  const T* g = static_cast<const T*>(d.gain);
  T* y = static_cast<T*>(d.out) + static_cast<size_t>(r) * d.Hd;
  const bool vec = d.Hd % 8 == 0 && d.Hd <= kKeep * 2048 &&
                   ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(y)) & 15) == 0;
  typedef T vec8 __attribute__((ext_vector_type(8)));
  vec8 keep[kKeep];
  float ss = 0.f;
  if (vec) {
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
      const int i = (k * 256 + threadIdx.x) * 8;
      if (i < d.Hd) {
        keep[k] = *reinterpret_cast<const vec8*>(x + i);
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float v = static_cast<float>(keep[k][e]); ss += v * v; }
      }
    }
  } else {
    for (int i = threadIdx.x; i < d.Hd; i += 256) {
      const float v = Elem<T>::load(x + i);
      ss += v * v;
    }
  }
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (part[0] + part[1]) + (part[2] + part[3]);
  const float scale = 1.0f / sqrtf(tot / static_cast<float>(d.Hd) + d.eps);
  if (vec) {
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
      const int i = (k * 256 + threadIdx.x) * 8;
      if (i < d.Hd) {
        const vec8 gv = *reinterpret_cast<const vec8*>(g + i);
        vec8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = static_cast<T>(static_cast<float>(keep[k][e]) * scale * static_cast<float>(gv[e]));
        *reinterpret_cast<vec8*>(y + i) = o;
      }
    }
  } else {
    for (int i = threadIdx.x; i < d.Hd; i += 256) Elem<T>::store(y + i, Elem<T>::load(x + i) * scale * Elem<T>::load(g + i));
  }
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

// ---- load-time re-layouts of projection weights (run once per weight; 16 bytes = 8 bf16 per thread) ----
typedef __bf16 wvec8 __attribute__((ext_vector_type(8)));

// out[n, k] = bf16(w[n, k] * gain[k]): the gain of an RMSNorm folded into the projection that follows it
__global__ __launch_bounds__(256) void fold_gain_kernel(const __bf16* __restrict__ w, const __bf16* __restrict__ gain,
                                                        __bf16* __restrict__ out, size_t n8, int k8) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i >= n8) return;
  const wvec8 x = reinterpret_cast<const wvec8*>(w)[i];
  const wvec8 g = reinterpret_cast<const wvec8*>(gain)[i % k8];
  wvec8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(static_cast<float>(x[e]) * static_cast<float>(g[e]));
  reinterpret_cast<wvec8*>(out)[i] = o;
}

// out[2j] = gate[j], out[2j+1] = up[j]: a lane of the projection kernel then holds both pre-activations of feature j
__global__ __launch_bounds__(256) void interleave_rows_kernel(const __bf16* __restrict__ gate, const __bf16* __restrict__ up,
                                                              __bf16* __restrict__ out, size_t n8, int k8) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;   // index into out, in 16-byte units
  if (i >= n8) return;
  const size_t row = i / k8, c = i - row * k8;
  const __bf16* src = (row & 1) ? up : gate;
  reinterpret_cast<wvec8*>(out)[i] = reinterpret_cast<const wvec8*>(src)[(row >> 1) * k8 + c];
}

}  // namespace

int launch_fold_rmsnorm_gain(const void* w, const void* gain, void* out, int N, int K, hipStream_t stream) {
  const size_t n8 = static_cast<size_t>(N) * K / 8;
  hipLaunchKernelGGL(fold_gain_kernel, dim3(static_cast<unsigned>((n8 + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const __bf16*>(w), static_cast<const __bf16*>(gain), static_cast<__bf16*>(out), n8, K / 8);
  return check_launch();
}

int launch_interleave_gate_up(const void* w_gate, const void* w_up, void* out, int F, int K, hipStream_t stream) {
  const size_t n8 = static_cast<size_t>(2) * F * K / 8;
  hipLaunchKernelGGL(interleave_rows_kernel, dim3(static_cast<unsigned>((n8 + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const __bf16*>(w_gate), static_cast<const __bf16*>(w_up), static_cast<__bf16*>(out), n8, K / 8);
  return check_launch();
}

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
