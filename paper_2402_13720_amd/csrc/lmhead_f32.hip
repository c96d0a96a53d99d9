// fp32 LM head with fused arg-max (correctness-grade path), and the cross-slab reduction
// shared by every LM-head variant.
//
// logits[r, v] = sum_k hidden[r, k] * w[v, k]  (Eq. (2): the target's next-token scores for
// every block row), greedy pick per row, lowest token id on ties.  A workgroup owns a slab
// of vocabulary rows; each of its 4 waves takes slab/4 of them and, for every hidden row of
// its grid.y slice, forms the dot product with lanes striding over k.  Only one
// (best value, best index) pair per (slab, row) leaves the kernel; a second tiny kernel
// reduces over slabs.
#include <math.h>

#include "ouro_internal.hpp"

namespace ouro {

namespace {

// (value, index) order used everywhere: larger value wins, equal values -> smaller index.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ __launch_bounds__(256) void lmhead_f32_kernel(ouro_lmhead_desc d, int slab, int rtile, float2* part) {
  extern __shared__ float smem[];                 // [4 waves][rtile] value, then [4 waves][rtile] index
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int R = d.R, Hd = d.Hd, V = d.V;
  const int r0 = blockIdx.y * rtile;
  const int nr = min(rtile, R - r0);
  float* best_v = smem + wave * rtile;
  int* best_i = reinterpret_cast<int*>(smem + 4 * rtile) + wave * rtile;
  for (int r = lane; r < nr; r += 64) { best_v[r] = -INFINITY; best_i[r] = 0x7fffffff; }
  const float* hidden = static_cast<const float*>(d.hidden);
  const float* w = static_cast<const float*>(d.w);
  const int per_wave = slab / 4;
  const int v_lo = blockIdx.x * slab + wave * per_wave;
  // Four hidden rows at a time against one vocabulary row: their loads are independent, so one memory round trip
  // serves four dot products and the four cross-lane sums overlap (each dot product keeps its own order of operations).
  for (int v = v_lo; v < min(v_lo + per_wave, V); ++v) {
    const float4* wrow = reinterpret_cast<const float4*>(w + static_cast<size_t>(v) * Hd);
    for (int rb = 0; rb < nr; rb += 4) {
      const float4* hrow[4];
      float dot[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        hrow[u] = reinterpret_cast<const float4*>(hidden + static_cast<size_t>(r0 + min(rb + u, nr - 1)) * Hd);
        dot[u] = 0.f;
      }
      for (int i = lane; i < Hd / 4; i += 64) {
        const float4 c = wrow[i];
        float4 a4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a4[u] = hrow[u][i];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          dot[u] = fmaf(a4[u].x, c.x, dot[u]);
          dot[u] = fmaf(a4[u].y, c.y, dot[u]);
          dot[u] = fmaf(a4[u].z, c.z, dot[u]);
          dot[u] = fmaf(a4[u].w, c.w, dot[u]);
        }
      }
      for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
        for (int u = 0; u < 4; ++u) dot[u] += __shfl_xor(dot[u], off);
      }
      if (lane == 0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = rb + u;
          if (r < nr && dot[u] > best_v[r]) { best_v[r] = dot[u]; best_i[r] = v; }   // v ascending: strict > keeps the lowest id
        }
      }
    }
  }
  __syncthreads();
  for (int r = threadIdx.x; r < nr; r += 256) {
    float bv = smem[r];
    int bi = reinterpret_cast<int*>(smem + 4 * rtile)[r];
    for (int wv = 1; wv < 4; ++wv) {
      const float v2 = smem[wv * rtile + r];
      const int i2 = reinterpret_cast<int*>(smem + 4 * rtile)[wv * rtile + r];
      if (better(v2, i2, bv, bi)) { bv = v2; bi = i2; }
    }
    part[static_cast<size_t>(blockIdx.x) * R + r0 + r] = make_float2(bv, __int_as_float(bi));
  }
}

// part [nslab][R] -> argmax_out[R], max_out[R].  One wave per row, lanes stride over slabs.
__global__ __launch_bounds__(256) void lmhead_final_kernel(const float2* part, int nslab, int R, int32_t* arg_out,
                                                           float* max_out) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= R) return;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  // loads in batches of 8 independent ones (one memory round trip per 512 slabs, not one per 64)
  for (int s0 = lane; s0 < nslab; s0 += 64 * 8) {
    float2 p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = s0 + 64 * u;
      p[u] = s < nslab ? part[static_cast<size_t>(s) * R + r] : make_float2(-INFINITY, __int_as_float(0x7fffffff));
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = __float_as_int(p[u].y);
      if (better(p[u].x, i, bv, bi)) { bv = p[u].x; bi = i; }
    }
  }
  for (int off = 32; off >= 1; off >>= 1) {
    const float ov = __shfl_xor(bv, off);
    const int oi = __shfl_xor(bi, off);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if (lane == 0) {
    arg_out[r] = bi;
    if (max_out) max_out[r] = bv;
  }
}

}  // namespace

int launch_lmhead_f32(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream) {
  dim3 grid(plan.nslab, plan.nrtile);
  const size_t smem = static_cast<size_t>(plan.rtile) * 4 * 2 * sizeof(float);
  hipLaunchKernelGGL(lmhead_f32_kernel, grid, dim3(256), smem, stream, d, plan.slab, plan.rtile,
                     static_cast<float2*>(d.workspace));
  return check_launch();
}

int launch_lmhead_final(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream) {
  hipLaunchKernelGGL(lmhead_final_kernel, dim3((d.R + 3) / 4), dim3(256), 0, stream,
                     static_cast<const float2*>(d.workspace),
                     plan.nslab, d.R, d.argmax_out, d.max_out);
  return check_launch();
}

}  // namespace ouro
