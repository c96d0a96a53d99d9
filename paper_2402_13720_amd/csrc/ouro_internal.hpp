// Internal declarations shared by the translation units of libouro (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "ouro.h"

namespace ouro {

// Records a failed HIP call for ouro_last_hip_error() and returns OURO_E_HIP.
int hip_failed(hipError_t e);

inline int check_launch() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? OURO_OK : hip_failed(e);
}

// One-time set-up per device, thread-safe: a kernel's dynamic shared-memory limit is an attribute of the function on
// one device, so it is raised on the first launch on each device and never again.  `init` returns an OURO status;
// a failed set-up is reported by every later call on that device as well.
constexpr int kMaxDevices = 64;
struct DeviceOnce {
  std::once_flag flag[kMaxDevices];
  int status[kMaxDevices];
};
template <typename F>
int device_once(DeviceOnce& s, F&& init) {
  int dev = 0;
  const hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_failed(e);
  if (dev < 0 || dev >= kMaxDevices) return init();        // beyond the table: set the attributes on every call
  std::call_once(s.flag[dev], [&] { s.status[dev] = init(); });
  return s.status[dev];
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Division by a divisor the host knows: floor(n / d) = (mulhi(n, mul) + n) >> shift for every 0 <= n < 2^31 (the
// multiply-and-shift form of division by an invariant integer; shift = ceil(log2 d)).  A kernel that decodes its
// workgroup id into (sequence, head, chunk, row block) pays two instructions per division instead of the ~25 of the
// generic expansion, all of which sat in front of its first memory access.
struct FastDiv {
  unsigned mul, shift;
};
inline FastDiv make_fastdiv(unsigned d) {
  unsigned l = 0;
  while ((1u << l) < d) ++l;
  const unsigned long long m = ((1ull << 32) * ((1ull << l) - d)) / d + 1;
  return FastDiv{static_cast<unsigned>(m), l};
}
__device__ __forceinline__ int fdiv(int n, FastDiv f) {
  return static_cast<int>((__umulhi(static_cast<unsigned>(n), f.mul) + static_cast<unsigned>(n)) >> f.shift);
}

// ---- attention ------------------------------------------------------------------------
// Launch plan of the bf16 split-KV kernel, derived on the host from shapes only.
struct AttnPlan {
  int rw;          // 32-row query blocks per workgroup: 1 (waves split the keys), 2 or 4 (waves split the rows)
  int waves;       // waves per workgroup: 4, or 8 (with rw = 4: two key groups per row block, two waves per SIMD)
  int rows_wg;     // query rows per workgroup: 32 * rw
  int nrb;         // row blocks per (sequence, KV head): ceil(T * G / rows_wg)
  int chunk;       // keys per workgroup (multiple of 128: four 32-key tiles, one per wave, at a time)
  int nch;         // chunk slots per sequence: ceil((max_seqlen + T) / chunk)
  size_t part_ml_bytes;  // fp32 (max, sum) pairs
  size_t part_o_bytes;   // fp32 partial outputs
  size_t total() const { return part_ml_bytes + part_o_bytes; }
};
AttnPlan plan_attn_bf16(const ouro_attn_desc& d);

int launch_attn_bf16(const ouro_attn_desc& d, const AttnPlan& plan, float scale, hipStream_t stream);
int launch_attn_f32(const ouro_attn_desc& d, float scale, hipStream_t stream);

// ---- LM head --------------------------------------------------------------------------
struct LmPlan {
  int variant;     // 0: fp32 VALU, 1: bf16 streaming (R tile 64), 2: bf16 streaming (R tile 128), 3: bf16 large tile
  int slab;        // vocabulary rows per workgroup
  int nslab;       // ceil(V / slab)
  int rtile;       // rows per grid.y slice
  int nrtile;
  size_t part_bytes;     // [nslab][R] (float value, int32 index) pairs
  size_t total() const { return part_bytes; }
};

LmPlan plan_lmhead(const ouro_lmhead_desc& d);
int validate_lmhead(const ouro_lmhead_desc* d, bool need_pointers);
int enqueue_lmhead(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);
int launch_lmhead_bf16(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);
int launch_lmhead_bf16_tile(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);
int launch_lmhead_f32(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);
int launch_pack_w(const void* src, void* dst, int V, int Hd, hipStream_t stream);
int launch_lmhead_final(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);

// ---- acceptance, commit ---------------------------------------------------------------
int launch_accept(const ouro_accept_desc& d, hipStream_t stream);
int launch_kv_commit(const ouro_kv_commit_desc& d, hipStream_t stream);

// ---- the rest of the verifying layer ---------------------------------------------------
int launch_rope_block(const ouro_rope_desc& d, hipStream_t stream);
int launch_rmsnorm(const ouro_rmsnorm_desc& d, hipStream_t stream);
int launch_silu_mul(const ouro_silu_mul_desc& d, hipStream_t stream);
int launch_linear_bf16(const ouro_linear_desc& d, hipStream_t stream);
size_t linear_workspace_bytes(int R, int K, int N, int ksplit_override);
int launch_fold_rmsnorm_gain(const void* w, const void* gain, void* out, int N, int K, hipStream_t stream);
int launch_interleave_gate_up(const void* w_gate, const void* w_up, void* out, int F, int K, hipStream_t stream);

}  // namespace ouro
