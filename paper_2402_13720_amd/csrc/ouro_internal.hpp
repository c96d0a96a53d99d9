// Internal declarations shared by the translation units of libouro (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ouro.h"

namespace ouro {

// Records a failed HIP call for ouro_last_hip_error() and returns OURO_E_HIP.
int hip_failed(hipError_t e);

inline int check_launch() {
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? OURO_OK : hip_failed(e);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- cross-workgroup hand-over without cache flushes ------------------------------------
// Partials that one workgroup writes and another (on any XCD) reads are moved with relaxed
// agent-scope atomic 64-bit accesses: each is a single store/load that is coherent at device
// level, so no L2 write-back or invalidate (which would evict the streamed operands of every
// other workgroup) is needed.  Order: writers store, wait for completion (workgroup-scope
// release = wait on the memory counter), barrier, one relaxed agent-scope ticket increment;
// the workgroup that draws the last ticket then reads with the same kind of loads.
#if defined(__HIPCC__)
__device__ __forceinline__ void st_agent_u64(void* p, unsigned long long v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_agent_u64(const void* p) {
  return __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent_f2(float* p, float x, float y) {
  st_agent_u64(p, (static_cast<unsigned long long>(__float_as_uint(y)) << 32) | __float_as_uint(x));
}
__device__ __forceinline__ void ld_agent_f2(const float* p, float& x, float& y) {
  const unsigned long long v = ld_agent_u64(p);
  x = __uint_as_float(static_cast<unsigned>(v));
  y = __uint_as_float(static_cast<unsigned>(v >> 32));
}
// Called by every thread after its partial stores and before the workgroup barrier that precedes the ticket.
__device__ __forceinline__ void partials_written() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }
__device__ __forceinline__ unsigned take_ticket(unsigned* counter) {
  return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void reset_ticket(unsigned* counter) {
  __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
#endif

// ---- attention ------------------------------------------------------------------------
// Launch plan of the bf16 split-KV kernel, derived on the host from shapes only.
struct AttnPlan {
  int qt;          // 32-row query tiles per wave (1 or 2)
  int rows_wg;     // query rows per workgroup: 32 * qt
  int nrb;         // row blocks per (sequence, KV head): ceil(T * G / rows_wg)
  int chunk;       // keys per workgroup (multiple of 128: the 4 waves take 32-key tiles round-robin)
  int nch;         // chunk slots per sequence: ceil((max_seqlen + T) / chunk)
  size_t counter_bytes;  // ticket counters, one per (sequence, KV head, row block); zero between calls
  size_t part_ml_bytes;  // fp32 (max, sum) pairs
  size_t part_o_bytes;   // fp32 partial outputs
  size_t total() const { return counter_bytes + part_ml_bytes + part_o_bytes; }
};
AttnPlan plan_attn_bf16(const ouro_attn_desc& d);

int launch_attn_bf16(const ouro_attn_desc& d, const AttnPlan& plan, float scale, hipStream_t stream);
int launch_attn_f32(const ouro_attn_desc& d, float scale, hipStream_t stream);

// ---- LM head --------------------------------------------------------------------------
struct LmPlan {
  int variant;     // 0: fp32 VALU, 1: bf16 skinny (R tile 64), 2: bf16 skinny (R tile 128)
  int slab;        // vocabulary rows per workgroup
  int nslab;       // ceil(V / slab)
  int rtile;       // rows per grid.y slice
  int nrtile;
  size_t counter_bytes;  // ticket counters, one per grid.y slice; zero between calls
  size_t part_bytes;     // [nslab][R] (float value, int32 index) pairs
  size_t total() const { return counter_bytes + part_bytes; }
};

// Bytes at the start of every workspace that hold ticket counters at most.
constexpr size_t kMaxCounterBytes = 1u << 20;
int launch_zero_fill(void* p, size_t bytes, hipStream_t stream);
LmPlan plan_lmhead(const ouro_lmhead_desc& d);
int launch_lmhead_bf16(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);
int launch_lmhead_f32(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);
int launch_lmhead_final(const ouro_lmhead_desc& d, const LmPlan& plan, hipStream_t stream);

// ---- acceptance -----------------------------------------------------------------------
int launch_accept(const ouro_accept_desc& d, hipStream_t stream);

}  // namespace ouro
