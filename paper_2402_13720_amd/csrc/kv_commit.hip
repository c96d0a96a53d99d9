// Commit of the accepted tokens: the keys/values of the accepted block tokens move to the tail of each
// sequence's cached tokens (the sentence after Eq. (3) and the rule after Eq. (9): the accepted draft is kept,
// every other block token is dropped).
//
// Pure data movement, a few hundred KB at most: one workgroup per (sequence, accepted slot) copies one K row
// and one V row (Hkv * D elements each) with 16-byte loads and stores; workgroups of slots past n_accept exit.
// The lengths are bumped by a second one-block kernel, so that no copy workgroup can read a length that
// another one has already advanced.
#include "ouro_internal.hpp"

namespace ouro {

namespace {

typedef unsigned __attribute__((ext_vector_type(4))) u32x4;

struct CommitArgs {
  const unsigned char* k_blk;
  const unsigned char* v_blk;
  const int32_t* accept_idx;
  const int32_t* n_accept;
  unsigned char* k_cache;
  unsigned char* v_cache;
  const int64_t* cu;
  int32_t* seq_len;
  int32_t* overflow;
  int B, T, max_accept;
  unsigned row_bytes;          // Hkv * D * element size, multiple of 16
  unsigned head_bytes;         // D * element size
  size_t cache_rows;           // 0: cache is [rows, Hkv, D]; else [Hkv, cache_rows, D]
};

__device__ __forceinline__ bool fits(const CommitArgs& a, int b, int have, int na) {
  return static_cast<long>(have) + na <= a.cu[b + 1] - a.cu[b];
}

__global__ __launch_bounds__(256) void kv_commit_copy_kernel(CommitArgs a) {
  const int b = blockIdx.x / a.max_accept, i = blockIdx.x - b * a.max_accept;
  const int na = a.n_accept[b];
  if (i >= na) return;
  const int have = a.seq_len[b];
  if (!fits(a, b, have, na)) return;
  const int t = a.accept_idx[b * a.max_accept + i];
  if (t < 0 || t >= a.T) return;                       // contract violation: never index outside the block
  const size_t src = (static_cast<size_t>(b) * a.T + t) * a.row_bytes;
  const size_t row = static_cast<size_t>(a.cu[b] + have + i);
  for (unsigned off = threadIdx.x * 16u; off < a.row_bytes; off += 256u * 16u) {
    size_t dst = row * a.row_bytes + off;
    if (a.cache_rows) {                                // head-major cache: head g of this row lives at [g][row]
      const unsigned g = off / a.head_bytes;
      dst = (g * a.cache_rows + row) * a.head_bytes + (off - g * a.head_bytes);
    }
    *reinterpret_cast<u32x4*>(a.k_cache + dst) = *reinterpret_cast<const u32x4*>(a.k_blk + src + off);
    *reinterpret_cast<u32x4*>(a.v_cache + dst) = *reinterpret_cast<const u32x4*>(a.v_blk + src + off);
  }
}

__global__ __launch_bounds__(256) void kv_commit_len_kernel(CommitArgs a) {
  for (int b = blockIdx.x * 256 + threadIdx.x; b < a.B; b += gridDim.x * 256) {
    const int na = a.n_accept[b], have = a.seq_len[b];
    const bool ok = fits(a, b, have, na);
    if (ok) a.seq_len[b] = have + na;
    a.overflow[b] = ok ? 0 : 1;
  }
}

}  // namespace

int launch_kv_commit(const ouro_kv_commit_desc& d, hipStream_t stream) {
  CommitArgs a{};
  a.k_blk = static_cast<const unsigned char*>(d.k_blk);
  a.v_blk = static_cast<const unsigned char*>(d.v_blk);
  a.accept_idx = d.accept_idx;
  a.n_accept = d.n_accept;
  a.k_cache = static_cast<unsigned char*>(d.k_cache);
  a.v_cache = static_cast<unsigned char*>(d.v_cache);
  a.cu = d.cu_seqlens;
  a.seq_len = d.seq_len;
  a.overflow = d.overflow;
  a.B = d.B;
  a.T = d.T;
  a.max_accept = d.max_accept;
  a.row_bytes = static_cast<unsigned>(d.Hkv) * d.D * (d.dtype == OURO_BF16 ? 2u : 4u);
  a.head_bytes = static_cast<unsigned>(d.D) * (d.dtype == OURO_BF16 ? 2u : 4u);
  a.cache_rows = d.kv_layout == OURO_KV_HEAD_MAJOR ? static_cast<size_t>(d.cache_rows) : 0;
  hipLaunchKernelGGL(kv_commit_copy_kernel, dim3(static_cast<unsigned>(d.B) * d.max_accept), dim3(256), 0, stream, a);
  int st = check_launch();
  if (st != OURO_OK) return st;
  hipLaunchKernelGGL(kv_commit_len_kernel, dim3(static_cast<unsigned>((d.B + 255) / 256)), dim3(256), 0, stream, a);
  return check_launch();
}

}  // namespace ouro
