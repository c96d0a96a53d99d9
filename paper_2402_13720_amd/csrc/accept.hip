// Acceptance: longest accepted prefix over the main draft and the candidate phrases
// (Eq. (3) for A, Eq. (9) for the per-phrase run, and the selection rule after Eq. (9)).
//
// One 64-lane wave per sequence.  Every lane first decides match[t] for its block
// positions (draft id == greedy token predicted by the row of the preceding token of the
// same lengthened draft).  Lane 0 then walks the main draft, lane j walks phrase j, and a
// wave-wide max over (length, lowest path id) picks the winner.
#include "ouro_internal.hpp"

namespace ouro {

namespace {

constexpr int kMaxT = 128;

__global__ __launch_bounds__(64) void accept_kernel(ouro_accept_desc d) {
  __shared__ unsigned char match[kMaxT];
  __shared__ int32_t tok[kMaxT], arg[kMaxT];            // the sequence's block, staged once: every later lookup is LDS
  __shared__ ouro_tok_meta meta[kMaxT];
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const int T = d.T, gamma = d.gamma, K = d.K, beta = d.beta;
  const bool have_root = d.root_pred != nullptr;
  {
    // all global loads of the kernel are issued here, back to back: one memory round trip
    const int32_t* gtok = d.draft_tok + static_cast<size_t>(b) * T;
    const int32_t* garg = d.argmax + static_cast<size_t>(b) * T;
    const ouro_tok_meta* gmeta = d.meta + static_cast<size_t>(b) * T;
    const int t0 = lane, t1 = lane + 64;
    const int32_t k0 = t0 < T ? gtok[t0] : 0, k1 = t1 < T ? gtok[t1] : 0;
    const int32_t a0 = t0 < T ? garg[t0] : 0, a1 = t1 < T ? garg[t1] : 0;
    const ouro_tok_meta z = {0, 0};
    const ouro_tok_meta m0 = t0 < T ? gmeta[t0] : z, m1 = t1 < T ? gmeta[t1] : z;
    tok[t0] = k0; tok[t1] = k1;
    arg[t0] = a0; arg[t1] = a1;
    meta[t0] = m0; meta[t1] = m1;
  }
  const int32_t root = have_root ? d.root_pred[b] : -1;
  __syncthreads();

  for (int t = lane; t < T; t += 64) {
    int parent;
    if (t < gamma) {
      parent = t - 1;                                   // main draft: previous main token (or the prefix)
    } else {
      const int within = (t - gamma) % beta;
      parent = within == 0 ? static_cast<int>(meta[t].branch_off) : t - 1;
    }
    bool m;
    // a position right after the prefix: checked against root_pred; without one, only main token 0 (declared
    // accepted by the caller) passes, a phrase hanging off the prefix has nothing to be checked against and fails
    if (parent < 0) m = have_root ? (tok[t] == root) : (t == 0);
    else m = tok[t] == arg[parent];
    match[t] = m ? 1 : 0;
  }
  __syncthreads();

  // lane 0: main draft; lane j (1..K): phrase j.
  int run = 0, start = 0, len = 0;
  if (lane == 0) { start = 0; len = gamma; }
  else if (lane <= K) { start = gamma + (lane - 1) * beta; len = beta; }
  while (run < len && match[start + run]) ++run;

  const int A = __shfl(run, 0);
  int bj = -1;
  int total = -1;
  if (lane == 0) total = A;
  else if (lane <= K) {
    bj = meta[start].branch_off;
    if (A >= bj + 1) total = bj + 1 + run;
  }
  // max over lanes of (total, lower lane first): key = total * 64 + (63 - lane); total >= -1.
  int key = (total + 1) * 64 + (63 - lane);
  for (int off = 32; off >= 1; off >>= 1) key = max(key, __shfl_xor(key, off));
  const int win = 63 - (key & 63);
  const int n_acc = (key >> 6) - 1;
  const int win_b = __shfl(bj, win);
  const int win_start = __shfl(start, win);

  // accepted block indices, in order
  const int width = gamma + beta;
  int32_t* idx = d.accept_idx + static_cast<size_t>(b) * width;
  const int n_main = win == 0 ? n_acc : win_b + 1;
  for (int i = lane; i < width; i += 64) {
    int v = -1;
    if (i < n_acc) v = i < n_main ? i : win_start + (i - n_main);
    idx[i] = v;
  }
  if (lane == 0) {
    int last = -1;
    if (n_acc > 0) last = (n_acc <= n_main) ? n_acc - 1 : win_start + (n_acc - n_main) - 1;
    d.n_accept[b] = n_acc;
    d.path[b] = win;
    d.bonus[b] = last >= 0 ? arg[last] : root;
    if (d.main_A) d.main_A[b] = A;
  }
  if (d.phrase_A && lane >= 1 && lane <= K) d.phrase_A[static_cast<size_t>(b) * K + (lane - 1)] = run;
  if (d.n_match) {
    int cnt = 0;
    for (int t = lane; t < gamma; t += 64) cnt += match[t];
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off);
    if (lane == 0) d.n_match[b] = cnt;
  }

  // ---- by-products for the phrase pool (Sec. 3.3) ----
  if (d.match_out)
    for (int t = lane; t < T; t += 64) d.match_out[static_cast<size_t>(b) * T + t] = match[t];
  if (d.n_seg) {
    // maximal runs of matches in the discarded part of the main draft (positions > A; A is the first mismatch)
    const int nmax = max(1, (gamma + 1) / 2);
    int32_t* ss = d.seg_start + static_cast<size_t>(b) * nmax;
    int32_t* sl = d.seg_len + static_cast<size_t>(b) * nmax;
    int base = 0;
    for (int i0 = 0; i0 < gamma; i0 += 64) {
      const int i = i0 + lane;
      const bool is_start = i < gamma && i > A && match[i] && !match[i - 1];
      const unsigned long long starts = __ballot(is_start);
      if (is_start) {
        const int k = base + __popcll(starts & ((1ull << lane) - 1ull));
        int e = i;
        while (e < gamma && match[e]) ++e;
        ss[k] = i;
        sl[k] = e - i;
      }
      base += __popcll(starts);
    }
    for (int k = base + lane; k < nmax; k += 64) { ss[k] = -1; sl[k] = 0; }
    if (lane == 0) d.n_seg[b] = base;
  }
  if (d.repaired && lane >= 1 && lane <= K) {
    // phrase o = lane: its first token (the main-draft token at its branch point) and the target's greedy token
    // at each of its block positions
    int32_t* rp = d.repaired + (static_cast<size_t>(b) * K + (lane - 1)) * (beta + 1);
    const int lo = gamma + (lane - 1) * beta;
    const int bo = meta[lo].branch_off;
    rp[0] = bo >= 0 ? tok[bo] : -1;
    for (int i = 0; i < beta; ++i) rp[1 + i] = i == 0 ? (bo >= 0 ? arg[bo] : root) : arg[lo + i - 1];
  }
}

}  // namespace

int launch_accept(const ouro_accept_desc& d, hipStream_t stream) {
  hipLaunchKernelGGL(accept_kernel, dim3(d.B), dim3(64), 0, stream, d);
  return check_launch();
}

}  // namespace ouro
