// Final draft tree (top-m rerank, order, parents, positions, attention mask), the greedy accept
// walk and sampled acceptance.  One workgroup per sequence; everything is integer work on at most
// DDD_POOL_MAX nodes, so it lives in LDS.
#include "tree_device.hpp"

namespace ddd {

__global__ __launch_bounds__(1024) void tree_finalize_kernel(FinalizeArgs a) {
  __shared__ TreeSmem sm;
  tree_finalize_block(a.st, a.tree, blockIdx.x, a.m, a.nmax, threadIdx.x, blockDim.x, sm);
}

hipError_t launch_tree_finalize(const FinalizeArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(tree_finalize_kernel, dim3(a.B), dim3(1024), 0, stream, a);
  return hipGetLastError();
}

// Section 1 / Section 3.1 (temperature 0): follow the child whose token equals the target's
// argmax at the current node until there is none; the argmax there is the bonus token.
__global__ __launch_bounds__(64) void verify_accept_kernel(VerifyArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int T = a.m + 1;
  const int n = a.tree.n_sel[b] + 1;
  const int32_t* tok = a.tree.tree_token + (size_t)b * T;
  const int32_t* par = a.tree.parent_idx + (size_t)b * T;
  const int32_t* tgt = a.target_argmax + (size_t)b * T;
  int32_t* path = a.accept_path + (size_t)b * (a.D + 1);
  int cur = 0, len = 0;
  if (lane == 0) path[0] = 0;
  for (int it = 0; it < a.D; ++it) {
    const int want = tgt[cur];
    int found = 0x7FFFFFFF;
    for (int c = 1 + lane; c < n; c += 64)
      if (par[c] == cur && tok[c] == want) found = min(found, c);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) found = min(found, __shfl_xor(found, off, 64));
    if (found == 0x7FFFFFFF) break;      // uniform
    cur = found;
    ++len;
    if (lane == 0) path[len] = cur;
  }
  if (lane == 0) {
    for (int i = len + 1; i <= a.D; ++i) path[i] = -1;
    a.accept_len[b] = len;
    a.bonus_token[b] = tgt[cur];
  }
}

hipError_t launch_verify_accept(const VerifyArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(verify_accept_kernel, dim3(a.B), dim3(64), 0, stream, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Sampled acceptance at temperature T > 0.  The paper measures at temperature 0 (Section 3.1) and
// fixes only that the emitted tokens follow the target model's distribution (Section 1).  The
// drafted children of a node are a deterministic function of the context, i.e. point-mass
// proposals: child x is accepted with probability p(x); after a rejection p continues without x,
// renormalised.  With w_j = exp((x_j - max x) / T) kept unnormalised and rem = sum of the
// weights not yet rejected:   accept child c  iff  u_accept[c] * rem < w[token_c];  when no child is
// accepted the bonus token is the first j whose prefix sum of the remaining weights exceeds
// u_bonus[node] * rem.  Every decision is taken in fp64.
//
// One workgroup of 16 waves per sequence; wave w owns the contiguous token segment
// [w*seg, (w+1)*seg) of the current node's logit row (coalesced loads, fixed summation order).
constexpr int kVsWaves = 16;
constexpr int kVsThreads = kVsWaves * kWave;
constexpr int kVsMaxRemoved = 128;     // children of one node <= beam width <= 128

__device__ __forceinline__ double wave_sum_f64(double x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
__device__ __forceinline__ double wave_scan_f64(double x, int lane) {   // inclusive prefix over the lanes
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const double t = __shfl_up(x, off, 64);
    if (lane >= off) x += t;
  }
  return x;
}

__global__ __launch_bounds__(kVsThreads) void verify_sample_kernel(VerifySampleArgs a) {
  __shared__ uint64_t s_key[kVsWaves];
  __shared__ double s_wsum[kVsWaves];
  __shared__ int s_rm_tok[kVsMaxRemoved];
  __shared__ double s_rm_w[kVsMaxRemoved];
  __shared__ int s_next, s_nrm, s_found[kVsWaves];
  __shared__ double s_rem;

  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int T = a.m + 1, V = a.V;
  const int n = min(a.tree.n_sel[b], a.m) + 1;
  const int32_t* tok = a.tree.tree_token + (size_t)b * T;
  const int32_t* par = a.tree.parent_idx + (size_t)b * T;
  int32_t* path = a.accept_path + (size_t)b * (a.D + 1);
  const int seg = ((V + kVsThreads - 1) / kVsThreads) * kWave;
  const int j0 = min(V, wv * seg), j1 = min(V, j0 + seg);
  const double Tt = (double)a.temperature;

  int cur = 0, len = 0, amax = 0;
  double Md = 0.0;
  const float* x = a.logits;
  if (tid == 0) path[0] = 0;

  for (int it = 0; it <= a.D; ++it) {
    x = a.logits + ((size_t)b * T + cur) * V;
    // row maximum (and the lowest token that attains it)
    uint64_t key = 0;
#pragma unroll 4
    for (int j = j0 + lane; j < j1; j += kWave) key = umax64(key, row_key(x[j], j));
    key = wave_max_u64(key);
    if (lane == 0) s_key[wv] = key;
    __syncthreads();
    uint64_t best = 0;
#pragma unroll
    for (int i = 0; i < kVsWaves; ++i) best = umax64(best, s_key[i]);
    Md = (double)key_value(best);
    amax = key_token(best);
    // weights: per-wave sums in a fixed order
    double acc = 0.0;
#pragma unroll 4
    for (int j = j0 + lane; j < j1; j += kWave) acc += exp(((double)x[j] - Md) / Tt);
    acc = wave_sum_f64(acc);
    if (lane == 0) s_wsum[wv] = acc;
    __syncthreads();
    if (wv == 0) {
      double rem = 0.0;
#pragma unroll
      for (int i = 0; i < kVsWaves; ++i) rem += s_wsum[i];
      int nxt = -1, nrm = 0;
      if (len < a.D) {
        for (int base = 1; base < n && nxt < 0; base += kWave) {
          const int c = base + lane;
          uint64_t kids = __ballot(c < n && par[c] == cur);
          while (kids) {
            const int cc = base + __ffsll((unsigned long long)kids) - 1;
            kids &= kids - 1;
            const int tk = min(max(tok[cc], 0), V - 1);
            const double w = exp(((double)x[tk] - Md) / Tt);
            if (a.u_accept[(size_t)b * T + cc] * rem < w) { nxt = cc; break; }
            rem -= w;
            if (lane == 0 && nrm < kVsMaxRemoved) { s_rm_tok[nrm] = tk; s_rm_w[nrm] = w; }
            ++nrm;
          }
        }
      }
      if (lane == 0) { s_next = nxt; s_rem = rem; s_nrm = min(nrm, kVsMaxRemoved); }
    }
    __syncthreads();
    const int nxt = s_next;
    if (nxt < 0) break;
    cur = nxt;
    ++len;
    if (tid == 0) path[len] = cur;
  }

  // Bonus token at `cur` (x, Md, amax, s_wsum, s_rm_* describe that node).
  const int nrm = s_nrm;
  const double thr = a.u_bonus[(size_t)b * T + cur] * s_rem;
  double pre = 0.0;               // remaining weight of the waves before this one
  for (int i = 0; i < wv; ++i) {
    double v = s_wsum[i];
    for (int r = 0; r < nrm; ++r)
      if (s_rm_tok[r] / seg == i) v -= s_rm_w[r];
    pre += v;
  }
  int found = 0x7FFFFFFF;
  double run = pre;
  for (int jb = j0; jb < j1; jb += kWave) {
    const int j = jb + lane;
    double w = 0.0;
    if (j < j1) {
      w = exp(((double)x[j] - Md) / Tt);
      for (int r = 0; r < nrm; ++r)
        if (s_rm_tok[r] == j) w = 0.0;
    }
    const double inc = wave_scan_f64(w, lane);
    const uint64_t over = __ballot(j < j1 && run + inc > thr);
    if (over != 0 && found == 0x7FFFFFFF) found = jb + __ffsll((unsigned long long)over) - 1;
    run += __shfl(inc, 63, 64);
  }
  if (lane == 0) s_found[wv] = found;
  __syncthreads();
  int bonus = 0x7FFFFFFF;
#pragma unroll
  for (int i = 0; i < kVsWaves; ++i) bonus = min(bonus, s_found[i]);
  if (bonus == 0x7FFFFFFF) {
    // rounding left no prefix above the threshold: the last token that still has weight, and if
    // the children covered everything the target's most likely token  (uniform branch)
    int last = -1;
    for (int j = j0 + lane; j < j1; j += kWave) {
      bool live = exp(((double)x[j] - Md) / Tt) > 0.0;
      for (int r = 0; r < nrm; ++r)
        if (s_rm_tok[r] == j) live = false;
      if (live) last = max(last, j);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) last = max(last, __shfl_xor(last, off, 64));
    __syncthreads();                 // every thread has read s_found
    if (lane == 0) s_found[wv] = last;
    __syncthreads();
    last = -1;
#pragma unroll
    for (int i = 0; i < kVsWaves; ++i) last = max(last, s_found[i]);
    bonus = last >= 0 ? last : amax;
  }
  if (tid == 0) {
    for (int i = len + 1; i <= a.D; ++i) path[i] = -1;
    a.accept_len[b] = len;
    a.bonus_token[b] = bonus;
  }
}

hipError_t launch_verify_sample(const VerifySampleArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(verify_sample_kernel, dim3(a.B), dim3(kVsThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
