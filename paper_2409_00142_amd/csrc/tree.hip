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

// Round statistics (Section 3.3 / Table 1: accepted length per round; Section 2: draft calls per round), added by
// the one thread per sequence that has the sequence's accepted length.  That thread calls stats_begin before its
// walk: the sequence's depth is read and goes into the round's running maximum while the walk runs, so that the end
// of the walk waits for nothing.  The sequence that arrives last closes the round: every sequence's depth has gone
// into the maximum before its arrival (the arrival's operand depends on the value the maximum returned, so the
// two atomics cannot pass each other), and the two words are zero again when the launch ends.  A batch of one has
// nothing to agree on.  Every update is an integer atomic without a returned value where none is needed.
struct StatsPre {
  int d;
  unsigned before;
};
__device__ __forceinline__ StatsPre stats_begin(const StatsArgs& s, int b, int B) {
  StatsPre p{0, 0u};
  if (s.sync == nullptr) return p;
  if (s.steps != nullptr) p.d = min(max(s.steps[b], 0), 31);
  if (B > 1) p.before = atomicMax(s.sync + 1, (unsigned)p.d);
  return p;
}
__device__ __forceinline__ void stats_end(const StatsArgs& s, const StatsPre& p, int B, int len) {
  if (s.sync == nullptr) return;
  typedef unsigned long long u64;
  if (s.accept_hist != nullptr) atomicAdd(reinterpret_cast<u64*>(s.accept_hist + min(max(len, 0), 31)), 1ull);
  if (s.depth_hist != nullptr && s.steps != nullptr) atomicAdd(reinterpret_cast<u64*>(s.depth_hist + p.d), 1ull);
  unsigned deepest = (unsigned)p.d;
  if (B > 1) {
    unsigned one = 1u;
    asm volatile("" : "+v"(one) : "v"(p.before));
    if (atomicAdd(s.sync, one) != (unsigned)(B - 1)) return;
    deepest = atomicExch(s.sync + 1, 0u);
    atomicExch(s.sync, 0u);
  }
  if (s.batch_depth_hist != nullptr && s.steps != nullptr) atomicAdd(reinterpret_cast<u64*>(s.batch_depth_hist + deepest), 1ull);
  if (s.rounds != nullptr) atomicAdd(reinterpret_cast<u64*>(s.rounds), 1ull);
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
  StatsPre sp{0, 0u};
  if (lane == 0) {
    path[0] = 0;
    sp = stats_begin(a.stats, b, a.B);
  }
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
    stats_end(a.stats, sp, a.B, len);
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
// One workgroup of 16 waves per sequence walks the accepted path.  Per node, one pass for the row
// maximum and one for the weights: the row is cut into 128 blocks of consecutive tokens (8 per
// wave, coalesced loads, fixed summation order) whose sums stay in LDS, so the bonus draw only has
// to look inside the one block in which the prefix sum passes the threshold.
constexpr int kVsWaves = 16;
constexpr int kVsThreads = kVsWaves * kWave;
constexpr int kVsSubPerWave = 8;
constexpr int kVsSub = kVsWaves * kVsSubPerWave;     // 128 = two per lane of the wave that draws the bonus
constexpr int kVsMaxRemoved = 128;                   // children of one node <= beam width <= 128

// exp(a) for a <= 0 to about 1e-14 relative: a = n ln2 + r, |r| <= ln2 / 2, Taylor polynomial of
// degree 11 in r (remainder below 7e-15), scaled by 2^n.  Arguments below -800 give 0.  Every
// instruction of a 64-wide wave costs four cycles here whatever its precision, and this function
// is most of what the kernel executes, hence the short polynomial: the decisions need the weights
// to about 1e-13, not to the last bit.
__device__ __forceinline__ double exp_nonpos(double a) {
  a = fmax(a, -800.0);
  const double n = __builtin_rint(a * 1.4426950408889634074);
  double r = fma(n, -6.93147180369123816490e-01, a);      // ln2, high part
  r = fma(n, -1.90821492927058770002e-10, r);             // ln2, low part
  double p = 1.0 / 39916800.0;
  p = fma(p, r, 1.0 / 3628800.0);
  p = fma(p, r, 1.0 / 362880.0);
  p = fma(p, r, 1.0 / 40320.0);
  p = fma(p, r, 1.0 / 5040.0);
  p = fma(p, r, 1.0 / 720.0);
  p = fma(p, r, 1.0 / 120.0);
  p = fma(p, r, 1.0 / 24.0);
  p = fma(p, r, 1.0 / 6.0);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  return ldexp(p, (int)n);
}

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

// Four consecutive logits starting at token j (a multiple of 4 past the row start); tokens at or
// beyond lim read as -inf, i.e. weight 0.  vec: the row is 16-byte aligned and V a multiple of 4.
__device__ __forceinline__ float4 load_logits4(const float* x, int j, int lim, bool vec) {
  const float ninf = -__builtin_inff();
  if (vec) return j < lim ? *reinterpret_cast<const float4*>(x + j) : make_float4(ninf, ninf, ninf, ninf);
  float4 v;
  v.x = j < lim ? x[j] : ninf;
  v.y = j + 1 < lim ? x[j + 1] : ninf;
  v.z = j + 2 < lim ? x[j + 2] : ninf;
  v.w = j + 3 < lim ? x[j + 3] : ninf;
  return v;
}

constexpr int kVsChunk = 4 * kWave;     // tokens one wave loads per instruction

__global__ __launch_bounds__(kVsThreads) void verify_sample_kernel(VerifySampleArgs a) {
  __shared__ float s_max[kVsWaves];
  __shared__ double s_sub[kVsSub];
  __shared__ int s_rm_tok[kVsMaxRemoved];
  __shared__ double s_rm_w[kVsMaxRemoved];
  __shared__ int s_next, s_nrm, s_bonus, s_last[kVsWaves];
  __shared__ uint64_t s_key[kVsWaves];
  __shared__ int s_par[DDD_MMAX + 1], s_tok[DDD_MMAX + 1];     // the sequence's tree, read once
  __shared__ double s_ua[DDD_MMAX + 1], s_ub[DDD_MMAX + 1];

  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int T = a.m + 1, V = a.V;
  if (tid < T) {
    s_par[tid] = a.tree.parent_idx[(size_t)b * T + tid];
    s_tok[tid] = min(max(a.tree.tree_token[(size_t)b * T + tid], 0), V - 1);
    s_ua[tid] = a.u_accept[(size_t)b * T + tid];
    s_ub[tid] = a.u_bonus[(size_t)b * T + tid];
  }
  const int n = min(a.tree.n_sel[b], a.m) + 1;
  StatsPre sp{0, 0u};
  if (tid == 0) sp = stats_begin(a.stats, b, a.B);
  __syncthreads();
  int32_t* path = a.accept_path + (size_t)b * (a.D + 1);
  const int cpb = (V + kVsSub * kVsChunk - 1) / (kVsSub * kVsChunk);      // chunks per block
  const int sb = cpb * kVsChunk;                                          // tokens per block
  const int j0 = wv * kVsSubPerWave * sb;                                 // may lie beyond V
  const bool vec = (V & 3) == 0 && (reinterpret_cast<uintptr_t>(a.logits) & 15) == 0;
  const double beta = 1.0 / (double)a.temperature;

  int cur = 0, len = 0, nrm = 0;
  double Md = 0.0, rem = 0.0;          // nrm, rem: meaningful in wave 0
  const float* x = a.logits;
  if (tid == 0) path[0] = 0;

  for (int it = 0; it <= a.D; ++it) {
    x = a.logits + ((size_t)b * T + cur) * V;
    // wave 0: what the children tests will need (tree indices 1..64; larger trees fetch the rest
    // when they get there), requested now so that it arrives behind the two passes
    bool kid = false;
    int ktok = 0;
    float kx = 0.0f;
    double ku = 0.0;
    if (wv == 0 && 1 + lane < n) {
      kid = s_par[1 + lane] == cur;
      ktok = s_tok[1 + lane];
      kx = x[ktok];
      ku = s_ua[1 + lane];
    }
    // row maximum
    float mx = -__builtin_inff();
#pragma unroll 8
    for (int c = 0; c < kVsSubPerWave * cpb; ++c) {
      const float4 v = load_logits4(x, j0 + c * kVsChunk + 4 * lane, V, vec);
      mx = fmaxf(fmaxf(mx, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
    }
    mx = wave_max_f32(mx);
    if (lane == 0) s_max[wv] = mx;
    __syncthreads();
    mx = s_max[0];
#pragma unroll
    for (int i = 1; i < kVsWaves; ++i) mx = fmaxf(mx, s_max[i]);
    Md = (double)mx;
    const double mb = -Md * beta;
    // weights: one sum per block of sb consecutive tokens, in a fixed order
#pragma unroll 2
    for (int i = 0; i < kVsSubPerWave; ++i) {
      double acc = 0.0;
      for (int c = 0; c < cpb; ++c) {
        const int j = j0 + (i * cpb + c) * kVsChunk + 4 * lane;
        const float4 v = load_logits4(x, j, V, vec);
        const double e0 = exp_nonpos(fma((double)v.x, beta, mb)), e1 = exp_nonpos(fma((double)v.y, beta, mb));
        const double e2 = exp_nonpos(fma((double)v.z, beta, mb)), e3 = exp_nonpos(fma((double)v.w, beta, mb));
        acc += (e0 + e1) + (e2 + e3);
      }
      acc = wave_sum_f64(acc);
      if (lane == 0) s_sub[wv * kVsSubPerWave + i] = acc;
    }
    __syncthreads();
    if (wv == 0) {
      rem = 0.0;
      for (int i = 0; i < kVsSub; ++i) rem += s_sub[i];
      int nxt = -1;
      nrm = 0;
      if (len < a.D) {
        for (int base = 1; base < n && nxt < 0; base += kWave) {
          if (base > 1) {
            const int c = base + lane;
            kid = c < n && s_par[c] == cur;
            ktok = c < n ? s_tok[c] : 0;
            kx = x[ktok];
            ku = c < n ? s_ua[c] : 0.0;
          }
          const double kw = exp_nonpos(fma((double)kx, beta, mb));       // this lane's tree index: base + lane
          uint64_t kids = __ballot(kid);
          while (kids) {
            const int l = __ffsll((unsigned long long)kids) - 1;
            kids &= kids - 1;
            const double w = __shfl(kw, l, 64);
            const int tk = __shfl(ktok, l, 64);
            if (__shfl(ku, l, 64) * rem < w) { nxt = base + l; break; }
            rem -= w;
            if (lane == 0 && nrm < kVsMaxRemoved) { s_rm_tok[nrm] = tk; s_rm_w[nrm] = w; }
            ++nrm;
          }
        }
      }
      nrm = min(nrm, kVsMaxRemoved);
      if (lane == 0) s_next = nxt;
    }
    __syncthreads();
    const int nxt = s_next;
    if (nxt < 0) break;
    cur = nxt;
    ++len;
    if (tid == 0) path[len] = cur;
  }

  // Bonus token at `cur` (x, Md, s_sub, s_rm_* describe that node): wave 0 finds the block in
  // which the prefix sum of the remaining weights passes the threshold, then the token inside it.
  if (wv == 0) {
    const double thr = s_ub[cur] * rem;
    double v0 = s_sub[2 * lane], v1 = s_sub[2 * lane + 1];
    for (int r = 0; r < nrm; ++r) {
      const int blk = s_rm_tok[r] / sb;
      if (blk == 2 * lane) v0 -= s_rm_w[r];
      if (blk == 2 * lane + 1) v1 -= s_rm_w[r];
    }
    const double inc = wave_scan_f64(v0 + v1, lane);        // prefix up to and including block 2*lane+1
    const double before = inc - (v0 + v1);
    const uint64_t hit = __ballot(inc > thr);
    int bonus = -1;
    if (hit != 0) {
      const int hl = __ffsll((unsigned long long)hit) - 1;
      const double bef = __shfl(before, hl, 64), first = __shfl(v0, hl, 64);
      const bool in_first = bef + first > thr;
      double run = in_first ? bef : bef + first;
      for (int jb = (2 * hl + (in_first ? 0 : 1)) * sb; jb < V; jb += kVsChunk) {   // ends inside the block but for rounding
        const int j = jb + 4 * lane;
        const float4 v = load_logits4(x, j, V, vec);
        const double mb = -Md * beta;
        double w[4] = {exp_nonpos(fma((double)v.x, beta, mb)), exp_nonpos(fma((double)v.y, beta, mb)),
                       exp_nonpos(fma((double)v.z, beta, mb)), exp_nonpos(fma((double)v.w, beta, mb))};
        for (int r = 0; r < nrm; ++r) {
          const int d = s_rm_tok[r] - j;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (d == e) w[e] = 0.0;
        }
        const double c0 = w[0], c1 = c0 + w[1], c2 = c1 + w[2], c3 = c2 + w[3];
        const double pre = run + (wave_scan_f64(c3, lane) - c3);     // remaining weight before this lane's tokens
        const int e = pre + c0 > thr ? 0 : pre + c1 > thr ? 1 : pre + c2 > thr ? 2 : pre + c3 > thr ? 3 : 4;
        const uint64_t over = __ballot(e < 4 && j + e < V);
        if (over != 0) {
          const int ol = __ffsll((unsigned long long)over) - 1;
          bonus = jb + 4 * ol + __shfl(e, ol, 64);
          break;
        }
        run = __shfl(pre + c3, 63, 64);
      }
    }
    if (lane == 0) { s_bonus = bonus; s_nrm = nrm; }
  }
  __syncthreads();
  int bonus = s_bonus;
  if (bonus < 0) {
    // rounding left no prefix above the threshold: the last token that still has weight, and if
    // the children covered everything the target's most likely token  (block-uniform branch)
    const int n_removed = s_nrm;
    int last = -1;
    uint64_t key = 0;
    for (int j = tid; j < V; j += kVsThreads) {
      key = umax64(key, row_key(x[j], j));
      bool live = exp(((double)x[j] - Md) * beta) > 0.0;
      for (int r = 0; r < n_removed; ++r)
        if (s_rm_tok[r] == j) live = false;
      if (live) last = max(last, j);
    }
    key = wave_max_u64(key);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) last = max(last, __shfl_xor(last, off, 64));
    if (lane == 0) { s_last[wv] = last; s_key[wv] = key; }
    __syncthreads();
    last = -1;
    key = 0;
#pragma unroll
    for (int i = 0; i < kVsWaves; ++i) { last = max(last, s_last[i]); key = umax64(key, s_key[i]); }
    bonus = last >= 0 ? last : key_token(key);
  }
  if (tid == 0) {
    for (int i = len + 1; i <= a.D; ++i) path[i] = -1;
    a.accept_len[b] = len;
    a.bonus_token[b] = bonus;
    stats_end(a.stats, sp, a.B, len);
  }
}

hipError_t launch_verify_sample(const VerifySampleArgs& a, hipStream_t stream) {
  if (a.m > DDD_MMAX) return hipErrorInvalidValue;      // the kernel keeps the tree in LDS
  hipLaunchKernelGGL(verify_sample_kernel, dim3(a.B), dim3(kVsThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
