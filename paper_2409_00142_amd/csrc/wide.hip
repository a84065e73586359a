// Wide beams (DDD_KMAX < k <= DDD_KWIDE_MAX): beam update, stop test and final tree of one
// sequence by one workgroup (Appendix, Table 2: draft speed against beam width).
//
// With up to 128 x 128 candidates per draft call and tens of thousands of pool nodes nothing fits
// in registers any more: the k*k candidate keys (score desc, token asc, flat index asc) are built
// in LDS and the k-th largest is found by a radix select (8-bit digits from the top: histogram in
// LDS, the digit holding the wanted rank narrows the prefix); the keys at or above it are the new
// beam, sorted by a small bitonic network.  The final rerank selects the m best pool nodes the
// same way with keys computed on the fly from the pool scores in global memory (L2-resident).
// Everything else (Eq. 1 in fp64 in index order, parents, ancestor rows, mask) is as for narrow
// beams.
#include "bookkeep_device.hpp"
#include "tree_device.hpp"

namespace ddd {

constexpr int kKW = DDD_KWIDE_MAX;
constexpr int kWideThreads = 1024;
constexpr int kGlobalChunk = 8;                    // loads in flight per thread when the keys come from global memory
constexpr int kFlatBits = 14;                      // k*k <= 16384 flat indices
constexpr uint32_t kFlatMask = (1u << kFlatBits) - 1u;
constexpr uint32_t kTokMaskW = (1u << (32 - kFlatBits)) - 1u;   // tokens below 2^18
// final tree of a large pool: sample, candidates and their ranks (tree_finalize_wide_block)
constexpr int kWSub = 512, kWCand = 1024;
constexpr int kWideWorkBytes = kWSub * 8 + kWCand * 8 + kWCand * 4;
static_assert(kWSub >= DDD_MMAX && kWSub <= kWCand, "the sample holds m keys and lies in the candidate list");
// LDS in front of WideSmem in the step kernel: the k*k candidate keys of a call, later the work area of the final tree
__host__ __device__ inline size_t wide_front_bytes(int k) {
  const size_t keys = ((size_t)k * k * 8 + 15) & ~(size_t)15;
  return keys > (size_t)kWideWorkBytes ? keys : (size_t)kWideWorkBytes;
}

__device__ __forceinline__ uint64_t wide_beam_key(float score, int token, int flat) {
  const uint32_t lo = ((kTokMaskW - (uint32_t)token) << kFlatBits) | (kFlatMask - (uint32_t)flat);
  return ((uint64_t)ord32(score) << 32) | lo;
}
__device__ __forceinline__ int wide_key_flat(uint64_t key) { return (int)(kFlatMask - ((uint32_t)key & kFlatMask)); }
__device__ __forceinline__ int wide_key_token(uint64_t key) {
  return (int)(kTokMaskW - (((uint32_t)key >> kFlatBits) & kTokMaskW));
}

struct WideSmem {
  unsigned hist[256];
  int digit, rem, alone, cnt, stopped;
  unsigned or_lo, or_hi, and_lo, and_hi, found_lo, found_hi;
  float lps_old[kKW];
  int node_old[kKW];
  uint64_t sel[kKW];
  double e[kKW];
  TreeEmitSmem te;
};

// One count for this lane's digit into the histogram.  Scores cluster (a handful of exponents), so
// most lanes of a wave often hit the same bin, which an LDS atomic serialises lane by lane: up to
// eight distinct digits per wave are therefore counted with a ballot and added once by a leader
// (`clustered`: the first digit examined, where the keys still share their leading bits); whatever
// is left, and every later digit, goes through plain atomics (spread digits rarely collide).
__device__ __forceinline__ void hist_add(unsigned* hist, unsigned digit, bool valid, int lane, bool clustered) {
  unsigned long long remaining = __ballot(valid);
  for (int it = 0; clustered && it < 8 && remaining != 0ull; ++it) {
    const int leader = __ffsll((long long)remaining) - 1;
    const unsigned d = (unsigned)__shfl((int)digit, leader, 64);
    const unsigned long long same = __ballot(valid && digit == d) & remaining;
    if (lane == leader) atomicAdd(&hist[d], (unsigned)__popcll(same));
    remaining &= ~same;
  }
  if ((remaining >> lane) & 1ull) atomicAdd(&hist[digit], 1u);
}

// The key of rank `want` (0-based, descending) among n distinct keys key_of(0..n-1), n > want.
// Every thread of the block calls it with the same arguments; the result is uniform.
// Radix select, 8-bit digits from the top; the bytes above the first one in which any two keys
// differ are skipped, and the search ends as soon as the wanted key is alone in its bin.
// One pass over keys 0..n-1 by the whole block (1024 threads): element i = tid + j * 1024.  CH
// keys are fetched before any is used, so a pass over keys that come from global memory pays one
// memory latency per CH elements.  fn(key, in) is called for every slot of a chunk that holds
// at least one element, by all threads (in == false past the end): it may use wave-wide operations.
template <int CH, class KeyFn, class Fn>
__device__ __forceinline__ void sweep_keys(int n, int tid, KeyFn key_of, Fn fn) {
  for (int j0 = 0; j0 * kWideThreads < n; j0 += CH) {
    uint64_t kk[CH];
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const int i = tid + (j0 + u) * kWideThreads;
      kk[u] = (i < n) ? key_of(i) : 0ull;
    }
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const int i0 = (j0 + u) * kWideThreads;
      if (i0 < n) fn(kk[u], tid + i0 < n);
    }
  }
}

// The key of rank `want` (0-based, descending) among the n distinct keys key_of(0..n-1), n > want.
// Every thread of the block calls it with the same arguments; the result is uniform.  Radix
// select, 8-bit digits from the top; the bytes above the first one in which any two keys differ
// are skipped, and the search ends as soon as the wanted key is alone in its bin.
template <int CH, class KeyFn>
__device__ __forceinline__ uint64_t block_select_kth(int n, int want, KeyFn key_of, WideSmem& sm, int tid) {
  const int lane = tid & 63;
  // bits in which the keys differ: OR of all keys against AND of all keys
  uint64_t vor = 0ull, vand = ~0ull;
  sweep_keys<CH>(n, tid, key_of, [&](uint64_t key, bool in) {
    if (in) {
      vor |= key;
      vand &= key;
    }
  });
  uint32_t olo = (uint32_t)vor, ohi = (uint32_t)(vor >> 32), alo = (uint32_t)vand, ahi = (uint32_t)(vand >> 32);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    olo |= (uint32_t)__shfl_xor((int)olo, off, 64);
    ohi |= (uint32_t)__shfl_xor((int)ohi, off, 64);
    alo &= (uint32_t)__shfl_xor((int)alo, off, 64);
    ahi &= (uint32_t)__shfl_xor((int)ahi, off, 64);
  }
  if (tid == 0) {
    sm.or_lo = 0u;
    sm.or_hi = 0u;
    sm.and_lo = ~0u;
    sm.and_hi = ~0u;
  }
  __syncthreads();
  if (lane == 0) {
    atomicOr(&sm.or_lo, olo);
    atomicOr(&sm.or_hi, ohi);
    atomicAnd(&sm.and_lo, alo);
    atomicAnd(&sm.and_hi, ahi);
  }
  __syncthreads();
  const uint64_t all_or = ((uint64_t)sm.or_hi << 32) | sm.or_lo, all_and = ((uint64_t)sm.and_hi << 32) | sm.and_lo;
  const uint64_t diff = all_or ^ all_and;
  if (diff == 0ull) return all_or;                    // a single key
  const int top_byte = (63 - __clzll((long long)diff)) >> 3;
  uint64_t prefix = (top_byte == 7) ? 0ull : (all_and & (~0ull << (8 * (top_byte + 1))));
  int rem = want;
  for (int shift = 8 * top_byte; shift >= 0; shift -= 8) {
    for (int i = tid; i < 256; i += kWideThreads) sm.hist[i] = 0u;
    __syncthreads();
    const uint64_t hi_mask = (shift == 56) ? 0ull : (~0ull << (shift + 8));
    sweep_keys<CH>(n, tid, key_of, [&](uint64_t key, bool in) {
      hist_add(sm.hist, (unsigned)(key >> shift) & 255u, in && (key & hi_mask) == prefix, lane, shift == 8 * top_byte);
    });
    __syncthreads();
    if (tid < 64) {   // wave 0: lane l owns digits 255-4l .. 252-4l; running count from the top digit down
      unsigned h[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) h[q] = sm.hist[255 - 4 * lane - q];
      const unsigned s = h[0] + h[1] + h[2] + h[3];
      unsigned incl = s;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
      }
      const unsigned excl = incl - s;
      if ((unsigned)rem >= excl && (unsigned)rem < incl) {   // exactly one lane
        unsigned c = excl;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if ((unsigned)rem >= c && (unsigned)rem < c + h[q]) {
            sm.digit = 255 - 4 * lane - q;
            sm.rem = (int)((unsigned)rem - c);
            sm.alone = (h[q] == 1u) ? 1 : 0;
          }
          c += h[q];
        }
      }
    }
    __syncthreads();
    prefix |= (uint64_t)(unsigned)sm.digit << shift;
    rem = sm.rem;
    if (sm.alone && shift > 0) {                      // uniform: the wanted key is the only one with this prefix
      const uint64_t pm = ~0ull << shift;
      sweep_keys<CH>(n, tid, key_of, [&](uint64_t key, bool in) {
        if (in && (key & pm) == prefix) {
          sm.found_lo = (uint32_t)key;
          sm.found_hi = (uint32_t)(key >> 32);
        }
      });
      __syncthreads();
      return ((uint64_t)sm.found_hi << 32) | sm.found_lo;
    }
  }
  return prefix;
}

// Descending bitonic sort of sm.sel[0..127] (unused slots hold 0) by one wave (all 64 lanes): each
// stage is one compare-exchange per lane, ordered by wave barriers instead of block barriers.
__device__ __forceinline__ void sort_sel_desc_wave(WideSmem& sm, int lane) {
  for (int size = 2; size <= kKW; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      const int pos = 2 * stride * (lane / stride) + (lane % stride);
      const int partner = pos + stride;
      const bool desc = ((pos & size) == 0);
      const uint64_t x = sm.sel[pos], y = sm.sel[partner];
      if ((x < y) == desc) {
        sm.sel[pos] = y;
        sm.sel[partner] = x;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// Final tree for a pool of any size.  The m best rerank keys are found as for narrow beams (tree_device.hpp): the
// m-th best key of the first kWSub nodes is a lower bound of the tree's keys (summed logprobs fall with depth), one
// sweep over the pool collects the keys at or above it, and the candidates are ranked by counting; a sweep over
// 50 000 scores takes about 20 us on the one CU that runs it, and the radix select needs five or six of them.  While
// more than kWCand keys pass the bound, the m-th best of kWSub of them tightens it (twice at most); after that the
// radix select takes over.  work: kWideWorkBytes of LDS.
__device__ __forceinline__ void tree_finalize_wide_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int nmax,
                                                         int tid, int nthr, WideSmem& sm, unsigned char* work) {
  const int N = st.n_nodes[b] - 1;
  const int m_eff = min(m, N);
  const float* psc = st.pool_score + (size_t)b * nmax;
  auto key_of = [&](int i) { return rerank_key(psc[i + 1], i + 1); };
  uint64_t* sample = reinterpret_cast<uint64_t*>(work);            // [kWSub]
  uint64_t* cand = sample + kWSub;                                   // [kWCand]
  int* rank = reinterpret_cast<int*>(cand + kWCand);                // [kWCand]
  bool ranked = false;
  if (m_eff < N && nthr == kWideThreads) {                           // uniform
    int n_sample = min(N, kWSub);
    for (int i = tid; i < n_sample; i += nthr) sample[i] = key_of(i);
    for (int attempt = 0; attempt < 3; ++attempt) {
      for (int i = tid; i < kWCand; i += nthr) rank[i] = 0;
      if (tid == 0) sm.cnt = 0;
      __syncthreads();
      count_larger_keys(sample, n_sample, rank, tid, nthr);
      __syncthreads();
      for (int i = tid; i < n_sample; i += nthr)
        if (rank[i] == min(m_eff, n_sample) - 1) {                   // exactly one key has this rank
          sm.found_lo = (uint32_t)sample[i];
          sm.found_hi = (uint32_t)(sample[i] >> 32);
        }
      __syncthreads();
      const uint64_t bound = ((uint64_t)sm.found_hi << 32) | sm.found_lo;
      sweep_keys<kGlobalChunk>(N, tid, key_of, [&](uint64_t key, bool in) {
        if (in && key >= bound) {
          const int p = atomicAdd(&sm.cnt, 1);
          if (p < kWCand) cand[p] = key;
        }
      });
      __syncthreads();
      const int C = sm.cnt;
      if (C <= kWCand) {                                             // uniform
        for (int i = tid; i < kWCand; i += nthr) rank[i] = 0;
        __syncthreads();
        count_larger_keys(cand, C, rank, tid, nthr);
        __syncthreads();
        for (int c = tid; c < C; c += nthr)
          if (rank[c] < m_eff) sm.te.pick[rank[c]] = (int)(0xFFFFFFFFu - (uint32_t)cand[c]);
        ranked = true;
        break;
      }
      for (int i = tid; i < kWSub; i += nthr) sample[i] = cand[i];  // the first kWSub candidates: all above the old bound
      n_sample = kWSub;
      __syncthreads();
    }
  }
  if (!ranked) {
    uint64_t kth = 0ull;                       // every key is at least 1
    if (m_eff < N) kth = block_select_kth<kGlobalChunk>(N, m_eff - 1, key_of, sm, tid);
    if (tid == 0) sm.cnt = 0;
    __syncthreads();
    sweep_keys<kGlobalChunk>(N, tid, key_of, [&](uint64_t key, bool in) {
      if (in && key >= kth) {
        const int p = atomicAdd(&sm.cnt, 1);
        if (p < kTreeMax) sm.te.pick[p] = (int)(0xFFFFFFFFu - (uint32_t)key);   // exactly m_eff: keys are distinct
      }
    });
  }
  __syncthreads();
  tree_emit_block(st, tree, b, m, m_eff, nmax, tid, nthr, sm.te);
}

// One draft call of one sequence by one workgroup; returns whether the sequence is still active after it
// (the same value in every thread; true when no stop test is asked for).
__device__ __forceinline__ bool step_wide_block(const WideStepArgs& a, unsigned char* wsm_raw) {
  const BeamArgs& g = a.beam;
  const int b = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  const int k = g.k, step = g.step;
  uint64_t* keys = reinterpret_cast<uint64_t*>(wsm_raw);                       // [k*k]
  WideSmem& sm = *reinterpret_cast<WideSmem*>(wsm_raw + wide_front_bytes(k));
  if (!g.st.active[b]) return false;         // uniform over the workgroup

  float* lps = g.st.logprobsum + (size_t)b * k;
  int32_t* bnode = g.st.beam_node + (size_t)b * k;
  int32_t* btok = g.st.beam_token + (size_t)b * k;
  int32_t* bslot = g.st.beam_parent_slot + (size_t)b * k;
  int32_t* ptok = g.st.pool_token + (size_t)b * g.nmax;
  int32_t* ppar = g.st.pool_parent + (size_t)b * g.nmax;
  int32_t* pdep = g.st.pool_depth + (size_t)b * g.nmax;
  float* psc = g.st.pool_score + (size_t)b * g.nmax;
  const bool from_keys = (a.part_key != nullptr);
  const size_t row0 = (step == 0) ? (size_t)b : (size_t)b * k;
  int steps_done = a.steps_done;

  if (a.do_select) {
    steps_done = step + 1;
    if (step == 0) {
      // the prompt call: nodes 1..k in rank order are the first beam
      for (int j = tid; j < k; j += nthr) {
        int t;
        float s;
        if (from_keys) {
          const uint64_t key = a.part_key[row0 * k + j];
          t = key_token(key);
          s = key_value(key) - a.part_lse[row0];
        } else {
          t = g.topk_token[row0 * k + j];
          s = g.topk_logprob[row0 * k + j];
        }
        const int nid = 1 + j;
        ptok[nid] = t;
        ppar[nid] = 0;
        pdep[nid] = 1;
        psc[nid] = s;
        bnode[j] = nid;
        btok[j] = t;
        bslot[j] = 0;
        lps[j] = s;
      }
      if (tid == 0) {
        g.st.n_nodes[b] = 1 + k;
        g.st.steps[b] = 1;
        if (a.lse_dbg != nullptr && from_keys) a.lse_dbg[row0] = a.part_lse[row0];
      }
    } else {
      const int base = 1 + k + (step - 1) * k * k;
      for (int i = tid; i < k; i += nthr) {
        sm.lps_old[i] = lps[i];
        sm.node_old[i] = bnode[i];
        if (a.lse_dbg != nullptr && from_keys) a.lse_dbg[row0 + i] = a.part_lse[row0 + i];
      }
      __syncthreads();
      for (int f0 = 0; f0 < k * k; f0 += 4 * nthr) {      // four candidates per thread in flight
        int t[4];
        float lp[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int f = f0 + u * nthr + tid;
          t[u] = 0;
          lp[u] = 0.f;
          if (f < k * k) {
            const int i = f / k, j = f - i * k;
            if (from_keys) {
              const uint64_t key = a.part_key[(row0 + i) * k + j];
              t[u] = key_token(key);
              lp[u] = key_value(key) - a.part_lse[row0 + i];
            } else {
              t[u] = g.topk_token[(row0 + i) * k + j];
              lp[u] = g.topk_logprob[(row0 + i) * k + j];
            }
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int f = f0 + u * nthr + tid;
          if (f < k * k) {
            const int i = f / k;
            const float sc = __fadd_rn(sm.lps_old[i], lp[u]);
            ptok[base + f] = t[u];
            ppar[base + f] = sm.node_old[i];
            pdep[base + f] = step + 1;
            psc[base + f] = sc;
            keys[f] = wide_beam_key(sc, t[u], f);
          }
        }
      }
      __syncthreads();
      const uint64_t kth = block_select_kth<8>(k * k, k - 1, [&](int i) { return keys[i]; }, sm, tid);
      for (int i = tid; i < kKW; i += nthr) sm.sel[i] = 0ull;
      if (tid == 0) sm.cnt = 0;
      __syncthreads();
      for (int f = tid; f < k * k; f += nthr)
        if (keys[f] >= kth) {
          const int p = atomicAdd(&sm.cnt, 1);
          if (p < kKW) sm.sel[p] = keys[f];     // exactly k of them: keys are distinct
        }
      __syncthreads();
      if (tid < 64) sort_sel_desc_wave(sm, tid);
      __syncthreads();
      for (int r = tid; r < k; r += nthr) {
        const uint64_t key = sm.sel[r];
        const int f = wide_key_flat(key);
        bnode[r] = base + f;
        btok[r] = wide_key_token(key);
        bslot[r] = f / k;
        lps[r] = key_value(key);
      }
      if (tid == 0) {
        g.st.n_nodes[b] = base + k * k;
        g.st.steps[b] = step + 1;
      }
    }
    __syncthreads();   // the new beam is visible to the block
  }

  if (tid == 0) sm.stopped = 0;
  if (a.do_stop) {
    for (int i = tid; i < k; i += nthr) sm.e[i] = exp((double)lps[i]);
    __syncthreads();
    if (tid == 0) {
      double P = 0.0;
      for (int i = 0; i < k; ++i) P += sm.e[i];   // index order
      bool cont = steps_done < g.D;
      if (cont && ((g.check_mask >> steps_done) & 1u) && P < (double)g.threshold) cont = false;
      g.st.conf[b] = P;
      g.st.active[b] = cont ? 1 : 0;
      sm.stopped = cont ? 0 : 1;
    }
    __syncthreads();
    const uint8_t on = sm.stopped ? 0 : 1;
    for (int i = tid; i < k; i += nthr) g.st.row_active[(size_t)b * k + i] = on;
  }
  __syncthreads();   // also orders the pool writes before the reads below
  const bool stopped = sm.stopped != 0;
  if (a.tree.mask != nullptr && stopped)   // the candidate keys of the beam update are no longer needed: their LDS is the work area
    tree_finalize_wide_block(g.st, a.tree, b, a.m, g.nmax, tid, nthr, sm, wsm_raw);
  return !stopped;
}

__global__ __launch_bounds__(kWideThreads) void step_wide_kernel(WideStepArgs a) {
  extern __shared__ __align__(16) unsigned char wsm_raw[];
  const bool active = step_wide_block(a, wsm_raw);
  if (a.call_count != nullptr && threadIdx.x == 0) {
    // report to the host that paces the round (see step_bookkeep_kernel): one atomic per sequence, arrivals in
    // the low half, active sequences in the high half; the last arrival clears the word and writes the host word
    const uint32_t mine = 1u | (active ? 0x10000u : 0u);
    const uint32_t seen = __hip_atomic_fetch_add(a.call_count, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((seen & 0xFFFFu) + 1u == gridDim.x) {
      __hip_atomic_store(a.call_count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t any = ((seen + mine) >> 16) != 0u ? 1u : 0u;
      __hip_atomic_store(a.progress, (a.round_tag << 2) | 2u | any, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
  }
}

__global__ __launch_bounds__(kWideThreads) void tree_finalize_wide_kernel(FinalizeArgs a) {
  __shared__ WideSmem sm;
  __shared__ __align__(16) unsigned char work[kWideWorkBytes];
  tree_finalize_wide_block(a.st, a.tree, blockIdx.x, a.m, a.nmax, threadIdx.x, blockDim.x, sm, work);
}

static size_t wide_lds_bytes(int k) { return wide_front_bytes(k) + sizeof(WideSmem); }

hipError_t prepare_wide() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&step_wide_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)wide_lds_bytes(kKW));
}

hipError_t launch_step_wide(const WideStepArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(step_wide_kernel, dim3(a.beam.B), dim3(kWideThreads), wide_lds_bytes(a.beam.k), stream, a);
  return hipGetLastError();
}

hipError_t launch_tree_finalize_wide(const FinalizeArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(tree_finalize_wide_kernel, dim3(a.B), dim3(kWideThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
