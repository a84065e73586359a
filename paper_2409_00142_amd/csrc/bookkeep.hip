// Stand-alone kernels of the per-call bookkeeping (device code in bookkeep_device.hpp) and the
// row reduction of materialised logits.
#include "bookkeep_device.hpp"

namespace ddd {

// ---- standalone merge: one wave per row ------------------------------------------------------
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs a) {
  __shared__ uint64_t s_mrg[4][kMergeWords];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= a.n_rows) return;                                 // wave-uniform
  if (a.row_active != nullptr && !a.row_active[row]) return;   // wave-uniform
  if (a.nslice == 0) {   // dense format: the keys are final (any k up to DDD_KWIDE_MAX)
    const float lse = a.part_sum[row];
    for (int j = lane; j < a.k; j += 64) {
      const uint64_t key = a.part_key[(size_t)row * a.k + j];
      a.topk_token[(size_t)row * a.k + j] = key_token(key);
      a.topk_logprob[(size_t)row * a.k + j] = key_value(key) - lse;
    }
    if (lane == 0) a.lse[row] = lse;
    return;
  }
  uint64_t key;
  float lse;
  {
    RowHeads heads;
    const uint64_t* pk = a.part_key + (size_t)row * a.nslice * a.k;
    merge_load_heads(pk, a.part_sum + (size_t)row * a.nslice, a.nslice, a.k, lane, heads);
    merge_row_dispatch(pk, heads, a.nslice, a.k, lane, key, lse, s_mrg[wave]);
  }
  if (lane < a.k) {
    a.topk_token[(size_t)row * a.k + lane] = key_token(key);
    a.topk_logprob[(size_t)row * a.k + lane] = key_value(key) - lse;
  }
  if (lane == 0) a.lse[row] = lse;
}

hipError_t launch_merge(const MergeArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(merge_kernel, dim3((a.n_rows + 3) / 4), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- row reduction of materialised logits (GEMM path) ------------------------------------------
// One workgroup per row.  The GEMM left, for every group of 64 consecutive vocabulary rows, the
// group's max and sum of exponentials.  lse follows from those alone.  The k-th largest group max
// T is a lower bound of the row's k-th largest logit (k distinct elements are >= T), and only the
// groups whose max reaches T - k of them, or a few more - can hold an element >= T: those groups'
// logits are read (64 values each), the candidates >= T collected, and the exact top-k by (logit
// desc, token asc) taken among them (a candidate's rank is the number of larger keys).  Massive ties (e.g. constant logits) overflow the lists: with
// too many candidate groups the whole row is scanned instead, and with too many candidates an
// exact but slow path takes over: k passes over the row, each finding the largest key below the
// previous winner.
constexpr int kCandMax = 2048;
constexpr int kGrpListMax = 256;   // groups that may hold a candidate; more than that: the row is scanned

// k-th largest of the group maxima as an ordered key (0 if there are fewer than k groups), by one
// wave: lane holds groups lane, lane + 64, ... (S slots).
template <int S>
__device__ __forceinline__ uint32_t kth_largest_group_max(const float* gmax, int ngrp_valid, int k, int lane) {
  uint32_t loc[S];
#pragma unroll
  for (int i = 0; i < S; ++i) {
    const int g = lane + 64 * i;
    loc[i] = (g < ngrp_valid) ? ord32(gmax[g]) : 0u;
  }
  uint32_t T = 0u;
  for (int round = 0; round < k; ++round) {
    uint32_t lm = 0u;
#pragma unroll
    for (int i = 0; i < S; ++i) lm = umax32(lm, loc[i]);
    T = wave_max_u32(lm);
    if (T == 0u) break;                                    // uniform: fewer than k groups
    // remove one holder of the maximum (the lowest lane, its lowest slot)
    const unsigned long long holders = __ballot(lm == T);
    if (lane == __ffsll((long long)holders) - 1) {
      bool done = false;
#pragma unroll
      for (int i = 0; i < S; ++i)
        if (!done && loc[i] == T) {
          loc[i] = 0u;
          done = true;
        }
    }
  }
  return T;
}

// Descending bitonic sort of n2 (a power of two) 64-bit keys in LDS by the whole block.
__device__ __forceinline__ void block_sort_desc(uint64_t* keys, int n2, int tid, int nthr) {
  for (int size = 2; size <= n2; size <<= 1)
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int p = tid; p < (n2 >> 1); p += nthr) {
        const int pos = 2 * stride * (p / stride) + (p % stride);
        const int partner = pos + stride;
        const bool desc = ((pos & size) == 0);
        const uint64_t x = keys[pos], y = keys[partner];
        if ((x < y) == desc) {
          keys[pos] = y;
          keys[partner] = x;
        }
      }
      __syncthreads();
    }
}

constexpr int kSortFromK = 17;   // beams wider than DDD_KMAX: sorts replace the k rounds of wave maxima

__global__ __launch_bounds__(256) void row_topk_kernel(RowTopkArgs a) {
  __shared__ uint64_t s_cand[kCandMax];
  __shared__ float s_red[8];
  __shared__ float s_T;
  __shared__ int s_cnt, s_ng;
  __shared__ int s_glist[kGrpListMax];
  __shared__ uint32_t s_bound[4];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (a.row_active != nullptr && !a.row_active[row]) return;   // uniform
  const int ngrp_valid = (a.V + 63) >> 6;
  const float* gmax = a.grp_max + (size_t)row * a.ngrp;
  const float* gsum = a.grp_sum + (size_t)row * a.ngrp;

  // ---- row max, lse ---------------------------------------------------------------------------
  float m = -INFINITY;
  for (int g = tid; g < ngrp_valid; g += 256) m = fmaxf(m, gmax[g]);
  m = wave_max_f32(m);
  if (lane == 0) s_red[wave] = m;
  __syncthreads();
  const float M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  float acc = 0.f;
  for (int g = tid; g < ngrp_valid; g += 256) acc += gsum[g] * __expf(gmax[g] - M);
  acc = wave_sum_f32(acc);
  if (lane == 0) s_red[4 + wave] = acc;
  // ---- T = k-th largest group max (or -inf if there are fewer than k groups): wave 0 -------------
  if (tid == 0) {
    s_cnt = 0;
    s_ng = 0;
  }
  if (a.k >= kSortFromK) {
    // wide beams: sort the group maxima (at most 2048) and read off the k-th
    int n2 = 64;
    while (n2 < ngrp_valid) n2 <<= 1;
    for (int g = tid; g < n2; g += 256) s_cand[g] = (g < ngrp_valid) ? (uint64_t)ord32(gmax[g]) : 0ull;
    __syncthreads();
    block_sort_desc(s_cand, n2, tid, 256);
    if (tid == 0) s_T = (a.k <= ngrp_valid) ? unord32((uint32_t)s_cand[a.k - 1]) : -INFINITY;
  } else {
    // Up to 2048 groups (V <= 131072), up to 8 per thread, as ordered keys.  A lower bound first: a quad of lanes
    // holds 4 to 32 groups, and the k-th largest of a wave's 16 quad maxima is reached by k distinct groups (k <= 16);
    // the best of the four waves' bounds is taken.  The group maxima at or above it - a few dozen - are ranked by
    // counting, and the one of rank k - 1 is T.  (k rounds of a wave maximum on one wave took three times as long.)
    uint32_t tm = 0u;
    for (int g = tid; g < ngrp_valid; g += 256) tm = umax32(tm, ord32(gmax[g]));
    uint32_t qm = umax32(tm, dpp_move_u32<0xB1>(tm));
    qm = umax32(qm, dpp_move_u32<0x4E>(qm));
    int larger = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) larger += ((uint32_t)__builtin_amdgcn_readlane((int)qm, 4 * q) > qm) ? 1 : 0;
    const uint32_t bound_w = ~wave_max_u32(~(larger < a.k ? qm : 0xFFFFFFFFu));
    if (lane == 0) s_bound[wave] = bound_w;
    __syncthreads();
    const uint32_t bound = umax32(umax32(s_bound[0], s_bound[1]), umax32(s_bound[2], s_bound[3]));
    for (int g = tid; g < ngrp_valid; g += 256) {
      const uint32_t v = ord32(gmax[g]);
      if (v >= bound) {
        const int p = atomicAdd(&s_ng, 1);
        if (p < kCandMax) s_cand[p] = ((uint64_t)v << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)g);   // distinct
      }
    }
    __syncthreads();
    const int ncg = s_ng;
    __syncthreads();                                             // everybody has the count: the counter is used again below
    if (ncg <= 256) {                                            // uniform
      if (tid < ncg) {
        const uint64_t mine = s_cand[tid];
        int rank = 0;
        for (int j = 0; j < ncg; ++j) rank += (s_cand[j] > mine) ? 1 : 0;
        if (rank == a.k - 1) s_T = unord32((uint32_t)(mine >> 32));
      }
      if (tid == 0) {
        if (ncg < a.k) s_T = -INFINITY;                          // fewer than k groups
        s_ng = 0;
      }
    } else if (wave == 0) {                                      // many equal maxima: the rounds
      const uint32_t T = (ngrp_valid <= 512)    ? kth_largest_group_max<8>(gmax, ngrp_valid, a.k, lane)
                         : (ngrp_valid <= 1024) ? kth_largest_group_max<16>(gmax, ngrp_valid, a.k, lane)
                                                : kth_largest_group_max<32>(gmax, ngrp_valid, a.k, lane);
      if (lane == 0) {
        s_T = (T == 0u) ? -INFINITY : unord32(T);
        s_ng = 0;
      }
    }
  }
  __syncthreads();
  const float lse = M + __logf(s_red[4] + s_red[5] + s_red[6] + s_red[7]);

  // ---- collect candidates >= T ------------------------------------------------------------------
  // Only groups whose max reaches T can hold one: usually k or a few more of them, so the row's
  // logits are read group by group (64 consecutive values, one per lane) rather than scanned.
  const float* x = a.logits + (size_t)row * a.V;
  const float T = s_T;
  for (int g = tid; g < ngrp_valid; g += 256)
    if (gmax[g] >= T) {
      const int p = atomicAdd(&s_ng, 1);
      if (p < kGrpListMax) s_glist[p] = g;
    }
  __syncthreads();
  const int ng = s_ng;
  if (ng <= kGrpListMax) {                                     // uniform
    for (int i0 = wave; i0 < ng; i0 += 16) {
      float xv[4];
      int vv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {                            // four independent loads in flight
        const int i = i0 + 4 * u;
        vv[u] = (i < ng) ? s_glist[i] * 64 + lane : a.V;
        xv[u] = (vv[u] < a.V) ? x[vv[u]] : -INFINITY;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (vv[u] < a.V && xv[u] >= T) {
          const int p = atomicAdd(&s_cnt, 1);
          if (p < kCandMax) s_cand[p] = row_key(xv[u], vv[u]);
        }
    }
  } else if ((a.V & 3) == 0) {                                 // too many groups tie at T: scan the row
    const int nchunk = a.V >> 2;
    for (int c0 = tid; c0 < nchunk; c0 += 8 * 256) {
      float4 q[8];   // eight independent 16-byte loads in flight before any is consumed
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = c0 + u * 256;
        q[u] = (c < nchunk) ? *reinterpret_cast<const float4*>(x + 4 * c)
                            : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int c = c0 + u * 256;
        const float xq[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
        if (c < nchunk && fmaxf(fmaxf(xq[0], xq[1]), fmaxf(xq[2], xq[3])) >= T) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (xq[e] >= T) {
              const int p = atomicAdd(&s_cnt, 1);
              if (p < kCandMax) s_cand[p] = row_key(xq[e], 4 * c + e);
            }
        }
      }
    }
  } else {
    for (int v = tid; v < a.V; v += 256) {
      const float xs = x[v];
      if (xs >= T) {
        const int p = atomicAdd(&s_cnt, 1);
        if (p < kCandMax) s_cand[p] = row_key(xs, v);
      }
    }
  }
  __syncthreads();
  const int cnt = s_cnt;

  if (cnt <= kCandMax && a.k >= kSortFromK) {                  // uniform
    // ---- wide beams: sort the candidates, the first k are the answer ------------------------------
    int n2 = 64;
    while (n2 < cnt) n2 <<= 1;
    for (int i = cnt + tid; i < n2; i += 256) s_cand[i] = 0ull;
    __syncthreads();
    block_sort_desc(s_cand, n2, tid, 256);
    for (int j = tid; j < a.k; j += 256) a.part_key[(size_t)row * a.k + j] = s_cand[j];
    if (tid == 0) a.part_sum[row] = lse;
  } else if (cnt <= 256) {                                     // uniform: the usual case, a few more than k candidates
    // ---- exact top-k among the candidates: a candidate's rank is the number of larger keys (keys are distinct) ---
    if (tid < cnt) {
      const uint64_t mine = s_cand[tid];
      int rank = 0;
      for (int j = 0; j < cnt; ++j) rank += (s_cand[j] > mine) ? 1 : 0;
      if (rank < a.k) a.part_key[(size_t)row * a.k + rank] = mine;
    } else if (tid < a.k) {
      a.part_key[(size_t)row * a.k + tid] = 0ull;              // fewer candidates than beams (V < k cannot happen; kept total)
    }
    if (tid == 0) a.part_sum[row] = lse;
  } else if (cnt <= kCandMax) {                                // uniform
    // ---- many candidates (ties at the threshold): wave 0, k rounds of wave max over its strided share ---
    if (wave == 0) {
      uint64_t mine[2] = {0ull, 0ull};                         // ranks lane and lane + 64
      for (int round = 0; round < a.k; ++round) {
        uint64_t loc = 0ull;
        for (int i = lane; i < cnt; i += 64) loc = umax64(loc, s_cand[i]);
        const uint64_t best = wave_max_u64(loc);
        if (lane == (round & 63)) mine[round >> 6] = best;
        for (int i = lane; i < cnt; i += 64)
          if (s_cand[i] == best) s_cand[i] = 0ull;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      if (lane < a.k) a.part_key[(size_t)row * a.k + lane] = mine[0];
      if (lane + 64 < a.k) a.part_key[(size_t)row * a.k + lane + 64] = mine[1];
      if (lane == 0) a.part_sum[row] = lse;
    }
  } else {
    // ---- more than kCandMax elements tie at or above T (e.g. constant logits): exact but slow ------
    // k rounds; each finds the largest key below the previous winner by a pass over the whole row.
    uint64_t* s_best = s_cand;   // [4] per-wave maxima
    uint64_t prev = ~0ull, mine = 0ull;
    for (int round = 0; round < a.k; ++round) {
      uint64_t loc = 0ull;
      for (int v = tid; v < a.V; v += 256) {
        const uint64_t key = row_key(x[v], v);
        if (key < prev) loc = umax64(loc, key);
      }
      loc = wave_max_u64(loc);
      __syncthreads();
      if (lane == 0) s_best[wave] = loc;
      __syncthreads();
      prev = umax64(umax64(s_best[0], s_best[1]), umax64(s_best[2], s_best[3]));
      if (tid == round) mine = prev;
    }
    if (tid < a.k) a.part_key[(size_t)row * a.k + tid] = mine;
    if (tid == 0) a.part_sum[row] = lse;
  }
}

hipError_t launch_row_topk(const RowTopkArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(row_topk_kernel, dim3(a.n_rows), dim3(256), 0, stream, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(64) void beam_select_kernel(BeamArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  if (!a.st.active[b]) return;
  const size_t row0 = (a.step == 0) ? (size_t)b : (size_t)b * a.k;
  const int li = min(lane, a.k - 1);
  const float old_lps = a.st.logprobsum[(size_t)b * a.k + li];
  const int old_node = a.st.beam_node[(size_t)b * a.k + li];
  beam_update(a, b, lane, a.topk_token + row0 * a.k, a.topk_logprob + row0 * a.k, a.k, old_lps, old_node);
}

__global__ __launch_bounds__(64) void depth_continue_kernel(BeamArgs a, int steps_done) {
  const int b = blockIdx.x, lane = threadIdx.x;
  if (!a.st.active[b]) return;
  const float v = (lane < a.k) ? a.st.logprobsum[(size_t)b * a.k + lane] : 0.f;
  stop_test(a, b, lane, v, steps_done);
}

hipError_t launch_beam_select(const BeamArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(beam_select_kernel, dim3(a.B), dim3(64), 0, stream, a);
  return hipGetLastError();
}
hipError_t launch_depth_continue(const BeamArgs& a, int steps_done, hipStream_t stream) {
  hipLaunchKernelGGL(depth_continue_kernel, dim3(a.B), dim3(64), 0, stream, a, steps_done);
  return hipGetLastError();
}

// ---- one launch per draft call (rows that came through the GEMM path, or a caller that runs
// the weight stream separately): one workgroup per sequence ---------------------------------------
__global__ __launch_bounds__(1024) void step_bookkeep_kernel(StepArgs a) {
  __shared__ StepSmem sm;
  __shared__ int s_last;
  __shared__ int s_word_base[DDD_BMAX / 64 + 1];
  __shared__ unsigned long long s_words[DDD_BMAX / 64];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (a.trace != nullptr && b == 0 && tid == 0) a.trace[0] = (uint64_t)wall_clock64();
  const bool active = step_bookkeep_block(a, b, tid, blockDim.x, sm);
  if (a.trace != nullptr && b == 0 && tid == 0) a.trace[5] = (uint64_t)wall_clock64();
  if (a.call_count == nullptr) return;               // uniform
  if (tid == 0) {
    // What the last workgroup needs from this one travels in atomics alone (performed at the device's
    // coherence point), so no fence is needed: the sequence's bit first, then - once that atomic has returned
    // its value - one add: arrivals in the low half, active sequences in the high half.
    uint32_t mine = 1u | (active ? 0x10000u : 0u);
    if (a.active_mask != nullptr && active) {
      const uint64_t before = __hip_atomic_fetch_or(a.active_mask + (b >> 6), 1ull << (b & 63), __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
      // the arrival below is made to depend on the value the first atomic returned: it cannot be issued earlier
      asm volatile("" : "+v"(mine) : "v"((uint32_t)before), "v"((uint32_t)(before >> 32)));
    }
    const uint32_t seen = __hip_atomic_fetch_add(a.call_count, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = (seen & 0xFFFFu) + 1u == gridDim.x;
    if (last) {
      __hip_atomic_store(a.call_count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next round
      if (a.progress != nullptr) {
        const uint32_t any = ((seen + mine) >> 16) != 0u ? 1u : 0u;
        __hip_atomic_store(a.progress, (a.round_tag << 2) | 2u | any, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      }
    }
    s_last = (last && a.active_mask != nullptr) ? 1 : 0;
  }
  __syncthreads();
  if (!s_last) return;                               // uniform
  // The last workgroup to arrive: the next call's active rows, ascending (rows b*k .. b*k+k-1 of every sequence
  // that goes on), for the GEMM path.  Every other workgroup's bit is in the mask: its arrival came after it.
  const int B = gridDim.x, k = a.beam.k, nwords = (B + 63) >> 6;
  for (int w = tid; w < nwords; w += blockDim.x) {
    s_words[w] = __hip_atomic_load(a.active_mask + w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(a.active_mask + w, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next call
  }
  __syncthreads();
  if (tid == 0) {
    int t = 0;
    for (int w = 0; w < nwords; ++w) {
      s_word_base[w] = t;
      t += __popcll(s_words[w]);
    }
    s_word_base[nwords] = t;
    *a.next_n_act = t * k;
  }
  __syncthreads();
  for (int q = tid; q < B; q += blockDim.x) {
    const unsigned long long word = s_words[q >> 6];
    if ((word >> (q & 63)) & 1ull) {
      const int pos = s_word_base[q >> 6] + __popcll(word & ((1ull << (q & 63)) - 1ull));
      for (int i = 0; i < k; ++i) a.next_row_list[pos * k + i] = q * k + i;
    }
  }
}

hipError_t launch_step_bookkeep(const StepArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(step_bookkeep_kernel, dim3(a.beam.B), dim3(64 * a.beam.k), 0, stream, a);
  return hipGetLastError();
}

// ---- poison fill of the scratch (debugging aid) -------------------------------------------------
__global__ __launch_bounds__(256) void poison_kernel(uint32_t* p, size_t n_words) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0xFFFFFFFFu;
}

hipError_t launch_poison(void* p, size_t bytes, hipStream_t stream) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  const size_t want = (n + 255) / 256;
  hipLaunchKernelGGL(poison_kernel, dim3((unsigned)(want < 2048 ? want : 2048)), dim3(256), 0, stream,
                     static_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

// ---- start of a round ------------------------------------------------------------------------
__global__ __launch_bounds__(64) void round_reset_kernel(ResetArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  if (lane == 0) {
    a.st.pool_token[(size_t)b * a.nmax] = a.root_token ? a.root_token[b] : -1;
    a.st.pool_parent[(size_t)b * a.nmax] = -1;
    a.st.pool_depth[(size_t)b * a.nmax] = 0;
    a.st.pool_score[(size_t)b * a.nmax] = 0.f;
    a.st.n_nodes[b] = 1;
    a.st.steps[b] = 0;
    a.st.active[b] = 1;
    a.st.conf[b] = 1.0;
  }
  if (lane < a.k) a.st.row_active[(size_t)b * a.k + lane] = 1;
}

hipError_t launch_round_reset(const ResetArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(round_reset_kernel, dim3(a.B), dim3(64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
