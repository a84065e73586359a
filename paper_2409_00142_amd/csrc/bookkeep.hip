// Per-row merge of the weight-stream partials, beam update and DDD stop test.
//
// merge_row      one wave per hidden row: combines the per-slice (max, sum of exponentials)
//                into lse, and picks the row's top-k tokens: the k slices with the best
//                heads contain every global top-k element, so only their k*k keys are ranked.
// beam_update    one wave per sequence: score = logprobsum[parent] + logprob (one fp32 add),
//                all k*k candidates go to the node pool, the k best by (score desc, token asc,
//                flat index asc) become the new beam (Algorithm 1, "postprocess ... to
//                produce the new beam", "calculate logprobsum").
// stop_test      Eq. 1 in the probability domain: P = sum_i exp(logprobsum[i]) in fp64, index
//                order; continue iff another call is allowed and (step not in S or P >= t).
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"
#include "tree_device.hpp"

namespace ddd {

constexpr int kKM = DDD_KMAX;

// All 64 lanes of the calling wave must be active.  On return lane j < k holds the rank-j key.
constexpr int kHPL = 8;   // heads per lane: up to 512 slices

// Issue the loads of a row's slice heads, runners-up and sums (lane handles slices lane, lane+64, ...).
__device__ __forceinline__ void merge_load_heads(const uint64_t* __restrict__ pk, const float* __restrict__ ps,
                                                 int nslice, int k, int lane, uint64_t (&head)[kHPL],
                                                 uint64_t (&second)[kHPL], float (&psum)[kHPL]) {
#pragma unroll
  for (int i = 0; i < kHPL; ++i) {
    const int s = lane + 64 * i;
    head[i] = (s < nslice) ? pk[(size_t)s * k] : 0ull;
    second[i] = (s < nslice && k > 1) ? pk[(size_t)s * k + 1] : 0ull;
    psum[i] = (s < nslice) ? ps[s] : 0.f;
  }
}

// All 64 lanes of the calling wave must be active.  On return lane j < k holds the rank-j key.
//
// The k slices with the best heads contain every global top-k element.  If none of their
// runners-up beats the k-th best head, the k best heads are the answer (the common case);
// otherwise the k*k keys of those slices are fetched and ranked.
template <int HPL>
__device__ __forceinline__ void merge_row(const uint64_t* __restrict__ pk, uint64_t (&head)[kHPL],
                                          const uint64_t (&second)[kHPL], const float (&psum)[kHPL], int k, int lane,
                                          int* wl, uint64_t& my_key, float& lse) {
  uint64_t loc = 0;
#pragma unroll
  for (int i = 0; i < HPL; ++i) loc = umax64(loc, head[i]);
  const float M = unord32(wave_max_u32((uint32_t)(loc >> 32)));
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < HPL; ++i)
    if (head[i] != 0ull) acc += psum[i] * __expf(key_value(head[i]) - M);
  lse = M + __logf(wave_sum_f32(acc));

  my_key = 0ull;
  uint64_t best = 0ull, sec_of_winners = 0ull;
  for (int round = 0; round < k; ++round) {
    loc = 0;
#pragma unroll
    for (int i = 0; i < HPL; ++i) loc = umax64(loc, head[i]);
    best = wave_max_u64(loc);
    if (lane == round) my_key = best;
    if (best == 0ull) {
      if (lane == 0) wl[round] = -1;
    } else {
#pragma unroll
      for (int i = 0; i < HPL; ++i)
        if (head[i] == best) {
          wl[round] = lane + 64 * i;
          head[i] = 0ull;
          sec_of_winners = umax64(sec_of_winners, second[i]);
        }
    }
  }
  // `best` is now the k-th best head (0 if there are fewer than k non-empty slices)
  const uint64_t best_second = wave_max_u64(sec_of_winners);
  if (best != 0ull && best_second < best) return;   // uniform: the heads are the top-k

  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  uint64_t cand[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int cidx = lane + 64 * i;
    cand[i] = 0ull;
    if (cidx < k * k) {
      const int s = wl[cidx / k];
      if (s >= 0) cand[i] = pk[(size_t)s * k + (cidx % k)];
    }
  }
  my_key = 0ull;
  for (int round = 0; round < k; ++round) {
    loc = umax64(umax64(cand[0], cand[1]), umax64(cand[2], cand[3]));
    best = wave_max_u64(loc);
    if (lane == round) my_key = best;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (cand[i] == best) cand[i] = 0ull;
  }
}

__device__ __forceinline__ void merge_row_dispatch(const uint64_t* pk, uint64_t (&head)[kHPL],
                                                   const uint64_t (&second)[kHPL], const float (&psum)[kHPL],
                                                   int nslice, int k, int lane, int* wl, uint64_t& my_key,
                                                   float& lse) {
  if (nslice <= 64)
    merge_row<1>(pk, head, second, psum, k, lane, wl, my_key, lse);
  else if (nslice <= 128)
    merge_row<2>(pk, head, second, psum, k, lane, wl, my_key, lse);
  else if (nslice <= 256)
    merge_row<4>(pk, head, second, psum, k, lane, wl, my_key, lse);
  else
    merge_row<8>(pk, head, second, psum, k, lane, wl, my_key, lse);
}

// ---- standalone merge: one wave per row ------------------------------------------------------
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs a) {
  __shared__ int wl[4][kKM];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= a.n_rows) return;                                 // wave-uniform
  if (a.row_active != nullptr && !a.row_active[row]) return;   // wave-uniform
  uint64_t key;
  float lse;
  if (a.nslice == 0) {   // dense format: the keys are final
    key = a.part_key[(size_t)row * a.k + min(lane, a.k - 1)];
    lse = a.part_sum[row];
  } else {
    uint64_t head[kHPL], second[kHPL];
    float psum[kHPL];
    const uint64_t* pk = a.part_key + (size_t)row * a.nslice * a.k;
    merge_load_heads(pk, a.part_sum + (size_t)row * a.nslice, a.nslice, a.k, lane, head, second, psum);
    merge_row_dispatch(pk, head, second, psum, a.nslice, a.k, lane, wl[wave], key, lse);
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
// T is a lower bound of the row's k-th largest logit (k distinct elements are >= T), so one
// compare-only pass over the row collects the few candidates >= T, and the exact top-k by
// (logit desc, token asc) is taken among them.  If more candidates than fit turn up (massive
// ties, e.g. constant logits), an exact but slow path takes over: k passes over the row, each
// finding the largest key below the previous winner.
constexpr int kCandMax = 1024;

__global__ __launch_bounds__(256) void row_topk_kernel(RowTopkArgs a) {
  __shared__ uint64_t s_cand[kCandMax];
  __shared__ float s_red[8];
  __shared__ float s_T;
  __shared__ int s_cnt;
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
  if (tid == 0) s_cnt = 0;
  if (wave == 0) {
    // up to 2048 groups (V <= 131072): 32 per lane, kept as ordered keys, k rounds of wave max
    uint32_t loc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const int g = lane + 64 * i;
      loc[i] = (g < ngrp_valid) ? ord32(gmax[g]) : 0u;
    }
    uint32_t T = 0u;
    for (int round = 0; round < a.k; ++round) {
      uint32_t lm = 0u;
#pragma unroll
      for (int i = 0; i < 32; ++i) lm = umax32(lm, loc[i]);
      T = wave_max_u32(lm);
      if (T == 0u) break;                                    // uniform: fewer than k groups
      // remove one holder of the maximum (the lowest lane, its lowest slot)
      const unsigned long long holders = __ballot(lm == T);
      if (lane == __ffsll((long long)holders) - 1) {
        bool done = false;
#pragma unroll
        for (int i = 0; i < 32; ++i)
          if (!done && loc[i] == T) {
            loc[i] = 0u;
            done = true;
          }
      }
    }
    if (lane == 0) s_T = (T == 0u) ? -INFINITY : unord32(T);
  }
  __syncthreads();
  const float lse = M + __logf(s_red[4] + s_red[5] + s_red[6] + s_red[7]);

  // ---- collect candidates >= T ------------------------------------------------------------------
  const float* x = a.logits + (size_t)row * a.V;
  const float T = s_T;
  if ((a.V & 3) == 0) {
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
        const float xv[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
        if (c < nchunk && fmaxf(fmaxf(xv[0], xv[1]), fmaxf(xv[2], xv[3])) >= T) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (xv[e] >= T) {
              const int p = atomicAdd(&s_cnt, 1);
              if (p < kCandMax) s_cand[p] = row_key(xv[e], 4 * c + e);
            }
        }
      }
    }
  } else {
    for (int v = tid; v < a.V; v += 256) {
      const float xv = x[v];
      if (xv >= T) {
        const int p = atomicAdd(&s_cnt, 1);
        if (p < kCandMax) s_cand[p] = row_key(xv, v);
      }
    }
  }
  __syncthreads();
  const int cnt = s_cnt;

  if (cnt <= kCandMax) {                                       // uniform
    // ---- exact top-k among the candidates: wave 0, k rounds of wave max over its strided share ---
    if (wave == 0) {
      uint64_t mine = 0ull;
      for (int round = 0; round < a.k; ++round) {
        uint64_t loc = 0ull;
        for (int i = lane; i < cnt; i += 64) loc = umax64(loc, s_cand[i]);
        const uint64_t best = wave_max_u64(loc);
        if (lane == round) mine = best;
        for (int i = lane; i < cnt; i += 64)
          if (s_cand[i] == best) s_cand[i] = 0ull;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      if (lane < a.k) a.part_key[(size_t)row * a.k + lane] = mine;
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

// ---- beam update by one wave (all 64 lanes active) -------------------------------------------
// tok/lp: rows of k entries with the given row stride (LDS or global).  old_lps / old_node: the
// current beam as loaded by lane i < k (ignored for step 0).
// Returns the new logprobsum of beam slot `lane` (lanes >= k: 0).
__device__ __forceinline__ float beam_update(const BeamArgs& a, int b, int lane, const int32_t* tok, const float* lp,
                                             int stride, float old_lps, int old_node) {
  const int k = a.k, step = a.step;
  float* lps = a.st.logprobsum + (size_t)b * k;
  int32_t* bnode = a.st.beam_node + (size_t)b * k;
  int32_t* btok = a.st.beam_token + (size_t)b * k;
  int32_t* bslot = a.st.beam_parent_slot + (size_t)b * k;
  int32_t* ptok = a.st.pool_token + (size_t)b * a.nmax;
  int32_t* ppar = a.st.pool_parent + (size_t)b * a.nmax;
  int32_t* pdep = a.st.pool_depth + (size_t)b * a.nmax;
  float* psc = a.st.pool_score + (size_t)b * a.nmax;

  float new_lps = 0.f;
  if (step == 0) {
    if (lane < k) {
      const int nid = 1 + lane;
      const int t = tok[lane];
      const float s = lp[lane];
      ptok[nid] = t;
      ppar[nid] = 0;
      pdep[nid] = 1;
      psc[nid] = s;
      bnode[lane] = nid;
      btok[lane] = t;
      bslot[lane] = 0;
      lps[lane] = s;
      new_lps = s;
    }
    if (lane == 0) a.st.n_nodes[b] = 1 + k;
  } else {
    const int base = 1 + k + (step - 1) * k * k;
    uint64_t cand[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int f = lane + 64 * i;
      cand[i] = 0ull;
      const int slot = min(f / k, k - 1), j = f - slot * k;
      const float plps = __shfl(old_lps, slot, 64);   // parent's logprobsum and pool id
      const int pnode = __shfl(old_node, slot, 64);
      if (f < k * k) {
        const int t = tok[slot * stride + j];
        const float sc = __fadd_rn(plps, lp[slot * stride + j]);
        ptok[base + f] = t;
        ppar[base + f] = pnode;
        pdep[base + f] = step + 1;
        psc[base + f] = sc;
        cand[i] = beam_key(sc, t, f);
      }
    }
    uint64_t mine = 0ull;
    for (int round = 0; round < k; ++round) {
      const uint64_t loc = umax64(umax64(cand[0], cand[1]), umax64(cand[2], cand[3]));
      const uint64_t best = wave_max_u64(loc);
      if (lane == round) mine = best;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (cand[i] == best) cand[i] = 0ull;
    }
    if (lane < k) {
      const int f = beam_key_flat(mine);
      const int t = (int)(0xFFFFFFu - (((uint32_t)mine >> 8) & 0xFFFFFFu));
      new_lps = key_value(mine);
      bnode[lane] = base + f;
      btok[lane] = t;
      bslot[lane] = f / k;
      lps[lane] = new_lps;
    }
    if (lane == 0) a.st.n_nodes[b] = base + k * k;
  }
  if (lane == 0) a.st.steps[b] = step + 1;
  return new_lps;
}

// Stop test by one wave; lane i < k passes its logprobsum.  steps_done = draft calls made so far.
__device__ __forceinline__ bool stop_test(const BeamArgs& a, int b, int lane, float my_lps, int steps_done) {
  const double e = (lane < a.k) ? exp((double)my_lps) : 0.0;
  const unsigned long long eb = (unsigned long long)__double_as_longlong(e);
  double P = 0.0;
#pragma unroll
  for (int i = 0; i < kKM; ++i) {   // index order; lanes >= k contribute exactly +0.0
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)eb, i);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(eb >> 32), i);
    P += __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
  }
  bool cont = steps_done < a.D;
  if (cont && ((a.check_mask >> steps_done) & 1u) && P < (double)a.threshold) cont = false;
  if (lane == 0) {
    a.st.conf[b] = P;
    a.st.active[b] = cont ? 1 : 0;
  }
  if (lane < a.k) a.st.row_active[(size_t)b * a.k + lane] = cont ? 1 : 0;
  return cont;
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

// ---- one launch per draft call: merge of the sequence's rows, beam update, stop test, and the
// final tree as soon as the sequence stops ---------------------------------------------------------
__global__ __launch_bounds__(1024) void step_bookkeep_kernel(StepArgs a) {
  __shared__ int wl[kKM][kKM];
  __shared__ int s_tok[kKM][kKM];
  __shared__ float s_lp[kKM][kKM];
  __shared__ int s_stopped;
  __shared__ TreeSmem tsm;
  const BeamArgs& g = a.beam;
  const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int rows = (g.step == 0) ? 1 : g.k;
  const size_t row0 = (g.step == 0) ? (size_t)b : (size_t)b * g.k;
  // Issue every independent load first: the flag, this wave's slice heads, the current beam.
  const uint8_t active = g.st.active[b];
  const size_t row = row0 + min(wave, rows - 1);
  const bool dense = (a.nslice == 0);             // keys already final (rows came through the GEMM path)
  const uint64_t* pk = a.part_key + row * (dense ? 1 : a.nslice) * g.k;
  uint64_t head[kHPL], second[kHPL];
  float psum[kHPL];
  uint64_t dkey = 0ull;
  float dlse = 0.f;
  if (dense) {
    dkey = pk[min(lane, g.k - 1)];
    dlse = a.part_sum[row];
  } else {
    merge_load_heads(pk, a.part_sum + row * a.nslice, a.nslice, g.k, lane, head, second, psum);
  }
  const int li = min(lane, g.k - 1);
  const float old_lps = g.st.logprobsum[(size_t)b * g.k + li];
  const int old_node = g.st.beam_node[(size_t)b * g.k + li];
  if (!active) return;                            // uniform over the workgroup
  if (threadIdx.x == 0) s_stopped = 0;
  if (wave < rows) {
    uint64_t key = dkey;
    float lse = dlse;
    if (!dense) merge_row_dispatch(pk, head, second, psum, a.nslice, g.k, lane, wl[wave], key, lse);
    if (lane < g.k) {
      s_tok[wave][lane] = key_token(key);
      s_lp[wave][lane] = key_value(key) - lse;
    }
    if (a.lse_dbg != nullptr && lane == 0) a.lse_dbg[row] = lse;
  }
  __syncthreads();
  if (wave == 0) {
    const float v = beam_update(g, b, lane, &s_tok[0][0], &s_lp[0][0], kKM, old_lps, old_node);
    const bool cont = stop_test(g, b, lane, v, g.step + 1);
    if (lane == 0 && !cont) s_stopped = 1;
  }
  __syncthreads();                                // also orders wave 0's pool writes before the reads below
  if (a.tree.mask != nullptr && s_stopped)
    tree_finalize_block(g.st, a.tree, b, a.m, g.nmax, threadIdx.x, blockDim.x, tsm);
}

hipError_t launch_step_bookkeep(const StepArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(step_bookkeep_kernel, dim3(a.beam.B), dim3(64 * a.beam.k), 0, stream, a);
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
