// Device code of the per-call bookkeeping: per-row merge of the stream partials, beam update,
// DDD stop test, and the step function that strings them together for one sequence.
//
// merge_row      one wave per hidden row: combines the per-slice (max, sum of exponentials)
//                into lse, and picks the row's top-k tokens by a k-way merge of the slices'
//                sorted lists (three keys per slice in registers).
// beam_update    one wave per sequence: score = logprobsum[parent] + logprob (one fp32 add),
//                all k*k candidates go to the node pool, the k best by (score desc, token asc,
//                flat index asc) become the new beam (Algorithm 1: the step that turns the draft
//                outputs into the next beam and its summed log-probabilities).
// stop_test      Eq. 1 in the probability domain: P = sum_i exp(logprobsum[i]) in fp64, index
//                order; continue iff another call is allowed and (step not in S or P >= t).
#pragma once
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"
#include "tree_device.hpp"

namespace ddd {

constexpr int kKM = DDD_KMAX;

constexpr int kHPL = 4;   // slices per lane: up to 256 slices (one per compute unit of the chip)

// The three best keys of each of a lane's slices (lane handles slices lane, lane + 64, ...) and the
// slices' sums of exponentials.
struct RowHeads {
  uint64_t q0[kHPL], q1[kHPL], q2[kHPL];
  float psum[kHPL];
};

// Issue the loads of a row's slice heads, their two runners-up and the sums.
__device__ __forceinline__ void merge_load_heads(const uint64_t* __restrict__ pk, const float* __restrict__ ps,
                                                 int nslice, int k, int lane, RowHeads& h) {
#pragma unroll
  for (int i = 0; i < kHPL; ++i) {
    const int s = lane + 64 * i;
    h.q0[i] = (s < nslice) ? pk[s] : 0ull;
    h.q1[i] = (s < nslice && k > 1) ? pk[nslice + s] : 0ull;
    h.q2[i] = (s < nslice && k > 2) ? pk[2 * nslice + s] : 0ull;
    h.psum[i] = (s < nslice) ? ps[s] : 0.f;
  }
}

// All 64 lanes of the calling wave must be active.  On return lane j < k holds the rank-j key.
//
// Every slice's list is sorted, so the next global best is always the front of some slice: k
// rounds of "wave-wide max of the fronts, the owner moves on to its slice's next key".  The first
// three keys of every slice are in registers; a slice that places more than three keys among the
// row's k best (for k = 10 and 256 slices about one row in 500) fetches its further keys one at
// a time as they are needed.
template <int HPL>
__device__ __forceinline__ void merge_row(const uint64_t* __restrict__ pk, RowHeads& h, int nslice, int k, int lane,
                                          uint64_t& my_key, float& lse) {
  uint64_t loc = 0;
#pragma unroll
  for (int i = 0; i < HPL; ++i) loc = umax64(loc, h.q0[i]);
  const float M = unord32(wave_max_u32((uint32_t)(loc >> 32)));
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < HPL; ++i)
    if (h.q0[i] != 0ull) acc += h.psum[i] * __expf(key_value(h.q0[i]) - M);
  lse = M + __logf(wave_sum_f32(acc));

  constexpr uint64_t kFetch = 1ull;    // "not in registers": no key has this value (its token would be 2^32 - 2)
  int taken[HPL];
#pragma unroll
  for (int i = 0; i < HPL; ++i) taken[i] = 0;
  my_key = 0ull;
  for (int round = 0; round < k; ++round) {
    loc = 0;
#pragma unroll
    for (int i = 0; i < HPL; ++i) loc = umax64(loc, h.q0[i]);
    // The high words (the logits) decide unless two slices' fronts tie in them: one 32-bit wave maximum and the
    // ballot of its holders; only a tie needs the second reduction over the low words (the tokens).
    const uint32_t hi = (uint32_t)(loc >> 32);
    const uint32_t M = wave_max_u32(hi);
    const unsigned long long holders = __ballot(hi == M);
    uint64_t best;
    int owner;
    if (__popcll(holders) == 1) {      // uniform
      owner = __ffsll(holders) - 1;
      best = ((uint64_t)M << 32) | (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)loc, owner);
    } else {
      const uint32_t L = wave_max_u32(hi == M ? (uint32_t)loc : 0u);
      best = ((uint64_t)M << 32) | L;
      owner = __ffsll((unsigned long long)__ballot(loc == best)) - 1;
    }
    if (lane == round) my_key = best;
    if (best == 0ull) break;           // uniform: fewer than k keys in the row
    // Keys are distinct (every token sits in one slice), so exactly one slot of the owner lane holds the best:
    // its index is made uniform and only that slot's update is issued (the wave would otherwise execute
    // the update of every slot for the sake of one lane).
    int which = -1;
#pragma unroll
    for (int i = 0; i < HPL; ++i)
      if (h.q0[i] == best) which = i;
    const int iu = __builtin_amdgcn_readlane(which, owner);
#pragma unroll
    for (int i = 0; i < HPL; ++i)
      if (iu == i) {                     // uniform
        if (which == i) {
          ++taken[i];
          h.q0[i] = h.q1[i];
          h.q1[i] = h.q2[i];
          h.q2[i] = (taken[i] + 2 < k) ? kFetch : 0ull;
          if (h.q0[i] == kFetch) h.q0[i] = pk[(size_t)taken[i] * nslice + lane + 64 * i];   // fourth key onwards
        }
      }
  }
}

// The same result without the k dependent rounds, for the usual row (all 64 lanes active; scratch: kMergeWords
// 64-bit words of LDS that belong to the calling wave).  A lower bound of the row's k-th best logit comes first: the
// 16 quads of lanes each hold 16 slices, the k-th largest of the 16 quad maxima is reached by k distinct keys (k <= 16).
// Every key at or above the bound is a candidate - the best fronts and a few runners-up, 20 to 30 keys -, the
// candidates are written to LDS, one per lane, and a candidate's rank is the number of larger candidates (keys are
// distinct).  The k rounds above are a chain of cross-lane reductions and scalar round trips (0.37 us each with ten
// waves on four SIMDs); the counting loops are independent iterations.  A slice whose third key is a candidate
// may hold more of them, and more than 64 candidates do not fit: such rows (about one in a hundred) take the rounds.
constexpr int kMergeWords = 64 + kKM;
template <int HPL>
__device__ __forceinline__ void merge_row_count(const uint64_t* __restrict__ pk, RowHeads& h, int nslice, int k, int lane,
                                                uint64_t& my_key, float& lse, uint64_t* scratch) {
  uint64_t loc = 0;
#pragma unroll
  for (int i = 0; i < HPL; ++i) loc = umax64(loc, h.q0[i]);
  const uint32_t lm = (uint32_t)(loc >> 32);
  // quad maxima (every lane of a quad holds its quad's), then how many of the 16 are larger than this one
  uint32_t qm = umax32(lm, dpp_move_u32<0xB1>(lm));
  qm = umax32(qm, dpp_move_u32<0x4E>(qm));
  int larger = 0;
#pragma unroll
  for (int q = 0; q < 16; ++q) larger += ((uint32_t)__builtin_amdgcn_readlane((int)qm, 4 * q) > qm) ? 1 : 0;
  // the smallest of the quad maxima that fewer than k others exceed = the k-th largest (ties included)
  const uint32_t bound = ~wave_max_u32(~(larger < k ? qm : 0xFFFFFFFFu));
  bool more = false;
  int base = 0;
  uint64_t* cand = scratch;          // [64]
  uint64_t* out = scratch + 64;      // [kKM]
  if (lane < kKM) out[lane] = 0ull;
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int i = 0; i < HPL; ++i) {
      const uint64_t key = (r == 0) ? h.q0[i] : (r == 1) ? h.q1[i] : h.q2[i];
      const bool in = key != 0ull && (uint32_t)(key >> 32) >= bound;
      const unsigned long long bal = __ballot(in);
      if (bal == 0ull) continue;                                   // uniform
      const int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
      if (in && pos < 64) cand[pos] = key;
      base += __popcll(bal);
      if (r == 2 && in && k > 3) more = true;
    }
  if (__ballot(more) != 0ull || base > 64) {                       // uniform
    merge_row<HPL>(pk, h, nslice, k, lane, my_key, lse);
    return;
  }
  // lse as in the rounds' version
  const float M = unord32(wave_max_u32(lm));
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < HPL; ++i)
    if (h.q0[i] != 0ull) acc += h.psum[i] * __expf(key_value(h.q0[i]) - M);
  lse = M + __logf(wave_sum_f32(acc));
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int C = base;
  const uint64_t mine = (lane < C) ? cand[lane] : 0ull;
  int rank = 0;
  for (int j = 0; j < C; ++j) rank += (cand[j] > mine) ? 1 : 0;
  if (lane < C && rank < k) out[rank] = mine;
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
  my_key = (lane < k) ? out[lane] : 0ull;
}

__device__ __forceinline__ void merge_row_dispatch(const uint64_t* pk, RowHeads& h, int nslice, int k, int lane,
                                                   uint64_t& my_key, float& lse, uint64_t* scratch) {
  merge_row_count<kHPL>(pk, h, nslice, k, lane, my_key, lse, scratch);
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

// ---- one draft call of one sequence by one workgroup: merge of the sequence's rows, beam update,
// stop test, and the final tree as soon as the sequence stops.  Every thread of the block must
// call it (nthr a multiple of 64, at least 64); the rows are dealt round-robin to the waves.
struct StepSmem {
  TreeSmem tsm;
  int tok[kKM][kKM];
  float lp[kKM][kKM];
  uint64_t cand[kKM * kKM];   // beam keys of the k*k candidates (beam update by the whole block)
  int rank[kKM * kKM];        // number of candidates with a larger key
  float newlps[kKM];          // logprobsum of the new beam
  uint64_t mrg[kKM][kMergeWords];   // per wave: candidates of the row merge and its result
  int stopped;
};

__device__ __forceinline__ void step_publish_row(const StepArgs& a, StepSmem& sm, int rw, size_t row, int lane,
                                                 uint64_t key, float lse) {
  if (lane < a.beam.k) {
    sm.tok[rw][lane] = key_token(key);
    sm.lp[rw][lane] = key_value(key) - lse;
  }
  if (a.lse_dbg != nullptr && lane == 0) a.lse_dbg[row] = lse;
}

// Returns whether the sequence is still active after this call (the same value in every thread).
__device__ __forceinline__ bool step_bookkeep_block(const StepArgs& a, int b, int tid, int nthr, StepSmem& sm) {
  const BeamArgs& g = a.beam;
  const int wave = tid >> 6, lane = tid & 63, nwaves = nthr >> 6;
  const int rows = (g.step == 0) ? 1 : g.k;
  const size_t row0 = (g.step == 0) ? (size_t)b : (size_t)b * g.k;
  // Issue every independent load first: the flag, this wave's slice heads, the current beam.
  const uint8_t active = g.st.active[b];
  const bool dense = (a.nslice == 0);             // keys already final (rows came through the GEMM path)
  const size_t row = row0 + min(wave, rows - 1);
  const uint64_t* pk = a.part_key + row * (dense ? 1 : a.nslice) * g.k;
  RowHeads heads;
  uint64_t key = 0ull;
  float lse = 0.f;
  if (dense) {
    key = pk[min(lane, g.k - 1)];
    lse = a.part_sum[row];
  } else {
    merge_load_heads(pk, a.part_sum + row * a.nslice, a.nslice, g.k, lane, heads);
  }
  const int li = min(lane, g.k - 1);
  const float old_lps = g.st.logprobsum[(size_t)b * g.k + li];
  const int old_node = g.st.beam_node[(size_t)b * g.k + li];
  if (!active) return false;                      // uniform over the workgroup
  if (tid == 0) sm.stopped = 0;
  uint64_t* const trace = (a.trace != nullptr && b == 0 && tid == 0) ? a.trace : nullptr;
  if (trace != nullptr) {   // the stamp must follow the arrival of this wave's keys: use one
    if (!dense && heads.q2[kHPL - 1] == 1ull) trace[7] = 1;       // (never true: keys are never 1)
    trace[1] = (uint64_t)wall_clock64();
  }
  // One wave per row (every call after the prompt call, launched with 64 * k threads): the whole block takes
  // part in the beam update.  Otherwise (the prompt call's single row; fewer waves than rows) wave 0 does it
  // from the rows' results in LDS.
  const bool by_block = g.step >= 1 && nwaves >= rows;
  if (wave < rows) {
    if (!dense) merge_row_dispatch(pk, heads, a.nslice, g.k, lane, key, lse, sm.mrg[wave]);
    if (!by_block) step_publish_row(a, sm, wave, row, lane, key, lse);
  }
  if (trace != nullptr) trace[2] = (uint64_t)wall_clock64();
  if (by_block) {
    // ---- Algorithm 1's beam update by all k waves: wave i holds row i's k candidates in its lanes j < k ------
    const int k = g.k, kk = k * k;
    const int base = 1 + k + (g.step - 1) * kk;
    const int wv = __builtin_amdgcn_readfirstlane(wave);
    const bool owner = wave < rows && lane < k;
    const int f = wv * k + lane;                       // flat index of this lane's candidate
    float sc = 0.f;
    int tkn = 0;
    if (wave < rows) {
      // the parent's logprobsum and pool id: lane i of every wave loaded slot i's
      const float plps = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(old_lps), wv));
      const int pnode = __builtin_amdgcn_readlane(old_node, wv);
      if (a.lse_dbg != nullptr && lane == 0) a.lse_dbg[row] = lse;
      if (owner) {
        tkn = key_token(key);
        sc = __fadd_rn(plps, key_value(key) - lse);    // logprob = logit - lse, then one fp32 add
        const size_t pn = (size_t)b * g.nmax + base + f;
        g.st.pool_token[pn] = tkn;
        g.st.pool_parent[pn] = pnode;
        g.st.pool_depth[pn] = g.step + 1;
        g.st.pool_score[pn] = sc;
        sm.cand[f] = beam_key(sc, tkn, f);
        sm.rank[f] = 0;
      }
    }
    __syncthreads();
    // rank = number of larger keys (keys are distinct: the flat index is part of them); the k*k comparisons of a
    // candidate are shared by the 64 / k lane groups of its wave
    if (wave < rows) {
      const int P = 64 / k, part = lane / k, j = lane - part * k;
      if (part < P) {
        const uint64_t mine = sm.cand[wv * k + j];
        const int chunk = (kk + P - 1) / P, lo = part * chunk, hi = min(kk, lo + chunk);
        int cnt = 0;
        for (int x = lo; x < hi; ++x) cnt += (sm.cand[x] > mine) ? 1 : 0;
        if (cnt != 0) atomicAdd(&sm.rank[wv * k + j], cnt);
      }
    }
    __syncthreads();
    if (owner) {
      const int rk = sm.rank[f];
      if (rk < k) {                                    // this candidate is slot rk of the new beam
        g.st.beam_node[(size_t)b * k + rk] = base + f;
        g.st.beam_token[(size_t)b * k + rk] = tkn;
        g.st.beam_parent_slot[(size_t)b * k + rk] = wv;
        g.st.logprobsum[(size_t)b * k + rk] = sc;
        sm.newlps[rk] = sc;
      }
    }
    if (tid == 0) {
      g.st.n_nodes[b] = base + kk;
      g.st.steps[b] = g.step + 1;
    }
    __syncthreads();
    if (wave == 0) {
      const bool cont = stop_test(g, b, lane, lane < k ? sm.newlps[lane] : 0.f, g.step + 1);
      if (lane == 0 && !cont) sm.stopped = 1;
    }
  } else {
  for (int rw = wave + nwaves; rw < rows; rw += nwaves) {   // fewer waves than rows: further passes
    const size_t row2 = row0 + rw;
    const uint64_t* pk2 = a.part_key + row2 * (dense ? 1 : a.nslice) * g.k;
    uint64_t key2;
    float lse2;
    if (dense) {
      key2 = pk2[min(lane, g.k - 1)];
      lse2 = a.part_sum[row2];
    } else {
      RowHeads heads2;
      merge_load_heads(pk2, a.part_sum + row2 * a.nslice, a.nslice, g.k, lane, heads2);
      merge_row_dispatch(pk2, heads2, a.nslice, g.k, lane, key2, lse2, sm.mrg[wave]);
    }
    step_publish_row(a, sm, rw, row2, lane, key2, lse2);
  }
  __syncthreads();
  if (wave == 0) {
    const float v = beam_update(g, b, lane, &sm.tok[0][0], &sm.lp[0][0], kKM, old_lps, old_node);
    const bool cont = stop_test(g, b, lane, v, g.step + 1);
    if (lane == 0 && !cont) sm.stopped = 1;
  }
  }
  __syncthreads();                                // also orders wave 0's pool writes before the reads below
  if (trace != nullptr) trace[3] = (uint64_t)wall_clock64();
  if (a.tree.mask != nullptr && sm.stopped)   // pool size after this call: 1 + k + step * k^2 (as beam_update just stored it)
    tree_finalize_block(g.st, a.tree, b, a.m, g.nmax, tid, nthr, sm.tsm, 1 + g.k + g.step * g.k * g.k);
  if (trace != nullptr) trace[4] = (uint64_t)wall_clock64();
  return !sm.stopped;
}

}  // namespace ddd
