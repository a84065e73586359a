// Final draft tree of one sequence, built by one workgroup (device functions shared by the
// stand-alone finalize kernels and the per-call bookkeeping kernels).
//
// Section 1: the m best nodes of the draft tree by summed logprob go to the target model in
// one pass; a node may attend to itself and its ancestors only.  Rerank key: (score desc,
// node id asc); tree order: ascending node id.
#pragma once
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"

namespace ddd {

constexpr int kPoolMax = DDD_POOL_MAX;
constexpr int kTreeMax = DDD_MMAX + 1;
constexpr int kMaskWords = (kTreeMax + 31) / 32;

// Working set of the part that follows the selection (at most m + 1 nodes).
struct TreeEmitSmem {
  int pick[kTreeMax];                   // pool ids of the m_eff best nodes, any order
  int sel[kTreeMax];                    // pool ids of tree indices 0..m_eff (0 = root), ascending
  int par[kTreeMax];                    // tree index of the parent
  uint32_t bits[kTreeMax][kMaskWords];  // ancestor bit rows
};

struct TreeSmem {
  uint64_t keys[kPoolMax + 2];          // rerank keys of pool nodes 1..N (+ padding)
  TreeEmitSmem e;
};

__device__ __forceinline__ uint64_t rerank_key(float score, int node) {
  return ((uint64_t)ord32(score) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)node);
}

// From the m_eff chosen pool ids in sm.pick (any order, already visible to the block): order
// them by id, find parents, ancestor rows, and write the tree.  Every thread of the block calls it.
__device__ __forceinline__ void tree_emit_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int m_eff,
                                                int nmax, int tid, int nthr, TreeEmitSmem& sm) {
  const int T = m + 1;
  const int32_t* ppar = st.pool_parent + (size_t)b * nmax;
  const int32_t* pdep = st.pool_depth + (size_t)b * nmax;
  const int32_t* ptok = st.pool_token + (size_t)b * nmax;
  // chosen ids in ascending order: rank by counting
  if (tid == 0) sm.sel[0] = 0;
  for (int i = tid; i < m_eff; i += nthr) {
    const int id = sm.pick[i];
    int rank = 0;
    for (int j = 0; j < m_eff; ++j) rank += (sm.pick[j] < id) ? 1 : 0;
    sm.sel[1 + rank] = id;
  }
  __syncthreads();
  // parents as tree indices (a parent has a smaller id, hence a smaller tree index); the node's
  // token and depth are requested in the same round trip as its parent's id and kept until the
  // tree is written (tree index tid; a block narrower than the tree takes the rest in a plain loop)
  const bool mine = tid <= m_eff;
  const int my_node = mine ? sm.sel[tid] : 0;
  const int my_pn = (mine && tid > 0) ? ppar[my_node] : -1;
  const int my_tok = mine ? ptok[my_node] : -1;
  const int my_dep = mine ? pdep[my_node] : 0;
  if (mine) {
    int par = -1;
    for (int j = 0; j < tid; ++j)
      if (sm.sel[j] == my_pn) par = j;
    sm.par[tid] = par;
  }
  for (int i = tid + nthr; i <= m_eff; i += nthr) {
    const int pn = ppar[sm.sel[i]];
    int par = -1;
    for (int j = 0; j < i; ++j)
      if (sm.sel[j] == pn) par = j;
    sm.par[i] = par;
  }
  __syncthreads();
  for (int i = tid; i < T; i += nthr) {
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) sm.bits[i][w] = 0u;
    if (i <= m_eff) {
      int c = i;
      while (c >= 0) {
        sm.bits[i][c >> 5] |= (1u << (c & 31));
        c = sm.par[c];
      }
    }
  }
  __syncthreads();
  if (tid == 0) tree.n_sel[b] = m_eff;
  for (int i = tid; i < m; i += nthr) tree.sel_node[(size_t)b * m + i] = (i < m_eff) ? sm.sel[1 + i] : -1;
  if (tid < T) {
    tree.tree_token[(size_t)b * T + tid] = my_tok;
    tree.pos[(size_t)b * T + tid] = my_dep;
    tree.parent_idx[(size_t)b * T + tid] = mine ? sm.par[tid] : -1;
  }
  for (int i = tid + nthr; i < T; i += nthr) {
    const bool ok = (i <= m_eff);
    const int node = ok ? sm.sel[i] : 0;
    tree.tree_token[(size_t)b * T + i] = ok ? ptok[node] : -1;
    tree.pos[(size_t)b * T + i] = ok ? pdep[node] : 0;
    tree.parent_idx[(size_t)b * T + i] = ok ? sm.par[i] : -1;
  }
  uint8_t* mask = tree.mask + (size_t)b * T * T;
  for (int e = tid; e < T * T; e += nthr) {
    const int i = e / T, j = e - i * T;
    mask[e] = (uint8_t)((sm.bits[i][j >> 5] >> (j & 31)) & 1u);
  }
}

// One compare-exchange of a bitonic network on keys in LDS: pair p of the stage with distance j
// inside sorted runs of length kk (descending overall).
__device__ __forceinline__ void bitonic_exchange(uint64_t* keys, int p, int j, int kk) {
  const int lo = ((p & ~(j - 1)) << 1) | (p & (j - 1)), hi = lo | j;
  const uint64_t x = keys[lo], y = keys[hi];
  const bool desc = (lo & kk) == 0;
  if ((x < y) == desc) {
    keys[lo] = y;
    keys[hi] = x;
  }
}

// Sorts keys[0 .. n2) (n2 a power of two >= 2) in descending order.  Every thread of the block
// calls it; nthr is a multiple of 64.  Pairs are dealt to the waves in blocks of 64 consecutive
// pairs; a stage with distance j <= 32 stays inside the 128 keys of such a block, so those stages
// need only the wave's own ordering, and only the stages with j >= 64 end in a block barrier.
__device__ __forceinline__ void bitonic_sort_desc(uint64_t* keys, int n2, int tid, int nthr) {
  const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
  const int npairs = n2 >> 1;
  for (int kk = 2; kk <= n2; kk <<= 1) {
    int j = kk >> 1;
    for (; j >= 64; j >>= 1) {
      for (int p = tid; p < npairs; p += nthr) bitonic_exchange(keys, p, j, kk);
      __syncthreads();
    }
    for (int pb = wave * 64; pb < npairs; pb += nwaves * 64) {
      const int p = pb + lane;
      for (int jj = j; jj >= 1; jj >>= 1) {
        if (p < npairs) bitonic_exchange(keys, p, jj, kk);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
    if (kk >= 64) __syncthreads();     // the next run length starts with a stage across blocks
  }
  if (n2 < 128) __syncthreads();
}

// Pools of at most DDD_POOL_MAX nodes: the rerank keys sit in LDS (they are distinct: the id is part
// of the key) and the m_eff largest are kept.
constexpr int kCountMax = 320;
// Must be called by every thread of the block.
// n_nodes: the sequence's pool size (st.n_nodes[b]) if the caller has it at hand, else -1.
__device__ __forceinline__ void tree_finalize_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int nmax,
                                                    int tid, int nthr, TreeSmem& sm, int n_nodes = -1) {
  if (n_nodes < 0) n_nodes = st.n_nodes[b];
  const int N = n_nodes - 1;
  const int m_eff = min(m, N);
  const float* psc = st.pool_score + (size_t)b * nmax;

  if (N <= kCountMax) {
    // Small pools: rank by counting (the number of larger keys is a node's position in the rerank
    // order); cheaper than the sort's chain of dependent stages up to a few hundred nodes.
    for (int i = tid; i < N; i += nthr) sm.keys[i] = rerank_key(psc[i + 1], i + 1);
    if (tid == 0) sm.keys[N] = 0ull;   // pad: the counting loop reads keys in pairs
    __syncthreads();
    for (int i = tid; i < N; i += nthr) {
      const uint64_t mine = sm.keys[i];
      int rank = 0;
      for (int j = 0; j < N; j += 2) {
        const uint64_t x = sm.keys[j], y = sm.keys[j + 1];
        rank += (x > mine ? 1 : 0) + (y > mine ? 1 : 0);
      }
      if (rank < m_eff) sm.e.pick[rank] = i + 1;
    }
  } else {
    int n2 = 2;
    while (n2 < N) n2 <<= 1;
    for (int i = tid; i < n2; i += nthr) sm.keys[i] = (i < N) ? rerank_key(psc[i + 1], i + 1) : 0ull;   // 0: below every key
    __syncthreads();
    bitonic_sort_desc(sm.keys, n2, tid, nthr);
    for (int i = tid; i < m_eff; i += nthr) sm.e.pick[i] = (int)(0xFFFFFFFFu - (uint32_t)sm.keys[i]);
  }
  __syncthreads();
  tree_emit_block(st, tree, b, m, m_eff, nmax, tid, nthr, sm.e);
}

}  // namespace ddd
