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
  // parents as tree indices (a parent has a smaller id, hence a smaller tree index)
  for (int i = tid; i <= m_eff; i += nthr) {
    int par = -1;
    if (i > 0) {
      const int pn = ppar[sm.sel[i]];
      for (int j = 0; j < i; ++j)
        if (sm.sel[j] == pn) par = j;
    }
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
  for (int i = tid; i < T; i += nthr) {
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

// Pools of at most DDD_POOL_MAX nodes: the keys sit in LDS and every node is ranked by counting.
// Must be called by every thread of the block.
__device__ __forceinline__ void tree_finalize_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int nmax,
                                                    int tid, int nthr, TreeSmem& sm) {
  const int n_nodes = st.n_nodes[b];
  const int N = n_nodes - 1;
  const int m_eff = min(m, N);
  const float* psc = st.pool_score + (size_t)b * nmax;

  for (int i = tid; i < N; i += nthr) sm.keys[i] = rerank_key(psc[i + 1], i + 1);
  if (tid == 0) sm.keys[N] = 0ull;   // pad: the counting loop below reads keys in pairs
  __syncthreads();
  // Rank by counting: keys are distinct (the id is part of the key), so the number of larger keys
  // is the node's position in the rerank order; the m_eff best are kept.
  for (int i = tid; i < N; i += nthr) {
    const uint64_t mine = sm.keys[i];
    int rank = 0;
    for (int j = 0; j < N; j += 2) {
      const uint64_t x = sm.keys[j], y = sm.keys[j + 1];
      rank += (x > mine ? 1 : 0) + (y > mine ? 1 : 0);
    }
    if (rank < m_eff) sm.e.pick[rank] = i + 1;
  }
  __syncthreads();
  tree_emit_block(st, tree, b, m, m_eff, nmax, tid, nthr, sm.e);
}

}  // namespace ddd
