// Final draft tree of one sequence, built by one workgroup (device function shared by the
// stand-alone finalize kernel and the per-call bookkeeping kernel).
#pragma once
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"

namespace ddd {

constexpr int kPoolMax = DDD_POOL_MAX;
constexpr int kTreeMax = DDD_MMAX + 1;
constexpr int kMaskWords = (kTreeMax + 31) / 32;

struct TreeSmem {
  uint64_t keys[kPoolMax];
  int sel[kTreeMax];                    // pool ids of tree indices 0..n_sel (0 = root)
  int par[kTreeMax];                    // tree index of the parent
  uint32_t bits[kTreeMax][kMaskWords];  // ancestor bit rows
};

// Section 1: the m best nodes of the draft tree by summed logprob go to the target model in
// one pass; a node may attend to itself and its ancestors only.  Rerank key: (score desc,
// node id asc); tree order: ascending node id.  Must be called by every thread of the block.
__device__ __forceinline__ void tree_finalize_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int nmax,
                                                    int tid, int nthr, TreeSmem& sm) {
  const int n_nodes = st.n_nodes[b];
  const int N = n_nodes - 1;
  const int m_eff = min(m, N), T = m + 1;
  const float* psc = st.pool_score + (size_t)b * nmax;
  const int32_t* ppar = st.pool_parent + (size_t)b * nmax;
  const int32_t* pdep = st.pool_depth + (size_t)b * nmax;
  const int32_t* ptok = st.pool_token + (size_t)b * nmax;

  int N2 = 64;
  while (N2 < N) N2 <<= 1;
  for (int i = tid; i < N2; i += nthr)
    sm.keys[i] =
        (i < N) ? (((uint64_t)ord32(psc[i + 1]) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)(i + 1))) : 0ull;
  __syncthreads();
  // bitonic sort, descending
  for (int size = 2; size <= N2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int p = tid; p < (N2 >> 1); p += nthr) {
        const int pos = 2 * stride * (p / stride) + (p % stride);
        const int partner = pos + stride;
        const bool desc = ((pos & size) == 0);
        const uint64_t x = sm.keys[pos], y = sm.keys[partner];
        if ((x < y) == desc) {
          sm.keys[pos] = y;
          sm.keys[partner] = x;
        }
      }
      __syncthreads();
    }
  }
  // chosen ids in ascending order: rank by counting
  if (tid == 0) sm.sel[0] = 0;
  for (int i = tid; i < m_eff; i += nthr) {
    const uint32_t id = 0xFFFFFFFFu - (uint32_t)sm.keys[i];
    int rank = 0;
    for (int j = 0; j < m_eff; ++j) rank += ((0xFFFFFFFFu - (uint32_t)sm.keys[j]) < id) ? 1 : 0;
    sm.sel[1 + rank] = (int)id;
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

}  // namespace ddd
