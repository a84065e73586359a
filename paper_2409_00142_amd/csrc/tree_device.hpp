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

// rank[i] = number of keys[0..n) larger than keys[i] (keys distinct, rank zeroed beforehand), by every thread of the block: with fewer keys than threads the comparisons of a key are shared
// by nthr / n threads.  No barrier inside.
__device__ __forceinline__ void count_larger_keys(const uint64_t* keys, int n, int* rank, int tid, int nthr) {
  if (n <= nthr) {                                               // uniform
    const int P = nthr / n, part = tid / n, i = tid - part * n;
    if (part < P) {
      const int chunk = ((n + P - 1) / P + 1) & ~1;              // even, so a pair never straddles two parts
      const int lo = part * chunk, hi = min(n, lo + chunk);
      const uint64_t mine = keys[i];
      int cnt = 0;
      for (int j = lo; j < hi; j += 2) {
        const uint64_t x = keys[j], y = (j + 1 < hi) ? keys[j + 1] : 0ull;
        cnt += (x > mine ? 1 : 0) + (y > mine ? 1 : 0);
      }
      if (cnt != 0) atomicAdd(&rank[i], cnt);
    }
  } else {
    for (int i = tid; i < n; i += nthr) {
      const uint64_t mine = keys[i];
      int cnt = 0;
      for (int j = 0; j < n; j += 2) {
        const uint64_t x = keys[j], y = (j + 1 < n) ? keys[j + 1] : 0ull;
        cnt += (x > mine ? 1 : 0) + (y > mine ? 1 : 0);
      }
      rank[i] = cnt;
    }
  }
}

// Pools of up to kSelMax nodes on a block with at least half as many threads: thread t looks after pool nodes
// t + 1 and t + 1 + nthr from their scores to their lines of the tree, so nothing is searched for and nothing is
// fetched twice.  One round trip brings a node's score, parent, token and depth.  Selection: the m-th best key
// among the first kSub nodes is a lower bound of the tree's keys (summed logprobs fall with depth, so the early
// nodes hold most of the tree and the bound is tight); the nodes at or above it - the candidates, usually little
// more than m - are ranked among themselves by counting (keys are distinct: the id is part of them), which costs
// kSub^2 + C^2 comparisons instead of N^2 or a sort's long chain of dependent stages (if more than kSelCand nodes
// pass the bound, the m-th best of kRefine of them is a tighter one: twice at most); up to kDirect nodes all are
// ranked at once, which saves the three barriers of the bound (7B shape, k = 10, microseconds inside the stopping
// call for 111 / 211 / 311 / 411 / 911 nodes: 3.6 / 5.7 / 6.3 / 6.7 / 9.5; ranking every node against all others
// took 3.5 / 5.2 / 7.8 / 15 / 34, the sort 16 at 911).  Still more than kSelCand candidates after two tightenings:
// the caller's general path takes over (returns false; nothing has been written to the tree).  The
// tree index of a selected node is 1 + the number of selected nodes with a smaller id (ballots and popcounts); a
// parent's tree index is read from the node -> index table (a selected node's parent is selected: its score is no
// smaller and its id is smaller).
constexpr int kSelMax = 2048, kSub = 128, kSelCand = 384, kDirect = 256, kRefine = 256;
static_assert(kRefine >= DDD_MMAX && kRefine <= kSelCand, "the refining sample holds m keys and lies in the candidate list");
static_assert(kDirect <= kSelCand, "the rank array holds every node of a directly ranked pool");
static_assert(kSub >= DDD_MMAX, "the subset must hold m keys");
__device__ __forceinline__ bool tree_select_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int nmax,
                                                  int tid, int nthr, TreeSmem& sm, int N) {
  const int m_eff = min(m, N), T = m + 1;
  // the upper half of the key array holds the working set of the selection
  int* tidx = reinterpret_cast<int*>(sm.keys + kSelMax + 2);     // [kSelMax + 1]  tree index of a pool node; -1: not in the tree
  uint64_t* ckey = reinterpret_cast<uint64_t*>(tidx + kSelMax + 2);   // [kSelCand] candidate keys
  int* cnode = reinterpret_cast<int*>(ckey + kSelCand);          // [kSelCand]     their pool ids
  int* rank = cnode + kSelCand;                                   // [kSelCand]     larger keys counted
  int* wtot = rank + kSelCand;                                    // [2][16]        selected nodes per wave and pass
  int* misc = wtot + 32;                                          // [0] candidates so far
  uint64_t* bound = reinterpret_cast<uint64_t*>(misc + 2);        // [1] the lower bound
  static_assert((kSelMax + 2) * 8 + (kSelMax + 2) * 4 + kSelCand * 16 + 34 * 4 + 8 <= (kPoolMax + 2) * 8, "working set");
  const int32_t* ppar = st.pool_parent + (size_t)b * nmax;
  const int32_t* pdep = st.pool_depth + (size_t)b * nmax;
  const int32_t* ptok = st.pool_token + (size_t)b * nmax;
  const float* psc = st.pool_score + (size_t)b * nmax;
  const int lane = tid & 63, wave = tid >> 6, nwaves = nthr >> 6;
  bool node[2];
  uint64_t my_key[2];
  int my_pn[2], my_tok[2], my_dep[2], root_tok = -1, root_dep = 0;
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int n = tid + q * nthr;                                 // pool node n + 1
    node[q] = n < N;
    my_key[q] = 0ull;
    my_pn[q] = 0;
    my_tok[q] = -1;
    my_dep[q] = 0;
    if (node[q]) {
      my_key[q] = rerank_key(psc[n + 1], n + 1);
      sm.keys[n] = my_key[q];
      tidx[n + 1] = -1;
      my_pn[q] = ppar[n + 1];
      my_tok[q] = ptok[n + 1];
      my_dep[q] = pdep[n + 1];
    }
  }
  const int S = min(N, kSub);
  if (tid < kSelCand) rank[tid] = 0;
  for (int i = tid + nthr; i < kSelCand; i += nthr) rank[i] = 0;
  if (tid == 0) {
    tidx[0] = 0;
    misc[0] = 0;
    sm.e.sel[0] = 0;
    sm.e.par[0] = -1;
    root_tok = ptok[0];
    root_dep = pdep[0];
  }
  __syncthreads();
  if (N <= kDirect) {                                             // uniform: few enough nodes to rank them all
    count_larger_keys(sm.keys, N, rank, tid, nthr);
    __syncthreads();
    for (int i = tid; i < N; i += nthr)
      if (rank[i] < m_eff) tidx[i + 1] = -2;                      // in the tree; its index follows
    __syncthreads();
  } else {
    // the bound: first from the early nodes, then - while more than kSelCand nodes pass it (a confident sequence: its
    // deep nodes score as well as the early ones) - from the first kRefine candidates, which lie above the old bound
    const uint64_t* sample = sm.keys;
    int n_sample = S, C = 0;
    for (int attempt = 0;; ++attempt) {
      count_larger_keys(sample, n_sample, rank, tid, nthr);
      __syncthreads();
      for (int i = tid; i < n_sample; i += nthr)
        if (rank[i] == min(m_eff, n_sample) - 1) bound[0] = sample[i];   // exactly one key has this rank
      if (tid == 0) misc[0] = 0;
      __syncthreads();
      const uint64_t lowest = bound[0];
      __syncthreads();                                              // everybody has the bound and is done with the ranks and the sample
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const bool cand = node[q] && my_key[q] >= lowest;
        const unsigned long long bal = __ballot(cand);
        int base = 0;
        if (lane == 0 && bal != 0ull) base = atomicAdd(&misc[0], __popcll(bal));
        base = __shfl(base, 0, 64);
        const int pos = base + __popcll(bal & ((1ull << lane) - 1ull));
        if (cand && pos < kSelCand) {
          ckey[pos] = my_key[q];
          cnode[pos] = tid + q * nthr + 1;
        }
      }
      if (tid < kSelCand) rank[tid] = 0;
      for (int i = tid + nthr; i < kSelCand; i += nthr) rank[i] = 0;
      __syncthreads();
      C = misc[0];
      if (C <= kSelCand) break;                                     // uniform
      if (attempt == 2) return false;                               // uniform: the general path
      sample = ckey;
      n_sample = kRefine;
    }
    count_larger_keys(ckey, C, rank, tid, nthr);
    __syncthreads();
    for (int c = tid; c < C; c += nthr)
      if (rank[c] < m_eff) tidx[cnode[c]] = -2;                     // in the tree; its index follows
    __syncthreads();
  }
  bool chosen[2];
  unsigned long long bal[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    chosen[q] = node[q] && tidx[tid + q * nthr + 1] == -2;
    bal[q] = __ballot(chosen[q]);
    if (lane == 0) wtot[q * 16 + wave] = __popcll(bal[q]);
  }
  __syncthreads();
  int ti[2] = {-1, -1};
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (chosen[q]) {
      int t = 1 + __popcll(bal[q] & ((1ull << lane) - 1ull));
      for (int w = 0; w < wave; ++w) t += wtot[q * 16 + w];
      if (q == 1)
        for (int w = 0; w < nwaves; ++w) t += wtot[w];
      ti[q] = t;
      sm.e.sel[t] = tid + q * nthr + 1;
      tidx[tid + q * nthr + 1] = t;
    }
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (chosen[q]) sm.e.par[ti[q]] = tidx[my_pn[q]];
  __syncthreads();
  for (int i = tid; i < T; i += nthr) {
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) sm.e.bits[i][w] = 0u;
    if (i <= m_eff) {
      int c = i;
      while (c >= 0) {
        sm.e.bits[i][c >> 5] |= (1u << (c & 31));
        c = sm.e.par[c];
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    tree.n_sel[b] = m_eff;
    tree.tree_token[(size_t)b * T] = root_tok;
    tree.pos[(size_t)b * T] = root_dep;
    tree.parent_idx[(size_t)b * T] = -1;
  }
  for (int i = tid; i < m; i += nthr) tree.sel_node[(size_t)b * m + i] = (i < m_eff) ? sm.e.sel[1 + i] : -1;
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (chosen[q]) {
      tree.tree_token[(size_t)b * T + ti[q]] = my_tok[q];
      tree.pos[(size_t)b * T + ti[q]] = my_dep[q];
      tree.parent_idx[(size_t)b * T + ti[q]] = sm.e.par[ti[q]];
    }
  for (int i = m_eff + 1 + tid; i < T; i += nthr) {     // padding
    tree.tree_token[(size_t)b * T + i] = -1;
    tree.pos[(size_t)b * T + i] = 0;
    tree.parent_idx[(size_t)b * T + i] = -1;
  }
  uint8_t* mask = tree.mask + (size_t)b * T * T;
  for (int e = tid; e < T * T; e += nthr) {
    const int i = e / T, j = e - i * T;
    mask[e] = (uint8_t)((sm.e.bits[i][j >> 5] >> (j & 31)) & 1u);
  }
  return true;
}

// Pools of at most DDD_POOL_MAX nodes: the rerank keys sit in LDS (they are distinct: the id is part
// of the key) and the m_eff largest are kept.
// Must be called by every thread of the block.
// n_nodes: the sequence's pool size (st.n_nodes[b]) if the caller has it at hand, else -1.
__device__ __forceinline__ void tree_finalize_block(const ddd_state& st, const ddd_tree& tree, int b, int m, int nmax,
                                                    int tid, int nthr, TreeSmem& sm, int n_nodes = -1) {
  if (n_nodes < 0) n_nodes = st.n_nodes[b];
  const int N = n_nodes - 1;
  const int m_eff = min(m, N);
  const float* psc = st.pool_score + (size_t)b * nmax;

  if (N >= 1 && N <= kSelMax && N <= 2 * nthr && nthr <= 1024) {   // uniform
    if (tree_select_block(st, tree, b, m, nmax, tid, nthr, sm, N)) return;
    __syncthreads();                                              // the general path reuses the key array
  }
  if (N <= 320) {
    // Small pools on a block much narrower than the pool: rank by counting (the number of larger keys is a node's
    // position in the rerank order); cheaper than the sort's chain of dependent stages up to a few hundred nodes.
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
