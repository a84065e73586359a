// Final draft tree (top-m rerank, order, parents, positions, attention mask) and the greedy
// accept walk.  One workgroup per sequence; everything is integer work on at most
// DDD_POOL_MAX nodes, so it lives in LDS.
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"

namespace ddd {

constexpr int kPoolMax = DDD_POOL_MAX;
constexpr int kTreeMax = DDD_MMAX + 1;
constexpr int kMaskWords = (kTreeMax + 31) / 32;

// Section 1: the m best nodes of the draft tree by summed logprob go to the target model in
// one pass; a node may attend to itself and its ancestors only.
__global__ __launch_bounds__(1024) void tree_finalize_kernel(FinalizeArgs a) {
  __shared__ uint64_t keys[kPoolMax];
  __shared__ int s_sel[kTreeMax];               // pool ids of tree indices 0..n_sel (0 = root)
  __shared__ int s_par[kTreeMax];               // tree index of the parent
  __shared__ uint32_t s_bits[kTreeMax][kMaskWords];
  const int b = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  const int n_nodes = a.st.n_nodes[b];
  const int N = n_nodes - 1;
  const int m = a.m, m_eff = min(m, N), T = m + 1;
  const float* psc = a.st.pool_score + (size_t)b * a.nmax;
  const int32_t* ppar = a.st.pool_parent + (size_t)b * a.nmax;
  const int32_t* pdep = a.st.pool_depth + (size_t)b * a.nmax;
  const int32_t* ptok = a.st.pool_token + (size_t)b * a.nmax;

  int N2 = 64;
  while (N2 < N) N2 <<= 1;
  // key: larger score first, then lower node id
  for (int i = tid; i < N2; i += nthr)
    keys[i] = (i < N) ? (((uint64_t)ord32(psc[i + 1]) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)(i + 1))) : 0ull;
  __syncthreads();
  // bitonic sort, descending
  for (int size = 2; size <= N2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int p = tid; p < (N2 >> 1); p += nthr) {
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
  // chosen ids in ascending order: rank by counting
  if (tid == 0) s_sel[0] = 0;
  if (tid < m_eff) {
    const uint32_t id = 0xFFFFFFFFu - (uint32_t)keys[tid];
    int rank = 0;
    for (int j = 0; j < m_eff; ++j) rank += ((0xFFFFFFFFu - (uint32_t)keys[j]) < id) ? 1 : 0;
    s_sel[1 + rank] = (int)id;
  }
  __syncthreads();
  // parents as tree indices
  if (tid <= m_eff) {
    int par = -1;
    if (tid > 0) {
      const int pn = ppar[s_sel[tid]];
      for (int j = 0; j < tid; ++j)
        if (s_sel[j] == pn) par = j;
    }
    s_par[tid] = par;
  }
  __syncthreads();
  // ancestor bit rows
  if (tid < T) {
#pragma unroll
    for (int w = 0; w < kMaskWords; ++w) s_bits[tid][w] = 0u;
    if (tid <= m_eff) {
      int c = tid;
      while (c >= 0) {
        s_bits[tid][c >> 5] |= (1u << (c & 31));
        c = s_par[c];
      }
    }
  }
  __syncthreads();
  // outputs
  if (tid == 0) a.tree.n_sel[b] = m_eff;
  if (tid < m) a.tree.sel_node[(size_t)b * m + tid] = (tid < m_eff) ? s_sel[1 + tid] : -1;
  if (tid < T) {
    const bool ok = (tid <= m_eff);
    const int node = ok ? s_sel[tid] : 0;
    a.tree.tree_token[(size_t)b * T + tid] = ok ? ptok[node] : -1;
    a.tree.pos[(size_t)b * T + tid] = ok ? pdep[node] : 0;
    a.tree.parent_idx[(size_t)b * T + tid] = ok ? s_par[tid] : -1;
  }
  uint8_t* mask = a.tree.mask + (size_t)b * T * T;
  for (int e = tid; e < T * T; e += nthr) {
    const int i = e / T, j = e - i * T;
    mask[e] = (uint8_t)((s_bits[i][j >> 5] >> (j & 31)) & 1u);
  }
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

}  // namespace ddd
