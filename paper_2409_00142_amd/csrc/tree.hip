// Final draft tree (top-m rerank, order, parents, positions, attention mask) and the greedy
// accept walk.  One workgroup per sequence; everything is integer work on at most
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
