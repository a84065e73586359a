// Synthetic stand-ins for the draft-model body and the target model (workload generators for
// tests and the benchmark; not part of the method), plus a plain read-stream kernel used as
// the practical HBM ceiling.  The hidden-state recipe is the documented counter-based one:
// SplitMix64-finaliser keys, four 16-bit fields summed per element, one fp32 multiply, an
// optional planted direction, RNE to bf16.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ddd_synth.h"

namespace {

constexpr uint64_t kGold = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kSeq = 0xD1B54A32D192ED03ull;
constexpr uint64_t kRoundPlant = 0xA5A5A5A5A5A5A5A5ull;
constexpr uint64_t kRowPlant = 0x5A5A5A5A5A5A5A5Aull;
constexpr uint64_t kTarget = 0x7A67E7ull;
constexpr uint32_t kRootParent = 0xFFFFFFFFu;
constexpr uint32_t kU24_070 = 11744051u;   // floor(0.70 * 2^24)
constexpr uint32_t kU24_085 = 14260633u;   // floor(0.85 * 2^24)

__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__device__ inline uint64_t stream_key(uint64_t seed, int b, int64_t rnd) {
  const uint64_t a = mix64(seed * kGold + (uint64_t)rnd + 1ull);
  return mix64(a ^ ((uint64_t)(b + 1) * kSeq));
}
__device__ inline uint64_t node_key(uint64_t skey, uint32_t parent, uint32_t token) {
  return mix64(skey ^ mix64(((uint64_t)parent << 32) | (uint64_t)token));
}
__device__ inline uint16_t f32_to_bf16_rne(float x) {
  const uint32_t u = __float_as_uint(x);
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

struct BodyArgs {
  ddd_synth_params p;
  ddd_state st;
  uint16_t* hid;
  int step;
};

// grid: (rows, parts of a row); block 256: a thread makes pairs of neighbouring elements (one 4-byte store each).
// With hundreds of rows a row is one workgroup: the chain of dependent loads that identifies the row's node (flag,
// beam entry, its parent) is walked once per row; a few rows are cut into parts so that the chip is still used.
__device__ inline float synth_element(uint64_t nk, int e, float scale) {
  const uint64_t z = mix64(nk + (uint64_t)(e + 1) * kGold);
  const int s = (int)((z & 0xFFFFu) + ((z >> 16) & 0xFFFFu) + ((z >> 32) & 0xFFFFu) + (z >> 48)) - 131070;
  return __fmul_rn((float)s, scale);
}

__global__ __launch_bounds__(256) void synth_body_kernel(BodyArgs a) {
  const int k = a.p.cfg.k, H = a.p.cfg.H;
  const int row = blockIdx.x;
  const int b = (a.step == 0) ? row : row / k;
  if (!a.st.active[b]) return;
  const uint64_t skey = stream_key(a.p.seed, b, *a.p.round_ctr);
  uint32_t parent, token;
  if (a.step == 0) {
    parent = kRootParent;
    token = (uint32_t)a.p.root_token;
  } else {
    const int i = row - b * k;
    const int node = a.st.beam_node[(size_t)b * k + i];
    const size_t nmax = 1 + (size_t)k + (size_t)(a.p.cfg.max_depth - 1) * k * k;
    parent = (uint32_t)a.st.pool_parent[(size_t)b * nmax + node];
    token = (uint32_t)a.st.beam_token[(size_t)b * k + i];
  }
  const uint64_t nk = node_key(skey, parent, token);
  int pi = -1;
  if (a.p.n_plant > 0) {
    const uint64_t ur = mix64(skey ^ kRoundPlant);
    if ((uint32_t)(ur >> 40) < a.p.plant_round_p24) {
      pi = (int)((ur & 0xFFFFu) % (uint32_t)a.p.n_plant);
    } else {
      const uint64_t un = mix64(nk ^ kRowPlant);
      if ((uint32_t)(un >> 40) < a.p.plant_row_p24) pi = (int)((un & 0xFFFFu) % (uint32_t)a.p.n_plant);
    }
  }
  const float scale = a.p.scale_depth[a.step];
  uint32_t* out = reinterpret_cast<uint32_t*>(a.hid + (size_t)row * H);   // H is even (a multiple of 128)
  for (int e = 512 * blockIdx.y + 2 * threadIdx.x; e < H; e += 512 * gridDim.y) {
    float v0 = synth_element(nk, e, scale), v1 = synth_element(nk, e + 1, scale);
    if (pi >= 0) {
      v0 = __fadd_rn(v0, a.p.plant_dir[(size_t)pi * H + e]);
      v1 = __fadd_rn(v1, a.p.plant_dir[(size_t)pi * H + e + 1]);
    }
    out[e >> 1] = (uint32_t)f32_to_bf16_rne(v0) | ((uint32_t)f32_to_bf16_rne(v1) << 16);
  }
}

struct TargetArgs {
  ddd_synth_params p;
  ddd_state st;
  ddd_tree tree;
  int32_t* out;
};

// grid: B; block 256.  The rank-0 / rank-1 children (the two lowest-id children) of every tree
// node are found by one pass over the pool: a node of sibling rank 0 or 1 looks its parent up in
// the sorted list of selected ids.  Then thread i handles tree index i.
__global__ __launch_bounds__(256) void synth_target_kernel(TargetArgs a) {
  __shared__ int sel[DDD_MMAX + 1], kid0[DDD_MMAX + 1], kid1[DDD_MMAX + 1];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int k = a.p.cfg.k, m = a.p.cfg.m, T = m + 1;
  const size_t nmax = 1 + (size_t)k + (size_t)(a.p.cfg.max_depth - 1) * k * k;
  const int32_t* ppar = a.st.pool_parent + (size_t)b * nmax;
  const int32_t* ptok = a.st.pool_token + (size_t)b * nmax;
  const int n_nodes = min(a.st.n_nodes[b], (int)nmax);
  const int n_sel = min(a.tree.n_sel[b], m);
  for (int i = tid; i <= n_sel; i += 256) {
    sel[i] = (i == 0) ? 0 : a.tree.sel_node[(size_t)b * m + i - 1];   // ascending ids
    kid0[i] = -1;
    kid1[i] = -1;
  }
  __syncthreads();
  // nodes of sibling rank 0 and 1 have ids 1, 2 (prompt call) and base_s + i*k + {0, 1} (later calls)
  const int kk = k * k;
  const int calls = (n_nodes - 1 - k) / kk;                  // later calls that have been made
  const int n_items = 2 + calls * k * 2;
  for (int it = tid; it < n_items; it += 256) {
    int c, j;
    if (it < 2) {
      c = 1 + it;
      j = it;
    } else {
      const int q = it - 2;
      j = q & 1;
      const int si = q >> 1;                                 // call index * k + beam slot
      c = 1 + k + si * k + j;
    }
    if (c >= n_nodes || (j == 1 && k < 2)) continue;
    const int p = ppar[c];
    int lo = 0, hi = n_sel;                                  // binary search of p in sel[0..n_sel]
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (sel[mid] < p)
        lo = mid + 1;
      else
        hi = mid;
    }
    if (sel[lo] == p) {
      if (j == 0) kid0[lo] = c;
      else kid1[lo] = c;
    }
  }
  __syncthreads();
  const int i = tid;
  if (i >= T) return;
  if (i > n_sel) {
    a.out[(size_t)b * T + i] = -1;
    return;
  }
  const int node = sel[i];
  const uint64_t skey = stream_key(a.p.seed, b, *a.p.round_ctr);
  const uint64_t tk = mix64(skey ^ mix64(kTarget + (uint64_t)node));
  const uint32_t u = (uint32_t)(tk >> 40);
  const int uni = (int)((tk & 0xFFFFFFFFull) % (uint64_t)a.p.cfg.V);
  int out = uni;
  if (u < kU24_070 && kid0[i] >= 0)
    out = ptok[kid0[i]];
  else if (u >= kU24_070 && u < kU24_085 && kid1[i] >= 0)
    out = ptok[kid1[i]];
  a.out[(size_t)b * T + i] = out;
}

__global__ void next_round_kernel(int64_t* ctr) { *ctr += 1; }

__global__ void round_stats_kernel(int64_t* ctr, const int32_t* steps, const int32_t* accept_len, int B,
                                   int64_t* depth_hist, int64_t* accept_hist, int64_t* batch_depth_hist) {
  // one workgroup; integer atomics, so the totals do not depend on the order
  __shared__ int s_max;
  if (threadIdx.x == 0) s_max = 0;
  __syncthreads();
  for (int b = threadIdx.x; b < B; b += blockDim.x) {
    if (steps != nullptr) atomicMax(&s_max, min(max(steps[b], 0), 31));
    if (depth_hist != nullptr && steps != nullptr)
      atomicAdd(reinterpret_cast<unsigned long long*>(depth_hist + min(max(steps[b], 0), 31)), 1ull);
    if (accept_hist != nullptr && accept_len != nullptr)
      atomicAdd(reinterpret_cast<unsigned long long*>(accept_hist + min(max(accept_len[b], 0), 31)), 1ull);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (batch_depth_hist != nullptr) batch_depth_hist[s_max] += 1;   // LM-head passes this round needed
    *ctr += 1;
  }
}

// Each thread reads 16-byte words with a grid stride and folds them into one word.
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9E3779B9u) *sink = acc;   // practically never: keeps the loads alive without a store
}

// Register-resident MFMA loop with pseudo-random bf16 operands: the matrix-core rate this chip
// sustains on data that toggles like real data (the clock drops under it), with no memory traffic.
typedef __attribute__((ext_vector_type(8))) __bf16 mr_bf16x8;
typedef __attribute__((ext_vector_type(16))) float mr_f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int mr_u32x4;
__device__ __forceinline__ unsigned mr_mix(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
__device__ __forceinline__ unsigned mr_pair(unsigned h) { return (h & 0x807f807fu) | 0x3f003f00u; }   // |x| in [0.5, 1)
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* sink, int iters, unsigned seed) {
  constexpr int NACC = 8;
  mr_bf16x8 a[NACC], b[NACC];
#pragma unroll
  for (int j = 0; j < NACC; ++j) {
    const unsigned h = mr_mix(seed + threadIdx.x * 131u + j * 977u + blockIdx.x * 7919u);
    const mr_u32x4 ua = {mr_pair(h), mr_pair(mr_mix(h + 1)), mr_pair(mr_mix(h + 2)), mr_pair(mr_mix(h + 3))};
    const mr_u32x4 ub = {mr_pair(mr_mix(h + 4)), mr_pair(mr_mix(h + 5)), mr_pair(mr_mix(h + 6)), mr_pair(mr_mix(h + 7))};
    a[j] = __builtin_bit_cast(mr_bf16x8, ua);
    b[j] = __builtin_bit_cast(mr_bf16x8, ub);
  }
  mr_f32x16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[(i * 3 + 1) % NACC], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  if (s == 1.2345f) sink[0] = s;   // practically never: keeps the loop alive without a store
}

// tokens[i] = hash(seed, round, i) mod V: a different last prompt token per sequence and round
__global__ void hash_tokens_kernel(const int64_t* round_ctr, int32_t* tokens, int V, uint64_t seed) {
  const uint64_t z = mix64(mix64(seed ^ (uint64_t)*round_ctr) + (uint64_t)threadIdx.x + 1ull);
  tokens[threadIdx.x] = (int32_t)(z % (uint64_t)V);
}

}  // namespace

extern "C" {

int ddd_synth_draft_body(void* user, int32_t step, const ddd_state* st, void* hid_out_bf16, void* stream) {
  const ddd_synth_params* p = static_cast<const ddd_synth_params*>(user);
  if (p == nullptr || st == nullptr || hid_out_bf16 == nullptr || p->round_ctr == nullptr) return DDD_ERR_INVALID_ARG;
  if (step < 0 || step >= p->cfg.max_depth || step >= 32) return DDD_ERR_INVALID_ARG;
  if (p->n_plant > 0 && p->plant_dir == nullptr) return DDD_ERR_INVALID_ARG;
  BodyArgs a;
  a.p = *p;
  a.st = *st;
  a.hid = static_cast<uint16_t*>(hid_out_bf16);
  a.step = step;
  const int rows = (step == 0) ? p->cfg.B : p->cfg.B * p->cfg.k;
  if (p->cfg.H % 2 != 0) return DDD_ERR_INVALID_ARG;
  int parts = 512 / rows;                                   // about 512 workgroups
  const int max_parts = (p->cfg.H + 511) / 512;
  parts = parts < 1 ? 1 : (parts > max_parts ? max_parts : parts);
  hipLaunchKernelGGL(synth_body_kernel, dim3(rows, parts), dim3(256), 0, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

int ddd_synth_target_argmax(const ddd_synth_params* p, const ddd_state* st, const ddd_tree* tree,
                            int32_t* target_argmax, void* stream) {
  if (p == nullptr || st == nullptr || tree == nullptr || target_argmax == nullptr || p->round_ctr == nullptr)
    return DDD_ERR_INVALID_ARG;
  if (p->cfg.m + 1 > 256) return DDD_ERR_INVALID_ARG;
  TargetArgs a;
  a.p = *p;
  a.st = *st;
  a.tree = *tree;
  a.out = target_argmax;
  hipLaunchKernelGGL(synth_target_kernel, dim3(p->cfg.B), dim3(256), 0, static_cast<hipStream_t>(stream), a);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

int ddd_synth_next_round(int64_t* round_ctr, void* stream) {
  if (round_ctr == nullptr) return DDD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(next_round_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), round_ctr);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

int ddd_synth_hash_tokens(const int64_t* round_ctr, int32_t* tokens, int32_t n, int32_t V, uint64_t seed, void* stream) {
  if (round_ctr == nullptr || tokens == nullptr || n < 1 || n > 1024 || V < 1) return DDD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(hash_tokens_kernel, dim3(1), dim3(n), 0, static_cast<hipStream_t>(stream), round_ctr, tokens, V,
                     seed);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

int ddd_synth_round_stats(int64_t* round_ctr, const int32_t* steps, const int32_t* accept_len, int32_t B,
                          int64_t* depth_hist, int64_t* accept_hist, int64_t* batch_depth_hist, void* stream) {
  if (round_ctr == nullptr || B < 1) return DDD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(round_stats_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), round_ctr, steps,
                     accept_len, B, depth_hist, accept_hist, batch_depth_hist);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

int ddd_synth_post(void* user, const ddd_state* st, const ddd_tree* tree, void* stream) {
  const ddd_synth_post_args* a = static_cast<const ddd_synth_post_args*>(user);
  if (a == nullptr || a->params == nullptr || a->ctx == nullptr || st == nullptr || tree == nullptr)
    return DDD_ERR_INVALID_ARG;
  int rc = ddd_synth_target_argmax(a->params, st, tree, a->target_argmax, stream);
  if (rc != DDD_OK) return rc;
  rc = ddd_verify_accept(a->ctx, tree, a->target_argmax, a->accept_len, a->accept_path, a->bonus_token, stream);
  if (rc != DDD_OK) return rc;
  if (a->depth_hist != nullptr || a->accept_hist != nullptr || a->batch_depth_hist != nullptr) {
    int64_t* ctr = const_cast<int64_t*>(a->params->round_ctr);   // the round's own counter: the statistics step advances it
    rc = ddd_synth_round_stats(ctr, st->steps, a->accept_len, a->params->cfg.B, a->depth_hist,
                               a->accept_hist, a->batch_depth_hist, stream);
    if (rc != DDD_OK) return rc;
  }
  if (a->hash_tokens != nullptr)
    rc = ddd_synth_hash_tokens(a->params->round_ctr, a->hash_tokens, a->params->cfg.B, a->params->cfg.V,
                               a->params->seed, stream);
  return rc;
}

int ddd_synth_read_stream(const void* src, size_t n_bytes, uint32_t* sink, int32_t n_blocks, void* stream) {
  if (src == nullptr || sink == nullptr || n_bytes % 16 != 0 || n_blocks < 1) return DDD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(read_stream_kernel, dim3(n_blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), n_bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

int ddd_synth_mfma_rate(float* sink, int32_t iters, int32_t n_blocks, void* stream) {
  if (sink == nullptr || iters < 1 || iters > (1 << 20) || n_blocks < 1 || n_blocks > 65536) return DDD_ERR_INVALID_ARG;
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(n_blocks), dim3(256), 0, static_cast<hipStream_t>(stream), sink, iters, 7u);
  return hipGetLastError() == hipSuccess ? DDD_OK : DDD_ERR_HIP;
}

}  // extern "C"
