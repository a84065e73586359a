// Tree attention of the verification pass: the consumer of the final tree's mask (Section 1, EAGLE
// paragraph: the whole draft tree goes through the target model in one pass, every node seeing
// the prompt, its ancestors and itself).
//
//   out[i] = sum_j softmax_j(q_i . k_j / sqrt(128)) v_j   over the L prompt keys and the tree keys
//                                                         j with mask[i][j] = 1, per sequence and head
//
// The prompt's keys and values are read once (HBM-bound: 2 * L * 256 bytes per head), so the
// kernel is a split-key ("flash decoding") pass: workgroup = 4 waves, every wave takes chunks of
// 32 keys for a tile of 64 queries and keeps a running max / sum / output per query.
// Both products run on v_mfma_f32_32x32x16_bf16 in transposed form, which puts one query in one
// lane, so the softmax rescaling is a per-lane scalar:
//   S^T[key][query]  = K[key][d]   Q^T[d][query]     (A = 32 keys x 16 d from the key cache as stored)
//   O^T[d][query]   += V^T[d][key] P^T[key][query]   (A = 32 d x 16 keys from the transposed value cache)
// The accumulator of the first product holds, per lane, keys g*8 + 4*lh + 0..3 (g = 0..3), which is
// not the 8 consecutive keys a B operand wants; the second product simply contracts over the keys
// in that order, by loading V^T as two 4-key pieces per operand.
// The four waves of a workgroup merge through LDS into one partial per workgroup; a second kernel
// merges the workgroups' partials.
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"

namespace ddd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int kAD = 128;        // head dimension
constexpr int kQT = 64;         // queries per tile
constexpr int kPartFloats = kAD * kQT + 2 * kQT;   // one partial: O^T[128][64], m[64], l[64]
constexpr int kLdsPitch = kQT + 1;                 // a wave's O^T in LDS: rows padded, so that reads along d are conflict-free too
constexpr int kLdsPart = kAD * kLdsPitch + 2 * kQT + 2 * kQT;   // ... + m[64], l[64], weight[64], spare
constexpr float kLazy = 11.0f;  // how far (in powers of two) a score may exceed a query's softmax reference before it moves

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {   // round to nearest even (one v_cvt_pk_bf16_f32)
  const f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// Operands of one chunk of 32 keys for one wave.
struct KeyOperands {
  bf16x8 kf[8];      // keys as A operands: lane (l32, lh) holds d = s*16 + lh*8 .. +7 of key c0 + l32
};
struct ValueOperands {
  bf16x8 vf[4][2];   // transposed values as A operands: lane (l32, lh) holds, for d = db*32 + l32 and 16-key step t,
                     // the keys c0 + 16t + 4*lh + 0..3 and c0 + 16t + 8 + 4*lh + 0..3 (the order the first product
                     // leaves them in)
};

// Prompt chunks come from the packed cache (fragment order: every operand of a wave is 1 KB of consecutive
// memory, 16 bytes per lane); the two tree chunks from the tree's own small arrays.
__device__ __forceinline__ void load_keys(const TreeAttnArgs& a, int c, int ncp, int b, int h, int lane,
                                          KeyOperands& x) {
  const int l32 = lane & 31, lh = lane >> 5;
  if (c < ncp) {
    const u32x4* kp = reinterpret_cast<const u32x4*>(a.k_prompt) + ((((size_t)b * a.nh + h) * ncp + c) * 8) * 64 + lane;
#pragma unroll
    for (int s = 0; s < 8; ++s) x.kf[s] = __builtin_bit_cast(bf16x8, kp[s * 64]);
  } else {
    const int kj = min((c - ncp) * 32 + l32, a.T - 1);
    const uint16_t* kp = a.k_tree + (((size_t)b * a.T + kj) * a.nh + h) * kAD + lh * 8;
#pragma unroll
    for (int s = 0; s < 8; ++s) x.kf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kp + s * 16));
  }
}

__device__ __forceinline__ void load_values(const TreeAttnArgs& a, int c, int ncp, int b, int h, int lane,
                                            ValueOperands& x) {
  const int l32 = lane & 31, lh = lane >> 5;
  if (c < ncp) {
    const u32x4* vp = reinterpret_cast<const u32x4*>(a.v_prompt) + ((((size_t)b * a.nh + h) * ncp + c) * 8) * 64 + lane;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int t = 0; t < 2; ++t) x.vf[db][t] = __builtin_bit_cast(bf16x8, vp[(db * 2 + t) * 64]);
  } else {
    const uint16_t* vp = a.vt_tree + (((size_t)b * a.nh + h) * kAD + l32) * a.Tp + (c - ncp) * 32 + lh * 4;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x2 lo = *reinterpret_cast<const u32x2*>(vp + (size_t)db * 32 * a.Tp + t * 16);
        const u32x2 hi = *reinterpret_cast<const u32x2*>(vp + (size_t)db * 32 * a.Tp + t * 16 + 8);
        const u32x4 u = {lo[0], lo[1], hi[0], hi[1]};
        x.vf[db][t] = __builtin_bit_cast(bf16x8, u);
      }
  }
}

// Running softmax state of the wave's 64 queries (one per lane and query block) and their outputs.
struct QueryState {
  f32x16 o[4][2];
  float m[2], l[2];
};

__device__ __forceinline__ void attend_chunk(const TreeAttnArgs& a, const KeyOperands& x, const ValueOperands& xv,
                                             const bf16x8 (&qf)[2][8], int c,
                                             int ncp, int b, int qt, int lane, QueryState& st) {
  const int l32 = lane & 31, lh = lane >> 5;
  const bool tree = c >= ncp;
  const int c0 = (tree ? c - ncp : c) * 32;
  const int nkeys = tree ? a.T : a.L;
  // scores are kept in units of ln 2: exp(s - m) = exp2(s' - m') with s' = s * log2(e) / sqrt(128)
  const float scale = 0.08838834764831845f * 1.4426950408889634f;
  const bool ragged = tree || c0 + 32 > nkeys;          // uniform: only such chunks have keys to hide
  bf16x8 pf[2][2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    f32x16 sacc;
#pragma unroll
    for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.kf[s], qf[qb][s], sacc, 0, 0, 0);
    // register e of the lane: key c0 + (e>>2)*8 + lh*4 + (e&3), query qb*32 + l32
    float sv[16];
    float cmax = -INFINITY;
    if (ragged) {
      const int qi = qt * kQT + qb * 32 + l32;
      const uint8_t* mrow = a.mask + ((size_t)b * a.T + min(qi, a.T - 1)) * a.T;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = c0 + (e >> 2) * 8 + lh * 4 + (e & 3);
        bool ok = key < nkeys;
        if (tree) ok = ok && qi < a.T && mrow[min(key, a.T - 1)] != 0;
        sv[e] = ok ? sacc[e] * scale : -INFINITY;
        cmax = fmaxf(cmax, sv[e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        sv[e] = sacc[e] * scale;
        cmax = fmaxf(cmax, sv[e]);
      }
    }
    cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));            // the other half of the query's keys
    // The reference m of a query only moves when a score exceeds it by more than kLazy: until then the
    // weights 2^(s - m) may grow to 2^kLazy (harmless in fp32 and in bf16), and the 64 accumulators of the
    // query need no rescaling, which for most chunks spares the whole wave the pass over its accumulators.
    const float m_new = (cmax > st.m[qb] + kLazy || st.m[qb] == -INFINITY) ? cmax : st.m[qb];
    const float alpha = (m_new == st.m[qb]) ? 1.f : exp2f(st.m[qb] - m_new);
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      sv[e] = __builtin_amdgcn_exp2f(sv[e] - m_new);                           // exp2(-inf) = 0 for hidden keys; m_new is finite
      psum += sv[e];                                          // whenever a key of the query has been seen
    }
    if (m_new == -INFINITY) {                                 // nothing visible yet: all weights are zero, not NaN
#pragma unroll
      for (int e = 0; e < 16; ++e) sv[e] = 0.f;
      psum = 0.f;
    }
    psum += __shfl_xor(psum, 32, 64);
    st.l[qb] = st.l[qb] * alpha + psum;
    st.m[qb] = m_new;
    if (__any(alpha != 1.f)) {                               // uniform
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) st.o[db][qb][e] *= alpha;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const u32x4 u = {pack_bf16x2(sv[8 * t], sv[8 * t + 1]), pack_bf16x2(sv[8 * t + 2], sv[8 * t + 3]),
                       pack_bf16x2(sv[8 * t + 4], sv[8 * t + 5]), pack_bf16x2(sv[8 * t + 6], sv[8 * t + 7])};
      pf[qb][t] = __builtin_bit_cast(bf16x8, u);
    }
  }
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
        st.o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xv.vf[db][t], pf[qb][t], st.o[db][qb], 0, 0, 0);
}

__global__ __launch_bounds__(256, 1) void tree_attn_partial_kernel(TreeAttnArgs a) {
  extern __shared__ __align__(16) float lds[];   // [4][kLdsPart]: the waves' partials at the end
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  const int nqt = (a.T + kQT - 1) / kQT;
  const int split = blockIdx.x / nqt, qt = blockIdx.x - split * nqt, h = blockIdx.y, b = blockIdx.z;
  const int gw = split * 4 + wave, ngw = a.nsplit * 4;
  const int ncp = (a.L + 31) >> 5, nct = (a.T + 31) >> 5;   // chunks of prompt keys, of tree keys
  const int nc = ncp + nct;

  // queries of this tile as B operands: lane (l32, lh) holds d = s*16 + lh*8 .. +7 of query qb*32 + l32
  bf16x8 qf[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int qi = qt * kQT + qb * 32 + l32;
    const uint16_t* qp = a.q + (((size_t)b * a.T + min(qi, a.T - 1)) * a.nh + h) * kAD + lh * 8;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      u32x4 u = {0u, 0u, 0u, 0u};
      if (qi < a.T) u = *reinterpret_cast<const u32x4*>(qp + s * 16);
      qf[qb][s] = __builtin_bit_cast(bf16x8, u);
    }
  }
  QueryState st;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) st.o[db][qb][e] = 0.f;
  st.m[0] = st.m[1] = -INFINITY;
  st.l[0] = st.l[1] = 0.f;

  for (int c = gw; c < nc; c += ngw) {   // chunks gw, gw + ngw, ...
    KeyOperands k;
    ValueOperands v;
    load_keys(a, c, ncp, b, h, lane, k);
    load_values(a, c, ncp, b, h, lane, v);
    attend_chunk(a, k, v, qf, c, ncp, b, qt, lane, st);
  }

  // the four waves' partials meet in LDS ...
  float* mine = lds + wave * kLdsPart;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int d = db * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
        mine[d * kLdsPitch + qb * 32 + l32] = st.o[db][qb][e];
      }
  if (lh == 0) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      mine[kAD * kLdsPitch + qb * 32 + l32] = st.m[qb];
      mine[kAD * kLdsPitch + kQT + qb * 32 + l32] = st.l[qb];
    }
  }
  __syncthreads();
  // ... and leave as one partial of the workgroup (fixed order): weight of every wave's partial per query first
  if (tid < kQT) {
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, lds[w * kLdsPart + kAD * kLdsPitch + tid]);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = lds[w * kLdsPart + kAD * kLdsPitch + tid];
      const float wg = (mw == -INFINITY) ? 0.f : exp2f(mw - M);
      lsum += wg * lds[w * kLdsPart + kAD * kLdsPitch + kQT + tid];
      lds[w * kLdsPart + kAD * kLdsPitch + 2 * kQT + tid] = wg;
    }
    lds[kAD * kLdsPitch + 3 * kQT + tid] = M;             // spare slots of wave 0's area
    lds[kLdsPart + kAD * kLdsPitch + 3 * kQT + tid] = lsum;   // ... and of wave 1's
  }
  __syncthreads();
  const float* wgt = lds + kAD * kLdsPitch + 2 * kQT;     // weight of wave w for query q at wgt[w * kLdsPart + q]
  const float* sM = lds + kAD * kLdsPitch + 3 * kQT;
  const float* sL = lds + kLdsPart + kAD * kLdsPitch + 3 * kQT;
  if (a.nsplit == 1) {
    // the only partial of its queries: finish here, no merge pass; consecutive threads write consecutive d
    const int d = tid & (kAD - 1);
    for (int q = tid >> 7; q < kQT; q += 2) {
      const int qi = qt * kQT + q;
      if (qi >= a.T) break;
      float acc = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) acc += wgt[w * kLdsPart + q] * lds[w * kLdsPart + d * kLdsPitch + q];
      // tree indices past n_sel are padding: zero rows
      a.out[(((size_t)b * a.T + qi) * a.nh + h) * kAD + d] = (qi <= a.n_sel[b]) ? acc / sL[q] : 0.f;
    }
    return;
  }
  float* part = a.part + ((((size_t)b * a.nh + h) * nqt + qt) * a.nsplit + split) * kPartFloats;
  const int qx = tid & (kQT - 1);
  for (int d = tid >> 6; d < kAD; d += 4) {
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) acc += wgt[w * kLdsPart + qx] * lds[w * kLdsPart + d * kLdsPitch + qx];
    part[d * kQT + qx] = acc;
  }
  if (tid < kQT) {
    part[kAD * kQT + qx] = sM[qx];
    part[kAD * kQT + kQT + qx] = sL[qx];
  }
}

// Merge of the workgroups' partials: one workgroup per (query tile x quarter of the head, head, sequence).
constexpr int kMaxSplits = 64;

__global__ __launch_bounds__(256) void tree_attn_merge_kernel(TreeAttnArgs a) {
  __shared__ float sw[kMaxSplits][kQT];   // weight of every partial for every query
  __shared__ float sden[kQT];
  const int nqt = (a.T + kQT - 1) / kQT;
  const int qt = blockIdx.x >> 2, dq0 = (blockIdx.x & 3) * 32, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const float* part = a.part + (((size_t)b * a.nh + h) * nqt + qt) * a.nsplit * kPartFloats;
  const int qx = tid & (kQT - 1), qi = qt * kQT + qx;
  if (tid < kQT) {
    float M = -INFINITY;
    for (int p = 0; p < a.nsplit; ++p) M = fmaxf(M, part[p * kPartFloats + kAD * kQT + qx]);
    float den = 0.f;
    for (int p = 0; p < a.nsplit; ++p) {   // fixed order
      const float mp = part[p * kPartFloats + kAD * kQT + qx];
      const float w = (mp == -INFINITY) ? 0.f : exp2f(mp - M);
      sw[p][qx] = w;
      den += w * part[p * kPartFloats + kAD * kQT + kQT + qx];
    }
    sden[qx] = den;
  }
  __syncthreads();
  if (qi >= a.T) return;
  const bool live = qi <= a.n_sel[b];     // tree indices past n_sel are padding: zero rows
  const float den = sden[qx];
  float* orow = a.out + (((size_t)b * a.T + qi) * a.nh + h) * kAD;
  float num[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) num[i] = 0.f;
  for (int p = 0; p < a.nsplit; ++p) {     // fixed order; the eight elements of a thread are independent loads
    const float w = sw[p][qx];
    const float* pp = part + (size_t)p * kPartFloats + (size_t)(dq0 + (tid >> 6)) * kQT + qx;
#pragma unroll
    for (int i = 0; i < 8; ++i) num[i] += w * pp[(size_t)4 * i * kQT];
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) orow[dq0 + (tid >> 6) + 4 * i] = live ? num[i] / den : 0.f;
}

// Prompt cache in fragment order: per (sequence, head, chunk of 32 keys) 8 KB of keys, [s][lane] x 8 bf16 =
// K[key c*32 + l32][d s*16 + lh*8 + 0..7], and 8 KB of values, [db*2 + t][lane] x 8 bf16 =
// V[key c*32 + 16t + 4*lh + 0..3, then c*32 + 16t + 8 + 4*lh + 0..3][d db*32 + l32]; keys past L are zero.
__global__ __launch_bounds__(64) void kv_pack_kernel(const uint16_t* k, const uint16_t* v, uint16_t* kp, uint16_t* vp,
                                                     int L, int nh) {
  const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x, l32 = lane & 31, lh = lane >> 5;
  const int ncp = gridDim.x;
  const size_t blk = (((size_t)b * nh + h) * ncp + c) * 8 * 64 * 8;   // in bf16 elements
  const int key = c * 32 + l32;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    u32x4 u = {0u, 0u, 0u, 0u};
    if (key < L) u = *reinterpret_cast<const u32x4*>(k + (((size_t)b * L + key) * nh + h) * kAD + s * 16 + lh * 8);
    *reinterpret_cast<u32x4*>(kp + blk + ((size_t)s * 64 + lane) * 8) = u;
  }
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint16_t e[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int kk = c * 32 + 16 * t + (i >> 2) * 8 + 4 * lh + (i & 3);
        e[i] = (kk < L) ? v[(((size_t)b * L + kk) * nh + h) * kAD + db * 32 + l32] : (uint16_t)0;
      }
      const u32x4 u = {(uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16),
                       (uint32_t)e[4] | ((uint32_t)e[5] << 16), (uint32_t)e[6] | ((uint32_t)e[7] << 16)};
      *reinterpret_cast<u32x4*>(vp + blk + ((size_t)(db * 2 + t) * 64 + lane) * 8) = u;
    }
}

hipError_t launch_kv_pack(const uint16_t* k, const uint16_t* v, uint16_t* kp, uint16_t* vp, int B, int L, int nh,
                          hipStream_t stream) {
  if (L <= 0) return hipSuccess;
  hipLaunchKernelGGL(kv_pack_kernel, dim3((L + 31) / 32, nh, B), dim3(64), 0, stream, k, v, kp, vp, L, nh);
  return hipGetLastError();
}

hipError_t prepare_tree_attention() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&tree_attn_partial_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kLdsPart * (int)sizeof(float));
}

size_t tree_attention_part_floats() { return (size_t)kPartFloats; }

hipError_t launch_tree_attention(const TreeAttnArgs& a, hipStream_t stream) {
  const int nqt = (a.T + kQT - 1) / kQT;
  hipLaunchKernelGGL(tree_attn_partial_kernel, dim3(a.nsplit * nqt, a.nh, a.B), dim3(256),
                     4 * kLdsPart * sizeof(float), stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.nsplit == 1) return e;
  hipLaunchKernelGGL(tree_attn_merge_kernel, dim3(nqt * 4, a.nh, a.B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
