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

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {   // round to nearest even, finite inputs
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7FFFu + ((a >> 16) & 1u);
  b += 0x7FFFu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xFFFF0000u);
}

__global__ __launch_bounds__(256, 1) void tree_attn_partial_kernel(TreeAttnArgs a) {
  extern __shared__ __align__(16) float lds[];   // [4][kPartFloats]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  const int nqt = (a.T + kQT - 1) / kQT;
  const int split = blockIdx.x / nqt, qt = blockIdx.x - split * nqt, h = blockIdx.y, b = blockIdx.z;
  const int gw = split * 4 + wave, ngw = a.nsplit * 4;
  const int ncp = (a.L + 31) >> 5, nct = (a.T + 31) >> 5;   // chunks of prompt keys, of tree keys

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
  f32x16 o[4][2];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[db][qb][e] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  const float scale = 0.08838834764831845f;   // 1 / sqrt(128)

  for (int c = gw; c < ncp + nct; c += ngw) {
    const bool tree = c >= ncp;
    const int c0 = (tree ? c - ncp : c) * 32;
    const int nkeys = tree ? a.T : a.L;
    // keys of the chunk as A operands: lane (l32, lh) holds d = s*16 + lh*8 .. +7 of key c0 + l32
    const int kj = min(c0 + l32, nkeys - 1);
    const uint16_t* kp = (tree ? a.k_tree + (((size_t)b * a.T + kj) * a.nh + h) * kAD
                               : a.k_prompt + (((size_t)b * a.L + kj) * a.nh + h) * kAD) + lh * 8;
    bf16x8 kf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kp + s * 16));
    // transposed values as A operands: lane (l32, lh) holds, for d = db*32 + l32 and 16-key step t, the keys
    // c0 + 16t + 4*lh + 0..3 and c0 + 16t + 8 + 4*lh + 0..3 (the order the first product leaves them in)
    const int xp = tree ? a.Tp : a.Lp;
    const uint16_t* vp = (tree ? a.vt_tree : a.vt_prompt) + (((size_t)b * a.nh + h) * kAD + l32) * xp + c0 + lh * 4;
    bf16x8 vf[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x2 lo = *reinterpret_cast<const u32x2*>(vp + (size_t)db * 32 * xp + t * 16);
        const u32x2 hi = *reinterpret_cast<const u32x2*>(vp + (size_t)db * 32 * xp + t * 16 + 8);
        const u32x4 u = {lo[0], lo[1], hi[0], hi[1]};
        vf[db][t] = __builtin_bit_cast(bf16x8, u);
      }

    bf16x8 pf[2][2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 sacc;
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[qb][s], sacc, 0, 0, 0);
      // register e of the lane: key c0 + (e>>2)*8 + lh*4 + (e&3), query qb*32 + l32
      const int qi = qt * kQT + qb * 32 + l32;
      const uint8_t* mrow = a.mask + ((size_t)b * a.T + min(qi, a.T - 1)) * a.T;
      float sv[16];
      float cmax = -INFINITY;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = c0 + (e >> 2) * 8 + lh * 4 + (e & 3);
        bool ok = key < nkeys;
        if (tree) ok = ok && qi < a.T && mrow[min(key, a.T - 1)] != 0;
        sv[e] = ok ? sacc[e] * scale : -INFINITY;
        cmax = fmaxf(cmax, sv[e]);
      }
      cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));            // the other half of the query's keys
      const float m_new = fmaxf(m_run[qb], cmax);
      const float alpha = (m_new == -INFINITY) ? 1.f : __expf(m_run[qb] - m_new);
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        sv[e] = (sv[e] == -INFINITY) ? 0.f : __expf(sv[e] - m_new);
        psum += sv[e];
      }
      psum += __shfl_xor(psum, 32, 64);
      l_run[qb] = l_run[qb] * alpha + psum;
      m_run[qb] = m_new;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][qb][e] *= alpha;
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
          o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][t], pf[qb][t], o[db][qb], 0, 0, 0);
  }

  // the four waves' partials meet in LDS ...
  float* mine = lds + wave * kPartFloats;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int d = db * 32 + (e >> 2) * 8 + lh * 4 + (e & 3);
        mine[d * kQT + qb * 32 + l32] = o[db][qb][e];
      }
  if (lh == 0) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      mine[kAD * kQT + qb * 32 + l32] = m_run[qb];
      mine[kAD * kQT + kQT + qb * 32 + l32] = l_run[qb];
    }
  }
  __syncthreads();
  // ... and leave as one partial of the workgroup (fixed order)
  float* part = a.part + ((((size_t)b * a.nh + h) * nqt + qt) * a.nsplit + split) * kPartFloats;
  const int qx = tid & (kQT - 1);
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) M = fmaxf(M, lds[w * kPartFloats + kAD * kQT + qx]);
  float wgt[4], lsum = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float mw = lds[w * kPartFloats + kAD * kQT + qx];
    wgt[w] = (mw == -INFINITY) ? 0.f : __expf(mw - M);
    lsum += wgt[w] * lds[w * kPartFloats + kAD * kQT + kQT + qx];
  }
  for (int d = tid >> 6; d < kAD; d += 4) {
    float acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) acc += wgt[w] * lds[w * kPartFloats + d * kQT + qx];
    part[d * kQT + qx] = acc;
  }
  if (tid < kQT) {
    part[kAD * kQT + qx] = M;
    part[kAD * kQT + kQT + qx] = lsum;
  }
}

// Merge of the workgroups' partials: one workgroup per (query tile, head, sequence).
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(TreeAttnArgs a) {
  const int nqt = (a.T + kQT - 1) / kQT;
  const int qt = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const float* part = a.part + (((size_t)b * a.nh + h) * nqt + qt) * a.nsplit * kPartFloats;
  const int qx = tid & (kQT - 1), qi = qt * kQT + qx;
  if (qi >= a.T) return;
  const bool live = qi <= a.n_sel[b];     // tree indices past n_sel are padding: zero rows
  float M = -INFINITY;
  for (int p = 0; p < a.nsplit; ++p) M = fmaxf(M, part[p * kPartFloats + kAD * kQT + qx]);
  float den = 0.f;
  for (int p = 0; p < a.nsplit; ++p) {
    const float mp = part[p * kPartFloats + kAD * kQT + qx];
    if (mp != -INFINITY) den += __expf(mp - M) * part[p * kPartFloats + kAD * kQT + kQT + qx];
  }
  float* orow = a.out + (((size_t)b * a.T + qi) * a.nh + h) * kAD;
  for (int d = tid >> 6; d < kAD; d += 4) {
    float num = 0.f;
    for (int p = 0; p < a.nsplit; ++p) {
      const float mp = part[p * kPartFloats + kAD * kQT + qx];
      if (mp != -INFINITY) num += __expf(mp - M) * part[p * kPartFloats + d * kQT + qx];
    }
    orow[d] = live ? num / den : 0.f;
  }
}

hipError_t prepare_tree_attention() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&tree_attn_partial_kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kPartFloats * (int)sizeof(float));
}

size_t tree_attention_part_floats() { return (size_t)kPartFloats; }

hipError_t launch_tree_attention(const TreeAttnArgs& a, hipStream_t stream) {
  const int nqt = (a.T + kQT - 1) / kQT;
  hipLaunchKernelGGL(tree_attn_partial_kernel, dim3(a.nsplit * nqt, a.nh, a.B), dim3(256),
                     4 * kPartFloats * sizeof(float), stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(tree_attn_merge_kernel, dim3(nqt, a.nh, a.B), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
