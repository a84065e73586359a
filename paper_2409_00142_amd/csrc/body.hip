// Stand-in draft layer: the kernels between two LM-head calls when the draft model's body is a
// real (synthetically weighted) EAGLE-shaped layer instead of a hook (Section 1, EAGLE paragraph:
// token embedding and parent feature -> FC -> one decoder layer -> the target's LM head; EAGLE-2
// paragraph: one input row per beam node, attending to the prompt and to its ancestors).
//
//   linear_stream_kernel   y (+)= x W^T for <= 16 rows: every weight matrix of the layer is read
//                          once per call, so these are HBM weight streams like the LM head
//                          (same streaming waves, plain store epilogue).
//   body_gather_kernel     x0 = [E[token], feature of the parent row]
//   rmsnorm_kernel         bf16(x / sqrt(mean x^2 + eps) * g)
//   body_attention_kernel  RoPE, bf16 key / value store, softmax over prompt + ancestors + self
//   silu_mul_kernel, body_final_kernel
// Rows of stopped sequences are skipped; a launch whose rows are all inactive exits at once.
#include "body_kernels.hpp"
#include "ddd_device.hpp"
#include "stream_tile.hpp"

namespace ddd {

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {   // finite inputs
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// ---- y (+)= x W^T ----------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(704) void linear_stream_kernel(LinearArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int NW = a.nw;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  if (a.row_active != nullptr) {   // uniform
    const int on = (lane < a.R) ? a.row_active[lane] : 0;
    if (__ballot(on != 0) == 0ull) return;
  }
  const int nslice = gridDim.x, slice = blockIdx.x;
  const int t0 = (int)(((long long)slice * a.ntiles) / nslice);
  const int t1 = (int)(((long long)(slice + 1) * a.ntiles) / nslice);
  const int nt = t1 - t0;

  float* red = reinterpret_cast<float*>(smem);      // [2][NW][256] fp32 partial tiles
  unsigned char* stage = smem + 2 * NW * 1024;      // [NW][kStageBytes]

  if (wave < NW) {
    // streaming wave: K-slice [wave*128*G, +128*G) of this pass, its share of x resident as B operands
    const int ks = wave * (128 * G);
    const int n = lane & 15, q = lane >> 4;
    bf16x8 bfrag[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x4 u = {0u, 0u, 0u, 0u};
        if (n < a.R) u = *reinterpret_cast<const u32x4*>(a.x + (size_t)n * a.ldx + ks + g * 128 + j * 32 + q * 8);
        bfrag[g][j] = __builtin_bit_cast(bf16x8, u);
      }
    const int lrow = lane >> 4, c = lane & 15;
    unsigned char* mystage = stage + wave * kStageBytes;
    const int wr_off = lrow * kStagePitch + c * 16;
    const int rd_off = n * kStagePitch + q * 16;
    const uint16_t* wbase = a.W + ks + c * 8;
    const int vlast = a.N - 1;

    u32x4 ring[G][4];
    {
      const int v0 = t0 * 16;
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = min(v0 + i * 4 + lrow, vlast);
          ring[g][i] = *reinterpret_cast<const u32x4*>(wbase + (size_t)row * a.ldw + g * 128);
        }
    }
    for (int t = 0; t + 1 < nt; ++t) {
      const f32x4 acc =
          stream_tile<G, true>(ring, bfrag, mystage, wr_off, rd_off, wbase, a.ldw, (t0 + t + 1) * 16 + lrow, vlast);
      *reinterpret_cast<f32x4*>(red + ((t & 1) * NW + wave) * 256 + lane * 4) = acc;
      __syncthreads();
    }
    if (nt > 0) {
      const int t = nt - 1;
      const f32x4 acc = stream_tile<G, false>(ring, bfrag, mystage, wr_off, rd_off, wbase, a.ldw, 0, vlast);
      *reinterpret_cast<f32x4*>(red + ((t & 1) * NW + wave) * 256 + lane * 4) = acc;
      __syncthreads();
    }
  } else {
    // epilogue wave: lane = (vb, r) owns outputs 4*vb .. 4*vb+3 of the tile for input row r
    const int r = lane & 15, vb = lane >> 4;
    for (int t = 0; t < nt; ++t) {
      __syncthreads();
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < NW; ++w)   // fixed order
        s += *reinterpret_cast<const f32x4*>(red + ((t & 1) * NW + w) * 256 + lane * 4);
      const int v0 = (t0 + t) * 16 + vb * 4;
      if (r < a.R) {
        float* yp = a.y + (size_t)r * a.ldy + v0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (v0 + e < a.N) yp[e] = a.accumulate ? yp[e] + s[e] : s[e];
      }
    }
  }
}

template <int G>
static hipError_t launch_linear_g(const LinearArgs& a, int nslice, hipStream_t stream) {
  const dim3 grid(nslice), block((a.nw + 1) * 64);
  const size_t lds = (size_t)2 * a.nw * 1024 + (size_t)a.nw * kStageBytes;
  hipLaunchKernelGGL((linear_stream_kernel<G>), grid, block, lds, stream, a);
  return hipGetLastError();
}

hipError_t launch_linear_stream(const LinearArgs& a, int G, int nslice, hipStream_t stream) {
  switch (G) {
    case 1: return launch_linear_g<1>(a, nslice, stream);
    case 2: return launch_linear_g<2>(a, nslice, stream);
    case 4: return launch_linear_g<4>(a, nslice, stream);
    default: return hipErrorInvalidValue;
  }
}

// ---- x0 = [E[token], parent feature] -----------------------------------------------------------
__global__ __launch_bounds__(256) void body_gather_kernel(BodyGatherArgs a) {
  const int r = blockIdx.x, tid = threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;
  int tok, prev_row, slot = 0;
  const uint16_t* feat;
  if (a.step == 0) {
    tok = a.root_token[r];
    feat = a.f_root + (size_t)r * a.H;
  } else {
    const int b = r / a.k;
    slot = a.beam_parent_slot[r];
    tok = a.beam_token[r];
    prev_row = (a.step == 1) ? b : b * a.k + slot;   // the prompt call has one row per sequence
    feat = a.h_prev + (size_t)prev_row * a.H;
    if (tid == 0) a.par_out[r] = slot;
  }
  const u32x4* e = reinterpret_cast<const u32x4*>(a.E + (size_t)tok * a.H);
  const u32x4* f = reinterpret_cast<const u32x4*>(feat);
  u32x4* x = reinterpret_cast<u32x4*>(a.x0 + (size_t)r * 2 * a.H);
  const int nv = a.H / 8;
  for (int i = tid; i < nv; i += 256) {
    x[i] = e[i];
    x[nv + i] = f[i];
  }
}

hipError_t launch_body_gather(const BodyGatherArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(body_gather_kernel, dim3(a.R), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- rmsnorm ----------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rmsnorm_kernel(RmsNormArgs a) {
  __shared__ float part[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;   // uniform over the block
  const float* x = a.x + (size_t)r * a.H;
  float ss = 0.f;
  for (int i = tid; i < a.H; i += 256) ss += x[i] * x[i];
  ss = wave_sum_f32(ss);
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  const float tot = ((part[0] + part[1]) + part[2]) + part[3];
  const float inv = 1.0f / sqrtf(tot / (float)a.H + 1e-6f);
  for (int i = tid; i < a.H; i += 256) a.out[(size_t)r * a.H + i] = f32_to_bf16_rne(x[i] * inv * a.g[i]);
}

hipError_t launch_rmsnorm(const RmsNormArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(rmsnorm_kernel, dim3(a.R), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- RoPE + key/value store + tree attention: one wave per (row, head) ---------------------------
__global__ __launch_bounds__(64) void body_attention_kernel(BodyAttnArgs a) {
  extern __shared__ __align__(16) float sm[];
  const int nh = a.H / kHeadDim;
  const int r = blockIdx.x / nh, h = blockIdx.x % nh, lane = threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;   // uniform
  const int b = (a.step == 0) ? r : r / a.k;
  const int n_vis = a.L + a.step + 1;
  float* qs = sm;                  // [128] rotated query
  float* ks = sm + 128;            // [128] own key as stored (bf16 values)
  float* vs = sm + 256;            // [128] own value as stored
  float* sc = sm + 384;            // [n_vis] scores, then weights
  int* anc = reinterpret_cast<int*>(sc + ((n_vis + 3) & ~3));   // [step] row of the ancestor in each earlier call

  {
    // pair (lane, lane + 64) of the head rotates by pos * base^(-2*lane/128)
    const float inv_freq = exp2f(-(float)(2 * lane) / (float)kHeadDim * 13.287712379549449f);   // log2(10000)
    float sn, cs;
    sincosf((float)(a.L + a.step) * inv_freq, &sn, &cs);
    const float* row = a.qkv + (size_t)r * 3 * a.H + h * kHeadDim;
    const float q0 = row[lane], q1 = row[lane + 64];
    const float k0 = row[a.H + lane], k1 = row[a.H + lane + 64];
    const float v0 = row[2 * a.H + lane], v1 = row[2 * a.H + lane + 64];
    qs[lane] = q0 * cs - q1 * sn;
    qs[lane + 64] = q1 * cs + q0 * sn;
    const uint16_t kb0 = f32_to_bf16_rne(k0 * cs - k1 * sn), kb1 = f32_to_bf16_rne(k1 * cs + k0 * sn);
    const uint16_t vb0 = f32_to_bf16_rne(v0), vb1 = f32_to_bf16_rne(v1);
    const size_t slot = ((size_t)a.step * kBodyRows + r) * a.H + h * kHeadDim;
    a.k_hist[slot + lane] = kb0;
    a.k_hist[slot + lane + 64] = kb1;
    a.v_hist[slot + lane] = vb0;
    a.v_hist[slot + lane + 64] = vb1;
    ks[lane] = bf16_to_f32(kb0);
    ks[lane + 64] = bf16_to_f32(kb1);
    vs[lane] = bf16_to_f32(vb0);
    vs[lane + 64] = bf16_to_f32(vb1);
    if (lane < a.step) {   // walk the parent slots back from this row to call number `lane`
      int cur = r;
      for (int s = a.step; s > lane; --s) {
        const int pslot = a.par_hist[s * kBodyRows + cur];
        cur = (s - 1 == 0) ? b : b * a.k + pslot;
      }
      anc[lane] = cur;
    }
  }
  __syncthreads();

  const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
  float mx = -INFINITY;
  for (int j = lane; j < n_vis; j += 64) {
    float dot = 0.f;
    if (j == n_vis - 1) {
      for (int i = 0; i < kHeadDim; ++i) dot += qs[i] * ks[i];
    } else {
      const uint16_t* kp = (j < a.L) ? a.Kp + ((size_t)(b * a.L + j) * a.H + h * kHeadDim)
                                     : a.k_hist + (((size_t)(j - a.L) * kBodyRows + anc[j - a.L]) * a.H + h * kHeadDim);
      for (int c = 0; c < kHeadDim / 8; ++c) {
        const u32x4 u = *reinterpret_cast<const u32x4*>(kp + c * 8);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          dot += qs[c * 8 + 2 * e] * __uint_as_float(u[e] << 16);
          dot += qs[c * 8 + 2 * e + 1] * __uint_as_float(u[e] & 0xFFFF0000u);
        }
      }
    }
    dot *= scale;
    sc[j] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = wave_max_f32(mx);
  float sum = 0.f;
  for (int j = lane; j < n_vis; j += 64) {
    const float p = __expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum_f32(sum);
  __syncthreads();

  float o0 = 0.f, o1 = 0.f;
  for (int j = 0; j < n_vis; ++j) {
    const float p = sc[j];
    if (j == n_vis - 1) {
      o0 += p * vs[lane];
      o1 += p * vs[lane + 64];
    } else {
      const uint16_t* vp = (j < a.L) ? a.Vp + ((size_t)(b * a.L + j) * a.H + h * kHeadDim)
                                     : a.v_hist + (((size_t)(j - a.L) * kBodyRows + anc[j - a.L]) * a.H + h * kHeadDim);
      o0 += p * bf16_to_f32(vp[lane]);
      o1 += p * bf16_to_f32(vp[lane + 64]);
    }
  }
  uint16_t* op = a.o + (size_t)r * a.H + h * kHeadDim;
  op[lane] = f32_to_bf16_rne(o0 / sum);
  op[lane + 64] = f32_to_bf16_rne(o1 / sum);
}

hipError_t launch_body_attention(const BodyAttnArgs& a, hipStream_t stream) {
  const int n_vis = a.L + a.step + 1;
  const size_t lds = (size_t)(384 + ((n_vis + 3) & ~3) + 32) * sizeof(float);
  hipLaunchKernelGGL(body_attention_kernel, dim3(a.R * (a.H / kHeadDim)), dim3(64), lds, stream, a);
  return hipGetLastError();
}

// ---- a = bf16(silu(gate) * up) ---------------------------------------------------------------------
__global__ __launch_bounds__(256) void silu_mul_kernel(SiluMulArgs a) {
  const int r = blockIdx.y, f = blockIdx.x * 256 + threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;
  if (f >= a.F) return;
  const float g = a.gu[(size_t)r * 2 * a.F + f], u = a.gu[(size_t)r * 2 * a.F + a.F + f];
  a.a[(size_t)r * a.F + f] = f32_to_bf16_rne(g / (1.0f + __expf(-g)) * u);
}

hipError_t launch_silu_mul(const SiluMulArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(silu_mul_kernel, dim3((a.F + 255) / 256, a.R), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- h = bf16(r) -------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void body_final_kernel(BodyFinalArgs a) {
  const int r = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;
  if (i >= a.H) return;
  const uint16_t hb = f32_to_bf16_rne(a.r[(size_t)r * a.H + i]);
  a.hid_out[(size_t)r * a.H + i] = hb;
  a.h_hist[(size_t)r * a.H + i] = hb;
}

hipError_t launch_body_final(const BodyFinalArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(body_final_kernel, dim3((a.H + 255) / 256, a.R), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
