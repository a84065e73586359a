// Stand-in draft layer: the kernels between two LM-head calls when the draft model's body is a
// real (synthetically weighted) EAGLE-shaped layer instead of a hook (Section 1, EAGLE paragraph:
// token embedding and parent feature -> FC -> one decoder layer -> the target's LM head; EAGLE-2
// paragraph: one input row per beam node, attending to the prompt and to its ancestors).
//
//   linear_stream_kernel   y (+)= x W^T for <= 16 rows: every weight matrix of the layer is read
//                          once per call, so these are HBM weight streams like the LM head
//                          (same streaming waves, plain store epilogue).
//                          Input rows are gathered in place (embedding row of the token, feature row of
//                          the parent).
//   rmsnorm_kernel         bf16(x / sqrt(mean x^2 + eps) * g)
//   body_attention_kernel  RoPE, bf16 key / value store, softmax over prompt + ancestors + self: one workgroup per
//                          (row, head); batched rounds: one per (sequence, head), by ordinary arithmetic
//                          (body_attention_seq_kernel) or with the prompt part on the matrix cores
//                          (body_attention_mfma_kernel, pack_prompt_values_kernel)
//   pack_x0_kernel         the FC's input rows assembled for the MFMA path of calls with more than 16 rows
//   The SiLU gate and the final bf16 rounding of the hidden rows ride in the epilogues of the
//   linears that produce their inputs.
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
  // Output rows are dealt to the workgroups in units of 4 (an epilogue lane's outputs, and whole gate/up
  // pairs), not in tiles of 16: every workgroup streams the same number of weight rows; a slice's last tile
  // is ragged, its missing rows repeat the slice's last row and are not written.
  const int nq = (a.N + 3) >> 2;
  const int n0 = (int)(((long long)slice * nq) / nslice) * 4;
  const int n1 = min((int)(((long long)(slice + 1) * nq) / nslice) * 4, a.N);
  const int nt = (n1 - n0 + 15) >> 4;

  float* red = reinterpret_cast<float*>(smem);      // [2][NW][256] fp32 partial tiles
  unsigned char* stage = smem + 2 * NW * 1024;      // [NW][kStageBytes]

  const int NR = a.n_ranges;
  const int total = nt * NR;          // (tile, range) steps of this workgroup, ranges innermost

  if (wave < NW) {
    // streaming wave: K-slice [wave*128*G, +128*G) of every range, its share of x resident as B operands
    const int ks = wave * (128 * G);
    const int n = lane & 15, q = lane >> 4;
    // the first tile of W is requested before anything else: it flies while the input rows are prepared
    const int lrow = lane >> 4, c = lane & 15;
    unsigned char* mystage = stage + wave * kStageBytes;
    const int wr_off = lrow * kStagePitch + c * 16;
    const int rd_off = n * kStagePitch + q * 16;
    const int woff = ks + c * 8;       // this lane's element offset inside a row of any range
    const uint16_t* wb0 = a.rg[0].W + woff;
    const int vlast = max(n1 - 1, 0);

    u32x4 ring[G][4];
    {
      const int v0 = n0;
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = min(v0 + i * 4 + lrow, vlast);
          ring[g][i] = *reinterpret_cast<const u32x4*>(wb0 + (size_t)row * a.ldw + g * 128);
        }
    }
    // source row of input row n in every range
    int src[kLinearRanges];
#pragma unroll
    for (int r = 0; r < kLinearRanges; ++r) {
      const LinearRange& rg = a.rg[r < NR ? r : 0];
      src[r] = n;
      if (n < a.R) {
        if (rg.gather_mode == kGatherIndex) src[r] = rg.gather_idx[n];
        else if (rg.gather_mode == kGatherInBlock) src[r] = (n / a.gather_k) * a.gather_k + rg.gather_idx[n];
        else if (rg.gather_mode == kGatherBlock) src[r] = n / a.gather_k;
      }
    }
    bf16x8 bfrag[G][4];
#pragma unroll 1
    for (int it = 0; it < total; ++it) {
      __builtin_amdgcn_sched_barrier(0);   // the previous step's operands are dead before the next ones are requested
      const int r = it % NR;
      if (NR > 1 || it == 0) {       // the input rows of this step's range
        const LinearRange& rg = a.rg[r];
        const uint16_t* xp = rg.x + (size_t)(r == 0 ? src[0] : r == 1 ? src[1] : src[2]) * rg.ldx + ks + q * 8;
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            u32x4 u = {0u, 0u, 0u, 0u};
            if (n < a.R) u = *reinterpret_cast<const u32x4*>(xp + g * 128 + j * 32);
            bfrag[g][j] = __builtin_bit_cast(bf16x8, u);
          }
      }
      f32x4 acc;
      if (it + 1 < total) {          // refill the ring with the next step's tile while this one is consumed
        const uint16_t* wn = a.rg[(it + 1) % NR].W + woff;
        acc = stream_tile<G, true>(ring, bfrag, mystage, wr_off, rd_off, wn, a.ldw, n0 + ((it + 1) / NR) * 16 + lrow, vlast);
      } else {
        acc = stream_tile<G, false>(ring, bfrag, mystage, wr_off, rd_off, wb0, a.ldw, 0, vlast);
      }
      *reinterpret_cast<f32x4*>(red + ((it & 1) * NW + wave) * 256 + lane * 4) = acc;
      __syncthreads();
    }
  } else {
    // epilogue wave: lane = (vb, r) owns outputs 4*vb .. 4*vb+3 of the tile for input row r
    const int r = lane & 15, vb = lane >> 4;
    for (int t = 0; t < nt; ++t) {
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      for (int rr = 0; rr < NR; ++rr) {
        const int it = t * NR + rr;
        __syncthreads();
        for (int w = 0; w < NW; ++w)   // fixed order
          s += *reinterpret_cast<const f32x4*>(red + ((it & 1) * NW + w) * 256 + lane * 4);
      }
      const int v0 = n0 + t * 16 + vb * 4;
      if (r < a.R && (a.row_active == nullptr || a.row_active[r] != 0)) {   // rows of stopped sequences stay untouched
        if (a.mode == kLinearSiluPairs) {   // outputs (v0, v0+1) and (v0+2, v0+3) are (gate, up) pairs
#pragma unroll
          for (int e = 0; e < 4; e += 2)
            if (v0 + e + 1 < n1) {
              const float g = s[e], u = s[e + 1];
              a.out16[(size_t)r * a.ld16 + ((v0 + e) >> 1)] = f32_to_bf16_rne(g / (1.0f + __expf(-g)) * u);
            }
        } else {
          float* yp = a.y + (size_t)r * a.ldy + v0;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (v0 + e < n1) {
              const float y = (a.mode == kLinearAccumulate) ? yp[e] + s[e] : s[e];
              yp[e] = y;
              if (a.out16 != nullptr) {
                const uint16_t yb = f32_to_bf16_rne(y);
                a.out16[(size_t)r * a.ld16 + v0 + e] = yb;
                if (a.out16b != nullptr) a.out16b[(size_t)r * a.ld16 + v0 + e] = yb;
              }
            }
        }
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

// ---- rmsnorm ----------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void rmsnorm_kernel(RmsNormArgs a) {
  __shared__ float part[16];
  const int r = blockIdx.x, tid = threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;   // uniform over the block
  const float* x = a.x + (size_t)r * a.H;
  float xv[8];                                                   // H <= 8192
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int i = tid + 1024 * j;
    xv[j] = (i < a.H) ? x[i] : 0.f;
    ss += xv[j] * xv[j];
  }
  ss = wave_sum_f32(ss);
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += part[w];                  // fixed order
  const float inv = 1.0f / sqrtf(tot / (float)a.H + 1e-6f);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int i = tid + 1024 * j;
    if (i < a.H) a.out[(size_t)r * a.H + i] = f32_to_bf16_rne(xv[j] * inv * a.g[i]);
  }
}

hipError_t launch_rmsnorm(const RmsNormArgs& a, hipStream_t stream) {
  if (a.H > 8192) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rmsnorm_kernel, dim3(a.R), dim3(1024), 0, stream, a);
  return hipGetLastError();
}

// ---- RoPE + key/value store + tree attention: one workgroup of 16 waves per (row, head) ----------
// Every phase is a few dependent memory round trips deep at most: keys are dealt one per thread,
// values to 8 groups of 128 threads (one per element of the head).
constexpr int kAttnThreads = 1024;

__device__ __forceinline__ float block_max_f32(float x, float* red, int tid) {
  x = wave_max_f32(x);
  __syncthreads();              // red may still be read from an earlier reduction
  if ((tid & 63) == 0) red[tid >> 6] = x;
  __syncthreads();
  float m = red[0];
#pragma unroll
  for (int w = 1; w < kAttnThreads / 64; ++w) m = fmaxf(m, red[w]);
  return m;
}
__device__ __forceinline__ float block_sum_f32(float x, float* red, int tid) {
  x = wave_sum_f32(x);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = x;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < kAttnThreads / 64; ++w) s += red[w];      // fixed order
  return s;
}

__global__ __launch_bounds__(kAttnThreads) void body_attention_kernel(BodyAttnArgs a) {
  extern __shared__ __align__(16) float sm[];
  const int nh = a.H / kHeadDim;
  const int r = blockIdx.x / nh, h = blockIdx.x % nh, tid = threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;   // uniform
  const int b = (a.step == 0) ? r : r / a.k;
  const int n_vis = a.L + a.step + 1;
  float* qs = sm;                  // [128] rotated query
  float* ks = sm + 128;            // [128] own key as stored (bf16 values)
  float* vs = sm + 256;            // [128] own value as stored
  float* red = sm + 384;           // [16] block reductions
  float* part = sm + 400;          // [8][128] partial outputs
  float* sc = sm + 400 + 8 * kHeadDim;                            // [n_vis] scores, then weights
  int* anc = reinterpret_cast<int*>(sc + ((n_vis + 3) & ~3));    // [step] row of the ancestor in each earlier call

  if (tid < 64) {
    // pair (tid, tid + 64) of the head rotates by pos * base^(-2*tid/128)
    const float inv_freq = exp2f(-(float)(2 * tid) / (float)kHeadDim * 13.287712379549449f);   // log2(10000)
    float sn, cs;
    sincosf((float)(a.L + a.step) * inv_freq, &sn, &cs);
    const float* row = a.qkv + (size_t)r * 3 * a.H + h * kHeadDim;
    const float q0 = row[tid], q1 = row[tid + 64];
    const float k0 = row[a.H + tid], k1 = row[a.H + tid + 64];
    const float v0 = row[2 * a.H + tid], v1 = row[2 * a.H + tid + 64];
    qs[tid] = q0 * cs - q1 * sn;
    qs[tid + 64] = q1 * cs + q0 * sn;
    const uint16_t kb0 = f32_to_bf16_rne(k0 * cs - k1 * sn), kb1 = f32_to_bf16_rne(k1 * cs + k0 * sn);
    const uint16_t vb0 = f32_to_bf16_rne(v0), vb1 = f32_to_bf16_rne(v1);
    const size_t slot = ((size_t)a.step * a.hist_rows + r) * a.H + h * kHeadDim;
    a.k_hist[slot + tid] = kb0;
    a.k_hist[slot + tid + 64] = kb1;
    a.v_hist[slot + tid] = vb0;
    a.v_hist[slot + tid + 64] = vb1;
    ks[tid] = bf16_to_f32(kb0);
    ks[tid + 64] = bf16_to_f32(kb1);
    vs[tid] = bf16_to_f32(vb0);
    vs[tid + 64] = bf16_to_f32(vb1);
  } else if (tid < 64 + a.step) {   // walk the parent slots back from this row to call number c
    const int c = tid - 64;
    int cur = r;
    for (int s = a.step; s > c; --s) {
      // this call's slots are still in the beam (and are recorded below); earlier calls' were recorded then
      const int pslot = (s == a.step) ? a.beam_parent_slot[cur] : a.par_hist[s * a.hist_rows + cur];
      cur = (s - 1 == 0) ? b : b * a.k + pslot;
    }
    anc[c] = cur;
  } else if (tid == 128 && h == 0 && a.step >= 1) {
    a.par_hist[a.step * a.hist_rows + r] = a.beam_parent_slot[r];
  }
  __syncthreads();

  // scores: one key per thread
  const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
  float mx = -INFINITY;
  for (int j = tid; j < n_vis; j += kAttnThreads) {
    float dot = 0.f;
    if (j == n_vis - 1) {
      for (int i = 0; i < kHeadDim; ++i) dot += qs[i] * ks[i];
    } else {
      const uint16_t* kp = (j < a.L) ? a.Kp + ((size_t)(b * a.L + j) * a.H + h * kHeadDim)
                                     : a.k_hist + (((size_t)(j - a.L) * a.hist_rows + anc[j - a.L]) * a.H + h * kHeadDim);
      u32x4 u[kHeadDim / 8];
#pragma unroll
      for (int c = 0; c < kHeadDim / 8; ++c) u[c] = *reinterpret_cast<const u32x4*>(kp + c * 8);
#pragma unroll
      for (int c = 0; c < kHeadDim / 8; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          dot += qs[c * 8 + 2 * e] * __uint_as_float(u[c][e] << 16);
          dot += qs[c * 8 + 2 * e + 1] * __uint_as_float(u[c][e] & 0xFFFF0000u);
        }
    }
    dot *= scale;
    sc[j] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = block_max_f32(mx, red, tid);
  float sum = 0.f;
  for (int j = tid; j < n_vis; j += kAttnThreads) {
    const float p = __expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = block_sum_f32(sum, red, tid);   // its barriers also publish the weights

  // values: element d of the head, keys grp, grp + 8, ...
  const int d = tid & (kHeadDim - 1), grp = tid >> 7;
  float o = 0.f;
  {
    const uint16_t* vbase = a.Vp + ((size_t)b * a.L * a.H + h * kHeadDim + d);
    int j = grp;
    for (; j + 8 * 15 < a.L; j += 8 * 16) {   // sixteen keys of this group in flight
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = bf16_to_f32(vbase[(size_t)(j + 8 * i) * a.H]);
#pragma unroll
      for (int i = 0; i < 16; ++i) o += sc[j + 8 * i] * v[i];
    }
    for (; j < a.L; j += 8) o += sc[j] * bf16_to_f32(vbase[(size_t)j * a.H]);
    for (int c = grp; c < a.step; c += 8)
      o += sc[a.L + c] * bf16_to_f32(a.v_hist[((size_t)c * a.hist_rows + anc[c]) * a.H + h * kHeadDim + d]);
    if (grp == 0) o += sc[n_vis - 1] * vs[d];
  }
  part[grp * kHeadDim + d] = o;
  __syncthreads();
  if (tid < kHeadDim) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 8; ++g) t += part[g * kHeadDim + tid];   // fixed order
    a.o[(size_t)r * a.H + h * kHeadDim + tid] = f32_to_bf16_rne(t / sum);
  }
}

// ---- rows of [E[token], parent feature] for the GEMM path: one workgroup per row ------------------------------
__global__ __launch_bounds__(256) void pack_x0_kernel(PackX0Args a) {
  const int r = blockIdx.x, tid = threadIdx.x;
  if (a.row_active != nullptr && a.row_active[r] == 0) return;   // uniform
  int fr = r;
  if (a.feat_mode == kGatherBlock) fr = r / a.k;
  else if (a.feat_mode == kGatherInBlock) fr = (r / a.k) * a.k + a.parent_slot[r];
  const u32x4* e = reinterpret_cast<const u32x4*>(a.E + (size_t)a.token[r] * a.H);
  const u32x4* f = reinterpret_cast<const u32x4*>(a.feat + (size_t)fr * a.H);
  u32x4* out = reinterpret_cast<u32x4*>(a.x0 + (size_t)r * 2 * a.H);
  const int n = a.H / 8;                                         // 16-byte pieces of a half
  for (int i = tid; i < n; i += 256) {
    out[i] = e[i];
    out[n + i] = f[i];
  }
}

hipError_t launch_pack_x0(const PackX0Args& a, hipStream_t stream) {
  hipLaunchKernelGGL(pack_x0_kernel, dim3(a.R), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---- the same attention for batched rounds: one workgroup per (sequence, head) ---------------------------------
// The k rows of a sequence share the prompt's keys and values, which are most of what the attention reads: with one
// workgroup per (row, head) they would be fetched k times and the launch would be hundreds of small latency-bound
// workgroups per CU (measured at B = 64, k = 10, L = 256: 510 us per call against 187 us).  Here each prompt key is
// read once and multiplied with all k queries (four threads per key, 32 elements each), each value once and
// weighted into all k outputs.  The arithmetic per row is that of body_attention_kernel (the same products and
// weights; sums in a different but fixed order).
constexpr int kSeqRows = 16;          // most rows per sequence (k) this kernel handles
constexpr int kSeqThreads = 1024;

__global__ __launch_bounds__(kSeqThreads) void body_attention_seq_kernel(BodyAttnArgs a) {
  extern __shared__ __align__(16) float sm[];
  const int nh = a.H / kHeadDim;
  const int b = blockIdx.x / nh, h = blockIdx.x % nh, tid = threadIdx.x;
  const int kk = (a.step == 0) ? 1 : a.k;                 // rows of this sequence
  const int r0 = (a.step == 0) ? b : b * a.k;
  if (a.row_active != nullptr && a.row_active[r0] == 0) return;   // uniform: a sequence's rows share their flag
  const int n_vis = a.L + a.step + 1;
  float* qs = sm;                                  // [kSeqRows][128] rotated queries
  float* ks = qs + kSeqRows * kHeadDim;            // [kSeqRows][128] own keys as stored (bf16 values)
  float* vs = ks + kSeqRows * kHeadDim;            // [kSeqRows][128] own values as stored
  float* part = vs + kSeqRows * kHeadDim;          // [8][kSeqRows][128] partial outputs
  float* rsum = part + 8 * kSeqRows * kHeadDim;    // [kSeqRows] sums of the weights
  int* anc = reinterpret_cast<int*>(rsum + kSeqRows);   // [kSeqRows][32] row of the ancestor in each earlier call
  float* sct = reinterpret_cast<float*>(anc + kSeqRows * 32);   // [n_vis][kSeqRows] scores, then weights

  if (tid < kk * 64) {
    // pair (p, p + 64) of the head of row i rotates by pos * base^(-2p/128)
    const int i = tid >> 6, p = tid & 63, r = r0 + i;
    const float inv_freq = exp2f(-(float)(2 * p) / (float)kHeadDim * 13.287712379549449f);   // log2(10000)
    float sn, cs;
    sincosf((float)(a.L + a.step) * inv_freq, &sn, &cs);
    const float* row = a.qkv + (size_t)r * 3 * a.H + h * kHeadDim;
    const float q0 = row[p], q1 = row[p + 64];
    const float k0 = row[a.H + p], k1 = row[a.H + p + 64];
    const float v0 = row[2 * a.H + p], v1 = row[2 * a.H + p + 64];
    qs[i * kHeadDim + p] = q0 * cs - q1 * sn;
    qs[i * kHeadDim + p + 64] = q1 * cs + q0 * sn;
    const uint16_t kb0 = f32_to_bf16_rne(k0 * cs - k1 * sn), kb1 = f32_to_bf16_rne(k1 * cs + k0 * sn);
    const uint16_t vb0 = f32_to_bf16_rne(v0), vb1 = f32_to_bf16_rne(v1);
    const size_t slot = ((size_t)a.step * a.hist_rows + r) * a.H + h * kHeadDim;
    a.k_hist[slot + p] = kb0;
    a.k_hist[slot + p + 64] = kb1;
    a.v_hist[slot + p] = vb0;
    a.v_hist[slot + p + 64] = vb1;
    ks[i * kHeadDim + p] = bf16_to_f32(kb0);
    ks[i * kHeadDim + p + 64] = bf16_to_f32(kb1);
    vs[i * kHeadDim + p] = bf16_to_f32(vb0);
    vs[i * kHeadDim + p + 64] = bf16_to_f32(vb1);
  }
  if (tid < kk * 32 && (tid & 31) < a.step) {   // walk the parent slots back from row i to call number c
    const int i = tid >> 5, c = tid & 31;
    int cur = r0 + i;
    for (int s = a.step; s > c; --s) {
      const int pslot = (s == a.step) ? a.beam_parent_slot[cur] : a.par_hist[s * a.hist_rows + cur];
      cur = (s - 1 == 0) ? b : b * a.k + pslot;
    }
    anc[i * 32 + c] = cur;
  }
  if (h == 0 && a.step >= 1 && tid >= 512 && tid < 512 + kk)
    a.par_hist[a.step * a.hist_rows + r0 + tid - 512] = a.beam_parent_slot[r0 + tid - 512];
  __syncthreads();

  // ---- scores.  Prompt keys: four threads per key, 32 elements each, all rows of the sequence ----------------
  const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
  {
    const int qd = tid & 3;
    for (int j = tid >> 2; j < a.L; j += kSeqThreads / 4) {
      const uint16_t* kp = a.Kp + ((size_t)(b * a.L + j) * a.H + h * kHeadDim + qd * 32);
      u32x4 u[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) u[c] = *reinterpret_cast<const u32x4*>(kp + c * 8);
      float kf[32];
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kf[c * 8 + 2 * e] = __uint_as_float(u[c][e] << 16);
          kf[c * 8 + 2 * e + 1] = __uint_as_float(u[c][e] & 0xFFFF0000u);
        }
      for (int i = 0; i < kk; ++i) {
        const float* q = qs + i * kHeadDim + qd * 32;
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 32; ++e) dot += q[e] * kf[e];
        dot += dpp_move_f32<0xB1>(dot);       // the four quarters of the key: lanes ^1, then ^2 (fixed order)
        dot += dpp_move_f32<0x4E>(dot);
        if (qd == 0) sct[j * kSeqRows + i] = dot * scale;
      }
    }
    // the rows' ancestors and themselves: one (row, key) pair per thread
    for (int e = tid; e < kk * (a.step + 1); e += kSeqThreads) {
      const int i = e / (a.step + 1), c = e - i * (a.step + 1);
      float dot = 0.f;
      if (c == a.step) {
        for (int x = 0; x < kHeadDim; ++x) dot += qs[i * kHeadDim + x] * ks[i * kHeadDim + x];
      } else {
        const uint16_t* kp = a.k_hist + (((size_t)c * a.hist_rows + anc[i * 32 + c]) * a.H + h * kHeadDim);
        for (int x = 0; x < kHeadDim; x += 2) {
          const uint32_t w = *reinterpret_cast<const uint32_t*>(kp + x);
          dot += qs[i * kHeadDim + x] * __uint_as_float(w << 16);
          dot += qs[i * kHeadDim + x + 1] * __uint_as_float(w & 0xFFFF0000u);
        }
      }
      sct[(a.L + c) * kSeqRows + i] = dot * scale;
    }
  }
  __syncthreads();
  // ---- softmax weights: wave i takes row i --------------------------------------------------------------------
  {
    const int i = tid >> 6, lane = tid & 63;
    if (i < kk) {
      float mx = -INFINITY;
      for (int j = lane; j < n_vis; j += 64) mx = fmaxf(mx, sct[j * kSeqRows + i]);
      mx = wave_max_f32(mx);
      float sum = 0.f;
      for (int j = lane; j < n_vis; j += 64) {
        const float p = __expf(sct[j * kSeqRows + i] - mx);
        sct[j * kSeqRows + i] = p;
        sum += p;
      }
      sum = wave_sum_f32(sum);
      if (lane == 0) rsum[i] = sum;
    }
  }
  __syncthreads();
  // ---- values: element d of the head, keys grp, grp + 8, ...; every value weighted into all rows ---------------
  const int d = tid & (kHeadDim - 1), grp = tid >> 7;
  float o[kSeqRows];
#pragma unroll
  for (int i = 0; i < kSeqRows; ++i) o[i] = 0.f;
  {
    const uint16_t* vbase = a.Vp + ((size_t)b * a.L * a.H + h * kHeadDim + d);
    int j = grp;
    for (; j + 8 * 7 < a.L; j += 8 * 8) {   // eight keys of this group in flight
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = bf16_to_f32(vbase[(size_t)(j + 8 * u) * a.H]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const f32x4* w = reinterpret_cast<const f32x4*>(sct + (j + 8 * u) * kSeqRows);
#pragma unroll
        for (int i4 = 0; i4 < kSeqRows / 4; ++i4) {
          const f32x4 ww = w[i4];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[i4 * 4 + e] += ww[e] * v[u];
        }
      }
    }
    for (; j < a.L; j += 8) {
      const float v = bf16_to_f32(vbase[(size_t)j * a.H]);
#pragma unroll
      for (int i = 0; i < kSeqRows; ++i) o[i] += sct[j * kSeqRows + i] * v;
    }
#pragma unroll
    for (int i = 0; i < kSeqRows; ++i)
      if (i < kk) {
        for (int c = grp; c < a.step; c += 8)
          o[i] += sct[(a.L + c) * kSeqRows + i] *
                  bf16_to_f32(a.v_hist[((size_t)c * a.hist_rows + anc[i * 32 + c]) * a.H + h * kHeadDim + d]);
        if (grp == 0) o[i] += sct[(n_vis - 1) * kSeqRows + i] * vs[i * kHeadDim + d];
      }
  }
#pragma unroll
  for (int i = 0; i < kSeqRows; ++i) part[(grp * kSeqRows + i) * kHeadDim + d] = o[i];
  __syncthreads();
  for (int e = tid; e < kk * kHeadDim; e += kSeqThreads) {
    const int i = e >> 7, x = e & (kHeadDim - 1);
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 8; ++g) t += part[(g * kSeqRows + i) * kHeadDim + x];   // fixed order
    a.o[(size_t)(r0 + i) * a.H + h * kHeadDim + x] = f32_to_bf16_rne(t / rsum[i]);
  }
}

// ---- batched rounds, the prompt part on the matrix cores ---------------------------------------------------------
// One workgroup of four waves per (sequence, head).  The L prompt keys are the same for every row of the sequence, so
// their scores and their part of the output are two small contractions, 16 rows at a time:
//   S[key][row] = sum_d K[key][d] q[row][d]      (v_mfma_f32_16x16x32_bf16: A = 16 keys x 32 d, B = 16 rows x 32 d)
//   O[d][row]   = sum_key V[key][d] p[row][key]  (A = 16 d x 32 keys, B = 16 rows x 32 keys)
// The fp32 operands (rotated queries, softmax weights) go in as two bf16 halves, x = hi + lo with |x - hi - lo| <=
// 2^-17 |x| (two MFMAs per tile), so no rounding point is added to the layer's definition.  Both A operands come
// straight from global memory, 16 bytes per lane: 8 consecutive d of one key for the first contraction (the cache's
// own layout), 8 consecutive keys of one d for the second, which needs the values with the keys of an element
// contiguous: pack_prompt_values_kernel writes that copy in the prompt call of every round.  No operand is staged in
// LDS, which leaves room for three workgroups per CU: each is a chain of dependent steps, and the others' loads run
// under it.  The rows' own keys and their ancestors' (at most 32 per row, different from row to row) are handled by
// ordinary arithmetic.  (With one workgroup per (row, head) the launch took 510 us at the 7B shape with 640 rows, with
// ordinary arithmetic per (sequence, head) 177 us.)
constexpr int kMfThreads = 256;

static size_t attention_mfma_lds(int Lp, int n_vis) {
  return (size_t)(kSeqRows * kHeadDim + kSeqRows + kSeqRows * 32 + (size_t)n_vis * kSeqRows) * sizeof(float) +
         (size_t)(2 * kSeqRows * kHeadDim + 2 * kSeqRows * (Lp + 8)) * sizeof(uint16_t);
}

__device__ __forceinline__ void split_bf16x8(const float* x, bool on, bf16x8& hi, bf16x8& lo) {
  u32x4 h, l;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float x0 = on ? x[2 * e] : 0.f, x1 = on ? x[2 * e + 1] : 0.f;
    const uint32_t h0 = f32_to_bf16_rne(x0), h1 = f32_to_bf16_rne(x1);
    const uint32_t l0 = f32_to_bf16_rne(x0 - bf16_to_f32((uint16_t)h0)), l1 = f32_to_bf16_rne(x1 - bf16_to_f32((uint16_t)h1));
    h[e] = h0 | (h1 << 16);
    l[e] = l0 | (l1 << 16);
  }
  hi = __builtin_bit_cast(bf16x8, h);
  lo = __builtin_bit_cast(bf16x8, l);
}

__global__ __launch_bounds__(kMfThreads) void body_attention_mfma_kernel(BodyAttnArgs a) {
  extern __shared__ __align__(16) unsigned char smb[];
  const int nh = a.H / kHeadDim;
  const int b = blockIdx.x / nh, h = blockIdx.x % nh, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kk = (a.step == 0) ? 1 : a.k;                 // rows of this sequence
  const int r0 = (a.step == 0) ? b : b * a.k;
  if (a.row_active != nullptr && a.row_active[r0] == 0) return;   // uniform: a sequence's rows share their flag
  const int L = a.L, Lp = a.Lp, n_vis = L + a.step + 1;
  const int ppitch = Lp + 8;
  float* qs = reinterpret_cast<float*>(smb);        // [kSeqRows][128] rotated queries; later the prompt's part of the outputs
  float* rsum = qs + kSeqRows * kHeadDim;           // [kSeqRows] sums of the weights
  int* anc = reinterpret_cast<int*>(rsum + kSeqRows);            // [kSeqRows][32] row of the ancestor in each earlier call
  float* sct = reinterpret_cast<float*>(anc + kSeqRows * 32);    // [n_vis][kSeqRows] scores; weights of the keys past the prompt
  uint16_t* ks = reinterpret_cast<uint16_t*>(sct + (size_t)n_vis * kSeqRows);   // [kSeqRows][128] own keys as stored
  uint16_t* vs = ks + kSeqRows * kHeadDim;                                      // [kSeqRows][128] own values as stored
  uint16_t* ph = vs + kSeqRows * kHeadDim;          // [kSeqRows][ppitch] weights of the prompt keys, high halves
  uint16_t* pl = ph + kSeqRows * ppitch;            // ... low halves

  // ---- the first 256 prompt keys: requested now, multiplied once the queries are rotated ------------------------
  // lane (row, dq) of the A operand holds 8 consecutive d of key `row` of the tile; tile t belongs to wave t mod 4
  const int ntile = (L + 15) >> 4;
  u32x4 kf[4][4];
  auto load_keys = [&](int t0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = min((t0 + wave + 4 * i) * 16 + (lane & 15), L - 1);
      const uint16_t* kp = a.Kp + ((size_t)(b * L + key) * a.H + h * kHeadDim + (lane >> 4) * 8);
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) kf[i][s4] = *reinterpret_cast<const u32x4*>(kp + s4 * 32);
    }
  };
  load_keys(0);
  // ---- own rows: rotate, store, ancestors (as in the kernels above) -----------------------------------------------
  for (int t = tid; t < kk * 64; t += kMfThreads) {
    const int i = t >> 6, p = t & 63, r = r0 + i;
    const float inv_freq = exp2f(-(float)(2 * p) / (float)kHeadDim * 13.287712379549449f);   // log2(10000)
    float sn, cs;
    sincosf((float)(L + a.step) * inv_freq, &sn, &cs);
    const float* row = a.qkv + (size_t)r * 3 * a.H + h * kHeadDim;
    const float q0 = row[p], q1 = row[p + 64];
    const float k0 = row[a.H + p], k1 = row[a.H + p + 64];
    const float v0 = row[2 * a.H + p], v1 = row[2 * a.H + p + 64];
    qs[i * kHeadDim + p] = q0 * cs - q1 * sn;
    qs[i * kHeadDim + p + 64] = q1 * cs + q0 * sn;
    const uint16_t kb0 = f32_to_bf16_rne(k0 * cs - k1 * sn), kb1 = f32_to_bf16_rne(k1 * cs + k0 * sn);
    const uint16_t vb0 = f32_to_bf16_rne(v0), vb1 = f32_to_bf16_rne(v1);
    const size_t slot = ((size_t)a.step * a.hist_rows + r) * a.H + h * kHeadDim;
    a.k_hist[slot + p] = kb0;
    a.k_hist[slot + p + 64] = kb1;
    a.v_hist[slot + p] = vb0;
    a.v_hist[slot + p + 64] = vb1;
    ks[i * kHeadDim + p] = kb0;
    ks[i * kHeadDim + p + 64] = kb1;
    vs[i * kHeadDim + p] = vb0;
    vs[i * kHeadDim + p + 64] = vb1;
  }
  for (int t = tid; t < kk * 32; t += kMfThreads) {   // walk the parent slots back from row i to call number c
    const int i = t >> 5, c = t & 31;
    if (c >= a.step) continue;
    int cur = r0 + i;
    for (int s = a.step; s > c; --s) {
      const int pslot = (s == a.step) ? a.beam_parent_slot[cur] : a.par_hist[s * a.hist_rows + cur];
      cur = (s - 1 == 0) ? b : b * a.k + pslot;
    }
    anc[i * 32 + c] = cur;
  }
  if (h == 0 && a.step >= 1 && tid < kk) a.par_hist[a.step * a.hist_rows + r0 + tid] = a.beam_parent_slot[r0 + tid];
  for (int e = tid; e < kSeqRows * ppitch / 2; e += kMfThreads) {   // rows and keys that do not exist weigh nothing
    reinterpret_cast<uint32_t*>(ph)[e] = 0u;
    reinterpret_cast<uint32_t*>(pl)[e] = 0u;
  }
  __syncthreads();

  // ---- scores of the prompt keys ------------------------------------------------------------------------------------
  const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
  const int row = lane & 15, q4 = lane >> 4;  // operand coordinates of the lane (B: row of the sequence; A: key or d)
  {
    bf16x8 qh[4], ql[4];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) split_bf16x8(qs + row * kHeadDim + s4 * 32 + q4 * 8, row < kk, qh[s4], ql[s4]);
    for (int t0 = 0; t0 < ntile; t0 += 16) {
      if (t0 > 0) load_keys(t0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int t = t0 + wave + 4 * i;
        if (t >= ntile) continue;                                    // wave-uniform
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const bf16x8 kfr = __builtin_bit_cast(bf16x8, kf[i][s4]);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr, qh[s4], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfr, ql[s4], acc, 0, 0, 0);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {                                // accumulator e: key 4 * (lane >> 4) + e, row lane & 15
          const int key = t * 16 + q4 * 4 + e;
          if (key < L) sct[key * kSeqRows + row] = acc[e] * scale;
        }
      }
    }
  }
  // ---- the prompt's values for this wave's two d tiles (first 256 keys): on their way from here on ----------------
  // lane (d, kq) of the A operand holds 8 consecutive keys of element d
  const int nstep = Lp >> 5;
  u32x4 vf[2][8];
  auto load_values = [&](int st0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const uint16_t* vp = a.Vt + ((size_t)b * a.H + h * kHeadDim + (wave * 2 + j) * 16 + row) * Lp + q4 * 8;
#pragma unroll
      for (int u = 0; u < 8; ++u) vf[j][u] = *reinterpret_cast<const u32x4*>(vp + min(st0 + u, nstep - 1) * 32);
    }
  };
  load_values(0);
  // ---- the rows' ancestors and themselves: four threads per (row, key) pair, 32 elements each ---------------------
  for (int e4 = tid; e4 < kk * (a.step + 1) * 4; e4 += kMfThreads) {
    const int e = e4 >> 2, qd = e4 & 3;
    const int i = e / (a.step + 1), c = e - i * (a.step + 1);
    const uint16_t* kp = (c == a.step) ? ks + i * kHeadDim + qd * 32
                                       : a.k_hist + (((size_t)c * a.hist_rows + anc[i * 32 + c]) * a.H + h * kHeadDim + qd * 32);
    u32x4 u[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) u[x] = *reinterpret_cast<const u32x4*>(kp + x * 8);
    const float* q = qs + i * kHeadDim + qd * 32;
    float dot = 0.f;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        dot += q[x * 8 + 2 * y] * __uint_as_float(u[x][y] << 16);
        dot += q[x * 8 + 2 * y + 1] * __uint_as_float(u[x][y] & 0xFFFF0000u);
      }
    dot += dpp_move_f32<0xB1>(dot);       // the four quarters of the key: lanes ^1, then ^2 (fixed order)
    dot += dpp_move_f32<0x4E>(dot);
    if (qd == 0) sct[(L + c) * kSeqRows + i] = dot * scale;
  }
  __syncthreads();
  // ---- softmax weights: wave w takes rows w, w + 4, ...; the prompt's weights as two bf16 halves ------------------
  for (int i = wave; i < kk; i += kMfThreads / 64) {
    float mx = -INFINITY;
    for (int j = lane; j < n_vis; j += 64) mx = fmaxf(mx, sct[j * kSeqRows + i]);
    mx = wave_max_f32(mx);
    float sum = 0.f;
    for (int j = lane; j < n_vis; j += 64) {
      const float p = __expf(sct[j * kSeqRows + i] - mx);
      sum += p;
      if (j < L) {
        const uint16_t hi = f32_to_bf16_rne(p);
        ph[i * ppitch + j] = hi;
        pl[i * ppitch + j] = f32_to_bf16_rne(p - bf16_to_f32(hi));
      } else {
        sct[j * kSeqRows + i] = p;
      }
    }
    sum = wave_sum_f32(sum);
    if (lane == 0) rsum[i] = sum;
  }
  __syncthreads();
  // ---- the prompt's part of the outputs: wave w takes d tiles 2w and 2w + 1 --------------------------------------
  {
    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    for (int st0 = 0; st0 < nstep; st0 += 8) {
      if (st0 > 0) load_values(st0);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int st = st0 + u;
        if (st >= nstep) continue;                                   // uniform
        // B operand: weights of row `row`, keys 32 st + 8 q4 .. + 7
        const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(ph + row * ppitch + st * 32 + q4 * 8));
        const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(pl + row * ppitch + st * 32 + q4 * 8));
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 af = __builtin_bit_cast(bf16x8, vf[j][u]);
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bh, acc[j], 0, 0, 0);
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bl, acc[j], 0, 0, 0);
        }
      }
    }
    // the queries are no longer needed: their place takes the outputs (accumulator e: d 4 * (lane >> 4) + e of the tile)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) qs[row * kHeadDim + (wave * 2 + j) * 16 + q4 * 4 + e] = acc[j][e];
  }
  __syncthreads();
  // ---- ancestors and the row itself, normalisation: the values of four ancestors in flight ------------------------
  {
    const int d = tid & (kHeadDim - 1);
    for (int i = tid >> 7; i < kk; i += kMfThreads / kHeadDim) {
      float o = qs[i * kHeadDim + d];
      const uint16_t* vh = a.v_hist + (size_t)h * kHeadDim + d;
      int c = 0;
      for (; c + 3 < a.step; c += 4) {
        uint16_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = vh[((size_t)(c + u) * a.hist_rows + anc[i * 32 + c + u]) * a.H];
#pragma unroll
        for (int u = 0; u < 4; ++u) o += sct[(L + c + u) * kSeqRows + i] * bf16_to_f32(v[u]);
      }
      for (; c < a.step; ++c) o += sct[(L + c) * kSeqRows + i] * bf16_to_f32(vh[((size_t)c * a.hist_rows + anc[i * 32 + c]) * a.H]);
      o += sct[(n_vis - 1) * kSeqRows + i] * bf16_to_f32(vs[i * kHeadDim + d]);
      a.o[(size_t)(r0 + i) * a.H + h * kHeadDim + d] = f32_to_bf16_rne(o / rsum[i]);
    }
  }
}

// Vt[b][e][key] = Vp[b][key][e]: one workgroup per (sequence, block of 128 elements, block of 128 keys); a thread
// writes 64 keys of one element, a whole cache line.
constexpr int kPackKeys = 128;
__global__ __launch_bounds__(256) void pack_prompt_values_kernel(const uint16_t* __restrict__ Vp, uint16_t* __restrict__ Vt,
                                                                 int H, int L, int Lp) {
  __shared__ uint16_t tile[kPackKeys][kHeadDim + 8];
  const int nhb = H / kHeadDim;
  const int b = blockIdx.x / nhb, hb = blockIdx.x % nhb, k0 = blockIdx.y * kPackKeys, tid = threadIdx.x;
  for (int c = tid; c < kPackKeys * 16; c += 256) {         // 16-byte pieces, whole rows of the cache
    const int kin = c >> 4, pc = c & 15, key = k0 + kin;
    u32x4 u = {0u, 0u, 0u, 0u};
    if (key < L) u = *reinterpret_cast<const u32x4*>(Vp + ((size_t)(b * L + key) * H + hb * kHeadDim + pc * 8));
    *reinterpret_cast<u32x4*>(&tile[kin][pc * 8]) = u;
  }
  __syncthreads();
  const int d = tid & (kHeadDim - 1), kh = tid >> 7;          // keys k0 + 64 kh .. + 63 of element d
  uint16_t* dst = Vt + ((size_t)b * H + hb * kHeadDim + d) * Lp + k0 + kh * 64;
#pragma unroll
  for (int g = 0; g < 8; ++g) {
    if (k0 + kh * 64 + g * 8 >= Lp) break;                    // Lp is a multiple of 32
    u32x4 o;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t lo = tile[kh * 64 + g * 8 + 2 * x][d], hi = tile[kh * 64 + g * 8 + 2 * x + 1][d];
      o[x] = lo | (hi << 16);
    }
    *reinterpret_cast<u32x4*>(dst + g * 8) = o;
  }
}

hipError_t launch_pack_prompt_values(const uint16_t* Vp, uint16_t* Vt, int B, int H, int L, int Lp, hipStream_t stream) {
  hipLaunchKernelGGL(pack_prompt_values_kernel, dim3(B * (H / kHeadDim), (Lp + kPackKeys - 1) / kPackKeys), dim3(256), 0,
                     stream, Vp, Vt, H, L, Lp);
  return hipGetLastError();
}

static size_t attention_seq_lds(int n_vis) {
  return (size_t)(3 * kSeqRows * kHeadDim + 8 * kSeqRows * kHeadDim + kSeqRows + kSeqRows * 32 + (size_t)n_vis * kSeqRows) *
         sizeof(float);
}

hipError_t launch_body_attention(const BodyAttnArgs& a, hipStream_t stream) {
  const int n_vis = a.L + a.step + 1;
  // batched rounds with a prompt: one workgroup per (sequence, head), the prompt part on the matrix cores
  if (a.R > kBodyRows && a.k <= kSeqRows && a.Vt != nullptr && attention_mfma_lds(a.Lp, n_vis) <= 150 * 1024) {
    static bool prepared_mf = false;
    if (!prepared_mf) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&body_attention_mfma_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
      if (e != hipSuccess) return e;
      prepared_mf = true;
    }
    const int n_seq = (a.step == 0) ? a.R : a.R / a.k;
    hipLaunchKernelGGL(body_attention_mfma_kernel, dim3(n_seq * (a.H / kHeadDim)), dim3(kMfThreads),
                       attention_mfma_lds(a.Lp, n_vis), stream, a);
    return hipGetLastError();
  }
  // ... without one (or with one too long for the LDS): the same by ordinary arithmetic
  if (a.R > kBodyRows && a.k <= kSeqRows && attention_seq_lds(n_vis) <= 150 * 1024) {
    static bool prepared = false;
    if (!prepared) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&body_attention_seq_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
      if (e != hipSuccess) return e;
      prepared = true;
    }
    const int n_seq = (a.step == 0) ? a.R : a.R / a.k;
    hipLaunchKernelGGL(body_attention_seq_kernel, dim3(n_seq * (a.H / kHeadDim)), dim3(kSeqThreads),
                       attention_seq_lds(n_vis), stream, a);
    return hipGetLastError();
  }
  const size_t lds = (size_t)(400 + 8 * kHeadDim + ((n_vis + 3) & ~3) + 32) * sizeof(float);
  hipLaunchKernelGGL(body_attention_kernel, dim3(a.R * (a.H / kHeadDim)), dim3(kAttnThreads), lds, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
