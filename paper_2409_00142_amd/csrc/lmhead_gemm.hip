// LM-head projection for more than 16 hidden rows (batched rounds): an MFMA GEMM with the same
// fused epilogue and the same partial-result format as the weight stream.
//
//   logits^T[V, R] = W[V, H] * hid^T[H, R]      (bf16 in, fp32 accumulate)
//
// Workgroup tile 128 (vocabulary rows) x 128 (hidden rows), K tile 64, 256 threads = 2 x 2 waves
// with 64 x 64 wave tiles of v_mfma_f32_32x32x16_bf16.  W is the A operand, so a lane of the
// accumulator owns one hidden row and 32 vocabulary rows per tile: the online logsoftmax
// statistics and the sorted top-k list of that (lane, row) live in registers.  Both operands
// are staged through double-buffered, padded (144-byte pitch) LDS tiles; the next K tile is
// loaded from global memory into registers while the current one is multiplied.  Two workgroups
// fit on a CU (about 74 KB of LDS, at most 256 VGPRs), so one workgroup's epilogue (vector ALU)
// overlaps the other's matrix work.
//
// A slice is a group of `tps` consecutive 128-row tiles of W; a unit of work is (slice, column
// tile).  Units are handed out so that workgroups of one XCD work on neighbouring units: the
// column tiles of one slice read the same W rows and share them through that XCD's L2, so W
// comes from HBM once.  Only active rows are multiplied: the columns are gathered through a
// compacted row list built on the device.
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"

namespace ddd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kBM = 128, kBN = 128, kBK = 64;
constexpr int kPitch = 72;                         // bf16 elements per LDS row: 64 + 8 pad
constexpr int kTileElems = 128 * kPitch;           // one operand tile
constexpr int kGemmLds = 4 * kTileElems * 2;       // A[2] + B[2], bytes

template <int KL>
__global__ __launch_bounds__(256, 2) void lmhead_gemm_kernel(GemmArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint16_t* As = reinterpret_cast<uint16_t*>(smem_raw);            // [2][128][kPitch]
  uint16_t* Bs = As + 2 * kTileElems;                              // [2][128][kPitch]

  const int n_act = *a.n_act_ptr;
  if (n_act <= 0) return;                                          // uniform
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave & 1, wn = wave >> 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const int NT = (n_act + kBN - 1) / kBN;
  const int nunits = a.nslice * NT;
  const int G = gridDim.x;
  const int vg = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);  // neighbours on one XCD get neighbouring units
  const int KT = a.H / kBK;
  const int ld_row = tid >> 3, ld_cc = tid & 7;                    // global->LDS copy coordinates

  for (int u = vg; u < nunits; u += G) {
    const int slice = u / NT, nt = u - slice * NT;
    const int mt0 = slice * a.tps, mt1 = min(a.nmt, mt0 + a.tps);

    const uint16_t* brow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = min(nt * kBN + ld_row + 32 * i, n_act - 1);
      brow[i] = a.hid + (size_t)a.row_list[n] * a.H + ld_cc * 8;
    }
    // per (lane, column block): hidden row, running max / sum, sorted top-k list
    int orow[2];
    bool rvalid[2];
    float m_run[2], s_run[2];
    uint64_t list[2][KL];
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
      const int n = nt * kBN + wn * 64 + bn * 32 + l32;
      rvalid[bn] = n < n_act;
      orow[bn] = a.row_list[min(n, n_act - 1)];
      m_run[bn] = -INFINITY;
      s_run[bn] = 0.f;
#pragma unroll
      for (int j = 0; j < KL; ++j) list[bn][j] = 0ull;
    }

    for (int mt = mt0; mt < mt1; ++mt) {
      const uint16_t* arow[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = min(mt * kBM + ld_row + 32 * i, a.V - 1);
        arow[i] = a.W + (size_t)v * a.H + ld_cc * 8;
      }
      f32x16 acc[2][2];
#pragma unroll
      for (int bm = 0; bm < 2; ++bm)
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0.f;

      u32x4 ra[4], rb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[i] = *reinterpret_cast<const u32x4*>(arow[i]);
        rb[i] = *reinterpret_cast<const u32x4*>(brow[i]);
      }
      __syncthreads();   // every wave is done with both LDS buffers (previous tile / final merge)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4*>(As + (ld_row + 32 * i) * kPitch + ld_cc * 8) = ra[i];
        *reinterpret_cast<u32x4*>(Bs + (ld_row + 32 * i) * kPitch + ld_cc * 8) = rb[i];
      }
      __syncthreads();

      for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        const bool more = (kt + 1 < KT);
        if (more) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            ra[i] = *reinterpret_cast<const u32x4*>(arow[i] + (kt + 1) * kBK);
            rb[i] = *reinterpret_cast<const u32x4*>(brow[i] + (kt + 1) * kBK);
          }
        }
        const uint16_t* Ab = As + buf * kTileElems + (wm * 64 + l32) * kPitch + lh * 8;
        const uint16_t* Bb = Bs + buf * kTileElems + (wn * 64 + l32) * kPitch + lh * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          bf16x8 af[2], bf[2];
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            af[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Ab + b * 32 * kPitch + ks * 16));
            bf[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bb + b * 32 * kPitch + ks * 16));
          }
#pragma unroll
          for (int bm = 0; bm < 2; ++bm)
#pragma unroll
            for (int bn = 0; bn < 2; ++bn)
              acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[bm], bf[bn], acc[bm][bn], 0, 0, 0);
        }
        if (more) {
          uint16_t* Aw = As + (buf ^ 1) * kTileElems;
          uint16_t* Bw = Bs + (buf ^ 1) * kTileElems;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<u32x4*>(Aw + (ld_row + 32 * i) * kPitch + ld_cc * 8) = ra[i];
            *reinterpret_cast<u32x4*>(Bw + (ld_row + 32 * i) * kPitch + ld_cc * 8) = rb[i];
          }
        }
        __syncthreads();
      }

      // ---- epilogue of this tile: accumulator element e of block (bm, bn) is
      //      vocabulary row vbase + bm*32 + (e/4)*8 + lh*4 + e%4, hidden-row column l32
      const int vbase = mt * kBM + wm * 64 + lh * 4;
#pragma unroll
      for (int bn = 0; bn < 2; ++bn) {
        if (!rvalid[bn]) continue;
        float tmax = -INFINITY;
#pragma unroll
        for (int bm = 0; bm < 2; ++bm)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int v = vbase + bm * 32 + (e >> 2) * 8 + (e & 3);
            const float x = acc[bm][bn][e] + 0.0f;   // -0 -> +0
            acc[bm][bn][e] = x;
            if (v < a.V) tmax = fmaxf(tmax, x);
          }
        if (a.logits_dbg != nullptr) {
#pragma unroll
          for (int bm = 0; bm < 2; ++bm)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const int v = vbase + bm * 32 + (e >> 2) * 8 + (e & 3);
              if (v < a.V) a.logits_dbg[(size_t)orow[bn] * a.V + v] = acc[bm][bn][e];
            }
        }
        const float m_new = fmaxf(m_run[bn], tmax);
        float s_new = (s_run[bn] == 0.f) ? 0.f : s_run[bn] * __expf(m_run[bn] - m_new);
        float tail = key_value(list[bn][KL - 1]);
        const bool full0 = list[bn][KL - 1] != 0ull;
        bool full = full0;
#pragma unroll
        for (int bm = 0; bm < 2; ++bm)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int v = vbase + bm * 32 + (e >> 2) * 8 + (e & 3);
            const float x = acc[bm][bn][e];
            if (v < a.V) {
              s_new += __expf(x - m_new);
              if (!full || x >= tail) {
                uint64_t cur = row_key(x, v);
                if (cur > list[bn][KL - 1]) {
#pragma unroll
                  for (int j = 0; j < KL; ++j) {
                    const bool gt = cur > list[bn][j];
                    const uint64_t hi = gt ? cur : list[bn][j];
                    cur = gt ? list[bn][j] : cur;
                    list[bn][j] = hi;
                  }
                  full = list[bn][KL - 1] != 0ull;
                  tail = key_value(list[bn][KL - 1]);
                }
              }
            }
          }
        m_run[bn] = m_new;
        s_run[bn] = s_new;
      }
    }

    // ---- end of the slice: the four (wave, half) owners of a hidden row merge through LDS ----
    __syncthreads();
    uint64_t* elist = reinterpret_cast<uint64_t*>(smem_raw);                       // [128][4][KL]
    float* estat = reinterpret_cast<float*>(smem_raw + (size_t)128 * 4 * KL * 8);  // [128][4][2]
    const int src = wm * 2 + lh;
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
      const int rl = wn * 64 + bn * 32 + l32;
#pragma unroll
      for (int j = 0; j < KL; ++j) elist[(rl * 4 + src) * KL + j] = list[bn][j];
      estat[(rl * 4 + src) * 2] = m_run[bn];
      estat[(rl * 4 + src) * 2 + 1] = s_run[bn];
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int rl = pass * 64 + (tid >> 2);          // quad = one hidden row, lane in quad = source
      const int n = nt * kBN + rl;
      const bool ok = n < n_act;
      const int row = a.row_list[min(n, n_act - 1)];
      const int slot = rl * 4 + (tid & 3);
      const float m_l = estat[slot * 2], s_l = estat[slot * 2 + 1];
      float m_q = fmaxf(m_l, dpp_move_f32<0xB1>(m_l));
      m_q = fmaxf(m_q, dpp_move_f32<0x4E>(m_q));
      float s_q = (s_l == 0.f) ? 0.f : s_l * __expf(m_l - m_q);
      s_q += dpp_move_f32<0xB1>(s_q);
      s_q += dpp_move_f32<0x4E>(s_q);
      uint64_t* pk = a.part_key + ((size_t)row * a.nslice + slice) * a.k;
      int cur = 0;
      for (int round = 0; round < a.k; ++round) {
        const uint64_t head = (cur < KL) ? elist[slot * KL + cur] : 0ull;
        uint64_t q = umax64(head, dpp_move_u64<0xB1>(head));
        q = umax64(q, dpp_move_u64<0x4E>(q));
        if (head == q && q != 0ull) ++cur;
        if (ok && (tid & 3) == 0) pk[round] = q;
      }
      if (ok && (tid & 3) == 0) a.part_sum[(size_t)row * a.nslice + slice] = s_q;
    }
    // the next unit starts with a barrier before it touches LDS
  }
}

// ---- compaction of the active rows ------------------------------------------------------------
__global__ __launch_bounds__(1024) void build_row_list_kernel(const uint8_t* row_active, int n_rows, int32_t* row_list,
                                                              int32_t* n_act) {
  __shared__ int wave_cnt[16];
  __shared__ int base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base = 0;
  __syncthreads();
  for (int r0 = 0; r0 < n_rows; r0 += 1024) {
    const int r = r0 + tid;
    const bool on = (r < n_rows) && (row_active == nullptr || row_active[r] != 0);
    const unsigned long long m = __ballot(on);
    if (lane == 0) wave_cnt[wave] = __popcll(m);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; ++w) off += wave_cnt[w];
    if (on) row_list[off + __popcll(m & ((1ull << lane) - 1ull))] = r;
    __syncthreads();
    if (tid == 0) {
      int t = 0;
      for (int w = 0; w < 16; ++w) t += wave_cnt[w];
      base += t;
    }
    __syncthreads();
  }
  if (tid == 0) *n_act = base;
}

hipError_t launch_build_row_list(const uint8_t* row_active, int n_rows, int32_t* row_list, int32_t* n_act,
                                 hipStream_t stream) {
  hipLaunchKernelGGL(build_row_list_kernel, dim3(1), dim3(1024), 0, stream, row_active, n_rows, row_list, n_act);
  return hipGetLastError();
}

template <int KL>
static hipError_t prepare_kl() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_gemm_kernel<KL>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
}

hipError_t prepare_lmhead_gemm(int k) {
  if (k <= 4) return prepare_kl<4>();
  if (k <= 8) return prepare_kl<8>();
  if (k <= 10) return prepare_kl<10>();
  return prepare_kl<16>();
}

hipError_t launch_lmhead_gemm(const GemmArgs& a, int grid, hipStream_t stream) {
  const dim3 g(grid), b(256);
  if (a.k <= 4)
    hipLaunchKernelGGL((lmhead_gemm_kernel<4>), g, b, kGemmLds, stream, a);
  else if (a.k <= 8)
    hipLaunchKernelGGL((lmhead_gemm_kernel<8>), g, b, kGemmLds, stream, a);
  else if (a.k <= 10)
    hipLaunchKernelGGL((lmhead_gemm_kernel<10>), g, b, kGemmLds, stream, a);
  else
    hipLaunchKernelGGL((lmhead_gemm_kernel<16>), g, b, kGemmLds, stream, a);
  return hipGetLastError();
}

}  // namespace ddd
