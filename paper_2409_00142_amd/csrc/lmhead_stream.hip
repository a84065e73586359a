// LM-head weight stream with fused online logsoftmax statistics and per-slice top-k.
//
// Computes, for R <= 16 hidden rows, logits[r,v] = sum_h hid[r,h] * W[v,h] (bf16 in, fp32
// accumulate) for every vocabulary row v, reading W exactly once, and leaves per
// (row, slice) partial results: the slice's k best (logit, token) keys in order and
// sum_v exp(logit - slice max).  A slice is the set of tiles (of at most 16 rows) owned by one
// workgroup: every nslice-th tile of the vocabulary.  The full logits are never written unless a debug buffer is given.
//
// Workgroup = NW streaming waves + 1 epilogue wave.
//  * Streaming wave w owns the K-slice [w*KS, (w+1)*KS) of the hidden dimension, KS = 128*G.
//    Its share of the hidden rows sits in registers as MFMA B operands for the whole
//    kernel.  For each 16-row tile of W it issues fully coalesced 16-byte loads (one
//    instruction = 4 rows x 256 contiguous bytes), keeps G*4 of them in flight (a register
//    ring that always holds the next tile), transposes each 16x128 group through a private
//    LDS stage into the MFMA A layout and accumulates v_mfma_f32_16x16x32_bf16 into one
//    16x16 fp32 tile; the tile is published to LDS and the workgroup meets at a barrier.
//  * The epilogue wave sums the NW partial tiles in a fixed order (so equal W rows give
//    bit-equal logits).  Lane (vb, r) owns 4 of the 16 logits of hidden row r per tile and
//    keeps their running max, running sum of exponentials and sorted top-k list in registers
//    while the streaming waves are already loading the next tile; after the last tile the
//    four lanes of a row merge their lists through LDS.
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"
#include "stream_tile.hpp"

namespace ddd {

template <int G, int KL>
__global__ __launch_bounds__(768) void lmhead_stream_kernel(StreamArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int NW = a.nw;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  // Nothing to do if every row of this pass is inactive (uniform): one load per lane and a ballot.  Normally that
  // round trip comes first, so that a skipped call retires at once.  A caller that knows skipped calls to be rare
  // (the host-paced round queues at most one per round) sets eager_loads: the first tile of W and the hidden rows
  // are requested before the flags are looked at, and the check costs an executed call nothing.
  const bool check_late = a.row_active != nullptr && a.eager_loads != 0;
  if (a.row_active != nullptr && !a.eager_loads) {
    const int on = (lane < a.R) ? a.row_active[lane] : 0;
    if (__ballot(on != 0) == 0ull) return;
  }
  int on_late = 1;     // requested now, looked at once the first tile's requests are out
  if (check_late) on_late = (lane < a.R) ? a.row_active[lane] : 0;

  const int nslice = gridDim.x, slice = blockIdx.x;
  uint64_t* const trace = a.trace ? a.trace + (size_t)slice * kTraceStreamWords : nullptr;
  if (trace != nullptr && tid == 0) trace[0] = (uint64_t)wall_clock64();
  // The vocabulary is cut into nslice * nt tiles of equal height (V / (nslice * nt) <= 16 rows, i.e. 15 or 16
  // rows each at 32000 rows over 256 slices) and slice i owns every nslice-th tile (the column rotated by one per
  // step): every workgroup fetches the same amount, and at any time the workgroups together read one contiguous
  // window of W that moves through the matrix (against one contiguous range of rows per workgroup: 53 -> 50 us per
  // launch at the 7B shape when W comes from HBM, 64 -> 60 us at the 13B shape).  A tile's missing rows repeat its
  // last row (the same cache lines) and are masked in the epilogue.  (Workgroups with an odd index - the odd XCDs -
  // finish about 3 us after the even ones whatever they read; the timestamps of ddd_trace_read show it.)
  const int nt = (a.V + 16 * nslice - 1) / (16 * nslice);
  const long long NT = (long long)nslice * nt;
  // Sweep direction: calls alternate, so that a call starts with the part of W its predecessor read
  // last, which the memory-side cache still holds.
  auto tile_lo = [&](int t) -> int {     // first row of this slice's t-th tile in walk order
    const int u = a.reverse ? nt - 1 - t : t;
    const long long j = (long long)u * nslice + (slice + u) % nslice;
    return (int)((j * a.V) / NT);
  };
  auto tile_hi = [&](int t) -> int {
    const int u = a.reverse ? nt - 1 - t : t;
    const long long j = (long long)u * nslice + (slice + u) % nslice + 1;
    return (int)((j * a.V) / NT);
  };

  float* red = reinterpret_cast<float*>(smem);      // [2][NW][256] fp32 partial tiles
  unsigned char* stage = smem + 2 * NW * 1024;      // [NW][kStageBytes]

  if (wave < NW) {
    // ------------------------------ streaming wave ------------------------------
    const int ks = wave * (128 * G);
    const int n = lane & 15, q = lane >> 4;          // MFMA operand coordinates
    bf16x8 bfrag[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        u32x4 u = {0u, 0u, 0u, 0u};
        if (n < a.R) u = *reinterpret_cast<const u32x4*>(a.hid + (size_t)n * a.H + ks + g * 128 + j * 32 + q * 8);
        bfrag[g][j] = __builtin_bit_cast(bf16x8, u);
      }

    const int lrow = lane >> 4, c = lane & 15;       // load coordinates: 4 rows x 16 chunks per instruction
    unsigned char* mystage = stage + wave * kStageBytes;
    const int wr_off = lrow * kStagePitch + c * 16;
    const int rd_off = n * kStagePitch + q * 16;
    const uint16_t* wbase = a.W + ks + c * 8;

    u32x4 ring[G][4];
    {
      const int lo = tile_lo(0), last = tile_hi(0) - 1;   // rows are clamped to the tile
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = min(lo + i * 4 + lrow, last);
          ring[g][i] = *reinterpret_cast<const u32x4*>(wbase + (size_t)row * a.H + g * 128);
        }
    }
    if (check_late) {   // the requests above are simply dropped if nothing is active
      asm volatile("" : "+v"(on_late));   // keeps the compiler from waiting for the flags before the requests are out
      if (__ballot(on_late != 0) == 0ull) return;
    }
    // every tile but the last refills the ring with the next tile while it is consumed
    for (int t = 0; t + 1 < nt; ++t) {
      const f32x4 acc = stream_tile<G, true>(ring, bfrag, mystage, wr_off, rd_off, wbase, a.H, tile_lo(t + 1) + lrow,
                                             tile_hi(t + 1) - 1);
      *reinterpret_cast<f32x4*>(red + ((t & 1) * NW + wave) * 256 + lane * 4) = acc;
      if (trace != nullptr && t == 0 && tid == 0) trace[1] = (uint64_t)wall_clock64();
      __syncthreads();
    }
    {
      const int t = nt - 1;
      const f32x4 acc = stream_tile<G, false>(ring, bfrag, mystage, wr_off, rd_off, wbase, a.H, 0, 0);
      *reinterpret_cast<f32x4*>(red + ((t & 1) * NW + wave) * 256 + lane * 4) = acc;
      if (trace != nullptr && tid == 0) {
        if (t == 0) trace[1] = (uint64_t)wall_clock64();
        trace[2] = (uint64_t)wall_clock64();
      }
      __syncthreads();
    }
  } else {
    // ------------------------------ epilogue wave ------------------------------
    // lane = (vb, r): rows 4*vb .. 4*vb+3 of the tile for hidden row r, exactly the MFMA C layout
    if (check_late && __ballot(on_late != 0) == 0ull) return;
    const int r = lane & 15, vb = lane >> 4;
    const bool row_ok = r < a.R;
    float m_run = -INFINITY, s_run = 0.f;
    uint64_t list[KL];
#pragma unroll
    for (int j = 0; j < KL; ++j) list[j] = 0;

    for (int t = 0; t < nt; ++t) {
      __syncthreads();
      if (trace != nullptr && t == nt - 1 && lane == 0) trace[6] = (uint64_t)wall_clock64();
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < NW; ++w)   // fixed order: equal W rows give bit-equal logits
        s += *reinterpret_cast<const f32x4*>(red + ((t & 1) * NW + w) * 256 + lane * 4);
      const int v0 = tile_lo(t) + vb * 4;
      const int nv = min(4, tile_hi(t) - v0);
      if (row_ok && nv > 0) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = s[e] + 0.0f;   // -0 -> +0
        if (a.logits_dbg != nullptr) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (e < nv) a.logits_dbg[(size_t)r * a.V + v0 + e] = x[e];
        }
        float tmax = x[0];
#pragma unroll
        for (int e = 1; e < 4; ++e)
          if (e < nv) tmax = fmaxf(tmax, x[e]);
        const float m_new = fmaxf(m_run, tmax);
        float s_new = s_run * __expf(m_run - m_new);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (e < nv) s_new += __expf(x[e] - m_new);
        m_run = m_new;
        s_run = s_new;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint64_t cur = row_key(x[e], v0 + e);
          if (e < nv && cur > list[KL - 1]) {
#pragma unroll
            for (int j = 0; j < KL; ++j) {
              const bool gt = cur > list[j];
              const uint64_t hi = gt ? cur : list[j];
              cur = gt ? list[j] : cur;
              list[j] = hi;
            }
          }
        }
      }
    }

    if (trace != nullptr && lane == 0) trace[3] = (uint64_t)wall_clock64();
    // The four lanes of a hidden row merge their lists: through LDS into quads (lane' = 4*r + vb).
    // Every streaming wave has passed its last barrier, so the stage area is free.
    uint64_t* elist = reinterpret_cast<uint64_t*>(stage);            // [64][KL]
    float* estat = reinterpret_cast<float*>(stage + 64 * KL * 8);    // [64][2]
    const int slot = r * 4 + vb;
#pragma unroll
    for (int j = 0; j < KL; ++j) elist[slot * KL + j] = list[j];
    estat[slot * 2] = m_run;
    estat[slot * 2 + 1] = s_run;
    wave_lds_fence();
    const int r2 = lane >> 2;
    const bool ok2 = r2 < a.R;
    const float m_l = estat[lane * 2], s_l = estat[lane * 2 + 1];
    float m_q = fmaxf(m_l, dpp_move_f32<0xB1>(m_l));
    m_q = fmaxf(m_q, dpp_move_f32<0x4E>(m_q));
    float s_q = (s_l == 0.f) ? 0.f : s_l * __expf(m_l - m_q);
    s_q += dpp_move_f32<0xB1>(s_q);
    s_q += dpp_move_f32<0x4E>(s_q);
    if (trace != nullptr && lane == 0) trace[4] = (uint64_t)wall_clock64();
    uint64_t* pk = a.part_key + (size_t)(ok2 ? r2 : 0) * nslice * a.k + slice;   // [row][rank][slice]
    int cur = 0;
    for (int round = 0; round < a.k; ++round) {
      const uint64_t head = (cur < KL) ? elist[lane * KL + cur] : 0ull;
      uint64_t q = umax64(head, dpp_move_u64<0xB1>(head));
      q = umax64(q, dpp_move_u64<0x4E>(q));
      if (head == q && q != 0ull) ++cur;
      if (ok2 && (lane & 3) == 0) pk[(size_t)round * nslice] = q;
    }
    if (ok2 && (lane & 3) == 0) a.part_sum[(size_t)r2 * nslice + slice] = s_q;
    if (trace != nullptr && lane == 0) trace[5] = (uint64_t)wall_clock64();
  }
}

template <int G>
static hipError_t launch_g(const StreamArgs& a, int nslice, hipStream_t stream) {
  const dim3 grid(nslice), block((a.nw + 1) * 64);
  // partial tiles + per-wave stages; the stage area is reused by the epilogue's final merge (<= 8.5 KB)
  const size_t stage_bytes = (size_t)a.nw * kStageBytes > 8704 ? (size_t)a.nw * kStageBytes : 8704;
  const size_t lds = (size_t)2 * a.nw * 1024 + stage_bytes;
  if (a.k <= 4)
    hipLaunchKernelGGL((lmhead_stream_kernel<G, 4>), grid, block, lds, stream, a);
  else if (a.k <= 8)
    hipLaunchKernelGGL((lmhead_stream_kernel<G, 8>), grid, block, lds, stream, a);
  else if (a.k <= 10)
    hipLaunchKernelGGL((lmhead_stream_kernel<G, 10>), grid, block, lds, stream, a);
  else
    hipLaunchKernelGGL((lmhead_stream_kernel<G, 16>), grid, block, lds, stream, a);
  return hipGetLastError();
}

hipError_t launch_lmhead_stream(const StreamArgs& a, int G, int nslice, hipStream_t stream) {
  switch (G) {
    case 1: return launch_g<1>(a, nslice, stream);
    case 2: return launch_g<2>(a, nslice, stream);
    case 4: return launch_g<4>(a, nslice, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace ddd
