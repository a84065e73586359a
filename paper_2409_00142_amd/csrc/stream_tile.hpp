// Streaming-wave building block shared by the weight-stream kernels (LM head, draft-layer
// linears): one 16-row tile of a row-major bf16 matrix against <= 16 resident input rows.
#pragma once
#include "ddd_device.hpp"

namespace ddd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kStagePitch = 272;               // 256 B of a row group + 16 B pad: conflict-free b128 reads
constexpr int kStageBytes = 16 * kStagePitch;  // one 16x128 bf16 group

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// One 16-row tile of one streaming wave: drain the register ring group by group through the
// LDS stage into MFMA operands; with REFILL each drained group is reloaded for the next tile.
template <int G, bool REFILL>
__device__ __forceinline__ f32x4 stream_tile(u32x4 (&ring)[G][4], const bf16x8 (&bfrag)[G][4], unsigned char* mystage,
                                             int wr_off, int rd_off, const uint16_t* wbase, int H, int next_row0,
                                             int vlast) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(mystage + wr_off + i * 4 * kStagePitch) = ring[g][i];
    if (REFILL) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = min(next_row0 + i * 4, vlast);
        ring[g][i] = *reinterpret_cast<const u32x4*>(wbase + (size_t)row * H + g * 128);
      }
    }
    wave_lds_fence();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32x4 u = *reinterpret_cast<const u32x4*>(mystage + rd_off + j * 64);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, u), bfrag[g][j], acc, 0, 0, 0);
    }
    wave_lds_fence();
  }
  return acc;
}

}  // namespace ddd
