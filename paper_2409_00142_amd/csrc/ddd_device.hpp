// Device-side helpers shared by the DDD kernels: ordered keys, wave-wide reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ddd {

constexpr int kWave = 64;

// ---- ordered keys ---------------------------------------------------------------------------
// fp32 -> uint32 whose unsigned order equals the float order (-inf lowest, +inf highest).
// -0 is mapped to +0 first, so keys compare like the floats themselves.
__device__ __forceinline__ uint32_t ord32(float x) {
  uint32_t b = __float_as_uint(x + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float unord32(uint32_t o) {
  uint32_t b = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
  return __uint_as_float(b);
}
// Row top-k key: larger key = larger logit, then lower token id.  0 is "no candidate".
__device__ __forceinline__ uint64_t row_key(float logit, int token) {
  return ((uint64_t)ord32(logit) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)token);
}
__device__ __forceinline__ int key_token(uint64_t key) { return (int)(0xFFFFFFFFu - (uint32_t)key); }
__device__ __forceinline__ float key_value(uint64_t key) { return unord32((uint32_t)(key >> 32)); }
// Beam key: larger score, then lower token id (< 2^24), then lower flat index (< 256).
__device__ __forceinline__ uint64_t beam_key(float score, int token, int flat) {
  uint32_t lo = ((0xFFFFFFu - (uint32_t)token) << 8) | (uint32_t)(0xFFu - (uint32_t)flat);
  return ((uint64_t)ord32(score) << 32) | lo;
}
__device__ __forceinline__ int beam_key_flat(uint64_t key) { return (int)(0xFFu - ((uint32_t)key & 0xFFu)); }

// ---- wave-wide max of a 64-bit key ----------------------------------------------------------
// Must be called with all 64 lanes of the wave active.  Returns the maximum in every lane.
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_move_u64(uint64_t x) {
  int lo = (int)(uint32_t)x, hi = (int)(uint32_t)(x >> 32);
  lo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
  return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}
__device__ __forceinline__ uint64_t umax64(uint64_t a, uint64_t b) { return a > b ? a : b; }

__device__ __forceinline__ uint64_t readlane_u64(uint64_t x, int lane) {
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, lane);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t x) {
  x = umax64(x, dpp_move_u64<0xB1>(x));    // quad_perm [1,0,3,2]  : lane ^ 1
  x = umax64(x, dpp_move_u64<0x4E>(x));    // quad_perm [2,3,0,1]  : lane ^ 2
  x = umax64(x, dpp_move_u64<0x141>(x));   // row_half_mirror      : other quad of each 8
  x = umax64(x, dpp_move_u64<0x140>(x));   // row_mirror           : other half of each 16
  uint64_t a = readlane_u64(x, 0), b = readlane_u64(x, 16), c = readlane_u64(x, 32), d = readlane_u64(x, 48);
  return umax64(umax64(a, b), umax64(c, d));
}

__device__ __forceinline__ float wave_max_f32(float x) {
  // ord32 keeps float order, reuse the integer path on the high word
  uint64_t k = (uint64_t)ord32(x) << 32;
  return unord32((uint32_t)(wave_max_u64(k) >> 32));
}

// Sum over the wave in a fixed butterfly order (deterministic).  All lanes active.
__device__ __forceinline__ float wave_sum_f32(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

}  // namespace ddd
