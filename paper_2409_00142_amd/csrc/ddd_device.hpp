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
// All of these must be called with all 64 lanes of the wave active; the result is the same in
// every lane.  The cross-lane steps are DPP moves (quad swaps, half-row and row mirrors), the
// four rows are combined through readlane.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u32(uint32_t x) {
  // every pattern used here has a valid source lane, so bound_ctrl never takes effect
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)x, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_move_u64(uint64_t x) {
  return ((uint64_t)dpp_move_u32<CTRL>((uint32_t)(x >> 32)) << 32) | dpp_move_u32<CTRL>((uint32_t)x);
}
template <int CTRL>
__device__ __forceinline__ float dpp_move_f32(float x) {
  return __uint_as_float(dpp_move_u32<CTRL>(__float_as_uint(x)));
}
__device__ __forceinline__ uint64_t umax64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umax32(uint32_t a, uint32_t b) { return a > b ? a : b; }

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
  x = umax32(x, dpp_move_u32<0xB1>(x));    // quad_perm [1,0,3,2]  : lane ^ 1
  x = umax32(x, dpp_move_u32<0x4E>(x));    // quad_perm [2,3,0,1]  : lane ^ 2
  x = umax32(x, dpp_move_u32<0x141>(x));   // row_half_mirror      : other quad of each 8
  x = umax32(x, dpp_move_u32<0x140>(x));   // row_mirror           : other half of each 16
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0);
  const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32);
  const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  return umax32(umax32(a, b), umax32(c, d));
}

// Max of 64-bit keys as two 32-bit reductions: the high words first, then the low words of the
// lanes that hold the maximal high word.  Valid keys have a non-zero low word; 0 means "none".
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t x) {
  const uint32_t hi = (uint32_t)(x >> 32), lo = (uint32_t)x;
  const uint32_t M = wave_max_u32(hi);
  const uint32_t L = wave_max_u32(hi == M ? lo : 0u);
  return ((uint64_t)M << 32) | L;
}

__device__ __forceinline__ float wave_max_f32(float x) { return unord32(wave_max_u32(ord32(x))); }

// Sum over the wave in a fixed butterfly order (deterministic).  All lanes active.
__device__ __forceinline__ float wave_sum_f32(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

}  // namespace ddd
