// Kernels of the stand-in draft layer (an EAGLE-shaped body with synthetic weights: embedding
// gather + FC, one decoder layer with tree attention over the beam's ancestors); host launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ddd {

constexpr int kBodyRows = 16;      // most rows of a call that go through the weight stream (one pass); more: MFMA GEMM
constexpr int kHeadDim = 128;

// y[r][n] (+)= sum_k x[r][k] * W[n][k] over up to three K ranges of 128*G*nw elements each: the LM
// head's weight stream with a plain store epilogue.
enum LinearMode {
  kLinearStore = 0,        // y = sum
  kLinearAccumulate = 1,   // y += sum
  kLinearSiluPairs = 2     // rows of W come in (gate_i, up_i) pairs: out16[r][i] = bf16(silu(gate) * up), y unused
};
// Where input row n of a linear comes from (the rows of [E[token], parent feature] are read in place).
enum GatherMode {
  kGatherNone = 0,     // source row n
  kGatherIndex = 1,    // source row idx[n]                              (embedding row of the row's token)
  kGatherInBlock = 2,  // source row (n / gk) * gk + idx[n]              (parent slot inside the sequence's block of gk rows)
  kGatherBlock = 3     // source row n / gk                              (the single row of the sequence's prompt call)
};
// One K range of a product: where its weights start and where its input rows come from.
struct LinearRange {
  const uint16_t* W;          // bf16, first element of the range in row 0 (row pitch LinearArgs::ldw)
  const uint16_t* x;          // bf16 source rows, first element of the range, row pitch ldx
  const int32_t* gather_idx;  // see GatherMode
  int gather_mode, ldx;
};
constexpr int kLinearRanges = 3;
// One launch covers n_ranges K ranges of the same length 128*G*nw and adds them up in order before
// the epilogue runs: y (+)= sum_ranges x_range W_range^T.
struct LinearArgs {
  LinearRange rg[kLinearRanges];
  int n_ranges, gather_k;
  const uint8_t* row_active;  // [R] or null: the launch does nothing if every row is inactive
  float* y;                   // fp32 [R], row pitch ldy
  uint16_t* out16;            // null, or bf16 [R] with row pitch ld16: the rounded result (modes 0/1), the activations (mode 2)
  uint16_t* out16b;           // null, or a second copy of out16 (same pitch)
  int ldw, ldy, ld16, N, R, ntiles, nw, mode;
};
hipError_t launch_linear_stream(const LinearArgs& a, int G, int nslice, hipStream_t stream);

// out[r] = bf16( x[r] / sqrt(mean(x[r]^2) + eps) * g )
struct RmsNormArgs {
  const float* x;             // fp32 [R][H]
  const float* g;             // fp32 [H]
  const uint8_t* row_active;
  uint16_t* out;              // bf16 [R][H]
  int H, R;
};
hipError_t launch_rmsnorm(const RmsNormArgs& a, hipStream_t stream);

// RoPE of q and k at position L + step, k and v stored as bf16, attention of every row over the
// prompt, its ancestors and itself.
struct BodyAttnArgs {
  const float* qkv;           // fp32 [R][3H]
  const uint16_t* Kp;         // bf16 [B][L][H] keys of the prompt (as cached)
  const uint16_t* Vp;
  uint16_t* k_hist;           // bf16 [D][hist_rows][H]
  uint16_t* v_hist;
  int32_t* par_hist;          // [D][hist_rows] parent slot of every row of every call; this call's row is written here
  const int32_t* beam_parent_slot;   // [B*k] of the current beam (read for step >= 1)
  const uint8_t* row_active;
  uint16_t* o;                // bf16 [R][H]
  int H, L, k, step, R;
  int hist_rows;              // rows per call in the histories (B*k)
  const uint16_t* Vt;         // null, or bf16 [B][H][Lp]: the prompt's values with the keys of one element contiguous
  int Lp;                     // L rounded up to a multiple of 32 (the keys past L are zero)
};
hipError_t launch_body_attention(const BodyAttnArgs& a, hipStream_t stream);
// Vt[b][e][key] = Vp[b][key][e] for key < L, 0 up to Lp (the A operand of the batched attention's second contraction).
hipError_t launch_pack_prompt_values(const uint16_t* Vp, uint16_t* Vt, int B, int H, int L, int Lp, hipStream_t stream);

// Input rows of the FC for calls that go through the MFMA GEMM: x0[r] = [E[token of r], feature of r's parent],
// assembled once (the GEMM gathers whole rows of one matrix).
struct PackX0Args {
  const uint16_t* E;          // bf16 [V][H]
  const int32_t* token;       // [R] token of every row (root tokens for the prompt call)
  const uint16_t* feat;       // bf16 feature rows of the previous call (f_root for the prompt call), row pitch H
  const int32_t* parent_slot; // [R] or null
  const uint8_t* row_active;  // [R] or null
  uint16_t* x0;               // bf16 [R][2H]
  int H, k, R;
  int feat_mode;              // GatherMode of the feature row: kGatherNone (prompt call), kGatherBlock, kGatherInBlock
};
hipError_t launch_pack_x0(const PackX0Args& a, hipStream_t stream);

}  // namespace ddd
