// Host-visible argument blocks and launchers of the DDD kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ddd.h"

namespace ddd {

// Device-timestamp trace (measurement aid, off unless the context enables it): 100 MHz wall-clock stamps.
// Weight stream, per workgroup: entry, first tile multiplied, last tile multiplied, last tile folded into the
// row statistics, the lanes' lists exchanged, partial results written; two unused.
// Bookkeeping, workgroup 0: entry, slice keys arrived, rows merged, beam and stop test done, tree done, exit.
constexpr int kTraceStreamWords = 8;
constexpr int kTraceStepWords = 8;
constexpr int kTraceCallWords = DDD_STATIC_SLICES * kTraceStreamWords + kTraceStepWords;   // one draft call

// ---- LM-head MFMA GEMM for more than 16 rows (lmhead_gemm.hip) --------------------------------
struct GemmArgs {
  const uint16_t* W;          // bf16 [V,H]
  const uint16_t* Wp;         // null, or the tile-major copy of W written by launch_pack_weights
  const uint16_t* hid;        // bf16 [rows,H]
  const int32_t* row_list;    // [n_act] ids of the active rows, ascending
  const int32_t* n_act_ptr;   // device scalar
  float* logits;              // fp32 [rows][V]: written for the active rows
  float* grp_max;             // fp32 [rows][ngrp]: max of each group of 64 consecutive vocabulary rows ...
  float* grp_sum;             // fp32 [rows][ngrp]: ... and sum of exp(logit - that max); ngrp = ceil(V/64) rounded up to 4
  int H, V, ngrp;
  int reverse;                // hand the row tiles of W out from the last to the first
  // What happens to the sums (the same product serves the draft layer's linears: W = a weight matrix [N = V][K = H],
  // hid = the input rows, logits = y).  kGemmLogits needs grp_max / grp_sum; the other modes ignore them.
  int epi;                    // GemmEpilogue
  uint16_t* out16;            // bf16 [rows][ld16]: the activations (kGemmSiluPairs), or null / the rounded result (kGemmAccumulate)
  uint16_t* out16b;           // null, or a second copy of out16 (kGemmAccumulate)
  int ld16;
};
enum GemmEpilogue {
  kGemmLogits = 0,       // logits = sum, plus max and sum of exponentials of every group of 64 vocabulary rows
  kGemmStore = 1,        // y = sum
  kGemmAccumulate = 2,   // y += sum; out16 / out16b (if not null) = bf16(y)
  kGemmSiluPairs = 3     // rows of W come in (gate_i, up_i) pairs: out16[r][i] = bf16(silu(gate) * up); y unused
};
hipError_t prepare_lmhead_gemm();   // once per process: enables the kernels' LDS sizes
// max_rows: the largest number of rows this call can have (picks the tile shape)
hipError_t launch_lmhead_gemm(const GemmArgs& a, int max_rows, int grid, hipStream_t stream);
// The same kernel for a linear of the draft layer: the tile shape is picked so that the launch has about as many
// work units as workgroups (N = a.V is a few thousand rows, not a vocabulary).
hipError_t launch_gemm_linear(const GemmArgs& a, int max_rows, int grid, hipStream_t stream);
// Tile-major copy of W for the GEMM: blocks of 256 vocabulary rows x 64 k, each 32 KB contiguous
// ([row in block][64 bf16]), blocks ordered (row block, k block); rows past V repeat row V-1.
// Wp holds ceil(V/256)*256*H elements.
hipError_t launch_pack_weights(const uint16_t* W, uint16_t* Wp, int V, int H, hipStream_t stream);
hipError_t launch_build_row_list(const uint8_t* row_active, int n_rows, int32_t* row_list, int32_t* n_act,
                                 hipStream_t stream);

// Row reduction of materialised logits: lse and top-k keys of every active row, in the "dense"
// partial format part_key[row][k] (final keys in order), part_sum[row] = lse.
struct RowTopkArgs {
  const float* logits;        // fp32 [n_rows][V]
  const float* grp_max;       // fp32 [n_rows][ngrp] per-group statistics written by the GEMM
  const float* grp_sum;
  const uint8_t* row_active;  // [n_rows] or null
  uint64_t* part_key;         // [n_rows][k]
  float* part_sum;            // [n_rows]
  int n_rows, V, k, ngrp;
};
hipError_t launch_row_topk(const RowTopkArgs& a, hipStream_t stream);

// ---- per-row merge, beam select, stop test (bookkeep.hip) -------------------------------------
// nslice == 0 selects the dense format above (nothing to merge).
struct MergeArgs {
  const uint64_t* part_key;   // [n_rows][k][nslice]: rank j of every slice together (the merge reads ranks 0..2)
  const float* part_sum;      // [n_rows][nslice]
  const uint8_t* row_active;  // [n_rows] or null
  int32_t* topk_token;        // [n_rows,k]
  float* topk_logprob;        // [n_rows,k]
  float* lse;                 // [n_rows]
  int n_rows, nslice, k;
};
hipError_t launch_merge(const MergeArgs& a, hipStream_t stream);

struct BeamArgs {
  ddd_state st;
  const int32_t* topk_token;  // [B] or [B*k] rows of k
  const float* topk_logprob;
  int B, k, D, nmax, step;
  float threshold;
  uint32_t check_mask;
};
hipError_t launch_beam_select(const BeamArgs& a, hipStream_t stream);
hipError_t launch_depth_continue(const BeamArgs& a, int steps_done, hipStream_t stream);

struct StepArgs {             // merge + beam select + stop test in one launch
  BeamArgs beam;              // topk_* unused
  const uint64_t* part_key;   // [B*k][k][nslice]
  const float* part_sum;
  float* lse_dbg;             // [B*k] or null: lse of every merged row
  ddd_tree tree;              // tree.mask == null: do not build the final tree here
  int nslice, m;
  uint32_t* call_count;       // null, or this call's arrival word (device): the last workgroup to arrive ...
  uint32_t* progress;         //   ... reports (round_tag << 2) | 2 | (some sequence still active) to this word in host
  uint32_t round_tag;         //       memory (if progress is not null), and
  uint64_t* active_mask;      //   ... if not null ([ceil(B/64)] device words, zero between calls: bit b = sequence b goes
  int32_t* next_row_list;     //       on) writes the next call's list of active rows b*k+i, ascending, and their
  int32_t* next_n_act;        //       number: what build_row_list_kernel would make of row_active after this launch
  uint64_t* trace;            // null, or [kTraceStepWords] device words: wall-clock stamps of workgroup 0's phases
};
hipError_t launch_step_bookkeep(const StepArgs& a, hipStream_t stream);

// ---- LM-head weight stream (lmhead_stream.hip) ------------------------------------------------
struct StreamArgs {
  const uint16_t* W;          // bf16 [V,H]
  const uint16_t* hid;        // bf16 [R,H], first row of this pass
  const uint8_t* row_active;  // [R] or null
  uint64_t* part_key;         // [R][k][nslice], first row of this pass
  float* part_sum;            // [R][nslice]
  float* logits_dbg;          // fp32 [R][V] or null
  int H, V, R, k, ntiles, nw;
  int reverse;                // walk every slice's tiles from the last to the first
  int eager_loads;            // request the first tile of W before the row flags are known (skipped calls are rare)
  uint64_t* trace;            // null, or [nslice][kTraceStreamWords] device words: wall-clock stamps of every workgroup
};
// G = 128-wide K groups per streaming wave (1, 2 or 4); H == 128 * G * nw.
hipError_t launch_lmhead_stream(const StreamArgs& a, int G, int nslice, hipStream_t stream);

// ---- wide beams, DDD_KMAX < k <= DDD_KWIDE_MAX (wide.hip) ---------------------------------------
// One workgroup per sequence; the k*k candidate keys sit in LDS and the new beam is found by a
// radix select.  Candidates come either as dense keys + lse (rows through the GEMM path) or as
// the top-k token / logprob arrays of the stand-alone call.
struct WideStepArgs {
  BeamArgs beam;
  const uint64_t* part_key;   // [rows][k] final keys in order, or null: use beam.topk_token / topk_logprob
  const float* part_lse;      // [rows] lse of each row (with part_key)
  float* lse_dbg;             // [rows] or null
  ddd_tree tree;              // tree.mask == null: do not build the final tree here
  int m;
  int do_select;              // run the beam update
  int do_stop;                // run the stop test (steps_done = beam.step + 1 after a beam update)
  int steps_done;             // draft calls made so far, for a stop test without a beam update
  uint32_t* call_count;       // null, or this call's arrival word: the last workgroup to arrive reports
  uint32_t* progress;         //   (round_tag << 2) | 2 | (some sequence still active) to this word in host memory
  uint32_t round_tag;
};
hipError_t prepare_wide();    // once per process: enables the kernels' LDS sizes
hipError_t launch_step_wide(const WideStepArgs& a, hipStream_t stream);

// Fills `bytes` (a multiple of 4) bytes with 0xFF: the context's scratch before a round when
// DDD_FLAG_POISON_SCRATCH is set (a kernel, not a memset node, so that it can be captured into a graph).
hipError_t launch_poison(void* p, size_t bytes, hipStream_t stream);

struct ResetArgs {
  ddd_state st;
  const int32_t* root_token;  // [B] or null
  int B, k, nmax;
};
hipError_t launch_round_reset(const ResetArgs& a, hipStream_t stream);

// ---- final tree and accept walk (tree.hip) ----------------------------------------------------
struct FinalizeArgs {
  ddd_state st;
  ddd_tree tree;
  int B, k, m, nmax;
};
hipError_t launch_tree_finalize(const FinalizeArgs& a, hipStream_t stream);
hipError_t launch_tree_finalize_wide(const FinalizeArgs& a, hipStream_t stream);   // pools beyond DDD_POOL_MAX

// Round statistics a verify launch adds to (all null: none kept).
struct StatsArgs {
  int64_t* rounds;
  int64_t* depth_hist;        // [32]
  int64_t* accept_hist;       // [32]
  int64_t* batch_depth_hist;  // [32]
  const int32_t* steps;       // [B] or null
  uint32_t* sync;             // device [2], zero between launches: arrivals, deepest sequence so far
};

struct VerifyArgs {
  ddd_tree tree;
  StatsArgs stats;
  const int32_t* target_argmax;  // [B,m+1]
  int32_t* accept_len;           // [B]
  int32_t* accept_path;          // [B,D+1]
  int32_t* bonus_token;          // [B]
  int B, m, D;
};
hipError_t launch_verify_accept(const VerifyArgs& a, hipStream_t stream);

struct VerifySampleArgs {
  ddd_tree tree;
  StatsArgs stats;
  const float* logits;           // fp32 [B,m+1,V]: the target model's logits after every tree node
  const double* u_accept;        // [B,m+1] uniforms in [0,1): acceptance test of each tree node
  const double* u_bonus;         // [B,m+1] uniforms in [0,1): bonus draw at each tree node
  int32_t* accept_len;           // [B]
  int32_t* accept_path;          // [B,D+1]
  int32_t* bonus_token;          // [B]
  float temperature;
  int B, m, D, V;
};
hipError_t launch_verify_sample(const VerifySampleArgs& a, hipStream_t stream);

// Tree attention over the final tree's mask (tree_attn.hip); heads of 128.
struct TreeAttnArgs {
  const uint16_t* q;          // bf16 [B][T][nh][128]   T = m + 1 tree indices
  const uint16_t* k_tree;     // bf16 [B][T][nh][128]
  const uint16_t* vt_tree;    // bf16 [B][nh][128][Tp]  values transposed, Tp = T rounded up to 32, padding zero
  const uint16_t* k_prompt;   // bf16 [B][nh][ceil(L/32)][8][64][8]  prompt keys in fragment order (launch_kv_pack)
  const uint16_t* v_prompt;   // bf16, the same shape: prompt values in fragment order
  const uint8_t* mask;        // [B][T][T]
  const int32_t* n_sel;       // [B]
  float* part;                // workspace: [B][nh][query tiles][nsplit][tree_attention_part_floats()]
  float* out;                 // fp32 [B][T][nh][128]
  int B, T, nh, L, Tp, nsplit;
};
hipError_t prepare_tree_attention();
// k, v: bf16 [B][L][nh][128] -> the fragment-order cache the attention reads (each ceil(L/32)*32*nh*128*B elements)
hipError_t launch_kv_pack(const uint16_t* k, const uint16_t* v, uint16_t* kp, uint16_t* vp, int B, int L, int nh,
                          hipStream_t stream);
size_t tree_attention_part_floats();
hipError_t launch_tree_attention(const TreeAttnArgs& a, hipStream_t stream);

}  // namespace ddd
