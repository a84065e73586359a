/*
 * ddd_synth.h - synthetic stand-ins for the two models the draft round talks to.
 *
 * These are workload generators for tests and the benchmark, not part of the method, and they
 * are built into a shared object of their own (libddd_synth.so, linked against libddd.so):
 * the paper's draft body is EAGLE's trained layer and its target is a Vicuna / LLaMA2
 * model (Section 3.1); neither is available, so a counter-based pseudo-Gaussian hidden
 * state and a hashed target argmax take their place on the device.  The recipe is the
 * one documented with the seeded input generators: SplitMix64 finaliser keys per
 * (seed, sequence, round) and per (parent node, token); each element sums the four
 * 16-bit fields of one mixed word, is centred, converted to fp32, multiplied by
 * gain*(1+0.3*depth)/(65536/sqrt(3)), optionally shifted by a planted direction and
 * rounded to bf16 (RNE).
 */
#ifndef DDD_SYNTH_H_
#define DDD_SYNTH_H_

#include "ddd.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ddd_synth_params {
  ddd_config cfg;
  uint64_t seed;
  const int64_t* round_ctr;   /* device int64[1]: current round id (read on the device)          */
  int32_t root_token;
  int32_t n_plant;            /* rows of plant_dir, 0 = no planting                              */
  float scale_depth[32];      /* fp32 scale for depth d, computed by the caller                  */
  const float* plant_dir;     /* device fp32[n_plant,H] or NULL                                  */
  uint32_t plant_round_p24;   /* a round is planted if its 24-bit hash is below this             */
  uint32_t plant_row_p24;     /* a row is planted if its 24-bit hash is below this               */
} ddd_synth_params;

/* ddd_draft_body_fn: user = const ddd_synth_params* (host memory that outlives the call). */
int ddd_synth_draft_body(void* user, int32_t step, const ddd_state* st, void* hid_out_bf16, void* stream);

/* Hashed target argmax for every tree node: device int32[B,m+1] (padding = -1). */
int ddd_synth_target_argmax(const ddd_synth_params* p, const ddd_state* st, const ddd_tree* tree,
                            int32_t* target_argmax, void* stream);

/* Adds 1 to *round_ctr on the device (enqueued; lets a captured round advance its own id). */
int ddd_synth_next_round(int64_t* round_ctr, void* stream);

/* tokens[i] = hash(seed, *round_ctr, i) mod V for i < n <= 1024 (device int32[n]): varies the last prompt
 * token of every sequence from round to round when the draft body is the stand-in layer. */
int ddd_synth_hash_tokens(const int64_t* round_ctr, int32_t* tokens, int32_t n, int32_t V, uint64_t seed, void* stream);

/* End-of-round statistics kept on the device (no host synchronisation): for every sequence
 * depth_hist[steps[b]] += 1 and accept_hist[accept_len[b]] += 1, and once per round
 * batch_depth_hist[max_b steps[b]] += 1 (the draft calls the batch executed); device int64[32]
 * each, any may be NULL; then *round_ctr += 1. */
int ddd_synth_round_stats(int64_t* round_ctr, const int32_t* steps, const int32_t* accept_len, int32_t B,
                          int64_t* depth_hist, int64_t* accept_hist, int64_t* batch_depth_hist, void* stream);

/* ddd_post_fn that runs the stand-in target and the accept walk in one host call: ddd_synth_target_argmax,
 * ddd_verify_accept, ddd_synth_round_stats (left out if its three histograms are all NULL: the round counter must
 * then advance by other means, e.g. as the `rounds` word of statistics bound to the context with ddd_stats_bind,
 * which the accept walk's own launch keeps) and, if hash_tokens is not NULL, ddd_synth_hash_tokens on it.
 * user = const ddd_synth_post_args* (host memory that outlives the call); every pointer inside is device memory
 * except params and ctx. */
typedef struct ddd_synth_post_args {
  const ddd_synth_params* params;
  ddd_ctx* ctx;
  int32_t* target_argmax;     /* [B,m+1] */
  int32_t* accept_len;        /* [B] */
  int32_t* accept_path;       /* [B,max_depth+1] */
  int32_t* bonus_token;       /* [B] */
  int64_t* depth_hist;        /* [32] or NULL */
  int64_t* accept_hist;       /* [32] or NULL */
  int64_t* batch_depth_hist;  /* [32] or NULL */
  int32_t* hash_tokens;       /* [B] or NULL */
} ddd_synth_post_args;
int ddd_synth_post(void* user, const ddd_state* st, const ddd_tree* tree, void* stream);

/* Plain coalesced read of n_bytes (multiple of 16) into a 4-byte checksum: the practical
 * HBM read ceiling the weight stream is compared with. */
int ddd_synth_read_stream(const void* src, size_t n_bytes, uint32_t* sink, int32_t n_blocks, void* stream);

/* Register-resident loop of bf16 32x32x16 MFMAs on pseudo-random operands, no memory traffic:
 * n_blocks workgroups of 4 waves, each wave issues iters * 8 MFMAs (32768 flop each).  The
 * practical matrix-core ceiling the batched LM-head GEMM is compared with.  sink: device fp32[1]. */
int ddd_synth_mfma_rate(float* sink, int32_t iters, int32_t n_blocks, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DDD_SYNTH_H_ */
