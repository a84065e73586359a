/*
 * ddd.h - C ABI of the MI355X (gfx950) Dynamic Depth Decoding draft-round library.
 *
 * The library implements the hot path of DDD (arXiv 2409.00142): the EAGLE-2 style
 * beam-search draft round of Section 1 made variable-depth by the confidence test of
 * Section 2 (Eq. 1, Algorithm 1), the final draft tree with its attention mask
 * (Section 1, EAGLE paragraph) and the temperature-0 accept walk (Section 1,
 * speculative-decoding paragraph; Section 3.1).
 *
 * Conventions for every entry point
 *  - All buffers named "device" are caller-owned HIP device memory on the current
 *    device; the library never frees or reallocates them.  The context owns only
 *    its own scratch (per-slice partial results) and an optional captured graph.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every
 *    call only enqueues work; none synchronises with the host.
 *  - Return value: 0 (DDD_OK) or a negative ddd_status.  Arguments are validated
 *    before anything is enqueued, so a failing call has no effect.  No C++
 *    exception crosses this boundary.
 *  - Notation follows the paper: beam width w is `k`, the maximum number of
 *    draft-model calls n is `max_depth` (D), the check set S is `check_mask`,
 *    the threshold x is given in the probability domain, t = exp(x).
 *  - NaN logits are outside the contract (ordering undefined).
 */
#ifndef DDD_H_
#define DDD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DDD_KMAX 16          /* largest beam width k of the register/LDS-resident path            */
#define DDD_KWIDE_MAX 128    /* largest beam width k at all (wide beams: Appendix, Table 2)       */
#define DDD_MMAX 128         /* largest final tree size m                                         */
#define DDD_DMAX 31          /* largest max_depth (check_mask has 32 bits)                        */
/* ddd_config.flags: every draft call walks W first row to last.  Default (bit clear): calls with
 * an odd index walk it last to first, so that a call starts in the part of W the previous call
 * left in the memory-side cache (on the weight-stream path the results are the same up to the
 * rounding order of the fp32 sum of exponentials, on the GEMM path they are bit-identical). */
#define DDD_FLAG_FORWARD_SWEEPS 1u
/* ddd_config.flags, debugging aid: ddd_round_reset (and so every round) first fills the context's scratch - per-slice
 * partial results, materialised logits and group statistics, list of active rows - with 0xFF bytes, so that a kernel
 * that read something an earlier round or call left there would give visibly wrong results.  Costs a fill of the
 * scratch per round (up to 82 MB at the B = 64 shape). */
#define DDD_FLAG_POISON_SCRATCH 2u
#define DDD_BMAX 4096        /* largest number of sequences B                                     */
#define DDD_POOL_MAX 4096    /* largest node pool per sequence for k <= DDD_KMAX                  */
#define DDD_POOL_WIDE_MAX 65536 /* largest node pool per sequence for wider beams                 */
#define DDD_STREAM_ROWS 16   /* rows handled by one pass of the weight stream                     */
#define DDD_STATIC_ROWS 16   /* most rows per call of ddd_lmhead_topk_static                      */
#define DDD_STATIC_SLICES 256 /* most weight-stream workgroups its static scratch has room for    */

typedef enum ddd_status {
  DDD_OK = 0,
  DDD_ERR_INVALID_ARG = -1,   /* null pointer, size out of range, unsupported shape */
  DDD_ERR_NO_DEVICE = -2,     /* no HIP device visible                               */
  DDD_ERR_WRONG_ARCH = -3,    /* the current device is not gfx950                    */
  DDD_ERR_HIP = -4,           /* a HIP runtime call failed (see ddd_last_hip_error)  */
  DDD_ERR_UNIMPLEMENTED = -5,
  DDD_ERR_STATE = -6,         /* e.g. ddd_round_launch before ddd_round_capture      */
  DDD_ERR_STATIC_LIMIT = -7   /* ddd_lmhead_topk_static: more rows or a wider beam than its static scratch holds */
} ddd_status;

/* Parameters of Algorithm 1 (its Require clause) plus the problem shape. */
typedef struct ddd_config {
  int32_t B;           /* independent sequences, each with its own beam and stop decision; B*k*H < 2^31 when
                          B*k > DDD_STREAM_ROWS or k > DDD_KMAX (hidden rows of the MFMA path: 32-bit byte offsets) */
  int32_t H;           /* hidden size: H = 128*G*nw with G in {1,2,4} and 1 <= nw <= 10 (so H <= 5120)    */
  int32_t V;           /* vocabulary size, k <= V < 2^24; V <= 2^17 if B*k > DDD_STREAM_ROWS or k > DDD_KMAX */
  int32_t k;           /* beam width w, 1..DDD_KWIDE_MAX; the node pool 1 + k + (max_depth-1)*k*k must
                          not exceed DDD_POOL_MAX (k <= DDD_KMAX) or DDD_POOL_WIDE_MAX (wider beams) */
  int32_t max_depth;   /* n: maximum number of draft-model calls per round, 1..DDD_DMAX   */
  int32_t m;           /* final tree size in draft nodes (root not counted), 1..DDD_MMAX  */
  float threshold;     /* t: continue iff sum_i exp(logprobsum[i]) >= t  (Eq. 1, t = exp(x)) */
  uint32_t check_mask; /* bit s set <=> s in S: test after the s-th draft call (s >= 1)   */
  uint32_t flags;      /* DDD_FLAG_* bits, other bits must be 0                           */
} ddd_config;

/* Per-round beam and node-pool state.  All members are device pointers (caller-owned).
 * Nmax = ddd_pool_capacity(cfg) = 1 + k + (max_depth-1)*k*k.  Node 0 is the root; the prompt
 * call creates nodes 1..k; the s-th later call (s >= 1) creates nodes
 * 1 + k + (s-1)*k*k + i*k + j for beam slot i and rank j. */
typedef struct ddd_state {
  float* logprobsum;         /* [B,k]    summed logprob of each beam sequence (Algorithm 1)   */
  int32_t* beam_node;        /* [B,k]    pool id of each beam entry                           */
  int32_t* beam_token;       /* [B,k]    its token                                            */
  int32_t* beam_parent_slot; /* [B,k]    slot of its parent in the previous beam              */
  int32_t* pool_token;       /* [B,Nmax] token of every generated node                        */
  int32_t* pool_parent;      /* [B,Nmax] pool id of its parent, -1 for the root               */
  int32_t* pool_depth;       /* [B,Nmax] depth, root 0                                        */
  float* pool_score;         /* [B,Nmax] summed logprob along the path, root 0                */
  int32_t* n_nodes;          /* [B]      nodes in the pool, root included                     */
  int32_t* steps;            /* [B]      draft calls made in this round                       */
  uint8_t* active;           /* [B]      1 while the sequence keeps drafting                  */
  uint8_t* row_active;       /* [B*k]    active[b] repeated for the k beam rows of b          */
  double* conf;              /* [B]      P = sum_i exp(logprobsum[i]) after the latest call   */
} ddd_state;

/* Final draft tree.  Tree index 0 is the root, indices 1..n_sel the selected nodes in
 * ascending pool id (parents precede children).  Entries past n_sel are padded
 * (-1 for ids and tokens, 0 for pos and mask). */
typedef struct ddd_tree {
  int32_t* sel_node;    /* [B,m]         pool ids of the selected nodes              */
  int32_t* n_sel;       /* [B]           min(m, n_nodes-1)                            */
  int32_t* tree_token;  /* [B,m+1]                                                    */
  int32_t* pos;         /* [B,m+1]       depth of each tree node (position offset)    */
  int32_t* parent_idx;  /* [B,m+1]       tree index of the parent, -1 for the root    */
  uint8_t* mask;        /* [B,m+1,m+1]   mask[i][j]=1 iff j is i or an ancestor of i  */
} ddd_tree;

typedef struct ddd_ctx ddd_ctx;

/* Host-only helpers (no device needed). */
const char* ddd_strerror(int code);
const char* ddd_last_hip_error(void);                 /* text of the last failing HIP call on this thread */
int ddd_config_validate(const ddd_config* cfg);       /* DDD_OK or DDD_ERR_INVALID_ARG                    */
size_t ddd_pool_capacity(const ddd_config* cfg);      /* 1 + k + (max_depth-1)*k*k ; 0 if cfg is invalid  */
size_t ddd_scratch_bytes(const ddd_config* cfg);      /* device scratch a context allocates               */

/* Create / destroy a context on the current device.  DDD_ERR_NO_DEVICE without a GPU,
 * DDD_ERR_WRONG_ARCH if it is not gfx950. */
int ddd_create(const ddd_config* cfg, ddd_ctx** out);
int ddd_destroy(ddd_ctx* ctx);

/* Start of a round (Algorithm 1, its state before the first draft call): pool := {root}, steps := 0, active := 1.
 * root_token: device int32[B] or NULL (root token recorded as -1). */
int ddd_round_reset(ddd_ctx* ctx, ddd_state* st, const int32_t* root_token, void* stream);

/* LM-head projection + logsoftmax + per-row top-k of one draft call (Section 2: the draft
 * output goes through a logsoftmax; Section 1: top-k continuations per sequence).
 *   W_bf16   device bf16[V,H] row-major (H contiguous): the target's LM head, reused by the draft model
 *   hid_bf16 device bf16[n_rows,H] row-major: the draft body's output rows, 1 <= n_rows <= B*k
 *   row_active device u8[n_rows] or NULL (all active); outputs of inactive rows are left untouched
 *   topk_token   device int32[n_rows,k]: ids of the k largest logits, (logit desc, id asc)
 *   topk_logprob device fp32[n_rows,k]:  logit - lse of those tokens
 *   lse          device fp32[n_rows]:    log sum_v exp(logit[r,v])
 *   logits_dbg   device fp32[n_rows,V] or NULL: full fp32 logits (bf16 inputs, fp32 accumulate) */
int ddd_lmhead_topk(ddd_ctx* ctx, const void* W_bf16, const void* hid_bf16, int32_t n_rows,
                    const uint8_t* row_active, int32_t* topk_token, float* topk_logprob, float* lse,
                    float* logits_dbg, void* stream);

/* ddd_lmhead_topk for callers that cannot allocate device memory or create a context: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same results, bit for
 * bit, as ddd_lmhead_topk on a context of this configuration, with the per-slice partial results in a static
 * device array of ddd_static_scratch_bytes() bytes (540 672) that every GPU the library runs on holds until
 * the process ends; the call allocates and frees nothing.
 *   cfg      only H, V and k are used; the whole configuration must be valid
 *   n_rows   1..DDD_STATIC_ROWS hidden rows, and k <= DDD_KMAX: anything larger returns DDD_ERR_STATIC_LIMIT
 *            (those sizes take the MFMA path, whose scratch is hundreds of megabytes: use a context)
 *   other arguments as for ddd_lmhead_topk (no debug buffer)
 * The first call on a device looks the array's address up (make that call outside stream capture).  All calls
 * on one GPU share the one array: calls that overlap on a GPU, on different streams or from different threads,
 * race; calls on one stream are ordered and safe.  Nothing in the array carries over between calls. */
int ddd_lmhead_topk_static(const ddd_config* cfg, const void* W_bf16, const void* hid_bf16, int32_t n_rows,
                           const uint8_t* row_active, int32_t* topk_token, float* topk_logprob, float* lse,
                           void* stream);
size_t ddd_static_scratch_bytes(void);

/* Beam update after draft call number step+1 (Algorithm 1: the first beam and its logprobsum after the
 * prompt call for step 0, the post-processing of the draft outputs inside the loop otherwise): adds logprobsum of the parents, appends all candidates to the pool, keeps the
 * k best by (score desc, token asc, flat index asc) as the new beam; steps[b] += 1.
 *   topk_token / topk_logprob: as written by ddd_lmhead_topk; rows [B] for step 0 (row b),
 *   rows [B*k] for step >= 1 (row b*k+i is beam slot i of sequence b).
 * Sequences with active[b] == 0 are left untouched. */
int ddd_beam_select(ddd_ctx* ctx, int32_t step, const int32_t* topk_token, const float* topk_logprob,
                    ddd_state* st, void* stream);

/* DDD stop test (Eq. 1; Algorithm 1: the check on H at the loop indices in S) taken after `steps_done` draft calls:
 * conf[b] = sum_i exp(logprobsum[b,i]) (fp64); active[b] stays 1 iff steps_done < max_depth and
 * (bit steps_done of check_mask is clear or conf[b] >= threshold).  Written on the device; the
 * host never needs to read it inside a round. */
int ddd_depth_continue(ddd_ctx* ctx, int32_t steps_done, ddd_state* st, void* stream);

/* One whole draft call for every active sequence: ddd_lmhead_topk + ddd_beam_select +
 * ddd_depth_continue with the per-row results kept on chip (two kernel launches for up to DDD_STREAM_ROWS rows:
 * weight stream, bookkeeping; with more rows: list of active rows, MFMA GEMM, row reduction, bookkeeping).
 * hid_bf16: [B,H] for step 0, [B*k,H] for step >= 1.
 * tree: NULL, or the output of ddd_tree_finalize: a sequence whose stop test fails in this call
 * (or that has made max_depth calls) gets its final tree written by the same launch.
 * logits_dbg as above or NULL; lse_dbg: device fp32[n_rows] or NULL, the lse of every row. */
int ddd_draft_step(ddd_ctx* ctx, int32_t step, const void* W_bf16, const void* hid_bf16, ddd_state* st,
                   ddd_tree* tree, float* logits_dbg, float* lse_dbg, void* stream);

/* Final top-m rerank of all pool nodes by (score desc, node id asc), tree order, mask,
 * positions (Section 1: the tree is fed to the target model under a tree attention mask). */
int ddd_tree_finalize(ddd_ctx* ctx, const ddd_state* st, ddd_tree* out, void* stream);

/* Greedy accept walk (Section 1: tokens are verified until one is incorrect, then the token
 * that should follow is emitted; Section 3.1: temperature 0).
 *   target_argmax device int32[B,m+1]: the target model's argmax after each tree node
 *   accept_len    device int32[B]:     accepted draft tokens
 *   accept_path   device int32[B,max_depth+1]: tree indices root..last accepted, -1 padded
 *   bonus_token   device int32[B]:     target_argmax at the last accepted node */
int ddd_verify_accept(ddd_ctx* ctx, const ddd_tree* tree, const int32_t* target_argmax, int32_t* accept_len,
                      int32_t* accept_path, int32_t* bonus_token, void* stream);

/* Running statistics of the rounds a context verifies, kept on the device (Section 3.3 and Table 1 report the
 * mean accepted length per round; the number of draft calls a round makes is the quantity Section 2 makes
 * dynamic).  All arrays are device memory owned by the caller, int64, any of them may be NULL:
 *   rounds            [1]   rounds verified (every sequence of the batch has been walked)
 *   depth_hist        [32]  sequences by their number of draft calls (ddd_state.steps; needs `steps`)
 *   accept_hist       [32]  sequences by accepted length
 *   batch_depth_hist  [32]  rounds by the number of draft calls of their deepest sequence (needs `steps`)
 *   steps             device int32[B]: the ddd_state.steps of the rounds being verified, or NULL
 * Values above 31 are counted in entry 31.  While a set is bound, ddd_verify_accept and ddd_verify_sample add
 * their round to it inside their own launch (integer atomics: the totals do not depend on the order; `rounds` and
 * `batch_depth_hist` are written once per launch, by the sequence that finishes last).  The caller zeroes the
 * arrays and reads them, ordered on the stream like any other output.  ddd_stats_bind(ctx, NULL) unbinds.  The
 * pointers are read when a verify call is enqueued (or captured): bind before capturing a graph that verifies.
 * Two verify launches of one context that overlap in time would share the round's arrival counter: keep them on
 * one stream. */
typedef struct ddd_round_stats {
  int64_t* rounds;
  int64_t* depth_hist;
  int64_t* accept_hist;
  int64_t* batch_depth_hist;
  const int32_t* steps;
} ddd_round_stats;
int ddd_stats_bind(ddd_ctx* ctx, const ddd_round_stats* stats);

/* Sampled accept walk at temperature T > 0.  The paper evaluates temperature 0 only (Section 3.1); what it
 * fixes is that the emitted tokens follow the target model's distribution (Section 1).  A drafted child is a
 * deterministic proposal, so it is accepted with the probability the target gives its token, and after a
 * rejection the target distribution continues without that token, renormalised.  With
 * w_j = exp((x_j - max x) / T) over the current node's logit row x and rem = the weight not yet rejected
 * (initially sum_j w_j), the children c of the current node are tried in tree-index order:
 *     accept c  iff  u_accept[c] * rem < w[token_c];      else rem -= w[token_c], w[token_c] = 0.
 * When none is accepted (or the node has no child) the bonus token is the smallest j whose prefix sum of the
 * remaining w exceeds u_bonus[node] * rem; if rounding leaves no such j, the last token with w > 0, else the
 * row's argmax.  All decisions are taken in fp64.
 *   target_logits device fp32 [B, m+1, V]: the target model's logits after each tree node; every row needs a
 *                 finite maximum (-inf entries are allowed)
 *   temperature   > 0, finite
 *   u_accept      device fp64 [B, m+1] uniforms in [0,1), entry i drives the test of tree index i
 *   u_bonus       device fp64 [B, m+1] uniforms in [0,1), entry i drives the bonus draw at tree index i
 *   outputs as for ddd_verify_accept.  Only the logit rows of the accepted path are read. */
int ddd_verify_sample(ddd_ctx* ctx, const ddd_tree* tree, const float* target_logits, float temperature,
                      const double* u_accept, const double* u_bonus, int32_t* accept_len, int32_t* accept_path,
                      int32_t* bonus_token, void* stream);

/* Tree attention of the verification pass: what consumes the final tree's mask (Section 1, EAGLE
 * paragraph: the whole tree is fed to the target model at once, the attention mask adjusted so that
 * a node sees the prompt, its ancestors and itself).  Per sequence, head and tree index i <= n_sel:
 *   out[i] = sum_j softmax_j(q_i . k_j / sqrt(128)) v_j  over the L prompt keys and the tree keys j
 *            with tree->mask[i][j] = 1; rows of tree indices past n_sel are written as zeros.
 * Heads have 128 elements; queries and keys arrive already rotated (tree->pos holds each node's
 * depth).  All device, bf16 unless noted:
 *   q, k_tree   [B, m+1, n_heads, 128]          tree index order
 *   vt_tree     [B, n_heads, 128, Tp]           tree values TRANSPOSED (element d, tree index), Tp = m+1
 *                                               rounded up to 32, the padding must be zero
 *   k_packed,   the prompt's keys and values as written by ddd_kv_pack, each B * n_heads * ceil(L/32) * 4096
 *   v_packed    elements; may be NULL if L = 0
 *   workspace   device scratch of at least ddd_tree_attention_workspace(ctx, n_heads, L) bytes
 *   out         fp32 [B, m+1, n_heads, 128]
 * The prompt cache is read once per call and is what the call's time is made of, so it is kept in the order
 * the matrix cores take their operands in (every load of a wavefront is 1 KB of consecutive memory): per
 * sequence, head and chunk c of 32 keys, 8 KB of keys [s = 0..7][lane = 0..63][8] = K[key 32c + lane%32]
 * [d = 16s + 8*(lane/32) + 0..7], and 8 KB of values [db*2 + t][lane][8] = V[key 32c + 16t + 4*(lane/32) + 0..3,
 * then 32c + 16t + 8 + 4*(lane/32) + 0..3][d = 32*db + lane%32] (db = 0..3, t = 0..1); keys past L are zero.
 * ddd_kv_pack writes this from row-major k, v [B, L, n_heads, 128]. */
int ddd_kv_pack(ddd_ctx* ctx, const void* k, const void* v, int32_t L, int32_t n_heads, void* k_packed, void* v_packed,
                void* stream);
size_t ddd_tree_attention_workspace(const ddd_ctx* ctx, int32_t n_heads, int32_t L);
int ddd_tree_attention(ddd_ctx* ctx, const ddd_tree* tree, const void* q, const void* k_tree, const void* vt_tree,
                       const void* k_packed, const void* v_packed, int32_t L, int32_t n_heads, void* workspace,
                       size_t workspace_bytes, float* out, void* stream);

/* Draft-model body supplied by the caller: must enqueue on `stream` the work that writes the
 * hidden rows for draft call number step+1 into hid_out_bf16 ([B,H] for step 0, [B*k,H] after)
 * from the current beam in *st; rows of inactive sequences may be left untouched.  It must not
 * synchronise.  Returns 0 or a negative status. */
typedef int (*ddd_draft_body_fn)(void* user, int32_t step, const ddd_state* st, void* hid_out_bf16, void* stream);
/* Optional work enqueued after the tree is final (e.g. target model + ddd_verify_accept). */
typedef int (*ddd_post_fn)(void* user, const ddd_state* st, const ddd_tree* tree, void* stream);

/* Algorithm 1 end to end: reset, then max_depth draft calls (later calls are skipped on the
 * device for sequences whose stop test failed; the call in which a sequence stops also builds
 * its final tree), then `post`.
 * Only enqueues; usable inside or outside graph capture.
 *   hid_buf    device bf16[B*k,H] scratch the draft body writes into
 *   logits_dbg device fp32[max_depth, B*k, V] or NULL
 *   lse_dbg    device fp32[max_depth, B*k] or NULL */
int ddd_round_enqueue(ddd_ctx* ctx, const void* W_bf16, ddd_state* st, ddd_tree* tree, const int32_t* root_token,
                      void* hid_buf, ddd_draft_body_fn body, void* body_user, ddd_post_fn post, void* post_user,
                      float* logits_dbg, float* lse_dbg, void* stream);

/* Capture ddd_round_enqueue into a HIP graph owned by the context (replacing any earlier
 * one), and launch it.  `stream` for capture must be a non-default stream. */
int ddd_round_capture(ddd_ctx* ctx, const void* W_bf16, ddd_state* st, ddd_tree* tree, const int32_t* root_token,
                      void* hid_buf, ddd_draft_body_fn body, void* body_user, ddd_post_fn post, void* post_user,
                      float* logits_dbg, float* lse_dbg, void* stream);
int ddd_round_launch(ddd_ctx* ctx, void* stream);

/* Algorithm 1 with the host pacing the launches instead of a captured graph: the same kernels as
 * ddd_round_enqueue, but draft call s (s >= 2) is put into the stream only after call s-2 has reported, through a
 * word in pinned host memory written by its bookkeeping launch, that some sequence is still active.  The stop test
 * (Eq. 1) stays on the device and call s-1 is already queued when the report of call s-2 arrives, so the device
 * never waits for the host (Section 2 and the Limitations section of the paper: on its runtime every check forces
 * evaluation, which is why it checks only at the steps in S); what is saved are the launches a graph of max_depth
 * calls spends on calls that every sequence skips: at most one such call is queued per round.  Results are those
 * of ddd_round_enqueue.
 * The host thread polls, occupying a core until the last draft call has been queued (the call returns then, not
 * when the round has finished).  A wait is bounded: 20 ms for the report of a call, 1 s for the first report of a
 * round (the stream may still hold earlier work, e.g. the target model's forward of the previous round, which has
 * to finish before call 0 runs; with more than a second of backlog drain the stream first).  When a limit passes
 * the remaining calls are queued unconditionally - the results are the same, the pacing is lost for that round -
 * and the expiry is counted, see ddd_round_run_stats.  One round per context at a time; not for use under stream
 * capture (nothing would run while the host waits).  Arguments as for ddd_round_enqueue, without the debug
 * buffers.  Returns the number of draft calls queued (>= 1), or a negative status. */
int ddd_round_run(ddd_ctx* ctx, const void* W_bf16, ddd_state* st, ddd_tree* tree, const int32_t* root_token,
                  void* hid_buf, ddd_draft_body_fn body, void* body_user, ddd_post_fn post, void* post_user,
                  void* stream);

/* Counters of ddd_round_run's host waits since the context was created (any pointer may be NULL): rounds run,
 * waits for a call's report, waits that ran into their limit (the round then lost its pacing, see above), and the
 * longest wait in microseconds. */
int ddd_round_run_stats(const ddd_ctx* ctx, uint64_t* rounds, uint64_t* waits, uint64_t* timeouts, double* max_wait_us);

/* Optional tile-major copy of the LM-head weights for the calls that take the MFMA path (more
 * than DDD_STREAM_ROWS rows, or wide beams).  Section 1's projection reads W once per draft call;
 * when W is too large for the chip's caches (a 128k vocabulary: 1 GB) the MFMA path would fetch it
 * from HBM in 128-byte pieces 2*H bytes apart, and reads the same bytes a quarter faster from a copy
 * whose tiles are contiguous.  Results are bit-identical with and without the copy.
 *   W_bf16  device, bf16 [V,H] row-major; NULL forgets the copy and frees it.
 * The context allocates ceil(V/256)*256*H*2 bytes on first use, fills them on `stream`, and from
 * then on reads the copy whenever a call passes this same pointer as W (the row-major W is still
 * needed: calls of up to DDD_STREAM_ROWS rows stream it).  Call again after changing W's contents,
 * and before ddd_round_capture (a captured graph keeps the operands it was captured with). */
int ddd_weights_pack(ddd_ctx* ctx, const void* W_bf16, void* stream);

/* Introspection used by the benchmark: number of weight-stream workgroups (slices). */
int ddd_num_slices(const ddd_ctx* ctx);

/* Measurement helper (the one call that synchronises): launches the LM-head kernel alone
 * `iters` times on `stream` for n_rows (<= B*k, all taken as active) rows of hid_bf16 - the weight
 * stream for n_rows <= DDD_STREAM_ROWS, the MFMA GEMM otherwise - each launch bracketed by its own
 * pair of HIP events recorded on that stream, waits for the last one and returns the mean and the
 * minimum elapsed time per launch in milliseconds (host pointers).  Partial results go to the
 * context scratch and are not consumed. */
int ddd_profile_lmhead(ddd_ctx* ctx, const void* W_bf16, const void* hid_bf16, int32_t n_rows, int32_t iters,
                       float* mean_ms, float* min_ms, void* stream);

/* Device-timestamp trace of the draft calls' kernels (measurement aid; the second call that synchronises).
 * While enabled, every draft call of the context (ddd_draft_step and the round calls) leaves 100 MHz wall-clock
 * stamps in a device buffer the context allocates on enabling: for call number s, at word s * DDD_TRACE_CALL_WORDS,
 * first DDD_STATIC_SLICES * 8 words of the weight stream (per workgroup: entry, first tile multiplied, last tile
 * multiplied (first streaming wave), last tile folded into the row statistics, the lanes' lists exchanged, partial
 * results written, last tile multiplied by every streaming wave, one unused; zero on the MFMA path), then 8 words of the bookkeeping launch's workgroup 0
 * (entry, slice keys arrived, rows merged, beam update and stop test done, final tree done - equal to the previous
 * stamp if none was built -, exit; two unused).  Kernels of a later round overwrite the stamps of an earlier one.
 * ddd_trace_enable waits for the device, then allocates / clears (on != 0) or frees (on == 0) the buffer: do not
 * call it between the capture and the last launch of a graph.  ddd_trace_read waits for the device, copies all
 * ddd_trace_words() words to host memory `out` (n_words must be that number) and clears the buffer. */
#define DDD_TRACE_CALL_WORDS (DDD_STATIC_SLICES * 8 + 8)
int ddd_trace_enable(ddd_ctx* ctx, int32_t on);
int ddd_trace_read(ddd_ctx* ctx, uint64_t* out, size_t n_words);
size_t ddd_trace_words(void);

#ifdef __cplusplus
}
#endif
#endif /* DDD_H_ */
