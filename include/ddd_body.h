/*
 * ddd_body.h - C ABI of a stand-in draft-model body for the DDD draft round.
 *
 * Section 1 (EAGLE paragraph) describes the draft model the round calls between two LM-head
 * projections: it takes the token sequence and the target model's feature sequence, runs one
 * transformer decoder layer and reuses the target's LM head; Section 1 (EAGLE-2 paragraph) makes
 * every beam node one input row whose context is the prompt plus the node's ancestors in the
 * draft tree.  The trained weights are not part of this library; with caller-supplied (here:
 * synthetic) weights of the same shapes this body makes a draft call stream what the real one
 * streams: the embedding rows of the beam tokens, an FC over [embedding, parent feature], and the
 * attention and MLP matrices of one layer, all bf16 with fp32 accumulation.
 *
 * Per row of a draft call (depth d = call number, L = prompt length):
 *   x0 = [E[token], f_parent]            r0 = x0 Wfc^T            xn = bf16(rmsnorm(r0) g1)
 *   [q,k,v] = xn Wqkv^T, q and k rotated to position L + d (rotate-half RoPE, base 10000, heads of
 *   128), k and v kept as bf16           o = bf16(softmax(q k_j / sqrt(128)) v_j) over the prompt, the
 *   row's ancestors and itself           r1 = r0 + o Wo^T          xn2 = bf16(rmsnorm(r1) g2)
 *   a = bf16(silu(xn2 Wg^T) * (xn2 Wu^T))  (gate and up rows interleaved in Wgu)   h = bf16(r1 + a Wd^T)
 * h is the hidden row handed to the LM head and the feature f of this node.  rmsnorm uses eps 1e-6.
 *
 * Conventions are those of ddd.h (device buffers are caller-owned, calls only enqueue, status
 * codes, `stream`).  Calls of up to DDD_STREAM_ROWS rows run every linear as a weight stream (each matrix
 * read once, HBM-bound); calls of more rows (batched rounds) run them on the matrix cores over the active rows.
 */
#ifndef DDD_BODY_H_
#define DDD_BODY_H_

#include "ddd.h"

#ifdef __cplusplus
extern "C" {
#endif

#define DDD_BODY_LMAX 2048   /* largest prompt length */
#define DDD_BODY_ROWS_MAX 4096 /* largest B*k */

typedef struct ddd_body_config {
  int32_t B, k;        /* as in ddd_config; B*k <= DDD_BODY_ROWS_MAX                     */
  int32_t H;           /* hidden size: H = 128*G*nw as in ddd_config (heads of 128)      */
  int32_t F;           /* MLP width, a multiple of 128                                   */
  int32_t V;           /* rows of the embedding                                          */
  int32_t max_depth;   /* draft calls per round, 1..DDD_DMAX                             */
  int32_t L;           /* prompt positions visible to every row, 0..DDD_BODY_LMAX        */
} ddd_body_config;

/* Device pointers, bf16 row-major unless noted; they must stay valid while bound. */
typedef struct ddd_body_weights {
  const void* E;      /* [V,H]   token embedding                    */
  const void* Wfc;    /* [H,2H]                                     */
  const float* g1;    /* [H] fp32                                   */
  const void* Wqkv;   /* [3H,H]  rows: q, then k, then v            */
  const void* Wo;     /* [H,H]                                      */
  const float* g2;    /* [H] fp32                                   */
  const void* Wgu;    /* [2F,H]  row 2i: gate i, row 2i+1: up i (this interleaving is the ABI's: it lets the
                                 product's epilogue form silu(gate)*up from neighbouring sums) */
  const void* Wd;     /* [H,F]                                      */
} ddd_body_weights;

typedef struct ddd_body_prompt {
  const void* K;              /* [B,L,H] cached keys of the prompt (already rotated) */
  const void* V;              /* [B,L,H] cached values                              */
  const void* f_root;         /* [B,H]   the target's feature at the last prompt token */
  const int32_t* root_token;  /* [B]     the last prompt token                      */
} ddd_body_prompt;

typedef struct ddd_body ddd_body;

/* Allocates the body's scratch and per-call history (features, keys, values and parent slots of
 * every row of every call of the current round: 3 * max_depth * max(B*k, 16) * H bf16). */
int ddd_body_create(const ddd_body_config* cfg, ddd_body** out);
int ddd_body_destroy(ddd_body* body);

/* Weights and prompt context used by the following calls (pointers are copied, not the data).  The prompt's keys
 * and values are read by every call of a round and must not change while a round is in flight; with more than 16
 * rows per call and a prompt of 32 positions or more, the prompt call (step 0) of every round also writes a copy of
 * the values laid out for the matrix cores (B * H * ceil(L / 32) * 32 bf16, allocated by ddd_body_create), which the
 * later calls of that round read. */
int ddd_body_bind(ddd_body* body, const ddd_body_weights* w, const ddd_body_prompt* p);

/* The body as a ddd_draft_body_fn: user = ddd_body*.  Enqueues the layer for the rows of draft
 * call number `step` (one row per sequence for step 0, B*k after) from the current beam in *st
 * and writes their hidden rows to hid_out_bf16; rows of stopped sequences are skipped.  Calls of
 * one round must come in order step = 0, 1, ... (each reads the history of the earlier ones). */
int ddd_body_step(void* user, int32_t step, const ddd_state* st, void* hid_out_bf16, void* stream);

/* y[r,n] = sum_k x[r,k] W[n,k]: one linear of the layer on its own (K a multiple of 128, N >= 1; W bf16 [N,K],
 * x bf16 [R,K], y fp32 [R,N], all device): the weight stream for R <= 16 rows, the MFMA path for
 * 16 < R <= B*k rows (N a multiple of 4 there).  accumulate != 0 adds to y. */
int ddd_body_linear(ddd_body* body, const void* W, int32_t N, int32_t K, const void* x, int32_t R, float* y,
                    int32_t accumulate, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DDD_BODY_H_ */
