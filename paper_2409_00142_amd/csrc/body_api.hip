// C ABI of the stand-in draft layer (include/ddd_body.h): argument checks, scratch, and the
// sequence of launches of one draft call.
#include <hip/hip_runtime.h>

#include <new>

#include "body_kernels.hpp"
#include "ddd_kernels.hpp"
#include "../../include/ddd_body.h"

using namespace ddd;

struct ddd_body {
  ddd_body_config cfg;
  int n_cu;
  int rows;          // B*k: rows of a call after the prompt call, and rows per call in the histories
  ddd_body_weights w;
  ddd_body_prompt p;
  bool bound;
  float* r;          // fp32 [rows][H]   residual stream
  uint16_t* xn;      // bf16 [rows][H]   normalised rows / attention output
  float* qkv;        // fp32 [rows][3H]
  uint16_t* act;     // bf16 [rows][F]
  uint16_t* h_hist;  // bf16 [D][rows][H]
  uint16_t* k_hist;
  uint16_t* v_hist;
  int32_t* par_hist; // [D][rows]
  // calls of more than kBodyRows rows go through the MFMA GEMM:
  uint16_t* x0;      // bf16 [rows][2H]  FC input rows, assembled (null if rows <= kBodyRows)
  int32_t* row_list; // [rows] ids of the active rows of the current call
  int32_t* n_act;    // [1]
  uint16_t* vt;      // bf16 [B][H][Lp] the prompt's values, keys contiguous (null if rows <= kBodyRows or L < 32);
  int Lp;            //   rewritten by the prompt call of every round
};

namespace {

int hip_status(hipError_t e) { return e == hipSuccess ? DDD_OK : DDD_ERR_HIP; }
#define BODY_HIP(call)                       \
  do {                                       \
    const int rc_ = hip_status(call);        \
    if (rc_ != DDD_OK) return rc_;           \
  } while (0)

// Largest K range one launch of the weight stream covers: 128 * G * nw with G in {1,2,4}, nw <= 10.
bool pick_range(int units, int* G, int* nw) {   // units = remaining K / 128
  int best = 0;
  for (int g = 4; g >= 1; g >>= 1)
    for (int w = 10; w >= 1; --w)
      if (g * w <= units && g * w > best) {
        best = g * w;
        *G = g;
        *nw = w;
      }
  return best > 0;
}

// One product y (+)= x W^T over K, cut into K ranges of 128 * G * nw elements; `a` describes the product: rg[0]
// holds W, x and the gather of the whole K extent.  Consecutive ranges of the same length go into one launch (at
// most kLinearRanges of them).  a.mode is the LinearMode of the whole product; a.out16 / a.out16b are written by
// the launch that completes it.
int enqueue_linear(const ddd_body* b, LinearArgs a, int K, hipStream_t s) {
  a.ntiles = (a.N + 15) / 16;
  const int nslice = a.ntiles < b->n_cu ? a.ntiles : b->n_cu;
  const LinearRange whole = a.rg[0];
  uint16_t* out16 = a.out16;
  uint16_t* out16b = a.out16b;
  const int mode = a.mode;
  int k0 = 0;
  while (k0 < K) {
    int G = 1, nw = 1;
    pick_range((K - k0) / 128, &G, &nw);
    const int len = 128 * G * nw;
    int nr = 1;
    while (nr < kLinearRanges && k0 + (nr + 1) * len <= K) ++nr;
    const bool last = k0 + nr * len >= K;
    // the gate needs complete sums: such a product must fit one launch
    if (mode == kLinearSiluPairs && !(k0 == 0 && last)) return DDD_ERR_INVALID_ARG;
    for (int r = 0; r < nr; ++r) {
      a.rg[r] = whole;
      a.rg[r].W = whole.W + k0 + r * len;
      a.rg[r].x = whole.x + k0 + r * len;
    }
    a.n_ranges = nr;
    a.out16 = last ? out16 : nullptr;
    a.out16b = last ? out16b : nullptr;
    a.nw = nw;
    a.mode = (k0 > 0) ? (int)kLinearAccumulate : mode;
    BODY_HIP(launch_linear_stream(a, G, nslice, s));
    k0 += nr * len;
  }
  return DDD_OK;
}

// One launch of a product whose K ranges come from different places: the ranges in a.rg[0 .. n_ranges) as given, each
// of K_range elements (one launch: K_range must be a single range length).
int enqueue_linear_ranges(const ddd_body* b, LinearArgs a, int K_range, hipStream_t s) {
  int G = 1, nw = 1;
  if (!pick_range(K_range / 128, &G, &nw) || 128 * G * nw != K_range) return DDD_ERR_INVALID_ARG;
  a.ntiles = (a.N + 15) / 16;
  a.nw = nw;
  const int nslice = a.ntiles < b->n_cu ? a.ntiles : b->n_cu;
  BODY_HIP(launch_linear_stream(a, G, nslice, s));
  return DDD_OK;
}

// y (+)= x W^T over the rows in b->row_list through the MFMA GEMM (calls of more than kBodyRows rows).
int enqueue_gemm_linear(const ddd_body* b, const void* W, int N, int K, const uint16_t* x, float* y, int epi,
                        uint16_t* out16, uint16_t* out16b, int ld16, hipStream_t s) {
  GemmArgs g;
  g.W = static_cast<const uint16_t*>(W);
  g.Wp = nullptr;
  g.hid = x;
  g.row_list = b->row_list;
  g.n_act_ptr = b->n_act;
  g.logits = y;
  g.grp_max = nullptr;
  g.grp_sum = nullptr;
  g.H = K;
  g.V = N;
  g.ngrp = 0;
  g.reverse = 0;
  g.epi = epi;
  g.out16 = out16;
  g.out16b = out16b;
  g.ld16 = ld16;
  BODY_HIP(launch_gemm_linear(g, b->rows, ((b->n_cu + 7) / 8) * 8, s));
  return DDD_OK;
}

LinearArgs linear_args(const void* W, int ldw, int N, int R, const uint8_t* row_active, float* y, int ldy, int mode) {
  LinearArgs a = {};
  a.rg[0].W = static_cast<const uint16_t*>(W);
  a.rg[0].gather_mode = kGatherNone;
  a.n_ranges = 1;
  a.ldw = ldw;
  a.N = N;
  a.R = R;
  a.row_active = row_active;
  a.y = y;
  a.ldy = ldy;
  a.mode = mode;
  a.gather_k = 1;
  return a;
}

}  // namespace

extern "C" {

int ddd_body_create(const ddd_body_config* cfg, ddd_body** out) {
  if (cfg == nullptr || out == nullptr) return DDD_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg->B < 1 || cfg->k < 1 || (long long)cfg->B * cfg->k > DDD_BODY_ROWS_MAX) return DDD_ERR_INVALID_ARG;
  if (cfg->H < 128 || cfg->H > 5120 || cfg->H % 128 != 0 || cfg->F < 128 || cfg->F % 128 != 0 || cfg->V < 1) return DDD_ERR_INVALID_ARG;
  {
    int G = 0, nw = 0;   // H must fit one K range of the weight stream (the gated linear needs complete sums)
    if (!pick_range(cfg->H / 128, &G, &nw) || G * nw != cfg->H / 128) return DDD_ERR_INVALID_ARG;
  }
  if (cfg->max_depth < 1 || cfg->max_depth > DDD_DMAX || cfg->L < 0 || cfg->L > DDD_BODY_LMAX)
    return DDD_ERR_INVALID_ARG;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return DDD_ERR_NO_DEVICE;
  hipDeviceProp_t prop;
  BODY_HIP(hipGetDeviceProperties(&prop, dev));
  ddd_body* b = new (std::nothrow) ddd_body();
  if (b == nullptr) return DDD_ERR_INVALID_ARG;
  b->cfg = *cfg;
  b->n_cu = prop.multiProcessorCount;
  b->bound = false;
  b->rows = cfg->B * cfg->k;
  // the stand-alone linear (ddd_body_linear) may be called with up to kBodyRows rows whatever B*k is
  const size_t H = cfg->H, F = cfg->F, D = cfg->max_depth, R = b->rows > kBodyRows ? b->rows : kBodyRows;
  hipError_t e = hipMalloc(&b->r, R * H * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&b->xn, R * H * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMalloc(&b->qkv, R * 3 * H * sizeof(float));
  if (e == hipSuccess) e = hipMalloc(&b->act, R * F * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMalloc(&b->h_hist, D * R * H * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMalloc(&b->k_hist, D * R * H * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMalloc(&b->v_hist, D * R * H * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMalloc(&b->par_hist, D * R * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemset(b->r, 0, R * H * sizeof(float));            // rows never written stay finite
  if (e == hipSuccess) e = hipMemset(b->xn, 0, R * H * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMemset(b->act, 0, R * F * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMemset(b->par_hist, 0, D * R * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(&b->row_list, R * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(&b->n_act, sizeof(int32_t));
  if (e == hipSuccess && b->rows > kBodyRows) {
    e = hipMalloc(&b->x0, R * 2 * H * sizeof(uint16_t));
    if (e == hipSuccess) e = prepare_lmhead_gemm();
    b->Lp = (cfg->L + 31) & ~31;
    if (e == hipSuccess && cfg->L >= 32) e = hipMalloc(&b->vt, (size_t)cfg->B * H * b->Lp * sizeof(uint16_t));
  }
  if (e != hipSuccess) {
    ddd_body_destroy(b);
    return DDD_ERR_HIP;
  }
  *out = b;
  return DDD_OK;
}

int ddd_body_destroy(ddd_body* b) {
  if (b == nullptr) return DDD_ERR_INVALID_ARG;
  (void)hipFree(b->r);
  (void)hipFree(b->xn);
  (void)hipFree(b->qkv);
  (void)hipFree(b->act);
  (void)hipFree(b->h_hist);
  (void)hipFree(b->k_hist);
  (void)hipFree(b->v_hist);
  (void)hipFree(b->par_hist);
  (void)hipFree(b->x0);
  (void)hipFree(b->vt);
  (void)hipFree(b->row_list);
  (void)hipFree(b->n_act);
  delete b;
  return DDD_OK;
}

int ddd_body_bind(ddd_body* b, const ddd_body_weights* w, const ddd_body_prompt* p) {
  if (b == nullptr || w == nullptr || p == nullptr) return DDD_ERR_INVALID_ARG;
  if (!w->E || !w->Wfc || !w->g1 || !w->Wqkv || !w->Wo || !w->g2 || !w->Wgu || !w->Wd) return DDD_ERR_INVALID_ARG;
  if (!p->f_root || !p->root_token || (b->cfg.L > 0 && (!p->K || !p->V))) return DDD_ERR_INVALID_ARG;
  b->w = *w;
  b->p = *p;
  b->bound = true;
  return DDD_OK;
}

int ddd_body_linear(ddd_body* b, const void* W, int32_t N, int32_t K, const void* x, int32_t R, float* y,
                    int32_t accumulate, void* stream) {
  if (b == nullptr || W == nullptr || x == nullptr || y == nullptr) return DDD_ERR_INVALID_ARG;
  if (N < 1 || K < 128 || K % 128 != 0 || R < 1) return DDD_ERR_INVALID_ARG;
  if (R > kBodyRows) {   // the MFMA path of calls with more rows, all R rows taken as active
    if (R > b->rows || N % 4 != 0) return DDD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    BODY_HIP(launch_build_row_list(nullptr, R, b->row_list, b->n_act, s));
    return enqueue_gemm_linear(b, W, N, K, static_cast<const uint16_t*>(x), y, accumulate ? kGemmAccumulate : kGemmStore,
                               nullptr, nullptr, 0, s);
  }
  LinearArgs a = linear_args(W, K, N, R, nullptr, y, N, accumulate ? kLinearAccumulate : kLinearStore);
  a.rg[0].x = static_cast<const uint16_t*>(x);
  a.rg[0].ldx = K;
  return enqueue_linear(b, a, K, static_cast<hipStream_t>(stream));
}

int ddd_body_step(void* user, int32_t step, const ddd_state* st, void* hid_out, void* stream) {
  ddd_body* b = static_cast<ddd_body*>(user);
  if (b == nullptr || st == nullptr || hid_out == nullptr) return DDD_ERR_INVALID_ARG;
  if (!b->bound) return DDD_ERR_STATE;
  if (step < 0 || step >= b->cfg.max_depth) return DDD_ERR_INVALID_ARG;
  if (st->beam_token == nullptr || st->beam_parent_slot == nullptr || st->row_active == nullptr)
    return DDD_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int H = b->cfg.H, F = b->cfg.F;
  const int R = (step == 0) ? b->cfg.B : b->cfg.B * b->cfg.k;
  const uint8_t* act = (step == 0) ? nullptr : st->row_active;   // a round starts with every sequence drafting
  const size_t hist_rows = b->rows > kBodyRows ? b->rows : kBodyRows;
  const size_t hist = (size_t)step * hist_rows * H;
  const bool gemm = R > kBodyRows;
  int rc = DDD_OK;

  RmsNormArgs n1;
  n1.x = b->r;
  n1.g = b->w.g1;
  n1.row_active = act;
  n1.out = b->xn;
  n1.H = H;
  n1.R = R;
  BodyAttnArgs t;
  t.qkv = b->qkv;
  t.Kp = static_cast<const uint16_t*>(b->p.K);
  t.Vp = static_cast<const uint16_t*>(b->p.V);
  t.k_hist = b->k_hist;
  t.v_hist = b->v_hist;
  t.par_hist = b->par_hist;
  t.beam_parent_slot = st->beam_parent_slot;
  t.row_active = act;
  t.o = b->xn;                     // the normalised rows are consumed: reuse their buffer
  t.H = H;
  t.L = b->cfg.L;
  t.k = b->cfg.k;
  t.step = step;
  t.R = R;
  t.hist_rows = (int)hist_rows;
  t.Vt = b->vt;
  t.Lp = b->Lp;
  if (step == 0 && b->vt != nullptr)   // the round's prompt, laid out for the batched attention's second contraction
    BODY_HIP(launch_pack_prompt_values(t.Vp, b->vt, b->cfg.B, H, b->cfg.L, b->Lp, s));
  RmsNormArgs n2 = n1;
  n2.g = b->w.g2;

  if (gemm) {
    // More than kBodyRows rows: the same sequence of operations with every linear on the matrix cores, over the
    // compacted list of active rows; the FC's input rows are assembled first (the GEMM gathers whole rows).
    BODY_HIP(launch_build_row_list(act, R, b->row_list, b->n_act, s));
    PackX0Args px;
    px.E = static_cast<const uint16_t*>(b->w.E);
    px.token = (step == 0) ? b->p.root_token : st->beam_token;
    px.feat = (step == 0) ? static_cast<const uint16_t*>(b->p.f_root) : b->h_hist + hist - hist_rows * H;
    px.parent_slot = st->beam_parent_slot;
    px.row_active = act;
    px.x0 = b->x0;
    px.H = H;
    px.k = b->cfg.k;
    px.R = R;
    px.feat_mode = (step == 0) ? kGatherNone : (step == 1) ? kGatherBlock : kGatherInBlock;
    BODY_HIP(launch_pack_x0(px, s));
    rc = enqueue_gemm_linear(b, b->w.Wfc, H, 2 * H, b->x0, b->r, kGemmStore, nullptr, nullptr, 0, s);
    if (rc != DDD_OK) return rc;
    BODY_HIP(launch_rmsnorm(n1, s));
    rc = enqueue_gemm_linear(b, b->w.Wqkv, 3 * H, H, b->xn, b->qkv, kGemmStore, nullptr, nullptr, 0, s);
    if (rc != DDD_OK) return rc;
    BODY_HIP(launch_body_attention(t, s));
    rc = enqueue_gemm_linear(b, b->w.Wo, H, H, b->xn, b->r, kGemmAccumulate, nullptr, nullptr, 0, s);   // r1 = r0 + o Wo^T
    if (rc != DDD_OK) return rc;
    BODY_HIP(launch_rmsnorm(n2, s));
    rc = enqueue_gemm_linear(b, b->w.Wgu, 2 * F, H, b->xn, nullptr, kGemmSiluPairs, b->act, nullptr, F, s);
    if (rc != DDD_OK) return rc;
    // h = bf16(r1 + a Wd^T), written to the hidden rows and to this call's features
    return enqueue_gemm_linear(b, b->w.Wd, H, F, b->act, b->r, kGemmAccumulate, static_cast<uint16_t*>(hid_out),
                               b->h_hist + hist, H, s);
  }

  // r0 = [E[token], parent feature] Wfc^T: one launch over two K ranges of H, the rows read where they are
  const uint16_t* Wfc = static_cast<const uint16_t*>(b->w.Wfc);
  LinearArgs fc = linear_args(Wfc, 2 * H, H, R, act, b->r, H, kLinearStore);
  fc.n_ranges = 2;
  fc.gather_k = b->cfg.k;
  fc.rg[0].x = static_cast<const uint16_t*>(b->w.E);
  fc.rg[0].ldx = H;
  fc.rg[0].gather_mode = kGatherIndex;
  fc.rg[0].gather_idx = (step == 0) ? b->p.root_token : st->beam_token;
  fc.rg[1].W = Wfc + H;
  fc.rg[1].x = (step == 0) ? static_cast<const uint16_t*>(b->p.f_root) : b->h_hist + hist - hist_rows * H;
  fc.rg[1].ldx = H;
  fc.rg[1].gather_mode = kGatherNone;
  fc.rg[1].gather_idx = nullptr;
  if (step == 1) fc.rg[1].gather_mode = kGatherBlock;      // the prompt call has one row per sequence
  if (step >= 2) {
    fc.rg[1].gather_mode = kGatherInBlock;
    fc.rg[1].gather_idx = st->beam_parent_slot;
  }
  rc = enqueue_linear_ranges(b, fc, H, s);
  if (rc != DDD_OK) return rc;

  BODY_HIP(launch_rmsnorm(n1, s));
  LinearArgs lq = linear_args(b->w.Wqkv, H, 3 * H, R, act, b->qkv, 3 * H, kLinearStore);
  lq.rg[0].x = b->xn;
  lq.rg[0].ldx = H;
  rc = enqueue_linear(b, lq, H, s);
  if (rc != DDD_OK) return rc;

  BODY_HIP(launch_body_attention(t, s));
  LinearArgs lo = linear_args(b->w.Wo, H, H, R, act, b->r, H, kLinearAccumulate);   // r1 = r0 + o Wo^T
  lo.rg[0].x = b->xn;
  lo.rg[0].ldx = H;
  rc = enqueue_linear(b, lo, H, s);
  if (rc != DDD_OK) return rc;

  // gate and up rows of Wgu alternate, so the epilogue of their linear forms a = bf16(silu(gate) * up) itself
  BODY_HIP(launch_rmsnorm(n2, s));
  LinearArgs lg = linear_args(b->w.Wgu, H, 2 * F, R, act, nullptr, 0, kLinearSiluPairs);
  lg.rg[0].x = b->xn;
  lg.rg[0].ldx = H;
  lg.out16 = b->act;
  lg.ld16 = F;
  rc = enqueue_linear(b, lg, H, s);
  if (rc != DDD_OK) return rc;

  // h = bf16(r1 + a Wd^T): the range that completes the sum also writes the hidden rows and this call's features
  LinearArgs ld = linear_args(b->w.Wd, F, H, R, act, b->r, H, kLinearAccumulate);
  ld.rg[0].x = b->act;
  ld.rg[0].ldx = F;
  ld.out16 = static_cast<uint16_t*>(hid_out);
  ld.out16b = b->h_hist + hist;
  ld.ld16 = H;
  rc = enqueue_linear(b, ld, F, s);
  if (rc != DDD_OK) return rc;
  return DDD_OK;
}

}  // extern "C"
