// C ABI of the DDD draft-round library: validation, context, dispatch, round orchestration.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "ddd_kernels.hpp"

using namespace ddd;

struct ddd_ctx {
  ddd_config cfg;
  int device;
  int n_cu;
  int G, nw;            // K split of the weight stream: H == 128 * G * nw
  int ntiles, nslice;   // 16-row tiles of W, workgroups of the weight stream (<= 16 rows)
  int g_grid;           // GEMM path (> 16 rows): one workgroup per CU
  int nmax;
  uint64_t* part_key;   // [B*k][k][nslice] (weight stream: rank-major, the slices' j-th keys together) or [B*k][k] (GEMM path, dense)
  float* part_sum;      // [B*k][nslice] or [B*k]
  int32_t* row_list;    // [B*k] active rows of the current call (GEMM path)
  int32_t* n_act;       // [1]
  float* logits;        // [B*k][V] fp32 logits of the GEMM path (null if B*k <= 16)
  float* grp_max;       // [B*k][ngrp] per-group max / sum-exp of the GEMM path
  float* grp_sum;
  int ngrp;
  const void* pack_src; // W pointer whose tile-major copy is in pack (null: none)
  uint16_t* pack;       // [ceil(V/256)*256][H] tile-major copy for the GEMM path, owned
  hipGraph_t graph;
  hipGraphExec_t graph_exec;
  // ddd_round_run: the kernels of draft call s publish "call s done, some sequence still active" to host memory
  uint32_t* call_count;          // device [DDD_DMAX + 1]: arrivals (low half) and active sequences (high half) per call
  uint64_t* active_mask;         // device [DDD_BMAX / 64]: bit b = sequence b goes on after the current call (zero between calls)
  volatile uint32_t* progress;   // pinned host [DDD_DMAX + 1]: (round tag << 2) | 2 | any_active
  uint32_t* progress_dev;        // the same words as the kernels address them
  uint32_t round_tag;
  // ddd_round_run's host waits, since the context was created (ddd_round_run_stats)
  uint64_t run_rounds, run_waits, run_timeouts;
  double run_max_wait_us;
  ddd_round_stats stats;         // caller's statistics arrays (all null: none bound)
  bool stats_on;
  uint32_t* stats_sync;          // device [2]: arrivals and deepest sequence of the verify launch in flight (zero between)
  uint64_t* trace;               // null, or device [DDD_DMAX + 1][kTraceCallWords]: stamps of every draft call's kernels
  size_t part_key_bytes, part_sum_bytes, logits_bytes, grp_bytes;   // sizes of the scratch arrays (DDD_FLAG_POISON_SCRATCH)
};

namespace {

thread_local char g_hip_err[256] = "";

int hip_fail(hipError_t e, const char* what) {
  std::snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
  return DDD_ERR_HIP;
}
#define DDD_HIP(call)                                 \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) return hip_fail(e_, #call); \
  } while (0)

// K split: the smallest G in {1,2,4} with H == 128*G*nw and nw <= 10 streaming waves
// (10 waves keep the dynamic LDS of the weight stream under 64 KB).
bool pick_split(int H, int* G, int* nw) {
  for (int g = 1; g <= 4; g <<= 1) {
    if (H % (128 * g) != 0) continue;
    const int w = H / (128 * g);
    if (w >= 1 && w <= 10) {
      *G = g;
      *nw = w;
      return true;
    }
  }
  return false;
}

bool state_ok(const ddd_state* s) {
  return s && s->logprobsum && s->beam_node && s->beam_token && s->beam_parent_slot && s->pool_token &&
         s->pool_parent && s->pool_depth && s->pool_score && s->n_nodes && s->steps && s->active && s->row_active &&
         s->conf;
}
bool tree_ok(const ddd_tree* t) {
  return t && t->sel_node && t->n_sel && t->tree_token && t->pos && t->parent_idx && t->mask;
}

BeamArgs beam_args(const ddd_ctx* c, const ddd_state* st, int step) {
  BeamArgs a;
  a.st = *st;
  a.topk_token = nullptr;
  a.topk_logprob = nullptr;
  a.B = c->cfg.B;
  a.k = c->cfg.k;
  a.D = c->cfg.max_depth;
  a.nmax = c->nmax;
  a.step = step;
  a.threshold = c->cfg.threshold;
  a.check_mask = c->cfg.check_mask;
  return a;
}

WideStepArgs wide_args(const ddd_ctx* c, const BeamArgs& beam) {
  WideStepArgs w;
  w.beam = beam;
  w.part_key = nullptr;
  w.part_lse = nullptr;
  w.lse_dbg = nullptr;
  std::memset(&w.tree, 0, sizeof(w.tree));
  w.m = c->cfg.m;
  w.do_select = 0;
  w.do_stop = 0;
  w.steps_done = 0;
  w.call_count = nullptr;
  w.progress = nullptr;
  w.round_tag = 0;
  return w;
}

// MFMA GEMM over the rows listed in the context's row list, logits into `out`.
int enqueue_gemm(ddd_ctx* c, const void* W, const void* hid, int max_rows, float* out, int reverse, hipStream_t s) {
  GemmArgs g;
  g.W = static_cast<const uint16_t*>(W);
  g.Wp = (c->pack_src != nullptr && c->pack_src == W) ? c->pack : nullptr;
  g.hid = static_cast<const uint16_t*>(hid);
  g.row_list = c->row_list;
  g.n_act_ptr = c->n_act;
  g.logits = out;
  g.grp_max = c->grp_max;
  g.grp_sum = c->grp_sum;
  g.H = c->cfg.H;
  g.V = c->cfg.V;
  g.ngrp = c->ngrp;
  g.reverse = (c->cfg.flags & DDD_FLAG_FORWARD_SWEEPS) ? 0 : reverse;
  g.epi = kGemmLogits;
  g.out16 = nullptr;
  g.out16b = nullptr;
  g.ld16 = 0;
  DDD_HIP(launch_lmhead_gemm(g, max_rows, c->g_grid, s));
  return DDD_OK;
}

// Slices of the path that handles n_rows rows (0 = dense results of the GEMM path).
// Wide beams always take the GEMM path: the weight stream keeps at most DDD_KMAX keys per row.
bool gemm_path(const ddd_ctx* c, int n_rows) { return n_rows > DDD_STREAM_ROWS || c->cfg.k > DDD_KMAX; }
int slices_for(const ddd_ctx* c, int n_rows) { return gemm_path(c, n_rows) ? 0 : c->nslice; }

// LM head over n_rows rows, partials into the context scratch: the weight stream for up to
// DDD_STREAM_ROWS rows, the MFMA GEMM over the compacted active rows otherwise.
// list_ready: the previous call's bookkeeping launch has already written the list of active rows (GEMM path).
int enqueue_stream(ddd_ctx* c, const void* W, const void* hid, int n_rows, const uint8_t* row_active, float* logits_dbg,
                   int reverse, hipStream_t s, bool list_ready = false, int trace_step = -1, bool eager_loads = false) {
  if (gemm_path(c, n_rows)) {
    float* out = logits_dbg ? logits_dbg : c->logits;
    if (!list_ready) DDD_HIP(launch_build_row_list(row_active, n_rows, c->row_list, c->n_act, s));
    int rc = enqueue_gemm(c, W, hid, n_rows, out, reverse, s);
    if (rc != DDD_OK) return rc;
    RowTopkArgs t;
    t.logits = out;
    t.grp_max = c->grp_max;
    t.grp_sum = c->grp_sum;
    t.ngrp = c->ngrp;
    t.row_active = row_active;
    t.part_key = c->part_key;
    t.part_sum = c->part_sum;
    t.n_rows = n_rows;
    t.V = c->cfg.V;
    t.k = c->cfg.k;
    DDD_HIP(launch_row_topk(t, s));
    return DDD_OK;
  }
  for (int r0 = 0; r0 < n_rows; r0 += DDD_STREAM_ROWS) {
    StreamArgs a;
    a.W = static_cast<const uint16_t*>(W);
    a.hid = static_cast<const uint16_t*>(hid) + (size_t)r0 * c->cfg.H;
    a.row_active = row_active ? row_active + r0 : nullptr;
    a.part_key = c->part_key + (size_t)r0 * c->nslice * c->cfg.k;
    a.part_sum = c->part_sum + (size_t)r0 * c->nslice;
    a.logits_dbg = logits_dbg ? logits_dbg + (size_t)r0 * c->cfg.V : nullptr;
    a.H = c->cfg.H;
    a.V = c->cfg.V;
    a.R = (n_rows - r0 < DDD_STREAM_ROWS) ? (n_rows - r0) : DDD_STREAM_ROWS;
    a.k = c->cfg.k;
    a.ntiles = c->ntiles;
    a.nw = c->nw;
    a.reverse = (c->cfg.flags & DDD_FLAG_FORWARD_SWEEPS) ? 0 : reverse;
    a.eager_loads = eager_loads ? 1 : 0;
    a.trace = (c->trace != nullptr && trace_step >= 0 && r0 == 0) ? c->trace + (size_t)trace_step * kTraceCallWords : nullptr;
    DDD_HIP(launch_lmhead_stream(a, c->G, c->nslice, s));
  }
  return DDD_OK;
}

}  // namespace

extern "C" {

const char* ddd_strerror(int code) {
  switch (code) {
    case DDD_OK: return "ok";
    case DDD_ERR_INVALID_ARG: return "invalid argument";
    case DDD_ERR_NO_DEVICE: return "no HIP device";
    case DDD_ERR_WRONG_ARCH: return "device is not gfx950";
    case DDD_ERR_HIP: return "HIP runtime error";
    case DDD_ERR_UNIMPLEMENTED: return "not implemented";
    case DDD_ERR_STATE: return "call not valid in the current state";
    case DDD_ERR_STATIC_LIMIT: return "size beyond the static scratch of the allocation-free entry point";
    default: return "unknown status";
  }
}

const char* ddd_last_hip_error(void) { return g_hip_err; }

int ddd_config_validate(const ddd_config* cfg) {
  if (cfg == nullptr) return DDD_ERR_INVALID_ARG;
  if (cfg->B < 1 || cfg->B > DDD_BMAX) return DDD_ERR_INVALID_ARG;
  if (cfg->k < 1 || cfg->k > DDD_KWIDE_MAX) return DDD_ERR_INVALID_ARG;
  const bool wide = cfg->k > DDD_KMAX;
  if (cfg->V < cfg->k || cfg->V >= (1 << 24)) return DDD_ERR_INVALID_ARG;
  // the GEMM path (more than DDD_STREAM_ROWS rows, or wide beams) keeps per-row statistics of at most
  // 2048 groups of 64 vocabulary rows; wide beam keys hold the token in 18 bits
  if ((wide || (long long)cfg->B * cfg->k > DDD_STREAM_ROWS) && cfg->V > (1 << 17)) return DDD_ERR_INVALID_ARG;
  // the MFMA path addresses the hidden rows by 32-bit byte offsets
  if ((wide || (long long)cfg->B * cfg->k > DDD_STREAM_ROWS) && (long long)cfg->B * cfg->k * cfg->H * 2 >= (1LL << 32))
    return DDD_ERR_INVALID_ARG;
  if (cfg->max_depth < 1 || cfg->max_depth > DDD_DMAX) return DDD_ERR_INVALID_ARG;
  if (cfg->m < 1 || cfg->m > DDD_MMAX) return DDD_ERR_INVALID_ARG;
  if (!(cfg->threshold >= 0.0f)) return DDD_ERR_INVALID_ARG;   // also rejects NaN
  if ((cfg->flags & ~(DDD_FLAG_FORWARD_SWEEPS | DDD_FLAG_POISON_SCRATCH)) != 0) return DDD_ERR_INVALID_ARG;
  int G, nw;
  if (cfg->H < 128 || !pick_split(cfg->H, &G, &nw)) return DDD_ERR_INVALID_ARG;
  const long long nmax = 1LL + cfg->k + (long long)(cfg->max_depth - 1) * cfg->k * cfg->k;
  if (nmax > (wide ? DDD_POOL_WIDE_MAX : DDD_POOL_MAX)) return DDD_ERR_INVALID_ARG;
  return DDD_OK;
}

size_t ddd_pool_capacity(const ddd_config* cfg) {
  if (ddd_config_validate(cfg) != DDD_OK) return 0;
  return (size_t)1 + cfg->k + (size_t)(cfg->max_depth - 1) * cfg->k * cfg->k;
}

size_t ddd_scratch_bytes(const ddd_config* cfg) {
  if (ddd_config_validate(cfg) != DDD_OK) return 0;
  const size_t rows = (size_t)cfg->B * cfg->k, max_slices = (cfg->k > DDD_KMAX) ? 1 : 512;
  size_t n = rows * max_slices * cfg->k * sizeof(uint64_t) + rows * max_slices * sizeof(float) + rows * 4 + 4;
  if (rows > DDD_STREAM_ROWS || cfg->k > DDD_KMAX)   // logits and per-group statistics of the GEMM path
    n += rows * (size_t)cfg->V * sizeof(float) + 2 * rows * (size_t)(((cfg->V + 63) / 64 + 3) & ~3) * sizeof(float);
  return n;
}

int ddd_create(const ddd_config* cfg, ddd_ctx** out) {
  if (out == nullptr) return DDD_ERR_INVALID_ARG;
  *out = nullptr;
  if (ddd_config_validate(cfg) != DDD_OK) return DDD_ERR_INVALID_ARG;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    return DDD_ERR_NO_DEVICE;
  }
  int dev = 0;
  DDD_HIP(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  DDD_HIP(hipGetDeviceProperties(&prop, dev));
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return DDD_ERR_WRONG_ARCH;

  ddd_ctx* c = new (std::nothrow) ddd_ctx();
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  c->cfg = *cfg;
  c->device = dev;
  c->n_cu = prop.multiProcessorCount;
  pick_split(cfg->H, &c->G, &c->nw);
  c->ntiles = (cfg->V + 15) / 16;
  c->nslice = c->n_cu < 256 ? c->n_cu : 256;   // the per-row merge takes four slices per lane
  if (c->nslice > c->ntiles) c->nslice = c->ntiles;
  c->nmax = (int)ddd_pool_capacity(cfg);
  c->graph = nullptr;
  c->graph_exec = nullptr;
  c->g_grid = ((c->n_cu + 7) / 8) * 8;
  c->logits = nullptr;
  c->grp_max = nullptr;
  c->grp_sum = nullptr;
  c->pack_src = nullptr;
  c->pack = nullptr;
  c->ngrp = ((cfg->V + 63) / 64 + 3) & ~3;
  const size_t rows = (size_t)cfg->B * cfg->k;
  const size_t ns = (cfg->k > DDD_KMAX) ? 1 : (size_t)c->nslice;   // wide beams only use the dense format
  c->part_key_bytes = rows * ns * cfg->k * sizeof(uint64_t);
  c->part_sum_bytes = rows * ns * sizeof(float);
  c->logits_bytes = c->grp_bytes = 0;
  hipError_t e = hipMalloc(&c->part_key, c->part_key_bytes);
  if (e == hipSuccess) e = hipMalloc(&c->part_sum, c->part_sum_bytes);
  if (e == hipSuccess) e = hipMalloc(&c->row_list, rows * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(&c->n_act, sizeof(int32_t));
  if (e == hipSuccess && (rows > DDD_STREAM_ROWS || cfg->k > DDD_KMAX)) {
    c->logits_bytes = rows * (size_t)cfg->V * sizeof(float);
    c->grp_bytes = rows * (size_t)c->ngrp * sizeof(float);
    e = hipMalloc(&c->logits, c->logits_bytes);
    if (e == hipSuccess) e = hipMalloc(&c->grp_max, c->grp_bytes);
    if (e == hipSuccess) e = hipMalloc(&c->grp_sum, c->grp_bytes);
    if (e == hipSuccess) e = prepare_lmhead_gemm();
    if (e == hipSuccess && cfg->k > DDD_KMAX) e = prepare_wide();
  }
  if (e == hipSuccess) e = prepare_tree_attention();
  c->call_count = nullptr;
  c->active_mask = nullptr;
  c->stats_sync = nullptr;
  c->stats_on = false;
  c->stats = ddd_round_stats{nullptr, nullptr, nullptr, nullptr, nullptr};
  c->progress = nullptr;
  c->progress_dev = nullptr;
  c->round_tag = 0;
  c->run_rounds = c->run_waits = c->run_timeouts = 0;
  c->run_max_wait_us = 0.0;
  c->trace = nullptr;
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->call_count), (DDD_DMAX + 1) * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(c->call_count, 0, (DDD_DMAX + 1) * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->stats_sync), 2 * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(c->stats_sync, 0, 2 * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->active_mask), (DDD_BMAX / 64) * sizeof(uint64_t));
  if (e == hipSuccess) e = hipMemset(c->active_mask, 0, (DDD_BMAX / 64) * sizeof(uint64_t));
  void* host_words = nullptr;
  if (e == hipSuccess)
    e = hipHostMalloc(&host_words, (DDD_DMAX + 1) * sizeof(uint32_t), hipHostMallocMapped | hipHostMallocCoherent);
  if (e == hipSuccess) {
    std::memset(host_words, 0, (DDD_DMAX + 1) * sizeof(uint32_t));
    c->progress = static_cast<volatile uint32_t*>(host_words);
    void* dev_words = nullptr;
    e = hipHostGetDevicePointer(&dev_words, host_words, 0);
    c->progress_dev = static_cast<uint32_t*>(dev_words);
  }
  if (e != hipSuccess) {
    if (c->call_count) (void)hipFree(c->call_count);
    if (c->active_mask) (void)hipFree(c->active_mask);
    if (c->stats_sync) (void)hipFree(c->stats_sync);
    if (host_words) (void)hipHostFree(host_words);
    if (c->logits) (void)hipFree(c->logits);
    if (c->grp_max) (void)hipFree(c->grp_max);
    if (c->grp_sum) (void)hipFree(c->grp_sum);
    if (c->part_key) (void)hipFree(c->part_key);
    if (c->part_sum) (void)hipFree(c->part_sum);
    if (c->row_list) (void)hipFree(c->row_list);
    if (c->n_act) (void)hipFree(c->n_act);
    delete c;
    return hip_fail(e, "context scratch");
  }
  *out = c;
  return DDD_OK;
}

int ddd_destroy(ddd_ctx* c) {
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  if (c->graph) (void)hipGraphDestroy(c->graph);
  (void)hipFree(c->part_key);
  (void)hipFree(c->part_sum);
  (void)hipFree(c->row_list);
  (void)hipFree(c->n_act);
  if (c->logits) (void)hipFree(c->logits);
  if (c->grp_max) (void)hipFree(c->grp_max);
  if (c->grp_sum) (void)hipFree(c->grp_sum);
  if (c->pack) (void)hipFree(c->pack);
  if (c->trace) (void)hipFree(c->trace);
  (void)hipFree(c->call_count);
  (void)hipFree(c->active_mask);
  (void)hipFree(c->stats_sync);
  (void)hipHostFree(const_cast<uint32_t*>(c->progress));
  delete c;
  return DDD_OK;
}

int ddd_weights_pack(ddd_ctx* c, const void* W, void* stream) {
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  c->pack_src = nullptr;
  if (W == nullptr) {   // forget the copy and give its memory back
    if (c->pack) DDD_HIP(hipFree(c->pack));
    c->pack = nullptr;
    return DDD_OK;
  }
  if (c->pack == nullptr) {
    const size_t elems = (size_t)((c->cfg.V + 255) / 256) * 256 * (size_t)c->cfg.H;
    DDD_HIP(hipMalloc(reinterpret_cast<void**>(&c->pack), elems * sizeof(uint16_t)));
  }
  DDD_HIP(launch_pack_weights(static_cast<const uint16_t*>(W), c->pack, c->cfg.V, c->cfg.H,
                              static_cast<hipStream_t>(stream)));
  c->pack_src = W;
  return DDD_OK;
}

namespace {
// Key splits of the tree attention: about two workgroups per CU, at least eight 32-key chunks per split.
int attn_splits(const ddd_ctx* c, int n_heads, int L) {
  const int T = c->cfg.m + 1, nqt = (T + 63) / 64;
  const int nchunks = (L + 31) / 32 + (T + 31) / 32;
  int ns = (2 * c->n_cu) / (c->cfg.B * n_heads * nqt);
  const int cap = nchunks / 8 > 1 ? nchunks / 8 : 1;
  if (ns > cap) ns = cap;
  if (ns > 64) ns = 64;
  return ns < 1 ? 1 : ns;
}
}  // namespace

size_t ddd_tree_attention_workspace(const ddd_ctx* c, int32_t n_heads, int32_t L) {
  if (c == nullptr || n_heads < 1 || L < 0) return 0;
  const size_t nqt = (size_t)(c->cfg.m + 1 + 63) / 64;
  return (size_t)c->cfg.B * n_heads * nqt * attn_splits(c, n_heads, L) * tree_attention_part_floats() * sizeof(float);
}

int ddd_kv_pack(ddd_ctx* c, const void* k, const void* v, int32_t L, int32_t n_heads, void* k_packed, void* v_packed,
                void* stream) {
  if (c == nullptr || L < 1 || L > (1 << 20) || n_heads < 1 || n_heads > 1024) return DDD_ERR_INVALID_ARG;
  if (k == nullptr || v == nullptr || k_packed == nullptr || v_packed == nullptr) return DDD_ERR_INVALID_ARG;
  DDD_HIP(launch_kv_pack(static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                         static_cast<uint16_t*>(k_packed), static_cast<uint16_t*>(v_packed), c->cfg.B, L, n_heads,
                         static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

int ddd_tree_attention(ddd_ctx* c, const ddd_tree* tree, const void* q, const void* k_tree, const void* vt_tree,
                       const void* k_packed, const void* v_packed, int32_t L, int32_t n_heads, void* workspace,
                       size_t workspace_bytes, float* out, void* stream) {
  if (c == nullptr || !tree_ok(tree) || q == nullptr || k_tree == nullptr || vt_tree == nullptr || out == nullptr ||
      workspace == nullptr)
    return DDD_ERR_INVALID_ARG;
  if (n_heads < 1 || n_heads > 1024 || L < 0 || L > (1 << 20) || (L > 0 && (k_packed == nullptr || v_packed == nullptr)))
    return DDD_ERR_INVALID_ARG;
  if (workspace_bytes < ddd_tree_attention_workspace(c, n_heads, L)) return DDD_ERR_INVALID_ARG;
  TreeAttnArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_tree = static_cast<const uint16_t*>(k_tree);
  a.vt_tree = static_cast<const uint16_t*>(vt_tree);
  a.k_prompt = static_cast<const uint16_t*>(k_packed);
  a.v_prompt = static_cast<const uint16_t*>(v_packed);
  a.mask = tree->mask;
  a.n_sel = tree->n_sel;
  a.part = static_cast<float*>(workspace);
  a.out = out;
  a.B = c->cfg.B;
  a.T = c->cfg.m + 1;
  a.nh = n_heads;
  a.L = L;
  a.Tp = (a.T + 31) & ~31;
  a.nsplit = attn_splits(c, n_heads, L);
  DDD_HIP(launch_tree_attention(a, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

int ddd_num_slices(const ddd_ctx* c) { return c ? c->nslice : DDD_ERR_INVALID_ARG; }

int ddd_profile_lmhead(ddd_ctx* c, const void* W, const void* hid, int32_t n_rows, int32_t iters, float* mean_ms,
                       float* min_ms, void* stream) {
  if (c == nullptr || W == nullptr || hid == nullptr || mean_ms == nullptr || min_ms == nullptr)
    return DDD_ERR_INVALID_ARG;
  if (n_rows < 1 || n_rows > c->cfg.B * c->cfg.k || iters < 1 || iters > 4096) return DDD_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool gemm = gemm_path(c, n_rows);
  if (gemm) DDD_HIP(launch_build_row_list(nullptr, n_rows, c->row_list, c->n_act, s));
  std::vector<hipEvent_t> ev(2 * (size_t)iters, nullptr);
  int rc = DDD_OK;
  for (size_t i = 0; i < ev.size() && rc == DDD_OK; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) rc = DDD_ERR_HIP;
  for (int i = 0; i < iters && rc == DDD_OK; ++i) {
    if (hipEventRecord(ev[2 * i], s) != hipSuccess) rc = DDD_ERR_HIP;
    if (rc == DDD_OK)
      rc = gemm ? enqueue_gemm(c, W, hid, n_rows, c->logits, i & 1, s) : enqueue_stream(c, W, hid, n_rows, nullptr, nullptr, i & 1, s);
    if (rc == DDD_OK && hipEventRecord(ev[2 * i + 1], s) != hipSuccess) rc = DDD_ERR_HIP;
  }
  if (rc == DDD_OK && hipEventSynchronize(ev[2 * (size_t)iters - 1]) != hipSuccess) rc = DDD_ERR_HIP;
  if (rc == DDD_OK) {
    double sum = 0.0;
    float mn = 1e30f;
    for (int i = 0; i < iters; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess) {
        rc = DDD_ERR_HIP;
        break;
      }
      sum += ms;
      mn = ms < mn ? ms : mn;
    }
    *mean_ms = (float)(sum / iters);
    *min_ms = mn;
  }
  for (hipEvent_t e : ev)
    if (e) (void)hipEventDestroy(e);
  return rc;
}

int ddd_trace_enable(ddd_ctx* c, int32_t on) {
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  DDD_HIP(hipDeviceSynchronize());   // no kernel in flight holds the old pointer
  const size_t bytes = (size_t)(DDD_DMAX + 1) * kTraceCallWords * sizeof(uint64_t);
  if (on) {
    if (c->trace == nullptr) DDD_HIP(hipMalloc(reinterpret_cast<void**>(&c->trace), bytes));
    DDD_HIP(hipMemset(c->trace, 0, bytes));
  } else if (c->trace != nullptr) {
    DDD_HIP(hipFree(c->trace));
    c->trace = nullptr;
  }
  return DDD_OK;
}

int ddd_trace_read(ddd_ctx* c, uint64_t* out, size_t n_words) {
  if (c == nullptr || out == nullptr) return DDD_ERR_INVALID_ARG;
  if (c->trace == nullptr) return DDD_ERR_STATE;
  const size_t total = (size_t)(DDD_DMAX + 1) * kTraceCallWords;
  if (n_words != total) return DDD_ERR_INVALID_ARG;
  DDD_HIP(hipDeviceSynchronize());
  DDD_HIP(hipMemcpy(out, c->trace, total * sizeof(uint64_t), hipMemcpyDeviceToHost));
  DDD_HIP(hipMemset(c->trace, 0, total * sizeof(uint64_t)));
  return DDD_OK;
}

size_t ddd_trace_words(void) { return (size_t)(DDD_DMAX + 1) * kTraceCallWords; }

int ddd_round_reset(ddd_ctx* c, ddd_state* st, const int32_t* root_token, void* stream) {
  if (c == nullptr || !state_ok(st)) return DDD_ERR_INVALID_ARG;
  ResetArgs a;
  a.st = *st;
  a.root_token = root_token;
  a.B = c->cfg.B;
  a.k = c->cfg.k;
  a.nmax = c->nmax;
  DDD_HIP(launch_round_reset(a, static_cast<hipStream_t>(stream)));
  if (c->cfg.flags & DDD_FLAG_POISON_SCRATCH) {
    // debugging aid: nothing a round reads from the context's scratch may predate the round
    hipStream_t s = static_cast<hipStream_t>(stream);
    DDD_HIP(launch_poison(c->part_key, c->part_key_bytes, s));
    DDD_HIP(launch_poison(c->part_sum, c->part_sum_bytes, s));
    if (c->logits != nullptr) {
      DDD_HIP(launch_poison(c->logits, c->logits_bytes, s));
      DDD_HIP(launch_poison(c->grp_max, c->grp_bytes, s));
      DDD_HIP(launch_poison(c->grp_sum, c->grp_bytes, s));
    }
    DDD_HIP(launch_poison(c->row_list, (size_t)c->cfg.B * c->cfg.k * sizeof(int32_t), s));
  }
  return DDD_OK;
}

int ddd_lmhead_topk(ddd_ctx* c, const void* W, const void* hid, int32_t n_rows, const uint8_t* row_active,
                    int32_t* topk_token, float* topk_logprob, float* lse, float* logits_dbg, void* stream) {
  if (c == nullptr || W == nullptr || hid == nullptr || topk_token == nullptr || topk_logprob == nullptr ||
      lse == nullptr)
    return DDD_ERR_INVALID_ARG;
  if (n_rows < 1 || n_rows > c->cfg.B * c->cfg.k) return DDD_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int rc = enqueue_stream(c, W, hid, n_rows, row_active, logits_dbg, 0, s);
  if (rc != DDD_OK) return rc;
  MergeArgs m;
  m.part_key = c->part_key;
  m.part_sum = c->part_sum;
  m.row_active = row_active;
  m.topk_token = topk_token;
  m.topk_logprob = topk_logprob;
  m.lse = lse;
  m.n_rows = n_rows;
  m.nslice = slices_for(c, n_rows);
  m.k = c->cfg.k;
  DDD_HIP(launch_merge(m, s));
  return DDD_OK;
}

int ddd_beam_select(ddd_ctx* c, int32_t step, const int32_t* topk_token, const float* topk_logprob, ddd_state* st,
                    void* stream) {
  if (c == nullptr || topk_token == nullptr || topk_logprob == nullptr || !state_ok(st)) return DDD_ERR_INVALID_ARG;
  if (step < 0 || step >= c->cfg.max_depth) return DDD_ERR_INVALID_ARG;
  BeamArgs a = beam_args(c, st, step);
  a.topk_token = topk_token;
  a.topk_logprob = topk_logprob;
  if (c->cfg.k > DDD_KMAX) {
    WideStepArgs w = wide_args(c, a);
    w.do_select = 1;
    DDD_HIP(launch_step_wide(w, static_cast<hipStream_t>(stream)));
    return DDD_OK;
  }
  DDD_HIP(launch_beam_select(a, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

int ddd_depth_continue(ddd_ctx* c, int32_t steps_done, ddd_state* st, void* stream) {
  if (c == nullptr || !state_ok(st)) return DDD_ERR_INVALID_ARG;
  if (steps_done < 1 || steps_done > c->cfg.max_depth) return DDD_ERR_INVALID_ARG;
  BeamArgs a = beam_args(c, st, steps_done - 1);
  if (c->cfg.k > DDD_KMAX) {
    WideStepArgs w = wide_args(c, a);
    w.do_stop = 1;
    w.steps_done = steps_done;
    DDD_HIP(launch_step_wide(w, static_cast<hipStream_t>(stream)));
    return DDD_OK;
  }
  DDD_HIP(launch_depth_continue(a, steps_done, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

}  // extern "C"

namespace {

// One draft call; publish: the bookkeeping launch also reports to c->progress[step] (ddd_round_run); in_round: the
// call is one of a round's consecutive calls 0, 1, 2, ... on this context, so on the GEMM path its bookkeeping
// launch leaves the next call's list of active rows behind and calls after the first do not build their own.
int draft_step(ddd_ctx* c, int32_t step, const void* W, const void* hid, ddd_state* st, ddd_tree* tree,
               float* logits_dbg, float* lse_dbg, bool publish, bool in_round, void* stream) {
  if (c == nullptr || W == nullptr || hid == nullptr || !state_ok(st)) return DDD_ERR_INVALID_ARG;
  if (tree != nullptr && !tree_ok(tree)) return DDD_ERR_INVALID_ARG;
  if (step < 0 || step >= c->cfg.max_depth) return DDD_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n_rows = (step == 0) ? c->cfg.B : c->cfg.B * c->cfg.k;
  // step 0 rows are one per sequence: active[] is the row flag; later rows use row_active[]
  const uint8_t* flags = (step == 0) ? st->active : st->row_active;
  StepArgs a;
  a.beam = beam_args(c, st, step);
  a.part_key = c->part_key;
  a.part_sum = c->part_sum;
  a.lse_dbg = lse_dbg;
  if (tree != nullptr)
    a.tree = *tree;
  else
    std::memset(&a.tree, 0, sizeof(a.tree));
  a.nslice = slices_for(c, n_rows);
  a.m = c->cfg.m;
  // rows of the calls after the prompt call go through the GEMM path and beams are narrow: the lists chain
  const bool chain = in_round && c->cfg.k <= DDD_KMAX && gemm_path(c, c->cfg.B * c->cfg.k);
  a.call_count = (publish || chain) ? c->call_count + step : nullptr;
  a.progress = publish ? c->progress_dev + step : nullptr;
  a.round_tag = c->round_tag;
  a.active_mask = chain ? c->active_mask : nullptr;
  a.next_row_list = c->row_list;
  a.next_n_act = c->n_act;
  a.trace = c->trace ? c->trace + (size_t)step * kTraceCallWords + DDD_STATIC_SLICES * kTraceStreamWords : nullptr;
  // publish = the host-paced round: it queues at most one call per round that every sequence skips
  int rc = enqueue_stream(c, W, hid, n_rows, flags, logits_dbg, step & 1, s, chain && step >= 1, step, publish);
  if (rc != DDD_OK) return rc;
  if (c->cfg.k > DDD_KMAX) {
    WideStepArgs w = wide_args(c, a.beam);
    w.part_key = c->part_key;
    w.part_lse = c->part_sum;
    w.lse_dbg = lse_dbg;
    w.tree = a.tree;
    w.do_select = 1;
    w.do_stop = 1;
    w.call_count = publish ? c->call_count + step : nullptr;
    w.progress = publish ? c->progress_dev + step : nullptr;
    w.round_tag = c->round_tag;
    DDD_HIP(launch_step_wide(w, s));
    return DDD_OK;
  }
  DDD_HIP(launch_step_bookkeep(a, s));
  return DDD_OK;
}

}  // namespace

extern "C" {

int ddd_draft_step(ddd_ctx* c, int32_t step, const void* W, const void* hid, ddd_state* st, ddd_tree* tree,
                   float* logits_dbg, float* lse_dbg, void* stream) {
  return draft_step(c, step, W, hid, st, tree, logits_dbg, lse_dbg, false, false, stream);
}

int ddd_tree_finalize(ddd_ctx* c, const ddd_state* st, ddd_tree* out, void* stream) {
  if (c == nullptr || !state_ok(st) || !tree_ok(out)) return DDD_ERR_INVALID_ARG;
  FinalizeArgs a;
  a.st = *st;
  a.tree = *out;
  a.B = c->cfg.B;
  a.k = c->cfg.k;
  a.m = c->cfg.m;
  a.nmax = c->nmax;
  if (c->nmax > DDD_POOL_MAX)
    DDD_HIP(launch_tree_finalize_wide(a, static_cast<hipStream_t>(stream)));
  else
    DDD_HIP(launch_tree_finalize(a, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

namespace {
StatsArgs stats_args(const ddd_ctx* c) {
  StatsArgs s{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  if (c->stats_on) {
    s.rounds = c->stats.rounds;
    s.depth_hist = c->stats.depth_hist;
    s.accept_hist = c->stats.accept_hist;
    s.batch_depth_hist = c->stats.batch_depth_hist;
    s.steps = c->stats.steps;
    s.sync = c->stats_sync;
  }
  return s;
}
}  // namespace

int ddd_stats_bind(ddd_ctx* c, const ddd_round_stats* stats) {
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  if (stats == nullptr) {
    c->stats_on = false;
    return DDD_OK;
  }
  c->stats = *stats;
  c->stats_on = stats->rounds != nullptr || stats->depth_hist != nullptr || stats->accept_hist != nullptr ||
                stats->batch_depth_hist != nullptr;
  return DDD_OK;
}

int ddd_verify_accept(ddd_ctx* c, const ddd_tree* tree, const int32_t* target_argmax, int32_t* accept_len,
                      int32_t* accept_path, int32_t* bonus_token, void* stream) {
  if (c == nullptr || !tree_ok(tree) || target_argmax == nullptr || accept_len == nullptr || accept_path == nullptr ||
      bonus_token == nullptr)
    return DDD_ERR_INVALID_ARG;
  VerifyArgs a;
  a.tree = *tree;
  a.stats = stats_args(c);
  a.target_argmax = target_argmax;
  a.accept_len = accept_len;
  a.accept_path = accept_path;
  a.bonus_token = bonus_token;
  a.B = c->cfg.B;
  a.m = c->cfg.m;
  a.D = c->cfg.max_depth;
  DDD_HIP(launch_verify_accept(a, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

int ddd_verify_sample(ddd_ctx* c, const ddd_tree* tree, const float* target_logits, float temperature,
                      const double* u_accept, const double* u_bonus, int32_t* accept_len, int32_t* accept_path,
                      int32_t* bonus_token, void* stream) {
  if (c == nullptr || !tree_ok(tree) || target_logits == nullptr || u_accept == nullptr || u_bonus == nullptr ||
      accept_len == nullptr || accept_path == nullptr || bonus_token == nullptr)
    return DDD_ERR_INVALID_ARG;
  if (!(temperature > 0.0f) || !(temperature < 3.0e38f)) return DDD_ERR_INVALID_ARG;
  VerifySampleArgs a;
  a.tree = *tree;
  a.stats = stats_args(c);
  a.logits = target_logits;
  a.u_accept = u_accept;
  a.u_bonus = u_bonus;
  a.accept_len = accept_len;
  a.accept_path = accept_path;
  a.bonus_token = bonus_token;
  a.temperature = temperature;
  a.B = c->cfg.B;
  a.m = c->cfg.m;
  a.D = c->cfg.max_depth;
  a.V = c->cfg.V;
  DDD_HIP(launch_verify_sample(a, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

namespace {
// Where a round builds the final trees.  Inside the bookkeeping launch of the call in which a sequence stops
// (no extra launch: right for a few sequences), or in one launch after the last call (with many sequences
// almost every call has some sequence stopping, and the slowest workgroup sets the time of the launch: the
// tree building would be on the critical path of every call).  A stopped sequence's pool no longer changes,
// so both give the same trees.
bool trees_after_the_calls(const ddd_ctx* c) { return c->cfg.B >= 8; }
// Limits of ddd_round_run's host waits for a draft call's report.
constexpr int kWaitMs = 20, kFirstWaitMs = 1000;
}  // namespace

int ddd_round_enqueue(ddd_ctx* c, const void* W, ddd_state* st, ddd_tree* tree, const int32_t* root_token,
                      void* hid_buf, ddd_draft_body_fn body, void* body_user, ddd_post_fn post, void* post_user,
                      float* logits_dbg, float* lse_dbg, void* stream) {
  if (c == nullptr || W == nullptr || !state_ok(st) || !tree_ok(tree) || hid_buf == nullptr || body == nullptr)
    return DDD_ERR_INVALID_ARG;
  int rc = ddd_round_reset(c, st, root_token, stream);
  if (rc != DDD_OK) return rc;
  const size_t dbg_stride = (size_t)c->cfg.B * c->cfg.k * c->cfg.V;
  const bool late_trees = trees_after_the_calls(c);
  for (int step = 0; step < c->cfg.max_depth; ++step) {
    rc = body(body_user, step, st, hid_buf, stream);
    if (rc != DDD_OK) return rc;
    rc = draft_step(c, step, W, hid_buf, st, late_trees ? nullptr : tree,
                    logits_dbg ? logits_dbg + dbg_stride * step : nullptr,
                    lse_dbg ? lse_dbg + (size_t)c->cfg.B * c->cfg.k * step : nullptr, false, true, stream);
    if (rc != DDD_OK) return rc;
  }
  if (late_trees) {
    rc = ddd_tree_finalize(c, st, tree, stream);
    if (rc != DDD_OK) return rc;
  }
  if (post != nullptr) rc = post(post_user, st, tree, stream);
  return rc;
}

int ddd_round_run(ddd_ctx* c, const void* W, ddd_state* st, ddd_tree* tree, const int32_t* root_token, void* hid_buf,
                  ddd_draft_body_fn body, void* body_user, ddd_post_fn post, void* post_user, void* stream) {
  if (c == nullptr || W == nullptr || !state_ok(st) || !tree_ok(tree) || hid_buf == nullptr || body == nullptr)
    return DDD_ERR_INVALID_ARG;
  const bool publish = true;
  c->round_tag = (c->round_tag + 1) & 0x3FFFFFFFu;
  if (c->round_tag == 0) c->round_tag = 1;
  int rc = ddd_round_reset(c, st, root_token, stream);
  if (rc != DDD_OK) return rc;
  const bool late_trees = trees_after_the_calls(c);
  int enqueued = 0;
  bool wait = publish;
  ++c->run_rounds;
  for (int step = 0; step < c->cfg.max_depth; ++step) {
    if (wait && step >= 2) {
      // Call step-1 is already in the queue; call `step` goes in once call step-2 has reported that
      // some sequence goes on.  The wait is bounded, so a stalled device cannot hang the host: when the
      // limit passes the rest is enqueued unconditionally (the device-side flags skip what is not needed)
      // and the expiry is counted (ddd_round_run_stats).  The first wait of a round also covers whatever
      // the stream still held when the round was queued, so its limit is the long one.
      const uint32_t want = c->round_tag << 2;
      const auto limit = std::chrono::milliseconds(step == 2 ? kFirstWaitMs : kWaitMs);
      const auto t0 = std::chrono::steady_clock::now();
      uint32_t v = c->progress[step - 2];
      for (unsigned spin = 0; (v & ~3u) != want; ++spin) {
        if ((spin & 1023u) == 1023u && std::chrono::steady_clock::now() - t0 > limit) {
          // the thread may have been off the CPU for most of that time: look once more before giving up
          v = c->progress[step - 2];
          if ((v & ~3u) != want) wait = false;
          break;
        }
        v = c->progress[step - 2];
      }
      const double waited_us =
          std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
      ++c->run_waits;
      if (waited_us > c->run_max_wait_us) c->run_max_wait_us = waited_us;
      if (!wait) ++c->run_timeouts;
      if (wait && (v & 1u) == 0u) break;           // every sequence has stopped
    }
    rc = body(body_user, step, st, hid_buf, stream);
    if (rc != DDD_OK) return rc;
    rc = draft_step(c, step, W, hid_buf, st, late_trees ? nullptr : tree, nullptr, nullptr, publish, true, stream);
    if (rc != DDD_OK) return rc;
    ++enqueued;
  }
  if (late_trees) {
    rc = ddd_tree_finalize(c, st, tree, stream);
    if (rc != DDD_OK) return rc;
  }
  if (post != nullptr) {
    rc = post(post_user, st, tree, stream);
    if (rc != DDD_OK) return rc;
  }
  return enqueued;
}

int ddd_round_run_stats(const ddd_ctx* c, uint64_t* rounds, uint64_t* waits, uint64_t* timeouts, double* max_wait_us) {
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  if (rounds) *rounds = c->run_rounds;
  if (waits) *waits = c->run_waits;
  if (timeouts) *timeouts = c->run_timeouts;
  if (max_wait_us) *max_wait_us = c->run_max_wait_us;
  return DDD_OK;
}

int ddd_round_capture(ddd_ctx* c, const void* W, ddd_state* st, ddd_tree* tree, const int32_t* root_token,
                      void* hid_buf, ddd_draft_body_fn body, void* body_user, ddd_post_fn post, void* post_user,
                      float* logits_dbg, float* lse_dbg, void* stream) {
  if (c == nullptr || stream == nullptr) return DDD_ERR_INVALID_ARG;
  if (W == nullptr || !state_ok(st) || !tree_ok(tree) || hid_buf == nullptr || body == nullptr)
    return DDD_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  DDD_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
  int rc = ddd_round_enqueue(c, W, st, tree, root_token, hid_buf, body, body_user, post, post_user, logits_dbg,
                             lse_dbg, stream);
  hipGraph_t g = nullptr;
  hipError_t e = hipStreamEndCapture(s, &g);
  if (rc != DDD_OK) {
    if (g) (void)hipGraphDestroy(g);
    return rc;
  }
  if (e != hipSuccess) return hip_fail(e, "hipStreamEndCapture");
  hipGraphExec_t ge = nullptr;
  e = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    (void)hipGraphDestroy(g);
    return hip_fail(e, "hipGraphInstantiate");
  }
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  if (c->graph) (void)hipGraphDestroy(c->graph);
  c->graph = g;
  c->graph_exec = ge;
  return DDD_OK;
}

int ddd_round_launch(ddd_ctx* c, void* stream) {
  if (c == nullptr) return DDD_ERR_INVALID_ARG;
  if (c->graph_exec == nullptr) return DDD_ERR_STATE;
  DDD_HIP(hipGraphLaunch(c->graph_exec, static_cast<hipStream_t>(stream)));
  return DDD_OK;
}

}  // extern "C"

// ---- allocation-free entry point ------------------------------------------------------------------
// The per-slice partial results of the weight stream (what a context keeps in memory it allocated) in a
// file-scope device array instead: DDD_STATIC_ROWS rows x DDD_KMAX ranks x DDD_STATIC_SLICES slices of
// 64-bit keys, then the slices' sums of exponentials.  Every device the library runs on holds its own copy
// until the process ends.
#define DDD_STATIC_KEY_BYTES ((size_t)DDD_STATIC_ROWS * DDD_KMAX * DDD_STATIC_SLICES * sizeof(uint64_t))
#define DDD_STATIC_SUM_BYTES ((size_t)DDD_STATIC_ROWS * DDD_STATIC_SLICES * sizeof(float))

static __device__ __align__(256) unsigned char scratch[DDD_STATIC_KEY_BYTES + DDD_STATIC_SUM_BYTES];

namespace {

constexpr size_t kStaticKeyBytes = DDD_STATIC_KEY_BYTES;
constexpr size_t kStaticBytes = DDD_STATIC_KEY_BYTES + DDD_STATIC_SUM_BYTES;

// In host code `scratch` is only a handle for the runtime: the array's device address is looked up once per
// device (with that device current) and host code uses nothing but that address.
constexpr int kMaxDevices = 64;
struct StaticDevice {
  bool ready;
  unsigned char* ptr;   // device address of `scratch` on this device
  int n_cu;
};
StaticDevice g_static[kMaxDevices];
std::mutex g_static_mutex;

// The current device's entry, set up on first use.  DDD_OK, or why the device cannot be used.
int static_device(StaticDevice* out) {
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    return DDD_ERR_NO_DEVICE;
  }
  int dev = 0;
  DDD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DDD_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticDevice& d = g_static[dev];
  if (!d.ready) {
    hipDeviceProp_t prop;
    DDD_HIP(hipGetDeviceProperties(&prop, dev));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return DDD_ERR_WRONG_ARCH;
    void* p = nullptr;
    DDD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return DDD_ERR_HIP;
    d.ptr = static_cast<unsigned char*>(p);
    d.n_cu = prop.multiProcessorCount;
    d.ready = true;
  }
  *out = d;
  return DDD_OK;
}

}  // namespace

extern "C" {

size_t ddd_static_scratch_bytes(void) { return kStaticBytes; }

int ddd_lmhead_topk_static(const ddd_config* cfg, const void* W, const void* hid, int32_t n_rows,
                           const uint8_t* row_active, int32_t* topk_token, float* topk_logprob, float* lse,
                           void* stream) {
  if (ddd_config_validate(cfg) != DDD_OK) return DDD_ERR_INVALID_ARG;
  if (W == nullptr || hid == nullptr || topk_token == nullptr || topk_logprob == nullptr || lse == nullptr)
    return DDD_ERR_INVALID_ARG;
  if (n_rows < 1) return DDD_ERR_INVALID_ARG;
  if (n_rows > DDD_STATIC_ROWS || cfg->k > DDD_KMAX) return DDD_ERR_STATIC_LIMIT;
  StaticDevice d;
  int rc = static_device(&d);
  if (rc != DDD_OK) return rc;
  int G = 0, nw = 0;
  pick_split(cfg->H, &G, &nw);
  const int ntiles = (cfg->V + 15) / 16;
  int nslice = d.n_cu < DDD_STATIC_SLICES ? d.n_cu : DDD_STATIC_SLICES;   // as a context picks it: same bits
  if (nslice > ntiles) nslice = ntiles;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // Nothing here has to start at zero: the stream kernel writes all k ranks and the sum of every
  // (row < n_rows, slice < nslice), which is exactly what the merge reads; leftovers of earlier calls lie outside.
  uint64_t* part_key = reinterpret_cast<uint64_t*>(d.ptr);
  float* part_sum = reinterpret_cast<float*>(d.ptr + kStaticKeyBytes);
  StreamArgs a;
  a.W = static_cast<const uint16_t*>(W);
  a.hid = static_cast<const uint16_t*>(hid);
  a.row_active = row_active;
  a.part_key = part_key;
  a.part_sum = part_sum;
  a.logits_dbg = nullptr;
  a.H = cfg->H;
  a.V = cfg->V;
  a.R = n_rows;
  a.k = cfg->k;
  a.ntiles = ntiles;
  a.nw = nw;
  a.reverse = 0;
  a.eager_loads = 0;
  a.trace = nullptr;
  DDD_HIP(launch_lmhead_stream(a, G, nslice, s));
  MergeArgs m;
  m.part_key = part_key;
  m.part_sum = part_sum;
  m.row_active = row_active;
  m.topk_token = topk_token;
  m.topk_logprob = topk_logprob;
  m.lse = lse;
  m.n_rows = n_rows;
  m.nslice = nslice;
  m.k = cfg->k;
  DDD_HIP(launch_merge(m, s));
  return DDD_OK;
}

}  // extern "C"
