// libarkv host side: the C ABI of include/arkv.h, argument checks, memory, count policy and the
// order of kernel launches.  No arithmetic of the method runs here except the scalar OQ-ratio /
// budget formulas (eqs. 6-8), which the paper defines on per-layer scalars.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <string>
#include <vector>

#include "arkv.h"
#include "arkv_dev.h"

using namespace arkv;

static thread_local std::string g_hip_error;

static int hip_fail(hipError_t e, const char* what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();
  return ARKV_EHIP;
}
#define HIP_TRY(expr)                                   \
  do {                                                  \
    hipError_t e_ = (expr);                             \
    if (e_ != hipSuccess) return hip_fail(e_, #expr);   \
  } while (0)

struct LayerState {
  bool scored = false, committed = false;
  bool failed = false;          // a launch of a decode step failed half way: the layer must be reset
  int scored_T = 0, T = 0, P = -1, live = 0, n_pending = 0, slot = 0, n_tailors = 0;
  int last_tailor = 0;          // 0 none, 1 at commit (keys in commit scratch), 2 during decode
  float2* pre = nullptr;        // [U][T] window sums from the prefill scorer
  size_t pre_cap = 0;
  std::vector<int32_t> n_o;     // [B] Original target per sequence
  // host mirror of the units' (Original, Quantized) token counts: exact after a commit and while only
  // appends happen; a decode-time tailor makes the split data dependent and invalidates it
  bool cnt_valid = false;
  std::vector<int32_t> cnt_o, cnt_q;   // [U]
  // after a decode-time tailor the counts are copied back asynchronously; the mirror is valid again once
  // the copy has landed (checked without waiting at the following steps)
  int2* cnt_host = nullptr;     // pinned, [U]
  hipEvent_t cnt_ev = nullptr;
  bool cnt_refresh = false;
  int cnt_refresh_P = 0;        // position of the step whose tailor the snapshot follows
};

struct arkv_cache {
  arkv_config cfg;
  Pools P;
  int L = 0, U = 0, b = 0;
  std::vector<LayerState> layers;
  std::vector<void*> allocs;
  // grow-only scratch shared by all layers (calls on one cache are stream-ordered)
  float2* rowstat = nullptr; size_t rowstat_cap = 0;
  float* rowc = nullptr; size_t rowc_cap = 0;
  int* stat_ticket = nullptr;     // [batch], zero between scorer calls
  uint64_t* ckeys = nullptr; size_t ckeys_cap = 0;
  int ckeys_layer = -1, ckeys_T = 0;
  hipStream_t last_stream = nullptr;
  // measurement hook: events around the attention kernel
  int prefill_chunk = 1024; // keys per workgroup of the prefill scorer (halved while the grid would be small)
  bool prefill_chunk_fixed = false;   // set through the launch-shape hook: taken as it is
  int wg_target = 512;      // workgroups per decode launch the split-K factor aims at
  int wq = 0;               // cost of a packed row in sixteenths of a bf16 row; 0 = by launch shape (decode_impl)
  float* attn_outf = nullptr;   // parity hook: fp32 copy of the prefill attention's output (caller's device buffer)
  bool timing = false;
  std::vector<hipEvent_t> ev_pool;   // pairs, reused after every read
  size_t ev_used = 0;
};

static int validate(const arkv_config* c) {
  if (!c) return ARKV_EINVAL;
  if (c->n_layers <= 0 || c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0)
    return ARKV_EINVAL;
  if (c->n_q_heads % c->n_kv_heads != 0) return ARKV_EINVAL;
  if (c->window < 1 || c->capacity_tokens < 3 || c->window >= c->capacity_tokens - 1) return ARKV_EINVAL;
  if (!(c->alpha > 0.0f && c->alpha <= 1.0f) || !(c->gamma >= 0.0f)) return ARKV_EINVAL;
  for (int i = 0; i < 3; ++i)
    if (!(c->tau[i] > 0.0f)) return ARKV_EINVAL;
  if (c->group_size != kGroup) return ARKV_EINVAL;
  if (c->tailor_policy != 0 && c->tailor_policy != 1) return ARKV_EINVAL;
  if (c->budget_mode != 0 && c->budget_mode != 1) return ARKV_EINVAL;
  const int G = c->n_q_heads / c->n_kv_heads;
  if (c->head_dim != 64 && c->head_dim != 128) return ARKV_EUNSUPPORTED;
  if (G != 1 && G != 2 && G != 4 && G != 8) return ARKV_EUNSUPPORTED;
  if (c->quant_bits != 2 && c->quant_bits != 4 && c->quant_bits != 8) return ARKV_EUNSUPPORTED;
  if (G * c->window > 512) return ARKV_EUNSUPPORTED;
  // the decode kernel's split cut points are 32-bit products of a unit's weighted row count and the split count
  // (<= 128); arkv_cache_create repeats the check with the real size of the Quantized pool
  if (c->capacity_tokens > (1 << 20) - 64) return ARKV_EUNSUPPORTED;
  return ARKV_OK;
}

static int survivors_b(const arkv_config* c) {
  const int nw = c->capacity_tokens - c->window;
  int b = c->tailor_policy == 1 ? nw - 1 : (int)floor((double)c->alpha * (double)nw);
  b = std::min(b, nw - 1);
  return std::max(b, 0);
}

template <typename T>
static int dev_alloc(arkv_cache* c, T** p, size_t count) {
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, std::max<size_t>(count, 1) * sizeof(T));
  if (e != hipSuccess) {
    hip_fail(e, "hipMalloc");
    return e == hipErrorOutOfMemory ? ARKV_ENOMEM : ARKV_EHIP;
  }
  c->allocs.push_back(q);
  *p = static_cast<T*>(q);
  return ARKV_OK;
}

template <typename T>
static int grow(T** p, size_t* cap, size_t count) {
  if (count <= *cap) return ARKV_OK;
  if (*p) HIP_TRY(hipFree(*p));
  *p = nullptr; *cap = 0;
  void* q = nullptr;
  hipError_t e = hipMalloc(&q, count * sizeof(T));
  if (e != hipSuccess) { hip_fail(e, "hipMalloc"); return e == hipErrorOutOfMemory ? ARKV_ENOMEM : ARKV_EHIP; }
  *p = static_cast<T*>(q); *cap = count;
  return ARKV_OK;
}

static int flush_and_sync(arkv_cache* c, int layer) {
  LayerState& ls = c->layers[(size_t)layer];
  if (ls.n_pending > 0) {
    HIP_TRY(launch_flush_scores(c->P, layer * c->U, c->U, ls.n_pending, ls.slot, c->last_stream));
    ls.n_pending = 0;
  }
  HIP_TRY(hipStreamSynchronize(c->last_stream));
  return ARKV_OK;
}

template <typename T>
static int fetch(std::vector<T>& h, const T* dev, size_t count) {
  h.resize(count);
  HIP_TRY(hipMemcpy(h.data(), dev, count * sizeof(T), hipMemcpyDeviceToHost));
  return ARKV_OK;
}

extern "C" {

int arkv_config_default(arkv_config* cfg) {
  if (!cfg) return ARKV_EINVAL;
  memset(cfg, 0, sizeof(*cfg));
  cfg->window = 32;
  cfg->alpha = 0.75f;
  cfg->gamma = 263.81f;
  cfg->tau[0] = 7.774f; cfg->tau[1] = 5.407f; cfg->tau[2] = 5.528f;
  cfg->quant_bits = 4;
  cfg->group_size = 32;
  return ARKV_OK;
}

// (C_orig, C_quant) of eq. 1 for one token of one kv-head
static void row_bytes(int d, int bits, int64_t* c_o, int64_t* c_q) {
  *c_o = 4 * (int64_t)d;
  *c_q = bits == 8 ? 2 * ((int64_t)d + 2) : 2 * ((int64_t)d * bits / 8 + ((int64_t)d / kGroup) * 4);
}

int arkv_budget_counts(const arkv_config* cfg, float rho, int32_t* n_o, int32_t* n_q, int32_t* b) {
  if (!cfg || !n_o || !n_q || !b) return ARKV_EINVAL;
  if (cfg->window < 1 || cfg->window >= cfg->capacity_tokens - 1) return ARKV_EINVAL;
  if (!(cfg->alpha > 0.0f && cfg->alpha <= 1.0f) || !(rho >= 0.0f && rho <= 1.0f)) return ARKV_EINVAL;
  const int bb = survivors_b(cfg);
  const int no = std::min((int)floor((double)rho * (double)(cfg->capacity_tokens - cfg->window)), bb);
  if (cfg->budget_mode == 1) {
    if (cfg->head_dim <= 0 || (cfg->quant_bits != 2 && cfg->quant_bits != 4 && cfg->quant_bits != 8)) return ARKV_EINVAL;
    int64_t co, cq;
    row_bytes(cfg->head_dim, cfg->quant_bits, &co, &cq);
    const int64_t nq = (int64_t)(bb - no) * co / cq;
    *n_o = no; *n_q = (int32_t)nq; *b = (int32_t)(no + nq);
    return ARKV_OK;
  }
  *n_o = no; *n_q = bb - no; *b = bb;
  return ARKV_OK;
}

int arkv_oq_ratio(const float* stats, int32_t n_layers, int32_t batch, const float tau[3], float* rho) {
  if (!stats || !tau || !rho || n_layers <= 0 || batch <= 0) return ARKV_EINVAL;
  for (int i = 0; i < 3; ++i)
    if (!(tau[i] > 0.0f)) return ARKV_EINVAL;
  std::vector<double> q((size_t)n_layers);
  for (int s = 0; s < batch; ++s) {
    double mx = 0.0;
    for (int l = 0; l < n_layers; ++l) {
      const float* st = stats + ((size_t)l * batch + s) * 3;
      if (!(st[0] >= 0.0f) || !(st[1] >= 0.0f) || !(st[2] >= 0.0f)) return ARKV_EINVAL;   // also rejects NaN
      q[l] = pow((double)st[0], 1.0 / (double)tau[0]) * pow((double)st[1], 1.0 / (double)tau[1]) *
             pow((double)st[2], 1.0 / (double)tau[2]);
      mx = std::max(mx, q[l]);
    }
    for (int l = 0; l < n_layers; ++l) rho[(size_t)l * batch + s] = mx > 0.0 ? (float)(q[l] / mx) : 1.0f;
  }
  return ARKV_OK;
}

int arkv_cache_create(const arkv_config* cfg, arkv_cache** out) {
  if (!out) return ARKV_EINVAL;
  *out = nullptr;
  int rc = validate(cfg);
  if (rc != ARKV_OK) return rc;
  arkv_cache* c = new (std::nothrow) arkv_cache();
  if (!c) return ARKV_ENOMEM;
  c->cfg = *cfg;
  c->L = cfg->n_layers;
  c->U = cfg->batch * cfg->n_kv_heads;
  c->b = survivors_b(cfg);
  c->layers.resize((size_t)c->L);
  for (auto& ls : c->layers) {
    ls.n_o.assign((size_t)cfg->batch, 0);
    ls.cnt_o.assign((size_t)c->U, 0);
    ls.cnt_q.assign((size_t)c->U, 0);
  }
  Pools& P = c->P;
  memset(&P, 0, sizeof(P));
  P.U = c->U;
  // 17 spare rows per unit: keeps the units' 2^k-byte regions from landing on the same HBM channels
  P.capO = cfg->capacity_tokens + 17;
  {
    int32_t no0, nq0, b0;
    if (arkv_budget_counts(cfg, 0.0f, &no0, &nq0, &b0) != ARKV_OK) { delete c; return ARKV_EINVAL; }
    P.capQ = std::max(b0, 1);             // every survivor may be Quantized
    P.capQv = (P.capQ + kVBlock - 1) / kVBlock * kVBlock;
  }
  // split cut points: (16 capO + 16 capQ + 16 * 32) * 128 must fit 32 bits (byte budgets keep up to
  // C_orig / C_quant times more Quantized rows than the token rule)
  if (((uint64_t)P.capO + (uint64_t)P.capQ + 32u) * 16u * (uint64_t)kMaxSplits > 0xFFFFFFFFull) { delete c; return ARKV_EUNSUPPORTED; }
  P.D = cfg->head_dim;
  P.G = cfg->n_q_heads / cfg->n_kv_heads;
  P.bits = cfg->quant_bits;
  const size_t LU = (size_t)c->L * c->U, D = (size_t)P.D, G = (size_t)P.G;
  const size_t CB = D * P.bits / 8, NG = (size_t)metas_per_row(P.D, P.bits);
  P.fin_stride = LU * G;
  P.plan_stride = kPlanHdr + 3 * P.capO + 2 * P.capQ;
  P.max_splits = std::max(1, std::min(kMaxSplits, (1024 + c->U - 1) / c->U));   // room for launch-shape sweeps
#define A(field, count) if ((rc = dev_alloc(c, &P.field, (count))) != ARKV_OK) { arkv_cache_destroy(c); return rc; }
  A(ok, LU * P.capO * D) A(ov, LU * P.capO * D)
  A(opos, LU * P.capO) A(oacc, LU * P.capO)
  const size_t MH = (size_t)vmeta_per_row(P.D, P.bits);
  A(qkc, LU * P.capQ * CB) A(qvc, LU * P.capQv * CB)
  A(qkm, LU * P.capQ * NG) A(qvm, LU * P.capQv * MH)
  A(qpos, LU * P.capQ) A(qacc, LU * P.capQ)
  A(cnt, LU) A(fin, kRing * LU * G) A(qprev, kRing * LU * G * D) A(qscale, kRing * LU) A(part, LU * (size_t)P.max_splits * G * (D + 2)) A(outf, LU * G * D) A(n_o, LU) A(nb, LU) A(ticket, LU)
  A(keys, LU * (size_t)(P.capO + P.capQ)) A(thr, LU * 2) A(plan, LU * (size_t)P.plan_stride)
#undef A
  hipError_t e = hipSuccess;
  for (auto& ls : c->layers) {
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ls.cnt_host), (size_t)c->U * sizeof(int2), hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ls.cnt_ev, hipEventDisableTiming);
  }
  // value blocks are read whole, stale slots included (their probabilities are zero): what they hold must be finite
  if (e == hipSuccess) e = hipMemset(P.qvc, 0, LU * P.capQv * CB);
  if (e == hipSuccess) e = hipMemset(P.qvm, 0, LU * P.capQv * MH * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMemset(P.cnt, 0, LU * sizeof(int2));
  if (e == hipSuccess) e = hipMemset(P.ticket, 0, LU * sizeof(int));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->stat_ticket), (size_t)c->cfg.batch * sizeof(int));
  if (e == hipSuccess) e = hipMemset(c->stat_ticket, 0, (size_t)c->cfg.batch * sizeof(int));
  if (e == hipSuccess) e = hipMemset(P.fin, 0, kRing * LU * G * sizeof(float2));
  if (e == hipSuccess) e = hipMemset(P.qprev, 0, kRing * LU * G * D * sizeof(uint16_t));
  if (e == hipSuccess) e = hipMemset(P.qscale, 0, kRing * LU * sizeof(float));
  if (e == hipSuccess) e = static_scratch_setup();      // device address of the static split-K scratch
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) { arkv_cache_destroy(c); return hip_fail(e, "cache set-up"); }
  *out = c;
  return ARKV_OK;
}

int arkv_cache_destroy(arkv_cache* c) {
  if (!c) return ARKV_OK;
  (void)hipDeviceSynchronize();
  for (void* p : c->allocs) (void)hipFree(p);
  for (auto& ls : c->layers) {
    if (ls.pre) (void)hipFree(ls.pre);
    if (ls.cnt_host) (void)hipHostFree(ls.cnt_host);
    if (ls.cnt_ev) (void)hipEventDestroy(ls.cnt_ev);
  }
  if (c->rowstat) (void)hipFree(c->rowstat);
  if (c->rowc) (void)hipFree(c->rowc);
  if (c->stat_ticket) (void)hipFree(c->stat_ticket);
  if (c->ckeys) (void)hipFree(c->ckeys);
  for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
  delete c;
  return ARKV_OK;
}

int arkv_cache_reset(arkv_cache* c, int32_t layer) {
  if (!c || layer < -1 || layer >= c->L) return ARKV_EINVAL;
  for (int l = 0; l < c->L; ++l) {
    if (layer >= 0 && l != layer) continue;
    LayerState& s = c->layers[(size_t)l];
    s.scored = s.committed = s.cnt_valid = s.cnt_refresh = s.failed = false;
    s.scored_T = s.T = s.live = s.n_pending = s.slot = s.n_tailors = s.last_tailor = 0;
    s.P = -1;
  }
  return ARKV_OK;
}

// Scorer of one layer (eqs. 2-5 + the window sums kept for the commit).  q_win: window query rows, heads
// q_head_stride elements apart.  attn != nullptr: run the causal attention pass first; it leaves the window
// rows' softmax constants in the scratch, so the scorer's own first pass over the keys is skipped.  lse != nullptr:
// the caller's attention produced those constants.
static int run_scorer(arkv_cache* c, int32_t layer, const uint16_t* q_win, size_t q_head_stride, const uint16_t* k,
                      int32_t T, float softmax_scale, float* stats, hipStream_t s, AttnLaunch* attn,
                      const float* lse = nullptr) {
  LayerState& ls = c->layers[(size_t)layer];
  const int U = c->U, G = c->P.G, W = c->cfg.window;
  int rc;
  if ((rc = grow(&ls.pre, &ls.pre_cap, (size_t)U * T)) != ARKV_OK) return rc;
  int MP = 32;
  while (MP < G * W) MP *= 2;
  int chunk = c->prefill_chunk;
  if (!c->prefill_chunk_fixed) {
    if (MP > 256) {
      // more than 256 query rows: the staged queries fill a CU's LDS, one workgroup (of 8 waves) per CU, and every
      // workgroup stages them again, so the grid is one round of the chip where the prompt allows it
      // (16K keys x 64 units at 512 rows: 173 us per pass with 4096 keys per workgroup, 185 us with 1024)
      const size_t per_wg = ((size_t)T * U + 255) / 256;
      chunk = (int)std::min<size_t>(8192, std::max<size_t>(1024, (per_wg + 127) / 128 * 128));
    }
    while (chunk > 128 && (size_t)((T + chunk - 1) / chunk) * U < (MP > 256 ? 256u : 1024u)) chunk >>= 1;
  }
  const int n_chunks = (T + chunk - 1) / chunk;
  if ((rc = grow(&c->rowstat, &c->rowstat_cap, (size_t)U * n_chunks * MP)) != ARKV_OK) return rc;
  // row constants [U][MP] floats (MP even, so what follows is 8-byte aligned) + statistics partials
  const size_t stat_doubles = (size_t)U * n_chunks + 3 * (size_t)c->cfg.batch * ((size_t)(T - W + 511) / 512);
  if ((rc = grow(&c->rowc, &c->rowc_cap, (size_t)U * MP + 2 * stat_doubles)) != ARKV_OK) return rc;
  if (attn) {
    attn->rowc = c->rowc; attn->MP = MP; attn->W = W;
    HIP_TRY(launch_prefill_attn(*attn, s));
  }
  PrefillLaunch a;
  a.q_win = q_win;
  a.q_head_stride = q_head_stride;
  a.have_rowc = (attn || lse) ? 1 : 0;
  a.lse = lse;
  a.k = k;
  a.pre = ls.pre; a.rowstat = c->rowstat; a.stats = stats; a.stat_ticket = c->stat_ticket;
  a.B = c->cfg.batch; a.Hkv = c->cfg.n_kv_heads; a.G = G; a.W = W; a.D = c->P.D; a.T = T;
  a.chunk = chunk; a.n_chunks = n_chunks;
  a.scale2 = softmax_scale * 1.4426950408889634f;
  HIP_TRY(launch_prefill_stats(a, c->rowc, s));
  ls.scored = true; ls.scored_T = T;
  c->last_stream = s;
  return ARKV_OK;
}

int arkv_prefill_stats(arkv_cache* c, int32_t layer, const void* q_win, const void* k, int32_t T,
                       float softmax_scale, float* stats, void* hip_stream) {
  if (!c || !q_win || !k || !stats || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  if (T <= c->cfg.window || !(softmax_scale > 0.0f)) return ARKV_EINVAL;
  if (c->layers[(size_t)layer].committed) return ARKV_ESTATE;
  return run_scorer(c, layer, static_cast<const uint16_t*>(q_win), (size_t)c->cfg.window * c->P.D,
                    static_cast<const uint16_t*>(k), T, softmax_scale, stats, static_cast<hipStream_t>(hip_stream),
                    nullptr);
}

int arkv_prefill_stats_lse(arkv_cache* c, int32_t layer, const void* q_win, const void* k, int32_t T,
                           float softmax_scale, const float* lse, float* stats, void* hip_stream) {
  if (!c || !q_win || !k || !lse || !stats || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  if (T <= c->cfg.window || !(softmax_scale > 0.0f)) return ARKV_EINVAL;
  if (c->layers[(size_t)layer].committed) return ARKV_ESTATE;
  return run_scorer(c, layer, static_cast<const uint16_t*>(q_win), (size_t)c->cfg.window * c->P.D,
                    static_cast<const uint16_t*>(k), T, softmax_scale, stats, static_cast<hipStream_t>(hip_stream),
                    nullptr, lse);
}

int arkv_prefill_attention(arkv_cache* c, int32_t layer, const void* q, const void* k, const void* v, int32_t T_q,
                           int32_t T, float softmax_scale, void* out, float* stats, void* hip_stream) {
  if (!c || !q || !k || !v || !out || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  if (T_q < 1 || T_q > T || !(softmax_scale > 0.0f)) return ARKV_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  AttnLaunch a;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.out = static_cast<uint16_t*>(out);
  a.outf = c->attn_outf;
  a.rowc = nullptr;
  a.B = c->cfg.batch; a.Hq = c->cfg.n_q_heads; a.Hkv = c->cfg.n_kv_heads; a.D = c->P.D;
  a.T = T; a.Tq = T_q; a.W = c->cfg.window; a.MP = 0;
  a.scale2 = softmax_scale * 1.4426950408889634f;
  if (!stats) {
    HIP_TRY(launch_prefill_attn(a, s));
    c->last_stream = s;
    return ARKV_OK;
  }
  if (T_q < c->cfg.window || T <= c->cfg.window) return ARKV_EINVAL;
  if (c->layers[(size_t)layer].committed) return ARKV_ESTATE;
  const size_t D = (size_t)c->P.D;
  return run_scorer(c, layer, a.q + (size_t)(T_q - c->cfg.window) * D, (size_t)T_q * D, a.k, T, softmax_scale, stats, s, &a);
}

int arkv_prefill_commit(arkv_cache* c, int32_t layer, const void* k, const void* v, int32_t T,
                        const float* rho, void* hip_stream) {
  if (!c || !k || !v || !rho || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  LayerState& ls = c->layers[(size_t)layer];
  if (ls.committed || !ls.scored || ls.scored_T != T) return ARKV_ESTATE;
  const arkv_config& cfg = c->cfg;
  const int N = cfg.capacity_tokens, W = cfg.window, U = c->U;
  std::vector<int32_t> no_units((size_t)U), nb_units((size_t)U), no_seq((size_t)cfg.batch), nb_seq((size_t)cfg.batch);
  for (int s = 0; s < cfg.batch; ++s) {
    int32_t no, nq, bb;
    int rc = arkv_budget_counts(&cfg, rho[s], &no, &nq, &bb);
    if (rc != ARKV_OK) return rc;
    no_seq[(size_t)s] = no; nb_seq[(size_t)s] = bb;
    for (int g = 0; g < cfg.n_kv_heads; ++g) {
      no_units[(size_t)s * cfg.n_kv_heads + g] = no;
      nb_units[(size_t)s * cfg.n_kv_heads + g] = bb;
    }
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (T >= N) {      // the key scratch of the first tailor; sized before anything is launched or recorded
    int rc = grow(&c->ckeys, &c->ckeys_cap, (size_t)U * T);
    if (rc != ARKV_OK) return rc;
  }
  for (int s = 0; s < cfg.batch; ++s) ls.n_o[(size_t)s] = no_seq[(size_t)s];
  HIP_TRY(launch_set_budgets(c->P, layer * U, cfg.n_kv_heads, cfg.batch, no_seq.data(), nb_seq.data(), st));
  CommitLaunch a;
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.pre = ls.pre;
  a.unit_begin = layer * U; a.n_units = U;
  a.T = T; a.window = W; a.gamma = cfg.gamma;
  a.select = T >= N ? 1 : 0;
  if (a.select) { c->ckeys_layer = layer; c->ckeys_T = T; }
  HIP_TRY(launch_commit(c->P, a, c->ckeys, st));
  ls.committed = true; ls.T = T; ls.P = T - 1; ls.n_pending = 0; ls.slot = 0;
  if (a.select) {
    ls.live = std::min(c->b, T - W) + W;
    ls.n_tailors = 1; ls.last_tailor = 1;
  } else {
    ls.live = T; ls.n_tailors = 0; ls.last_tailor = 0;
  }
  // every prompt token starts Original, so the first tailor's split is known without looking at the data
  for (int u = 0; u < U; ++u) {
    if (a.select) {
      const int nel = T - W, keep = std::min(nb_units[(size_t)u], nel), no = std::min(no_units[(size_t)u], nel);
      ls.cnt_o[(size_t)u] = W + no;
      ls.cnt_q[(size_t)u] = keep - no;
    } else {
      ls.cnt_o[(size_t)u] = T;
      ls.cnt_q[(size_t)u] = 0;
    }
  }
  ls.cnt_valid = true;
  c->last_stream = st;
  return ARKV_OK;
}

// One decode step of n layers in the same state.  static_scratch: the split-K partials and tickets of this launch
// live in the library's static device array instead of the cache's own buffers.
static int decode_impl(arkv_cache* c, int32_t layer_begin, int32_t n, const void* q, const void* k_new,
                       const void* v_new, const float* softmax_scale, void* out, void* hip_stream,
                       bool static_scratch) {
  if (!c || !q || !k_new || !v_new || !softmax_scale || !out) return ARKV_EINVAL;
  if (n < 1 || n > kMaxLayersPerLaunch || layer_begin < 0 || layer_begin + n > c->L) return ARKV_EINVAL;
  LayerState& l0 = c->layers[(size_t)layer_begin];
  for (int i = 0; i < n; ++i) {
    const LayerState& li = c->layers[(size_t)(layer_begin + i)];
    if (!li.committed || li.failed) return ARKV_ESTATE;
    if (li.T != l0.T || li.P != l0.P || li.live != l0.live || li.n_pending != l0.n_pending || li.slot != l0.slot)
      return ARKV_ESTATE;
    if (!(softmax_scale[i] > 0.0f)) return ARKV_EINVAL;
  }
  const arkv_config& cfg = c->cfg;
  const int N = cfg.capacity_tokens, W = cfg.window, U = c->U;
  if (l0.live >= N) return ARKV_ESTATE;   // cannot happen: a tailor always frees a slot
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  DecodeLaunch a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.out = static_cast<uint16_t*>(out);
  a.unit_begin = layer_begin * U; a.n_units = n * U; a.units_per_layer = U;
  // split-K factor: enough workgroups to fill the chip, at least 128 rows (two tiles per wave) each: below
  // that the merge of more partials costs more than the shorter loops save (measured on the 8K-context shape)
  int splits = (c->wg_target + a.n_units / 2) / a.n_units;
  // few units: beyond 32 splits the merge (one workgroup pulls every partial of its unit) costs more than the
  // second workgroup per CU gains, so such launches use one workgroup per CU
  if (splits > 32) splits = (splits + 1) / 2;
  splits = std::min(splits, std::max(1, l0.live / 128));
  a.splits = std::max(1, std::min(splits, c->P.max_splits));
  a.part_unit0 = 0;
  Pools pools = c->P;                 // by value: the launch may point the split-K scratch elsewhere
  if (static_scratch) {
    float* sp = nullptr; int* stk = nullptr; size_t cap = 0;
    HIP_TRY(static_scratch_get(&sp, &stk, &cap));
    const size_t row = (size_t)pools.G * ((size_t)pools.D + 2);
    if (a.n_units > kStaticUnits || (size_t)a.n_units * row > cap) return ARKV_ESCRATCH;
    // as many splits as fit (never more than the cache's own buffers would get)
    a.splits = (int)std::min<size_t>((size_t)a.splits, cap / ((size_t)a.n_units * row));
    pools.part = sp; pools.ticket = stk; pools.max_splits = a.splits;
    a.part_unit0 = a.unit_begin;
  }
  // Measured cost of a packed row in sixteenths of a bf16 row.  With two workgroups per CU the bf16 rows stream
  // at the HBM limit and a packed row costs about 10/16 of one (8 to 14 measure within 1 %); with one workgroup
  // per CU (few units) the bf16 rows are not bandwidth-bound and a packed row costs as much as a bf16 row
  // (128K-context shape, 8 units: 18.1 us per launch at 16 against 19.4 at 10).
  a.wq = c->wq > 0 ? c->wq : (a.splits * a.n_units <= 256 ? 16 : 10);
  { const SplitRecip rc = split_recip(a.splits, a.wq); a.inv_splits = rc.inv_s; a.inv_wq = rc.inv_wq; }
  for (int i = 0; i < n; ++i) {
    LayerState& li = c->layers[(size_t)(layer_begin + i)];
    if (li.cnt_valid || !li.cnt_refresh) continue;
    if (hipEventQuery(li.cnt_ev) != hipSuccess) { (void)hipGetLastError(); continue; }   // not landed yet
    const int steps = li.P - li.cnt_refresh_P;
    for (int u = 0; u < U; ++u) { li.cnt_o[(size_t)u] = li.cnt_host[u].x + steps; li.cnt_q[(size_t)u] = li.cnt_host[u].y; }
    li.cnt_valid = true; li.cnt_refresh = false;
  }
  a.cnt_known = 0;
  if (n == 1 && a.n_units <= kMaxUnitsKnown) {   // one layer: the kernel indexes the counts by its block index
    bool known = true;
    for (int i = 0; i < n; ++i) known = known && c->layers[(size_t)(layer_begin + i)].cnt_valid;
    if (known) {
      a.cnt_known = 1;
      for (int i = 0; i < n; ++i) {
        const LayerState& li = c->layers[(size_t)(layer_begin + i)];
        for (int u = 0; u < U; ++u) { a.cnt_o[i * U + u] = li.cnt_o[(size_t)u]; a.cnt_q[i * U + u] = li.cnt_q[(size_t)u]; }
      }
    }
  }
  a.position = l0.P + 1;
  a.n_pending = l0.n_pending;
  a.slot = l0.slot;
  a.fold = l0.n_pending == kRing - 1 ? 1 : 0;   // the ring is full: add the waiting steps now
  for (int i = 0; i < n; ++i) a.scale2[i] = softmax_scale[i] * 1.4426950408889634f;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (c->timing && !static_scratch) {        // the event pool grows by allocation
    if (c->ev_used + 2 > c->ev_pool.size()) {
      for (int i = 0; i < 2; ++i) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        c->ev_pool.push_back(e);
      }
    }
    e0 = c->ev_pool[c->ev_used]; e1 = c->ev_pool[c->ev_used + 1];
    c->ev_used += 2;
  }
  HIP_TRY(launch_decode(pools, a, st, e0, e1));
  const int P = l0.P + 1, live = l0.live + 1;
  const int n_pending = (a.fold ? 0 : l0.n_pending) + 1, slot = (l0.slot + 1) % kRing;
  bool tailor = live >= N;
  int live_after = live;
  if (tailor) {
    TailorLaunch t;
    t.unit_begin = a.unit_begin; t.n_units = a.n_units;
    t.position = P; t.t_prefill = l0.T; t.window = W; t.gamma = cfg.gamma;
    t.n_pending = n_pending; t.slot = slot;
    const hipError_t te = launch_tailor(c->P, t, st);
    if (te != hipSuccess) {
      // the attention of this step is on the stream, the tailor is not (or only partly): the device-side state of
      // these layers is no longer what the host would book, so they refuse further steps until they are reset
      for (int i = 0; i < n; ++i) c->layers[(size_t)(layer_begin + i)].failed = true;
      return hip_fail(te, "launch_tailor");
    }
    const int wcount = std::min(W, P + 1);
    live_after = std::min(c->b, live - wcount) + wcount;
  }
  for (int i = 0; i < n; ++i) {
    LayerState& li = c->layers[(size_t)(layer_begin + i)];
    li.P = P; li.live = live_after; li.slot = slot; li.n_pending = tailor ? 0 : n_pending;
    for (auto& v : li.cnt_o) v += 1;
    if (tailor) {
      li.n_tailors += 1; li.last_tailor = 2; li.cnt_valid = false; li.cnt_refresh = false;
      if (cfg.tailor_policy == 0) {       // with a tailor at every step the snapshot would never be used
        HIP_TRY(hipMemcpyAsync(li.cnt_host, c->P.cnt + (size_t)(layer_begin + i) * U, (size_t)U * sizeof(int2),
                               hipMemcpyDeviceToHost, st));
        HIP_TRY(hipEventRecord(li.cnt_ev, st));
        li.cnt_refresh = true; li.cnt_refresh_P = P;
      }
    }
  }
  c->last_stream = st;
  return ARKV_OK;
}

int arkv_decode_step_layers(arkv_cache* c, int32_t layer_begin, int32_t n, const void* q, const void* k_new,
                            const void* v_new, const float* softmax_scale, void* out, void* hip_stream) {
  return decode_impl(c, layer_begin, n, q, k_new, v_new, softmax_scale, out, hip_stream, false);
}

int arkv_decode_step(arkv_cache* c, int32_t layer, const void* q, const void* k_new, const void* v_new,
                     float softmax_scale, void* out, void* hip_stream) {
  return decode_impl(c, layer, 1, q, k_new, v_new, &softmax_scale, out, hip_stream, false);
}

int arkv_decode_step_static(arkv_cache* c, int32_t layer, const void* q, const void* k_new, const void* v_new,
                            float softmax_scale, void* out, void* hip_stream) {
  return decode_impl(c, layer, 1, q, k_new, v_new, &softmax_scale, out, hip_stream, true);
}

// ---- observability ---------------------------------------------------------------------------

int arkv_cache_counters(arkv_cache* c, int32_t layer, int32_t* n_original, int32_t* n_quantized,
                        int32_t* n_evicted, int64_t* live_bytes) {
  if (!c || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  if (!c->layers[(size_t)layer].committed) return ARKV_ESTATE;
  HIP_TRY(hipStreamSynchronize(c->last_stream));
  std::vector<int2> cnt;
  int rc = fetch(cnt, c->P.cnt + (size_t)layer * c->U, (size_t)c->U);
  if (rc != ARKV_OK) return rc;
  int64_t co, cq;
  row_bytes(c->P.D, c->P.bits, &co, &cq);
  for (int u = 0; u < c->U; ++u) {
    if (n_original) n_original[u] = cnt[(size_t)u].x;
    if (n_quantized) n_quantized[u] = cnt[(size_t)u].y;
    if (n_evicted) n_evicted[u] = c->layers[(size_t)layer].P + 1 - cnt[(size_t)u].x - cnt[(size_t)u].y;
    if (live_bytes) live_bytes[u] = cnt[(size_t)u].x * co + cnt[(size_t)u].y * cq;
  }
  return ARKV_OK;
}

int arkv_cache_progress(arkv_cache* c, int32_t layer, int32_t* n_tailors, int32_t* n_live, int32_t* position) {
  if (!c || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  const LayerState& ls = c->layers[(size_t)layer];
  if (n_tailors) *n_tailors = ls.n_tailors;
  if (n_live) *n_live = ls.live;
  if (position) *position = ls.P;
  return ARKV_OK;
}

int arkv_cache_export(arkv_cache* c, int32_t layer, int32_t max_tokens, int32_t* n_live, int32_t* pos,
                      uint8_t* state, float* s1, float* s2, uint16_t* rows_k, uint16_t* rows_v,
                      uint8_t* codes_k, uint8_t* codes_v, uint16_t* scale_k, uint16_t* zero_k,
                      uint16_t* scale_v, uint16_t* zero_v) {
  if (!c || layer < 0 || layer >= c->L || max_tokens < c->cfg.capacity_tokens) return ARKV_EINVAL;
  if (!c->layers[(size_t)layer].committed) return ARKV_ESTATE;
  int rc = flush_and_sync(c, layer);
  if (rc != ARKV_OK) return rc;
  const Pools& P = c->P;
  const size_t U = (size_t)c->U, off = (size_t)layer * U, D = (size_t)P.D;
  const size_t CB = D * P.bits / 8, NG = (size_t)metas_per_row(P.D, P.bits), cO = (size_t)P.capO, cQ = (size_t)P.capQ;
  std::vector<int2> cnt;
  std::vector<int32_t> opos, qpos;
  std::vector<float2> oacc, qacc;
  std::vector<uint16_t> ok, ov;
  std::vector<uint8_t> qkc, qvc;
  std::vector<uint32_t> qkm;
  std::vector<uint16_t> qvm;
  const size_t cQv = (size_t)P.capQv, MH = (size_t)vmeta_per_row(P.D, P.bits);
  if ((rc = fetch(cnt, P.cnt + off, U)) || (rc = fetch(opos, P.opos + off * cO, U * cO)) ||
      (rc = fetch(qpos, P.qpos + off * cQ, U * cQ)) || (rc = fetch(oacc, P.oacc + off * cO, U * cO)) ||
      (rc = fetch(qacc, P.qacc + off * cQ, U * cQ)))
    return rc;
  if (rows_k && (rc = fetch(ok, P.ok + off * cO * D, U * cO * D))) return rc;
  if (rows_v && (rc = fetch(ov, P.ov + off * cO * D, U * cO * D))) return rc;
  if (codes_k && (rc = fetch(qkc, P.qkc + off * cQ * CB, U * cQ * CB))) return rc;
  if (codes_v && (rc = fetch(qvc, P.qvc + off * cQv * CB, U * cQv * CB))) return rc;
  if ((scale_k || zero_k) && (rc = fetch(qkm, P.qkm + off * cQ * NG, U * cQ * NG))) return rc;
  if ((scale_v || zero_v) && (rc = fetch(qvm, P.qvm + off * cQv * MH, U * cQv * MH))) return rc;
  const size_t MT = (size_t)max_tokens;
  struct Ent { int32_t pos; int32_t slot; uint8_t st; };
  std::vector<Ent> ents;
  for (size_t u = 0; u < U; ++u) {
    ents.clear();
    for (int i = 0; i < cnt[u].x; ++i) ents.push_back({opos[u * cO + i], i, ARKV_STATE_ORIGINAL});
    for (int i = 0; i < cnt[u].y; ++i) ents.push_back({qpos[u * cQ + i], i, ARKV_STATE_QUANTIZED});
    std::sort(ents.begin(), ents.end(), [](const Ent& a, const Ent& b) { return a.pos < b.pos; });
    if (ents.size() > MT) return ARKV_EINVAL;
    if (n_live) n_live[u] = (int32_t)ents.size();
    for (size_t t = 0; t < ents.size(); ++t) {
      const Ent& e = ents[t];
      const size_t o = u * MT + t;
      const bool isq = e.st == ARKV_STATE_QUANTIZED;
      const size_t so = u * cO + (size_t)e.slot, sq = u * cQ + (size_t)e.slot;
      if (pos) pos[o] = e.pos;
      if (state) state[o] = e.st;
      if (s1) s1[o] = isq ? qacc[sq].x : oacc[so].x;
      if (s2) s2[o] = isq ? qacc[sq].y : oacc[so].y;
      if (rows_k) { if (isq) memset(rows_k + o * D, 0, D * 2); else memcpy(rows_k + o * D, &ok[so * D], D * 2); }
      if (rows_v) { if (isq) memset(rows_v + o * D, 0, D * 2); else memcpy(rows_v + o * D, &ov[so * D], D * 2); }
      if (codes_k) {      // the row's bytes back into canonical order
        for (size_t bcol = 0; bcol < CB; ++bcol)
          codes_k[o * CB + bcol] = isq ? qkc[sq * CB + (size_t)kcode_index((int)bcol, P.D, P.bits)] : (uint8_t)0;
      }
      if (codes_v) {      // gather the row's bytes out of the token-minor value blocks
        for (size_t bcol = 0; bcol < CB; ++bcol)
          codes_v[o * CB + bcol] = isq ? qvc[u * cQv * CB + vcode_index(e.slot, (int)bcol, (int)CB, P.bits)] : (uint8_t)0;
      }
      for (size_t g = 0; g < NG; ++g) {
        if (scale_k) scale_k[o * NG + g] = isq ? (uint16_t)(qkm[sq * NG + g] & 0xffffu) : 0;
        if (zero_k) zero_k[o * NG + g] = isq ? (uint16_t)(qkm[sq * NG + g] >> 16) : 0;
        if (scale_v) scale_v[o * NG + g] = isq ? qvm[u * cQv * MH + vmeta_index(e.slot, (int)g, (int)MH)] : (uint16_t)0;
        if (zero_v) zero_v[o * NG + g] = (isq && MH > 1) ? qvm[u * cQv * MH + vmeta_index(e.slot, (int)(NG + g), (int)MH)] : (uint16_t)0;
      }
    }
  }
  return ARKV_OK;
}

int arkv_debug_last_tailor_scores(arkv_cache* c, int32_t layer, int32_t max_tokens, int32_t* count,
                                  int32_t* pos, float* score) {
  if (!c || layer < 0 || layer >= c->L || !count || max_tokens < 1) return ARKV_EINVAL;
  const LayerState& ls = c->layers[(size_t)layer];
  const size_t U = (size_t)c->U;
  if (ls.last_tailor == 0) {
    for (size_t u = 0; u < U; ++u) count[u] = -1;
    return ARKV_OK;
  }
  HIP_TRY(hipStreamSynchronize(c->last_stream));
  std::vector<uint64_t> keys;
  size_t per;
  int rc;
  if (ls.last_tailor == 1) {
    if (c->ckeys_layer != layer) return ARKV_ESTATE;   // scratch reused by another layer's commit
    per = (size_t)c->ckeys_T;
    rc = fetch(keys, (const uint64_t*)c->ckeys, U * per);
  } else {
    per = (size_t)(c->P.capO + c->P.capQ);
    rc = fetch(keys, (const uint64_t*)c->P.keys + (size_t)layer * U * per, U * per);
  }
  if (rc != ARKV_OK) return rc;
  for (size_t u = 0; u < U; ++u) {
    int n = 0;
    for (size_t i = 0; i < per; ++i) {
      const uint64_t k = keys[u * per + i];
      if (!k) continue;
      if (n >= max_tokens) return ARKV_EINVAL;
      const uint32_t sb = (uint32_t)(k >> 32);
      float S;
      memcpy(&S, &sb, 4);
      if (pos) pos[u * (size_t)max_tokens + n] = (int32_t)(0xFFFFFFFFu - (uint32_t)(k & 0xFFFFFFFFu));
      if (score) score[u * (size_t)max_tokens + n] = S;
      ++n;
    }
    count[u] = n;
  }
  return ARKV_OK;
}

int arkv_debug_last_out_f32(arkv_cache* c, int32_t layer, float* out) {
  if (!c || !out || layer < 0 || layer >= c->L) return ARKV_EINVAL;
  HIP_TRY(hipStreamSynchronize(c->last_stream));
  const size_t n = (size_t)c->U * c->P.G * c->P.D;
  HIP_TRY(hipMemcpy(out, c->P.outf + (size_t)layer * n, n * sizeof(float), hipMemcpyDeviceToHost));
  return ARKV_OK;
}

int arkv_debug_prefill_attention_f32(arkv_cache* c, float* out_f32) {
  if (!c) return ARKV_EINVAL;
  c->attn_outf = out_f32;
  return ARKV_OK;
}

int arkv_debug_set_launch_shape(arkv_cache* c, int32_t wg_target, int32_t packed_weight, int32_t prefill_chunk) {
  if (!c || packed_weight > 16 || (prefill_chunk > 0 && (prefill_chunk % 128 != 0 || prefill_chunk > 8192))) return ARKV_EINVAL;
  if (wg_target > 0) c->wg_target = wg_target;
  if (packed_weight > 0) c->wq = packed_weight;
  if (prefill_chunk > 0) { c->prefill_chunk = prefill_chunk; c->prefill_chunk_fixed = true; }
  return ARKV_OK;
}

int arkv_debug_time_attend(arkv_cache* c, int32_t enable) {
  if (!c) return ARKV_EINVAL;
  c->timing = enable != 0;
  c->ev_used = 0;
  return ARKV_OK;
}

int arkv_debug_attend_time(arkv_cache* c, double* total_ms, int64_t* launches) {
  if (!c || !total_ms || !launches) return ARKV_EINVAL;
  HIP_TRY(hipStreamSynchronize(c->last_stream));
  double tot = 0.0;
  for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->ev_pool[i], c->ev_pool[i + 1]));
    tot += (double)ms;
  }
  *total_ms = tot;
  *launches = (int64_t)(c->ev_used / 2);
  c->ev_used = 0;
  return ARKV_OK;
}

int arkv_debug_phase_trace(int32_t which, unsigned long long* host_words, int32_t n_rows) {
  if (!host_words || which < 0 || which > 2 || n_rows < 1 || n_rows > 8192) return ARKV_EINVAL;
  bool built = false;
  const hipError_t e = which == 2 ? phase_trace_attn(host_words, &built)
                                  : phase_trace_decode(which, host_words, n_rows, &built);
  if (!built) return ARKV_EUNSUPPORTED;
  return e == hipSuccess ? ARKV_OK : hip_fail(e, "arkv_debug_phase_trace");
}

const char* arkv_strerror(int code) {
  switch (code) {
    case ARKV_OK: return "ok";
    case ARKV_EINVAL: return "invalid argument";
    case ARKV_ESTATE: return "call out of order for this layer";
    case ARKV_ENOMEM: return "out of memory";
    case ARKV_EHIP: return "HIP runtime error (see arkv_last_hip_error)";
    case ARKV_EUNSUPPORTED: return "configuration not supported by this build";
    case ARKV_ESCRATCH: return "the launch needs more static scratch memory than the library holds";
  }
  return "unknown error code";
}

const char* arkv_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
