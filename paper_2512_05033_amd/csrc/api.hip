// The C ABI of libarb (include/arb.h): argument validation, workspace carving
// and the launch sequence of the step-scoring forward.  No allocation, no
// synchronisation and no read-back happen in the hot calls.
#include "common.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include <new>
#include <vector>

// ------------------------------------------------------------------------- errors

static thread_local char g_err[512] = "";

arb_status arb_fail(arb_status st, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return st;
}

extern "C" const char *arb_last_error(void) { return g_err; }

// -------------------------------------------------------------------------- model

struct arb_model {
  arb_model_cfg cfg;
  const bf16 *embed;
  std::vector<const bf16 *> wqkv, wo, wgu, wd;              // packed uint32 when w4
  std::vector<const bf16 *> sqkv, so, sgu, sd;              // group scales of 4-bit weights
  std::vector<const bf16 *> wgu_blocked;                    // K-blocked copies of wgu (empty: none)
  bool w4 = false;
  bool debug_ids = false;                                 // ARB_DEBUG_IDS: range-check ids before every forward
  std::vector<const float *> g_attn, g_mlp;
  const float *g_final, *w_head;
  float b_head;
  int trace_stage = -1, trace_cap = 0, trace_n = 0;      // timing hook (arb_model_trace)
  std::vector<hipEvent_t> trace_start, trace_stop;
  int qkv_rows() const { return (cfg.n_q_heads + 2 * cfg.n_kv_heads) * cfg.head_dim; }
};

extern "C" arb_status arb_model_create(const arb_model_cfg *cfg, const arb_weights *w, arb_model **out) {
  if (!cfg || !w || !out) return arb_fail(ARB_EINVAL, "arb_model_create: null argument");
  *out = nullptr;
  const arb_model_cfg &c = *cfg;
  if (c.n_layers <= 0 || c.d_model <= 0 || c.n_q_heads <= 0 || c.n_kv_heads <= 0 || c.head_dim <= 0 ||
      c.d_ffn <= 0 || c.vocab <= 0)
    return arb_fail(ARB_ESHAPE, "arb_model_create: non-positive dimension");
  if (c.n_q_heads % c.n_kv_heads != 0)
    return arb_fail(ARB_ESHAPE, "arb_model_create: n_q_heads %d is not a multiple of n_kv_heads %d", c.n_q_heads,
                    c.n_kv_heads);
  if (c.head_dim % 2 != 0) return arb_fail(ARB_ESHAPE, "arb_model_create: odd head_dim %d", c.head_dim);
  if (!(c.rms_eps >= 0.f) || !(c.rope_base > 0.f))
    return arb_fail(ARB_EINVAL, "arb_model_create: rms_eps %g / rope_base %g", c.rms_eps, c.rope_base);
  if (c.pool != ARB_POOL_MEAN && c.pool != ARB_POOL_LAST)
    return arb_fail(ARB_EINVAL, "arb_model_create: pool mode %d", c.pool);
  if (c.kv_block != ARB_KV_BLOCK) return arb_fail(ARB_EUNSUPPORTED, "arb_model_create: kv_block %d (16 only)", c.kv_block);
  if (c.head_dim != 64 && c.head_dim != 128)
    return arb_fail(ARB_EUNSUPPORTED, "arb_model_create: head_dim %d (64 or 128 only)", c.head_dim);
  if (c.d_model % 128 != 0 || c.d_ffn % 128 != 0 || (c.n_q_heads * c.head_dim) % 128 != 0 || c.d_model > 8192)
    return arb_fail(ARB_EUNSUPPORTED, "arb_model_create: d_model %d, d_ffn %d, n_q_heads*head_dim %d must be multiples of 128 (d_model <= 8192)",
                    c.d_model, c.d_ffn, c.n_q_heads * c.head_dim);
  if (((c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim) % 128 != 0)
    return arb_fail(ARB_EUNSUPPORTED, "arb_model_create: (Hq + 2 Hkv) * head_dim must be a multiple of 128");
  if (!w->embed || !w->wqkv || !w->wo || !w->wgu || !w->wd || !w->g_attn || !w->g_mlp || !w->g_final)
    return arb_fail(ARB_EINVAL, "arb_model_create: null weight pointer");
  if (c.has_router_head < 0 || c.has_router_head > ARB_HEAD_TWO_CLASS)
    return arb_fail(ARB_EINVAL, "arb_model_create: has_router_head = %d", c.has_router_head);
  if (c.has_router_head && !w->w_head) return arb_fail(ARB_EINVAL, "arb_model_create: has_router_head but w_head is null");
  for (int l = 0; l < c.n_layers; ++l)
    if (!w->wqkv[l] || !w->wo[l] || !w->wgu[l] || !w->wd[l] || !w->g_attn[l] || !w->g_mlp[l])
      return arb_fail(ARB_EINVAL, "arb_model_create: null weight pointer in layer %d", l);
  const int n_scale = (w->wqkv_scale != nullptr) + (w->wo_scale != nullptr) + (w->wgu_scale != nullptr) + (w->wd_scale != nullptr);
  if (n_scale != 0 && n_scale != 4) return arb_fail(ARB_EINVAL, "arb_model_create: either all four scale tables or none");
  if (n_scale == 4) {
    for (int l = 0; l < c.n_layers; ++l)
      if (!w->wqkv_scale[l] || !w->wo_scale[l] || !w->wgu_scale[l] || !w->wd_scale[l])
        return arb_fail(ARB_EINVAL, "arb_model_create: null scale pointer in layer %d", l);
  }
  arb_model *m = new (std::nothrow) arb_model;
  if (!m) return arb_fail(ARB_EINVAL, "arb_model_create: out of host memory");
  m->cfg = c;
  m->w4 = n_scale == 4;
  const char *dbg = getenv("ARB_DEBUG_IDS");
  m->debug_ids = dbg && dbg[0] && dbg[0] != '0';
  m->embed = (const bf16 *)w->embed;
  for (int l = 0; l < c.n_layers; ++l) {
    m->wqkv.push_back((const bf16 *)w->wqkv[l]);
    m->wo.push_back((const bf16 *)w->wo[l]);
    m->wgu.push_back((const bf16 *)w->wgu[l]);
    m->wd.push_back((const bf16 *)w->wd[l]);
    if (m->w4) {
      m->sqkv.push_back((const bf16 *)w->wqkv_scale[l]);
      m->so.push_back((const bf16 *)w->wo_scale[l]);
      m->sgu.push_back((const bf16 *)w->wgu_scale[l]);
      m->sd.push_back((const bf16 *)w->wd_scale[l]);
    }
    m->g_attn.push_back(w->g_attn[l]);
    m->g_mlp.push_back(w->g_mlp[l]);
    if (w->wgu_blocked) {
      if (!w->wgu_blocked[l] || m->w4 || c.d_model % 32 != 0) {
        delete m;
        return arb_fail(ARB_EINVAL, "arb_model_create: wgu_blocked needs bf16 weights and a pointer for every layer (layer %d)", l);
      }
      m->wgu_blocked.push_back((const bf16 *)w->wgu_blocked[l]);
    }
  }
  m->g_final = w->g_final;
  m->w_head = c.has_router_head ? w->w_head : nullptr;
  m->b_head = w->b_head;
  *out = m;
  return ARB_OK;
}

extern "C" arb_status arb_model_destroy(arb_model *m) {
  delete m;
  return ARB_OK;
}

extern "C" arb_status arb_model_trace(arb_model *m, int32_t stage, void *const *start, void *const *stop, int32_t n) {
  if (!m || n < 0 || (n > 0 && (!start || !stop))) return arb_fail(ARB_EINVAL, "arb_model_trace: bad argument");
  m->trace_stage = n > 0 ? stage : -1;
  m->trace_cap = n;
  m->trace_n = 0;
  m->trace_start.assign((hipEvent_t const *)start, (hipEvent_t const *)start + n);
  m->trace_stop.assign((hipEvent_t const *)stop, (hipEvent_t const *)stop + n);
  return ARB_OK;
}

extern "C" int32_t arb_model_trace_count(const arb_model *m) { return m ? m->trace_n : 0; }

// Brackets one launch with the caller's events when its stage is being traced.
struct TraceScope {
  arb_model *m;
  hipStream_t st;
  bool on;
  TraceScope(arb_model *m_, int stage, hipStream_t st_) : m(m_), st(st_) {
    on = m->trace_stage == stage && m->trace_n < m->trace_cap;
    if (on) (void)hipEventRecord(m->trace_start[m->trace_n], st);
  }
  ~TraceScope() {
    if (on) (void)hipEventRecord(m->trace_stop[m->trace_n++], st);
  }
};

// ---------------------------------------------------------------------- workspace

struct Workspace {
  float *h;          // fp32 [T, d] residual stream
  bf16 *x;           // bf16 [T, d] normed activations
  bf16 *qkv;         // bf16 [T, (Hq+2Hkv)*hd]
  bf16 *attn;        // bf16 [T, Hq*hd]
  bf16 *act;         // bf16 [T, F]
  int32_t *tok_pos, *tok_slot;
  f32x2 *cs;         // [T, hd/2] rotary table
  float *tok_dot;    // [T]
  float *parts;      // fp32 [8, T, d] split-K partial products of the residual projections
  void *attn_ws;
  size_t attn_ws_bytes, total;
};

// attn_splits: the number of key splits whose partial results the attention part must hold.
static Workspace carve(const arb_model_cfg &c, int T, int attn_splits, void *base) {
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void *p = base ? (char *)base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  const size_t t = (size_t)T;
  w.h = (float *)take(t * c.d_model * sizeof(float));
  w.x = (bf16 *)take(t * c.d_model * sizeof(bf16));
  w.qkv = (bf16 *)take(t * (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * sizeof(bf16));
  w.attn = (bf16 *)take(t * c.n_q_heads * c.head_dim * sizeof(bf16));
  w.act = (bf16 *)take(t * c.d_ffn * sizeof(bf16));
  w.tok_pos = (int32_t *)take(t * sizeof(int32_t));
  w.tok_slot = (int32_t *)take(t * sizeof(int32_t));
  w.cs = (f32x2 *)take(t * (c.head_dim / 2) * sizeof(f32x2));
  w.tok_dot = (float *)take(t * sizeof(float));
  w.parts = (float *)take(8 * t * c.d_model * sizeof(float));
  w.attn_ws_bytes = attention_ws_bytes(attn_splits, T, c.n_q_heads, c.head_dim);
  w.attn_ws = take(w.attn_ws_bytes);
  w.total = off;
  return w;
}

extern "C" size_t arb_workspace_bytes(const arb_model *m, int32_t max_batch, int32_t max_total_tokens,
                                      int32_t max_ctx) {
  if (!m || max_batch < 0 || max_total_tokens < 0 || max_ctx < 0) return 0;
  return carve(m->cfg, max_total_tokens, attention_splits_cap(max_ctx), nullptr).total;
}

// --------------------------------------------------------------- batch validation

struct BatchInfo {
  int max_ctx, max_step;
};

static arb_status check_batch(const arb_batch *bt, int kv_block, BatchInfo *info, bool need_tokens) {
  if (!bt) return arb_fail(ARB_EINVAL, "null batch");
  if (bt->batch < 0 || bt->total_tokens < 0 || bt->max_blocks_per_seq < 0)
    return arb_fail(ARB_EINVAL, "negative batch size / token count / table width");
  info->max_ctx = info->max_step = 0;
  if (bt->batch == 0) {
    if (bt->total_tokens != 0) return arb_fail(ARB_EINVAL, "empty batch with %d tokens", bt->total_tokens);
    return ARB_OK;
  }
  if (!bt->block_tables || !bt->prefix_lens || !bt->cu_step_lens || !bt->prefix_lens_host || !bt->cu_step_lens_host ||
      (need_tokens && !bt->token_ids))
    return arb_fail(ARB_EINVAL, "null pointer in batch");
  const int32_t *cu = bt->cu_step_lens_host, *p = bt->prefix_lens_host;
  if (cu[0] != 0) return arb_fail(ARB_EINVAL, "cu_step_lens[0] = %d, expected 0", cu[0]);
  for (int b = 0; b < bt->batch; ++b) {
    const long long s = (long long)cu[b + 1] - cu[b];
    if (s < 1) return arb_fail(ARB_EINVAL, "sequence %d has a step of %lld tokens (need >= 1)", b, s);
    if (p[b] < 0) return arb_fail(ARB_EINVAL, "sequence %d has prefix length %d", b, p[b]);
    const long long ctx = (long long)p[b] + s;
    if (ctx > (1 << 30)) return arb_fail(ARB_ECAPACITY, "sequence %d: context of %lld tokens", b, ctx);
    if ((ctx + kv_block - 1) / kv_block > bt->max_blocks_per_seq)
      return arb_fail(ARB_ECAPACITY, "sequence %d needs %lld blocks, table rows hold %d", b,
                      (ctx + kv_block - 1) / kv_block, bt->max_blocks_per_seq);
    if (ctx > info->max_ctx) info->max_ctx = (int)ctx;
    if (s > info->max_step) info->max_step = (int)s;
  }
  if (cu[bt->batch] != bt->total_tokens)
    return arb_fail(ARB_EINVAL, "cu_step_lens[batch] = %d but total_tokens = %d", cu[bt->batch], bt->total_tokens);
  return ARB_OK;
}

// ------------------------------------------------------------------------ forward

// Runs decoder layers [l0, l1).  With h_in == nullptr the pass starts from the token embeddings (l0 must be 0)
// and ends with the final norm (+ head); otherwise it starts from the given fp32 residual stream and hands the
// residual stream after layer l1 - 1 back through h_out, with no final norm.
static arb_status forward(arb_model *m, const arb_kv *kv, const arb_batch *bt, bool with_head, float tau,
                          float *scores, uint8_t *escalate, void *hidden_out, void *ws, size_t ws_bytes,
                          hipStream_t st, int l0, int l1, const float *h_in = nullptr, float *h_out = nullptr,
                          bool ws_is_static = false) {
  if (!m || !kv) return arb_fail(ARB_EINVAL, "null model or kv");
  const arb_model_cfg &c = m->cfg;
  BatchInfo info;
  if (arb_status s = check_batch(bt, c.kv_block, &info, h_in == nullptr)) return s;
  if (bt->batch == 0) return ARB_OK;
  if (with_head && !scores) return arb_fail(ARB_EINVAL, "model has a router head but scores is null");
  if (!with_head && (scores || escalate)) return arb_fail(ARB_EINVAL, "scores/escalate given but no router head is applied");
  if (!kv->k_pool || !kv->v_pool) return arb_fail(ARB_EINVAL, "null kv pool table");
  for (int l = l0; l < l1; ++l)
    if (!kv->k_pool[l] || !kv->v_pool[l]) return arb_fail(ARB_EINVAL, "null kv pool in layer %d", l);
  const int T = bt->total_tokens, B = bt->batch, d = c.d_model;
  const int G = c.n_q_heads / c.n_kv_heads;
  const AttnPlan plan = plan_attention(B, bt->prefix_lens_host, bt->cu_step_lens_host, G, c.n_kv_heads);
  // the attention part is sized by this call's own split count (never above what arb_workspace_bytes assumed)
  const Workspace w = carve(c, T, plan.max_splits, ws);
  if (ws_is_static && ws_bytes < w.total)
    return arb_fail(ARB_ECAPACITY, "arb_score_steps_noalloc: this batch needs %zu bytes of scratch but the static buffer "
                    "holds %zu (ARB_NOALLOC_SCRATCH_BYTES); use arb_score_steps with a workspace", w.total, ws_bytes);
  if (!ws || ws_bytes < w.total) return arb_fail(ARB_ECAPACITY, "workspace %zu < %zu bytes", ws_bytes, w.total);
  if (m->debug_ids) {
    // Debug mode (environment variable ARB_DEBUG_IDS at arb_model_create): the ids the kernels would
    // index with are range-checked on the device first, and this call waits for the verdict, so that a
    // bad id becomes an error instead of an out-of-bounds access.  The error word borrows the
    // workspace's partial-product area, which nothing has written yet.
    if (kv->n_blocks <= 0) return arb_fail(ARB_EINVAL, "debug id check: arb_kv.n_blocks = %d", kv->n_blocks);
    int32_t *err = (int32_t *)w.parts, host[4] = {0, 0, 0, 0};
    if (arb_status s0 = launch_check_ids(h_in ? nullptr : bt->token_ids, T, c.vocab, bt->block_tables, B,
                                         bt->max_blocks_per_seq, bt->prefix_lens, bt->cu_step_lens, c.kv_block,
                                         kv->n_blocks, err, st))
      return s0;
    ARB_CHECK_HIP(hipMemcpyAsync(host, err, sizeof host, hipMemcpyDeviceToHost, st));
    ARB_CHECK_HIP(hipStreamSynchronize(st));
    if (host[0] & 1)
      return arb_fail(ARB_EINVAL, "debug id check: token_ids[%d] is outside [0, %d)", host[1], c.vocab);
    if (host[0] & 2)
      return arb_fail(ARB_EINVAL, "debug id check: block_tables[%d][%d] is outside [0, %d)",
                      host[2] / bt->max_blocks_per_seq, host[2] % bt->max_blocks_per_seq, kv->n_blocks);
  }
  if (h_in) ARB_CHECK_HIP(hipMemcpyAsync(w.h, h_in, (size_t)T * d * sizeof(float), hipMemcpyDeviceToDevice, st));

  // The residual projections (O, down) are split along K when their N is too narrow to fill the
  // chip; their fp32 products (one per split; a single one when not split: a plain store is cheaper
  // in the GEMM epilogue than a read-modify-write of the stream) are added to the residual stream by
  // the norm kernel that follows.
  const int so = gemm_residual_splits(T, d, c.n_q_heads * c.head_dim), sd = gemm_residual_splits(T, d, c.d_ffn);
  // The QKV projection is narrow as well; when its tiles leave half the CUs idle it is split along K
  // into fp32 partial products (in `parts`, free at that point) that rope_append adds up, which also
  // spares q and k a rounding.
  int sq = 256 / (ceil_div(T, 128) * (m->qkv_rows() / 128));
  if (sq > d / 256) sq = d / 256;
  if (sq > 8 * d / m->qkv_rows()) sq = 8 * d / m->qkv_rows();
  if (sq > 4) sq = 4;
  // ... unless 64-row tiles alone occupy at least three quarters of the CUs: then the unsplit projection in
  // 64-row tiles is as fast, and rope_append reads bf16 instead of partial products (1.5B shape, 1024 tokens: -0.8 %)
  if (ceil_div(T, 64) * (m->qkv_rows() / 128) >= 192) sq = 1;
  if (sq < 2) sq = 1;
  // one projection: bf16 weights, or packed 4-bit weights with their group scales
  auto project = [&](const bf16 *a, const bf16 *wt, const bf16 *scale, void *out, int N, int K, int epi, int splits,
                     int part, const bf16 *wt_blocked = nullptr) {
    if (!m->w4) return launch_gemm(a, wt, out, T, N, K, epi, st, splits, part, wt_blocked);
    if (part == GEMM_PART_SMALL) return (arb_status)ARB_OK;            // the 4-bit kernel is one launch
    return launch_gemm_w4(a, (const uint32_t *)wt, scale, out, T, N, K, epi, st, splits);
  };
  auto scale_of = [&](const std::vector<const bf16 *> &v, int l) { return m->w4 ? v[l] : (const bf16 *)nullptr; };
  int pending = 0;
  arb_status s;
  if ((s = launch_token_meta(bt->prefix_lens, bt->cu_step_lens, bt->block_tables, B, T, bt->max_blocks_per_seq,
                             c.kv_block, w.tok_pos, w.tok_slot, st)))
    return s;
  if ((s = launch_rope_table(w.tok_pos, T, c.head_dim, c.rope_base, w.cs, st))) return s;
  for (int l = l0; l < l1; ++l) {
    {
      TraceScope t(m, ARB_STAGE_NORM, st);
      if (l == 0 && !h_in)
        s = launch_embed_rmsnorm(m->embed, bt->token_ids, m->g_attn[0], c.rms_eps, T, d, w.h, w.x, st);
      else
        s = launch_rmsnorm(w.h, w.parts, pending, m->g_attn[l], c.rms_eps, T, d, w.x, st);
      pending = 0;
    }
    if (s) return s;
    {
      TraceScope t(m, ARB_STAGE_QKV, st);
      if (sq > 1)
        s = project(w.x, m->wqkv[l], scale_of(m->sqkv, l), w.parts, m->qkv_rows(), d, ARB_EPI_STORE_F32, sq, GEMM_PART_ALL);
      else
        s = project(w.x, m->wqkv[l], scale_of(m->sqkv, l), w.qkv, m->qkv_rows(), d, ARB_EPI_STORE_BF16, 1, GEMM_PART_ALL);
    }
    if (s) return s;
    {
      TraceScope t(m, ARB_STAGE_ROPE_APPEND, st);
      // the queries leave the rotary kernel multiplied by log2(e)/sqrt(hd) (in fp32, before their one rounding)
      s = launch_rope_append(w.qkv, w.parts, sq > 1 ? sq : 0, w.cs, w.tok_slot, (bf16 *)kv->k_pool[l], (bf16 *)kv->v_pool[l], T, c.n_q_heads,
                             c.n_kv_heads, c.head_dim, attention_q_scale(c.head_dim), st);
    }
    if (s) return s;
    {
      TraceScope t(m, ARB_STAGE_ATTENTION, st);
      s = launch_attention(w.qkv, m->qkv_rows(), (const bf16 *)kv->k_pool[l], (const bf16 *)kv->v_pool[l],
                           bt->block_tables, bt->max_blocks_per_seq, bt->prefix_lens, bt->cu_step_lens, B, T,
                           c.n_q_heads, c.n_kv_heads, c.head_dim, plan, w.tok_pos, w.attn, w.attn_ws, w.attn_ws_bytes, st, true);
    }
    if (s) return s;
    {
      TraceScope t(m, ARB_STAGE_OPROJ, st);
      s = project(w.attn, m->wo[l], scale_of(m->so, l), w.parts, d, c.n_q_heads * c.head_dim,
                  so > 1 ? ARB_EPI_RESIDUAL_F32 : ARB_EPI_STORE_F32, so, GEMM_PART_ALL);
      pending = so;
    }
    if (s) return s;
    if ((s = launch_rmsnorm(w.h, w.parts, pending, m->g_mlp[l], c.rms_eps, T, d, w.x, st))) return s;
    pending = 0;
    {
      TraceScope t(m, ARB_STAGE_GATE_UP, st);
      {
        TraceScope large(m, ARB_STAGE_GATE_UP_LARGE, st);
        s = project(w.x, m->wgu[l], scale_of(m->sgu, l), w.act, c.d_ffn, d, ARB_EPI_SWIGLU_BF16, 1, GEMM_PART_LARGE,
                    m->wgu_blocked.empty() ? nullptr : m->wgu_blocked[l]);
      }
      if (!s) s = project(w.x, m->wgu[l], scale_of(m->sgu, l), w.act, c.d_ffn, d, ARB_EPI_SWIGLU_BF16, 1, GEMM_PART_SMALL);
    }
    if (s) return s;
    {
      TraceScope t(m, ARB_STAGE_DOWN, st);
      s = project(w.act, m->wd[l], scale_of(m->sd, l), w.parts, d, c.d_ffn,
                  sd > 1 ? ARB_EPI_RESIDUAL_F32 : ARB_EPI_STORE_F32, sd, GEMM_PART_ALL);
      pending = sd;
    }
    if (s) return s;
  }
  if (h_in) {
    // fold the last projection's partial products into the residual stream, then hand it back
    if (pending && (s = launch_rmsnorm(w.h, w.parts, pending, m->g_final, c.rms_eps, T, d, w.x, st))) return s;
    ARB_CHECK_HIP(hipMemcpyAsync(h_out, w.h, (size_t)T * d * sizeof(float), hipMemcpyDeviceToDevice, st));
    return ARB_OK;
  }
  const bool two_class = c.has_router_head == ARB_HEAD_TWO_CLASS;
  if ((s = launch_final_norm_head(w.h, w.parts, pending, m->g_final, c.rms_eps, T, d, with_head ? m->w_head : nullptr,
                                  with_head && two_class ? m->w_head + d : nullptr,
                                  (bf16 *)hidden_out, with_head ? w.tok_dot : nullptr, st)))
    return s;
  if (with_head)
    if ((s = launch_pool_route(w.tok_dot, bt->cu_step_lens, B, m->b_head, c.pool, two_class, tau, scores, escalate, st))) return s;
  return ARB_OK;
}

extern "C" arb_status arb_score_steps(arb_model *m, const arb_kv *kv, const arb_batch *batch, float tau, float *scores,
                                      uint8_t *escalate, void *hidden_out, void *ws, size_t ws_bytes, void *stream) {
  if (!m) return arb_fail(ARB_EINVAL, "null model");
  return forward(m, kv, batch, m->cfg.has_router_head != 0, tau, scores, escalate, hidden_out, ws, ws_bytes,
                 (hipStream_t)stream, 0, m->cfg.n_layers);
}

// ---- the entry point that allocates nothing: the workspace is a static device array ----

// Every GPU the library runs on holds its own copy of this array (at its own address) until the process
// ends.  In host code the name is only a handle for hipGetSymbolAddress: kernels and copies get the
// per-device address resolved below, never the name.
static __device__ __align__(256) unsigned char scratch[ARB_NOALLOC_SCRATCH_BYTES];

static const int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, once resolved
static std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch`, looked up once per device.
static arb_status static_scratch(void **out) {
  int dev = -1;
  ARB_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return arb_fail(ARB_EUNSUPPORTED, "arb_score_steps_noalloc: device index %d", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    ARB_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return arb_fail(ARB_EHIP, "arb_score_steps_noalloc: the static scratch buffer has no address on device %d", dev);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ARB_OK;
}

extern "C" arb_status arb_score_steps_noalloc(arb_model *m, const arb_kv *kv, const arb_batch *batch, float tau,
                                              float *scores, uint8_t *escalate, void *hidden_out, void *stream) {
  if (!m) return arb_fail(ARB_EINVAL, "null model");
  void *ws = nullptr;
  if (arb_status s = static_scratch(&ws)) return s;
  // Nothing in the workspace is read before this call has written it (every buffer is a kernel's output
  // before it is another's input), so the previous call's contents need no clearing.
  return forward(m, kv, batch, m->cfg.has_router_head != 0, tau, scores, escalate, hidden_out, ws,
                 ARB_NOALLOC_SCRATCH_BYTES, (hipStream_t)stream, 0, m->cfg.n_layers, nullptr, nullptr, true);
}

extern "C" arb_status arb_prefill(arb_model *m, const arb_kv *kv, const arb_batch *batch, void *hidden_out, void *ws,
                                  size_t ws_bytes, void *stream) {
  if (!m) return arb_fail(ARB_EINVAL, "null model");
  return forward(m, kv, batch, false, 0.f, nullptr, nullptr, hidden_out, ws, ws_bytes, (hipStream_t)stream, 0,
                 m->cfg.n_layers);
}

extern "C" arb_status arb_route(const float *scores, int32_t n, float tau, int32_t sense, uint8_t *escalate,
                                void *stream) {
  if (n < 0) return arb_fail(ARB_EINVAL, "arb_route: n = %d", n);
  if (n == 0) return ARB_OK;
  if (!scores || !escalate) return arb_fail(ARB_EINVAL, "arb_route: null pointer");
  if (sense != ARB_ESCALATE_IF_GT && sense != ARB_ACCEPT_IF_GT) return arb_fail(ARB_EINVAL, "arb_route: sense %d", sense);
  return launch_route(scores, n, tau, sense, escalate, (hipStream_t)stream);
}

extern "C" arb_status arb_advantage_route(const float *s_t, const float *s_d, int32_t n, float tau,
                                       const float *tau_device, float *delta, uint8_t *escalate, float *realized,
                                       void *stream) {
  if (n < 0) return arb_fail(ARB_EINVAL, "arb_advantage_route: n = %d", n);
  if (n == 0) return ARB_OK;
  if (!s_t || !s_d) return arb_fail(ARB_EINVAL, "arb_advantage_route: null score array");
  if (!delta && !escalate && !realized) return arb_fail(ARB_EINVAL, "arb_advantage_route: no output requested");
  return launch_advantage_route(s_t, s_d, n, tau, tau_device, delta, escalate, realized, (hipStream_t)stream);
}

extern "C" arb_status arb_budget_threshold(const float *delta, int32_t n, int32_t budget, float *tau_out,
                                           void *stream) {
  if (n < 0 || budget < 0) return arb_fail(ARB_EINVAL, "arb_budget_threshold: n = %d, budget = %d", n, budget);
  if (!tau_out || (n > 0 && !delta)) return arb_fail(ARB_EINVAL, "arb_budget_threshold: null pointer");
  return launch_budget_threshold(delta, n, budget, tau_out, (hipStream_t)stream);
}

extern "C" size_t arb_next_token_workspace_bytes(int32_t n, int32_t d_model, int32_t vocab) {
  if (n < 0 || d_model <= 0 || vocab <= 0) return 0;
  return align_up((size_t)n * d_model * sizeof(bf16), 256) + align_up((size_t)n * vocab * sizeof(float), 256);
}

extern "C" arb_status arb_next_token(const void *hidden, const int32_t *rows, int32_t n, int32_t d_model,
                                     const void *w_lm, int32_t vocab, float temperature, const float *uniforms,
                                     int32_t *token, float *chosen_logit, void *ws, size_t ws_bytes, void *stream) {
  if (n < 0) return arb_fail(ARB_EINVAL, "arb_next_token: n = %d", n);
  if (n == 0) return ARB_OK;
  if (!hidden || !rows || !w_lm || !token) return arb_fail(ARB_EINVAL, "arb_next_token: null pointer");
  if (d_model <= 0 || vocab <= 0) return arb_fail(ARB_ESHAPE, "arb_next_token: d_model %d, vocab %d", d_model, vocab);
  if (temperature > 0.f && !uniforms) return arb_fail(ARB_EINVAL, "arb_next_token: sampling needs uniforms");
  const size_t need = arb_next_token_workspace_bytes(n, d_model, vocab);
  if (!ws || ws_bytes < need) return arb_fail(ARB_ECAPACITY, "arb_next_token: workspace %zu < %zu bytes", ws_bytes, need);
  bf16 *x = (bf16 *)ws;
  float *logits = (float *)((char *)ws + align_up((size_t)n * d_model * sizeof(bf16), 256));
  hipStream_t st = (hipStream_t)stream;
  arb_status s;
  if ((s = launch_gather_rows((const bf16 *)hidden, rows, n, d_model, x, st))) return s;
  if ((s = launch_gemm(x, (const bf16 *)w_lm, logits, n, vocab, d_model, ARB_EPI_STORE_F32, st))) return s;
  return launch_sample_token(logits, n, vocab, temperature, uniforms, token, chosen_logit, st);
}

extern "C" arb_status arb_first_stop(const int32_t *tokens, int32_t n, int32_t max_len, int32_t sep, int32_t eos,
                                     int32_t *len, uint8_t *ended, void *stream) {
  if (n < 0 || max_len < 0) return arb_fail(ARB_EINVAL, "arb_first_stop: n = %d, max_len = %d", n, max_len);
  if (n == 0) return ARB_OK;
  if (!len || (max_len > 0 && !tokens)) return arb_fail(ARB_EINVAL, "arb_first_stop: null pointer");
  return launch_first_stop(tokens, n, max_len, sep, eos, len, ended, (hipStream_t)stream);
}

extern "C" arb_status arb_step_advance(const int32_t *open_rows, const int32_t *chosen, int32_t n_open, int32_t n,
                                       int32_t max_len, int32_t sep, int32_t eos, int32_t *steps, int32_t *len,
                                       uint8_t *done, int32_t *next_rows, int32_t *next_ids, int32_t *n_next,
                                       void *stream) {
  if (n < 0 || n_open < 0 || n_open > n || max_len <= 0)
    return arb_fail(ARB_EINVAL, "arb_step_advance: n = %d, n_open = %d, max_len = %d", n, n_open, max_len);
  if (!n_next) return arb_fail(ARB_EINVAL, "arb_step_advance: null pointer");
  if (n_open > 0 && (!open_rows || !chosen || !steps || !len || !done || !next_rows || !next_ids))
    return arb_fail(ARB_EINVAL, "arb_step_advance: null pointer");
  return launch_step_advance(open_rows, chosen, n_open, max_len, sep, eos, steps, len, done, next_rows, next_ids, n_next,
                             (hipStream_t)stream);
}

extern "C" arb_status arb_pack_steps(const int32_t *steps, int32_t max_len, const int32_t *rows, const int32_t *cu,
                                     int32_t n_rows, int32_t *ids, void *stream) {
  if (n_rows < 0 || max_len <= 0) return arb_fail(ARB_EINVAL, "arb_pack_steps: n_rows = %d, max_len = %d", n_rows, max_len);
  if (n_rows == 0) return ARB_OK;
  if (!steps || !rows || !cu || !ids) return arb_fail(ARB_EINVAL, "arb_pack_steps: null pointer");
  return launch_pack_steps(steps, max_len, rows, cu, n_rows, ids, (hipStream_t)stream);
}

extern "C" arb_status arb_slot_mapping(const arb_batch *batch, int32_t kv_block, int32_t *slots, void *stream) {
  BatchInfo info;
  if (kv_block <= 0) return arb_fail(ARB_EINVAL, "arb_slot_mapping: kv_block %d", kv_block);
  if (arb_status s = check_batch(batch, kv_block, &info, false)) return s;
  if (batch->batch == 0) return ARB_OK;
  if (!slots) return arb_fail(ARB_EINVAL, "arb_slot_mapping: null output");
  return launch_token_meta(batch->prefix_lens, batch->cu_step_lens, batch->block_tables, batch->batch,
                           batch->total_tokens, batch->max_blocks_per_seq, kv_block, nullptr, slots,
                           (hipStream_t)stream);
}

// ------------------------------------------------------------------------- stages

extern "C" arb_status arb_stage_gemm(const void *A, const void *B, const void *B_blocked, void *C, int32_t M,
                                     int32_t N, int32_t K, int32_t epilogue, void *stream) {
  if (M == 0) return ARB_OK;
  if (!A || !B || !C) return arb_fail(ARB_EINVAL, "arb_stage_gemm: null pointer");
  return launch_gemm((const bf16 *)A, (const bf16 *)B, C, M, N, K, epilogue, (hipStream_t)stream, 1, GEMM_PART_ALL,
                     (const bf16 *)B_blocked);
}

extern "C" arb_status arb_pack_k_blocked(const void *W, int64_t rows, int32_t K, void *packed, void *stream) {
  if (rows < 0) return arb_fail(ARB_EINVAL, "arb_pack_k_blocked: rows = %lld", (long long)rows);
  if (rows > 0 && (!W || !packed)) return arb_fail(ARB_EINVAL, "arb_pack_k_blocked: null pointer");
  return launch_pack_k_blocked((const bf16 *)W, (size_t)rows, K, (bf16 *)packed, (hipStream_t)stream);
}

extern "C" arb_status arb_w4_quantize(const void *W, int32_t N, int32_t K, void *packed, void *scales, void *stream) {
  if (N == 0) return ARB_OK;
  if (!W || !packed || !scales) return arb_fail(ARB_EINVAL, "arb_w4_quantize: null pointer");
  return launch_w4_quantize((const bf16 *)W, N, K, (uint32_t *)packed, (bf16 *)scales, 4, (hipStream_t)stream);
}

extern "C" arb_status arb_w3_quantize(const void *W, int32_t N, int32_t K, void *packed, void *scales, void *stream) {
  if (N == 0) return ARB_OK;
  if (!W || !packed || !scales) return arb_fail(ARB_EINVAL, "arb_w3_quantize: null pointer");
  return launch_w4_quantize((const bf16 *)W, N, K, (uint32_t *)packed, (bf16 *)scales, 3, (hipStream_t)stream);
}

extern "C" arb_status arb_stage_gemm_w4(const void *A, const void *packed, const void *scales, void *C, int32_t M,
                                        int32_t N, int32_t K, int32_t epilogue, void *stream) {
  if (M == 0) return ARB_OK;
  if (!A || !packed || !scales || !C) return arb_fail(ARB_EINVAL, "arb_stage_gemm_w4: null pointer");
  return launch_gemm_w4((const bf16 *)A, (const uint32_t *)packed, (const bf16 *)scales, C, M, N, K, epilogue,
                        (hipStream_t)stream);
}

extern "C" int32_t arb_gemm_large_tile_columns(int32_t M, int32_t N, int32_t K, int32_t epilogue) {
  return gemm_large_cols(M, N, K, epilogue, 1);
}

extern "C" arb_status arb_stage_attention(const arb_model *m, const void *q, int32_t q_row_stride, int32_t q_scaled,
                                          const void *k_pool, const void *v_pool, const arb_batch *batch, void *out,
                                          void *ws, size_t ws_bytes, void *stream) {
  if (!m) return arb_fail(ARB_EINVAL, "null model");
  const arb_model_cfg &c = m->cfg;
  BatchInfo info;
  if (arb_status s = check_batch(batch, c.kv_block, &info, false)) return s;
  if (batch->batch == 0) return ARB_OK;
  if (!q || !k_pool || !v_pool || !out) return arb_fail(ARB_EINVAL, "arb_stage_attention: null pointer");
  if (q_row_stride < c.n_q_heads * c.head_dim || q_row_stride % 8 != 0)
    return arb_fail(ARB_EINVAL, "arb_stage_attention: q_row_stride %d", q_row_stride);
  const AttnPlan plan = plan_attention(batch->batch, batch->prefix_lens_host, batch->cu_step_lens_host,
                                       c.n_q_heads / c.n_kv_heads, c.n_kv_heads);
  return launch_attention((const bf16 *)q, q_row_stride, (const bf16 *)k_pool, (const bf16 *)v_pool,
                          batch->block_tables, batch->max_blocks_per_seq, batch->prefix_lens, batch->cu_step_lens,
                          batch->batch, batch->total_tokens, c.n_q_heads, c.n_kv_heads, c.head_dim, plan, nullptr, (bf16 *)out,
                          ws, ws_bytes, (hipStream_t)stream, q_scaled != 0);
}

extern "C" arb_status arb_stage_rmsnorm(const float *x, const float *g, float eps, int32_t T, int32_t d, void *out,
                                        void *stream) {
  if (T < 0) return arb_fail(ARB_EINVAL, "arb_stage_rmsnorm: T = %d", T);
  if (T == 0) return ARB_OK;
  if (!x || !g || !out) return arb_fail(ARB_EINVAL, "arb_stage_rmsnorm: null pointer");
  return launch_rmsnorm(const_cast<float *>(x), nullptr, 0, g, eps, T, d, (bf16 *)out, (hipStream_t)stream);
}

extern "C" arb_status arb_stage_rope_append(const arb_model *m, void *qkv, void *k_pool, void *v_pool,
                                            const arb_batch *batch, void *ws, size_t ws_bytes, void *stream) {
  if (!m) return arb_fail(ARB_EINVAL, "null model");
  const arb_model_cfg &c = m->cfg;
  BatchInfo info;
  if (arb_status s = check_batch(batch, c.kv_block, &info, false)) return s;
  if (batch->batch == 0) return ARB_OK;
  if (!qkv || !k_pool || !v_pool) return arb_fail(ARB_EINVAL, "arb_stage_rope_append: null pointer");
  const size_t T = batch->total_tokens;
  const size_t need = 2 * align_up(T * sizeof(int32_t), 256) + align_up(T * (c.head_dim / 2) * sizeof(f32x2), 256);
  if (!ws || ws_bytes < need) return arb_fail(ARB_ECAPACITY, "arb_stage_rope_append: workspace %zu < %zu bytes", ws_bytes, need);
  int32_t *tok_pos = (int32_t *)ws;
  int32_t *tok_slot = (int32_t *)((char *)ws + align_up(T * sizeof(int32_t), 256));
  f32x2 *cs = (f32x2 *)((char *)ws + 2 * align_up(T * sizeof(int32_t), 256));
  hipStream_t st = (hipStream_t)stream;
  arb_status s;
  if ((s = launch_token_meta(batch->prefix_lens, batch->cu_step_lens, batch->block_tables, batch->batch, (int)T,
                             batch->max_blocks_per_seq, c.kv_block, tok_pos, tok_slot, st)))
    return s;
  if ((s = launch_rope_table(tok_pos, (int)T, c.head_dim, c.rope_base, cs, st))) return s;
  return launch_rope_append((bf16 *)qkv, nullptr, 0, cs, tok_slot, (bf16 *)k_pool, (bf16 *)v_pool, (int)T, c.n_q_heads,
                            c.n_kv_heads, c.head_dim, 1.0f, st);
}

extern "C" arb_status arb_stage_layers(arb_model *m, const arb_kv *kv, const arb_batch *batch, int32_t layer_begin,
                                       int32_t layer_end, const float *h_in, float *h_out, void *ws, size_t ws_bytes,
                                       void *stream) {
  if (!m) return arb_fail(ARB_EINVAL, "null model");
  if (layer_begin < 0 || layer_end > m->cfg.n_layers || layer_begin >= layer_end)
    return arb_fail(ARB_EINVAL, "arb_stage_layers: layers [%d, %d) of %d", layer_begin, layer_end, m->cfg.n_layers);
  if (batch && batch->batch > 0 && (!h_in || !h_out)) return arb_fail(ARB_EINVAL, "arb_stage_layers: null residual stream");
  return forward(m, kv, batch, false, 0.f, nullptr, nullptr, nullptr, ws, ws_bytes, (hipStream_t)stream, layer_begin,
                 layer_end, h_in, h_out);
}

extern "C" arb_status arb_stage_norm_pool_head(const float *h, const float *g_final, float eps, const arb_batch *batch,
                                               int32_t d, const float *w_head, float b_head, int32_t pool, float tau,
                                               void *hidden_out, float *scores, uint8_t *escalate, void *ws,
                                               size_t ws_bytes, void *stream) {
  BatchInfo info;
  if (arb_status s = check_batch(batch, ARB_KV_BLOCK, &info, false)) return s;
  if (batch->batch == 0) return ARB_OK;
  if (!h || !g_final || !w_head || !scores) return arb_fail(ARB_EINVAL, "arb_stage_norm_pool_head: null pointer");
  if (pool != ARB_POOL_MEAN && pool != ARB_POOL_LAST) return arb_fail(ARB_EINVAL, "arb_stage_norm_pool_head: pool %d", pool);
  const size_t need = (size_t)batch->total_tokens * sizeof(float);
  if (!ws || ws_bytes < need) return arb_fail(ARB_ECAPACITY, "arb_stage_norm_pool_head: workspace %zu < %zu bytes", ws_bytes, need);
  hipStream_t st = (hipStream_t)stream;
  if (arb_status s = launch_final_norm_head(h, nullptr, 0, g_final, eps, batch->total_tokens, d, w_head, nullptr, (bf16 *)hidden_out,
                                            (float *)ws, st))
    return s;
  return launch_pool_route((const float *)ws, batch->cu_step_lens, batch->batch, b_head, pool, 0, tau, scores, escalate, st);
}
