// C-ABI of libsurelock: argument validation, buffer carving and the launch sequence of one
// SureLock step.  Everything here runs on the host; no device memory is allocated.
#include "sl_common.h"
#include <new>
#include <string.h>

thread_local int g_sl_last_hip_error = 0;

extern "C" int sl_last_hip_error(void) { return g_sl_last_hip_error; }

extern "C" const char* sl_strerror(int status) {
  switch (status) {
    case SL_OK: return "ok";
    case SL_EINVAL: return "invalid argument (null pointer, shape, dtype or alignment)";
    case SL_ENOSPC: return "caller-provided buffer too small";
    case SL_EHIP: return "HIP runtime error (see sl_last_hip_error)";
    case SL_ESTATE: return "call order violated (weights, K/V cache or posterior store not bound)";
    default: return "unknown status";
  }
}

static bool cfg_ok(const sl_config* c) {
  if (!c) return false;
  if (c->n_layers < 1 || c->d_model < 8 || c->n_heads < 1 || c->d_head < 2 || c->d_ff < 8 || c->vocab < 8) return false;
  if (c->dtype != SL_F32 && c->dtype != SL_BF16) return false;
  if (!(c->d_head == 32 || c->d_head == 64 || c->d_head == 128 || c->d_head == 256)) return false;
  if (c->vocab % 8 || c->d_model % 8 || c->d_ff % 8) return false;
  if (c->mask_id < 0 || c->mask_id >= c->vocab) return false;
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return false;
  if (c->candidates_pre_update != 0 && c->candidates_pre_update != 1) return false;
  if (!(c->gate_percentile >= 0.f) || c->gate_percentile > 100.f) return false;
  if (!(c->temperature >= 0.f)) return false;
  return true;
}

extern "C" int sl_init(const sl_config* cfg, sl_ctx** out) {
  if (!out) return SL_EINVAL;
  *out = nullptr;
  if (!cfg_ok(cfg)) return SL_EINVAL;
  sl_ctx* c = new (std::nothrow) sl_ctx();
  if (!c) return SL_ENOSPC;
  memset(c, 0, sizeof(*c));
  c->cfg = *cfg;
  c->layers = new (std::nothrow) sl_layer_weights[cfg->n_layers];
  c->packed = new (std::nothrow) sl_packed_layer[cfg->n_layers];
  if (!c->layers || !c->packed) { delete[] c->layers; delete[] c->packed; delete c; return SL_ENOSPC; }
  memset(c->packed, 0, sizeof(sl_packed_layer) * cfg->n_layers);
  c->use_mfma = sl_mfma_supported(cfg);
  *out = c;
  return SL_OK;
}

static void prof_free(sl_ctx* ctx) {
  if (!ctx->prof) return;
  for (int i = 0; i < 2 * ctx->prof->cap; ++i)
    if (ctx->prof->ev[i]) (void)hipEventDestroy(ctx->prof->ev[i]);
  delete[] ctx->prof->ev;
  delete[] ctx->prof->slot;
  delete ctx->prof;
  ctx->prof = nullptr;
}

extern "C" int sl_profile_begin(sl_ctx* ctx, int32_t max_launches) {
  if (!ctx || max_launches < 1 || max_launches > (1 << 20)) return SL_EINVAL;
  prof_free(ctx);
  sl_prof* p = new (std::nothrow) sl_prof();
  if (!p) return SL_ENOSPC;
  p->cap = max_launches;
  p->n = 0;
  p->ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_launches]();
  p->slot = new (std::nothrow) int[max_launches];
  ctx->prof = p;
  if (!p->ev || !p->slot) { prof_free(ctx); return SL_ENOSPC; }
  for (int i = 0; i < 2 * max_launches; ++i) {
    const hipError_t e = hipEventCreate(&p->ev[i]);
    if (e != hipSuccess) { g_sl_last_hip_error = (int)e; prof_free(ctx); return SL_EHIP; }
  }
  return SL_OK;
}

extern "C" int sl_profile_end(sl_ctx* ctx, float* ms, int32_t* launches) {
  if (!ctx || !ms || !launches) return SL_EINVAL;
  if (!ctx->prof) return SL_ESTATE;
  for (int i = 0; i < SL_PROF_SLOTS; ++i) { ms[i] = 0.f; launches[i] = 0; }
  sl_prof* p = ctx->prof;
  int rc = SL_OK;
  if (p->n > 0) {
    hipError_t e = hipEventSynchronize(p->ev[2 * p->n - 1]);
    for (int i = 0; i < p->n && e == hipSuccess; ++i) {
      float t = 0.f;
      e = hipEventElapsedTime(&t, p->ev[2 * i], p->ev[2 * i + 1]);
      ms[p->slot[i]] += t;
      launches[p->slot[i]] += 1;
    }
    if (e != hipSuccess) { g_sl_last_hip_error = (int)e; rc = SL_EHIP; }
  }
  prof_free(ctx);
  return rc;
}

extern "C" int sl_destroy(sl_ctx* ctx) {
  if (!ctx) return SL_EINVAL;
  prof_free(ctx);
  delete[] ctx->layers;
  delete[] ctx->packed;
  delete ctx;
  return SL_OK;
}

// ---- weights -----------------------------------------------------------------------------------
extern "C" int sl_packed_weights_bytes(const sl_ctx* ctx, size_t* out) {
  if (!ctx || !out) return SL_EINVAL;
  *out = ctx->use_mfma ? sl_mfma_packed_bytes(&ctx->cfg) : 0;
  return SL_OK;
}

extern "C" int sl_bind_weights(sl_ctx* ctx, void* stream, const sl_weights* w, void* packed, size_t packed_bytes) {
  if (!ctx || !w || !w->emb || !w->final_norm || !w->lm_head || !w->layers) return SL_EINVAL;
  for (int l = 0; l < ctx->cfg.n_layers; ++l) {
    const sl_layer_weights& L = w->layers[l];
    if (!L.attn_norm || !L.wq || !L.wk || !L.wv || !L.wo || !L.ffn_norm || !L.w_gate || !L.w_up || !L.w_down)
      return SL_EINVAL;
  }
  if (ctx->use_mfma) {
    if (!packed) return SL_EINVAL;
    if (packed_bytes < sl_mfma_packed_bytes(&ctx->cfg)) return SL_ENOSPC;
    if ((uintptr_t)packed % 256) return SL_EINVAL;
  }
  ctx->plain = *w;
  memcpy(ctx->layers, w->layers, sizeof(sl_layer_weights) * ctx->cfg.n_layers);
  ctx->plain.layers = ctx->layers;
  if (ctx->use_mfma) {
    const int rc = sl_mfma_pack_all(ctx, (hipStream_t)stream, packed);
    if (rc != SL_OK) return rc;
  }
  ctx->weights_bound = true;
  return SL_OK;
}

// ---- K/V cache ---------------------------------------------------------------------------------
static size_t rope_tab_bytes(const sl_config& c, int n_pad) {
  return sl_align_up((size_t)n_pad * (c.d_head / 2) * sizeof(float2), 256);
}

extern "C" int sl_kv_cache_bytes(const sl_ctx* ctx, int32_t batch, int32_t n_seq, size_t* out) {
  if (!ctx || !out || batch < 1 || batch > SL_MAX_BATCH || n_seq < 1) return SL_EINVAL;
  const sl_config& c = ctx->cfg;
  const int n_pad = (int)sl_align_up(n_seq, 64);
  const size_t layer = (size_t)batch * c.n_heads * n_pad * c.d_head;
  *out = rope_tab_bytes(c, n_pad) + 2 * (size_t)c.n_layers * layer * sl_tsize(c.dtype);
  return SL_OK;
}

extern "C" int sl_kv_cache_bind(sl_ctx* ctx, void* stream, void* kv, size_t bytes, int32_t batch, int32_t n_seq) {
  size_t need = 0;
  const int rc = sl_kv_cache_bytes(ctx, batch, n_seq, &need);
  if (rc != SL_OK) return rc;
  if (!kv || (uintptr_t)kv % 256) return SL_EINVAL;
  if (bytes < need) return SL_ENOSPC;
  if ((size_t)batch * n_seq > (size_t)1 << 30) return SL_EINVAL;
  const sl_config& c = ctx->cfg;
  ctx->kv = kv;
  ctx->batch = batch;
  ctx->n_seq = n_seq;
  ctx->n_pad = (int)sl_align_up(n_seq, 64);
  ctx->kv_layer_elems = (size_t)batch * c.n_heads * ctx->n_pad * c.d_head;
  int r2 = slk_fill_zero((hipStream_t)stream, kv, need);
  if (r2 != SL_OK) return r2;
  return slk_rope_table((hipStream_t)stream, kv, ctx->n_pad, c.d_head, c.rope_theta);
}

static inline char* kv_k_layer(const sl_ctx* ctx, int l) {
  const size_t ts = sl_tsize(ctx->cfg.dtype);
  return (char*)ctx->kv + rope_tab_bytes(ctx->cfg, ctx->n_pad) + (size_t)l * ctx->kv_layer_elems * ts;
}
static inline char* kv_v_layer(const sl_ctx* ctx, int l) {
  const size_t ts = sl_tsize(ctx->cfg.dtype);
  return kv_k_layer(ctx, ctx->cfg.n_layers) + (size_t)l * ctx->kv_layer_elems * ts;
}

extern "C" int sl_kv_cache_read(const sl_ctx* ctx, void* stream, int32_t layer, void* k_out, void* v_out) {
  if (!ctx || !k_out || !v_out) return SL_EINVAL;
  if (!ctx->kv) return SL_ESTATE;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return SL_EINVAL;
  return slk_kv_read((hipStream_t)stream, ctx->cfg.dtype, kv_k_layer(ctx, layer), kv_v_layer(ctx, layer), ctx->batch,
                     ctx->cfg.n_heads, ctx->n_seq, ctx->n_pad, ctx->cfg.d_head, k_out, v_out, ctx->use_mfma ? 1 : 0);
}

// ---- posterior store -----------------------------------------------------------------------------
// Rows per buffer: B*N rounded up until a buffer is a whole number of 256-byte units, so that the
// second buffer starts aligned AND a whole number of rows after the first (row index B*N' + g of
// the first buffer is row g of the second).
static size_t post_rows(const sl_ctx* ctx, int32_t batch, int32_t n_seq) {
  const size_t row_bytes = (size_t)ctx->cfg.vocab * sl_tsize(ctx->cfg.dtype);
  size_t unit = 256;
  while (unit > 1 && row_bytes % unit) unit >>= 1;          // largest power of two <= 256 dividing a row
  return sl_align_up((size_t)batch * n_seq, 256 / unit);
}

extern "C" int sl_posterior_bytes(const sl_ctx* ctx, int32_t batch, int32_t n_seq, size_t* out) {
  if (!ctx || !out || batch < 1 || n_seq < 1) return SL_EINVAL;
  *out = 2 * post_rows(ctx, batch, n_seq) * ctx->cfg.vocab * sl_tsize(ctx->cfg.dtype);
  return SL_OK;
}

extern "C" int sl_posterior_bind(sl_ctx* ctx, void* store, size_t bytes) {
  if (!ctx || !store || (uintptr_t)store % 256) return SL_EINVAL;
  if (!ctx->kv) return SL_ESTATE;          // batch / n_seq come from the cache binding
  size_t need = 0;
  sl_posterior_bytes(ctx, ctx->batch, ctx->n_seq, &need);
  if (bytes < need) return SL_ENOSPC;
  ctx->post = store;
  ctx->post_buf_elems = post_rows(ctx, ctx->batch, ctx->n_seq) * ctx->cfg.vocab;
  return SL_OK;
}

extern "C" int sl_logits_ptr(const sl_ctx* ctx, int32_t t, void** out) {
  if (!ctx || !out || t < 0) return SL_EINVAL;
  if (!ctx->post) return SL_ESTATE;
  *out = (char*)ctx->post + (size_t)(t & 1) * ctx->post_buf_elems * sl_tsize(ctx->cfg.dtype);
  return SL_OK;
}

// ---- workspace -----------------------------------------------------------------------------------
struct Workspace {
  char *x, *h, *q, *o, *a;
  float *f32, *attn;
  void* score;                      // partial states of rows split over several workgroups
  size_t bytes;
};

static Workspace carve(const sl_ctx* ctx, void* base, int rows, int batch, int n_seq) {
  const sl_config& c = ctx->cfg;
  const size_t ts = sl_tsize(c.dtype);
  const size_t hd = (size_t)c.n_heads * c.d_head;
  size_t f32_cols = 3 * hd;
  if ((size_t)2 * c.d_ff > f32_cols) f32_cols = (size_t)2 * c.d_ff;
  if ((size_t)c.d_model > f32_cols) f32_cols = c.d_model;
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t n) { char* p = (char*)base + off; off += sl_align_up(n, 256); return p; };
  const size_t rows32 = sl_align_up((size_t)rows, 32);     // tiled activation buffers hold whole 32-row blocks
  w.x = take((size_t)rows * c.d_model * ts);
  w.h = take(rows32 * c.d_model * ts);
  // q doubles as scratch once the layers are done (token draws: ids + per-part candidates; probe: row indices)
  size_t q_bytes = (size_t)rows * hd * ts;
  const size_t draw_bytes = sl_align_up((size_t)rows * sizeof(int32_t), 256) + slk_sample_scratch_bytes(rows);
  if (draw_bytes > q_bytes) q_bytes = draw_bytes;
  w.q = take(q_bytes);
  w.o = take(rows32 * hd * ts);
  w.a = take(rows32 * c.d_ff * ts);
  size_t f32_elems = (size_t)rows * f32_cols;
  if (ctx->use_mfma) {
    // the plans' need grows with the row bound: one evaluation for the largest bound seen serves every smaller one
    if (rows > ctx->f32_plan_rows) {
      ctx->f32_plan_elems = sl_mfma_f32_elems(&c, rows);
      ctx->f32_plan_rows = rows;
    }
    if (ctx->f32_plan_elems > f32_elems) f32_elems = ctx->f32_plan_elems;
  }
  w.f32 = (float*)take(f32_elems * sizeof(float));
  w.attn = nullptr;
  if (ctx->use_mfma) {
    const int n_pad = (int)sl_align_up((size_t)n_seq, 64);
    w.attn = (float*)take(slk_attention_scratch_elems(rows, batch, c.n_heads, n_pad) * sizeof(float));
  }
  w.score = take(slk_score_scratch_bytes());
  w.bytes = off;
  return w;
}

extern "C" int sl_workspace_bytes(const sl_ctx* ctx, int32_t batch, int32_t n_seq, size_t* out) {
  if (!ctx || !out || batch < 1 || n_seq < 1) return SL_EINVAL;
  *out = carve(ctx, nullptr, batch * n_seq, batch, n_seq).bytes;
  return SL_OK;
}

// ---- the restricted forward ------------------------------------------------------------------------
#define SL_TRY(expr) do { const int rc_ = (expr); if (rc_ != SL_OK) return rc_; } while (0)

// Layers [lo, hi) on the rows held in ws.x, with ws.h = RMSNorm(ws.x) by layer lo's attention
// gain on entry.  On exit ws.x is the block output and ws.h its RMSNorm by the next gain
// (layer hi's attention gain, or the final gain after the last layer).
static int run_layers(sl_ctx* ctx, hipStream_t s, const Workspace& ws, const int32_t* active_idx,
                      const int32_t* m_dev, int mu, int lo, int hi) {
  const sl_config& c = ctx->cfg;
  const int dt = c.dtype, d = c.d_model, H = c.n_heads, dh = c.d_head, hd = H * dh, dff = c.d_ff;
  const void* rope_tab = ctx->kv;
  for (int l = lo; l < hi; ++l) {
    const sl_layer_weights& L = ctx->layers[l];
    const void* next_gain = (l + 1 < c.n_layers) ? ctx->layers[l + 1].attn_norm : ctx->plain.final_norm;
    if (ctx->use_mfma) {
      SL_TRY(sl_mfma_layer(ctx, s, l, ws.x, ws.h, ws.q, ws.o, ws.a, ws.f32, ws.attn, active_idx, m_dev, mu, next_gain));
      continue;
    }
    // Q, K, V projections of the active rows (fp32 results side by side)
    SL_RUN(ctx, s, SL_PROF_GEMM_QKV, slk_gemm_generic(s, dt, ws.h, L.wq, m_dev, mu, hd, d, ws.f32, nullptr, nullptr, 3 * (size_t)hd));
    SL_RUN(ctx, s, SL_PROF_GEMM_QKV, slk_gemm_generic(s, dt, ws.h, L.wk, m_dev, mu, hd, d, ws.f32 + hd, nullptr, nullptr, 3 * (size_t)hd));
    SL_RUN(ctx, s, SL_PROF_GEMM_QKV, slk_gemm_generic(s, dt, ws.h, L.wv, m_dev, mu, hd, d, ws.f32 + 2 * hd, nullptr, nullptr, 3 * (size_t)hd));
    // RoPE; live K/V overwrite the rows' own cache slots (locked slots are never touched)
    SL_RUN(ctx, s, SL_PROF_ROPE_KV, slk_rope_kv_write(s, dt, ws.f32, 1, 0, active_idx, m_dev, mu, H, dh, ctx->n_seq, ctx->n_pad, rope_tab, ws.q,
                             ctx->probe_read_only ? nullptr : kv_k_layer(ctx, l),
                             ctx->probe_read_only ? nullptr : kv_v_layer(ctx, l), 0));
    SL_RUN(ctx, s, SL_PROF_ATTENTION, slk_attention_generic(s, dt, ws.q, kv_k_layer(ctx, l), kv_v_layer(ctx, l), active_idx, m_dev, mu, H, dh,
                                 ctx->n_seq, ctx->n_pad, ws.o));
    SL_RUN(ctx, s, SL_PROF_GEMM_OUT, slk_gemm_generic(s, dt, ws.o, L.wo, m_dev, mu, d, hd, ws.f32, nullptr, nullptr, d));
    SL_RUN(ctx, s, SL_PROF_ADD_NORM, slk_add_rmsnorm(s, dt, ws.x, ws.f32, 1, 0, m_dev, mu, d, L.ffn_norm, c.rms_eps, ws.h, 0));
    SL_RUN(ctx, s, SL_PROF_GEMM_GATE_UP, slk_gemm_generic(s, dt, ws.h, L.w_gate, m_dev, mu, dff, d, ws.f32, nullptr, nullptr, 2 * (size_t)dff));
    SL_RUN(ctx, s, SL_PROF_GEMM_GATE_UP, slk_gemm_generic(s, dt, ws.h, L.w_up, m_dev, mu, dff, d, ws.f32 + dff, nullptr, nullptr, 2 * (size_t)dff));
    SL_RUN(ctx, s, SL_PROF_SWIGLU, slk_swiglu(s, dt, ws.f32, 1, 0, m_dev, mu, dff, ws.a, 0, 0));
    SL_RUN(ctx, s, SL_PROF_GEMM_DOWN, slk_gemm_generic(s, dt, ws.a, L.w_down, m_dev, mu, d, dff, ws.f32, nullptr, nullptr, d));
    SL_RUN(ctx, s, SL_PROF_ADD_NORM, slk_add_rmsnorm(s, dt, ws.x, ws.f32, 1, 0, m_dev, mu, d, next_gain, c.rms_eps, ws.h, 0));
  }
  return SL_OK;
}

static int check_ready(const sl_ctx* ctx, bool need_post) {
  if (!ctx) return SL_EINVAL;
  if (!ctx->weights_bound || !ctx->kv) return SL_ESTATE;
  if (need_post && !ctx->post) return SL_ESTATE;
  return SL_OK;
}

extern "C" int sl_forward_layers(sl_ctx* ctx, void* stream, const void* x_in, void* x_out, const int32_t* active_idx,
                                 const int32_t* m_dev, int32_t m_upper, int32_t layer_lo, int32_t layer_hi,
                                 void* workspace, size_t workspace_bytes) {
  SL_TRY(check_ready(ctx, false));
  if (!x_in || !x_out || !active_idx || !m_dev || !workspace) return SL_EINVAL;
  if (m_upper < 0 || m_upper > ctx->batch * ctx->n_seq) return SL_EINVAL;
  if (layer_lo < 0 || layer_hi > ctx->cfg.n_layers || layer_lo >= layer_hi) return SL_EINVAL;
  if ((uintptr_t)workspace % 256) return SL_EINVAL;
  if (m_upper == 0) return SL_OK;
  const Workspace ws = carve(ctx, workspace, m_upper, ctx->batch, ctx->n_seq);
  if (workspace_bytes < ws.bytes) return SL_ENOSPC;
  hipStream_t s = (hipStream_t)stream;
  const sl_config& c = ctx->cfg;
  SL_TRY(slk_copy_rows(s, c.dtype, x_in, ws.x, m_dev, m_upper, c.d_model));
  SL_TRY(slk_rmsnorm(s, c.dtype, ws.x, m_dev, m_upper, c.d_model, ctx->layers[layer_lo].attn_norm, c.rms_eps, ws.h, ctx->use_mfma));
  SL_TRY(run_layers(ctx, s, ws, active_idx, m_dev, m_upper, layer_lo, layer_hi));
  return slk_copy_rows(s, c.dtype, ws.x, x_out, m_dev, m_upper, c.d_model);
}

// ---- controller pieces -----------------------------------------------------------------------------
extern "C" int sl_compact_active(void* stream, const uint8_t* lock, int32_t batch, int32_t n_seq,
                                 int32_t* active_idx, int32_t* cu_active) {
  if (!lock || !active_idx || !cu_active || batch < 1 || n_seq < 1) return SL_EINVAL;
  if ((size_t)batch * n_seq > (size_t)1 << 30) return SL_EINVAL;
  return slk_compact_active((hipStream_t)stream, lock, batch, n_seq, batch * n_seq, active_idx, cu_active);
}

extern "C" int sl_score_posteriors(void* stream, const void* logits_cur, int32_t cur_packed, const void* logits_prev,
                                   int32_t dtype, int32_t vocab, const int32_t* active_idx, const int32_t* m_dev,
                                   int32_t m_upper, int32_t first_step, float* kl, float* conf, int32_t* argmax) {
  if (!logits_cur || !active_idx || !m_dev || !kl || !conf || !argmax) return SL_EINVAL;
  if (!first_step && !logits_prev) return SL_EINVAL;
  if (dtype != SL_F32 && dtype != SL_BF16) return SL_EINVAL;
  if (vocab < 8 || vocab % 8 || m_upper < 0) return SL_EINVAL;
  if ((uintptr_t)logits_cur % 16 || (uintptr_t)logits_prev % 16) return SL_EINVAL;
  return slk_score((hipStream_t)stream, logits_cur, cur_packed, logits_prev, dtype, vocab, active_idx, m_dev, m_upper,
                   first_step, kl, conf, argmax, nullptr);
}

extern "C" int sl_unmask_topk(void* stream, int32_t* tokens, uint8_t* masked, const int32_t* active_idx,
                              const int32_t* cu_active, const float* conf, const int32_t* argmax, int32_t batch,
                              int32_t n_seq, int32_t block_lo, int32_t block_hi, int32_t k) {
  if (!tokens || !masked || !active_idx || !cu_active || !conf || !argmax) return SL_EINVAL;
  if (batch < 1 || n_seq < 1 || block_lo < 0 || block_hi > n_seq || block_lo > block_hi || k < 0) return SL_EINVAL;
  if ((size_t)(block_hi - block_lo) * 8 > 60 * 1024) return SL_EINVAL;
  return slk_unmask_topk((hipStream_t)stream, tokens, masked, active_idx, cu_active, conf, argmax, batch, n_seq,
                         block_lo, block_hi, k, batch * n_seq);
}

extern "C" int sl_lock_rule(void* stream, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                            const int32_t* m_dev, int32_t m_upper, const float* kl, const float* eps, int32_t batch,
                            int32_t n_seq, int32_t first_step, uint8_t* new_lock) {
  if (!lock || !masked || !active_idx || !m_dev || !kl || !eps || !new_lock) return SL_EINVAL;
  if (batch < 1 || n_seq < 1 || m_upper < 0) return SL_EINVAL;
  return slk_lock_rule((hipStream_t)stream, lock, masked, active_idx, m_dev, m_upper, kl, eps, batch, n_seq,
                       first_step, new_lock);
}

extern "C" int sl_lock_rule_gated(void* stream, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                                  const int32_t* cu_active, int32_t m_upper, const float* kl, const float* conf,
                                  const float* eps, float gate_percentile, int32_t batch, int32_t n_seq,
                                  int32_t first_step, uint8_t* new_lock) {
  if (!lock || !masked || !active_idx || !cu_active || !kl || !conf || !eps || !new_lock) return SL_EINVAL;
  if (batch < 1 || n_seq < 1 || m_upper < 0) return SL_EINVAL;
  if (!(gate_percentile > 0.f) || gate_percentile > 100.f) return SL_EINVAL;
  return slk_lock_rule_gated((hipStream_t)stream, lock, masked, active_idx, cu_active, m_upper, kl, conf, eps,
                             gate_percentile, batch, n_seq, first_step, new_lock);
}

extern "C" int sl_sample_tokens(void* stream, const void* logits_cur, int32_t cur_packed, int32_t dtype, int32_t vocab,
                               const int32_t* active_idx, const int32_t* m_dev, int32_t m_upper, const uint8_t* masked,
                               int32_t n_seq, int32_t block_lo, int32_t block_hi, float temperature, uint64_t seed,
                               int32_t t, const int32_t* argmax, int32_t* write_id, void* scratch, size_t scratch_bytes) {
  if (!logits_cur || !active_idx || !m_dev || !masked || !argmax || !write_id || !scratch) return SL_EINVAL;
  if (m_upper > 0 && scratch_bytes < slk_sample_scratch_bytes(m_upper)) return SL_ENOSPC;
  if ((dtype != SL_F32 && dtype != SL_BF16) || vocab < 8 || vocab % 8 || m_upper < 0 || n_seq < 1) return SL_EINVAL;
  if (block_lo < 0 || block_hi > n_seq || block_lo > block_hi || !(temperature > 0.f) || t < 1) return SL_EINVAL;
  return slk_sample_tokens((hipStream_t)stream, logits_cur, cur_packed, dtype, vocab, active_idx, m_dev, m_upper, masked,
                           n_seq, block_lo, block_hi, temperature, seed, t, argmax, write_id, scratch);
}

extern "C" int sl_sample_tokens_noalloc(void* stream, const void* logits_cur, int32_t cur_packed, int32_t dtype,
                                       int32_t vocab, const int32_t* active_idx, const int32_t* m_dev, int32_t m_upper,
                                       const uint8_t* masked, int32_t n_seq, int32_t block_lo, int32_t block_hi,
                                       float temperature, uint64_t seed, int32_t t, const int32_t* argmax,
                                       int32_t* write_id) {
  if (!logits_cur || !active_idx || !m_dev || !masked || !argmax || !write_id) return SL_EINVAL;
  if ((dtype != SL_F32 && dtype != SL_BF16) || vocab < 8 || vocab % 8 || m_upper < 0 || n_seq < 1) return SL_EINVAL;
  if (block_lo < 0 || block_hi > n_seq || block_lo > block_hi || !(temperature > 0.f) || t < 1) return SL_EINVAL;
  if (m_upper > slk_sample_static_rows()) return SL_ENOSPC;       // beyond the static buffer: use sl_sample_tokens
  void* parts = nullptr;
  SL_TRY(slk_sample_static_ptr(&parts));
  return slk_sample_tokens((hipStream_t)stream, logits_cur, cur_packed, dtype, vocab, active_idx, m_dev, m_upper, masked,
                           n_seq, block_lo, block_hi, temperature, seed, t, argmax, write_id, parts);
}

extern "C" int sl_select_rows(void* stream, const uint8_t* lock, const uint8_t* masked, const float* d_last,
                             int32_t batch, int32_t n_seq, int32_t block_lo, int32_t block_hi, float select_fraction,
                             uint8_t* compute_mask) {
  if (!lock || !masked || !d_last || !compute_mask || batch < 1 || n_seq < 1) return SL_EINVAL;
  if (block_lo < 0 || block_hi > n_seq || block_lo > block_hi) return SL_EINVAL;
  if (!(select_fraction > 0.f) || select_fraction > 1.f || compute_mask == lock) return SL_EINVAL;
  return slk_select_rows((hipStream_t)stream, lock, masked, d_last, batch, n_seq, block_lo, block_hi, select_fraction,
                         compute_mask);
}

extern "C" int sl_lock_rule_relock(void* stream, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                                   const int32_t* cu_active, int32_t m_upper, const float* kl, const float* conf,
                                   const float* eps, float gate_percentile, const uint8_t* relocked,
                                   const int32_t* cool_until, float rho, int32_t t, int32_t batch, int32_t n_seq,
                                   uint8_t* new_lock, int32_t* t_lock) {
  if (!lock || !masked || !active_idx || !cu_active || !kl || !conf || !eps || !new_lock) return SL_EINVAL;
  if (!relocked || !cool_until || !t_lock) return SL_EINVAL;
  if (batch < 1 || n_seq < 1 || m_upper < 0 || t < 1) return SL_EINVAL;
  if (gate_percentile > 100.f || !(rho > 0.f) || rho > 1.f) return SL_EINVAL;
  return slk_lock_rule_relock((hipStream_t)stream, lock, masked, active_idx, cu_active, m_upper, kl, conf, eps,
                              gate_percentile, relocked, cool_until, rho, t, batch, n_seq, new_lock, t_lock);
}

extern "C" int sl_lock_test(void* stream, const void* logits_cur, int32_t cur_packed, const void* logits_prev,
                            int32_t dtype, int32_t vocab, int32_t* tokens, uint8_t* masked, const uint8_t* lock,
                            const int32_t* active_idx, const int32_t* cu_active, int32_t m_upper, const float* eps,
                            int32_t batch, int32_t n_seq, int32_t first_step, int32_t block_lo, int32_t block_hi,
                            int32_t k, float* kl, float* conf, int32_t* argmax, uint8_t* new_lock) {
  if (!cu_active || batch < 1) return SL_EINVAL;
  if (!tokens || !masked || !lock || !eps || !new_lock) return SL_EINVAL;
  if (n_seq < 1 || block_lo < 0 || block_hi > n_seq || block_lo > block_hi || k < 0) return SL_EINVAL;
  const int32_t* m_dev = cu_active + batch;
  SL_TRY(sl_score_posteriors(stream, logits_cur, cur_packed, logits_prev, dtype, vocab, active_idx, m_dev, m_upper,
                             first_step, kl, conf, argmax));
  SL_TRY(sl_unmask_topk(stream, tokens, masked, active_idx, cu_active, conf, argmax, batch, n_seq, block_lo, block_hi,
                        k));
  return sl_lock_rule(stream, lock, masked, active_idx, m_dev, m_upper, kl, eps, batch, n_seq, first_step, new_lock);
}

// ---- standalone projection ---------------------------------------------------------------------------
extern "C" int sl_linear_pack(void* stream, const void* w, int32_t n, int32_t k, void* packed, size_t packed_bytes) {
  if (!w || !packed || n < 32 || k < 64 || n % 32 || k % 64) return SL_EINVAL;
  if ((uintptr_t)w % 16 || (uintptr_t)packed % 16) return SL_EINVAL;
  if (packed_bytes < (size_t)n * k * 2) return SL_ENOSPC;
  return slk_pack_weight((hipStream_t)stream, w, n, k, packed, 0, 1);
}

extern "C" int sl_linear_splits(int32_t m_upper, int32_t n, int32_t k) {
  if (m_upper < 1 || n < 32 || k < 64 || n % 32 || k % 64) return SL_EINVAL;
  return slk_gemm_splits(m_upper, n, k);
}

extern "C" int sl_linear_plan(int32_t m_upper, int32_t n, int32_t k, int32_t* kernel, int32_t* splits, int32_t* tile_rows,
                              int32_t* tile_cols, int32_t* tail_tile) {
  if (m_upper < 1 || n < 32 || k < 64 || n % 32 || k % 64) return SL_EINVAL;
  if (!kernel || !splits || !tile_rows || !tile_cols || !tail_tile) return SL_EINVAL;
  return slk_gemm_describe(m_upper, n, k, kernel, splits, tile_rows, tile_cols, tail_tile);
}

extern "C" int sl_linear_forward(void* stream, const void* x, int32_t x_tiled, const void* packed, const int32_t* m_dev,
                                 int32_t m_upper, int32_t n, int32_t k, int32_t splits, float* y_f32, void* y_bf16,
                                 const int32_t* row_map) {
  if (!x || !packed || !m_dev || m_upper < 0 || n < 32 || k < 64 || n % 32 || k % 64) return SL_EINVAL;
  if ((y_f32 == nullptr) == (y_bf16 == nullptr)) return SL_EINVAL;
  if ((uintptr_t)x % 16 || (uintptr_t)packed % 16 || (uintptr_t)y_bf16 % 16) return SL_EINVAL;
  if (splits == 0) splits = y_f32 ? slk_gemm_splits(m_upper, n, k) : 1;
  if (splits < 1 || k % (64 * splits) || (y_bf16 && splits != 1)) return SL_EINVAL;
  return slk_gemm_mfma((hipStream_t)stream, x, x_tiled ? 1 : 0, packed, m_dev, m_upper, n, k, splits, y_f32, y_bf16, row_map, n);
}

extern "C" int sl_linear_clock_probe(void* stream, const void* x, int32_t x_tiled, const void* packed, const int32_t* m_dev,
                                     int32_t m_upper, int32_t n, int32_t k, void* y_bf16, const int32_t* row_map,
                                     int64_t* counters) {
  if (!x || !packed || !m_dev || !y_bf16 || !counters || m_upper < 65 || n < 32 || k < 256 || n % 32 || k % 64) return SL_EINVAL;
  if ((uintptr_t)x % 16 || (uintptr_t)packed % 16 || (uintptr_t)y_bf16 % 16 || (uintptr_t)counters % 8) return SL_EINVAL;
  return slk_gemm_mfma256_probe((hipStream_t)stream, x, x_tiled ? 1 : 0, packed, m_dev, m_upper, n, k, y_bf16, row_map, n,
                                (long long*)counters);
}

// ---- the step --------------------------------------------------------------------------------------
// compute_mask / d_last: null for the plain step; otherwise the step computes only the rows the selection
// keeps (Exp-5, combined setting) and maintains d_last and the posterior buffers for the skipped ones.
static int step_impl(sl_ctx* ctx, void* stream, int32_t* tokens, uint8_t* masked, const uint8_t* lock,
                     const float* eps, int32_t t, int32_t block_lo, int32_t block_hi, int32_t k,
                     int32_t m_upper, int32_t* active_idx, int32_t* cu_active, float* kl, float* conf,
                     int32_t* argmax, uint8_t* new_lock, void* workspace, size_t workspace_bytes,
                     float select_fraction, float* d_last, uint8_t* compute_mask) {
  SL_TRY(check_ready(ctx, true));
  if (!tokens || !masked || !lock || !eps || !active_idx || !cu_active || !kl || !conf || !argmax || !new_lock ||
      !workspace)
    return SL_EINVAL;
  const int B = ctx->batch, N = ctx->n_seq;
  if (t < 1 || m_upper < 1 || m_upper > B * N) return SL_EINVAL;
  if (block_lo < 0 || block_hi > N || block_lo > block_hi || k < 0) return SL_EINVAL;
  if ((size_t)(block_hi - block_lo) * 8 > 60 * 1024) return SL_EINVAL;
  if ((uintptr_t)workspace % 256) return SL_EINVAL;
  const Workspace ws = carve(ctx, workspace, m_upper, ctx->batch, ctx->n_seq);
  if (workspace_bytes < ws.bytes) return SL_ENOSPC;
  hipStream_t s = (hipStream_t)stream;
  const sl_config& c = ctx->cfg;
  const int32_t* m_dev = cu_active + B;
  // A_t (with selection: the rows of A_t the selection keeps; from step 2 on, once scores exist)
  const uint8_t* rows_mask = lock;
  if (compute_mask != nullptr) {
    SL_RUN(ctx, s, SL_PROF_COMPACT, slk_select_rows(s, lock, masked, d_last, B, N, block_lo, block_hi,
                                                    t == 1 ? 1.0f : select_fraction, compute_mask));
    const size_t ts = sl_tsize(c.dtype);
    SL_RUN(ctx, s, SL_PROF_COMPACT, slk_posterior_carry_skipped(s, ctx->post, ctx->post_buf_elems * ts,
                                                                (size_t)c.vocab * ts, lock, compute_mask, B * N, t));
    rows_mask = compute_mask;
  }
  SL_RUN(ctx, s, SL_PROF_COMPACT, slk_compact_active(s, rows_mask, B, N, m_upper, active_idx, cu_active));
  // block input of the active rows + first LN
  SL_RUN(ctx, s, SL_PROF_EMBED_NORM, slk_embed_rmsnorm(s, c.dtype, ctx->plain.emb, tokens, active_idx, m_dev, m_upper, c.d_model, c.vocab,
                           ctx->layers[0].attn_norm, c.rms_eps, ws.x, ws.h, ctx->use_mfma));
  SL_TRY(run_layers(ctx, s, ws, active_idx, m_dev, m_upper, 0, c.n_layers));
  // logits of the active rows, written to their rows of this step's posterior buffer
  void *cur = nullptr, *prev = nullptr;
  sl_logits_ptr(ctx, t, &cur);
  sl_logits_ptr(ctx, t - 1, &prev);
  if (ctx->use_mfma)
    SL_RUN(ctx, s, SL_PROF_LM_HEAD, sl_mfma_lm_head(ctx, s, ws.h, active_idx, m_dev, m_upper, cur));
  else
    SL_RUN(ctx, s, SL_PROF_LM_HEAD, slk_gemm_generic(s, c.dtype, ws.h, ctx->plain.lm_head, m_dev, m_upper, c.vocab, c.d_model, nullptr, cur,
                            active_idx, c.vocab));
  // score -> UpdateMASK -> candidates -> lock
  SL_RUN(ctx, s, SL_PROF_SCORE, slk_score(s, cur, 0, prev, c.dtype, c.vocab, active_idx, m_dev, m_upper, t == 1, kl, conf, argmax, ws.score));
  if (d_last != nullptr) SL_RUN(ctx, s, SL_PROF_SCORE, slk_scatter_rows_f32(s, active_idx, m_dev, m_upper, kl, d_last));
  // (with candidates_pre_update the lock rule simply runs first: it then sees `masked` as it
  // was before UpdateMASK, and neither kernel reads what the other writes)
  auto lock_rule = [&]() -> int {
    // the rule kernels write the locked positions and the computed rows; skipped rows (selection) are
    // neither, so a separate output starts as a copy of the input mask
    if (compute_mask != nullptr && new_lock != lock)
      SL_HIP(hipMemcpyAsync(new_lock, lock, (size_t)B * N, hipMemcpyDeviceToDevice, s));
    if (c.gate_percentile > 0.f)
      return slk_lock_rule_gated(s, lock, masked, active_idx, cu_active, m_upper, kl, conf, eps, c.gate_percentile, B, N,
                                 t == 1, new_lock);
    return slk_lock_rule(s, lock, masked, active_idx, m_dev, m_upper, kl, eps, B, N, t == 1, new_lock);
  };
  if (c.candidates_pre_update) SL_RUN(ctx, s, SL_PROF_LOCK_RULE, lock_rule());
  const int32_t* write_id = argmax;
  if (c.temperature > 0.f) {
    // the tokens UpdateMASK may write are drawn from softmax(z / temperature); ranking stays on conf
    // the query buffer is free once the layers are done: [m_upper] drawn ids, then the per-part candidates
    int32_t* drawn = (int32_t*)ws.q;
    void* parts = ws.q + sl_align_up((size_t)m_upper * sizeof(int32_t), 256);
    SL_RUN(ctx, s, SL_PROF_UNMASK, slk_sample_tokens(s, cur, 0, c.dtype, c.vocab, active_idx, m_dev, m_upper, masked, N,
                                                     block_lo, block_hi, c.temperature, c.seed, t, argmax, drawn, parts));
    write_id = drawn;
  }
  // the plain rule in Alg. 1's order shares UpdateMASK's launch (one workgroup per sequence does both)
  if (!c.candidates_pre_update && !(c.gate_percentile > 0.f) && compute_mask == nullptr && block_hi > block_lo && k > 0) {
    SL_RUN(ctx, s, SL_PROF_UNMASK, slk_unmask_lock(s, tokens, masked, active_idx, cu_active, conf, write_id, B, N, block_lo,
                                                   block_hi, k, m_upper, lock, kl, eps, t == 1, new_lock));
    return SL_OK;
  }
  SL_RUN(ctx, s, SL_PROF_UNMASK, slk_unmask_topk(s, tokens, masked, active_idx, cu_active, conf, write_id, B, N, block_lo, block_hi, k, m_upper));
  if (!c.candidates_pre_update) SL_RUN(ctx, s, SL_PROF_LOCK_RULE, lock_rule());
  return SL_OK;
}

extern "C" int sl_surelock_step(sl_ctx* ctx, void* stream, int32_t* tokens, uint8_t* masked, const uint8_t* lock,
                                const float* eps, int32_t t, int32_t block_lo, int32_t block_hi, int32_t k,
                                int32_t m_upper, int32_t* active_idx, int32_t* cu_active, float* kl, float* conf,
                                int32_t* argmax, uint8_t* new_lock, void* workspace, size_t workspace_bytes) {
  return step_impl(ctx, stream, tokens, masked, lock, eps, t, block_lo, block_hi, k, m_upper, active_idx, cu_active, kl,
                   conf, argmax, new_lock, workspace, workspace_bytes, 1.0f, nullptr, nullptr);
}

extern "C" int sl_surelock_step_selected(sl_ctx* ctx, void* stream, int32_t* tokens, uint8_t* masked,
                                         const uint8_t* lock, const float* eps, int32_t t, int32_t block_lo,
                                         int32_t block_hi, int32_t k, float select_fraction, float* d_last,
                                         uint8_t* compute_mask, int32_t m_upper, int32_t* active_idx,
                                         int32_t* cu_active, float* kl, float* conf, int32_t* argmax,
                                         uint8_t* new_lock, void* workspace, size_t workspace_bytes) {
  if (!d_last || !compute_mask || !(select_fraction > 0.f) || select_fraction > 1.f) return SL_EINVAL;
  if (compute_mask == lock || compute_mask == new_lock) return SL_EINVAL;
  if (ctx && ctx->kv && (size_t)ctx->n_seq * 8 > 60 * 1024) return SL_EINVAL;
  return step_impl(ctx, stream, tokens, masked, lock, eps, t, block_lo, block_hi, k, m_upper, active_idx, cu_active, kl,
                   conf, argmax, new_lock, workspace, workspace_bytes, select_fraction, d_last, compute_mask);
}

// ---- optional unlocking ------------------------------------------------------------------------------
extern "C" int sl_unlock_probe(sl_ctx* ctx, void* stream, const int32_t* tokens, const uint8_t* lock,
                               const int32_t* t_lock, int32_t m_upper, int32_t* probe_idx, int32_t* cu_probe,
                               void* probe_logits, float* kl, float* conf, int32_t* argmax, void* workspace,
                               size_t workspace_bytes) {
  SL_TRY(check_ready(ctx, true));
  if (!tokens || !lock || !t_lock || !probe_idx || !cu_probe || !probe_logits || !kl || !conf || !argmax || !workspace)
    return SL_EINVAL;
  const int B = ctx->batch, N = ctx->n_seq;
  if (m_upper < 1 || m_upper > B * N) return SL_EINVAL;
  if ((uintptr_t)workspace % 256 || (uintptr_t)probe_logits % 16) return SL_EINVAL;
  const Workspace ws = carve(ctx, workspace, m_upper, B, N);
  if (workspace_bytes < ws.bytes) return SL_ENOSPC;
  hipStream_t s = (hipStream_t)stream;
  const sl_config& c = ctx->cfg;
  const int32_t* m_dev = cu_probe + B;
  // L_t, the rows the probe visits
  SL_TRY(slk_compact_active(s, lock, B, N, m_upper, probe_idx, cu_probe, 1));
  SL_TRY(slk_embed_rmsnorm(s, c.dtype, ctx->plain.emb, tokens, probe_idx, m_dev, m_upper, c.d_model, c.vocab,
                           ctx->layers[0].attn_norm, c.rms_eps, ws.x, ws.h, ctx->use_mfma));
  // queries only: keys and values of every slot come from the cache, nothing is written
  ctx->probe_read_only = true;
  const int rc = run_layers(ctx, s, ws, probe_idx, m_dev, m_upper, 0, c.n_layers);
  ctx->probe_read_only = false;
  SL_TRY(rc);
  // proxy logits, packed in probe order
  if (ctx->use_mfma)
    SL_TRY(sl_mfma_lm_head(ctx, s, ws.h, nullptr, m_dev, m_upper, probe_logits));
  else
    SL_TRY(slk_gemm_generic(s, c.dtype, ws.h, ctx->plain.lm_head, m_dev, m_upper, c.vocab, c.d_model, nullptr,
                            probe_logits, nullptr, c.vocab));
  // u~ (as conf) and D~ = KL(p^_t || p_{t*}): the kept row of a position locked at t* lies in buffer t* & 1
  int32_t* prev_rows = (int32_t*)ws.q;                   // the query buffer is free again
  SL_TRY(slk_probe_prev_rows(s, probe_idx, m_dev, m_upper, t_lock, (int)(ctx->post_buf_elems / c.vocab), prev_rows));
  return slk_score(s, probe_logits, 1, ctx->post, c.dtype, c.vocab, prev_rows, m_dev, m_upper, 0, kl, conf, argmax,
                   ws.score);
}

extern "C" int sl_unlock_rule(sl_ctx* ctx, void* stream, uint8_t* lock, uint8_t* relocked, int32_t* cool_until,
                              const int32_t* t_lock, const int32_t* probe_idx, const int32_t* cu_probe,
                              int32_t m_upper_probe, const float* kl_probe, const float* conf_probe,
                              const int32_t* cu_active, int32_t m_upper_active, const float* conf_active,
                              float percentile, float eps_unlock, int32_t t, int32_t d_interval, int32_t d_cool,
                              uint8_t* unlocked) {
  SL_TRY(check_ready(ctx, true));
  if (!lock || !relocked || !cool_until || !t_lock || !probe_idx || !cu_probe || !kl_probe || !conf_probe ||
      !cu_active || !conf_active || !unlocked)
    return SL_EINVAL;
  const int B = ctx->batch, N = ctx->n_seq;
  if (m_upper_probe < 1 || m_upper_probe > B * N || m_upper_active < 0 || m_upper_active > B * N) return SL_EINVAL;
  if (!(percentile > 0.f) || percentile > 100.f || t < 1 || d_interval < 0 || d_cool < 0) return SL_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  SL_TRY(slk_unlock_rule(s, lock, relocked, cool_until, t_lock, probe_idx, cu_probe, m_upper_probe, kl_probe,
                         conf_probe, cu_active, m_upper_active, conf_active, percentile, eps_unlock, t, d_interval,
                         d_cool, B, N, unlocked));
  const size_t ts = sl_tsize(ctx->cfg.dtype);
  return slk_posterior_carry(s, ctx->post, ctx->post_buf_elems * ts, (size_t)ctx->cfg.vocab * ts, probe_idx,
                             cu_probe + B, m_upper_probe, t_lock, unlocked, t);
}
