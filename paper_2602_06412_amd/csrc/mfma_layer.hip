// The bf16 / MFMA route through one Transformer block and the LM head: which kernels run,
// in which order, on which buffers.  Host code only.
#include "sl_common.h"

bool sl_mfma_supported(const sl_config* c) {
  const int hd = c->n_heads * c->d_head;
  return c->dtype == SL_BF16 && c->d_head == 128 && c->d_model % 64 == 0 && c->d_ff % 64 == 0 && hd % 64 == 0 &&
         c->vocab % 32 == 0;
}

// Packed buffer: per layer [wqkv | wo | w_gate_up | w_down], then lm_head; each matrix keeps
// its element count (re-tiling is a permutation), sections aligned to 256 bytes.
struct PackedLayout {
  size_t qkv, wo, wgu, wdown, layer_bytes, lm_head, total;
};
static PackedLayout packed_layout(const sl_config* c) {
  const size_t d = c->d_model, hd = (size_t)c->n_heads * c->d_head, dff = c->d_ff, V = c->vocab;
  PackedLayout p;
  size_t off = 0;
  auto take = [&](size_t elems) { const size_t o = off; off += sl_align_up(elems * 2, 256); return o; };
  p.qkv = take(3 * hd * d);
  p.wo = take(d * hd);
  p.wgu = take(2 * dff * d);
  p.wdown = take(d * dff);
  p.layer_bytes = off;
  p.lm_head = p.layer_bytes * c->n_layers;
  p.total = p.lm_head + sl_align_up(V * d * 2, 256);
  return p;
}

size_t sl_mfma_packed_bytes(const sl_config* cfg) { return packed_layout(cfg).total; }

#define SL_TRY(expr) do { const int rc_ = (expr); if (rc_ != SL_OK) return rc_; } while (0)

int sl_mfma_pack_all(sl_ctx* ctx, hipStream_t s, void* packed) {
  const sl_config& c = ctx->cfg;
  const PackedLayout p = packed_layout(&c);
  const int d = c.d_model, hd = c.n_heads * c.d_head, dff = c.d_ff;
  char* base = (char*)packed;
  for (int l = 0; l < c.n_layers; ++l) {
    const sl_layer_weights& L = ctx->layers[l];
    char* lb = base + (size_t)l * p.layer_bytes;
    SL_TRY(slk_pack_weight(s, L.wq, hd, d, lb + p.qkv, 0, 1));
    SL_TRY(slk_pack_weight(s, L.wk, hd, d, lb + p.qkv, hd / 32, 1));
    SL_TRY(slk_pack_weight(s, L.wv, hd, d, lb + p.qkv, 2 * hd / 32, 1));
    SL_TRY(slk_pack_weight(s, L.wo, d, hd, lb + p.wo, 0, 1));
    // gate and up interleaved by 32-column blocks (gate j, up j, gate j+1, ..): the thread that holds
    // gate column c of a row also holds up column c, so SwiGLU can run in the GEMM epilogue
    SL_TRY(slk_pack_weight(s, L.w_gate, dff, d, lb + p.wgu, 0, 2));
    SL_TRY(slk_pack_weight(s, L.w_up, dff, d, lb + p.wgu, 1, 2));
    SL_TRY(slk_pack_weight(s, L.w_down, d, dff, lb + p.wdown, 0, 1));
    ctx->packed[l] = sl_packed_layer{lb + p.qkv, lb + p.wo, lb + p.wgu, lb + p.wdown};
  }
  SL_TRY(slk_pack_weight(s, ctx->plain.lm_head, c.vocab, d, base + p.lm_head, 0, 1));
  ctx->packed_lm_head = base + p.lm_head;
  return SL_OK;
}

// fp32 scratch needed by any launch bounded by at most `rows` rows: the widest
// [splits][mu][n] partial block over the four projections
size_t sl_mfma_f32_elems(const sl_config* c, int rows) {
  const int d = c->d_model, hd = c->n_heads * c->d_head, dff = c->d_ff;
  const int shapes[4][2] = {{3 * hd, d}, {d, hd}, {2 * dff, d}, {d, dff}};
  size_t best = 0;
  for (int mu = 1; mu <= rows; ++mu)
    for (auto& sh : shapes) {
      int S = slk_gemm_splits(mu, sh[0], sh[1]);
      if (sh[0] == 2 * dff) {                        // the gate|up launch follows its own plan
        const int Sg = slk_gemm_splits_gate_up(mu, sh[0], sh[1]);
        S = Sg > S ? Sg : S;
      }
      const size_t e = (size_t)S * mu * sh[0];
      if (e > best) best = e;
    }
  return best;
}

static inline char* kv_k(const sl_ctx* ctx, int l) {
  const sl_config& c = ctx->cfg;
  const size_t tab = sl_align_up((size_t)ctx->n_pad * (c.d_head / 2) * sizeof(float2), 256);
  return (char*)ctx->kv + tab + (size_t)l * ctx->kv_layer_elems * 2;
}
static inline char* kv_v(const sl_ctx* ctx, int l) { return kv_k(ctx, ctx->cfg.n_layers) + (size_t)l * ctx->kv_layer_elems * 2; }

int sl_mfma_layer(sl_ctx* ctx, hipStream_t s, int l, void* x, void* h, void* q, void* o, void* a, float* f32,
                  float* attn_scratch, const int32_t* active_idx, const int32_t* m_dev, int mu, const void* next_gain) {
  const sl_config& c = ctx->cfg;
  const int d = c.d_model, H = c.n_heads, dh = c.d_head, hd = H * dh, dff = c.d_ff;
  const sl_packed_layer& P = ctx->packed[l];
  const sl_layer_weights& L = ctx->layers[l];
  void* kc_w = ctx->probe_read_only ? nullptr : kv_k(ctx, l);      // read-only probe: queries only
  void* vc_w = ctx->probe_read_only ? nullptr : kv_v(ctx, l);
  if (H % 2 == 0 && slk_gemm_unsplit_thick(mu, 3 * hd, d)) {
    // thick launches: Q | K | V projection, RoPE and the scatter into q and the caches in one kernel
    SL_RUN(ctx, s, SL_PROF_GEMM_QKV, slk_gemm_mfma256_qkv_rope(s, h, P.wqkv, m_dev, mu, H, d, active_idx, ctx->n_seq, ctx->n_pad,
                                                             ctx->kv, q, kc_w, vc_w));
  } else {
    // Q | K | V projections in one launch (fp32 partial planes), then RoPE + cache write
    const int S = slk_gemm_splits(mu, 3 * hd, d);
    SL_RUN(ctx, s, SL_PROF_GEMM_QKV, slk_gemm_mfma(s, h, 1, P.wqkv, m_dev, mu, 3 * hd, d, S, f32, nullptr, nullptr, 3 * (size_t)hd));
    SL_RUN(ctx, s, SL_PROF_ROPE_KV, slk_rope_kv_write(s, SL_BF16, f32, S, (size_t)mu * 3 * hd, active_idx, m_dev, mu, H, dh, ctx->n_seq, ctx->n_pad,
                             ctx->kv, q, kc_w, vc_w, 1));
  }
  SL_RUN(ctx, s, SL_PROF_ATTENTION, slk_attention_mfma(s, q, kv_k(ctx, l), kv_v(ctx, l), active_idx, m_dev, mu, ctx->batch, H, ctx->n_seq,
                            ctx->n_pad, o, attn_scratch));
  int S = 1;
  if (slk_gemm_unsplit_thick(mu, d, hd)) {
    // thick launches: the residual add runs in the projection's epilogue, the norm reads the new x
    SL_RUN(ctx, s, SL_PROF_GEMM_OUT, slk_gemm_mfma256_residual(s, o, P.wo, m_dev, mu, d, hd, x));
    SL_RUN(ctx, s, SL_PROF_ADD_NORM, slk_rmsnorm(s, SL_BF16, x, m_dev, mu, d, L.ffn_norm, c.rms_eps, h, 1));
  } else {
    S = slk_gemm_splits(mu, d, hd);
    SL_RUN(ctx, s, SL_PROF_GEMM_OUT, slk_gemm_mfma(s, o, 1, P.wo, m_dev, mu, d, hd, S, f32, nullptr, nullptr, d));
    SL_RUN(ctx, s, SL_PROF_ADD_NORM, slk_add_rmsnorm(s, SL_BF16, x, f32, S, (size_t)mu * d, m_dev, mu, d, L.ffn_norm, c.rms_eps, h, 1));
  }
  if (slk_gemm_unsplit_thick(mu, 2 * dff, d)) {
    SL_RUN(ctx, s, SL_PROF_GEMM_GATE_UP, slk_gemm_mfma256_swiglu(s, h, P.wgu, m_dev, mu, dff, d, a));
  } else if (slk_gemm_stream_swiglu_ok(mu, dff, d)) {
    // thin launches whose gate|up projection runs unsplit: SwiGLU in the weight-stream kernel's epilogue
    SL_RUN(ctx, s, SL_PROF_GEMM_GATE_UP, slk_gemm_stream_swiglu(s, h, P.wgu, m_dev, mu, dff, d, a));
  } else {
    S = slk_gemm_splits_gate_up(mu, 2 * dff, d);
    SL_RUN(ctx, s, SL_PROF_GEMM_GATE_UP, slk_gemm_mfma(s, h, 1, P.wgu, m_dev, mu, 2 * dff, d, S, f32, nullptr, nullptr, 2 * (size_t)dff));
    SL_RUN(ctx, s, SL_PROF_SWIGLU, slk_swiglu(s, SL_BF16, f32, S, (size_t)mu * 2 * dff, m_dev, mu, dff, a, 1, 1));
  }
  if (slk_gemm_unsplit_thick(mu, d, dff)) {
    SL_RUN(ctx, s, SL_PROF_GEMM_DOWN, slk_gemm_mfma256_residual(s, a, P.wdown, m_dev, mu, d, dff, x));
    SL_RUN(ctx, s, SL_PROF_ADD_NORM, slk_rmsnorm(s, SL_BF16, x, m_dev, mu, d, next_gain, c.rms_eps, h, 1));
  } else {
    S = slk_gemm_splits(mu, d, dff);
    SL_RUN(ctx, s, SL_PROF_GEMM_DOWN, slk_gemm_mfma(s, a, 1, P.wdown, m_dev, mu, d, dff, S, f32, nullptr, nullptr, d));
    SL_RUN(ctx, s, SL_PROF_ADD_NORM, slk_add_rmsnorm(s, SL_BF16, x, f32, S, (size_t)mu * d, m_dev, mu, d, next_gain, c.rms_eps, h, 1));
  }
  return SL_OK;
}

int sl_mfma_lm_head(sl_ctx* ctx, hipStream_t s, const void* h, const int32_t* active_idx, const int32_t* m_dev, int mu,
                    void* logits_buf) {
  const sl_config& c = ctx->cfg;
  return slk_gemm_mfma(s, h, 1, ctx->packed_lm_head, m_dev, mu, c.vocab, c.d_model, 1, nullptr, logits_buf, active_idx,
                       c.vocab);
}
