/*
 * libsurelock: the per-step hot path of SureLock (Oba et al., "Stopping
 * Computation for Converged Tokens in Masked Diffusion-LM Decoding") as HIP
 * kernels for gfx950 (MI355X), behind a plain C ABI.
 *
 * One diffusion step (Algorithm 1, body of the loop over t) restricted to the
 * M unlocked ("active") positions of B sequences of N slots each:
 *   active-set compaction -> embedding gather -> L x [ RMSNorm, Q/K/V projection,
 *   RoPE, K/V write into the frozen-plus-live cache, bidirectional M x N
 *   attention over all N cached slots, Out projection, SwiGLU FFN ] -> final
 *   RMSNorm + LM head -> posterior scoring (step-wise KL, confidence, argmax)
 *   -> UpdateMASK -> candidates and the lock rule.
 *
 * Conventions for every entry point
 *  - All tensor arguments are DEVICE pointers unless the comment says "host".
 *    The library never allocates or frees device memory: the caller owns every
 *    buffer (weights, caches, workspace, outputs) and passes raw pointers.
 *  - `stream` is a hipStream_t passed as void*; calls only enqueue work on it
 *    and return without synchronising.  Buffers must stay valid until the
 *    stream has drained.
 *  - Return value: 0 (SL_OK) or a negative sl_status.  Arguments are validated
 *    on the host before anything is launched, so SL_EINVAL / SL_ENOSPC never
 *    leave partial work behind.  Nothing throws or aborts.
 *  - Row ids: a position i of sequence b has the flat row id g = b*N + i.
 *    "Packed" arrays have one entry per active row, in the order of active_idx.
 *  - Storage type T is bf16 (SL_BF16) or fp32 (SL_F32); all arithmetic
 *    accumulates in fp32.  Tensors that live in memory between operators are
 *    rounded to T (nearest-even) at: RMSNorm output; q and k after RoPE, v;
 *    attention output; the residual stream after each add; silu(gate)*up; logits.
 */
#ifndef SURELOCK_H
#define SURELOCK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sl_status {
  SL_OK = 0,
  SL_EINVAL = -1,   /* null pointer, bad shape, bad dtype, misaligned pointer      */
  SL_ENOSPC = -2,   /* a caller-provided buffer (workspace, cache, store) too small */
  SL_EHIP = -3,     /* a HIP call failed; see sl_last_hip_error()                   */
  SL_ESTATE = -4    /* call order violated (e.g. step before the cache is bound)    */
} sl_status;

enum { SL_F32 = 0, SL_BF16 = 1 };

/* Largest batch (sequences stepped together): the attention kernels keep the row range of every sequence in
 * LDS.  sl_kv_cache_bytes / sl_kv_cache_bind and the stand-alone calls that take a batch return SL_EINVAL
 * beyond it. */
enum { SL_MAX_BATCH = 255 };

/* Model shape.  The block is the pre-RMSNorm / RoPE / SwiGLU block with multi-head
 * attention (H_kv = H), the one whose GEMMs the paper's algorithmic-FLOP count
 * lists (Sec. 2.4): Q, K, V, Out projections and a three-matrix FFN. */
typedef struct sl_config {
  int32_t n_layers, d_model, n_heads, d_head, d_ff, vocab;
  int32_t dtype;        /* SL_F32 or SL_BF16: storage type T of weights and activations */
  int32_t mask_id;      /* token id of [MASK] (only used for validation)                */
  float rms_eps;
  float rope_theta;
  int32_t candidates_pre_update; /* 0: Alg. 1 as printed, UpdateMASK precedes the candidate line, so a
                                  * position unmasked at step t may lock at step t; 1: candidates
                                  * are taken from the unmasked set as it was BEFORE UpdateMASK    */
  float gate_percentile;         /* 0: the optional confidence gate of the lock rule is off (the
                                  * step then uses sl_lock_rule); m in (0, 100]: the step uses
                                  * sl_lock_rule_gated with this m (Sec. 2.2)                      */
  float temperature;             /* 0: UpdateMASK writes the argmax (the paper's setting); tau > 0: it
                                  * writes a token drawn from softmax(z / tau), see sl_sample_tokens.
                                  * Scores and the lock test always use the raw posterior.          */
  uint64_t seed;                 /* key of the draws (temperature > 0)                              */
} sl_config;

/* Plain weights, caller-owned device memory of type T, `[out_features, in_features]`
 * row-major (y = x W^T).  Norm gains are vectors of d_model. */
typedef struct sl_layer_weights {
  const void *attn_norm;            /* [d]        */
  const void *wq, *wk, *wv;         /* [H*d_h, d] */
  const void *wo;                   /* [d, H*d_h] */
  const void *ffn_norm;             /* [d]        */
  const void *w_gate, *w_up;        /* [d_ff, d]  */
  const void *w_down;               /* [d, d_ff]  */
} sl_layer_weights;

typedef struct sl_weights {
  const void *emb;                  /* [vocab, d] */
  const void *final_norm;           /* [d]        */
  const void *lm_head;              /* [vocab, d] */
  const sl_layer_weights *layers;   /* HOST array of n_layers entries */
} sl_weights;

typedef struct sl_ctx sl_ctx;       /* host-side descriptors only */

/* ---- lifetime ------------------------------------------------------------------ */

/* Create a context for one model shape.  Allocates host memory only. */
int sl_init(const sl_config *cfg, sl_ctx **out);
int sl_destroy(sl_ctx *ctx);
const char *sl_strerror(int status);
/* hipError_t value of the most recent failed HIP call on this thread (0 if none). */
int sl_last_hip_error(void);

/* Size of, and conversion into, the library's private weight layout.  For bf16
 * models whose dimensions are multiples of the MFMA tile the projection matrices
 * are re-tiled so that each wavefront's MFMA operand fragment is one contiguous,
 * fully coalesced 1 KiB read (Q/K/V fused into one matrix, gate/up fused into
 * one); other models reference the plain matrices and need 0 extra bytes.  The
 * plain weights (at least emb and the norm gains) must outlive the context.
 * Enqueues the re-tiling kernels on `stream`. */
int sl_packed_weights_bytes(const sl_ctx *ctx, size_t *out);
int sl_bind_weights(sl_ctx *ctx, void *stream, const sl_weights *plain /* host struct */,
                    void *packed, size_t packed_bytes);

/* ---- state: Alg. 1 'State' lines ---------------------------------------------------
 * K/V cache (the caches C for (k, v), all layers): "frozen plus live".  Every active
 * row overwrites its own cache row at every step (the 'assemble' line); a locked row
 * is simply never written again, which is the cache commit of the lock line.
 * Layout (T elements), n_pad = N rounded up to 64:
 *   K: [L][B][H][n_pad/32][d_h/8][32][8]  post-RoPE keys; 32 slots x 8 dims interleaved so a
 *                                         32-key MFMA operand fragment of QK^T is contiguous
 *   V: [L][B][H][n_pad/16][2][d_h][8]     values; the 8 slots {8a+4h+i} of a 16-slot block are
 *                                         stored together at [h][dim][4a+i], the key order in
 *                                         which one lane holds the K Q^T accumulator, so P.V
 *                                         needs no transpose
 * (sl_kv_cache_read returns the plain layout.)
 * On the matrix-core route (bf16, d_h = 128) a V element is the value rounded to bf16, held in the
 * 16 bits of an IEEE half: the attention kernels multiply V by half-precision probabilities and the
 * matrix cores take both operands in one format.  Every bf16 value with 2^-14 <= |v| <= 65504 is held
 * exactly; smaller magnitudes are kept to a multiple of 2^-24; larger ones are stored as +-65504 (never
 * as infinity).  sl_kv_cache_read converts back to bf16.  K elements and everything on the other routes
 * are plain values of type T.
 * sl_kv_cache_bind zero-fills the buffer (enqueued on `stream`). */
int sl_kv_cache_bytes(const sl_ctx *ctx, int32_t batch, int32_t n_seq, size_t *out);
int sl_kv_cache_bind(sl_ctx *ctx, void *stream, void *kv, size_t bytes, int32_t batch, int32_t n_seq);
/* Copy layer `layer`'s K and V out in the plain layout [B, N, H, d_h] (type T). */
int sl_kv_cache_read(const sl_ctx *ctx, void *stream, int32_t layer, void *k_out, void *v_out);

/* Previous posteriors p_{t-1} (Alg. 1 state; Sec. 2.1: a locked row keeps p_{t*}).
 * Stored in factored form as the rows' logits (type T): log p = z - logsumexp(z) is
 * recomputed on the fly by the KL pass, which needs both rows anyway.  Two buffers
 * [2][R][vocab] alternate (R = B*N rounded up so that a buffer is a multiple of 256 bytes;
 * sl_posterior_bytes / 2 apart): step t writes the logits of its active rows into buffer
 * t & 1 (rows by flat id) and reads p_{t-1} from buffer (t-1) & 1. */
int sl_posterior_bytes(const sl_ctx *ctx, int32_t batch, int32_t n_seq, size_t *out);
int sl_posterior_bind(sl_ctx *ctx, void *store, size_t bytes);
/* Device pointer to the [B*N, vocab] logits buffer that step t writes (host out). */
int sl_logits_ptr(const sl_ctx *ctx, int32_t t, void **out);

int sl_workspace_bytes(const sl_ctx *ctx, int32_t batch, int32_t n_seq, size_t *out);

/* ---- the step ---------------------------------------------------------------------
 * One iteration of the loop of Alg. 1 for all B sequences.
 *   tokens  [B*N] i32  in/out  current token ids; UpdateMASK writes argmax ids
 *   masked  [B*N] u8   in/out  1 = still [MASK] (the set M_t); UpdateMASK clears
 *   lock    [B*N] u8   in      lock mask at the start of the step
 *   eps     [B]   f32  in      per-sequence KL threshold (lock iff D <= eps)
 *   t                  host    1-based step index; at t = 1 D = +inf and nothing locks
 *   block_lo/hi, k     host    UpdateMASK unmasks the k most confident still-masked
 *                              positions with block_lo <= i < block_hi in each sequence
 *   m_upper            host    an upper bound on the number of active rows (B*N is
 *                              always valid); launches are sized by it, rows beyond
 *                              the true M exit early.  The bound is the caller's
 *                              promise: if the true count exceeds it, only the first
 *                              m_upper active rows (in active_idx order) are computed,
 *                              scored, unmasked and tested, nothing is written past
 *                              m_upper entries of the packed arrays, and cu_active
 *                              still reports the true counts (cu_active[B] > m_upper
 *                              tells the caller the step was incomplete)
 *   active_idx [>=m_upper] i32 out  flat ids of active rows, ascending
 *   cu_active  [B+1]   i32 out  exclusive prefix sums of per-sequence counts; [B] = M
 *   kl, conf [>=m_upper] f32 out  D_t and max_v p_t per active row (u = 1 - conf)
 *   argmax   [>=m_upper] i32 out  argmax_v p_t (lowest id on ties)
 *   new_lock [B*N] u8  out     lock | F_t   (may alias lock)
 * Logits of the active rows land in the posterior store (sl_logits_ptr(t)). */
int sl_surelock_step(sl_ctx *ctx, void *stream, int32_t *tokens, uint8_t *masked,
                     const uint8_t *lock, const float *eps, int32_t t,
                     int32_t block_lo, int32_t block_hi, int32_t k, int32_t m_upper,
                     int32_t *active_idx, int32_t *cu_active, float *kl, float *conf,
                     int32_t *argmax, uint8_t *new_lock, void *workspace, size_t workspace_bytes);

/* The step combined with selection-based sparsification (Exp-5, the setting that selects a fixed
 * fraction k of the positions not yet locked): from t = 2 on, per sequence only ceil(k n) of the n
 * non-locked positions are computed: the still-masked positions inside [block_lo, block_hi)
 * always, the rest of the budget in decreasing order of d_last, ties to the lower position (the
 * paper's surrogate names no order; this one recomputes what moved most).  A skipped position
 * keeps its K/V, its posterior, its d_last and its lock state; its next KL is taken against the
 * posterior of the step it was last computed at.
 *   select_fraction    host    k, 0 < k <= 1
 *   d_last   [B*N] f32 in/out  the KL each position scored when last computed; the caller fills
 *                              it with +inf before step 1 (every step overwrites the computed rows)
 *   compute_mask [B*N] u8 out  0 = computed at this step, 1 = locked or skipped (must not alias
 *                              lock / new_lock)
 *   m_upper                    bounds the number of COMPUTED rows; n_seq <= 7680
 * active_idx / cu_active / kl / conf / argmax describe the computed rows.  Everything else as
 * sl_surelock_step.  Not meant to be mixed with the unlocking entry points in one run. */
int sl_surelock_step_selected(sl_ctx *ctx, void *stream, int32_t *tokens, uint8_t *masked,
                              const uint8_t *lock, const float *eps, int32_t t,
                              int32_t block_lo, int32_t block_hi, int32_t k, float select_fraction,
                              float *d_last, uint8_t *compute_mask, int32_t m_upper,
                              int32_t *active_idx, int32_t *cu_active, float *kl, float *conf,
                              int32_t *argmax, uint8_t *new_lock, void *workspace, size_t workspace_bytes);

/* The restricted forward alone (Alg. 1, 'Compute on active positions'), layers
 * [layer_lo, layer_hi) on given block inputs: x_in [m_upper, d] (type T, packed in
 * active order) -> x_out [m_upper, d].  Writes the active rows' K/V into the cache.
 * m_dev points to the device int holding the true M (e.g. cu_active + B). */
int sl_forward_layers(sl_ctx *ctx, void *stream, const void *x_in, void *x_out,
                      const int32_t *active_idx, const int32_t *m_dev, int32_t m_upper,
                      int32_t layer_lo, int32_t layer_hi, void *workspace, size_t workspace_bytes);

/* ---- the controller pieces, callable on given logits ---------------------------- */

/* Alg. 1 'A_t <- {i | lock_i = 0}': stable compaction of the unlocked flat ids. */
int sl_compact_active(void *stream, const uint8_t *lock, int32_t batch, int32_t n_seq,
                      int32_t *active_idx, int32_t *cu_active);

/* Alg. 1 'Score on active positions' (+ argmax): for each active row r with flat id
 * g = active_idx[r]:  D = KL(softmax(cur row) || softmax(prev row)) in nats, conf =
 * max softmax(cur row), argmax.  cur row = logits_cur + (cur_packed ? r : g)*vocab,
 * prev row = logits_prev + g*vocab; dtype SL_F32 / SL_BF16; vocab % 8 == 0.
 * first_step != 0: logits_prev is not read and D = +inf. */
int sl_score_posteriors(void *stream, const void *logits_cur, int32_t cur_packed,
                        const void *logits_prev, int32_t dtype, int32_t vocab,
                        const int32_t *active_idx, const int32_t *m_dev, int32_t m_upper,
                        int32_t first_step, float *kl, float *conf, int32_t *argmax);

/* UpdateMASK (confidence-ordered unmasking at temperature 0): per sequence, the k
 * still-masked positions inside [block_lo, block_hi) with the highest conf (ties:
 * lowest position) get tokens[g] = argmax[r], masked[g] = 0. */
int sl_unmask_topk(void *stream, int32_t *tokens, uint8_t *masked, const int32_t *active_idx,
                   const int32_t *cu_active, const float *conf, const int32_t *argmax,
                   int32_t batch, int32_t n_seq, int32_t block_lo, int32_t block_hi, int32_t k);

/* The token UpdateMASK writes at temperature tau > 0 (appendix on sampling temperature): for every
 * active row r whose position is still masked and inside [block_lo, block_hi), write_id[r] = a token
 * drawn from softmax(z_r / tau) in Gumbel-max form, argmax_v (z_v + tau * G_v), G_v = -ln(-ln U_v)
 * (fp32, lowest id on ties); every other row gets write_id[r] = argmax[r].  U_v is word v % 4 of the
 * Philox4x32-10 block with counter (v / 4, flat row id g, t, 0) and key (seed low word, seed high
 * word), mapped to (2 (x >> 9) + 1) / 2^24: the draw depends on (seed, t, g) only, not on the launch.
 * Rows as in sl_score_posteriors (cur_packed, dtype, vocab % 8 == 0); pass write_id as the `argmax`
 * argument of sl_unmask_topk.  The step does both when sl_config.temperature > 0.
 * scratch: 64 * m_upper bytes of device memory, 8-byte aligned (a row is streamed by eight workgroups,
 * each leaves a candidate there). */
int sl_sample_tokens(void *stream, const void *logits_cur, int32_t cur_packed, int32_t dtype, int32_t vocab,
                     const int32_t *active_idx, const int32_t *m_dev, int32_t m_upper,
                     const uint8_t *masked, int32_t n_seq, int32_t block_lo, int32_t block_hi,
                     float temperature, uint64_t seed, int32_t t, const int32_t *argmax, int32_t *write_id,
                     void *scratch, size_t scratch_bytes);

/* sl_sample_tokens for callers that cannot allocate device memory or bring a scratch buffer: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical write_id; the per-part candidates go to a buffer that is part of the
 * library's device code (1 MiB, held by every GPU the library runs on until the process ends) instead
 * of a caller's scratch.  Calls no allocating routine.  m_upper <= 16384, otherwise SL_ENOSPC (nothing
 * is launched).  All calls on one GPU share that buffer: nothing in it has to start at zero (every
 * entry that is read is written earlier in the same call), but two calls whose kernels overlap on
 * one GPU (different streams) race on it; calls on one stream are ordered and safe.  The first call
 * on a device looks the buffer's address up (hipGetSymbolAddress, no allocation) with that device
 * current; SL_EHIP if that fails. */
int sl_sample_tokens_noalloc(void *stream, const void *logits_cur, int32_t cur_packed, int32_t dtype, int32_t vocab,
                             const int32_t *active_idx, const int32_t *m_dev, int32_t m_upper,
                             const uint8_t *masked, int32_t n_seq, int32_t block_lo, int32_t block_hi,
                             float temperature, uint64_t seed, int32_t t, const int32_t *argmax, int32_t *write_id);

/* Candidates Z_t = active and unmasked; F_t = {i in Z_t : D_i <= eps_b}; new_lock =
 * lock | F_t (gate disabled).  first_step != 0 locks nothing. */
int sl_lock_rule(void *stream, const uint8_t *lock, const uint8_t *masked,
                 const int32_t *active_idx, const int32_t *m_dev, int32_t m_upper,
                 const float *kl, const float *eps, int32_t batch, int32_t n_seq,
                 int32_t first_step, uint8_t *new_lock);

/* The lock rule with the optional confidence gate (Alg. 1, the percentile line and the lock
 * line; Sec. 2.2): per sequence, theta = the gate_percentile-th percentile of u = 1 - conf over
 * the candidates Z_t, by nearest rank (the ceil(m n / 100)-th smallest of the n values, at least
 * the first; ties at theta pass); F_t = {i in Z_t : u_i <= theta and D_i <= eps_b}.
 * u is formed in fp32 as max(0, 1 - conf).  gate_percentile in (0, 100].  conf [>= m_upper] and
 * cu_active [batch + 1] as the step or sl_score_posteriors / sl_compact_active produce them;
 * n_seq <= 15360.  new_lock may alias lock. */
int sl_lock_rule_gated(void *stream, const uint8_t *lock, const uint8_t *masked,
                       const int32_t *active_idx, const int32_t *cu_active, int32_t m_upper,
                       const float *kl, const float *conf, const float *eps, float gate_percentile,
                       int32_t batch, int32_t n_seq, int32_t first_step, uint8_t *new_lock);

/* The selection of sl_surelock_step_selected alone: compute_mask[g] = 0 for the ceil(k n) non-locked
 * positions of each sequence that are computed (still-masked ones inside [block_lo, block_hi)
 * always, then by decreasing d_last, ties to the lower position), 1 for locked and skipped ones.
 * 0 < select_fraction <= 1; n_seq <= 7680; compute_mask must not alias lock. */
int sl_select_rows(void *stream, const uint8_t *lock, const uint8_t *masked, const float *d_last,
                   int32_t batch, int32_t n_seq, int32_t block_lo, int32_t block_hi,
                   float select_fraction, uint8_t *compute_mask);

/* ---- optional unlocking (appendix 'Optional Unlocking') --------------------------------------
 * Per-position state, device arrays [B*N] owned by the caller and zero-initialised:
 *   t_lock     i32  the step at which the position locked (t*_i); written by
 *                   sl_lock_rule_relock, read by the probe and the unlock rule
 *   relocked   u8   1 = the position has been unlocked before: it re-locks only on
 *                   D <= rho * eps (product formed in fp32)
 *   cool_until i32  the position cannot lock while t <= cool_until (= unlock step + D_cool)
 * A run with unlocking calls, per step t: sl_surelock_step (its new_lock output pointed at
 * scratch), sl_lock_rule_relock (the rule that counts), and after every P-th step
 * sl_unlock_probe then sl_unlock_rule.  All three leave the K/V cache untouched; an unlocked
 * position is simply active again at step t + 1, whose forward overwrites its K/V rows. */

/* The lock rule with the re-lock state: F_t = {i in Z_t : [u_i <= theta_b] and
 * D_i <= (relocked_i ? rho * eps_b : eps_b) and t > cool_until_i}; new_lock = lock | F_t (may
 * alias lock); t_lock[i] = t for i in F_t.  gate_percentile <= 0 switches the bracketed gate off,
 * otherwise it is sl_lock_rule_gated's.  t = 1 locks nothing.  0 < rho <= 1; n_seq <= 15360. */
int sl_lock_rule_relock(void *stream, const uint8_t *lock, const uint8_t *masked,
                        const int32_t *active_idx, const int32_t *cu_active, int32_t m_upper,
                        const float *kl, const float *conf, const float *eps, float gate_percentile,
                        const uint8_t *relocked, const int32_t *cool_until, float rho, int32_t t,
                        int32_t batch, int32_t n_seq, uint8_t *new_lock, int32_t *t_lock);

/* The budgeted proxy on the locked rows: their current tokens run through all layers and the
 * LM head with queries only (keys and values of every slot, their own included, are read from
 * the cache; nothing is written to it or to the posterior store).  Outputs, packed in the order
 * of probe_idx:
 *   probe_idx [>= m_upper] i32  flat ids of the locked rows, ascending; cu_probe [B+1] their
 *                               per-sequence prefix sums ([B] = count)
 *   probe_logits [m_upper, vocab] T  proxy logits (16-byte aligned, caller's scratch)
 *   conf, argmax                max and argmax of the proxy posterior (u~ = 1 - conf)
 *   kl                          D~ = KL(p^_t || p_{t*}) against the row the store kept from
 *                               step t_lock (buffer t_lock & 1)
 * m_upper bounds the number of locked rows (B*N is always valid); workspace as for the step. */
int sl_unlock_probe(sl_ctx *ctx, void *stream, const int32_t *tokens, const uint8_t *lock,
                    const int32_t *t_lock, int32_t m_upper, int32_t *probe_idx, int32_t *cu_probe,
                    void *probe_logits, float *kl, float *conf, int32_t *argmax,
                    void *workspace, size_t workspace_bytes);

/* The unlock rule (the appendix's displayed condition, a conjunction): per sequence, theta =
 * the percentile-th percentile (nearest rank, as for the gate) of u = max(0, 1 - conf_active)
 * over ALL active rows of step t (cu_active / conf_active as the step left them; no active row:
 * the first test passes); a probed position g unlocks iff
 *   u~ > theta  and  D~ > eps_unlock  and  t - t_lock[g] > d_interval      (all strict).
 * Then lock[g] = 0, relocked[g] = 1, cool_until[g] = t + d_cool, unlocked[r] = 1 (else 0; r the
 * probe row), and if the row's kept posterior lies in the buffer step t + 1 will not read
 * (t_lock and t of different parity) it is copied to the other, so that D_{t+1} is taken
 * against p_{t*}.  lock is updated in place. */
int sl_unlock_rule(sl_ctx *ctx, void *stream, uint8_t *lock, uint8_t *relocked, int32_t *cool_until,
                   const int32_t *t_lock, const int32_t *probe_idx, const int32_t *cu_probe,
                   int32_t m_upper_probe, const float *kl_probe, const float *conf_probe,
                   const int32_t *cu_active, int32_t m_upper_active, const float *conf_active,
                   float percentile, float eps_unlock, int32_t t, int32_t d_interval, int32_t d_cool,
                   uint8_t *unlocked);

/* lock_test(eps): Alg. 1 from 'Unmasking' to 'Lock' on given logits = score ->
 * UpdateMASK -> candidates -> lock rule, in that order. */
int sl_lock_test(void *stream, const void *logits_cur, int32_t cur_packed, const void *logits_prev,
                 int32_t dtype, int32_t vocab, int32_t *tokens, uint8_t *masked, const uint8_t *lock,
                 const int32_t *active_idx, const int32_t *cu_active, int32_t m_upper,
                 const float *eps, int32_t batch, int32_t n_seq, int32_t first_step,
                 int32_t block_lo, int32_t block_hi, int32_t k,
                 float *kl, float *conf, int32_t *argmax, uint8_t *new_lock);

/* ---- the M-row projection alone ---------------------------------------------------------
 * y = x W^T for the packed active rows on the MFMA units (the GEMM terms Q, K, V, Out, FFN
 * of Sec. 2.4), bf16 only; n % 32 == 0, k % 64 == 0.  sl_linear_pack re-tiles W [n, k] into
 * the fragment layout (same byte count).  sl_linear_forward: x [m_upper, k] bf16, row-major
 * (x_tiled = 0) or in the same 32 x 16 fragment tiling as the weights, rows padded to a
 * multiple of 32 (x_tiled = 1: element (r, c) at
 * (((r/32)*(k/16) + c/16)*64 + r%32 + 32*((c%16)/8))*8 + c%8); splits = 0
 * picks the k-split count (query it with sl_linear_splits); exactly one of
 *   y_f32  [splits][m_upper][n] fp32 partial sums (16-byte aligned; caller adds the splits), or
 *   y_bf16 [*, n] bf16 rows (16-byte aligned), row r written to row row_map[r] (row_map may
 *          be null; splits must resolve to 1: pass splits = 1)
 * must be non-null. */
int sl_linear_pack(void *stream, const void *w, int32_t n, int32_t k, void *packed, size_t packed_bytes);
int sl_linear_splits(int32_t m_upper, int32_t n, int32_t k);
/* The launch sl_linear_forward(.., splits = 0, y_f32) makes for a row bound (host outputs; nothing is
 * launched), so that tests can tell which kernel form a shape reaches and check that every form a
 * model shape can reach is covered:
 *   kernel     0 = weight-stream kernel (rows <= 64: no LDS, operands global -> registers),
 *              1 = ring kernel (operands through an LDS ring, one workgroup per CU),
 *              2 = LDS kernel for reductions too short for the ring
 *   splits     k-split count (= sl_linear_splits)
 *   tile_rows  rows per workgroup tile (ring kernel: a multiple of 32 from 64 to 256, fitted to m_upper)
 *   tile_cols  columns per workgroup tile (128 or 256)
 *   tail_tile  1: full-height row tiles plus one half-height tile for the row tail (ring kernel) */
int sl_linear_plan(int32_t m_upper, int32_t n, int32_t k, int32_t *kernel, int32_t *splits, int32_t *tile_rows,
                   int32_t *tile_cols, int32_t *tail_tile);
int sl_linear_forward(void *stream, const void *x, int32_t x_tiled, const void *packed, const int32_t *m_dev,
                      int32_t m_upper, int32_t n, int32_t k, int32_t splits, float *y_f32, void *y_bf16,
                      const int32_t *row_map);

/* Measurement aid for the roofline of the projections (Sec. 2.4 GEMM terms): the same product as
 * sl_linear_forward with a bf16 destination, through the thick-M (256 x 256 tile) kernel only
 * (m_upper >= 65, k >= 256), with one workgroup in the middle of the grid recording into
 * counters[0..7] (device memory, 8 x int64, written when the kernel finishes; zero them first):
 *   [0..2] shader-clock cycles of its prologue (first tiles in flight), k loop, epilogue
 *   [3..5] the same three spans in ticks of the constant 100 MHz counter
 *   [6]    workgroups in the launch                        [7] k-tiles (32 deep) in the loop
 * counters[1] / counters[4] * 100 is the shader clock in MHz that the power management grants
 * under this kernel; 1024 * counters[7] / counters[1] is the matrix pipe's busy fraction in the
 * loop.  y_bf16 receives the ordinary result.  SL_EINVAL for shapes the thick kernel does not take. */
int sl_linear_clock_probe(void *stream, const void *x, int32_t x_tiled, const void *w_packed, const int32_t *m_dev,
                          int32_t m_upper, int32_t n, int32_t k, void *y_bf16, const int32_t *row_map,
                          int64_t *counters);

/* Measurement aids for the rooflines of Sec. 2.4's terms: what the chip sustains on the matrix units
 * and on HBM with nothing else in the way, so that a kernel's rate can be read against the published
 * peak and against the achievable one.
 * sl_peak_probe_mfma: one launch of one workgroup per compute unit with 4 x waves_per_simd waves, each
 *   wave running iters x 16 independent v_mfma_f32_16x16x32_bf16 on register operands.
 *   operands: device, >= 8192 bytes (operand_bytes), 16-byte aligned: eight 64-lane bf16x8 fragments,
 *   any finite values (the clock the power management grants depends on them: use the distribution of
 *   the workload).  iters in [1, 2^24]; waves_per_simd 1 or 2.  sink: device floats, one per launched
 *   thread (sink_bytes >= compute units x waves_per_simd x 1024; 1 MiB covers this chip).
 *   *flops (host) receives the floating-point operations of the launch.
 * sl_peak_probe_stream: one grid-stride pass of 16-byte loads over src[bytes] (device, 16-byte aligned,
 *   bytes a multiple of 16); dst null: read only, the words XOR-folded into sink; dst non-null (same
 *   size, no overlap with src): copied.  sink: device uint32, one per launched thread (sink_bytes >=
 *   compute units x 8192; 2 MiB covers this chip).  HBM bytes moved: bytes (read only), 2 x bytes (copy).
 * Both enqueue on stream and return; the caller times them.  SL_EINVAL for null / misaligned /
 * out-of-range arguments, SL_ENOSPC for an operand or sink buffer that is too small. */
int sl_peak_probe_mfma(void *stream, const void *operands, size_t operand_bytes, int32_t iters, int32_t waves_per_simd,
                       float *sink, size_t sink_bytes, int64_t *flops);
int sl_peak_probe_stream(void *stream, const void *src, void *dst, size_t bytes, uint32_t *sink, size_t sink_bytes);

/* ---- measurement support ------------------------------------------------------------
 * Per-kernel timing of the step's launches with HIP events on the step's own stream.
 * Between sl_profile_begin and sl_profile_end every kernel the library launches for this
 * context is bracketed by an event pair; sl_profile_end synchronises on the last event,
 * adds the elapsed times up per kernel slot and releases the events.  Host arrays:
 * ms[SL_PROF_SLOTS], launches[SL_PROF_SLOTS].  Profiling adds host work per launch, so
 * whole-step latency is measured with profiling off. */
enum {
  SL_PROF_COMPACT = 0, SL_PROF_EMBED_NORM, SL_PROF_GEMM_QKV, SL_PROF_ROPE_KV, SL_PROF_ATTENTION,
  SL_PROF_GEMM_OUT, SL_PROF_ADD_NORM, SL_PROF_GEMM_GATE_UP, SL_PROF_SWIGLU, SL_PROF_GEMM_DOWN,
  SL_PROF_LM_HEAD, SL_PROF_SCORE, SL_PROF_UNMASK, SL_PROF_LOCK_RULE, SL_PROF_SLOTS
};
int sl_profile_begin(sl_ctx *ctx, int32_t max_launches);
int sl_profile_end(sl_ctx *ctx, float *ms /* host */, int32_t *launches /* host */);

#ifdef __cplusplus
}
#endif
#endif /* SURELOCK_H */
