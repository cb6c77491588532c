// Shared host/device declarations of libsurelock (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/surelock.h"

typedef __bf16 bf16_t;

// ---- storage-type traits: load to fp32, round-to-nearest-even store -------------
template <typename T> struct st;
template <> struct st<float> {
  static constexpr int kDtype = SL_F32;
  static constexpr int kVec = 4;                       // elements per 16-byte access
  __device__ static inline float ld(const float* p) { return *p; }
  __device__ static inline void stv(float* p, float v) { *p = v; }
  __device__ static inline float rnd(float v) { return v; }
};
template <> struct st<bf16_t> {
  static constexpr int kDtype = SL_BF16;
  static constexpr int kVec = 8;
  __device__ static inline float ld(const bf16_t* p) { return (float)*p; }
  __device__ static inline void stv(bf16_t* p, float v) { *p = (bf16_t)v; }
  __device__ static inline float rnd(float v) { return (float)(bf16_t)v; }
};

__device__ inline float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// ---- K/V cache addressing (elements of T inside one (sequence, head) slab of n_pad slots) ---
// K: [n_pad/32][d_h/8][32 slots][8]   -> a 32-key x 16-dim MFMA A-operand fragment of QK^T is
//                                       one contiguous 1 KiB block (lane = slot + 32*(chunk&1))
// V: [n_pad/16][2][d_h][8]             -> the 8 slots {8a + 4h + i : a<2, i<4} of a 16-slot block
//                                       sit together at [h][dim][4a + i]: exactly the 8 keys
//                                       one lane of the S^T = K Q^T accumulator holds, so the
//                                       P V product needs no transpose or shuffle
__host__ __device__ inline size_t kc_index(int slot, int dim, int dh) {
  return (((size_t)(slot >> 5) * (dh >> 3) + (dim >> 3)) * 32 + (slot & 31)) * 8 + (dim & 7);
}
__host__ __device__ inline size_t vc_index(int slot, int dim, int dh) {
  return (((size_t)(slot >> 4) * 2 + ((slot >> 2) & 1)) * dh + dim) * 8 + ((slot >> 3) & 1) * 4 + (slot & 3);
}

// V element of the MFMA route.  The attention kernels multiply V by half-precision probabilities (the
// matrix cores take both operands in one format), so on that route the cache holds each V value, rounded
// to bf16 like every stored activation, in an IEEE half container: exact for 2^-14 <= |v| <= 65504
// (a bf16 value has 8 significant bits, a half 11), kept to a multiple of 2^-24 below that, saturated
// above (an infinity would turn a zero probability into NaN).  These helpers carry the 16 bits in a
// bf16_t, which is what the cache pointers are typed as.
typedef _Float16 f16_t;
__device__ inline bf16_t vcache_half_bits(float v) {
  const float r = (float)(bf16_t)v;
  const float c = r != r ? r : fminf(fmaxf(r, -65504.f), 65504.f);
  return __builtin_bit_cast(bf16_t, (f16_t)c);
}
__device__ inline bf16_t vcache_half_value(bf16_t bits) { return (bf16_t)(float)__builtin_bit_cast(f16_t, bits); }
template <bool VH>
__device__ inline bf16_t vcache_elem(float v) { return VH ? vcache_half_bits(v) : (bf16_t)v; }

// ---- activation matrices feeding the MFMA GEMMs ------------------------------------------
// "Tiled" layout of an [rows, K] bf16 matrix: MFMA A-operand fragments [rows/32][K/16][64][8],
// lane = row%32 + 32*((col%16)/8).  A GEMM workgroup then fetches each 32 x 16 fragment as one
// contiguous 1 KiB block instead of gathering 32 B from 32 different rows.  Rows are padded
// to a multiple of 32 by the allocation.
__host__ __device__ inline size_t afrag_index(int row, int col, int K) {
  return (((size_t)(row >> 5) * (K >> 4) + (col >> 4)) * 64 + (row & 31) + 32 * ((col >> 3) & 1)) * 8 + (col & 7);
}
template <bool TILED>
__host__ __device__ inline size_t act_index(int row, int col, int K) {
  return TILED ? afrag_index(row, col, K) : (size_t)row * K + col;
}

// ---- wave / block reductions (wave = 64 lanes) ------------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over a block of NT threads; every thread gets the result.  `sh` has NT/64 floats.
template <int NT>
__device__ inline float block_sum(float v, float* sh) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  __syncthreads();
  if (l == 0) sh[w] = v;
  __syncthreads();
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) r += sh[i];
  return r;
}
template <int NT>
__device__ inline float block_max(float v, float* sh) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  __syncthreads();
  if (l == 0) sh[w] = v;
  __syncthreads();
  float r = sh[0];
#pragma unroll
  for (int i = 1; i < NT / 64; ++i) r = fmaxf(r, sh[i]);
  return r;
}

// ---- 8- and 16-byte accesses of the row-wise code (bf16 rows, fp32 partial planes) --------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
__device__ inline void ld8(const bf16_t* p, float (&v)[8]) {
  const bf16x8_t u = *reinterpret_cast<const bf16x8_t*>(p);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)u[e];
}
__device__ inline void st8(bf16_t* p, const float (&v)[8]) {
  bf16x8_t u;
#pragma unroll
  for (int e = 0; e < 8; ++e) u[e] = (bf16_t)v[e];
  *reinterpret_cast<bf16x8_t*>(p) = u;
}
__device__ inline void ld8f(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ inline void st4(bf16_t* p, const float (&v)[4]) {
  bf16x4_t u;
#pragma unroll
  for (int e = 0; e < 4; ++e) u[e] = (bf16_t)v[e];
  *reinterpret_cast<bf16x4_t*>(p) = u;
}
__device__ inline void ld4f(const float* p, float (&v)[4]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
}

// ---- host side -------------------------------------------------------------------------
extern thread_local int g_sl_last_hip_error;
#define SL_HIP(call)                                   \
  do {                                                 \
    hipError_t e_ = (call);                            \
    if (e_ != hipSuccess) {                            \
      g_sl_last_hip_error = (int)e_;                   \
      return SL_EHIP;                                  \
    }                                                  \
  } while (0)
#define SL_LAUNCH_CHECK() SL_HIP(hipGetLastError())
// Raise a kernel's dynamic-LDS limit the first time it is launched on a device (the attribute is
// per device and function; `done` is a launcher-owned bit mask over device ids; two first calls
// racing only repeat an idempotent call).  Kept out of the steady-state launch path.
#define SL_ALLOW_DYNAMIC_LDS(done, kern, bytes)                                                          \
  do {                                                                                                   \
    int dev_ = 0;                                                                                        \
    SL_HIP(hipGetDevice(&dev_));                                                                         \
    if (dev_ >= 64 || !(((done) >> dev_) & 1ull)) {                                                      \
      SL_HIP(hipFuncSetAttribute((const void*)(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes))); \
      if (dev_ < 64) (done) |= 1ull << dev_;                                                             \
    }                                                                                                    \
  } while (0)
#define SL_REQUIRE(cond) do { if (!(cond)) return SL_EINVAL; } while (0)

static inline size_t sl_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int sl_cdiv(int a, int b) { return (a + b - 1) / b; }
static inline size_t sl_tsize(int dtype) { return dtype == SL_BF16 ? 2 : 4; }

struct sl_packed_layer {            // device pointers into the caller's packed buffer (MFMA path)
  const void *wqkv, *wo, *wgu, *wdown;
};

struct sl_prof {                    // event pairs recorded while profiling is on
  hipEvent_t* ev;                   // 2 * cap events
  int* slot;
  int cap, n;
};

struct sl_ctx {
  sl_config cfg;
  sl_prof* prof;
  bool weights_bound, use_mfma;
  sl_weights plain;                 // copy of the caller's struct (layers -> own host array)
  sl_layer_weights* layers;         // host array, n_layers
  sl_packed_layer* packed;          // host array, n_layers (use_mfma only)
  const void* packed_lm_head;
  // K/V cache
  void* kv; int32_t batch, n_seq, n_pad; size_t kv_layer_elems;   // elements of T per layer per K (= per V)
  // posterior store
  void* post; size_t post_buf_elems;
  // true while the read-only unlock probe runs: the forward stores queries only, no K/V
  bool probe_read_only;
  // fp32 partial-plane elements the launch plans need for any launch of at most f32_plan_rows rows
  // (evaluating the plans for every row count is host work that must stay off the per-step path)
  mutable int f32_plan_rows;
  mutable size_t f32_plan_elems;
};

// Run one launcher call, bracketed by an event pair when profiling is on.
#define SL_RUN(ctx, stream, slot_id, call)                                                   \
  do {                                                                                       \
    sl_prof* pf_ = (ctx)->prof;                                                              \
    const bool on_ = pf_ && pf_->n < pf_->cap;                                               \
    if (on_) SL_HIP(hipEventRecord(pf_->ev[2 * pf_->n], (stream)));                          \
    const int rc_ = (call);                                                                  \
    if (rc_ != SL_OK) return rc_;                                                            \
    if (on_) {                                                                               \
      SL_HIP(hipEventRecord(pf_->ev[2 * pf_->n + 1], (stream)));                             \
      pf_->slot[pf_->n++] = (slot_id);                                                       \
    }                                                                                        \
  } while (0)

// ---- kernel launchers (one translation unit each) ------------------------------------------
// control_kernels.hip
int slk_lock_rule_gated(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                        const int32_t* cu_active, int m_upper, const float* kl, const float* conf, const float* eps,
                        float gate_m, int B, int N, int first_step, uint8_t* new_lock);
int slk_compact_active(hipStream_t s, const uint8_t* lock, int B, int N, int cap, int32_t* active_idx,
                       int32_t* cu_active, int select_locked = 0);
int slk_lock_rule_relock(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                         const int32_t* cu_active, int m_upper, const float* kl, const float* conf, const float* eps,
                         float gate_m, const uint8_t* relocked, const int32_t* cool_until, float rho, int t, int B,
                         int N, uint8_t* new_lock, int32_t* t_lock);
int slk_unlock_rule(hipStream_t s, uint8_t* lock, uint8_t* relocked, int32_t* cool_until, const int32_t* t_lock,
                    const int32_t* probe_idx, const int32_t* cu_probe, int mp_upper, const float* kl_probe,
                    const float* conf_probe, const int32_t* cu_active, int ma_upper, const float* conf_active, float m,
                    float eps_unlock, int t, int d_interval, int d_cool, int B, int N, uint8_t* unlocked);
int slk_sample_tokens(hipStream_t s, const void* logits, int cur_packed, int dtype, int V, const int32_t* active_idx,
                      const int32_t* m_dev, int m_upper, const uint8_t* masked, int N, int lo, int hi, float tau,
                      unsigned long long seed, int t, const int32_t* argmax, int32_t* write_id, void* scratch);
size_t slk_sample_scratch_bytes(int m_upper);
int slk_sample_static_rows();
int slk_sample_static_ptr(void** out);
int slk_select_rows(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const float* d_last, int B, int N,
                    int lo, int hi, float k_frac, uint8_t* compute_mask);
int slk_posterior_carry_skipped(hipStream_t s, void* store, size_t buf_bytes, size_t row_bytes, const uint8_t* lock,
                                const uint8_t* compute_mask, int total, int t);
int slk_scatter_rows_f32(hipStream_t s, const int32_t* active_idx, const int32_t* m_dev, int m_upper, const float* src,
                         float* dst);
int slk_probe_prev_rows(hipStream_t s, const int32_t* probe_idx, const int32_t* m_dev, int m_upper,
                        const int32_t* t_lock, int buf_rows, int32_t* prev_rows);
int slk_posterior_carry(hipStream_t s, void* store, size_t buf_bytes, size_t row_bytes, const int32_t* probe_idx,
                        const int32_t* m_dev, int m_upper, const int32_t* t_lock, const uint8_t* unlocked, int t);
int slk_unmask_topk(hipStream_t s, int32_t* tokens, uint8_t* masked, const int32_t* active_idx,
                    const int32_t* cu_active, const float* conf, const int32_t* argmax,
                    int B, int N, int lo, int hi, int k, int m_upper);
int slk_unmask_lock(hipStream_t s, int32_t* tokens, uint8_t* masked, const int32_t* active_idx,
                    const int32_t* cu_active, const float* conf, const int32_t* argmax, int B, int N, int lo, int hi,
                    int k, int m_upper, const uint8_t* lock, const float* kl, const float* eps, int first_step,
                    uint8_t* new_lock);
int slk_lock_rule(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                  const int32_t* m_dev, int m_upper, const float* kl, const float* eps, int B, int N,
                  int first_step, uint8_t* new_lock);
// score_kernel.hip
int slk_score(hipStream_t s, const void* cur, int cur_packed, const void* prev, int dtype, int V,
              const int32_t* active_idx, const int32_t* m_dev, int m_upper, int first_step,
              float* kl, float* conf, int32_t* argmax, void* scratch);
size_t slk_score_scratch_bytes();
// rowwise_kernels.hip
// `tiled`: write h / a in the fragment-tiled layout (afrag_index) instead of row-major
int slk_embed_rmsnorm(hipStream_t s, int dtype, const void* emb, const int32_t* tokens, const int32_t* active_idx,
                      const int32_t* m_dev, int m_upper, int d, int vocab, const void* gain, float eps, void* x,
                      void* h, int tiled);
// delta / qkv / gu may be S k-split partials, `sstride` floats apart; they are summed in split order
int slk_add_rmsnorm(hipStream_t s, int dtype, void* x, const float* delta, int S, size_t sstride,
                    const int32_t* m_dev, int m_upper, int d, const void* gain, float eps, void* h, int tiled);
int slk_rmsnorm(hipStream_t s, int dtype, const void* x, const int32_t* m_dev, int m_upper, int d,
                const void* gain, float eps, void* h, int tiled);
int slk_rope_table(hipStream_t s, void* tab, int n_pad, int dh, float theta);
int slk_gemm_mfma256_residual(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                              void* x);
int slk_gemm_mfma256_qkv_rope(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int H, int k,
                              const int32_t* active_idx, int N, int n_pad, const void* rope_tab, void* q, void* kc,
                              void* vc);
int slk_rope_kv_write(hipStream_t s, int dtype, const float* qkv, int S, size_t sstride, const int32_t* active_idx,
                      const int32_t* m_dev, int m_upper, int H, int dh, int N, int n_pad, const void* rope_tab, void* q, void* kc, void* vc,
                      int v_half);
int slk_swiglu(hipStream_t s, int dtype, const float* gu, int S, size_t sstride, const int32_t* m_dev, int m_upper,
               int dff, void* a, int tiled, int interleaved);
int slk_kv_read(hipStream_t s, int dtype, const void* kc, const void* vc, int B, int H, int N, int n_pad, int dh,
                void* k_out, void* v_out, int v_half);
int slk_fill_zero(hipStream_t s, void* p, size_t bytes);
int slk_copy_rows(hipStream_t s, int dtype, const void* src, void* dst, const int32_t* m_dev, int m_upper, int d);
// gemm_generic.hip:  C[m, n] (fp32, ldc) = A[m, k] (T) . W[n, k]^T (T); optional row map for the output
int slk_gemm_generic(hipStream_t s, int dtype, const void* A, const void* W, const int32_t* m_dev, int m_upper,
                     int n, int k, float* C_f32, void* C_T, const int32_t* out_row_map, size_t ldc);
// attention_generic.hip
int slk_attention_generic(hipStream_t s, int dtype, const void* q, const void* kc, const void* vc,
                          const int32_t* active_idx, const int32_t* m_dev, int m_upper,
                          int H, int dh, int N, int n_pad, void* o);

// gemm_mfma.hip
int slk_pack_weight(hipStream_t s, const void* W, int n, int k, void* P, int nb_off, int nb_stride);
int slk_gemm_unsplit_thick(int mu, int n, int k);
int slk_gemm_stream_swiglu_ok(int mu, int dff, int k);
int slk_gemm_stream_swiglu(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int dff, int k,
                           void* a);
int slk_gemm_splits_gate_up(int mu, int n, int k);
// gate|up projection with interleaved 32-column blocks (gate j, up j, gate j+1, ..) and SwiGLU in the
// epilogue: a[row, c] = silu(g) * u as bf16 in the fragment-tiled layout; no k-split
int slk_gemm_mfma256_probe(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n,
                           int k, void* Cb, const int32_t* row_map, size_t ldc, long long* probe);
int slk_gemm_mfma256_swiglu(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int dff, int k,
                            void* a);
int slk_gemm_splits(int mu, int n, int k);
int slk_gemm_describe(int mu, int n, int k, int* kind, int* splits, int* rows, int* cols, int* tail);
// a_tiled: A is in the fragment-tiled layout (rows padded to 32) instead of row-major
int slk_gemm_mfma(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                  int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc);
int slk_gemm_mfma256(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n,
                     int k, int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc);
// attention_mfma.hip
int slk_attention_mfma(hipStream_t s, const void* q, const void* kc, const void* vc, const int32_t* active_idx,
                       const int32_t* m_dev, int m_upper, int B, int H, int N, int n_pad, void* o, float* scratch);
size_t slk_attention_scratch_elems(int m_upper, int B, int H, int n_pad);
// mfma path (mfma_layer.hip)
size_t sl_mfma_f32_elems(const sl_config* cfg, int mu);
bool sl_mfma_supported(const sl_config* cfg);
size_t sl_mfma_packed_bytes(const sl_config* cfg);
int sl_mfma_pack_all(sl_ctx* ctx, hipStream_t s, void* packed);
int sl_mfma_layer(sl_ctx* ctx, hipStream_t s, int layer, void* x, void* h, void* q, void* o, void* a, float* f32,
                  float* attn_scratch, const int32_t* active_idx, const int32_t* m_dev, int mu, const void* next_gain);
int sl_mfma_lm_head(sl_ctx* ctx, hipStream_t s, const void* h, const int32_t* active_idx, const int32_t* m_dev, int mu,
                    void* logits_buf);
