// Row-wise (HBM-streaming) kernels of the restricted forward: embedding gather fused with
// the first RMSNorm, residual-add fused with the next RMSNorm, RoPE fused with the K/V
// cache write, SwiGLU, and cache maintenance.  One workgroup per active row; rows beyond
// the true M (read from device memory) exit at once.
#include "sl_common.h"

constexpr int kRowThreads = 256;

// Alg. 1 'Initialize block input' for the active rows, fused with the first layer's LN:
// x = Emb[token], h = rnd(x * rsqrt(mean(x^2) + eps) * gain).  The row (a few KB) is read a
// second time from cache for the scaling pass instead of being held in registers.
template <typename T, bool TILED>
__global__ __launch_bounds__(kRowThreads) void embed_rmsnorm_kernel(const T* __restrict__ emb,
                                                                    const int32_t* __restrict__ tokens,
                                                                    const int32_t* __restrict__ active_idx,
                                                                    const int32_t* __restrict__ m_dev, int m_upper,
                                                                    int d, int vocab, const T* __restrict__ gain,
                                                                    float eps, T* __restrict__ x, T* __restrict__ h) {
  __shared__ float sh[kRowThreads / 64];
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  // token ids are device data nobody validated: an id outside the table (a caller's mistake, or
  // an argmax over non-finite logits) must not become an out-of-bounds read
  const int tok = min(max(tokens[active_idx[r]], 0), vocab - 1);
  const T* src = emb + (size_t)tok * d;
  float ssq = 0.f;
  for (int c = threadIdx.x; c < d; c += kRowThreads) {
    const T v = src[c];
    x[(size_t)r * d + c] = v;
    ssq += (float)v * (float)v;
  }
  ssq = block_sum<kRowThreads>(ssq, sh);
  const float rstd = 1.0f / sqrtf(ssq / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += kRowThreads)
    st<T>::stv(h + act_index<TILED>(r, c, d), st<T>::ld(src + c) * rstd * st<T>::ld(gain + c));
}

// x <- rnd(x + delta) (residual add in fp32; delta may arrive as S k-split partials),
// then h = RMSNorm of the STORED x.
template <typename T, bool ADD, bool TILED>
__global__ __launch_bounds__(kRowThreads) void add_rmsnorm_kernel(T* x, const float* __restrict__ delta, int S,
                                                                  size_t sstride,
                                                                  const int32_t* __restrict__ m_dev, int m_upper,
                                                                  int d, const T* __restrict__ gain, float eps,
                                                                  T* __restrict__ h) {
  __shared__ float sh[kRowThreads / 64];
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  T* xr = x + (size_t)r * d;
  float ssq = 0.f;
  for (int c = threadIdx.x; c < d; c += kRowThreads) {
    float v = st<T>::ld(xr + c);
    if (ADD) {
      const float* dp = delta + (size_t)r * d + c;
      float dl = dp[0];
      int sp = 1;
      for (; sp + 3 < S; sp += 4) {             // k-split partials, fixed order, 4 loads in flight
        const float p0 = dp[sp * sstride], p1 = dp[(sp + 1) * sstride], p2 = dp[(sp + 2) * sstride],
                    p3 = dp[(sp + 3) * sstride];
        dl = (((dl + p0) + p1) + p2) + p3;
      }
      for (; sp < S; ++sp) dl += dp[sp * sstride];
      v = st<T>::rnd(v + dl);
      st<T>::stv(xr + c, v);
    }
    ssq += v * v;
  }
  ssq = block_sum<kRowThreads>(ssq, sh);
  const float rstd = 1.0f / sqrtf(ssq / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += kRowThreads)   // each thread re-reads what it wrote itself
    st<T>::stv(h + act_index<TILED>(r, c, d), st<T>::ld(xr + c) * rstd * st<T>::ld(gain + c));
}

// q, k <- rnd(RoPE(q, k)) at the row's fixed slot; v <- rnd(v); k, v go to the row's own
// cache slot (the only cache rows this step may touch), q to the packed query buffer.
// Half-split pairing (j, j + d_h/2); angles come from a table built in fp64 at bind time.
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_write_kernel(const float* __restrict__ qkv, int S, size_t sstride,
                                                            const int32_t* __restrict__ active_idx,
                                                            const int32_t* __restrict__ m_dev, int m_upper, int H,
                                                            int dh, int N, int n_pad,
                                                            const float2* __restrict__ rope_tab, T* __restrict__ q,
                                                            T* __restrict__ kc, T* __restrict__ vc) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  const int g = active_idx[r];
  const int b = g / N, i = g - b * N;
  const int half = dh >> 1, hd = H * dh;
  const float* row = qkv + (size_t)r * 3 * hd;
  for (int e = threadIdx.x; e < H * half; e += blockDim.x) {
    const int hh = e / half, j = e - hh * half;
    const float2 cs = rope_tab[(size_t)i * half + j];
    const int c0 = hh * dh + j, c1 = c0 + half;
    float q0 = row[c0], q1 = row[c1];
    float k0 = row[hd + c0], k1 = row[hd + c1];
    float v0 = row[2 * hd + c0], v1 = row[2 * hd + c1];
    for (int sp = 1; sp < S; ++sp) {                     // k-split partials, fixed order
      const float* pr = row + sp * sstride;
      q0 += pr[c0]; q1 += pr[c1];
      k0 += pr[hd + c0]; k1 += pr[hd + c1];
      v0 += pr[2 * hd + c0]; v1 += pr[2 * hd + c1];
    }
    st<T>::stv(q + (size_t)r * hd + c0, q0 * cs.x - q1 * cs.y);
    st<T>::stv(q + (size_t)r * hd + c1, q1 * cs.x + q0 * cs.y);
    const size_t head_base = ((size_t)b * H + hh) * n_pad * dh;
    st<T>::stv(kc + head_base + kc_index(i, j, dh), k0 * cs.x - k1 * cs.y);
    st<T>::stv(kc + head_base + kc_index(i, j + half, dh), k1 * cs.x + k0 * cs.y);
    st<T>::stv(vc + head_base + vc_index(i, j, dh), v0);
    st<T>::stv(vc + head_base + vc_index(i, j + half, dh), v1);
  }
}

// cos/sin of pos * theta^(-2j/d_h), evaluated in fp64 once per (slot, pair).
__global__ void rope_table_kernel(float2* tab, int n_pad, int half, int dh, double theta) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_pad * half) return;
  const int i = t / half, j = t - i * half;
  const double ang = (double)i * pow(theta, -2.0 * (double)j / (double)dh);
  tab[t] = make_float2((float)cos(ang), (float)sin(ang));
}

template <typename T, bool TILED>
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ gu, int S, size_t sstride,
                                                     const int32_t* __restrict__ m_dev, int m_upper, int dff,
                                                     T* __restrict__ a) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.y;
  if (r >= M) return;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= dff) return;
  float g = gu[(size_t)r * 2 * dff + c], u = gu[(size_t)r * 2 * dff + dff + c];
  for (int sp = 1; sp < S; ++sp) {
    g += gu[sp * sstride + (size_t)r * 2 * dff + c];
    u += gu[sp * sstride + (size_t)r * 2 * dff + dff + c];
  }
  st<T>::stv(a + act_index<TILED>(r, c, dff), g / (1.0f + expf(-g)) * u);
}

template <typename T>
__global__ void kv_read_kernel(const T* __restrict__ kc, const T* __restrict__ vc, int B, int H, int N, int n_pad,
                               int dh, T* __restrict__ k_out, T* __restrict__ v_out) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)B * N * H * dh;
  if (t >= total) return;
  const int dd = t % dh;
  const int hh = (t / dh) % H;
  const int i = (t / ((size_t)dh * H)) % N;
  const int b = t / ((size_t)dh * H * N);
  const size_t head_base = ((size_t)b * H + hh) * n_pad * dh;
  k_out[t] = kc[head_base + kc_index(i, dd, dh)];
  v_out[t] = vc[head_base + vc_index(i, dd, dh)];
}

__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < n16; t += stride) p[t] = make_uint4(0, 0, 0, 0);
}

template <typename T>
__global__ void copy_rows_kernel(const T* __restrict__ src, T* __restrict__ dst, const int32_t* __restrict__ m_dev,
                                 int m_upper, int d) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  for (int c = threadIdx.x; c < d; c += blockDim.x) dst[(size_t)r * d + c] = src[(size_t)r * d + c];
}

// ---- launchers ---------------------------------------------------------------------------------
#define DISPATCH_T(dtype, ...)                                  \
  do {                                                          \
    if ((dtype) == SL_BF16) { using T = bf16_t; __VA_ARGS__; }  \
    else { using T = float; __VA_ARGS__; }                      \
  } while (0)

#define DISPATCH_TILED(tiled, ...)                      \
  do {                                                  \
    if (tiled) { constexpr bool TL = true; __VA_ARGS__; } \
    else { constexpr bool TL = false; __VA_ARGS__; }    \
  } while (0)

int slk_embed_rmsnorm(hipStream_t s, int dtype, const void* emb, const int32_t* tokens, const int32_t* active_idx,
                      const int32_t* m_dev, int m_upper, int d, int vocab, const void* gain, float eps, void* x,
                      void* h, int tiled) {
  if (m_upper <= 0) return SL_OK;
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((embed_rmsnorm_kernel<T, TL>), dim3(m_upper),
                                                             dim3(kRowThreads), 0, s, (const T*)emb, tokens,
                                                             active_idx, m_dev, m_upper, d, vocab, (const T*)gain,
                                                             eps, (T*)x, (T*)h)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_add_rmsnorm(hipStream_t s, int dtype, void* x, const float* delta, int S, size_t sstride,
                    const int32_t* m_dev, int m_upper, int d, const void* gain, float eps, void* h, int tiled) {
  if (m_upper <= 0) return SL_OK;
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_kernel<T, true, TL>), dim3(m_upper),
                                                             dim3(kRowThreads), 0, s, (T*)x, delta, S, sstride,
                                                             m_dev, m_upper, d, (const T*)gain, eps, (T*)h)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_rmsnorm(hipStream_t s, int dtype, const void* x, const int32_t* m_dev, int m_upper, int d, const void* gain,
                float eps, void* h, int tiled) {
  if (m_upper <= 0) return SL_OK;
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_kernel<T, false, TL>), dim3(m_upper),
                                                             dim3(kRowThreads), 0, s, (T*)const_cast<void*>(x),
                                                             (const float*)nullptr, 1, (size_t)0, m_dev, m_upper, d,
                                                             (const T*)gain, eps, (T*)h)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_rope_table(hipStream_t s, void* tab, int n_pad, int dh, float theta) {
  const int half = dh / 2, n = n_pad * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3(sl_cdiv(n, 256)), dim3(256), 0, s, (float2*)tab, n_pad, half, dh,
                     (double)theta);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_rope_kv_write(hipStream_t s, int dtype, const float* qkv, int S, size_t sstride, const int32_t* active_idx,
                      const int32_t* m_dev, int m_upper, int H, int dh, int N, int n_pad, const void* rope_tab, void* q, void* kc,
                      void* vc) {
  if (m_upper <= 0) return SL_OK;
  DISPATCH_T(dtype, hipLaunchKernelGGL((rope_kv_write_kernel<T>), dim3(m_upper), dim3(256), 0, s, qkv, S, sstride,
                                       active_idx, m_dev, m_upper, H, dh, N, n_pad, (const float2*)rope_tab, (T*)q, (T*)kc,
                                       (T*)vc));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_swiglu(hipStream_t s, int dtype, const float* gu, int S, size_t sstride, const int32_t* m_dev, int m_upper,
               int dff, void* a, int tiled) {
  if (m_upper <= 0) return SL_OK;
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((swiglu_kernel<T, TL>), dim3(sl_cdiv(dff, 256), m_upper),
                                                             dim3(256), 0, s, gu, S, sstride, m_dev, m_upper, dff,
                                                             (T*)a)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_kv_read(hipStream_t s, int dtype, const void* kc, const void* vc, int B, int H, int N, int n_pad, int dh,
                void* k_out, void* v_out) {
  const size_t total = (size_t)B * N * H * dh;
  DISPATCH_T(dtype, hipLaunchKernelGGL((kv_read_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                                       (const T*)kc, (const T*)vc, B, H, N, n_pad, dh, (T*)k_out, (T*)v_out));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_fill_zero(hipStream_t s, void* p, size_t bytes) {
  if (bytes == 0) return SL_OK;
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, n16);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_copy_rows(hipStream_t s, int dtype, const void* src, void* dst, const int32_t* m_dev, int m_upper, int d) {
  if (m_upper <= 0) return SL_OK;
  DISPATCH_T(dtype, hipLaunchKernelGGL((copy_rows_kernel<T>), dim3(m_upper), dim3(256), 0, s, (const T*)src, (T*)dst,
                                       m_dev, m_upper, d));
  SL_LAUNCH_CHECK();
  return SL_OK;
}
