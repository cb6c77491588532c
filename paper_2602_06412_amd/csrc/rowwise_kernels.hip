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
template <typename T, bool VH>
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
    if (kc == nullptr) continue;                         // read-only probe: queries only
    const size_t head_base = ((size_t)b * H + hh) * n_pad * dh;
    st<T>::stv(kc + head_base + kc_index(i, j, dh), k0 * cs.x - k1 * cs.y);
    st<T>::stv(kc + head_base + kc_index(i, j + half, dh), k1 * cs.x + k0 * cs.y);
    if constexpr (VH) {                                  // bf16 storage only (see vcache_half_bits)
      vc[head_base + vc_index(i, j, dh)] = vcache_half_bits(v0);
      vc[head_base + vc_index(i, j + half, dh)] = vcache_half_bits(v1);
    } else {
      st<T>::stv(vc + head_base + vc_index(i, j, dh), v0);
      st<T>::stv(vc + head_base + vc_index(i, j + half, dh), v1);
    }
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

// gu holds gate and up side by side ([gate dff | up dff], interleaved = 0) or interleaved by
// 32-column blocks (gate j, up j, gate j+1, .., interleaved = 1).
template <typename T, bool TILED>
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ gu, int S, size_t sstride,
                                                     const int32_t* __restrict__ m_dev, int m_upper, int dff,
                                                     int interleaved, T* __restrict__ a) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.y;
  if (r >= M) return;
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= dff) return;
  const size_t gi = (size_t)r * 2 * dff + (interleaved ? (c >> 5) * 64 + (c & 31) : c);
  const size_t ui = gi + (interleaved ? 32 : dff);
  float g = gu[gi], u = gu[ui];
  for (int sp = 1; sp < S; ++sp) {
    g += gu[sp * sstride + gi];
    u += gu[sp * sstride + ui];
  }
  st<T>::stv(a + act_index<TILED>(r, c, dff), g / (1.0f + expf(-g)) * u);
}

template <typename T, bool VH>
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
  if constexpr (VH) v_out[t] = vcache_half_value(vc[head_base + vc_index(i, dd, dh)]);
  else v_out[t] = vc[head_base + vc_index(i, dd, dh)];
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

// ---- bf16 variants with 16-byte accesses ---------------------------------------------------------
// Same arithmetic, in the same order, as the element-wise kernels above; a thread owns chunks of
// consecutive columns, so loads and stores are 8 or 16 bytes wide (also in the fragment-tiled
// layout, where the eight columns starting at a multiple of eight are contiguous) and all loads
// of a thread are in flight together.  Used when shapes and pointers allow, else the kernels above.
// bf16, fragment-tiled output, gate/up interleaved by 32-column blocks: a thread owns eight consecutive
// output columns (32-byte loads of the gate and the up sums per plane, one 16-byte store); same arithmetic.
__global__ __launch_bounds__(256) void swiglu_vec_kernel(const float* __restrict__ gu, int S, size_t sstride,
                                                         const int32_t* __restrict__ m_dev, int m_upper, int dff,
                                                         bf16_t* __restrict__ a) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.y;
  if (r >= M) return;
  const int c = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
  if (c >= dff) return;
  const float* gp = gu + (size_t)r * 2 * dff + (c >> 5) * 64 + (c & 31);
  float g[8], u[8], o[8];
  ld8f(gp, g);
  ld8f(gp + 32, u);
  for (int sp = 1; sp < S; ++sp) {
    float t[8], v[8];
    ld8f(gp + sp * sstride, t);
    ld8f(gp + sp * sstride + 32, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) { g[e] += t[e]; u[e] += v[e]; }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
  st8(a + afrag_index(r, c, dff), o);
}

constexpr int kMaxChunks = 4;             // chunks of 8 columns per thread: rows up to 8192 columns

template <bool TILED>
__global__ __launch_bounds__(kRowThreads) void embed_rmsnorm_vec_kernel(
    const bf16_t* __restrict__ emb, const int32_t* __restrict__ tokens, const int32_t* __restrict__ active_idx,
    const int32_t* __restrict__ m_dev, int m_upper, int d, int vocab, const bf16_t* __restrict__ gain, float eps,
    bf16_t* __restrict__ x, bf16_t* __restrict__ h) {
  __shared__ float sh[kRowThreads / 64];
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  const int tok = min(max(tokens[active_idx[r]], 0), vocab - 1);     // see embed_rmsnorm_kernel
  const bf16_t* src = emb + (size_t)tok * d;
  const int nch = d >> 3;
  float v[kMaxChunks][8];
  float ssq = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c8 = threadIdx.x + j * kRowThreads;
    if (c8 < nch) {
      const bf16x8_t u = *reinterpret_cast<const bf16x8_t*>(src + c8 * 8);
      *reinterpret_cast<bf16x8_t*>(x + (size_t)r * d + c8 * 8) = u;
#pragma unroll
      for (int e = 0; e < 8; ++e) { v[j][e] = (float)u[e]; ssq += v[j][e] * v[j][e]; }
    }
  }
  ssq = block_sum<kRowThreads>(ssq, sh);
  const float rstd = 1.0f / sqrtf(ssq / (float)d + eps);
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c8 = threadIdx.x + j * kRowThreads;
    if (c8 < nch) {
      float g[8], o[8];
      ld8(gain + c8 * 8, g);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = v[j][e] * rstd * g[e];
      st8(h + act_index<TILED>(r, c8 * 8, d), o);
    }
  }
}

__device__ inline void ld4(const bf16_t* p, float (&v)[4]) {
  const bf16x4_t u = *reinterpret_cast<const bf16x4_t*>(p);
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = (float)u[e];
}
template <bool ADD, bool TILED>
__global__ __launch_bounds__(kRowThreads) void add_rmsnorm_vec_kernel(bf16_t* x, const float* __restrict__ delta, int S,
                                                                      size_t sstride,
                                                                      const int32_t* __restrict__ m_dev, int m_upper,
                                                                      int d, const bf16_t* __restrict__ gain,
                                                                      float eps, bf16_t* __restrict__ h) {
  __shared__ float sh[kRowThreads / 64];
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  bf16_t* xr = x + (size_t)r * d;
  const int nch = d >> 3;
  float v[kMaxChunks][8];
  float ssq = 0.f;
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c8 = threadIdx.x + j * kRowThreads;
    if (c8 < nch) {
      ld8(xr + c8 * 8, v[j]);
      if (ADD) {
        const float* dp = delta + (size_t)r * d + c8 * 8;
        float dl[8];
        ld8f(dp, dl);
        // k-split partials, added in plane order; up to seven loads are issued before the first add (one
        // load per trip made the launch a chain of S memory latencies: 7.4 us at 16 rows and S = 8)
        for (int sp0 = 1; sp0 < S; sp0 += 7) {
          float pp[7][8];
#pragma unroll
          for (int i = 0; i < 7; ++i)
            if (sp0 + i < S) ld8f(dp + (size_t)(sp0 + i) * sstride, pp[i]);
#pragma unroll
          for (int i = 0; i < 7; ++i)
            if (sp0 + i < S) {
#pragma unroll
              for (int e = 0; e < 8; ++e) dl[e] += pp[i][e];
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[j][e] = st<bf16_t>::rnd(v[j][e] + dl[e]);
        st8(xr + c8 * 8, v[j]);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) ssq += v[j][e] * v[j][e];
    }
  }
  ssq = block_sum<kRowThreads>(ssq, sh);
  const float rstd = 1.0f / sqrtf(ssq / (float)d + eps);
#pragma unroll
  for (int j = 0; j < kMaxChunks; ++j) {
    const int c8 = threadIdx.x + j * kRowThreads;
    if (c8 < nch) {
      float g[8], o[8];
      ld8(gain + c8 * 8, g);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = v[j][e] * rstd * g[e];
      st8(h + act_index<TILED>(r, c8 * 8, d), o);
    }
  }
}

// Thick-launch variant of the kernel above for d = 512 CH: one wave per row (four rows per workgroup),
// the row held in registers (CH chunks of 8 per lane), the sum of squares reduced by shuffles, no LDS and
// no barrier.  With thousands of rows the block-per-row kernel is bound by workgroup turnover (8 KB of
// traffic per workgroup in the norm-only form); this one keeps a wave streaming: norm-only at 8192 rows
// 65 -> 38 us.  Taken from 2048 rows on (at 512 rows its 128 workgroups leave half the chip idle).
template <bool ADD, bool TILED, int CH>
__global__ __launch_bounds__(256) void add_rmsnorm_wave_kernel(bf16_t* x, const float* __restrict__ delta, int S,
                                                               size_t sstride, const int32_t* __restrict__ m_dev,
                                                               int m_upper, const bf16_t* __restrict__ gain, float eps,
                                                               bf16_t* __restrict__ h) {
  constexpr int d = 512 * CH;
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= M) return;
  bf16_t* xr = x + (size_t)r * d;
  float v[CH][8];
  float ssq = 0.f;
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int c8 = lane + j * 64;
    ld8(xr + c8 * 8, v[j]);
    if (ADD) {
      const float* dp = delta + (size_t)r * d + c8 * 8;
      float dl[8];
      ld8f(dp, dl);
      for (int sp = 1; sp < S; ++sp) {            // k-split partials, fixed order
        float pp[8];
        ld8f(dp + sp * sstride, pp);
#pragma unroll
        for (int e = 0; e < 8; ++e) dl[e] += pp[e];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) v[j][e] = st<bf16_t>::rnd(v[j][e] + dl[e]);
      st8(xr + c8 * 8, v[j]);
    }
  }
  // The sum of squares is taken in the order of the block-per-row kernels (thread t of 256 sums chunks t
  // and t + 256, wave totals are added in wave order), so that a row's result does not depend on which
  // kernel the launch size selects.
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float part = 0.f;
#pragma unroll
    for (int jj = w; jj < CH; jj += 4)
#pragma unroll
      for (int e = 0; e < 8; ++e) part += v[jj][e] * v[jj][e];
    ssq += wave_sum(part);
  }
  const float rstd = 1.0f / sqrtf(ssq / (float)d + eps);
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int c8 = lane + j * 64;
    float g[8], o[8];
    ld8(gain + c8 * 8, g);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = v[j][e] * rstd * g[e];
    st8(h + act_index<TILED>(r, c8 * 8, d), o);
  }
}

// Thin-launch variant.  One thread per (head, four rotation pairs): fp32 loads are 16 bytes and
// those of a wave contiguous, q and K leave as 8-byte stores (consecutive dims
// of one slot are contiguous in the K layout); V keeps 2-byte stores, its layout puts eight
// SLOTS side by side, not eight dims.
template <bool VH>
__global__ __launch_bounds__(256) void rope_kv_write_vec_kernel(const float* __restrict__ qkv, int S, size_t sstride,
                                                                const int32_t* __restrict__ active_idx,
                                                                const int32_t* __restrict__ m_dev, int m_upper, int H,
                                                                int dh, int N, int n_pad,
                                                                const float2* __restrict__ rope_tab,
                                                                bf16_t* __restrict__ q, bf16_t* __restrict__ kc,
                                                                bf16_t* __restrict__ vc) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  const int g = active_idx[r];
  const int b = g / N, i = g - b * N;
  const int half = dh >> 1, hd = H * dh, per_head = half >> 2;
  const float* row = qkv + (size_t)r * 3 * hd;
  // gridDim.y workgroups share a row (a launch of few rows would otherwise leave most CUs without a workgroup)
  const int per_wg = (H * per_head + gridDim.y - 1) / gridDim.y, t_end = min(H * per_head, (int)(blockIdx.y + 1) * per_wg);
  for (int t = blockIdx.y * per_wg + threadIdx.x; t < t_end; t += blockDim.x) {
    const int hh = t / per_head, j = (t - hh * per_head) * 4;
    const int c0 = hh * dh + j, c1 = c0 + half;
    float q0[4], q1[4], k0[4], k1[4], v0[4], v1[4], cs0[4], cs1[4];
    ld4f(row + c0, q0); ld4f(row + c1, q1);
    ld4f(row + hd + c0, k0); ld4f(row + hd + c1, k1);
    ld4f(row + 2 * hd + c0, v0); ld4f(row + 2 * hd + c1, v1);
    const float* tab = reinterpret_cast<const float*>(rope_tab + (size_t)i * half + j);   // (cos, sin) x 4
    ld4f(tab, cs0); ld4f(tab + 4, cs1);
    for (int sp = 1; sp < S; ++sp) {                     // k-split partials, fixed order
      const float* pr = row + sp * sstride;
      float p[4];
#define SL_ACC4(dst, src) do { ld4f(src, p); _Pragma("unroll") for (int e = 0; e < 4; ++e) dst[e] += p[e]; } while (0)
      SL_ACC4(q0, pr + c0); SL_ACC4(q1, pr + c1);
      SL_ACC4(k0, pr + hd + c0); SL_ACC4(k1, pr + hd + c1);
      SL_ACC4(v0, pr + 2 * hd + c0); SL_ACC4(v1, pr + 2 * hd + c1);
#undef SL_ACC4
    }
    float qa[4], qb[4], ka[4], kb[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float c = e < 2 ? cs0[2 * e] : cs1[2 * (e - 2)], sn = e < 2 ? cs0[2 * e + 1] : cs1[2 * (e - 2) + 1];
      qa[e] = q0[e] * c - q1[e] * sn;
      qb[e] = q1[e] * c + q0[e] * sn;
      ka[e] = k0[e] * c - k1[e] * sn;
      kb[e] = k1[e] * c + k0[e] * sn;
    }
    st4(q + (size_t)r * hd + c0, qa);
    st4(q + (size_t)r * hd + c1, qb);
    if (kc == nullptr) continue;                         // read-only probe: queries only
    const size_t head_base = ((size_t)b * H + hh) * n_pad * dh;
    st4(kc + head_base + kc_index(i, j, dh), ka);
    st4(kc + head_base + kc_index(i, j + half, dh), kb);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vc[head_base + vc_index(i, j + e, dh)] = vcache_elem<VH>(v0[e]);
      vc[head_base + vc_index(i, j + half + e, dh)] = vcache_elem<VH>(v1[e]);
    }
  }
}

// Thick-launch variant: one workgroup per 16 consecutive packed rows, one head at a time.
// Loads are 16 bytes per thread and contiguous along a row; q leaves directly (8-byte stores);
// K and V of the head are staged in LDS as 16-bit cache elements and leave in the order of the cache layouts:
//   K: a thread writes the 16-byte unit (slot, 8 dims); the 16 rows of a unit column are 16
//      lanes, so consecutive slots give 256 contiguous bytes;
//   V: the cache puts eight SLOTS side by side per dim (slots 16A + 4c + {0..3} and 16A + 8 + 4c +
//      {0..3} form the 16-byte group c of block A).  When the 16 rows are the 16 consecutive
//      slots of one aligned block (the common case while large parts of a sequence are still
//      active) a thread writes one group as a 16-byte store, a wave 1 KiB contiguous; otherwise V
//      falls back to 2-byte stores.
// Requires d_h = 128 (256 threads = 16 rows x 16 chunks of four rotation pairs).
template <bool VH>
__global__ __launch_bounds__(256) void rope_kv_write_block_kernel(const float* __restrict__ qkv, int S, size_t sstride,
                                                                  const int32_t* __restrict__ active_idx,
                                                                  const int32_t* __restrict__ m_dev, int m_upper, int H,
                                                                  int N, int n_pad, const float2* __restrict__ rope_tab,
                                                                  bf16_t* __restrict__ q, bf16_t* __restrict__ kc,
                                                                  bf16_t* __restrict__ vc) {
  constexpr int RB = 16, dh = 128, half = 64;
  const int M = min(*m_dev, m_upper);
  const int r0 = blockIdx.x * RB;
  if (r0 >= M) return;
  const int nrows = min(RB, M - r0);
  __shared__ int slot_sh[RB];
  __shared__ int dense_sh;
  __shared__ __align__(16) bf16_t kbuf[RB][dh + 8];     // +8: rows 272 bytes apart, 16-byte aligned, banks spread
  __shared__ __align__(16) bf16_t vbuf[RB][dh + 8];
  if (threadIdx.x < RB) slot_sh[threadIdx.x] = threadIdx.x < nrows ? active_idx[r0 + threadIdx.x] : -1;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int g0 = slot_sh[0];
    bool dense = nrows == RB && (g0 % N) % RB == 0 && (g0 % N) + RB <= N;
    for (int j = 1; j < RB && dense; ++j) dense = slot_sh[j] == g0 + j;
    dense_sh = dense;
  }
  __syncthreads();
  const bool dense = dense_sh != 0;
  const int hd = H * dh;
  // compute role: row j, rotation pairs jj .. jj+3
  const int j = threadIdx.x >> 4, jj = (threadIdx.x & 15) * 4;
  const bool live = j < nrows;
  const int g = live ? slot_sh[j] : 0;
  const int b = g / N, i = g - b * N;
  float cs0[4] = {0.f, 0.f, 0.f, 0.f}, cs1[4] = {0.f, 0.f, 0.f, 0.f};
  if (live) {
    const float* tab = reinterpret_cast<const float*>(rope_tab + (size_t)i * half + jj);   // (cos, sin) x 4
    ld4f(tab, cs0); ld4f(tab + 4, cs1);
  }
  // K store role: unit (slot js, dims 8 dg .. 8 dg + 7); V store role: group vcg of the block, dim vdim
  const int js = threadIdx.x & 15, dg = threadIdx.x >> 4;
  const int vcg = threadIdx.x >> 7, vdim = threadIdx.x & 127;
  const int gs = js < nrows ? slot_sh[js] : -1;
  const int g0 = slot_sh[0];
  // the heads are divided over gridDim.y workgroups (thin launches would otherwise leave CUs idle)
  const int h_per = H / gridDim.y;
  for (int hh = blockIdx.y * h_per; hh < (blockIdx.y + 1) * h_per; ++hh) {
    if (live) {
      const float* row = qkv + (size_t)(r0 + j) * 3 * hd;
      const int c0 = hh * dh + jj, c1 = c0 + half;
      float q0[4], q1[4], k0[4], k1[4], v0[4], v1[4];
      ld4f(row + c0, q0); ld4f(row + c1, q1);
      ld4f(row + hd + c0, k0); ld4f(row + hd + c1, k1);
      ld4f(row + 2 * hd + c0, v0); ld4f(row + 2 * hd + c1, v1);
      for (int sp = 1; sp < S; ++sp) {                     // k-split partials, fixed order
        const float* pr = row + sp * sstride;
        float p[4];
#define SL_ACC4(dst, src) do { ld4f(src, p); _Pragma("unroll") for (int e = 0; e < 4; ++e) dst[e] += p[e]; } while (0)
        SL_ACC4(q0, pr + c0); SL_ACC4(q1, pr + c1);
        SL_ACC4(k0, pr + hd + c0); SL_ACC4(k1, pr + hd + c1);
        SL_ACC4(v0, pr + 2 * hd + c0); SL_ACC4(v1, pr + 2 * hd + c1);
#undef SL_ACC4
      }
      float qa[4], qb[4], ka[4], kb[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float c = e < 2 ? cs0[2 * e] : cs1[2 * (e - 2)], sn = e < 2 ? cs0[2 * e + 1] : cs1[2 * (e - 2) + 1];
        qa[e] = q0[e] * c - q1[e] * sn;
        qb[e] = q1[e] * c + q0[e] * sn;
        ka[e] = k0[e] * c - k1[e] * sn;
        kb[e] = k1[e] * c + k0[e] * sn;
      }
      st4(q + (size_t)(r0 + j) * hd + c0, qa);
      st4(q + (size_t)(r0 + j) * hd + c1, qb);
      st4(&kbuf[j][jj], ka);
      st4(&kbuf[j][jj + half], kb);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vbuf[j][jj + e] = vcache_elem<VH>(v0[e]);
        vbuf[j][jj + half + e] = vcache_elem<VH>(v1[e]);
      }
    }
    __syncthreads();
    if (gs >= 0) {
      const int bs = gs / N, is = gs - bs * N;
      const size_t head_base = ((size_t)bs * H + hh) * n_pad * dh;
      *reinterpret_cast<bf16x8_t*>(kc + head_base + kc_index(is, dg * 8, dh)) =
          *reinterpret_cast<const bf16x8_t*>(&kbuf[js][dg * 8]);
    }
    if (dense) {
      const int bb = g0 / N, i0 = g0 - bb * N;
      const size_t head_base = ((size_t)bb * H + hh) * n_pad * dh;
      bf16x8_t out;
#pragma unroll
      for (int e = 0; e < 8; ++e) out[e] = vbuf[(e >> 2) * 8 + 4 * vcg + (e & 3)][vdim];
      *reinterpret_cast<bf16x8_t*>(vc + head_base + vc_index(i0 + 4 * vcg, vdim, dh)) = out;
    } else {
      // 16 rows x 128 dims as 2-byte stores, eight per thread
      for (int u = threadIdx.x; u < RB * dh; u += blockDim.x) {
        const int jr = u >> 7, dd = u & 127;
        if (jr < nrows) {
          const int gr = slot_sh[jr], br = gr / N, ir = gr - br * N;
          vc[((size_t)br * H + hh) * n_pad * dh + vc_index(ir, dd, dh)] = vbuf[jr][dd];
        }
      }
    }
    __syncthreads();
  }
}

// ---- launchers ---------------------------------------------------------------------------------
static inline bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

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
  if (dtype == SL_BF16 && d % 8 == 0 && d <= 8 * kRowThreads * kMaxChunks && al16(emb) && al16(gain) && al16(x) && al16(h)) {
    DISPATCH_TILED(tiled, hipLaunchKernelGGL((embed_rmsnorm_vec_kernel<TL>), dim3(m_upper), dim3(kRowThreads), 0, s,
                                             (const bf16_t*)emb, tokens, active_idx, m_dev, m_upper, d, vocab,
                                             (const bf16_t*)gain, eps, (bf16_t*)x, (bf16_t*)h));
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((embed_rmsnorm_kernel<T, TL>), dim3(m_upper),
                                                             dim3(kRowThreads), 0, s, (const T*)emb, tokens,
                                                             active_idx, m_dev, m_upper, d, vocab, (const T*)gain,
                                                             eps, (T*)x, (T*)h)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

constexpr int kWaveRowsMin = 2048;     // the wave-per-row norm kernel from this many rows on (see add_rmsnorm_wave_kernel)
int slk_add_rmsnorm(hipStream_t s, int dtype, void* x, const float* delta, int S, size_t sstride,
                    const int32_t* m_dev, int m_upper, int d, const void* gain, float eps, void* h, int tiled) {
  if (m_upper <= 0) return SL_OK;
  if (dtype == SL_BF16 && d == 4096 && m_upper >= kWaveRowsMin && sstride % 4 == 0 && al16(x) && al16(delta) && al16(gain) &&
      al16(h)) {
    DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_wave_kernel<true, TL, 8>), dim3(sl_cdiv(m_upper, 4)), dim3(256), 0, s,
                                             (bf16_t*)x, delta, S, sstride, m_dev, m_upper, (const bf16_t*)gain, eps,
                                             (bf16_t*)h));
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  if (dtype == SL_BF16 && d % 8 == 0 && d <= 8 * kRowThreads * kMaxChunks && sstride % 4 == 0 && al16(x) && al16(delta) &&
      al16(gain) && al16(h)) {
    DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_vec_kernel<true, TL>), dim3(m_upper), dim3(kRowThreads), 0, s,
                                             (bf16_t*)x, delta, S, sstride, m_dev, m_upper, d, (const bf16_t*)gain,
                                             eps, (bf16_t*)h));
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_kernel<T, true, TL>), dim3(m_upper),
                                                             dim3(kRowThreads), 0, s, (T*)x, delta, S, sstride,
                                                             m_dev, m_upper, d, (const T*)gain, eps, (T*)h)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_rmsnorm(hipStream_t s, int dtype, const void* x, const int32_t* m_dev, int m_upper, int d, const void* gain,
                float eps, void* h, int tiled) {
  if (m_upper <= 0) return SL_OK;
  if (dtype == SL_BF16 && d == 4096 && m_upper >= kWaveRowsMin && al16(x) && al16(gain) && al16(h)) {
    DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_wave_kernel<false, TL, 8>), dim3(sl_cdiv(m_upper, 4)), dim3(256), 0,
                                             s, (bf16_t*)const_cast<void*>(x), (const float*)nullptr, 1, (size_t)0, m_dev,
                                             m_upper, (const bf16_t*)gain, eps, (bf16_t*)h));
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  if (dtype == SL_BF16 && d % 8 == 0 && d <= 8 * kRowThreads * kMaxChunks && al16(x) && al16(gain) && al16(h)) {
    DISPATCH_TILED(tiled, hipLaunchKernelGGL((add_rmsnorm_vec_kernel<false, TL>), dim3(m_upper), dim3(kRowThreads), 0, s,
                                             (bf16_t*)const_cast<void*>(x), (const float*)nullptr, 1, (size_t)0, m_dev,
                                             m_upper, d, (const bf16_t*)gain, eps, (bf16_t*)h));
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
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
                      void* vc, int v_half) {
  if (m_upper <= 0) return SL_OK;
  if ((kc == nullptr) != (vc == nullptr)) return SL_EINVAL;
  if (v_half && dtype != SL_BF16) return SL_EINVAL;     // the half container is a 16-bit format
  // kc = vc = null: rotate and store the queries only (the row-per-workgroup kernels skip the cache stores)
  // thin launches are latency-bound (wide accesses, few instructions win); thick ones are bound by the
  // scattered 2-byte V stores, where the element-wise kernel's many threads per row do better
  if ((m_upper <= 256 || kc == nullptr) && dtype == SL_BF16 && dh % 8 == 0 && sstride % 4 == 0 && al16(rope_tab) && al16(qkv) && al16(q) && al16(kc) && al16(vc)) {
    const int per_row = H * (dh / 8), wgs = per_row >= 512 && m_upper <= 256 ? 2 : 1;   // (head, four pairs) items per row
    hipLaunchKernelGGL(v_half ? rope_kv_write_vec_kernel<true> : rope_kv_write_vec_kernel<false>, dim3(m_upper, wgs), dim3(256), 0,
                       s, qkv, S, sstride, active_idx, m_dev, m_upper, H, dh, N, n_pad, (const float2*)rope_tab, (bf16_t*)q,
                       (bf16_t*)kc, (bf16_t*)vc);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  if (kc != nullptr && dtype == SL_BF16 && dh == 128 && sstride % 4 == 0 && N % 16 == 0 && al16(rope_tab) && al16(qkv) && al16(q) && al16(kc) && al16(vc)) {
    const int row_blocks = sl_cdiv(m_upper, 16);
    int hs = 1;                                          // head groups: aim at two workgroups per CU
    while (hs < H && H % (hs * 2) == 0 && row_blocks * hs < 512) hs *= 2;
    hipLaunchKernelGGL(v_half ? rope_kv_write_block_kernel<true> : rope_kv_write_block_kernel<false>, dim3(row_blocks, hs),
                       dim3(256), 0, s, qkv, S, sstride, active_idx, m_dev, m_upper, H, N, n_pad, (const float2*)rope_tab,
                       (bf16_t*)q, (bf16_t*)kc, (bf16_t*)vc);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  if (v_half) {
    hipLaunchKernelGGL((rope_kv_write_kernel<bf16_t, true>), dim3(m_upper), dim3(256), 0, s, qkv, S, sstride, active_idx, m_dev,
                       m_upper, H, dh, N, n_pad, (const float2*)rope_tab, (bf16_t*)q, (bf16_t*)kc, (bf16_t*)vc);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  DISPATCH_T(dtype, hipLaunchKernelGGL((rope_kv_write_kernel<T, false>), dim3(m_upper), dim3(256), 0, s, qkv, S, sstride,
                                       active_idx, m_dev, m_upper, H, dh, N, n_pad, (const float2*)rope_tab, (T*)q, (T*)kc,
                                       (T*)vc));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_swiglu(hipStream_t s, int dtype, const float* gu, int S, size_t sstride, const int32_t* m_dev, int m_upper,
               int dff, void* a, int tiled, int interleaved) {
  if (m_upper <= 0) return SL_OK;
  if (dtype == SL_BF16 && tiled && interleaved && dff % 32 == 0 && sstride % 4 == 0 && al16(gu) && al16(a)) {
    hipLaunchKernelGGL(swiglu_vec_kernel, dim3(sl_cdiv(dff / 8, 256), m_upper), dim3(256), 0, s, gu, S, sstride, m_dev, m_upper,
                       dff, (bf16_t*)a);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  DISPATCH_T(dtype, DISPATCH_TILED(tiled, hipLaunchKernelGGL((swiglu_kernel<T, TL>), dim3(sl_cdiv(dff, 256), m_upper),
                                                             dim3(256), 0, s, gu, S, sstride, m_dev, m_upper, dff,
                                                             interleaved, (T*)a)));
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_kv_read(hipStream_t s, int dtype, const void* kc, const void* vc, int B, int H, int N, int n_pad, int dh,
                void* k_out, void* v_out, int v_half) {
  const size_t total = (size_t)B * N * H * dh;
  if (v_half) {
    if (dtype != SL_BF16) return SL_EINVAL;
    hipLaunchKernelGGL((kv_read_kernel<bf16_t, true>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       (const bf16_t*)kc, (const bf16_t*)vc, B, H, N, n_pad, dh, (bf16_t*)k_out, (bf16_t*)v_out);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  DISPATCH_T(dtype, hipLaunchKernelGGL((kv_read_kernel<T, false>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
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
