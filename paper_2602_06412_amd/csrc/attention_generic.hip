// Shape-generic bidirectional attention for the active rows (Alg. 1 'attention' line; Sec. 2.1):
// o[r, h] = softmax(q[r, h] . K[b, h, 0..N)^T / sqrt(d_h)) V[b, h, 0..N), no mask, all N slots of
// the row's own sequence (cached and live alike).  One workgroup per (row, head); fp32
// throughout.  Correctness path for the fp32 configuration and for head sizes other than 128.
#include "sl_common.h"

template <typename T>
__global__ __launch_bounds__(256) void attention_generic_kernel(const T* __restrict__ q, const T* __restrict__ kc,
                                                                const T* __restrict__ vc,
                                                                const int32_t* __restrict__ active_idx,
                                                                const int32_t* __restrict__ m_dev, int m_upper, int H,
                                                                int dh, int N, int n_pad, T* __restrict__ o) {
  extern __shared__ float smem[];
  float* qs = smem;              // [dh]
  float* sc = smem + dh;         // [n_pad] scores / probabilities
  float* part = sc + n_pad;      // [256] partial outputs
  __shared__ float red[4];
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x, hh = blockIdx.y;
  if (r >= M) return;
  const int tid = threadIdx.x;
  const int g = active_idx[r];
  const int b = g / N;
  const size_t head_base = ((size_t)b * H + hh) * n_pad * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int c = tid; c < dh; c += 256) qs[c] = st<T>::ld(q + ((size_t)r * H + hh) * dh + c);
  __syncthreads();
  float lmax = -INFINITY;
  for (int n = tid; n < N; n += 256) {
    float s = 0.f;
    for (int c = 0; c < dh; ++c) s = fmaf(qs[c], st<T>::ld(kc + head_base + kc_index(n, c, dh)), s);
    s *= scale;
    sc[n] = s;
    lmax = fmaxf(lmax, s);
  }
  const float mx = block_max<256>(lmax, red);
  float lsum = 0.f;
  for (int n = tid; n < N; n += 256) {
    const float p = expf(sc[n] - mx);
    sc[n] = p;
    lsum += p;
  }
  const float tot = block_sum<256>(lsum, red);   // also orders the sc[] writes before the reads below
  const int G = 256 / dh;                        // thread groups splitting the slots
  const int grp = tid / dh, c = tid - grp * dh;
  float acc = 0.f;
  if (grp < G) {
    for (int n = grp; n < N; n += G) acc = fmaf(sc[n], st<T>::ld(vc + head_base + vc_index(n, c, dh)), acc);
  }
  part[tid] = acc;
  __syncthreads();
  if (tid < dh) {
    float v = 0.f;
    for (int gg = 0; gg < G; ++gg) v += part[gg * dh + tid];
    st<T>::stv(o + ((size_t)r * H + hh) * dh + tid, v / tot);
  }
}

int slk_attention_generic(hipStream_t s, int dtype, const void* q, const void* kc, const void* vc,
                          const int32_t* active_idx, const int32_t* m_dev, int m_upper, int H, int dh, int N,
                          int n_pad, void* o) {
  if (m_upper <= 0) return SL_OK;
  if (!(dh == 32 || dh == 64 || dh == 128 || dh == 256)) return SL_EINVAL;
  const size_t sh = (size_t)(dh + n_pad + 256) * sizeof(float);
  if (sh > 64 * 1024) return SL_EINVAL;
  dim3 grid(m_upper, H), block(256);
  if (dtype == SL_BF16)
    hipLaunchKernelGGL((attention_generic_kernel<bf16_t>), grid, block, sh, s, (const bf16_t*)q, (const bf16_t*)kc,
                       (const bf16_t*)vc, active_idx, m_dev, m_upper, H, dh, N, n_pad, (bf16_t*)o);
  else
    hipLaunchKernelGGL((attention_generic_kernel<float>), grid, block, sh, s, (const float*)q, (const float*)kc,
                       (const float*)vc, active_idx, m_dev, m_upper, H, dh, N, n_pad, (float*)o);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
