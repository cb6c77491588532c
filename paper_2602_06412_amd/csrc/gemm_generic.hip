// Shape-generic projection kernel: C[m, n] = sum_k A[m, k] * W[n, k]  (y = x W^T), any m/n/k,
// storage type fp32 or bf16, fp32 FMA accumulation in ascending k.  This is the path of the
// fp32 configuration and of shapes the MFMA kernels do not tile; it is written for
// correctness on every shape, not for speed.
#include "sl_common.h"

constexpr int GT = 64;    // tile edge
constexpr int GK = 16;    // k step

template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T* __restrict__ A, const T* __restrict__ W,
                                                           const int32_t* __restrict__ m_dev, int m_upper, int n,
                                                           int k, float* __restrict__ C_f32, T* __restrict__ C_T,
                                                           const int32_t* __restrict__ out_row_map, size_t ldc) {
  __shared__ float As[GK][GT + 1];
  __shared__ float Ws[GK][GT + 1];
  const int M = min(*m_dev, m_upper);
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  if (m0 >= M) return;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;          // thread owns rows ty*4.., cols tx*4..
  float acc[4][4] = {};
  for (int k0 = 0; k0 < k; k0 += GK) {
    // 64 x 16 elements of each operand, 4 per thread
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int e = tid + it * 256;
      const int row = e >> 4, kk = e & 15;
      const int gm = m0 + row, gn = n0 + row, gk = k0 + kk;
      As[kk][row] = (gm < M && gk < k) ? st<T>::ld(A + (size_t)gm * k + gk) : 0.f;
      Ws[kk][row] = (gn < n && gk < k) ? st<T>::ld(W + (size_t)gn * k + gk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; w[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    const size_t orow = out_row_map ? (size_t)out_row_map[gm] : (size_t)gm;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= n) continue;
      if (C_f32) C_f32[orow * ldc + gn] = acc[i][j];
      else st<T>::stv(C_T + orow * ldc + gn, acc[i][j]);
    }
  }
}

int slk_gemm_generic(hipStream_t s, int dtype, const void* A, const void* W, const int32_t* m_dev, int m_upper, int n,
                     int k, float* C_f32, void* C_T, const int32_t* out_row_map, size_t ldc) {
  if (m_upper <= 0) return SL_OK;
  dim3 grid(sl_cdiv(n, GT), sl_cdiv(m_upper, GT)), block(256);
  if (dtype == SL_BF16)
    hipLaunchKernelGGL((gemm_generic_kernel<bf16_t>), grid, block, 0, s, (const bf16_t*)A, (const bf16_t*)W, m_dev,
                       m_upper, n, k, C_f32, (bf16_t*)C_T, out_row_map, ldc);
  else
    hipLaunchKernelGGL((gemm_generic_kernel<float>), grid, block, 0, s, (const float*)A, (const float*)W, m_dev,
                       m_upper, n, k, C_f32, (float*)C_T, out_row_map, ldc);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
