// Measurement aids: what this chip sustains on the two resources the rooflines of the step's
// kernels are drawn against, measured with nothing else in the way.
//   mfma_peak_kernel   a bare loop of v_mfma_f32_16x16x32_bf16 (the instruction of the projection
//                      kernels, Sec. 2.4 GEMM terms) on register operands: 16 independent
//                      accumulators per wave, no memory traffic inside the loop
//   stream_peak_kernel a grid-stride pass of 16-byte loads over a buffer, read-only (the access
//                      pattern of the posterior scoring, Alg. 1 'Score on active positions', and of
//                      the thin-M weight streams) or copied to a second buffer
// Both write a small per-thread result so that the work cannot be dropped.
#include "sl_common.h"

typedef __bf16 pk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int pk_u32x4 __attribute__((ext_vector_type(4)));

#define SL_TRY(expr) do { const int rc_ = (expr); if (rc_ != SL_OK) return rc_; } while (0)

constexpr int kPeakThreads = 256;          // 4 waves: one per SIMD of a CU; also the stream kernel's workgroup
constexpr int kPeakMfmaPerIter = 16;
constexpr int kStreamWgPerCu = 8;

// One workgroup per CU, four or eight waves (one or two per SIMD).  The launch bound of 512 keeps the 16
// accumulators in ordinary vector registers: at 256 the compiler moves them to accumulation registers and
// pads the loop with copies between the two files.
__global__ __launch_bounds__(512) void mfma_peak_kernel(const pk_bf16x8* __restrict__ operands, int iters,
                                                        float* __restrict__ sink) {
  // operands: 8 fragments x 64 lanes x 16 bytes, the same for every wave
  const int lane = threadIdx.x & 63;
  pk_bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[i * 64 + lane];
    b[i] = operands[(4 + i) * 64 + lane];
  }
  pk_f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = pk_f32x4{0.f, 0.f, 0.f, 0.f};
  int it = iters;                            // >= 1 (checked on the host)
  do {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  } while (--it > 0);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Each workgroup takes contiguous 16 KiB blocks (four 16-byte loads in flight per thread, 256 B per wave and
// load), workgroup-strided over the buffer.
template <bool COPY>
__global__ __launch_bounds__(kPeakThreads) void stream_peak_kernel(const pk_u32x4* __restrict__ src, pk_u32x4* __restrict__ dst,
                                                                   size_t n16, unsigned int* __restrict__ sink) {
  constexpr size_t kBlock = 4 * kPeakThreads;                 // 16-byte words per workgroup trip
  pk_u32x4 x = pk_u32x4{0u, 0u, 0u, 0u};
  size_t base = (size_t)blockIdx.x * kBlock;
  for (; base + kBlock <= n16; base += (size_t)gridDim.x * kBlock) {
    const size_t i = base + threadIdx.x;
    const pk_u32x4 v0 = __builtin_nontemporal_load(src + i);
    const pk_u32x4 v1 = __builtin_nontemporal_load(src + i + kPeakThreads);
    const pk_u32x4 v2 = __builtin_nontemporal_load(src + i + 2 * kPeakThreads);
    const pk_u32x4 v3 = __builtin_nontemporal_load(src + i + 3 * kPeakThreads);
    if (COPY) {
      __builtin_nontemporal_store(v0, dst + i);
      __builtin_nontemporal_store(v1, dst + i + kPeakThreads);
      __builtin_nontemporal_store(v2, dst + i + 2 * kPeakThreads);
      __builtin_nontemporal_store(v3, dst + i + 3 * kPeakThreads);
    } else {
      x ^= v0 ^ v1 ^ v2 ^ v3;
    }
  }
  // the last, partial block belongs to the workgroup whose turn it would be
  for (size_t i = base + threadIdx.x; i < n16 && base < n16; i += kPeakThreads) {
    const pk_u32x4 v = __builtin_nontemporal_load(src + i);
    if (COPY) __builtin_nontemporal_store(v, dst + i);
    else x ^= v;
  }
  if (!COPY) sink[(size_t)blockIdx.x * kPeakThreads + threadIdx.x] = x[0] ^ x[1] ^ x[2] ^ x[3];
}

static int cu_count(int* out) {
  int dev = 0;
  SL_HIP(hipGetDevice(&dev));
  SL_HIP(hipDeviceGetAttribute(out, hipDeviceAttributeMultiprocessorCount, dev));
  return *out > 0 ? SL_OK : SL_EHIP;
}

extern "C" int sl_peak_probe_mfma(void* stream, const void* operands, size_t operand_bytes, int32_t iters,
                                  int32_t waves_per_simd, float* sink, size_t sink_bytes, int64_t* flops) {
  if (!operands || !sink || !flops || iters < 1 || iters > (1 << 24) || waves_per_simd < 1 || waves_per_simd > 2)
    return SL_EINVAL;
  if ((uintptr_t)operands % 16 || (uintptr_t)sink % 4) return SL_EINVAL;
  if (operand_bytes < (size_t)8 * 64 * 16) return SL_ENOSPC;
  int cus = 0;
  SL_TRY(cu_count(&cus));
  const int threads = kPeakThreads * waves_per_simd;
  if (sink_bytes < (size_t)cus * threads * sizeof(float)) return SL_ENOSPC;
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(cus), dim3(threads), 0, (hipStream_t)stream,
                     (const pk_bf16x8*)operands, (int)iters, sink);
  SL_LAUNCH_CHECK();
  *flops = (int64_t)cus * (threads / 64) * iters * kPeakMfmaPerIter * (2LL * 16 * 16 * 32);
  return SL_OK;
}

extern "C" int sl_peak_probe_stream(void* stream, const void* src, void* dst, size_t bytes, uint32_t* sink,
                                    size_t sink_bytes) {
  if (!src || !sink || bytes < 16 || bytes % 16) return SL_EINVAL;
  if ((uintptr_t)src % 16 || (uintptr_t)dst % 16 || (uintptr_t)sink % 4) return SL_EINVAL;
  if (dst) {                                                   // the two buffers must not overlap
    const uintptr_t a = (uintptr_t)src, b = (uintptr_t)dst;
    if (a < b + bytes && b < a + bytes) return SL_EINVAL;
  }
  int cus = 0;
  SL_TRY(cu_count(&cus));
  const int grid = cus * kStreamWgPerCu;
  if (sink_bytes < (size_t)grid * kPeakThreads * sizeof(uint32_t)) return SL_ENOSPC;
  const size_t n16 = bytes / 16;
  if (dst)
    hipLaunchKernelGGL(stream_peak_kernel<true>, dim3(grid), dim3(kPeakThreads), 0, (hipStream_t)stream,
                       (const pk_u32x4*)src, (pk_u32x4*)dst, n16, sink);
  else
    hipLaunchKernelGGL(stream_peak_kernel<false>, dim3(grid), dim3(kPeakThreads), 0, (hipStream_t)stream,
                       (const pk_u32x4*)src, (pk_u32x4*)nullptr, n16, sink);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
