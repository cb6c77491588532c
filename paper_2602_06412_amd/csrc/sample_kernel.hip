// Token sampling at temperature tau > 0 (appendix on sampling temperature): the token UpdateMASK
// writes at a still-masked position of the current block is drawn from softmax(z / tau); everything
// the lock test uses stays on the raw posterior.  The draw is the Gumbel-max form
//   argmax_v ( z_v + tau * G_v ),  G_v = -ln(-ln U_v),
// one streaming pass over the row's logits.  U_v comes from the counter-based generator
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), written out here from its published round
// function: word v % 4 of the block with counter (v / 4, flat row id, step, 0) and key = the two
// halves of the seed; U = (2 (x >> 9) + 1) / 2^24 (an odd multiple of 2^-24: exact in fp32, never 0 or 1).
#include "sl_common.h"

__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                     uint32_t (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ inline void load4(const float* p, float (&z)[4]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  z[0] = a.x; z[1] = a.y; z[2] = a.z; z[3] = a.w;
}
__device__ inline void load4(const bf16_t* p, float (&z)[4]) {
  const uint2 a = *reinterpret_cast<const uint2*>(p);
  z[0] = bf16_bits_to_f32(a.x & 0xffffu); z[1] = bf16_bits_to_f32(a.x >> 16);
  z[2] = bf16_bits_to_f32(a.y & 0xffffu); z[3] = bf16_bits_to_f32(a.y >> 16);
}

// A row's V logits are streamed by kSampleParts workgroups (grid.y), each over a contiguous share of the
// Philox blocks; rows that cannot be unmasked at this step (not masked, or outside the block) exit at
// once.  Only a block's worth of rows draws at a step (tens of rows), and the generator's 32 x 32 -> 64
// bit multiplies run at a quarter of the vector rate, so spreading a row over several CUs is what keeps
// the latency down (64 eligible rows at V = 126464: 48 us unsplit with 256 or 1024 threads per row).
// Each part leaves its best (score, id); sample_finish_kernel takes the best part, lowest id on ties.
constexpr int kSampleThreads = 256;
constexpr int kSampleParts = 8;

struct SamplePart { float s; int v; };

template <typename T>
__global__ __launch_bounds__(kSampleThreads) void sample_tokens_kernel(const T* __restrict__ logits, int cur_packed, int V,
                                                                       const int32_t* __restrict__ active_idx,
                                                                       const int32_t* __restrict__ m_dev, int m_upper,
                                                                       const uint8_t* __restrict__ masked, int N, int lo,
                                                                       int hi, float tau, uint32_t seed_lo, uint32_t seed_hi,
                                                                       int t, SamplePart* __restrict__ part) {
  __shared__ float best_s[kSampleThreads / 64];
  __shared__ int best_v[kSampleThreads / 64];
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  const int g = active_idx[r];
  const int i = g % N;
  if (!(masked[g] && i >= lo && i < hi)) return;
  const T* row = logits + (size_t)(cur_packed ? r : g) * V;
  const int nblk = V >> 2;
  const int b0 = (int)((long long)nblk * blockIdx.y / gridDim.y), b1 = (int)((long long)nblk * (blockIdx.y + 1) / gridDim.y);
  float bs = -INFINITY;
  int bv = 0x7fffffff;
  for (int blk = b0 + threadIdx.x; blk < b1; blk += kSampleThreads) {
    uint32_t x[4];
    philox4x32_10((uint32_t)blk, (uint32_t)g, (uint32_t)t, 0u, seed_lo, seed_hi, x);
    float z[4];
    load4(row + 4 * blk, z);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float u = (float)(2u * (x[w] >> 9) + 1u) * 5.9604644775390625e-8f;      // * 2^-24, exact
      // inner log: full accuracy (u close to 1 gives the large G that win draws); outer: the fast one,
      // whose absolute error (~1e-7 |log2|) is what matters for a term added to a logit
      const float s = z[w] + tau * (-__logf(-logf(u)));
      if (s > bs) { bs = s; bv = 4 * blk + w; }          // ascending v within a thread: first maximum kept
    }
  }
  // (value descending, index ascending) over the wave, then over the waves
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float os = __shfl_xor(bs, o, 64);
    const int ov = __shfl_xor(bv, o, 64);
    if (os > bs || (os == bs && ov < bv)) { bs = os; bv = ov; }
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { best_s[w] = bs; best_v[w] = bv; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int j = 1; j < kSampleThreads / 64; ++j)
      if (best_s[j] > bs || (best_s[j] == bs && best_v[j] < bv)) { bs = best_s[j]; bv = best_v[j]; }
    part[(size_t)r * gridDim.y + blockIdx.y] = SamplePart{bs, bv};
  }
}

__global__ void sample_finish_kernel(const int32_t* __restrict__ active_idx, const int32_t* __restrict__ m_dev, int m_upper,
                                     const uint8_t* __restrict__ masked, int N, int lo, int hi, int parts,
                                     const SamplePart* __restrict__ part, const int32_t* __restrict__ argmax,
                                     int32_t* __restrict__ write_id) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= min(*m_dev, m_upper)) return;
  const int g = active_idx[r];
  const int i = g % N;
  int out = argmax[r];
  if (masked[g] && i >= lo && i < hi) {
    float bs = -INFINITY;
    int bv = 0x7fffffff;
    for (int p = 0; p < parts; ++p) {
      const SamplePart q = part[(size_t)r * parts + p];
      if (q.s > bs || (q.s == bs && q.v < bv)) { bs = q.s; bv = q.v; }
    }
    if (bv != 0x7fffffff) out = bv;                      // a row without a comparable score keeps its argmax
  }
  write_id[r] = out;
}

size_t slk_sample_scratch_bytes(int m_upper) { return (size_t)m_upper * kSampleParts * sizeof(SamplePart); }

// scratch: slk_sample_scratch_bytes(m_upper) of device memory
int slk_sample_tokens(hipStream_t s, const void* logits, int cur_packed, int dtype, int V, const int32_t* active_idx,
                      const int32_t* m_dev, int m_upper, const uint8_t* masked, int N, int lo, int hi, float tau,
                      unsigned long long seed, int t, const int32_t* argmax, int32_t* write_id, void* scratch) {
  if (m_upper <= 0) return SL_OK;
  if (V % 4 || !(tau > 0.f) || !scratch || (uintptr_t)scratch % 8 || (uintptr_t)logits % 16) return SL_EINVAL;
  const uint32_t k0 = (uint32_t)(seed & 0xffffffffull), k1 = (uint32_t)(seed >> 32);
  dim3 grid(m_upper, kSampleParts);
  if (dtype == SL_BF16)
    hipLaunchKernelGGL((sample_tokens_kernel<bf16_t>), grid, dim3(kSampleThreads), 0, s, (const bf16_t*)logits, cur_packed,
                       V, active_idx, m_dev, m_upper, masked, N, lo, hi, tau, k0, k1, t, (SamplePart*)scratch);
  else
    hipLaunchKernelGGL((sample_tokens_kernel<float>), grid, dim3(kSampleThreads), 0, s, (const float*)logits, cur_packed, V,
                       active_idx, m_dev, m_upper, masked, N, lo, hi, tau, k0, k1, t, (SamplePart*)scratch);
  SL_LAUNCH_CHECK();
  hipLaunchKernelGGL(sample_finish_kernel, dim3(sl_cdiv(m_upper, 256)), dim3(256), 0, s, active_idx, m_dev, m_upper, masked, N,
                     lo, hi, kSampleParts, (const SamplePart*)scratch, argmax, write_id);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- the same draw for callers that cannot allocate ----------------------------------------------
// The per-part candidates live in a file-scope device array instead of a caller's buffer.  Every
// GPU holds its own copy of the array at its own address; the address is looked up once per device
// (with that device current) and kept.  The array's name is only a host-side handle: device code
// and HIP calls always get the looked-up pointer.
constexpr int kSampleStaticRows = 16384;                       // largest m_upper the static buffer serves (1 MiB)
static __device__ __align__(256) unsigned char scratch[(size_t)kSampleStaticRows * kSampleParts * sizeof(SamplePart)];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];                       // per device; null until first use there

int slk_sample_static_rows() { return kSampleStaticRows; }

// Device address of this device's copy of `scratch` (no allocation: the array is part of the code object).
int slk_sample_static_ptr(void** out) {
  int dev = 0;
  SL_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SL_EINVAL;
  void* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    SL_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SL_EHIP;
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);  // racing first calls store the same address
  }
  *out = p;
  return SL_OK;
}
