// Index-set and mask kernels of the SureLock controller (Alg. 1: the active-set
// line, UpdateMASK, the candidate line and the lock rule).  All integer work; these
// launches move a few KB and are latency-bound, so each is a single small kernel.
#include "sl_common.h"

// ---- A_t = {i | lock_i = 0}: stable stream compaction over the flat [B*N] mask -------
// One 1024-thread block walks the mask in chunks of 1024: wave ballot + popcount gives
// the rank inside a wave, an LDS scan over the 16 wave totals gives the rank inside the
// chunk, a running base carries across chunks.  cu_active[b] is the rank of flat id b*N.
__global__ __launch_bounds__(1024) void compact_active_kernel(const uint8_t* __restrict__ lock, int B, int N,
                                                              int32_t* __restrict__ active_idx,
                                                              int32_t* __restrict__ cu_active) {
  __shared__ int wave_tot[16];
  __shared__ int base_sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int total = B * N;
  if (tid == 0) base_sh = 0;
  __syncthreads();
  for (int start = 0; start < total; start += 1024) {
    const int g = start + tid;
    const bool act = (g < total) && (lock[g] == 0);
    const unsigned long long bal = __ballot(act);
    const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(bal);
    __syncthreads();
    int before = 0, chunk_tot = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int c = wave_tot[w];
      before += (w < wave) ? c : 0;
      chunk_tot += c;
    }
    const int base = base_sh;
    const int rank = base + before + in_wave;
    if (g < total) {
      if (act) active_idx[rank] = g;
      if (g % N == 0) cu_active[g / N] = rank;
    }
    __syncthreads();
    if (tid == 0) base_sh = base + chunk_tot;
    __syncthreads();
  }
  if (tid == 0) cu_active[B] = base_sh;
}

int slk_compact_active(hipStream_t s, const uint8_t* lock, int B, int N, int32_t* active_idx, int32_t* cu_active) {
  hipLaunchKernelGGL(compact_active_kernel, dim3(1), dim3(1024), 0, s, lock, B, N, active_idx, cu_active);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- UpdateMASK: top-k by confidence inside the current block, one workgroup per sequence --
// Every eligible row gets the 64-bit key (conf bits << 32) | ~row: keys are distinct, a larger
// key means more confident, and among equal confidences the lower position (= lower packed
// row) wins.  The k-th largest key (or a lower bound of it that no unwanted key reaches) is
// found by an 8-bit-per-pass radix select over LDS histograms; rows whose key reaches it are
// unmasked.  Confidences are probabilities
// (non-negative floats), whose bit patterns order like the values.
__global__ __launch_bounds__(256) void unmask_topk_kernel(int32_t* __restrict__ tokens, uint8_t* __restrict__ masked,
                                                          const int32_t* __restrict__ active_idx,
                                                          const int32_t* __restrict__ cu_active,
                                                          const float* __restrict__ conf,
                                                          const int32_t* __restrict__ argmax, int N, int lo, int hi,
                                                          int k) {
  extern __shared__ unsigned long long keys[];     // [hi - lo]
  __shared__ int count;
  __shared__ int hist[256];
  __shared__ unsigned long long prefix_sh;
  __shared__ int want_sh, done_sh;
  __shared__ int wave_tot[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int r0 = cu_active[b], r1 = cu_active[b + 1];
  if (tid == 0) count = 0;
  __syncthreads();
  for (int r = r0 + tid; r < r1; r += 256) {
    const int g = active_idx[r];
    const int i = g - b * N;
    if (i >= lo && i < hi && masked[g]) {
      const int slot = atomicAdd(&count, 1);
      keys[slot] = ((unsigned long long)__float_as_uint(conf[r]) << 32) | (unsigned)(~(unsigned)r);
    }
  }
  __syncthreads();
  const int n = count;
  if (n == 0) return;
  unsigned long long thresh = 0;                   // k >= n: everything eligible is taken
  if (k < n) {
    // radix select of the k-th largest key, most significant byte first.  Thread b owns bin b:
    // a suffix sum over the histogram (wave shuffles + the four wave totals) tells each thread
    // how many keys sit in higher bins; exactly one thread finds the k-th largest in its bin.
    // Once a bin holds exactly the keys still wanted, every key in it qualifies and the
    // remaining bytes need not be examined.
    const int lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { prefix_sh = 0; want_sh = k; done_sh = 0; }
    for (int shift = 56; shift >= 0; shift -= 8) {
      hist[tid] = 0;
      __syncthreads();
      const unsigned long long prefix = prefix_sh;
      const int want = want_sh;
      const unsigned long long himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
      for (int e = tid; e < n; e += 256) {
        const unsigned long long key = keys[e];
        if ((key & himask) == prefix) atomicAdd(&hist[(int)((key >> shift) & 0xff)], 1);
      }
      __syncthreads();
      const int c = hist[tid];
      int incl = c;                                // keys in bins tid .. 64*wave+63
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += y;
      }
      if (lane == 0) wave_tot[wave] = incl;
      __syncthreads();
      for (int w = wave + 1; w < 4; ++w) incl += wave_tot[w];      // keys in bins >= tid
      const int above = incl - c;                  // keys in bins > tid
      if (above < want && want <= incl) {
        prefix_sh = prefix | ((unsigned long long)tid << shift);
        want_sh = want - above;
        if (want - above == c) done_sh = 1;
      }
      __syncthreads();
      if (done_sh) break;
    }
    thresh = prefix_sh;
  }
  for (int e = tid; e < n; e += 256) {
    const unsigned long long key = keys[e];
    if (key >= thresh) {
      const int r = (int)(~(unsigned)(key & 0xffffffffu));
      const int g = active_idx[r];
      tokens[g] = argmax[r];
      masked[g] = 0;
    }
  }
}

int slk_unmask_topk(hipStream_t s, int32_t* tokens, uint8_t* masked, const int32_t* active_idx,
                    const int32_t* cu_active, const float* conf, const int32_t* argmax, int B, int N, int lo, int hi,
                    int k) {
  if (hi <= lo || k <= 0) return SL_OK;
  const size_t sh = (size_t)(hi - lo) * 8;
  hipLaunchKernelGGL(unmask_topk_kernel, dim3(B), dim3(256), sh, s, tokens, masked, active_idx, cu_active, conf,
                     argmax, N, lo, hi, k);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- candidates and lock rule: Z_t = active & unmasked, F_t = {i in Z_t : D_i <= eps_b} ------
// Thread p < B*N carries an already-locked position over; thread r < M decides row r.
// The two roles write disjoint positions, so new_lock may alias lock.
__global__ void lock_rule_kernel(const uint8_t* lock, const uint8_t* __restrict__ masked,
                                 const int32_t* __restrict__ active_idx, const int32_t* __restrict__ m_dev,
                                 int m_upper, const float* __restrict__ kl, const float* __restrict__ eps, int total,
                                 int N, int first_step, uint8_t* new_lock) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int M = min(*m_dev, m_upper);
  if (t < total && lock[t]) new_lock[t] = 1;
  if (t < M) {
    const int g = active_idx[t];
    const bool F = !first_step && masked[g] == 0 && kl[t] <= eps[g / N];
    new_lock[g] = F ? 1 : 0;
  }
}

int slk_lock_rule(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                  const int32_t* m_dev, int m_upper, const float* kl, const float* eps, int B, int N, int first_step,
                  uint8_t* new_lock) {
  const int total = B * N;
  const int n = total > m_upper ? total : m_upper;
  hipLaunchKernelGGL(lock_rule_kernel, dim3(sl_cdiv(n, 256)), dim3(256), 0, s, lock, masked, active_idx, m_dev,
                     m_upper, kl, eps, total, N, first_step, new_lock);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- lock rule with the confidence gate: theta_b = nearest-rank percentile of u over Z_t -----
// One workgroup per sequence.  The candidates' u = max(0, 1 - conf) (non-negative floats, whose bit
// patterns order like the values) are collected in LDS; the rank-th smallest is found by a 4-pass
// radix select (thread b owns bin b, shuffle prefix sums); then F_t = {u <= theta and D <= eps}.
__global__ __launch_bounds__(256) void lock_rule_gated_kernel(const uint8_t* lock, const uint8_t* __restrict__ masked,
                                                              const int32_t* __restrict__ active_idx,
                                                              const int32_t* __restrict__ cu_active, int m_upper,
                                                              const float* __restrict__ kl,
                                                              const float* __restrict__ conf,
                                                              const float* __restrict__ eps, double gate_m, int N,
                                                              int first_step, uint8_t* new_lock) {
  extern __shared__ unsigned int ukeys[];          // [N]
  __shared__ int count, want_sh, done_sh;
  __shared__ unsigned int prefix_sh;
  __shared__ int hist[256];
  __shared__ int wave_tot[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r0 = min(cu_active[b], m_upper), r1 = min(cu_active[b + 1], m_upper);
  // positions locked before stay locked (threads beyond the row range take no part in the rest)
  for (int p = tid; p < N; p += 256)
    if (lock[(size_t)b * N + p]) new_lock[(size_t)b * N + p] = 1;
  if (tid == 0) count = 0;
  __syncthreads();
  if (!first_step) {
    for (int r = r0 + tid; r < r1; r += 256) {
      if (masked[active_idx[r]] == 0) {
        const int slot = atomicAdd(&count, 1);
        ukeys[slot] = __float_as_uint(fmaxf(0.f, 1.0f - conf[r]));
      }
    }
  }
  __syncthreads();
  const int n = count;
  unsigned int theta = 0;
  if (n > 0) {
    int rank = (int)ceil(gate_m * (double)n / 100.0);
    rank = rank < 1 ? 1 : (rank > n ? n : rank);
    if (tid == 0) { prefix_sh = 0; want_sh = rank; done_sh = 0; }
    for (int shift = 24; shift >= 0; shift -= 8) {
      hist[tid] = 0;
      __syncthreads();
      const unsigned int prefix = prefix_sh;
      const int want = want_sh;
      const unsigned int himask = shift == 24 ? 0u : (~0u << (shift + 8));
      for (int e = tid; e < n; e += 256) {
        const unsigned int key = ukeys[e];
        if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 0xff], 1);
      }
      __syncthreads();
      const int c = hist[tid];
      int incl = c;                                // keys in bins 64*wave .. tid
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
      }
      if (lane == 63) wave_tot[wave] = incl;
      __syncthreads();
      for (int w = 0; w < wave; ++w) incl += wave_tot[w];      // keys in bins <= tid
      const int below = incl - c;
      if (below < want && want <= incl) {
        // everything in this bin that is still wanted: if that is the whole bin, the bin's largest
        // possible key is a valid threshold and the remaining bytes need not be examined
        prefix_sh = prefix | ((unsigned int)tid << shift);
        want_sh = want - below;
        if (want - below == c) { prefix_sh = prefix | ((unsigned int)tid << shift) | (shift ? ((1u << shift) - 1u) : 0u); done_sh = 1; }
      }
      __syncthreads();
      if (done_sh) break;
    }
    theta = prefix_sh;
  }
  for (int r = r0 + tid; r < r1; r += 256) {
    const int g = active_idx[r];
    bool F = false;
    if (!first_step && masked[g] == 0)
      F = __float_as_uint(fmaxf(0.f, 1.0f - conf[r])) <= theta && kl[r] <= eps[b];
    new_lock[g] = F ? 1 : 0;
  }
}

int slk_lock_rule_gated(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                        const int32_t* cu_active, int m_upper, const float* kl, const float* conf, const float* eps,
                        float gate_m, int B, int N, int first_step, uint8_t* new_lock) {
  if ((size_t)N * 4 > 60 * 1024) return SL_EINVAL;
  hipLaunchKernelGGL(lock_rule_gated_kernel, dim3(B), dim3(256), (size_t)N * 4, s, lock, masked, active_idx, cu_active,
                     m_upper, kl, conf, eps, (double)gate_m, N, first_step, new_lock);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
