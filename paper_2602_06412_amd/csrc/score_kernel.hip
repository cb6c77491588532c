// Posterior scoring (Alg. 1 'Score on active positions'; Sec. 2.2): one streaming pass
// over the current and the previous logits row of every active position gives
//   D    = KL(p_t || p_{t-1})           (nats)
//   conf = max_v p_t(v)                  (u = 1 - conf)
//   argmax_v p_t(v)                      (lowest id on ties)
// HBM-bound: each row pair is read exactly once with 16-byte loads, nothing is written
// but three scalars per row.
//
// Arithmetic.  With a = z_t(v), b = z_{t-1}(v) and any common shift m,
//   S  = sum e^{a-m},   dS = sum (e^{b-m} - e^{a-m}),   W = sum e^{a-m} (a - b)
//   KL = sum p_t (log p_t - log p_{t-1}) = W/S + log(1 + dS/S).
// a - b is exact in fp32 for bf16 inputs, and both dS and W are sums of terms that vanish
// with a - b, so the result keeps its relative accuracy when successive posteriors are
// close (the regime the lock test works in) instead of cancelling two O(1) logsumexps.
// The shift m is a running maximum over both rows, raised chunk by chunk (online
// rescaling), so one pass suffices for any vocabulary size.
#include "sl_common.h"

struct ScoreAcc {
  float m, S, Sc, dS, W, bestv;   // Sc: compensation term of S (S + Sc is the sum)
  int besti;
};

__device__ inline void acc_merge(ScoreAcc& x, const ScoreAcc& y) {
  const float m = fmaxf(x.m, y.m);
  const float fx = (x.m == m) ? 1.f : __expf(x.m - m);
  const float fy = (y.m == m) ? 1.f : __expf(y.m - m);
  x.S = (x.S + x.Sc) * fx + (y.S + y.Sc) * fy;
  x.Sc = 0.f;
  x.dS = x.dS * fx + y.dS * fy;
  x.W = x.W * fx + y.W * fy;
  x.m = m;
  if (y.bestv > x.bestv || (y.bestv == x.bestv && y.besti < x.besti)) {
    x.bestv = y.bestv;
    x.besti = y.besti;
  }
}

// 16-byte chunks: `raw` is what a load leaves in registers, unpack() turns it into E floats.
// The loads are streaming (non-temporal): both posterior buffers are read exactly once per step,
// and keeping them out of the caches measured 99 -> 89 us at M = 1024.
typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
typedef float f32x4_nt __attribute__((ext_vector_type(4)));
template <typename T> struct chunk_io;
template <> struct chunk_io<bf16_t> {
  typedef uint4 raw;
  __device__ static inline raw load_raw(const bf16_t* p) {
    const u32x4_nt t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
  }
  __device__ static inline void unpack(const raw& u, float (&v)[8]) {
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
    v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xffff0000u);
    v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xffff0000u);
  }
};
template <> struct chunk_io<float> {
  typedef float4 raw;
  __device__ static inline raw load_raw(const float* p) {
    const f32x4_nt t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_nt*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
  }
  __device__ static inline void unpack(const raw& u, float (&v)[4]) { v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w; }
};


// NT threads per row: 256 when there are rows enough to fill the chip, 1024 for thin launches
// (a row is ~0.5 MB of loads; a single small workgroup would be latency-bound on it).
template <typename T, bool FIRST, int NT>
__global__ __launch_bounds__(NT) void score_kernel(const T* __restrict__ cur, int cur_packed,
                                                               const T* __restrict__ prev, int V,
                                                               const int32_t* __restrict__ active_idx,
                                                               const int32_t* __restrict__ m_dev, int m_upper,
                                                               float* __restrict__ kl, float* __restrict__ conf,
                                                               int32_t* __restrict__ argmax, int parts,
                                                               ScoreAcc* __restrict__ partial) {
  constexpr int E = st<T>::kVec;
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x;
  if (r >= M) return;
  const int g = active_idx[r];
  const T* a_row = cur + (size_t)(cur_packed ? r : g) * V;
  const T* b_row = prev + (size_t)g * V;
  ScoreAcc acc{-INFINITY, 0.f, 0.f, 0.f, 0.f, -INFINITY, 0x7fffffff};
  // blockIdx.y = which of `parts` equal shares of the row this workgroup streams
  const int c_lo = (int)((long long)(V / E) * blockIdx.y / parts);
  const int n_chunks = (int)((long long)(V / E) * (blockIdx.y + 1) / parts);
  // Exponentials are taken in base 2 (one fma + v_exp per term): e^{a-m} = 2^{a L - m L}, L = log2 e.
  // The same expression serves both rows, so equal logits give exactly equal terms and KL(p||p) = 0.
  constexpr float L2E = 1.4426950408889634f;
  auto consume = [&](const float (&a)[E], const float (&b)[E], int c) {
    float amax = a[0];
#pragma unroll
    for (int j = 1; j < E; ++j) amax = fmaxf(amax, a[j]);
    float cm = amax;
    if (!FIRST) {
#pragma unroll
      for (int j = 0; j < E; ++j) cm = fmaxf(cm, b[j]);
    }
    if (cm > acc.m) {
      const float f = __expf(acc.m - cm);      // 0 on the first chunk (acc.m = -inf)
      acc.S *= f; acc.Sc *= f; acc.dS *= f; acc.W *= f;
      acc.m = cm;
    }
    if (amax > acc.bestv) {                     // rare after the first chunks; first (lowest) index wins ties
      int jb = E - 1;
#pragma unroll
      for (int j = E - 2; j >= 0; --j) jb = (a[j] == amax) ? j : jb;
      acc.bestv = amax;
      acc.besti = c * E + jb;
    }
    const float m2 = -acc.m * L2E;
    float cs = 0.f;                             // this chunk's share of S
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float ea = __builtin_amdgcn_exp2f(fmaf(a[j], L2E, m2));
      cs += ea;
      if (!FIRST) {
        const float eb = __builtin_amdgcn_exp2f(fmaf(b[j], L2E, m2));
        acc.dS += eb - ea;
        acc.W = fmaf(ea, a[j] - b[j], acc.W);
      }
    }
    // S += cs with an error-free two-sum: once a dominant term (e^0 = 1) is in S, plain
    // adds of the many ~1e-8 terms of a peaked posterior would be rounded away
    const float t = acc.S + cs;
    const float bp = t - acc.S;
    acc.Sc += (acc.S - (t - bp)) + (cs - bp);
    acc.S = t;
  };
  // two chunks per trip so that four 16-byte loads are in flight per thread (issuing the next
  // trip's loads ahead of the arithmetic as well was measured and gained nothing)
  typedef typename chunk_io<T>::raw Raw;
  auto eat = [&](const Raw& ra, const Raw& rb, int c) {
    float a[E], b[E];
    chunk_io<T>::unpack(ra, a);
    chunk_io<T>::unpack(FIRST ? ra : rb, b);
    consume(a, b, c);
  };
  int c = c_lo + threadIdx.x;
  for (; c + NT < n_chunks; c += 2 * NT) {
    const Raw a0 = chunk_io<T>::load_raw(a_row + (size_t)c * E);
    const Raw a1 = chunk_io<T>::load_raw(a_row + (size_t)(c + NT) * E);
    const Raw b0 = FIRST ? a0 : chunk_io<T>::load_raw(b_row + (size_t)c * E);
    const Raw b1 = FIRST ? a1 : chunk_io<T>::load_raw(b_row + (size_t)(c + NT) * E);
    eat(a0, b0, c);
    eat(a1, b1, c + NT);
  }
  if (c < n_chunks) {
    const Raw ra = chunk_io<T>::load_raw(a_row + (size_t)c * E);
    const Raw rb = FIRST ? ra : chunk_io<T>::load_raw(b_row + (size_t)c * E);
    eat(ra, rb, c);
  }
  // wave reduction, then across the block's waves through LDS
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ScoreAcc y;
    y.m = __shfl_xor(acc.m, o, 64); y.S = __shfl_xor(acc.S, o, 64); y.Sc = __shfl_xor(acc.Sc, o, 64); y.dS = __shfl_xor(acc.dS, o, 64);
    y.W = __shfl_xor(acc.W, o, 64); y.bestv = __shfl_xor(acc.bestv, o, 64); y.besti = __shfl_xor(acc.besti, o, 64);
    acc_merge(acc, y);
  }
  __shared__ ScoreAcc sh[NT / 64];
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    ScoreAcc t = sh[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) acc_merge(t, sh[w]);
    t.S += t.Sc;
    t.Sc = 0.f;
    if (parts > 1) {                             // score_merge_kernel finishes the row
      partial[(size_t)r * parts + blockIdx.y] = t;
      return;
    }
    conf[r] = __expf(t.bestv - t.m) / t.S;
    argmax[r] = t.besti < V ? t.besti : 0;     // a row without any comparable logit (all NaN) still yields a valid id
    kl[r] = FIRST ? INFINITY : fmaxf(0.f, t.W / t.S + log1pf(t.dS / t.S));
  }
}

// Thin launches: a row is ~0.5 MB, and with fewer rows than CUs one workgroup per row leaves
// most of the chip idle.  Each row is then streamed by `parts` workgroups and this kernel merges
// their partial states in part order (one thread per row).
template <bool FIRST>
__global__ void score_merge_kernel(const ScoreAcc* __restrict__ partial, int parts, const int32_t* __restrict__ m_dev,
                                   int m_upper, int V, float* __restrict__ kl, float* __restrict__ conf,
                                   int32_t* __restrict__ argmax) {
  const int M = min(*m_dev, m_upper);
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= M) return;
  ScoreAcc t = partial[(size_t)r * parts];
  for (int q = 1; q < parts; ++q) acc_merge(t, partial[(size_t)r * parts + q]);
  conf[r] = __expf(t.bestv - t.m) / t.S;
  argmax[r] = t.besti < V ? t.besti : 0;
  kl[r] = FIRST ? INFINITY : fmaxf(0.f, t.W / t.S + log1pf(t.dS / t.S));
}

template <typename T, int NT>
static int launch_score_nt(hipStream_t s, const void* cur, int cur_packed, const void* prev, int V,
                           const int32_t* active_idx, const int32_t* m_dev, int m_upper, int first_step, float* kl,
                           float* conf, int32_t* argmax, int parts, ScoreAcc* partial) {
  dim3 grid(m_upper, parts), block(NT);
  if (first_step)
    hipLaunchKernelGGL((score_kernel<T, true, NT>), grid, block, 0, s, (const T*)cur, cur_packed, (const T*)cur, V,
                       active_idx, m_dev, m_upper, kl, conf, argmax, parts, partial);
  else
    hipLaunchKernelGGL((score_kernel<T, false, NT>), grid, block, 0, s, (const T*)cur, cur_packed, (const T*)prev, V,
                       active_idx, m_dev, m_upper, kl, conf, argmax, parts, partial);
  SL_LAUNCH_CHECK();
  if (parts > 1) {
    if (first_step)
      hipLaunchKernelGGL(score_merge_kernel<true>, dim3(sl_cdiv(m_upper, 64)), dim3(64), 0, s, partial, parts, m_dev,
                         m_upper, V, kl, conf, argmax);
    else
      hipLaunchKernelGGL(score_merge_kernel<false>, dim3(sl_cdiv(m_upper, 64)), dim3(64), 0, s, partial, parts, m_dev,
                         m_upper, V, kl, conf, argmax);
    SL_LAUNCH_CHECK();
  }
  return SL_OK;
}

// Rows per launch at or below which a row is split (needs the caller's scratch), and how far.
int slk_score_parts(int m_upper, int V) {
  if (m_upper > 128 || V < 65536) return 1;
  int parts = sl_cdiv(512, m_upper);
  return parts > 16 ? 16 : parts;
}
size_t slk_score_scratch_bytes() { return (size_t)128 * 16 * sizeof(ScoreAcc); }

template <typename T>
static int launch_score(hipStream_t s, const void* cur, int cur_packed, const void* prev, int V,
                        const int32_t* active_idx, const int32_t* m_dev, int m_upper, int first_step, float* kl,
                        float* conf, int32_t* argmax, void* scratch) {
  if (m_upper <= 0) return SL_OK;
  const int parts = scratch ? slk_score_parts(m_upper, V) : 1;
  if (parts > 1)
    return launch_score_nt<T, 256>(s, cur, cur_packed, prev, V, active_idx, m_dev, m_upper, first_step, kl, conf,
                                   argmax, parts, (ScoreAcc*)scratch);
  if (m_upper <= 512 && V >= 16384)
    return launch_score_nt<T, 1024>(s, cur, cur_packed, prev, V, active_idx, m_dev, m_upper, first_step, kl, conf,
                                    argmax, 1, nullptr);
  return launch_score_nt<T, 256>(s, cur, cur_packed, prev, V, active_idx, m_dev, m_upper, first_step, kl, conf, argmax,
                                 1, nullptr);
}

// scratch: slk_score_scratch_bytes() of device memory, or null (rows are then never split)
int slk_score(hipStream_t s, const void* cur, int cur_packed, const void* prev, int dtype, int V,
              const int32_t* active_idx, const int32_t* m_dev, int m_upper, int first_step, float* kl, float* conf,
              int32_t* argmax, void* scratch) {
  if (dtype == SL_BF16)
    return launch_score<bf16_t>(s, cur, cur_packed, prev, V, active_idx, m_dev, m_upper, first_step, kl, conf, argmax,
                                scratch);
  return launch_score<float>(s, cur, cur_packed, prev, V, active_idx, m_dev, m_upper, first_step, kl, conf, argmax,
                             scratch);
}
