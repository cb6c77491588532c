// Index-set and mask kernels of the SureLock controller (Alg. 1: the active-set
// line, UpdateMASK, the candidate line and the lock rule).  All integer work; these
// launches move a few KB and are latency-bound, so each is a single small kernel.
#include "sl_common.h"

// ---- A_t = {i | lock_i = 0}: stable stream compaction over the flat [B*N] mask -------
// One 1024-thread block walks the mask in chunks of 1024: wave ballot + popcount gives
// the rank inside a wave, an LDS scan over the 16 wave totals gives the rank inside the
// chunk, a running base carries across chunks.  cu_active[b] is the rank of flat id b*N.
// active_idx holds `cap` entries: ranks beyond it are counted (cu_active stays the true prefix sums, so the
// caller can see the overflow) but not stored.
__global__ __launch_bounds__(1024) void compact_active_kernel(const uint8_t* __restrict__ lock, int B, int N,
                                                              int select_locked, int cap,
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
    const bool act = (g < total) && ((lock[g] != 0) == (select_locked != 0));
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
      if (act && rank < cap) active_idx[rank] = g;
      if (g % N == 0) cu_active[g / N] = rank;
    }
    __syncthreads();
    if (tid == 0) base_sh = base + chunk_tot;
    __syncthreads();
  }
  if (tid == 0) cu_active[B] = base_sh;
}

// select_locked = 0: the unlocked positions (A_t); 1: the locked ones (L_t, the rows the unlock probe visits)
int slk_compact_active(hipStream_t s, const uint8_t* lock, int B, int N, int cap, int32_t* active_idx,
                       int32_t* cu_active, int select_locked) {
  hipLaunchKernelGGL(compact_active_kernel, dim3(1), dim3(1024), 0, s, lock, B, N, select_locked, cap, active_idx,
                     cu_active);
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
__device__ __forceinline__ void unmask_topk_body(int32_t* __restrict__ tokens, uint8_t* masked,
                                                 const int32_t* __restrict__ active_idx,
                                                 const int32_t* __restrict__ cu_active,
                                                 const float* __restrict__ conf,
                                                 const int32_t* __restrict__ argmax, int N, int lo, int hi,
                                                 int k, int m_upper) {
  extern __shared__ unsigned long long keys[];     // [hi - lo]
  __shared__ int count;
  __shared__ int hist[256];
  __shared__ unsigned long long prefix_sh;
  __shared__ int want_sh, done_sh;
  __shared__ int wave_tot[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  // packed arrays hold m_upper rows: rows beyond the caller's bound do not exist
  const int r0 = min(cu_active[b], m_upper), r1 = min(cu_active[b + 1], m_upper);
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

__global__ __launch_bounds__(256) void unmask_topk_kernel(int32_t* __restrict__ tokens, uint8_t* __restrict__ masked,
                                                          const int32_t* __restrict__ active_idx,
                                                          const int32_t* __restrict__ cu_active,
                                                          const float* __restrict__ conf,
                                                          const int32_t* __restrict__ argmax, int N, int lo, int hi,
                                                          int k, int m_upper) {
  unmask_topk_body(tokens, masked, active_idx, cu_active, conf, argmax, N, lo, hi, k, m_upper);
}

// UpdateMASK followed by the candidates + lock rule of the same sequence in one launch (the order of Alg. 1):
// one workgroup per sequence unmasks its top k, then decides its own active rows on the updated flags and
// carries its already-locked positions over.  A sequence's rule reads only that sequence's flags, which
// this workgroup itself has just written (visible after the barrier).  Same decisions as
// unmask_topk_kernel + lock_rule_kernel; new_lock may alias lock.
__global__ __launch_bounds__(256) void unmask_lock_kernel(int32_t* __restrict__ tokens, uint8_t* masked,
                                                          const int32_t* __restrict__ active_idx,
                                                          const int32_t* __restrict__ cu_active,
                                                          const float* __restrict__ conf,
                                                          const int32_t* __restrict__ argmax, int N, int lo, int hi,
                                                          int k, int m_upper, const uint8_t* lock,
                                                          const float* __restrict__ kl, const float* __restrict__ eps,
                                                          int first_step, uint8_t* new_lock) {
  unmask_topk_body(tokens, masked, active_idx, cu_active, conf, argmax, N, lo, hi, k, m_upper);
  __threadfence_block();
  __syncthreads();
  const int b = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < N; i += 256)
    if (lock[(size_t)b * N + i]) new_lock[(size_t)b * N + i] = 1;
  const int r0 = min(cu_active[b], m_upper), r1 = min(cu_active[b + 1], m_upper);
  const float e = eps[b];
  for (int r = r0 + tid; r < r1; r += 256) {
    const int g = active_idx[r];
    const bool F = !first_step && masked[g] == 0 && kl[r] <= e;
    new_lock[g] = F ? 1 : 0;
  }
}

int slk_unmask_lock(hipStream_t s, int32_t* tokens, uint8_t* masked, const int32_t* active_idx,
                    const int32_t* cu_active, const float* conf, const int32_t* argmax, int B, int N, int lo, int hi,
                    int k, int m_upper, const uint8_t* lock, const float* kl, const float* eps, int first_step,
                    uint8_t* new_lock) {
  if (hi <= lo || k <= 0 || m_upper <= 0) return SL_EINVAL;      // nothing to unmask: the caller runs the rule alone
  const size_t sh = (size_t)(hi - lo) * 8;
  hipLaunchKernelGGL(unmask_lock_kernel, dim3(B), dim3(256), sh, s, tokens, masked, active_idx, cu_active, conf,
                     argmax, N, lo, hi, k, m_upper, lock, kl, eps, first_step, new_lock);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_unmask_topk(hipStream_t s, int32_t* tokens, uint8_t* masked, const int32_t* active_idx,
                    const int32_t* cu_active, const float* conf, const int32_t* argmax, int B, int N, int lo, int hi,
                    int k, int m_upper) {
  if (hi <= lo || k <= 0 || m_upper <= 0) return SL_OK;
  const size_t sh = (size_t)(hi - lo) * 8;
  hipLaunchKernelGGL(unmask_topk_kernel, dim3(B), dim3(256), sh, s, tokens, masked, active_idx, cu_active, conf,
                     argmax, N, lo, hi, k, m_upper);
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

// ---- nearest-rank selection over non-negative floats held in LDS as their bit patterns --------
// The rank-th smallest of keys[0..n) (1 <= rank <= n) by a 4-pass radix select: thread b owns bin b,
// a shuffle prefix sum over the histogram tells it how many keys sit in lower bins, exactly one thread
// finds the wanted rank in its bin.  exact = false may stop early and return an upper bound of the
// value that no larger key reaches (enough for "key <= result" tests on the keys themselves);
// exact = true returns the value itself.  Called by all 256 threads of the workgroup.
struct SelectShared {
  int hist[256];
  int wave_tot[4];
  int want, done;
  unsigned int prefix;
};

__device__ static unsigned int select_rank_smallest(const unsigned int* keys, int n, int rank, bool exact,
                                                    SelectShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __syncthreads();
  if (tid == 0) { sh.prefix = 0; sh.want = rank; sh.done = 0; }
  for (int shift = 24; shift >= 0; shift -= 8) {
    sh.hist[tid] = 0;
    __syncthreads();
    const unsigned int prefix = sh.prefix;
    const int want = sh.want;
    const unsigned int himask = shift == 24 ? 0u : (~0u << (shift + 8));
    for (int e = tid; e < n; e += 256) {
      const unsigned int key = keys[e];
      if ((key & himask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 0xff], 1);
    }
    __syncthreads();
    const int c = sh.hist[tid];
    int incl = c;                                // keys in bins 64*wave .. tid
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_up(incl, o, 64);
      if (lane >= o) incl += y;
    }
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += sh.wave_tot[w];      // keys in bins <= tid
    const int below = incl - c;
    if (below < want && want <= incl) {
      sh.prefix = prefix | ((unsigned int)tid << shift);
      sh.want = want - below;
      // everything in this bin is still wanted: the bin's largest possible key is a valid bound and
      // the remaining bytes need not be examined
      if (!exact && want - below == c) {
        sh.prefix = prefix | ((unsigned int)tid << shift) | (shift ? ((1u << shift) - 1u) : 0u);
        sh.done = 1;
      }
    }
    __syncthreads();
    if (sh.done) break;
  }
  return sh.prefix;
}

__device__ static inline int nearest_rank(double m, int n) {
  int rank = (int)ceil(m * (double)n / 100.0);
  return rank < 1 ? 1 : (rank > n ? n : rank);
}

// ---- lock rule with the confidence gate and the re-lock state -------------------------------------
// One workgroup per sequence.  Gate (gate_m > 0): the candidates' u = max(0, 1 - conf) (non-negative
// floats, whose bit patterns order like the values) are collected in LDS, theta_b = their nearest-rank
// percentile, F_t = {u <= theta and D <= eps}.  Re-lock state (relocked != null; optional unlocking):
// a position unlocked before needs D <= rho * eps and cannot lock while t <= cool_until.  t_lock, if
// given, receives t at the positions locked by this call.
struct RelockArgs {
  const uint8_t* relocked;
  const int32_t* cool_until;
  float rho;
  int t;
  int32_t* t_lock;
};

__global__ __launch_bounds__(256) void lock_rule_gated_kernel(const uint8_t* lock, const uint8_t* __restrict__ masked,
                                                              const int32_t* __restrict__ active_idx,
                                                              const int32_t* __restrict__ cu_active, int m_upper,
                                                              const float* __restrict__ kl,
                                                              const float* __restrict__ conf,
                                                              const float* __restrict__ eps, double gate_m, int N,
                                                              int first_step, uint8_t* new_lock, RelockArgs rs) {
  extern __shared__ unsigned int ukeys[];          // [N]
  __shared__ int count;
  __shared__ SelectShared sel;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int r0 = min(cu_active[b], m_upper), r1 = min(cu_active[b + 1], m_upper);
  // positions locked before stay locked (threads beyond the row range take no part in the rest)
  for (int p = tid; p < N; p += 256)
    if (lock[(size_t)b * N + p]) new_lock[(size_t)b * N + p] = 1;
  if (tid == 0) count = 0;
  __syncthreads();
  const bool gate = gate_m > 0.0;
  if (!first_step && gate) {
    for (int r = r0 + tid; r < r1; r += 256) {
      if (masked[active_idx[r]] == 0) {
        const int slot = atomicAdd(&count, 1);
        ukeys[slot] = __float_as_uint(fmaxf(0.f, 1.0f - conf[r]));
      }
    }
  }
  __syncthreads();
  const int n = count;
  unsigned int theta = gate ? 0u : 0xffffffffu;
  if (n > 0) theta = select_rank_smallest(ukeys, n, nearest_rank(gate_m, n), false, sel);
  for (int r = r0 + tid; r < r1; r += 256) {
    const int g = active_idx[r];
    bool F = false;
    if (!first_step && masked[g] == 0) {
      float e = eps[b];
      bool cooled = true;
      if (rs.relocked != nullptr) {
        if (rs.relocked[g]) e = rs.rho * e;
        cooled = rs.t > rs.cool_until[g];
      }
      F = cooled && __float_as_uint(fmaxf(0.f, 1.0f - conf[r])) <= theta && kl[r] <= e;
    }
    new_lock[g] = F ? 1 : 0;
    if (F && rs.t_lock != nullptr) rs.t_lock[g] = rs.t;
  }
}

int slk_lock_rule_gated(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                        const int32_t* cu_active, int m_upper, const float* kl, const float* conf, const float* eps,
                        float gate_m, int B, int N, int first_step, uint8_t* new_lock) {
  if ((size_t)N * 4 > 60 * 1024) return SL_EINVAL;
  hipLaunchKernelGGL(lock_rule_gated_kernel, dim3(B), dim3(256), (size_t)N * 4, s, lock, masked, active_idx, cu_active,
                     m_upper, kl, conf, eps, (double)gate_m, N, first_step, new_lock,
                     RelockArgs{nullptr, nullptr, 1.f, 0, nullptr});
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// gate_m <= 0: no gate
int slk_lock_rule_relock(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const int32_t* active_idx,
                         const int32_t* cu_active, int m_upper, const float* kl, const float* conf, const float* eps,
                         float gate_m, const uint8_t* relocked, const int32_t* cool_until, float rho, int t, int B,
                         int N, uint8_t* new_lock, int32_t* t_lock) {
  if ((size_t)N * 4 > 60 * 1024) return SL_EINVAL;
  hipLaunchKernelGGL(lock_rule_gated_kernel, dim3(B), dim3(256), (size_t)N * 4, s, lock, masked, active_idx, cu_active,
                     m_upper, kl, conf, eps, (double)gate_m, N, t == 1 ? 1 : 0, new_lock,
                     RelockArgs{relocked, cool_until, rho, t, t_lock});
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- the unlock rule (optional unlocking): one workgroup per sequence -------------------------------
// theta_b = nearest-rank percentile of u = max(0, 1 - conf) over ALL active rows of the sequence (exact
// value: the probed rows compared with it are not among the keys); a probed locked position g unlocks iff
//   u~ > theta  and  D~ > eps_unlock  and  t - t_lock[g] > d_interval.
// An unlocked position gets lock = 0, relocked = 1, cool_until = t + d_cool; unlocked[r] flags the row.
__global__ __launch_bounds__(256) void unlock_rule_kernel(uint8_t* lock, uint8_t* relocked, int32_t* cool_until,
                                                          const int32_t* __restrict__ t_lock,
                                                          const int32_t* __restrict__ probe_idx,
                                                          const int32_t* __restrict__ cu_probe, int mp_upper,
                                                          const float* __restrict__ kl_probe,
                                                          const float* __restrict__ conf_probe,
                                                          const int32_t* __restrict__ cu_active, int ma_upper,
                                                          const float* __restrict__ conf_active, double m,
                                                          float eps_unlock, int t, int d_interval, int d_cool,
                                                          uint8_t* __restrict__ unlocked) {
  extern __shared__ unsigned int ukeys[];          // [N]
  __shared__ SelectShared sel;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int a0 = min(cu_active[b], ma_upper), a1 = min(cu_active[b + 1], ma_upper);
  const int n = a1 - a0;
  for (int r = tid; r < n; r += 256) ukeys[r] = __float_as_uint(fmaxf(0.f, 1.0f - conf_active[a0 + r]));
  __syncthreads();
  unsigned int theta = 0;
  if (n > 0) theta = select_rank_smallest(ukeys, n, nearest_rank(m, n), true, sel);
  const int p0 = min(cu_probe[b], mp_upper), p1 = min(cu_probe[b + 1], mp_upper);
  for (int r = p0 + tid; r < p1; r += 256) {
    const int g = probe_idx[r];
    const unsigned int uk = __float_as_uint(fmaxf(0.f, 1.0f - conf_probe[r]));
    const bool un = (n == 0 || uk > theta) && kl_probe[r] > eps_unlock && t - t_lock[g] > d_interval;
    unlocked[r] = un ? 1 : 0;
    if (un) {
      lock[g] = 0;
      relocked[g] = 1;
      cool_until[g] = t + d_cool;
    }
  }
}

int slk_unlock_rule(hipStream_t s, uint8_t* lock, uint8_t* relocked, int32_t* cool_until, const int32_t* t_lock,
                    const int32_t* probe_idx, const int32_t* cu_probe, int mp_upper, const float* kl_probe,
                    const float* conf_probe, const int32_t* cu_active, int ma_upper, const float* conf_active, float m,
                    float eps_unlock, int t, int d_interval, int d_cool, int B, int N, uint8_t* unlocked) {
  if ((size_t)N * 4 > 60 * 1024) return SL_EINVAL;
  hipLaunchKernelGGL(unlock_rule_kernel, dim3(B), dim3(256), (size_t)N * 4, s, lock, relocked, cool_until, t_lock,
                     probe_idx, cu_probe, mp_upper, kl_probe, conf_probe, cu_active, ma_upper, conf_active, (double)m,
                     eps_unlock, t, d_interval, d_cool, unlocked);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- where a probed row's kept posterior lies ---------------------------------------------------------
// The posterior store holds two buffers of buf_rows rows each; the step taken at time t writes buffer
// t & 1, so a position locked at t* keeps p_{t*} in buffer t* & 1.  prev_rows[r] = that row's index
// counted from the start of the first buffer.
__global__ void probe_prev_rows_kernel(const int32_t* __restrict__ probe_idx, const int32_t* __restrict__ m_dev,
                                       int m_upper, const int32_t* __restrict__ t_lock, int buf_rows,
                                       int32_t* __restrict__ prev_rows) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= min(*m_dev, m_upper)) return;
  const int g = probe_idx[r];
  prev_rows[r] = (t_lock[g] & 1) * buf_rows + g;
}

int slk_probe_prev_rows(hipStream_t s, const int32_t* probe_idx, const int32_t* m_dev, int m_upper,
                        const int32_t* t_lock, int buf_rows, int32_t* prev_rows) {
  if (m_upper <= 0) return SL_OK;
  hipLaunchKernelGGL(probe_prev_rows_kernel, dim3(sl_cdiv(m_upper, 256)), dim3(256), 0, s, probe_idx, m_dev, m_upper,
                     t_lock, buf_rows, prev_rows);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- carrying p_{t*} of an unlocked position to where step t + 1 looks for p_t -----------------------
// Step t + 1 reads the previous posterior from buffer t & 1.  A position unlocked at t whose kept row
// lies in the other buffer (t_lock and t of different parity) has it copied across; 16-byte units.
__global__ __launch_bounds__(256) void posterior_carry_kernel(uint4* __restrict__ store, size_t buf_units,
                                                              size_t row_units,
                                                              const int32_t* __restrict__ probe_idx,
                                                              const int32_t* __restrict__ m_dev, int m_upper,
                                                              const int32_t* __restrict__ t_lock,
                                                              const uint8_t* __restrict__ unlocked, int t) {
  const int r = blockIdx.x;
  if (r >= min(*m_dev, m_upper) || !unlocked[r]) return;
  const int g = probe_idx[r];
  const int from = t_lock[g] & 1, to = t & 1;
  if (from == to) return;
  const uint4* src = store + from * buf_units + (size_t)g * row_units;
  uint4* dst = store + to * buf_units + (size_t)g * row_units;
  for (size_t e = (size_t)blockIdx.y * 256 + threadIdx.x; e < row_units; e += (size_t)gridDim.y * 256) dst[e] = src[e];
}

int slk_posterior_carry(hipStream_t s, void* store, size_t buf_bytes, size_t row_bytes, const int32_t* probe_idx,
                        const int32_t* m_dev, int m_upper, const int32_t* t_lock, const uint8_t* unlocked, int t) {
  if (m_upper <= 0) return SL_OK;
  if (row_bytes % 16 || buf_bytes % 16 || (uintptr_t)store % 16) return SL_EINVAL;
  const int chunks = (int)((row_bytes / 16 + 2047) / 2048);
  hipLaunchKernelGGL(posterior_carry_kernel, dim3(m_upper, chunks > 0 ? chunks : 1), dim3(256), 0, s, (uint4*)store,
                     buf_bytes / 16, row_bytes / 16, probe_idx, m_dev, m_upper, t_lock, unlocked, t);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- selection on top of the lock mask (Exp-5, combined setting): which non-locked rows to compute ----
// One workgroup per sequence.  Of the n non-locked positions, ceil(k n) are computed: the still-masked
// positions of the current block always, the rest of the budget by decreasing d_last (the KL a position
// scored when last computed; non-negative floats order like their bit patterns), ties to the lower
// position.  Keys (d_last bits << 32) | ~position are distinct; the (budget - #must)-th largest is found by
// an 8-pass radix select in LDS.  compute_mask[g] = 0 for the rows to compute, 1 for locked and skipped ones.
struct Select64Shared {
  int hist[256];
  int wave_tot[4];
  int want, done;
  unsigned long long prefix;
};

// the k-th largest of n distinct keys (1 <= k <= n), or a lower bound of it that no smaller key reaches
__device__ static unsigned long long select_kth_largest(const unsigned long long* keys, int n, int k,
                                                        Select64Shared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __syncthreads();
  if (tid == 0) { sh.prefix = 0; sh.want = k; sh.done = 0; }
  for (int shift = 56; shift >= 0; shift -= 8) {
    sh.hist[tid] = 0;
    __syncthreads();
    const unsigned long long prefix = sh.prefix;
    const int want = sh.want;
    const unsigned long long himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
    for (int e = tid; e < n; e += 256) {
      const unsigned long long key = keys[e];
      if ((key & himask) == prefix) atomicAdd(&sh.hist[(int)((key >> shift) & 0xff)], 1);
    }
    __syncthreads();
    const int c = sh.hist[tid];
    int incl = c;                                // keys in bins tid .. 64*wave+63
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int y = __shfl_down(incl, o, 64);
      if (lane + o < 64) incl += y;
    }
    if (lane == 0) sh.wave_tot[wave] = incl;
    __syncthreads();
    for (int w = wave + 1; w < 4; ++w) incl += sh.wave_tot[w];      // keys in bins >= tid
    const int above = incl - c;                  // keys in bins > tid
    if (above < want && want <= incl) {
      sh.prefix = prefix | ((unsigned long long)tid << shift);
      sh.want = want - above;
      if (want - above == c) sh.done = 1;          // the whole bin is wanted: its lowest possible key will do
    }
    __syncthreads();
    if (sh.done) break;
  }
  return sh.prefix;
}

__global__ __launch_bounds__(256) void select_rows_kernel(const uint8_t* __restrict__ lock,
                                                          const uint8_t* __restrict__ masked,
                                                          const float* __restrict__ d_last, int N, int lo, int hi,
                                                          double k_frac, uint8_t* __restrict__ compute_mask) {
  extern __shared__ unsigned long long skeys[];    // [N]
  __shared__ int n_active, n_must, count;
  __shared__ Select64Shared sel;
  const int b = blockIdx.x, tid = threadIdx.x;
  if (tid == 0) { n_active = 0; n_must = 0; count = 0; }
  __syncthreads();
  for (int p = tid; p < N; p += 256) {
    const size_t g = (size_t)b * N + p;
    if (lock[g]) { compute_mask[g] = 1; continue; }
    atomicAdd(&n_active, 1);
    if (masked[g] && p >= lo && p < hi) {
      compute_mask[g] = 0;
      atomicAdd(&n_must, 1);
    } else {
      const int slot = atomicAdd(&count, 1);
      skeys[slot] = ((unsigned long long)__float_as_uint(d_last[g]) << 32) | (unsigned)(~(unsigned)p);
    }
  }
  __syncthreads();
  const int n = n_active, cnt = count;
  int budget = (int)ceil(k_frac * (double)n);
  budget = budget > n ? n : budget;
  const int want = budget - n_must;
  unsigned long long thresh = 0;                   // want >= cnt: every other row is computed too
  bool none = want <= 0;
  if (!none && want < cnt) thresh = select_kth_largest(skeys, cnt, want, sel);
  for (int e = tid; e < cnt; e += 256) {
    const unsigned long long key = skeys[e];
    const unsigned p = ~(unsigned)(key & 0xffffffffu);
    compute_mask[(size_t)b * N + p] = (!none && key >= thresh) ? 0 : 1;
  }
}

int slk_select_rows(hipStream_t s, const uint8_t* lock, const uint8_t* masked, const float* d_last, int B, int N,
                    int lo, int hi, float k_frac, uint8_t* compute_mask) {
  if ((size_t)N * 8 > 60 * 1024) return SL_EINVAL;
  hipLaunchKernelGGL(select_rows_kernel, dim3(B), dim3(256), (size_t)N * 8, s, lock, masked, d_last, N, lo, hi,
                     (double)k_frac, compute_mask);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// A skipped position (not locked, not computed at step t) has its newest posterior row copied from the
// buffer step t - 1 wrote to the one step t writes, so that the next step that computes it finds the
// posterior of the step it was last computed at where every step looks for p_{t-1}.  16-byte units.
__global__ __launch_bounds__(256) void posterior_carry_skipped_kernel(uint4* __restrict__ store, size_t buf_units,
                                                                      size_t row_units,
                                                                      const uint8_t* __restrict__ lock,
                                                                      const uint8_t* __restrict__ compute_mask,
                                                                      int total, int t) {
  const int g = blockIdx.x;
  if (g >= total || lock[g] || !compute_mask[g]) return;
  const uint4* src = store + (size_t)((t - 1) & 1) * buf_units + (size_t)g * row_units;
  uint4* dst = store + (size_t)(t & 1) * buf_units + (size_t)g * row_units;
  for (size_t e = (size_t)blockIdx.y * 256 + threadIdx.x; e < row_units; e += (size_t)gridDim.y * 256) dst[e] = src[e];
}

int slk_posterior_carry_skipped(hipStream_t s, void* store, size_t buf_bytes, size_t row_bytes, const uint8_t* lock,
                                const uint8_t* compute_mask, int total, int t) {
  if (total <= 0 || t < 2) return SL_OK;
  if (row_bytes % 16 || buf_bytes % 16 || (uintptr_t)store % 16) return SL_EINVAL;
  const int chunks = (int)((row_bytes / 16 + 2047) / 2048);
  hipLaunchKernelGGL(posterior_carry_skipped_kernel, dim3(total, chunks > 0 ? chunks : 1), dim3(256), 0, s,
                     (uint4*)store, buf_bytes / 16, row_bytes / 16, lock, compute_mask, total, t);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// d_last[active_idx[r]] = kl[r] for the computed rows
__global__ void scatter_rows_f32_kernel(const int32_t* __restrict__ active_idx, const int32_t* __restrict__ m_dev,
                                        int m_upper, const float* __restrict__ src, float* __restrict__ dst) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < min(*m_dev, m_upper)) dst[active_idx[r]] = src[r];
}

int slk_scatter_rows_f32(hipStream_t s, const int32_t* active_idx, const int32_t* m_dev, int m_upper, const float* src,
                         float* dst) {
  if (m_upper <= 0) return SL_OK;
  hipLaunchKernelGGL(scatter_rows_f32_kernel, dim3(sl_cdiv(m_upper, 256)), dim3(256), 0, s, active_idx, m_dev, m_upper,
                     src, dst);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
