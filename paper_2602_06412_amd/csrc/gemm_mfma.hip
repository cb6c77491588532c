// M-row projection GEMMs on the MFMA units (gfx950, bf16 in / fp32 accumulate):
//   C[m, n] = sum_k A[m, k] * W[n, k],   m = active rows only (Alg. 1 'main projections',
//   Out projection, FFN, LM head; the GEMM terms of the algorithmic-FLOP count, Sec. 2.4).
//
// Design for thin, shrinking M (the paper's 'thin slices' regime):
//  * The weight matrix is pre-tiled once into MFMA B-operand fragments
//    [n/32][k/16][64 lanes][8 bf16], so a wavefront streams its weight slab with fully
//    coalesced 1 KiB reads straight into registers; weights never pass through LDS and
//    every weight byte is read by exactly one wavefront per M-tile.
//  * A workgroup is 4 wavefronts that share one BM x 64 activation tile in LDS (stored in
//    A-operand fragment order, so LDS reads are conflict-free 16-byte accesses) and own
//    disjoint 32*WNB-column slices: block tile BM x (128*WNB), BM in {32, 64, 128, 256} picked from
//    the launch's row bound.
//  * k can be split across workgroups (grid.y) so that small-M launches still put >= 2
//    workgroups on every CU while the weights stream once; partial sums go to fp32
//    [split][row][n] and the consumer kernel adds them in a fixed order (deterministic).
//  * Workgroup ids are mapped so that all M-tiles of one weight slab run back to back on
//    the same XCD (ids are dealt round-robin over the 8 XCDs), i.e. re-reads hit that L2.
#include "sl_common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;      // k per LDS tile = 4 MFMA k-steps of 16

typedef bf16x8 Frag;        // one lane's 16-byte share of an MFMA operand fragment

// ---- weight pre-tiling -------------------------------------------------------------------
// One thread moves one 16-byte chunk W[nrow][k8*8 .. k8*8+7] to its fragment slot.
__global__ void pack_weight_kernel(const bf16_t* __restrict__ W, int n, int k, bf16_t* __restrict__ P, int nb_off,
                                   int nb_stride) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int k8n = k / 8;
  if (t >= (size_t)n * k8n) return;
  const int row = t / k8n, k8 = t - (size_t)row * k8n;
  const int nb = (row / 32) * nb_stride + nb_off, kb = k8 / 2;
  const int lane = (row & 31) + 32 * (k8 & 1);
  const uint4 v = *reinterpret_cast<const uint4*>(W + (size_t)row * k + (size_t)k8 * 8);
  reinterpret_cast<uint4*>(P)[((size_t)nb * (k / 16) + kb) * 64 + lane] = v;
}

// 32-row block j of W becomes column block j * nb_stride + nb_off of the packed matrix (several
// matrices can share one packed matrix side by side or interleaved).
int slk_pack_weight(hipStream_t s, const void* W, int n, int k, void* P, int nb_off, int nb_stride) {
  const size_t chunks = (size_t)n * (k / 8);
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, (const bf16_t*)W, n,
                     k, (bf16_t*)P, nb_off, nb_stride);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- the kernel ----------------------------------------------------------------------------
// OUT = 0: fp32 partials Cf[split][row][n] (ldc = n, split stride = m_upper * n)
// OUT = 1: bf16 rows Cb[row_map ? row_map[row] : row][n] (no split-k)
template <int BM, int WNB, int OUT>
__global__ __launch_bounds__(256, (BM <= 128 ? 2 : 1)) void gemm_mfma_kernel(
    const bf16_t* __restrict__ A, int a_tiled, const bf16_t* __restrict__ Wp, int n, int k, int k_per_split,
    const int32_t* __restrict__ m_dev, int m_upper, float* __restrict__ Cf, bf16_t* __restrict__ Cb,
    const int32_t* __restrict__ row_map, size_t ldc, int tiles_m, int tiles_n) {
  constexpr int MB = BM / 32;          // 32-row blocks per tile
  constexpr int BN = 128 * WNB;
  constexpr int NF = MB;               // A fragments each wave fetches per k-tile (MB*4 / 4 waves)
  // Two LDS stages as separate arrays, so the compiler can tell which stage an in-flight
  // direct-to-LDS load targets and does not make reads of the other stage wait for it.
  __shared__ Frag stage0[MB * 4 * 64];
  __shared__ Frag stage1[MB * 4 * 64];

  const int M = min(*m_dev, m_upper);
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int tn = (j / tiles_m) * 8 + xcd, tm = j % tiles_m;
  if (tn >= tiles_n) return;
  const int m0 = tm * BM;
  if (m0 >= M) return;
  const int n0 = tn * BN;
  const int kbeg = blockIdx.y * k_per_split;
  const int ktiles = k_per_split / BK;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int K16 = k / 16, NB32 = n / 32;

  // Per-lane 32-bit offsets from wave-uniform bases keep the address registers few.
  const Frag* Wf = reinterpret_cast<const Frag*>(Wp) + (size_t)(kbeg / 16) * 64;
  uint32_t b_off[WNB];
#pragma unroll
  for (int i = 0; i < WNB; ++i) {
    int nb = n0 / 32 + wave * WNB + i;
    nb = nb < NB32 ? nb : NB32 - 1;                      // column tail: load something valid, never stored
    b_off[i] = (uint32_t)nb * (uint32_t)K16 * 64u + (uint32_t)lane;
  }
  // Activation fragments go global -> LDS directly (no register staging): the hardware puts
  // lane L's 16 bytes at (wave-uniform LDS base) + 16*L, which is the fragment order.
  // A is row-major [m_upper, k] (a 32 x 16 fragment is gathered from 32 rows) or already
  // fragment-tiled (one contiguous 1 KiB block per fragment).
  const bf16_t* Ab = a_tiled ? A : A + kbeg;
  const int a_kt_stride = a_tiled ? 4 * 512 : BK;         // elements per k-tile
  uint32_t a_off[NF];
  int a_frag[NF];                                         // fragment index (mb*4 + kb) inside a stage
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const int f = wave + 4 * i, mb = f % MB, kb = f / MB;
    if (a_tiled) {
      int mbg = m0 / 32 + mb;
      const int mb_last = (m_upper + 31) / 32 - 1;
      mbg = mbg < mb_last ? mbg : mb_last;                // row tail: stay inside the (32-row padded) buffer
      a_off[i] = (((uint32_t)mbg * (uint32_t)K16 + (uint32_t)(kbeg / 16 + kb)) * 64u + (uint32_t)lane) * 8u;
    } else {
      int row = m0 + mb * 32 + (lane & 31);
      row = row < m_upper ? row : m_upper - 1;            // row tail: stay inside the buffer
      a_off[i] = (uint32_t)row * (uint32_t)k + (uint32_t)(kb * 16 + (lane >> 5) * 8);
    }
    a_frag[i] = mb * 4 + kb;
  }

  f32x16 acc[MB][WNB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < WNB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  Frag b0[WNB][4], b1[WNB][4];          // weight fragments of the even / odd k-tile (ping-pong, no copies)

  auto load_a = [&](int kt, Frag* stage) {
    const bf16_t* base = Ab + (size_t)kt * a_kt_stride;
#pragma unroll
    for (int i = 0; i < NF; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + a_off[i]),
                                       (__attribute__((address_space(3))) void*)(stage + a_frag[i] * 64), 16, 0, 0);
  };
  auto load_b = [&](int kt, Frag (&b)[WNB][4]) {
    const Frag* base = Wf + kt * 256;
#pragma unroll
    for (int i = 0; i < WNB; ++i)
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) b[i][kb] = __builtin_nontemporal_load(&base[b_off[i] + kb * 64]);   // streamed once
  };
  // One k-tile: A fragments are read one k-step ahead of the MFMAs that use them.
  auto compute = [&](const Frag* stage, const Frag (&b)[WNB][4]) {
    Frag af[2][MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) af[0][mb] = stage[(mb * 4) * 64 + lane];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      if (kb < 3) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) af[(kb + 1) & 1][mb] = stage[(mb * 4 + kb + 1) * 64 + lane];
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < WNB; ++i)
          acc[mb][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kb & 1][mb], b[i][kb], acc[mb][i], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  load_b(0, b0);
  load_a(0, stage0);
#pragma unroll
  for (int i = 0; i < WNB; ++i)
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) asm volatile("" : "+v"(b0[i][kb]));   // pin: loads stay above the wait
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): every load issued so far has landed
  __syncthreads();

  // Two k-tiles per trip (the tile count per split is even).  While tile kt is multiplied out
  // of one LDS stage and one register set, tile kt+1 is in flight towards the other stage /
  // set; the last trip re-fetches the final tile instead of branching (never used).  The
  // direct-to-LDS loads must have landed (vmcnt) before the barrier that publishes them.
  const int last = ktiles - 1;
  for (int kt = 0; kt < ktiles; kt += 2) {
    load_b(kt + 1, b1);
    load_a(kt + 1, stage1);
    compute(stage0, b0);
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): every load issued so far has landed
    __syncthreads();
    const int nk = kt + 2 < ktiles ? kt + 2 : last;
    load_b(nk, b0);
    load_a(nk, stage0);
    compute(stage1, b1);
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): every load issued so far has landed
    __syncthreads();
  }

  // epilogue.  Accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
  const int col_in = lane & 31, row_in = 4 * (lane >> 5);
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = m0 + mb * 32 + 8 * (v / 4) + row_in + (v % 4);
      if (row >= M) continue;
#pragma unroll
      for (int i = 0; i < WNB; ++i) {
        const int col = n0 + (wave * WNB + i) * 32 + col_in;
        if (col >= n) continue;
        if (OUT == 0) {
          Cf[((size_t)blockIdx.y * m_upper + row) * ldc + col] = acc[mb][i][v];
        } else {
          const size_t orow = row_map ? (size_t)row_map[row] : (size_t)row;
          Cb[orow * ldc + col] = (bf16_t)acc[mb][i][v];
        }
      }
    }
  }
}

// Wait until at most N younger loads are outstanding; the asm names the registers of the slot it releases, which
// keeps the MFMAs that read them behind it.
template <int N, int NBW, int MB>
__device__ __forceinline__ void stream_landed(Frag (&b)[NBW], Frag (&a)[MB]) {
  static_assert(N >= 0 && N <= 63, "vmcnt range");
  if constexpr (NBW == 2 && MB == 1)
    asm volatile("s_waitcnt vmcnt(%3)" : "+v"(b[0]), "+v"(b[1]), "+v"(a[0]) : "n"(N));
  else if constexpr (NBW == 2)
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(b[0]), "+v"(b[1]), "+v"(a[0]), "+v"(a[MB - 1]) : "n"(N));
  else if constexpr (MB == 1)
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(b[0]), "+v"(a[0]) : "n"(N));
  else
    asm volatile("s_waitcnt vmcnt(%3)" : "+v"(b[0]), "+v"(a[0]), "+v"(a[MB - 1]) : "n"(N));
}

// ---- thin launches (at most 32 MB rows, MB = 1 or 2): a pure weight stream ---------------------
// Below ~300 rows the projection is bound by reading the weights once (2 n k bytes), so the only
// thing that matters is keeping enough loads in flight.  Here every wave streams its own 64
// columns with no LDS and no barrier: operand fragments go global -> registers, DEPTH k-steps
// (16 deep each) ahead of the MFMAs that consume them, in a register ring the compiler tracks
// load by load (vmcnt(n) waits, never a drain).  The activation fragments (1 KiB per 32 rows and
// k-step) are fetched by all four waves of a workgroup; they are a few hundred KB in total and
// stay in L1/L2, while the weights come from HBM exactly once.
// NBW = 32-column blocks per wave: 2 (workgroup tile 256 columns, 8 k-steps in flight) or 1 (128 columns, 16
// k-steps in flight: the same bytes in flight per wave over twice as many workgroups, for launches whose
// 256-column tiles would leave CUs without a workgroup).
template <int MB, int OUT, int NBW>
__global__ __launch_bounds__(256, 2) void gemm_stream_kernel(
    const bf16_t* __restrict__ A, int a_tiled, const bf16_t* __restrict__ Wp, int n, int k, int k_per_split,
    const int32_t* __restrict__ m_dev, int m_upper, float* __restrict__ Cf, bf16_t* __restrict__ Cb,
    const int32_t* __restrict__ row_map, size_t ldc, int tiles_n) {
  constexpr int DEPTH = 16 / NBW;
  const int M = min(*m_dev, m_upper);
  const int tn = blockIdx.x;
  if (tn >= tiles_n || M <= 0) return;
  const int n0 = tn * 128 * NBW;
  const int kbeg = blockIdx.y * k_per_split;
  const int ksteps = k_per_split / 16;                 // a multiple of DEPTH
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int K16 = k / 16, NB32 = n / 32;

  const Frag* bp[NBW];
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    int nb = n0 / 32 + wave * NBW + i;
    nb = nb < NB32 ? nb : NB32 - 1;                    // column tail: load something valid, never stored
    bp[i] = reinterpret_cast<const Frag*>(Wp) + ((size_t)nb * K16 + kbeg / 16) * 64 + lane;
  }
  // activation fragment of row block mb at k-step s: tiled -> one contiguous 1 KiB block,
  // row-major -> 16 bytes from row (lane % 32), columns 16 s + 8 (lane / 32) ..
  const bf16_t* ap[MB];
  size_t a_step;                                       // elements between consecutive k-steps
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    if (a_tiled) {
      int mbg = mb;
      const int mb_last = (m_upper + 31) / 32 - 1;
      mbg = mbg < mb_last ? mbg : mb_last;
      ap[mb] = A + (((size_t)mbg * K16 + kbeg / 16) * 64 + lane) * 8;
    } else {
      int row = mb * 32 + (lane & 31);
      row = row < m_upper ? row : m_upper - 1;
      ap[mb] = A + (size_t)row * k + kbeg + (lane >> 5) * 8;
    }
  }
  a_step = a_tiled ? 512 : 16;

  f32x16 acc[MB][NBW];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < NBW; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // The loads are issued as inline assembly and waited for with explicit vmcnt counts: left to
  // the compiler, loads that cross the loop's back edge are drained (vmcnt(0)) at the top of
  // every trip, which empties the pipeline DEPTH k-steps at a time.  Loads return in order and
  // each k-step issues NBW + MB of them, so the operands of a step have landed once at most
  // (DEPTH-1)(NBW+MB) younger loads are outstanding (at most 45: the counter holds 63).
  // The weight loads carry the non-temporal hint: every weight byte is used once per launch, and
  // streaming them past the caches measured 191 -> 165 us on the LM head at M = 16 (6.3 TB/s).
  // Register-ring contract.  The compiler cannot see that a register is still being written after the load
  // instruction has issued, so the code must never give it a reason to touch fa / fb between a fetch and the
  // stream_landed that waits for it:
  //  * every fetched slot is consumed (no dummy fetches: a destination the compiler counts as dead may be
  //    handed to another value while the load is still in flight);
  //  * the ring registers are read-write operands ("+v") of both the load and the wait, i.e. one live value
  //    from the first fetch to the last MFMA, never dead, never rematerialised;
  //  * the kernel must not spill (a spill or a copy of a ring register before its wait would read bytes that
  //    have not landed): the build fails if the compiler reports scratch for this kernel.
  Frag fa[DEPTH][MB], fb[DEPTH][NBW];
#pragma unroll
  for (int u = 0; u < DEPTH; ++u) {
#pragma unroll
    for (int i = 0; i < NBW; ++i) fb[u][i] = Frag{};
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) fa[u][mb] = Frag{};
  }
  auto fetch = [&](int step, int slot) {
#pragma unroll
    for (int i = 0; i < NBW; ++i)
      asm volatile("global_load_dwordx4 %0, %1, off nt" : "+v"(fb[slot][i]) : "v"(bp[i] + (size_t)step * 64) : "memory");
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
      asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(fa[slot][mb]) : "v"(ap[mb] + (size_t)step * a_step) : "memory");
  };
#pragma unroll
  for (int u = 0; u < DEPTH; ++u) fetch(u, u);
  auto mfma_step = [&](int u) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int i = 0; i < NBW; ++i)
        acc[mb][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[u][mb], fb[u][i], acc[mb][i], 0, 0, 0);
  };
  // Every trip but the last refills each slot DEPTH steps ahead as soon as its MFMAs are issued.
  for (int s0 = 0; s0 + DEPTH < ksteps; s0 += DEPTH) {
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      stream_landed<(DEPTH - 1) * (NBW + MB), NBW, MB>(fb[u], fa[u]);
      mfma_step(u);
      fetch(s0 + u + DEPTH, u);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // The last trip fetches nothing: slot u has landed once at most DEPTH-1-u younger steps are outstanding, and
  // after its last wait no load is in flight.  (Re-fetching a dummy step here instead, to keep one wait count,
  // left loads in flight into registers the compiler already counted as free: it placed the epilogue's row
  // index in one of them ahead of the final wait, and a late load could overwrite it.)
#define SL_LAST_STEP(U)                                                            \
  if constexpr (U < DEPTH) {                                                       \
    stream_landed<(DEPTH - 1 - U) * (NBW + MB), NBW, MB>(fb[U], fa[U]);            \
    mfma_step(U);                                                                  \
    __builtin_amdgcn_sched_barrier(0);                                             \
  }
  SL_LAST_STEP(0) SL_LAST_STEP(1) SL_LAST_STEP(2) SL_LAST_STEP(3) SL_LAST_STEP(4) SL_LAST_STEP(5) SL_LAST_STEP(6)
  SL_LAST_STEP(7) SL_LAST_STEP(8) SL_LAST_STEP(9) SL_LAST_STEP(10) SL_LAST_STEP(11) SL_LAST_STEP(12)
  SL_LAST_STEP(13) SL_LAST_STEP(14) SL_LAST_STEP(15)
#undef SL_LAST_STEP
  static_assert(DEPTH <= 16, "last trip is written out for 16 slots");

  const int col_in = lane & 31, row_in = 4 * (lane >> 5);
  if constexpr (OUT == 2) {
    // SwiGLU of an unsplit gate|up launch in the epilogue (columns interleaved by 32-column blocks: gate
    // c .. c+31, then up c .. c+31; n = 2 d_ff, ldc = d_ff, Cb = the fragment-tiled activation matrix a).
    // With two blocks per wave a lane holds gate and up of its column; with one, waves 0/1 and 2/3 of the
    // workgroup hold the gate and the up block of a pair, and the up values cross through LDS.
    static_assert(MB == 1, "thin launches only");
    __shared__ float up_sh[NBW == 1 ? 2 * 16 * 64 : 1];
    if constexpr (NBW == 1) {
      if (wave & 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) up_sh[((wave >> 1) * 16 + v) * 64 + lane] = acc[0][0][v];
      }
      __syncthreads();
      if (wave & 1) return;
    }
    const int pair = NBW == 1 ? (n0 >> 6) + (wave >> 1) : (n0 >> 6) + wave;      // which 32 output columns
    const int c = pair * 32 + col_in;
    if (c >= (n >> 1)) return;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = 8 * (v / 4) + row_in + (v % 4);
      if (row >= M) continue;
      const float g = acc[0][0][v];
      const float u = NBW == 1 ? up_sh[((wave >> 1) * 16 + v) * 64 + lane] : acc[0][NBW - 1][v];
      Cb[afrag_index(row, c, (int)ldc)] = (bf16_t)(g / (1.0f + expf(-g)) * u);
    }
    return;
  }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = mb * 32 + 8 * (v / 4) + row_in + (v % 4);
      if (row >= M) continue;
#pragma unroll
      for (int i = 0; i < NBW; ++i) {
        const int col = n0 + (wave * NBW + i) * 32 + col_in;
        if (col >= n) continue;
        if (OUT == 0) {
          Cf[((size_t)blockIdx.y * m_upper + row) * ldc + col] = acc[mb][i][v];
        } else {
          const size_t orow = row_map ? (size_t)row_map[row] : (size_t)row;
          Cb[orow * ldc + col] = (bf16_t)acc[mb][i][v];
        }
      }
    }
  }
}

template <int MB, int OUT, int NBW = 2>
static int launch_stream(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n,
                         int k, int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc) {
  const int tiles_n = sl_cdiv(n, 128 * NBW);
  if ((k / splits) % (16 * (16 / NBW))) return SL_EINVAL;        // whole trips of the register ring
  hipLaunchKernelGGL((gemm_stream_kernel<MB, OUT, NBW>), dim3(tiles_n, splits), dim3(256), 0, s, (const bf16_t*)A,
                     a_tiled, (const bf16_t*)Wp, n, k, k / splits, m_dev, mu, Cf, (bf16_t*)Cb, row_map, ldc, tiles_n);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- host side ------------------------------------------------------------------------------
constexpr int kThinMax = 32;   // launches bounded by at most this many rows take the thin (weight-stream) kernels
static int pick_bm(int mu) { return mu <= 32 ? 32 : mu <= 64 ? 64 : 128; }

// Launch plan for a projection bounded by mu rows: which kernel and how many k-splits.
//  * thin launches (mu <= kThinMax) are weight-stream bound: the k split (and the 128-column tile
//    form) that brings the launch closest to about one workgroup per CU with few fp32 planes, the
//    partial traffic capped at a fraction of the weight bytes (k >= 16*S*mu);
//  * thicker launches take the ring kernel (one workgroup per CU, ~0.8 us per 32-deep k-tile and round
//    of full-height workgroups; its tile height is fitted to the rows by that launcher, whose cost
//    model is shared here) with the split count that minimises  rounds * tile cost * (k-tiles per split
//    + fixed) * t_tile + bytes of fp32 partials written and read back / 5 TB/s; reductions too short
//    for its ring (fewer than 8 k-tiles per split) go to the 128 x 256 LDS kernel (two per CU, ~1.8 us
//    per 64-deep k-tile).
//  The thin limit is 32 rows: from 33 rows on the ring's short tiles are ahead of the two-block
//  weight-stream kernel (whole step at 64 rows 0.39 -> 0.36 ms, at 33 rows 0.365 -> 0.337 ms).
struct GemmPlan {
  int thick256;   // 1: gemm_mfma256_kernel
  int splits;
};
double slk_ring_cost(int mu, int n, int splits);     // gemm_mfma256.hip
// swiglu_consumer: the output is the gate|up pair that SwiGLU consumes; an unsplit launch of the
// ring kernel then writes bf16 activations from its epilogue, every other plan writes fp32
// planes that a second kernel reads back.
// Thin launches: 128-column tiles when 256-column ones would give at most 160 workgroups (and the split's
// reduction is whole trips of the deeper register ring); the workgroup count that results.
static bool thin_narrow(int n, int k, int splits) {
  return sl_cdiv(n, 256) * splits <= 160 && (k / splits) % 256 == 0;
}
static long thin_workgroups(int n, int k, int splits) {
  return (long)sl_cdiv(n, thin_narrow(n, k, splits) ? 128 : 256) * splits;
}

static GemmPlan gemm_plan(int mu, int n, int k, bool swiglu_consumer = false) {
  GemmPlan p{0, 1};
  if (mu <= kThinMax) {
    // Measured at the LLaDA-8B shapes (16 and 32 rows): a weight stream is fastest with about one workgroup
    // per CU (192-256 workgroups: 100 MB in 23-24 us); 96-128 workgroups leave CUs idle (29-36 us) and 384-768
    // are slower again (26-28 us; 201 MB: 44-46 us against 37-39 us), as is every extra fp32 plane.
    int best_s = 1;
    long best_cost = -1;
    for (int s = 1; s <= 16; s *= 2) {
      if (k % (128 * s) || k / s < 256) break;
      if (s > 1 && (size_t)s * 16 * mu > (size_t)k) break;         // fp32 partial traffic capped against the weights
      const long wgs = thin_workgroups(n, k, s);
      const long cost = (wgs > 224 ? wgs - 224 : 224 - wgs) + 4 * s;
      if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_s = s; }
    }
    p.splits = best_s;
    return p;
  }
  // The ring kernel wherever its k loop is long enough (at least 8 k-tiles per split); its half-height
  // variant covers ragged and small row counts.  Measured over ragged row counts at the LLaDA-8B shapes
  // the 128 x 256 LDS kernel never won where the ring was eligible (LM head at 820 rows: 1.19 ms
  // against 0.79 ms), so it is kept for short reductions only.
  double best = 1e30;
  const int t128 = sl_cdiv(mu, 128) * sl_cdiv(n, 256);
  for (int s = 1; s <= 8; s *= 2) {
    if (k % (2 * BK * s)) break;
    if (k / (32 * s) < 8) break;
    const double traffic_us = 2.0 * s * (double)mu * n * 4.0 / 5.0e6 * (s > 1 ? 1.0 : 0.5);
    const double fused_us = (double)mu * n / 5.0e6;      // bf16 activations of half the width, written once
    const double ring_us = slk_ring_cost(mu, n, s) * (k / (32.0 * s) + 4.0) * 0.8;
    const double t = ring_us + (swiglu_consumer && s == 1 ? fused_us : traffic_us);
    if (t < best) { best = t; p.thick256 = 1; p.splits = s; }
  }
  if (p.thick256) return p;
  for (int s = 1; s <= 8; s *= 2) {
    if (k % (2 * BK * s)) break;
    if (k / (BK * s) < 4) break;
    const double traffic_us = 2.0 * s * (double)mu * n * 4.0 / 5.0e6 * (s > 1 ? 1.0 : 0.5);
    const double t = sl_cdiv(t128 * s, 512) * (k / (64.0 * s) + 3.0) * 1.8 + traffic_us;
    if (t < best) { best = t; p.thick256 = 0; p.splits = s; }
  }
  return p;
}

int slk_gemm_splits(int mu, int n, int k) { return gemm_plan(mu, n, k).splits; }
// 1 if the launch plan for (mu, n, k) is the 256 x 256 ring kernel without a k-split (the only
// form whose epilogue can apply SwiGLU to finished sums)
int slk_gemm_unsplit_thick(int mu, int n, int k) {
  if (mu <= kThinMax || k < 256) return 0;
  const GemmPlan p = gemm_plan(mu, n, k, true);
  return p.thick256 && p.splits == 1;
}
// split count of the gate|up projection when it is NOT fused with SwiGLU
int slk_gemm_splits_gate_up(int mu, int n, int k) { return gemm_plan(mu, n, k, true).splits; }

template <int BM, int WNB, int OUT>
static int launch_gemm(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                       int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc) {
  constexpr int BN = 128 * WNB;
  const int tiles_m = sl_cdiv(mu, BM), tiles_n = sl_cdiv(n, BN);
  const size_t sh = 0;
  auto kern = gemm_mfma_kernel<BM, WNB, OUT>;
  dim3 grid(8 * tiles_m * sl_cdiv(tiles_n, 8), splits), block(256);
  hipLaunchKernelGGL(kern, grid, block, sh, s, (const bf16_t*)A, a_tiled, (const bf16_t*)Wp, n, k, k / splits, m_dev, mu, Cf,
                     (bf16_t*)Cb, row_map, ldc, tiles_m, tiles_n);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// Which kernel a launch bounded by mu rows takes (one decision, shared by the launcher and by
// sl_linear_plan): kind 0 = weight-stream kernel (rows = 32 or 64, cols = 128 or 256 per workgroup),
// 1 = ring kernel (rows / tail as its launcher chooses), 2 = 128 x 256 LDS kernel (short reductions).
struct KernelPick { int kind, rows, cols, tail; };
void slk_ring_describe(int mu, int n, int splits, int* rows, int* tail);     // gemm_mfma256.hip
static KernelPick pick_kernel(int mu, int n, int k, int splits, bool f32_out) {
  if (mu > kThinMax && k / splits >= 256) {
    const GemmPlan plan = gemm_plan(mu, n, k);
    const bool use256 = plan.splits == splits ? plan.thick256 != 0 : true;
    if (use256) {
      KernelPick p{1, 256, 256, 0};
      slk_ring_describe(mu, n, splits, &p.rows, &p.tail);
      return p;
    }
  }
  // the barrier-free weight stream with one 32-row block (at most 32 rows) or two (33..64 rows, reached
  // only where the reduction is too short for the ring kernel)
  if (f32_out && mu <= 32 && thin_narrow(n, k, splits)) return KernelPick{0, 32, 128, 0};
  if (mu <= 32 && (k / splits) % 128 == 0) return KernelPick{0, 32, 256, 0};
  if (mu <= 64 && (k / splits) % 128 == 0) return KernelPick{0, 64, 256, 0};
  return KernelPick{2, pick_bm(mu), 256, 0};
}

// Thin unsplit gate|up projection with SwiGLU in its epilogue: a [mu <= 32 rows, dff] bf16, fragment-tiled.
// Returns SL_EINVAL when the plan for this launch is not the unsplit weight-stream kernel (the caller then
// runs the projection into fp32 planes and the SwiGLU kernel).
int slk_gemm_stream_swiglu(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int dff, int k,
                           void* a) {
  const int n = 2 * dff;
  if (mu <= 0 || mu > kThinMax || dff % 32 || k % (2 * BK)) return SL_EINVAL;
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;
  if (gemm_plan(mu, n, k, true).splits != 1) return SL_EINVAL;
  const KernelPick p = pick_kernel(mu, n, k, 1, true);
  if (p.kind != 0 || p.rows != 32) return SL_EINVAL;
  if (p.cols == 128) return launch_stream<1, 2, 1>(s, A, 1, Wp, m_dev, mu, n, k, 1, nullptr, a, nullptr, (size_t)dff);
  return launch_stream<1, 2, 2>(s, A, 1, Wp, m_dev, mu, n, k, 1, nullptr, a, nullptr, (size_t)dff);
}
// 1 if slk_gemm_stream_swiglu takes this launch
int slk_gemm_stream_swiglu_ok(int mu, int dff, int k) {
  const int n = 2 * dff;
  if (mu <= 0 || mu > kThinMax || dff % 32 || k % (2 * BK)) return 0;
  if (gemm_plan(mu, n, k, true).splits != 1) return 0;
  const KernelPick p = pick_kernel(mu, n, k, 1, true);
  return p.kind == 0 && p.rows == 32;
}

// kind / splits / rows / cols / tail of the launch sl_linear_forward(.., splits = 0, y_f32) would make
int slk_gemm_describe(int mu, int n, int k, int* kind, int* splits, int* rows, int* cols, int* tail) {
  const int S = gemm_plan(mu, n, k).splits;
  const KernelPick p = pick_kernel(mu, n, k, S, true);
  *kind = p.kind; *splits = S; *rows = p.rows; *cols = p.cols; *tail = p.tail;
  return SL_OK;
}

// C = A . Wp^T for a launch bounded by mu rows.  Cf != null: fp32 partials [splits][mu][n];
// else bf16 rows into Cb through row_map (splits must be 1).
int slk_gemm_mfma(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                  int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc) {
  if (mu <= 0) return SL_OK;
  if (splits < 1 || n % 32 || k % (2 * BK * splits)) return SL_EINVAL;     // even number of k-tiles per split
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;   // 32-bit offsets
  if (!Cf && splits != 1) return SL_EINVAL;
  const KernelPick p = pick_kernel(mu, n, k, splits, Cf != nullptr);
  if (p.kind == 1) return slk_gemm_mfma256(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc);
  if (p.kind == 0 && p.cols == 128)
    return launch_stream<1, 0, 1>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, nullptr, nullptr, ldc);
  if (p.kind == 0 && p.rows == 32)
    return Cf ? launch_stream<1, 0>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, nullptr, nullptr, ldc)
              : launch_stream<1, 1>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, nullptr, Cb, row_map, ldc);
  if (p.kind == 0)
    return Cf ? launch_stream<2, 0>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, nullptr, nullptr, ldc)
              : launch_stream<2, 1>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, nullptr, Cb, row_map, ldc);
#define GO(BM)                                                                                             \
  return Cf ? launch_gemm<BM, 2, 0>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, nullptr, nullptr, ldc)          \
            : launch_gemm<BM, 2, 1>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, nullptr, Cb, row_map, ldc)
  if (p.rows == 32) { GO(32); }
  if (p.rows == 64) { GO(64); }
  GO(128);
#undef GO
}
