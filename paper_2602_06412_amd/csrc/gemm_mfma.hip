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
__global__ void pack_weight_kernel(const bf16_t* __restrict__ W, int n, int k, bf16_t* __restrict__ P, int nb_off) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int k8n = k / 8;
  if (t >= (size_t)n * k8n) return;
  const int row = t / k8n, k8 = t - (size_t)row * k8n;
  const int nb = row / 32 + nb_off, kb = k8 / 2;
  const int lane = (row & 31) + 32 * (k8 & 1);
  const uint4 v = *reinterpret_cast<const uint4*>(W + (size_t)row * k + (size_t)k8 * 8);
  reinterpret_cast<uint4*>(P)[((size_t)nb * (k / 16) + kb) * 64 + lane] = v;
}

int slk_pack_weight(hipStream_t s, const void* W, int n, int k, void* P, int nb_off) {
  const size_t chunks = (size_t)n * (k / 8);
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, (const bf16_t*)W, n,
                     k, (bf16_t*)P, nb_off);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- the kernel ----------------------------------------------------------------------------
// OUT = 0: fp32 partials Cf[split][row][n] (ldc = n, split stride = m_upper * n)
// OUT = 1: bf16 rows Cb[row_map ? row_map[row] : row][n] (no split-k)
template <int BM, int WNB, int OUT>
__global__ __launch_bounds__(256, (BM <= 64 ? 2 : 1)) void gemm_mfma_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ Wp, int n, int k, int k_per_split,
    const int32_t* __restrict__ m_dev, int m_upper, float* __restrict__ Cf, bf16_t* __restrict__ Cb,
    const int32_t* __restrict__ row_map, size_t ldc, int tiles_m, int tiles_n) {
  constexpr int MB = BM / 32;          // 32-row blocks per tile
  constexpr int BN = 128 * WNB;
  constexpr int NF = MB;               // A fragments each wave stages per k-tile (MB*4 / 4 waves)
  extern __shared__ Frag lds[];       // [2 stages][MB][4 kb][64 lanes] x 16 B

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

  const Frag* Bp[WNB];
#pragma unroll
  for (int i = 0; i < WNB; ++i) {
    int nb = n0 / 32 + wave * WNB + i;
    nb = nb < NB32 ? nb : NB32 - 1;                      // column tail: load something valid, never stored
    Bp[i] = reinterpret_cast<const Frag*>(Wp) + ((size_t)nb * K16 + kbeg / 16) * 64 + lane;
  }
  const bf16_t* Ap[NF];
  int a_slot[NF];
#pragma unroll
  for (int i = 0; i < NF; ++i) {
    const int f = wave + 4 * i, mb = f % MB, kb = f / MB;
    int row = m0 + mb * 32 + (lane & 31);
    row = row < m_upper ? row : m_upper - 1;              // row tail: stay inside the buffer
    Ap[i] = A + (size_t)row * k + kbeg + kb * 16 + (lane >> 5) * 8;
    a_slot[i] = (mb * 4 + kb) * 64 + lane;
  }

  f32x16 acc[MB][WNB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < WNB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  Frag a_reg[NF];
  Frag b_cur[WNB][4], b_nxt[WNB][4];
  // prologue: tile 0
#pragma unroll
  for (int i = 0; i < NF; ++i) a_reg[i] = *reinterpret_cast<const Frag*>(Ap[i]);
#pragma unroll
  for (int i = 0; i < WNB; ++i)
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) b_cur[i][kb] = Bp[i][kb * 64];
#pragma unroll
  for (int i = 0; i < NF; ++i) lds[a_slot[i]] = a_reg[i];
  __syncthreads();

  for (int kt = 0; kt < ktiles; ++kt) {
    const bool more = kt + 1 < ktiles;
    if (more) {
#pragma unroll
      for (int i = 0; i < NF; ++i) a_reg[i] = *reinterpret_cast<const Frag*>(Ap[i] + (kt + 1) * BK);
#pragma unroll
      for (int i = 0; i < WNB; ++i)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) b_nxt[i][kb] = Bp[i][((kt + 1) * 4 + kb) * 64];
    }
    const Frag* stage = lds + (kt & 1) * (MB * 4 * 64);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const Frag a = stage[(mb * 4 + kb) * 64 + lane];
#pragma unroll
        for (int i = 0; i < WNB; ++i)
          acc[mb][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b_cur[i][kb], acc[mb][i], 0, 0, 0);
      }
    }
    if (more) {
      Frag* nstage = lds + ((kt + 1) & 1) * (MB * 4 * 64);
#pragma unroll
      for (int i = 0; i < NF; ++i) nstage[a_slot[i]] = a_reg[i];
#pragma unroll
      for (int i = 0; i < WNB; ++i)
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) b_cur[i][kb] = b_nxt[i][kb];
    }
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

// ---- host side ------------------------------------------------------------------------------
// Number of k-splits for a launch bounded by mu rows: enough workgroups to cover the chip
// twice over, capped so that the fp32 partial traffic stays under a quarter of the weight
// bytes and each split keeps at least two k-tiles.
int slk_gemm_splits(int mu, int n, int k) {
  const int bm = mu <= 32 ? 32 : mu <= 64 ? 64 : mu <= 128 ? 128 : 256;
  const int tiles = sl_cdiv(mu, bm) * sl_cdiv(n, 256);
  const int target = bm <= 64 ? 512 : 256;
  int s = 1;
  while (s < 16 && tiles * s < target && (k % (BK * s * 2) == 0) && (k / (BK * s * 2) >= 2) &&
         (size_t)(s * 2) * 16 * mu <= (size_t)k)
    s *= 2;
  return s;
}

template <int BM, int WNB, int OUT>
static int launch_gemm(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                       int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc) {
  constexpr int BN = 128 * WNB;
  const int tiles_m = sl_cdiv(mu, BM), tiles_n = sl_cdiv(n, BN);
  const size_t sh = (size_t)2 * (BM / 32) * 4 * 64 * 16;
  auto kern = gemm_mfma_kernel<BM, WNB, OUT>;
  if (sh > 48 * 1024) SL_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh));
  dim3 grid(8 * tiles_m * sl_cdiv(tiles_n, 8), splits), block(256);
  hipLaunchKernelGGL(kern, grid, block, sh, s, (const bf16_t*)A, (const bf16_t*)Wp, n, k, k / splits, m_dev, mu, Cf,
                     (bf16_t*)Cb, row_map, ldc, tiles_m, tiles_n);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// C = A . Wp^T for a launch bounded by mu rows.  Cf != null: fp32 partials [splits][mu][n];
// else bf16 rows into Cb through row_map (splits must be 1).
int slk_gemm_mfma(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int n, int k, int splits,
                  float* Cf, void* Cb, const int32_t* row_map, size_t ldc) {
  if (mu <= 0) return SL_OK;
  if (n % 32 || k % (BK * splits) || splits < 1) return SL_EINVAL;
  if (!Cf && splits != 1) return SL_EINVAL;
#define GO(BM)                                                                                             \
  return Cf ? launch_gemm<BM, 2, 0>(s, A, Wp, m_dev, mu, n, k, splits, Cf, nullptr, nullptr, ldc)          \
            : launch_gemm<BM, 2, 1>(s, A, Wp, m_dev, mu, n, k, splits, nullptr, Cb, row_map, ldc)
  if (mu <= 32) { GO(32); }
  if (mu <= 64) { GO(64); }
  if (mu <= 128) { GO(128); }
  GO(256);
#undef GO
}
