// Bidirectional M x N attention of the active rows on the MFMA units (bf16, d_h = 128):
//   o[r, h] = softmax(q[r, h] . K[b, h, 0..N)^T / sqrt(d_h)) V[b, h, 0..N)
// for the packed active rows r of each sequence b against ALL N cached slots of that
// sequence, no mask (Alg. 1 'attention' line; Sec. 2.1: locked slots are served from the
// cache, live slots were just overwritten by this step's K/V write).
//
// Flash-style, computed transposed so that softmax statistics live in one lane:
//   S^T[key, q] = K Q^T   (MFMA A = K fragment from LDS, B = Q^T fragment kept in registers)
//   lane l of the accumulator owns query q = l%32 and 16 keys per 32-key block, so the row
//   max / sum of the online softmax need one cross-lane exchange (lanes l, l^32) only;
//   O^T[dim, q] += V^T P^T  (A = V^T fragment from LDS, B = P^T = the accumulator registers
//   of the first product rounded to bf16, used in place: no LDS round trip, no transpose).
// The K/V cache layouts (kc_index / vc_index) make every fragment of a 64-slot tile a
// contiguous block, so a tile is a straight 16 KiB + 16 KiB copy into LDS.
//
// One workgroup = 4 waves x 32 queries of ONE sequence and one head; packed rows of
// different sequences never share a tile (the varlen case of a ragged batch).
#include "sl_common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

typedef bf16x8 FragA;       // one lane's 16-byte share of an MFMA operand fragment

constexpr int QT = 128;          // queries per workgroup
constexpr int KT = 64;           // slots per K/V tile
constexpr int DH = 128;
constexpr int kMaxBatch = 255;

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// SPLIT: the key tiles are divided over gridDim.z workgroups (thin launches would otherwise
// leave most CUs idle and walk all N slots serially); each writes its unnormalised O, running
// max and sum, and attention_merge_kernel combines them.
template <bool SPLIT>
__global__ __launch_bounds__(256) void attention_mfma_kernel(const bf16_t* __restrict__ q,
                                                             const bf16_t* __restrict__ kc,
                                                             const bf16_t* __restrict__ vc,
                                                             const int32_t* __restrict__ active_idx,
                                                             const int32_t* __restrict__ m_dev, int m_upper, int B,
                                                             int H, int N, int n_pad, bf16_t* __restrict__ o,
                                                             int tiles_per_split, float* __restrict__ part_o,
                                                             float* __restrict__ part_ml) {
  __shared__ FragA ldsK[KT * DH / 8];        // 16 KiB
  __shared__ FragA ldsV[KT * DH / 8];        // 16 KiB
  __shared__ int cu[kMaxBatch + 2];
  const int M = min(*m_dev, m_upper);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // blockIdx.x = head: consecutive workgroup ids go to different XCDs, so the query tiles of
  // one head (same K/V) land on one XCD and share its L2
  const int hh = blockIdx.x;
  // per-sequence row ranges: cu[b] = first packed row whose flat id >= b*N
  if (B == 1) {
    if (tid <= 1) cu[tid] = tid ? M : 0;
  } else if (tid <= B) {
    int lo = 0, hi = M;
    const long long key = (long long)tid * N;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if ((long long)active_idx[mid] < key) lo = mid + 1; else hi = mid;
    }
    cu[tid] = lo;
  }
  __syncthreads();
  int b = 0, tile = blockIdx.y, row0 = -1, row_end = 0;
  for (; b < B; ++b) {
    const int cnt = cu[b + 1] - cu[b];
    const int nt = (cnt + QT - 1) / QT;
    if (tile < nt) { row0 = cu[b] + tile * QT; row_end = cu[b + 1]; break; }
    tile -= nt;
  }
  if (row0 < 0) return;                       // uniform across the workgroup

  const size_t head_base = ((size_t)b * H + hh) * n_pad * DH;
  const FragA* kg = reinterpret_cast<const FragA*>(kc + head_base);
  const FragA* vg = reinterpret_cast<const FragA*>(vc + head_base);

  // Q^T fragments: lane holds query (lane&31), dims ks*16 + (lane>>5)*8 .. +7
  const int my_row = row0 + wave * 32 + (lane & 31);
  const int ld_row = my_row < row_end ? my_row : row_end - 1;
  FragA qf[8];
  {
    const bf16_t* qp = q + ((size_t)ld_row * H + hh) * DH + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const FragA*>(qp + ks * 16);
  }

  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_o[i][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = 1.4426950408889634f / sqrtf((float)DH);   // log2(e) / sqrt(d_h)

  const int kt_lo = SPLIT ? blockIdx.z * tiles_per_split : 0;
  const int n_tiles = SPLIT ? min(n_pad / KT, kt_lo + tiles_per_split) : n_pad / KT;
  FragA kreg[4], vreg[4];
  {
    const FragA* k0 = kg + (size_t)kt_lo * (KT * DH / 8);
    const FragA* v0 = vg + (size_t)kt_lo * (KT * DH / 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) { kreg[i] = k0[tid + 256 * i]; vreg[i] = v0[tid + 256 * i]; }
  }

  for (int kt = kt_lo; kt < n_tiles; ++kt) {
    __syncthreads();                          // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 4; ++i) { ldsK[tid + 256 * i] = kreg[i]; ldsV[tid + 256 * i] = vreg[i]; }
    __syncthreads();
    if (kt + 1 < n_tiles) {
      const FragA* kn = kg + (size_t)(kt + 1) * (KT * DH / 8);
      const FragA* vn = vg + (size_t)(kt + 1) * (KT * DH / 8);
#pragma unroll
      for (int i = 0; i < 4; ++i) { kreg[i] = kn[tid + 256 * i]; vreg[i] = vn[tid + 256 * i]; }
    }
    // S^T = K Q^T : two 32-key blocks
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const FragA a = ldsK[(kb * 16 + 2 * ks) * 32 + lane];
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
      }
    }
    // accumulator register v of block kb is key 32*kb + 8*(v/4) + 4*(lane>>5) + v%4
    if ((kt + 1) * KT > N) {
      const int kbase = kt * KT + 4 * (lane >> 5);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kbase + 32 * kb + 8 * (v / 4) + (v % 4) >= N) s[kb][v] = -INFINITY;
    }
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);     // finite: every tile holds at least one real key
    const float alpha = exp2f((m_run - m_new) * sc);
    const float mb_ = m_new * sc;
    float psum = 0.f;
    // The probabilities enter the second product as a bf16 pair hi + lo (lo = the bf16 of what
    // hi's rounding lost): one bf16 alone carries a relative error of 2^-9 per probability,
    // enough to move ~30% of the attention outputs to the neighbouring bf16 value.
    FragA pf[4], pl[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[v] = exp2f(fmaf(s[kb][v], sc, -mb_));
        psum += p[v];
      }
      // step st = 2*kb + j uses registers 8j .. 8j+7: keys 16*st + 8a + 4h + i  <->  e = 4a + i
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const __bf16 hi = (__bf16)p[8 * j + e];
          pf[2 * kb + j][e] = hi;
          pl[2 * kb + j][e] = (__bf16)(p[8 * j + e] - (float)hi);
        }
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__any(alpha != 1.0f)) {                // the running max rarely moves after the first tiles
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[i][v] *= alpha;
    }
    // O^T += V^T P^T
#pragma unroll
    for (int st = 0; st < 4; ++st) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const FragA a = ldsV[(2 * st + (lane >> 5)) * DH + mb * 32 + (lane & 31)];
        acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[st], acc_o[mb], 0, 0, 0);
        acc_o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pl[st], acc_o[mb], 0, 0, 0);
      }
    }
  }
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (SPLIT) {
    if (my_row < row_end) {
      const size_t slot = ((size_t)blockIdx.z * m_upper + my_row) * H + hh;
      float* po = part_o + slot * DH + 4 * (lane >> 5);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<float4*>(po + mb * 32 + 8 * g) =
              make_float4(acc_o[mb][4 * g], acc_o[mb][4 * g + 1], acc_o[mb][4 * g + 2], acc_o[mb][4 * g + 3]);
      if (lane < 32) {
        part_ml[slot * 2] = m_run * sc;          // running max in the exp2 domain
        part_ml[slot * 2 + 1] = l_tot;
      }
    }
    return;
  }
  const float inv = 1.0f / l_tot;
  if (my_row < row_end) {
    // o is written in the fragment-tiled activation layout the Out-projection GEMM reads
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc_o[mb][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(o + afrag_index(my_row, hh * DH + mb * 32 + 8 * g + 4 * (lane >> 5), H * DH)) = w;
      }
  }
}

// o[row, h, :] = sum_z 2^(m_z - m) O_z / sum_z 2^(m_z - m) l_z over the key splits z
__global__ __launch_bounds__(128) void attention_merge_kernel(const float* __restrict__ part_o,
                                                              const float* __restrict__ part_ml,
                                                              const int32_t* __restrict__ m_dev, int m_upper, int H,
                                                              int Z, bf16_t* __restrict__ o) {
  const int M = min(*m_dev, m_upper);
  const int row = blockIdx.x, hh = blockIdx.y, dd = threadIdx.x;
  if (row >= M) return;
  float mx = -INFINITY;
  for (int z = 0; z < Z; ++z) mx = fmaxf(mx, part_ml[(((size_t)z * m_upper + row) * H + hh) * 2]);
  float num = 0.f, den = 0.f;
  for (int z = 0; z < Z; ++z) {
    const size_t slot = ((size_t)z * m_upper + row) * H + hh;
    const float w = exp2f(part_ml[slot * 2] - mx);
    num = fmaf(w, part_o[slot * DH + dd], num);
    den = fmaf(w, part_ml[slot * 2 + 1], den);
  }
  o[afrag_index(row, hh * DH + dd, H * DH)] = (bf16_t)(num / den);
}

// Key-split plan for a launch bounded by m_upper rows: split while fewer than ~2 workgroups
// per CU would run.  Returns Z (1 = no split) and the tiles per split.
int slk_attention_splits(int m_upper, int B, int H, int n_pad, int* tiles_per_split) {
  const int n_tiles = n_pad / KT;
  const int blocks = (sl_cdiv(m_upper, QT) + B - 1) * H;
  int Z = 1;
  if (blocks < 256) Z = sl_cdiv(512, blocks);
  if (Z > n_tiles) Z = n_tiles;
  const int tps = sl_cdiv(n_tiles, Z);
  *tiles_per_split = tps;
  return sl_cdiv(n_tiles, tps);
}

// fp32 scratch floats the split path may need for any launch of at most m_upper rows
size_t slk_attention_scratch_elems(int m_upper, int B, int H, int n_pad) {
  size_t best = 0;
  for (int mu = 1; mu <= m_upper; ++mu) {
    int tps;
    const int Z = slk_attention_splits(mu, B, H, n_pad, &tps);
    if (Z > 1 && (size_t)Z * mu * H * (DH + 2) > best) best = (size_t)Z * mu * H * (DH + 2);
  }
  return best;
}

int slk_attention_mfma(hipStream_t s, const void* q, const void* kc, const void* vc, const int32_t* active_idx,
                       const int32_t* m_dev, int m_upper, int B, int H, int N, int n_pad, void* o, float* scratch) {
  if (m_upper <= 0) return SL_OK;
  if (B > kMaxBatch || n_pad % KT) return SL_EINVAL;
  int tps;
  const int Z = scratch ? slk_attention_splits(m_upper, B, H, n_pad, &tps) : 1;
  dim3 grid(H, sl_cdiv(m_upper, QT) + B - 1, Z), block(256);
  if (Z == 1) {
    hipLaunchKernelGGL(attention_mfma_kernel<false>, grid, block, 0, s, (const bf16_t*)q, (const bf16_t*)kc,
                       (const bf16_t*)vc, active_idx, m_dev, m_upper, B, H, N, n_pad, (bf16_t*)o, 0, nullptr, nullptr);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  float* part_o = scratch;
  float* part_ml = scratch + (size_t)Z * m_upper * H * DH;
  hipLaunchKernelGGL(attention_mfma_kernel<true>, grid, block, 0, s, (const bf16_t*)q, (const bf16_t*)kc,
                     (const bf16_t*)vc, active_idx, m_dev, m_upper, B, H, N, n_pad, (bf16_t*)o, tps, part_o, part_ml);
  SL_LAUNCH_CHECK();
  hipLaunchKernelGGL(attention_merge_kernel, dim3(m_upper, H), dim3(DH), 0, s, part_o, part_ml, m_dev, m_upper, H, Z,
                     (bf16_t*)o);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
