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
//   of the first product rounded to half precision, used in place: no LDS round trip, no
//   transpose).
// The K/V cache layouts (kc_index / vc_index) make every fragment of a 64-slot tile a
// contiguous block, so a tile is a straight 16 KiB + 16 KiB copy into LDS.
//
// Precision of P.  The second product runs on half-precision operands: V is cached as the half
// image of its bf16 values (vcache_half_bits: exact in the range activations live in), P is
// rounded to half precision (11 significant bits, round to nearest even) by the two thick-launch
// kernels and carried as a pair of halves (22 bits) by the thin one, where the second half costs
// nothing.  One bf16 value per probability (8 bits, what a plain bf16 attention does) is not
// enough against an fp64 softmax: measured on one full-size layer, the rms error of the logits
// grows by 17 % with bf16 probabilities, by 5-8 % with one half, by nothing with two; the largest
// error and the share of logits beyond 2e-2 stay where the bf16 roundings of the activations put
// them with one half or two.
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
constexpr int kMaxBatch = SL_MAX_BATCH;

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
constexpr float kMaxLag = 8.0f;   // probabilities may exceed 1 by up to 2^8 before the reference moves
typedef uint32_t PFrag __attribute__((ext_vector_type(4)));   // eight half-precision probabilities, packed in pairs

// O^T += V^T P^T on one fragment pair: V is cached as half-precision images of its bf16 values, P is
// rounded to half precision (see the kernels), the product accumulates in fp32.
__device__ inline f32x16 mfma_pv(const FragA& v, const PFrag& p, const f32x16& acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, v), __builtin_bit_cast(f16x8, p), acc, 0, 0, 0);
}
// Two probabilities as a packed pair of halves, round to nearest even.
__device__ inline uint32_t pack_half2(float a, float b) {
  const f32x2 pp = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, f16x2));
}
// What the halves of such a pair leave of (a, b), again as a packed pair: P = hi + lo carries 22 bits.
__device__ inline uint32_t pack_half2_rest(float a, float b, uint32_t hi) {
  const f16x2 h = __builtin_bit_cast(f16x2, hi);
  return pack_half2(a - (float)h[0], b - (float)h[1]);
}

// SPLIT: the key tiles are divided over gridDim.z workgroups (thin launches would otherwise
// leave most CUs idle and walk all N slots serially); each writes its unnormalised O, running
// max and sum, and attention_merge_kernel combines them.
//
// Software pipeline.  With one wave per SIMD nothing else can hide the softmax arithmetic, so
// each wave overlaps its own work: iteration t issues the MFMAs of O += V(t-1)^T P(t-1)^T and of
// S(t+1) = K(t+1) Q^T while the vector ALU turns S(t) into P(t) (MFMAs run asynchronously once
// issued).  O is kept relative to the running max of the tiles already ADDED, so the rescale by
// alpha(t) follows the accumulation of tile t-1 and happens only when some lane's max moved.
// K and V tiles arrive by direct-to-LDS loads into three-slot rings (K(t+3) and V(t+1) are issued
// in iteration t, two iterations ahead of their use); one barrier per tile.
template <bool SPLIT>
__global__ __launch_bounds__(256, 1) void attention_mfma_kernel(const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ kc,
                                                                const bf16_t* __restrict__ vc,
                                                                const int32_t* __restrict__ active_idx,
                                                                const int32_t* __restrict__ m_dev, int m_upper, int B,
                                                                int H, int N, int n_pad, bf16_t* __restrict__ o,
                                                                int tiles_per_split, float* __restrict__ part_o,
                                                                float* __restrict__ part_ml) {
  extern __shared__ FragA lds[];             // K ring [R][16 KiB] | V ring [R][16 KiB]
  __shared__ int cu[kMaxBatch + 2];
  constexpr int TILE_F = KT * DH / 8;        // FragA elements per tile
  FragA* const ldsK = lds;
  constexpr int R = 3;                       // ring depth: tiles are requested R-1 iterations ahead
  FragA* const ldsV = lds + R * TILE_F;
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
  const int kt_lo = SPLIT ? blockIdx.z * tiles_per_split : 0;
  const int kt_hi = SPLIT ? min(n_pad / KT, kt_lo + tiles_per_split) : n_pad / KT;
  const int T = kt_hi - kt_lo;               // >= 1 tiles for this workgroup

  // a 16 KiB tile is a straight copy: 16 chunks of 1 KiB, four per wave, lane L's 16 bytes land at
  // chunk base + 16 L
  // Addressing is scalar except for one per-lane byte offset: the tile pointer g is uniform
  // (instruction form "vgpr offset + sgpr base"), and the LDS destination is a scalar sum on the
  // wave's LDS base, read once.  l is a slot of the K or V ring, given as its index into lds.
  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) FragA*)(lds + wave * 4 * 64));
  const uint32_t lane_voff = (uint32_t)((wave * 4 * 64 + lane) * 16);
  auto load_chunk = [&](const FragA* g, const FragA* l, int c) {
    const uint32_t laddr = lds_wave + (uint32_t)((l - lds) + c * 64) * 16u;
    const uint64_t gbase = (uint64_t)(uintptr_t)g + (uint64_t)(c * 1024);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_voff), "s"(gbase), "s"(laddr)
                 : "memory", "m0");
  };
  auto load_tile = [&](const FragA* g, FragA* l) {
#pragma unroll
    for (int c = 0; c < 4; ++c) load_chunk(g, l, c);
  };
  // prologue loads: K(0..R-1), V(0..R-3); V(0) also into the slot iteration 0 multiplies by P = 0
#pragma unroll
  for (int j = 0; j < R; ++j) load_tile(kg + (size_t)min(kt_lo + j, kt_hi - 1) * TILE_F, ldsK + j * TILE_F);
#pragma unroll
  for (int j = 0; j < R - 2; ++j) load_tile(vg + (size_t)min(kt_lo + j, kt_hi - 1) * TILE_F, ldsV + j * TILE_F);
  load_tile(vg + (size_t)kt_lo * TILE_F, ldsV + (R - 1) * TILE_F);

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

  // S^T = K Q^T for one tile: two 32-key blocks
  auto scores = [&](const FragA* kt_lds, f32x16 (&sv)[2]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const FragA a = kt_lds[(kb * 8 + ks) * 64 + lane];
        sv[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sv[kb], 0, 0, 0);
      }
    }
  };
  // accumulator register v of block kb is key 32*kb + 8*(v/4) + 4*(lane>>5) + v%4
  auto mask_tail = [&](int kt, f32x16 (&sv)[2]) {
    const int kbase = kt * KT + 4 * (lane >> 5);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (kbase + 32 * kb + 8 * (v / 4) + (v % 4) >= N) sv[kb][v] = -INFINITY;
  };
  // O^T += V^T P^T
  auto pv = [&](const FragA* vt_lds, const PFrag (&ph)[4]) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      FragA a[4];
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) a[mb] = vt_lds[(2 * st + (lane >> 5)) * DH + mb * 32 + (lane & 31)];
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) acc_o[mb] = mfma_pv(a[mb], ph[st], acc_o[mb]);
    }
  };
  // One pipeline step for tile t: scores sc_cur -> probabilities p_new, while the MFMAs add tile t-1
  // (p_old) and compute the scores of tile t+1 (sc_next).
  auto step = [&](int t, f32x16 (&sc_cur)[2], f32x16 (&sc_next)[2], const PFrag (&p_old)[4], PFrag (&p_new)[4]) {
    // loads complete in order, eight chunks per wave per iteration: all but those of the last
    // R-2 iterations have landed, which covers K(t+1) and V(t-1)
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(8 * (R - 2)) : "memory");
    __syncthreads();      // ... for everyone; the slots of K(t) and V(t-2) are free
    // K(t+R) and V(t+R-2) go into the two slots the barrier just freed, one 1 KiB chunk every second
    // MFMA slot below (a burst of eight would fill the load queue and stall the wave at issue).
    // Past the last tile K re-fetches the last one; nothing reads it.
    const FragA* k_src = kg + (size_t)min(kt_lo + t + R, kt_hi - 1) * TILE_F;
    const FragA* v_src = vg + (size_t)min(kt_lo + t + R - 2, kt_hi - 1) * TILE_F;
    FragA* const k_dst = ldsK + (t % R) * TILE_F;
    FragA* const v_dst = ldsV + ((t + R - 2) % R) * TILE_F;
    const FragA* vt_lds = ldsV + ((t + R - 1) % R) * TILE_F + (lane >> 5) * DH + (lane & 31);
    const FragA* kt_lds = ldsK + ((t + 1) % R) * TILE_F + lane;
    // The block below is laid out by hand as 32 slots, one MFMA each, fenced so that the compiler
    // keeps the order: slots 0..15 add tile t-1 (V fragment groups of four), slots 16..31 compute the
    // scores of tile t+1; LDS fragments are read 8..12 slots ahead of their MFMA; the softmax of tile
    // t rides along, one pair of probabilities every second slot (an MFMA occupies the matrix pipe
    // for 32 cycles and leaves the vector ALU about 20 of them).
    FragA va[3][4], kf[16];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) va[0][mb] = vt_lds[mb * 32];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) va[1][mb] = vt_lds[2 * DH + mb * 32];
    // The reference point of the exponentials follows the running max only in jumps of more than
    // kMaxLag (in the exp2 domain): a stale reference is exact mathematics (numerator and
    // denominator carry the same factor, at most 2^kMaxLag), and O is then rescaled on a tile only
    // when some query of the wave really jumped.  With near-uniform scores the max of 32 queries
    // creeps up on almost every tile, and rescaling 64 accumulators each time cost a quarter of
    // the kernel.  First tile: m_run = -inf, so every query jumps (alpha = 0 on a zero O).
    float mx = sc_cur[0][0], m_new = 0.f, alpha = 1.f, mb_ = 0.f;
    float psum = 0.f, pa = 0.f, pb = 0.f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if (i < 16 && i % 2 == 0) {
        if (i < 8) load_chunk(k_src, k_dst, i / 2);
        else load_chunk(v_src, v_dst, i / 2 - 4);
      }
      if (i < 8) {                                   // V fragments of group st + 2, eight slots ahead
        const int st = i >> 2, r = i & 3;
        va[(st + 2) % 3][r] = vt_lds[(2 * (st + 2)) * DH + r * 32];
      }
      if (i >= 4 && i < 20) {                        // K fragments of tile t+1, twelve slots ahead
        const int q = i - 4, jr = (q & 1) * 8 + (q >> 1);
        kf[jr] = kt_lds[jr * 64];
      }
      if (i < 16) {
        const int st = i >> 2, mb = i & 3;
        acc_o[mb] = mfma_pv(va[st % 3][mb], p_old[st], acc_o[mb]);
      } else {
        const int jj = i - 16, kb = jj & 1, ks = jj >> 1, j = kb * 8 + ks;   // the two score blocks alternate
        if (ks == 0) {
          f32x16 z;
#pragma unroll
          for (int v = 0; v < 16; ++v) z[v] = 0.f;
          sc_next[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[ks], z, 0, 0, 0);
        } else {
          sc_next[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qf[ks], sc_next[kb], 0, 0, 0);
        }
      }
      // Vector work of tile t, tied to its slot by the empty asm statements (without them the compiler
      // sinks all of it below the last MFMA).  Slots 0..3: the tile's row max, a dependent chain that
      // would otherwise hold the first MFMA back (the MFMAs of these slots add tile t-1 and do not need
      // it); the two lanes of a query exchange their halves with a lane-half swap, a vector-ALU
      // instruction.  Slots 4..31: the softmax, one pair of probabilities (2pr, 2pr+1 of this lane:
      // register v of block kb, for P^T step 2*kb + v/8) at a time, exponentials in one slot, sum and
      // rounding to a pair of halves in the next; the last four slots carry two such pieces each.
      if (i < 4) {
        const int kb = i >> 1, v0 = (i & 1) * 8;
#pragma unroll
        for (int v = 0; v < 8; ++v) mx = fmaxf(mx, sc_cur[kb][v0 + v]);
        if (i == 3) {
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
          mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
          const float m_cand = fmaxf(m_run, mx);    // finite: every tile holds at least one real key
          m_new = (m_cand - m_run) * sc > kMaxLag ? m_cand : m_run;
          alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
          mb_ = m_new * sc;
          asm volatile("" : "+v"(m_new), "+v"(alpha), "+v"(mb_));
        } else {
          asm volatile("" : "+v"(mx));
        }
      } else {
#pragma unroll
        for (int u = 0; u < (i < 28 ? 1 : 2); ++u) {
          const int piece = i < 28 ? i - 4 : 24 + 2 * (i - 28) + u;      // 32 pieces: (pair, half of its work)
          const int pr = piece >> 1;
          const int x = 2 * pr, kb = x >> 4, v = x & 15, stp = 2 * kb + (v >> 3), e = v & 7;
          if ((piece & 1) == 0) {
            pa = __builtin_amdgcn_exp2f(fmaf(sc_cur[kb][v], sc, -mb_));
            pb = __builtin_amdgcn_exp2f(fmaf(sc_cur[kb][v + 1], sc, -mb_));
            asm volatile("" : "+v"(pa), "+v"(pb));
          } else {
            psum += pa + pb;
            uint32_t hw = pack_half2(pa, pb);
            asm volatile("" : "+v"(hw), "+v"(psum));
            p_new[stp][e >> 1] = hw;
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__any(alpha != 1.0f)) {                // the running max rarely moves after the first tiles
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[i][v] *= alpha;
    }
    if ((kt_lo + t + 2) * KT > N) mask_tail(kt_lo + t + 1, sc_next);
  };

  f32x16 s0[2], s1[2];
  PFrag p0[4], p1[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) p0[i][e] = 0u;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  scores(ldsK, s0);
  if ((kt_lo + 1) * KT > N) mask_tail(kt_lo, s0);
  for (int t = 0; t < T; t += 2) {
    step(t, s0, s1, p0, p1);
    if (t + 1 < T) step(t + 1, s1, s0, p1, p0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                            // V(T-1) landed
  if (T & 1) pv(ldsV + ((T - 1) % R) * TILE_F, p1);
  else pv(ldsV + ((T - 1) % R) * TILE_F, p0);

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

// Second form of the same product for launches with more workgroups than CUs: the wave does not
// pipeline its own tile steps (scores, softmax, P.V in sequence) and THREE workgroups share a CU, so
// that one's softmax runs under the others' MFMAs and barrier waits.  What lets three fit: P is one
// half-precision value per probability (no lo half: 32 MFMAs per tile instead of 48, no vector work to
// form it; 151 registers), and V has ONE 16 KiB slot next to K's two (48 KiB per workgroup): V(t) is
// requested at the top of step t, when the barrier has shown that everyone is done with V(t-1), and
// arrives under the scores and the softmax of the step; a second barrier per step makes it visible.
// Measured at sum M = 8192 rows of N = 1024: 220 us (two workgroups per CU, P as two halves) ->
// 206 us (three per CU) -> 157 us (one half).  Same fragment layouts as above.
template <bool SPLIT>
__global__ __launch_bounds__(256, 3) void attention_trio_kernel(const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ kc,
                                                                const bf16_t* __restrict__ vc,
                                                                const int32_t* __restrict__ active_idx,
                                                                const int32_t* __restrict__ m_dev, int m_upper, int B,
                                                                int H, int N, int n_pad, bf16_t* __restrict__ o,
                                                                int tiles_per_split, float* __restrict__ part_o,
                                                                float* __restrict__ part_ml) {
  extern __shared__ FragA lds[];             // K ring [2][16 KiB] | V slot [16 KiB]
  __shared__ int cu[kMaxBatch + 2];
  constexpr int TILE_F = KT * DH / 8;
  FragA* const ldsK = lds;
  FragA* const ldsV = lds + 2 * TILE_F;
  const int M = min(*m_dev, m_upper);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hh = blockIdx.x;
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
  const int kt_lo = SPLIT ? blockIdx.z * tiles_per_split : 0;
  const int kt_hi = SPLIT ? min(n_pad / KT, kt_lo + tiles_per_split) : n_pad / KT;
  const int T = kt_hi - kt_lo;               // >= 1 tiles for this workgroup

  const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) FragA*)(lds + wave * 4 * 64));
  const uint32_t lane_voff = (uint32_t)((wave * 4 * 64 + lane) * 16);
  auto load_tile = [&](const FragA* g, const FragA* l) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t laddr = lds_wave + (uint32_t)((l - lds) + c * 64) * 16u;
      const uint64_t gbase = (uint64_t)(uintptr_t)g + (uint64_t)(c * 1024);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                   :
                   : "v"(lane_voff), "s"(gbase), "s"(laddr)
                   : "memory", "m0");
    }
  };
  load_tile(kg + (size_t)kt_lo * TILE_F, ldsK);

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

  for (int t = 0; t < T; ++t) {
    const int slot = t & 1;
    // K(t) has landed (it was requested one iteration ago) ...
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();       // ... for everyone, and everyone is done with tile t-1: V's slot and K(t-1)'s are free
    // V(t) first, then K(t+1): loads complete in order, so "all but the last four" below means V(t)
    load_tile(vg + (size_t)(kt_lo + t) * TILE_F, ldsV);
    if (t + 1 < T) load_tile(kg + (size_t)(kt_lo + t + 1) * TILE_F, ldsK + (slot ^ 1) * TILE_F);
    // S^T = K Q^T: two 32-key blocks; register v of block kb is key 32*kb + 8*(v/4) + 4*(lane>>5) + v%4
    f32x16 sv[2];
    const FragA* kt_lds = ldsK + slot * TILE_F + lane;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        sv[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_lds[(kb * 8 + ks) * 64], qf[ks], sv[kb], 0, 0, 0);
    }
    if ((kt_lo + t + 1) * KT > N) {
      const int kbase = (kt_lo + t) * KT + 4 * (lane >> 5);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kbase + 32 * kb + 8 * (v / 4) + (v % 4) >= N) sv[kb][v] = -INFINITY;
    }
    float mx = sv[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sv[kb][v]);
    {   // the two lanes of a query exchange their halves' maxima (a lane-half swap: vector ALU, no LDS trip)
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    // the reference of the exponentials follows the running max only in jumps (see kMaxLag)
    const float m_cand = fmaxf(m_run, mx);
    const float m_new = (m_cand - m_run) * sc > kMaxLag ? m_cand : m_run;
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
    const float mb_ = m_new * sc;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[i][v] *= alpha;
    }
    // P in half precision, round to nearest even; pair (v, v+1) of block kb belongs to P^T step 2*kb + v/8
    PFrag ph[4];
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float pa = __builtin_amdgcn_exp2f(fmaf(sv[kb][v], sc, -mb_));
        const float pb = __builtin_amdgcn_exp2f(fmaf(sv[kb][v + 1], sc, -mb_));
        psum += pa + pb;
        ph[2 * kb + (v >> 3)][(v & 7) >> 1] = pack_half2(pa, pb);
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    // V(t) has landed (K(t+1)'s four chunks may still be in flight) ...
    if (t + 1 < T) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();       // ... for everyone
    // O^T += V^T P^T
    const FragA* vt_lds = ldsV + (lane >> 5) * DH + (lane & 31);
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      FragA a[4];
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) a[mb] = vt_lds[(2 * st) * DH + mb * 32];
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) acc_o[mb] = mfma_pv(a[mb], ph[st], acc_o[mb]);
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
        part_ml[slot * 2] = m_run * sc;
        part_ml[slot * 2 + 1] = l_tot;
      }
    }
    return;
  }
  const float inv = 1.0f / l_tot;
  if (my_row < row_end) {
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

// Third form, for launches of few rows (late steps of a schedule, where the whole product is a few
// MFLOP and its time is launches and memory latency): one workgroup = ONE head and 32 queries of one
// sequence; its four waves split the key tiles (wave w takes tiles w, w + 4, ..), each with the full
// flash recurrence on its own tiles, and merge their (O, max, sum) through LDS, so there is no
// partial-result buffer and no merge launch.  K and V fragments go global -> registers directly (the
// cache layouts make every MFMA fragment of a tile one contiguous 1 KiB block: no LDS staging, no
// barrier in the loop), the next tile's fragments are requested before the current tile is computed.
// Same fragment layouts as the kernels above; P is carried as two halves (hi + lo, 22 bits: the
// matrix pipe idles here anyway), with the exact running max as the reference of the exponentials.
constexpr int QTT = 32;          // queries per workgroup of the thin kernel
__global__ __launch_bounds__(256, 1) void attention_thin_kernel(const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ kc,
                                                                const bf16_t* __restrict__ vc,
                                                                const int32_t* __restrict__ active_idx,
                                                                const int32_t* __restrict__ m_dev, int m_upper, int B,
                                                                int H, int N, int n_pad, bf16_t* __restrict__ o) {
  extern __shared__ FragA lds[];             // reused as float: partial O [4 waves][64 lanes][64] | (m, l) [4][64][2]
  __shared__ int cu[kMaxBatch + 2];
  constexpr int TILE_F = KT * DH / 8;
  const int M = min(*m_dev, m_upper);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hh = blockIdx.x;
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
    const int nt = (cnt + QTT - 1) / QTT;
    if (tile < nt) { row0 = cu[b] + tile * QTT; row_end = cu[b + 1]; break; }
    tile -= nt;
  }
  if (row0 < 0) return;                       // uniform across the workgroup

  const size_t head_base = ((size_t)b * H + hh) * n_pad * DH;
  const FragA* kg = reinterpret_cast<const FragA*>(kc + head_base) + lane;
  const FragA* vg = reinterpret_cast<const FragA*>(vc + head_base) + (lane >> 5) * DH + (lane & 31);
  const int n_tiles = n_pad / KT;

  // every wave holds the same 32 queries: lane = query (lane & 31), dims ks*16 + (lane>>5)*8 .. +7
  const int my_row = row0 + (lane & 31);
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

  // fragments of tile t: K block (kb, ks) at (kb*8 + ks)*64 + lane, V^T block (st, mb) at (2*st + lane>>5)*DH + mb*32 + lane&31
  auto load_kv = [&](int t, FragA (&kf)[16], FragA (&vf)[16]) {
    const FragA* kt = kg + (size_t)t * TILE_F;
    const FragA* vt = vg + (size_t)t * TILE_F;
#pragma unroll
    for (int j = 0; j < 16; ++j) kf[j] = kt[j * 64];
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) vf[st * 4 + mb] = vt[(2 * st) * DH + mb * 32];
  };
  auto tile_step = [&](int t, const FragA (&kf)[16], const FragA (&vf)[16]) {
    f32x16 sv[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) sv[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb * 8 + ks], qf[ks], sv[kb], 0, 0, 0);
    }
    if ((t + 1) * KT > N) {                  // register v of block kb is key 32*kb + 8*(v/4) + 4*(lane>>5) + v%4
      const int kbase = t * KT + 4 * (lane >> 5);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kbase + 32 * kb + 8 * (v / 4) + (v % 4) >= N) sv[kb][v] = -INFINITY;
    }
    float mx = sv[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sv[kb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);     // finite: every tile holds at least one real key
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
    const float mb_ = m_new * sc;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_o[i][v] *= alpha;
    PFrag ph[4], pl[4];
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; v += 2) {
        const float pa = __builtin_amdgcn_exp2f(fmaf(sv[kb][v], sc, -mb_));
        const float pb = __builtin_amdgcn_exp2f(fmaf(sv[kb][v + 1], sc, -mb_));
        psum += pa + pb;
        const uint32_t hw = pack_half2(pa, pb);
        const uint32_t lw = pack_half2_rest(pa, pb, hw);
        ph[2 * kb + (v >> 3)][(v & 7) >> 1] = hw;
        pl[2 * kb + (v >> 3)][(v & 7) >> 1] = lw;
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int st = 0; st < 4; ++st) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
        acc_o[mb] = mfma_pv(vf[st * 4 + mb], ph[st], acc_o[mb]);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
        acc_o[mb] = mfma_pv(vf[st * 4 + mb], pl[st], acc_o[mb]);
    }
  };
  // this wave's tiles: wave, wave + 4, ..; two register sets, the next tile is requested before the current one is used
  {
    FragA k0[16], v0[16], k1[16], v1[16];
    int t = wave;
    if (t < n_tiles) load_kv(t, k0, v0);
    while (t < n_tiles) {
      if (t + 4 < n_tiles) load_kv(t + 4, k1, v1);
      tile_step(t, k0, v0);
      t += 4;
      if (t >= n_tiles) break;
      if (t + 4 < n_tiles) load_kv(t + 4, k0, v0);
      tile_step(t, k1, v1);
      t += 4;
    }
  }
  // merge the four waves' partial results: wave w finishes dims 32 w .. 32 w + 31
  float* part_o = reinterpret_cast<float*>(lds);          // [4][64][64]
  float* part_ml = part_o + 4 * 64 * 64;                  // [4][64][2]
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  {
    float* po = part_o + ((size_t)wave * 64 + lane) * 64;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<float4*>(po + mb * 16 + 4 * g) =
            make_float4(acc_o[mb][4 * g], acc_o[mb][4 * g + 1], acc_o[mb][4 * g + 2], acc_o[mb][4 * g + 3]);
    part_ml[(wave * 64 + lane) * 2] = m_run * sc;           // running max in the exp2 domain (-inf: no tile)
    part_ml[(wave * 64 + lane) * 2 + 1] = l_tot;
  }
  __syncthreads();
  float mz[4], mx = -INFINITY;
#pragma unroll
  for (int z = 0; z < 4; ++z) { mz[z] = part_ml[(z * 64 + lane) * 2]; mx = fmaxf(mx, mz[z]); }
  float num[16], den = 0.f;
#pragma unroll
  for (int v = 0; v < 16; ++v) num[v] = 0.f;
#pragma unroll
  for (int z = 0; z < 4; ++z) {
    const float w = __builtin_amdgcn_exp2f(mz[z] - mx);
    den = fmaf(w, part_ml[(z * 64 + lane) * 2 + 1], den);
    const float* pz = part_o + ((size_t)z * 64 + lane) * 64 + wave * 16;
#pragma unroll
    for (int v = 0; v < 16; ++v) num[v] = fmaf(w, pz[v], num[v]);
  }
  const float inv = 1.0f / den;
  if (my_row < row_end) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 w4;
#pragma unroll
      for (int e = 0; e < 4; ++e) w4[e] = (__bf16)(num[4 * g + e] * inv);
      *reinterpret_cast<bf16x4*>(o + afrag_index(my_row, hh * DH + wave * 32 + 8 * g + 4 * (lane >> 5), H * DH)) = w4;
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

// Which kernel a launch of `blocks` (row tile, head) workgroups takes: the three-per-CU kernel as
// soon as there are more workgroups than CUs, the pipelined one otherwise (at N = 2048 and 857 rows,
// 224 workgroups: 46 us against 62 us for the three-per-CU kernel with the keys split three ways).
static bool attention_use_trio(int blocks) { return blocks > 256; }

// The thin kernel (32 queries and one head per workgroup, key tiles split over its waves) while its
// workgroups fit the chip in one round and a wave's share of the keys stays short.
static bool attention_use_thin(int m_upper, int B, int H, int n_pad) {
  const int blocks = (sl_cdiv(m_upper, QTT) + B - 1) * H;
  return blocks <= 512 && n_pad / KT <= 16;
}

// Key-split plan for a launch bounded by m_upper rows: the keys are split just far enough to
// give every CU one workgroup of the pipelined kernel (LDS rings, 370 registers per lane: one per
// CU) or three of the other; splitting further only adds partial-result traffic and more
// rounds of workgroups.  Returns Z (1 = no split) and the tiles per split.
int slk_attention_splits(int m_upper, int B, int H, int n_pad, int* tiles_per_split) {
  const int n_tiles = n_pad / KT;
  const int blocks = (sl_cdiv(m_upper, QT) + B - 1) * H;
  int Z = (attention_use_trio(blocks) ? 768 : 256) / blocks;
  if (Z < 1) Z = 1;
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
  if (attention_use_thin(m_upper, B, H, n_pad)) {
    const size_t sh_thin = (size_t)(4 * 64 * 64 + 4 * 64 * 2) * sizeof(float);
    static unsigned long long lds_thin = 0;
    SL_ALLOW_DYNAMIC_LDS(lds_thin, attention_thin_kernel, sh_thin);
    hipLaunchKernelGGL(attention_thin_kernel, dim3(H, sl_cdiv(m_upper, QTT) + B - 1), dim3(256), sh_thin, s, (const bf16_t*)q,
                       (const bf16_t*)kc, (const bf16_t*)vc, active_idx, m_dev, m_upper, B, H, N, n_pad, (bf16_t*)o);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  int tps;
  const int Z = scratch ? slk_attention_splits(m_upper, B, H, n_pad, &tps) : 1;
  dim3 grid(H, sl_cdiv(m_upper, QT) + B - 1, Z), block(256);
  const bool trio = attention_use_trio((int)(grid.x * grid.y));
  const size_t sh = (trio ? 3 : 6) * (size_t)KT * DH * 2;   // 16 KiB slots: K 2 + V 1, or three each
  static unsigned long long lds_ok[4] = {0, 0, 0, 0};
  SL_ALLOW_DYNAMIC_LDS(lds_ok[0], attention_mfma_kernel<false>, 6 * (size_t)KT * DH * 2);
  SL_ALLOW_DYNAMIC_LDS(lds_ok[1], attention_mfma_kernel<true>, 6 * (size_t)KT * DH * 2);
  SL_ALLOW_DYNAMIC_LDS(lds_ok[2], attention_trio_kernel<false>, 3 * (size_t)KT * DH * 2);
  SL_ALLOW_DYNAMIC_LDS(lds_ok[3], attention_trio_kernel<true>, 3 * (size_t)KT * DH * 2);
  if (Z == 1) {
    hipLaunchKernelGGL(trio ? attention_trio_kernel<false> : attention_mfma_kernel<false>, grid, block, sh, s,
                       (const bf16_t*)q, (const bf16_t*)kc, (const bf16_t*)vc, active_idx, m_dev, m_upper, B, H, N, n_pad,
                       (bf16_t*)o, 0, nullptr, nullptr);
    SL_LAUNCH_CHECK();
    return SL_OK;
  }
  float* part_o = scratch;
  float* part_ml = scratch + (size_t)Z * m_upper * H * DH;
  hipLaunchKernelGGL(trio ? attention_trio_kernel<true> : attention_mfma_kernel<true>, grid, block, sh, s,
                     (const bf16_t*)q, (const bf16_t*)kc, (const bf16_t*)vc, active_idx, m_dev, m_upper, B, H, N, n_pad,
                     (bf16_t*)o, tps, part_o, part_ml);
  SL_LAUNCH_CHECK();
  hipLaunchKernelGGL(attention_merge_kernel, dim3(m_upper, H), dim3(DH), 0, s, part_o, part_ml, m_dev, m_upper, H, Z,
                     (bf16_t*)o);
  SL_LAUNCH_CHECK();
  return SL_OK;
}
