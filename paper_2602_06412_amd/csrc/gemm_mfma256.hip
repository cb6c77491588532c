// The ring kernel of the projection GEMM (launches bounded by more than 32 rows): one TM x 256 output tile
// per workgroup and CU, TM any multiple of 32 from 64 to 256, fed through a ring of LDS stages.
//
// Why a ring.  Measured on the older 128-row-tile kernel (gemm_mfma.hip): with loads switched off
// the MFMA loop runs at ~75% of peak, with them at ~45%, although neither HBM nor L2 bandwidth is
// near its limit.  Every weight byte is touched for the first time exactly once (an L2 miss
// served from HBM, ~2 us under load), all row tiles sharing the slab wait on that same miss,
// and with a prefetch distance of one k-tile (~0.4-0.9 us of MFMA work) the latency is exposed
// on every tile.  This kernel therefore keeps NS-1 k-tiles in flight:
//  * eight waves (two per SIMD) own (TM/2) x 64 sub-tiles of the TM x 256 tile;
//  * BOTH operands are staged in LDS by direct-to-LDS loads (no registers are tied up by
//    loads in flight; each byte crosses the vector L1 once per CU: 32 B/clk at full MFMA
//    rate for the full-height tile, half of what the 128-row kernel needs);
//  * k-tiles are 32 deep ((TM + 256) * 64 bytes per stage) and the stages fill the 160 KiB LDS: five
//    of 32 KiB at TM = 256 (four tiles = 128 KiB per CU in flight while one is multiplied), up to
//    eight at TM = 64 (for the short tiles a depth beyond four measured no different: their k-tile
//    step is held at ~0.4 us by the CU's miss path whatever is in flight);
//  * one barrier per k-tile, placed between the two halves of its MFMAs (the first and the last 16-row
//    blocks of a wave's sub-tile), so the LDS reads on either side of it are covered by MFMAs;
//    fragments are read half a tile ahead.
// Operands land in LDS as 32 x 16 blocks of 1 KiB (activation rows gathered 32 x 16 per
// instruction, pre-tiled weights copied linearly): element (r, k) of a block sits in the 16-byte
// slot (r % 32) + 32 * ((k % 16) / 8).
//
// The products are v_mfma_f32_16x16x32_bf16, not 32x32x16: same flops per cycle, but measured
// on this chip with random operands a loop of 16x16x32 sustains ~1.93 PFLOP/s at ~1.95 GHz where
// 32x32x16 sustains ~1.65 at ~1.65 GHz (the clock is managed by power, and the deeper dot
// product moves a quarter of the accumulator data per flop).  A 16 x 32 operand of that
// instruction (lane l: row l % 16, k = 8 * (l / 16) .. +7) is gathered from two neighbouring
// 32 x 16 blocks by giving every lane its own slot address; each group of 16 lanes still reads
// 256 contiguous bytes.  The weight fragment is passed as the first operand, so a lane ends up
// with four consecutive columns of one output row (16-byte fp32 / 8-byte bf16 pieces).
#include "sl_common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef bf16x8 Frag;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int BK2 = 32;                   // k per stage: one 16x16x32 MFMA k-step
constexpr int TILE = 256;                 // columns per tile, and rows of the full-height tile
// Rows per tile TM: any multiple of 32 from 64 to 256, so that a launch can fit its row tiles to the
// number of active rows (320 rows = two tiles of 160, not two of 256) and latency follows M.  A
// shorter tile costs more per row (the weight half of the operand traffic and the per-k-tile barrier
// do not shrink: kTileCost below); its smaller stages allow a deeper ring.
template <int TM> struct TileCfg {
  static_assert(TM % 32 == 0 && TM >= 64 && TM <= 256, "tile height");
  static constexpr int A_FR = TM / 16;              // A fragments (32 x 16, 1 KiB) per stage
  static constexpr int STAGE = (A_FR + 16) * 64;    // Frag elements per stage: A, then 16 B fragments
  static constexpr int NA = TM / 32;                // 16-row accumulator blocks per wave (sub-tile TM/2 x 64)
  static constexpr int HL = (NA + 1) / 2;           // ... in the first half of a k-tile step
  static constexpr int HH = NA / 2;                 // ... in the second half
  static constexpr int DMA = TM > 128 ? 4 : 3;      // direct-to-LDS loads per wave and k-tile (2 B + 1 or 2 A)
  static constexpr int NS0 = (160 * 1024) / (STAGE * 16);
  static constexpr int NS = NS0 > 8 ? 8 : NS0;      // ring stages: all of the 160 KiB LDS (5 .. 8)
};

// PROBE: one workgroup in the middle of the grid also records shader-clock cycles and 100 MHz
// wall ticks of its prologue, k loop and epilogue into probe[0..7] (a measurement aid: the
// clock under this kernel is set by the chip's power management, not by the nominal 2.4 GHz).
// OUT = 3: the Q|K|V projection with RoPE and the scatter into q / the K and V caches in its epilogue
// (the launch then replaces the projection's fp32 output and the separate RoPE + cache-write kernel).
struct RopeScatter {
  const int32_t* active_idx;   // [M] flat row ids
  const float2* rope_tab;      // [n_pad][64] (cos, sin)
  bf16_t* q;                   // [M, H*128] packed
  bf16_t* kc;                  // this layer's K cache, or null (queries only)
  bf16_t* vc;                  // this layer's V cache, or null
  int N, n_pad, H;
};

// One TM x 256 output tile (rows m0 .., column tile tn) by the whole 512-thread workgroup.
template <int OUT, int TM, bool PROBE>
__device__ __forceinline__ void ring_tile(
    const bf16_t* __restrict__ A, int a_tiled, const bf16_t* __restrict__ Wp, int n, int k, int k_per_split,
    const int M, int m_upper, float* __restrict__ Cf, bf16_t* __restrict__ Cb,
    const int32_t* __restrict__ row_map, size_t ldc, const int m0, const int tn, long long* __restrict__ probe,
    const RopeScatter& rs) {
  typedef TileCfg<TM> TC;
  constexpr int STAGE = TC::STAGE, NA = TC::NA, HL = TC::HL, HH = TC::HH, NS = TC::NS, A_FR = TC::A_FR;
  extern __shared__ Frag lds[];           // [NS stages][A: TM/32 mb x 2 kb | B: 8 nb x 2 kb][64 lanes]

  const int n0 = tn * TILE;
  const int kbeg = blockIdx.y * k_per_split;
  const int ktiles = k_per_split / BK2;
  const int last = ktiles - 1;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 2, wn = wave & 3;          // this wave's (TM/2) x 64 sub-tile
  const int K16 = k / 16, NB32 = n / 32;

  // global -> LDS: wave w moves the two B fragments of column block w and one or two of the A_FR
  // fragments of A (fragment f = row block f / 2, k half f % 2, at byte f * 1024 of the stage): f = w
  // for tiles of at most 128 rows, f = 2 w and 2 w + 1 above, taken modulo A_FR (a wave without a
  // fragment of its own repeats another wave's load, same bytes to the same place, so that every wave
  // issues the same number of loads per k-tile and one wait count serves all).
  // A is row-major [m_upper, k] (a 32 x 16 fragment is gathered from 32 rows) or already
  // fragment-tiled (one contiguous 1 KiB block per fragment, rows padded to 32).
  const bf16_t* Ab = a_tiled ? A : A + kbeg;
  const int a_kt_stride = a_tiled ? 2 * 512 : BK2, a_kb_stride = a_tiled ? 512 : 16;   // elements
  constexpr int NAF = TC::DMA - 2;                    // A fragments this wave fetches per k-tile
  uint32_t a_off[NAF], a_slot[NAF];                   // per-lane element offset, byte offset inside the stage
#pragma unroll
  for (int i = 0; i < NAF; ++i) {
    const int f = (NAF == 2 ? 2 * wave + i : wave) % A_FR;
    const int a_mb = f >> 1, a_kb = f & 1;
    a_slot[i] = (uint32_t)f * 1024u;
    if (a_tiled) {
      int mbg = m0 / 32 + a_mb;
      // row tail: stay inside the buffer (blocks past the end read valid blocks; their products are never stored)
      const int n_mb = (m_upper + 31) / 32;
      mbg = mbg < n_mb ? mbg : mbg % n_mb;
      a_off[i] = (((uint32_t)mbg * (uint32_t)K16 + (uint32_t)(kbeg / 16)) * 64u + (uint32_t)lane) * 8u +
                 (uint32_t)(a_kb * a_kb_stride);
    } else {
      int row = m0 + a_mb * 32 + (lane & 31);
      row = row < m_upper ? row : row % m_upper;        // row tail: stay inside the buffer
      a_off[i] = (uint32_t)row * (uint32_t)k + (uint32_t)((lane >> 5) * 8) + (uint32_t)(a_kb * a_kb_stride);
    }
  }
  const Frag* Wf = reinterpret_cast<const Frag*>(Wp) + (size_t)(kbeg / 16) * 64;
  uint32_t b_off;
  {
    int nb = n0 / 32 + wave;
    nb = nb < NB32 ? nb : NB32 - 1;                   // column tail: valid but unused data
    b_off = (uint32_t)nb * (uint32_t)K16 * 64u + (uint32_t)lane;
  }
  // Direct-to-LDS loads are issued as inline assembly on purpose: when the compiler sees an
  // LDS-DMA instruction it makes every later LDS read wait for ALL of them (vmcnt(0)), which
  // would collapse the ring to a depth of one.  Here the code itself guarantees, with explicit
  // vmcnt waits and the barrier, that a stage is read only after its loads have landed.
  // The hardware writes lane L's 16 bytes at M0 + 16*L.
  // Addressing is split so that almost all of it is scalar work: the per-lane part of a global
  // address is a 32-bit byte offset computed once, the per-tile part a 64-bit scalar base
  // (instruction form "vgpr offset + sgpr base"), and the LDS destination a scalar sum on a
  // base read once per wave.
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) Frag*)lds);
  const uint32_t wave_u = __builtin_amdgcn_readfirstlane((uint32_t)wave);
  uint32_t lds_a[NAF], a_voff[NAF];
#pragma unroll
  for (int i = 0; i < NAF; ++i) {
    lds_a[i] = lds_base + __builtin_amdgcn_readfirstlane(a_slot[i]);                      // this wave's A slot(s)
    a_voff[i] = a_off[i] * 2u;                                                            // bytes
  }
  const uint32_t lds_b = lds_base + (uint32_t)A_FR * 1024u + wave_u * 2048u;              // ... and B slots
  const uint32_t b_voff0 = b_off * 16u, b_voff1 = b_voff0 + 1024u;
  const uint64_t a_base = (uint64_t)(uintptr_t)Ab, b_base = (uint64_t)(uintptr_t)Wf;
  const uint32_t a_kt_bytes = (uint32_t)a_kt_stride * 2u;
  // (no immediate offsets: an instruction offset would be added to the LDS address as well)
  // Weight loads carry the non-temporal hint (each weight byte is wanted by at most a few
  // workgroups at about the same time and never again in the launch): measured 1 % at 1024
  // rows to 4 % at 256 rows on the whole step.
#define SL_DMA(voff, sbase, m0val, hint)                                                        \
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" hint               \
               :                                                                                \
               : "v"(voff), "s"(sbase), "s"(m0val)                                              \
               : "memory", "m0")
  auto issue = [&](int kt, int st) {
    kt = kt < last ? kt : last;                       // past the end: re-fetch the last tile (never used)
    const uint32_t so = (uint32_t)(st * STAGE) * 16u, lb = lds_b + so;
    const uint64_t ga = a_base + (uint64_t)kt * a_kt_bytes, gb = b_base + (uint64_t)kt * (128u * 16u);
    SL_DMA(a_voff[0], ga, lds_a[0] + so, "");
    SL_DMA(b_voff0, gb, lb, " nt");
    if (NAF == 2) SL_DMA(a_voff[NAF - 1], ga, lds_a[NAF - 1] + so, "");
    SL_DMA(b_voff1, gb, lb + 1024u, " nt");
  };
#undef SL_DMA

  // acc[a][b]: rows 16a .. 16a+15, columns 16b .. 16b+15 of this wave's sub-tile; lane l
  // holds row l % 16, columns 4 * (l / 16) .. +3
  f32x4 acc[NA][4];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  // 16 x 32 operand out of the 32 x 16 blocks of a stage: lane l wants row l % 16 and the 8 k of
  // group g = l / 16, i.e. slot (l % 16) + 32 * (g % 2) of k-block g / 2; a second 16-row half
  // of a block is 16 slots further on
  const int frag_lane = (lane >> 5) * 64 + ((lane >> 4) & 1) * 32 + (lane & 15);
  const Frag* sa0 = lds + frag_lane;                                 // 32-row block j of the tile at j * 128
  const Frag* sb0 = lds + A_FR * 64 + wn * 2 * 128 + frag_lane;      // 32-column block 2*wn + i
  // 16-row block a of this wave's sub-tile is 16-row block wm * NA + a of the tile: half (.. & 1) of 32-row block (.. >> 1)
  auto a_frag = [&](int st, int a) { const int g = wm * NA + a; return sa0[st * STAGE + (g >> 1) * 128 + (g & 1) * 16]; };
  auto b_frag = [&](int st, int b) { return sb0[st * STAGE + (b >> 1) * 128 + (b & 1) * 16]; };
  // A fragments of the first HL / the last HH 16-row blocks of the sub-tile, B fragments of two successive k-tiles
  Frag a_lo[HL], a_hi[HH], b_even[4], b_odd[4];
  // in the order the MFMAs consume them: (a0,b0) (a0,b1) (a0,b2) (a0,b3) (a1,*) ...
  auto read_tile_head = [&](int st, Frag (&af)[HL], Frag (&bf)[4]) {
    bf[0] = b_frag(st, 0);
    af[0] = a_frag(st, 0);
#pragma unroll
    for (int b = 1; b < 4; ++b) bf[b] = b_frag(st, b);
#pragma unroll
    for (int a = 1; a < HL; ++a) af[a] = a_frag(st, a);
  };
  auto read_tile_rest = [&](int st, Frag (&af)[HH]) {
#pragma unroll
    for (int a = 0; a < HH; ++a) af[a] = a_frag(st, HL + a);
  };
  auto mma_lo = [&](const Frag (&af)[HL], const Frag (&bf)[4]) {
#pragma unroll
    for (int a = 0; a < HL; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[b], af[a], acc[a][b], 0, 0, 0);
  };
  auto mma_hi = [&](const Frag (&af)[HH], const Frag (&bf)[4]) {
#pragma unroll
    for (int a = 0; a < HH; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        acc[HL + a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[b], af[a], acc[HL + a][b], 0, 0, 0);
  };
  // "s_waitcnt vmcnt(DMA*(NS-2))": all but this wave's newest NS-2 tiles have landed (loads
  // complete in order, DMA per tile per wave)
#define SL_WAIT_RING() asm volatile("s_waitcnt vmcnt(%0)" ::"n"(TC::DMA * (NS - 2)) : "memory")

  // NR LDS reads slotted one each behind the first MFMAs of a group of NM: the wave's issue slot is blocked
  // while the MFMA pipe is busy anyway, so the reads issue for free (short tiles have fewer MFMAs than reads
  // in their second half: the reads left over follow the group)
#define SL_INTERLEAVE(NR, NM)                                                              \
  do {                                                                                     \
    constexpr int nr_ = (NR) < (NM) ? (NR) : (NM);                                         \
    _Pragma("unroll") for (int q_ = 0; q_ < nr_; ++q_) {                                   \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   \
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                   \
    }                                                                                      \
    if constexpr ((NM) > nr_) __builtin_amdgcn_sched_group_barrier(0x008, (NM) - nr_, 0);   \
    if constexpr ((NR) > nr_) __builtin_amdgcn_sched_group_barrier(0x100, (NR) - nr_, 0);   \
  } while (0)
  long long pc0 = 0, pw0 = 0, pc1 = 0, pw1 = 0, pc2 = 0, pw2 = 0;
  if (PROBE) { pc0 = clock64(); pw0 = wall_clock64(); }
  // prologue: tiles 0 .. NS-2 in flight, tile 0 landed and published, its first fragments read
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) issue(t, t);
  SL_WAIT_RING();
  __syncthreads();
  read_tile_head(0, a_lo, b_even);

  // One k-tile per step: refill the stage every wave finished reading before the previous
  // barrier, multiply the first HL 16-row blocks of the sub-tile while reading the A fragments of
  // the other HH, wait for tile kt+1 and publish it, multiply the upper half while reading the
  // first fragments of tile kt+1.  B fragments alternate between two register sets, hence two steps per trip.
  if (PROBE) { pc1 = clock64(); pw1 = wall_clock64(); }
  int st = 0;                                         // stage of tile kt
  auto step = [&](int kt, Frag (&b_cur)[4], Frag (&b_next)[4]) {
    const int st_prev = st == 0 ? NS - 1 : st - 1;
    const int st_next = st == NS - 1 ? 0 : st + 1;
    issue(kt + NS - 1, st_prev);
    read_tile_rest(st, a_hi);
    mma_lo(a_lo, b_cur);
    SL_INTERLEAVE(HH, 4 * HL);
    __builtin_amdgcn_sched_barrier(0);
    SL_WAIT_RING();                                   // this wave's share of tile kt+1 has landed
    __syncthreads();                                  // ... and so has everyone else's
    read_tile_head(st_next, a_lo, b_next);
    mma_hi(a_hi, b_cur);
    SL_INTERLEAVE(4 + HL, 4 * HH);
    __builtin_amdgcn_sched_barrier(0);
    st = st_next;
  };
  int kt = 0;
  for (; kt + 1 < ktiles; kt += 2) {
    step(kt, b_even, b_odd);
    step(kt + 1, b_odd, b_even);
  }
  if (kt < ktiles) step(kt, b_even, b_odd);
  if (PROBE) { pc2 = clock64(); pw2 = wall_clock64(); }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // drain the (unused) tail re-fetches
#undef SL_WAIT_RING
#undef SL_INTERLEAVE

  const int row_in = lane & 15, col_in = 4 * (lane >> 4);   // this lane's place in a 16 x 16 block
  if (OUT == 1 || OUT == 4) {
    // OUT = 4: the residual add in the epilogue, Cb [m, n] row-major <- rnd(Cb + sums) in place (each
    // element belongs to exactly one workgroup, which reads it before it writes it).
    // bf16 rows: a lane's piece of a row is 8 bytes, scattered over 16 rows per instruction.  The
    // ring is drained, so each wave stages its 128 x 64 sub-tile in LDS as bf16 (row stride 144
    // bytes) with 8-byte writes and sends it out as 16-byte stores, eight lanes per 128-byte
    // row segment.
    __syncthreads();                                  // every wave is done reading operand stages
    constexpr int RS = 72;                            // bf16 elements per staged row
    bf16_t* stage = reinterpret_cast<bf16_t*>(lds) + (size_t)wave * (TM / 2) * RS;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        bf16x4 v4;
        if (OUT == 4) {
          const int row = m0 + wm * (TM / 2) + a * 16 + row_in, col = n0 + wn * 64 + b * 16 + col_in;
          bf16x4 x4 = {(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
          if (row < M && col < n) x4 = *reinterpret_cast<const bf16x4*>(Cb + (size_t)row * ldc + col);
#pragma unroll
          for (int v = 0; v < 4; ++v) v4[v] = (bf16_t)((float)x4[v] + acc[a][b][v]);
        } else {
#pragma unroll
          for (int v = 0; v < 4; ++v) v4[v] = (bf16_t)acc[a][b][v];
        }
        *reinterpret_cast<bf16x4*>(stage + (a * 16 + row_in) * RS + b * 16 + col_in) = v4;
      }
    // same-wave LDS traffic is ordered; no barrier needed between a wave's writes and its reads
    const int chunk = lane & 7, rsub = lane >> 3;
    const int col = n0 + wn * 64 + chunk * 8;
#pragma unroll
    for (int it = 0; it < TM / 16; ++it) {
      const int r = it * 8 + rsub;
      const int row = m0 + wm * (TM / 2) + r;
      const Frag val = *reinterpret_cast<const Frag*>(stage + r * RS + chunk * 8);
      if (row < M && col < n) {
        const size_t orow = row_map ? (size_t)row_map[row] : (size_t)row;
        // streaming store: these rows (the step's logits, 259 MB at M = 1024) are read once by the
        // next kernel and would otherwise sit dirty in the memory-side cache and be written back
        // under that kernel's reads (scoring 111 -> 99 us)
        if (OUT == 4) *reinterpret_cast<Frag*>(Cb + orow * ldc + col) = val;     // read again by the norm kernel
        else __builtin_nontemporal_store(val, reinterpret_cast<Frag*>(Cb + orow * ldc + col));
      }
    }
    if (PROBE) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 // the stores have left
      const long long pc3 = clock64(), pw3 = wall_clock64();
      if (blockIdx.x == ((gridDim.x >> 1) & ~7u) && threadIdx.x == 0) {
        probe[0] = pc1 - pc0; probe[1] = pc2 - pc1; probe[2] = pc3 - pc2;
        probe[3] = pw1 - pw0; probe[4] = pw2 - pw1; probe[5] = pw3 - pw2;
        probe[6] = gridDim.x; probe[7] = ktiles;
      }
    }
    return;
  }
  if (OUT == 2) {
    // columns are gate/up interleaved by 32-column blocks: of a wave's 64 columns the first 32
    // are gate columns c .. c+31 and the last 32 the up columns of the same c (n = 2 d_ff,
    // ldc = d_ff), so accumulators b and b+2 of a lane pair up.  silu(g) * u is staged per wave
    // as a 128 x 32 bf16 block and leaves as 16-byte stores: eight consecutive columns of a row
    // are contiguous in the fragment-tiled layout.
    __syncthreads();
    constexpr int RS = 40;
    bf16_t* stage = reinterpret_cast<bf16_t*>(lds) + (size_t)wave * (TM / 2) * RS;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        bf16x4 v4;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float g = acc[a][b][v], u = acc[a][b + 2][v];
          v4[v] = (bf16_t)(g / (1.0f + expf(-g)) * u);
        }
        *reinterpret_cast<bf16x4*>(stage + (a * 16 + row_in) * RS + b * 16 + col_in) = v4;
      }
    const int chunk = lane & 3, rsub = lane >> 2;
    const int c = (n0 / 64 + wn) * 32 + chunk * 8;
#pragma unroll
    for (int it = 0; it < TM / 32; ++it) {
      const int r = it * 16 + rsub;
      const int row = m0 + wm * (TM / 2) + r;
      const Frag val = *reinterpret_cast<const Frag*>(stage + r * RS + chunk * 8);
      if (row < M && c < (n >> 1)) *reinterpret_cast<Frag*>(Cb + afrag_index(row, c, (int)ldc)) = val;
    }
    return;
  }
  if (OUT == 3) {
    // n = 3 H 128 columns = [q | k | v], each a whole number of 256-column tiles: this tile holds two
    // heads of one of the three.  RoPE pairs dims j and j + 64 of a head, which sit in two different
    // waves, and the caches want 16-byte units along dims (K) or along slots (V): the fp32 sums go
    // through LDS 128 rows at a time (the drained ring's space), then all 512 threads rotate, round
    // and store.  RoPE is applied to the unrounded sums, like the stand-alone kernel does.
    constexpr int RSf = 260;                          // floats per staged row (16-byte aligned, banks spread)
    float* stage = reinterpret_cast<float*>(lds);
    int* slot_sh = reinterpret_cast<int*>(stage + 128 * RSf);      // [128] flat ids of the staged rows, -1 past M
    int* dense_sh = slot_sh + 128;                                 // [8] per 16-row group (V stores)
    const int hd = rs.H * 128;
    const int sec = n0 / hd;                          // 0 q, 1 k, 2 v
    const int head0 = (n0 - sec * hd) >> 7;
    const int tid = threadIdx.x;
#pragma unroll 1
    for (int p = 0; p < (TM + 127) / 128; ++p) {
      __syncthreads();                                // operand stages (or the previous pass) are done with
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        const int trow = wm * (TM / 2) + a * 16;      // this 16-row block's first row inside the tile
        if (trow / 128 != p) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b)
          *reinterpret_cast<f32x4*>(stage + (trow - p * 128 + row_in) * RSf + wn * 64 + b * 16 + col_in) = acc[a][b];
      }
      if (tid < 128) {
        const int row = m0 + p * 128 + tid;
        slot_sh[tid] = (p * 128 + tid < TM && row < M) ? rs.active_idx[row] : -1;
      }
      __syncthreads();
      if (sec < 2) {
        if (sec == 1 && rs.kc == nullptr) continue;   // queries only (uniform over the workgroup)
#pragma unroll 1
        for (int it = 0; it < 4; ++it) {
          const int item = tid + it * 512;
          const int r = item >> 4, hh = (item >> 3) & 1, c = item & 7;
          const int g = slot_sh[r];
          if (g < 0) continue;
          const int bb = g / rs.N, i = g - bb * rs.N;
          const float* x1 = stage + r * RSf + hh * 128 + c * 8;
          const float4* cs = reinterpret_cast<const float4*>(rs.rope_tab + (size_t)i * 64 + c * 8);
          bf16x8 o1, o2;
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const float4 t = cs[e2];                  // (cos, sin) of pairs 2 e2 and 2 e2 + 1
            const float a0 = x1[2 * e2], b0 = x1[64 + 2 * e2], a1 = x1[2 * e2 + 1], b1 = x1[64 + 2 * e2 + 1];
            o1[2 * e2] = (bf16_t)(a0 * t.x - b0 * t.y);
            o2[2 * e2] = (bf16_t)(b0 * t.x + a0 * t.y);
            o1[2 * e2 + 1] = (bf16_t)(a1 * t.z - b1 * t.w);
            o2[2 * e2 + 1] = (bf16_t)(b1 * t.z + a1 * t.w);
          }
          const int head = head0 + hh;
          if (sec == 0) {
            bf16_t* qr = rs.q + (size_t)(m0 + p * 128 + r) * hd + head * 128 + c * 8;
            *reinterpret_cast<bf16x8*>(qr) = o1;
            *reinterpret_cast<bf16x8*>(qr + 64) = o2;
          } else {
            bf16_t* kb = rs.kc + ((size_t)bb * rs.H + head) * rs.n_pad * 128;
            *reinterpret_cast<bf16x8*>(kb + kc_index(i, c * 8, 128)) = o1;
            *reinterpret_cast<bf16x8*>(kb + kc_index(i, 64 + c * 8, 128)) = o2;
          }
        }
      } else {
        if (rs.vc == nullptr) continue;
        // V: 16 consecutive rows that are the 16 consecutive slots of one aligned block leave as
        // 16-byte groups of eight slots per dim; other rows as 2-byte stores
        if (tid < 8) {
          const int g0 = slot_sh[tid * 16];
          bool dense = g0 >= 0 && (g0 % rs.N) % 16 == 0 && (g0 % rs.N) + 16 <= rs.N;
          for (int jx = 1; jx < 16 && dense; ++jx) dense = slot_sh[tid * 16 + jx] == g0 + jx;
          dense_sh[tid] = dense;
        }
        __syncthreads();
#pragma unroll 1
        for (int it = 0; it < 8; ++it) {
          const int item = tid + it * 512;
          const int vdim = item & 127, vcg = (item >> 7) & 1, hh = (item >> 8) & 1, gi = item >> 9;
          const int head = head0 + hh;
          const float* col = stage + (gi * 16) * RSf + hh * 128 + vdim;
          if (dense_sh[gi]) {
            const int g0 = slot_sh[gi * 16];
            const int bb = g0 / rs.N, i0 = g0 - bb * rs.N;
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = vcache_half_bits(col[((e >> 2) * 8 + 4 * vcg + (e & 3)) * RSf]);
            *reinterpret_cast<bf16x8*>(rs.vc + ((size_t)bb * rs.H + head) * rs.n_pad * 128 + vc_index(i0 + 4 * vcg, vdim, 128)) = o;
          } else {
#pragma unroll 1
            for (int e = 0; e < 8; ++e) {
              const int lr = (e >> 2) * 8 + 4 * vcg + (e & 3);
              const int g = slot_sh[gi * 16 + lr];
              if (g < 0) continue;
              const int bb = g / rs.N, i = g - bb * rs.N;
              rs.vc[((size_t)bb * rs.H + head) * rs.n_pad * 128 + vc_index(i, vdim, 128)] = vcache_half_bits(col[lr * RSf]);
            }
          }
        }
      }
    }
    return;
  }
  // fp32 partial plane of this k-split: 16 bytes per lane, 64 contiguous bytes per row
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    const int row = m0 + wm * (TM / 2) + a * 16 + row_in;
    if (row >= M) continue;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int col = n0 + wn * 64 + b * 16 + col_in;
      if (col < n) *reinterpret_cast<f32x4*>(Cf + ((size_t)blockIdx.y * m_upper + row) * ldc + col) = acc[a][b];
    }
  }
}

// Workgroup -> tile.  Consecutive workgroups go to consecutive XCDs (blockIdx.x = 8 * j + xcd), each with an
// L2 of its own that holds a few k-steps of the ~32 tiles its CUs work on at a time; XCD x owns the column
// tiles 8 c + x.  Operand bytes that leave an L2 are about (distinct row tiles + distinct column tiles) among
// those 32, per k-step: 33 when an XCD walks down one column tile after the other, 12 for 8 x 4 tiles.  An
// XCD therefore walks bands of gn of its column tiles, column fastest, so that the tiles in flight form a
// block of about (32 / gn) x gn.  Measured at 8192 rows: L2 fetch bytes of the layer projections halve from
// gn = 1 to gn = 4 and the launches get 2 to 5 % faster; wider bands and splitting the rows over XCDs
// (which fetches every weight tile into several L2s) are slower at few row tiles.
struct TileMap {
  int gn, cn;        // band width; column tiles per XCD
};
__device__ inline bool tile_of_workgroup(const TileMap& tmap, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int full = tmap.cn / tmap.gn * tmap.gn;     // column tiles in whole bands
  int c;
  if (j < tiles_m * full) {
    const int band = j / (tiles_m * tmap.gn), q = j - band * tiles_m * tmap.gn;
    tm = q / tmap.gn;
    c = band * tmap.gn + q % tmap.gn;
  } else {
    const int q = j - tiles_m * full, w = tmap.cn - full;
    tm = q / w;
    c = full + q % w;
  }
  tn = c * 8 + xcd;
  return tm < tiles_m && tn < tiles_n;
}
static TileMap pick_tile_map(int tiles_m, int tiles_n) {
  const int cn = sl_cdiv(tiles_n, 8), gn = tiles_m >= 16 ? 4 : 2;
  return TileMap{gn < cn ? gn : cn, cn};
}

template <int OUT, int TM, bool PROBE = false>
__global__ __launch_bounds__(512, 2) void gemm_mfma256_kernel(
    const bf16_t* __restrict__ A, int a_tiled, const bf16_t* __restrict__ Wp, int n, int k, int k_per_split,
    const int32_t* __restrict__ m_dev, int m_upper, float* __restrict__ Cf, bf16_t* __restrict__ Cb,
    const int32_t* __restrict__ row_map, size_t ldc, int tiles_m, int tiles_n, TileMap tmap,
    long long* __restrict__ probe, RopeScatter rs) {
  const int M = min(*m_dev, m_upper);
  int tm, tn;
  if (!tile_of_workgroup(tmap, tiles_m, tiles_n, tm, tn) || tm * TM >= M) return;
  ring_tile<OUT, TM, PROBE>(A, a_tiled, Wp, n, k, k_per_split, M, m_upper, Cf, Cb, row_map, ldc, tm * TM, tn, probe, rs);
}

// Full-height row tiles followed by ONE half-height tile for a row tail of at most 128 rows
// (tiles_m counts both kinds): the tail then costs 0.565 of a full tile instead of a whole one.
template <int OUT>
__global__ __launch_bounds__(512, 2) void gemm_mfma256_tail_kernel(
    const bf16_t* __restrict__ A, int a_tiled, const bf16_t* __restrict__ Wp, int n, int k, int k_per_split,
    const int32_t* __restrict__ m_dev, int m_upper, float* __restrict__ Cf, bf16_t* __restrict__ Cb,
    const int32_t* __restrict__ row_map, size_t ldc, int tiles_m, int tiles_n, TileMap tmap, RopeScatter rs) {
  const int M = min(*m_dev, m_upper);
  int tm, tn;
  if (!tile_of_workgroup(tmap, tiles_m, tiles_n, tm, tn) || tm * TILE >= M) return;
  if (tm == tiles_m - 1)
    ring_tile<OUT, 128, false>(A, a_tiled, Wp, n, k, k_per_split, M, m_upper, Cf, Cb, row_map, ldc, tm * TILE, tn, nullptr, rs);
  else
    ring_tile<OUT, 256, false>(A, a_tiled, Wp, n, k, k_per_split, M, m_upper, Cf, Cb, row_map, ldc, tm * TILE, tn, nullptr, rs);
}

template <int OUT, int TM>
static int launch_ring(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                       int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc, const RopeScatter& rs) {
  const int tiles_m = sl_cdiv(mu, TM), tiles_n = sl_cdiv(n, TILE);
  const size_t sh = (size_t)TileCfg<TM>::NS * TileCfg<TM>::STAGE * 16;
  auto kern = gemm_mfma256_kernel<OUT, TM>;
  static unsigned long long lds_ok = 0;              // one per kernel instantiation
  SL_ALLOW_DYNAMIC_LDS(lds_ok, kern, sh);
  const TileMap tmap = pick_tile_map(tiles_m, tiles_n);
  dim3 grid(8 * tiles_m * tmap.cn, splits), block(512);
  hipLaunchKernelGGL(kern, grid, block, sh, s, (const bf16_t*)A, a_tiled, (const bf16_t*)Wp, n, k, k / splits, m_dev, mu, Cf,
                     (bf16_t*)Cb, row_map, ldc, tiles_m, tiles_n, tmap, (long long*)nullptr, rs);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

// ---- tile heights of a launch ------------------------------------------------------------------
// Cost model in units of one full-height tile's time on 256 CUs: a full round of workgroups costs 1, a
// last partial round 0.9 whatever its fill (measured: the busy CUs of a partial round run at a higher
// clock), a tile of TM rows kTileCost[TM / 32] of a full one.
// A launch runs either uniform tiles of one height (any multiple of 32 from 64 to 256: the smallest
// number of row tiles that covers the rows, or more and shorter ones where that saves a round of
// workgroups), or, for many rows, full-height tiles plus ONE half-height tile for a row tail of at
// most 128 rows.  Fewer, taller tiles win near-ties (less operand traffic per flop).
static double ring_rounds_cost(int workgroups) {
  return workgroups / 256 + (workgroups % 256 ? 0.9 : 0.0);
}
// measured on the LM head (one row tile of TM rows) and on the layer projections: a k-tile step has a
// floor of about 0.4 us however short the tile (barrier, LDS latency, the 16 KiB of weights per step)
static const double kTileCost[9] = {0, 0, 0.51, 0.55, 0.565, 0.70, 0.78, 0.86, 1.0};   // by TM / 32

struct RingChoice {
  int tail;        // 1: full-height tiles + one half-height tail tile
  int tm;          // rows per tile (uniform launches)
  double cost;     // in full-tile rounds
};
static RingChoice ring_choice(int mu, int n, int splits) {
  const int tn = sl_cdiv(n, TILE) * splits;
  RingChoice best{0, 256, 1e30};
  const int t_min = sl_cdiv(mu, 256), t_max = sl_cdiv(mu, 64);
  for (int t = t_min; t <= t_max; ++t) {
    int tm = (int)sl_align_up((size_t)sl_cdiv(mu, t), 32);
    if (tm < 64) tm = 64;
    if (sl_cdiv(mu, tm) != t) continue;              // the same height with fewer tiles was already priced
    const double c = ring_rounds_cost(t * tn) * kTileCost[tm / 32];
    if (c < 0.97 * best.cost) best = RingChoice{0, tm, c};
  }
  const int t_full = sl_cdiv(mu, 256);
  const int tail = mu - (t_full - 1) * 256;          // rows of the last full-height tile
  if (t_full > 1 && tail <= 128) {
    // Every workgroup takes a CU's one slot whatever its tile height, so the rounds are those of the
    // workgroup COUNT; a CU's share is a mix of full tiles and half tiles in the launch's proportion.
    // (Pricing the launch by its work alone, as if the short tiles packed into the gaps, chose this form
    // for 640 rows x 96 column tiles, 288 workgroups in two rounds: 145 us where five 128-row tiles per
    // column tile take 117 us.)
    // (one round: the launch lasts as long as its full tiles do)
    const double half_share = t_full * tn > 256 ? 1.0 / t_full : 0.0;
    const double mixed = ring_rounds_cost(t_full * tn) * (1.0 - half_share * (1.0 - kTileCost[4]));
    if (mixed < 0.95 * best.cost) best = RingChoice{1, 256, mixed};
  }
  return best;
}

// cost of the cheapest ring launch for (mu rows, n columns, `splits` k-splits), in full-tile rounds
double slk_ring_cost(int mu, int n, int splits) { return ring_choice(mu, n, splits).cost; }
void slk_ring_describe(int mu, int n, int splits, int* rows, int* tail) {
  const RingChoice c = ring_choice(mu, n, splits);
  *rows = c.tm;
  *tail = c.tail;
}

template <int OUT>
static int launch_ring_tail(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n,
                            int k, int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc, const RopeScatter& rs) {
  const int tiles_m = sl_cdiv(mu, TILE), tiles_n = sl_cdiv(n, TILE);
  const size_t sh = 160 * 1024;                                                // the larger of the two rings
  auto kern = gemm_mfma256_tail_kernel<OUT>;
  static unsigned long long lds_ok = 0;
  SL_ALLOW_DYNAMIC_LDS(lds_ok, kern, sh);
  const TileMap tmap = pick_tile_map(tiles_m, tiles_n);
  dim3 grid(8 * tiles_m * tmap.cn, splits), block(512);
  hipLaunchKernelGGL(kern, grid, block, sh, s, (const bf16_t*)A, a_tiled, (const bf16_t*)Wp, n, k, k / splits, m_dev, mu, Cf,
                     (bf16_t*)Cb, row_map, ldc, tiles_m, tiles_n, tmap, rs);
  SL_LAUNCH_CHECK();
  return SL_OK;
}

template <int OUT>
static int launch256(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                     int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc,
                     const RopeScatter& rs = RopeScatter{}) {
  const RingChoice c = ring_choice(mu, n, splits);
  if (c.tail) return launch_ring_tail<OUT>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
  switch (c.tm) {
    case 64: return launch_ring<OUT, 64>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
    case 96: return launch_ring<OUT, 96>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
    case 128: return launch_ring<OUT, 128>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
    case 160: return launch_ring<OUT, 160>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
    case 192: return launch_ring<OUT, 192>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
    case 224: return launch_ring<OUT, 224>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
    default: return launch_ring<OUT, 256>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, Cb, row_map, ldc, rs);
  }
}

int slk_gemm_mfma256(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n,
                     int k, int splits, float* Cf, void* Cb, const int32_t* row_map, size_t ldc) {
  if (mu <= 0) return SL_OK;
  if (splits < 1 || n % 32 || k % (BK2 * splits) || k / (BK2 * splits) < 8) return SL_EINVAL;
  if (!Cf && splits != 1) return SL_EINVAL;
  if (Cf && ((uintptr_t)Cf % 16 || ldc % 4)) return SL_EINVAL;       // 16-byte fp32 stores
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;
  return Cf ? launch256<0>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, Cf, nullptr, nullptr, ldc)
            : launch256<1>(s, A, a_tiled, Wp, m_dev, mu, n, k, splits, nullptr, Cb, row_map, ldc);
}

// The LM-head launch (bf16 rows, no split) with the cycle probe switched on; probe = 8 int64 on the device.
int slk_gemm_mfma256_probe(hipStream_t s, const void* A, int a_tiled, const void* Wp, const int32_t* m_dev, int mu, int n,
                           int k, void* Cb, const int32_t* row_map, size_t ldc, long long* probe) {
  if (mu <= 0 || !probe || !Cb) return SL_EINVAL;
  if (n % 32 || k % BK2 || k / BK2 < 8) return SL_EINVAL;
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;
  const int tiles_m = sl_cdiv(mu, TILE), tiles_n = sl_cdiv(n, TILE);
  const size_t sh = (size_t)TileCfg<256>::NS * TileCfg<256>::STAGE * 16;
  auto kern = gemm_mfma256_kernel<1, 256, true>;
  static unsigned long long lds_ok = 0;
  SL_ALLOW_DYNAMIC_LDS(lds_ok, kern, sh);
  const TileMap tmap = pick_tile_map(tiles_m, tiles_n);
  dim3 grid(8 * tiles_m * tmap.cn, 1), block(512);
  hipLaunchKernelGGL(kern, grid, block, sh, s, (const bf16_t*)A, a_tiled, (const bf16_t*)Wp, n, k, k, m_dev, mu,
                     (float*)nullptr, (bf16_t*)Cb, row_map, ldc, tiles_m, tiles_n, tmap, probe, RopeScatter{});
  SL_LAUNCH_CHECK();
  return SL_OK;
}

int slk_gemm_mfma256_swiglu(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int dff, int k,
                            void* a) {
  if (mu <= 0) return SL_OK;
  const int n = 2 * dff;
  if (dff % 32 || k % BK2 || k / BK2 < 8) return SL_EINVAL;
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;
  return launch256<2>(s, A, 1, Wp, m_dev, mu, n, k, 1, nullptr, a, nullptr, (size_t)dff);
}

// Q|K|V projection + RoPE + scatter in one launch: q [mu, H*128] packed bf16, K / V into the layer's
// cache at the rows' own slots (kc = vc = null: queries only).  Unsplit only (k / 32 >= 8); H even, so
// that a 256-column tile is two whole heads of q, k or v.
int slk_gemm_mfma256_qkv_rope(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int H, int k,
                              const int32_t* active_idx, int N, int n_pad, const void* rope_tab, void* q, void* kc,
                              void* vc) {
  if (mu <= 0) return SL_OK;
  const int n = 3 * H * 128;
  if (H < 2 || H % 2 || k % BK2 || k / BK2 < 8 || !active_idx || !rope_tab || !q) return SL_EINVAL;
  if ((kc == nullptr) != (vc == nullptr)) return SL_EINVAL;
  if ((uintptr_t)q % 16 || (uintptr_t)kc % 16 || (uintptr_t)vc % 16 || (uintptr_t)rope_tab % 16) return SL_EINVAL;
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;
  const RopeScatter rs{active_idx, (const float2*)rope_tab, (bf16_t*)q, (bf16_t*)kc, (bf16_t*)vc, N, n_pad, H};
  return launch256<3>(s, A, 1, Wp, m_dev, mu, n, k, 1, nullptr, nullptr, nullptr, (size_t)n, rs);
}

// x [mu, n] bf16 row-major <- rnd(x + A W^T) in place: a projection with the residual add in its
// epilogue (unsplit only; n % 8 == 0 for the 16-byte row pieces).
int slk_gemm_mfma256_residual(hipStream_t s, const void* A, const void* Wp, const int32_t* m_dev, int mu, int n, int k,
                              void* x) {
  if (mu <= 0) return SL_OK;
  if (n % 32 || k % BK2 || k / BK2 < 8 || !x || (uintptr_t)x % 16) return SL_EINVAL;
  if ((size_t)n * k >= ((size_t)1 << 31) * 8 || (size_t)mu * k >= ((size_t)1 << 32)) return SL_EINVAL;
  return launch256<4>(s, A, 1, Wp, m_dev, mu, n, k, 1, nullptr, x, nullptr, (size_t)n);
}
