// bf16 matrix-core GEMM whose operand tiles go from global memory straight into LDS (gfx950's 16-byte
// global_load_lds), for all three operand layouts of the path step.
//
// Tile 256 x 256 (A tile | B tile per stage), eight waves of 128 x 64 outputs, and a ring of LDS stages: K tiles of 32
// in a ring of four stages of 32 KB, or K tiles of 64 in a ring of two of 64 KB.  One wave-level load writes 1024
// consecutive LDS bytes (lane l writes bytes [16 l, 16 l + 16)), so the LDS layout is linear in the lane and
// every permutation is applied on the global side, by choosing which 16 bytes a lane fetches:
//   * operand contiguous along K ([rows, K] in memory): tile row r is 64 bytes = 4 chunks, chunk c at chunk position
//     c ^ ((r >> 2) & 3) (K tile 32), or 128 bytes = 8 chunks = one whole cache line per row and request, chunk c at
//     c ^ ((r >> 1) & 7) (K tile 64).  A fragment is one ds_read_b128, free of bank conflicts for the lane groups
//     the LDS serves together: lane l reads row l % 32, K half l / 32 of a 16-deep step for v_mfma_f32_32x32x16_bf16,
//     row l % 16, K quarter l / 16 of a 32-deep step for v_mfma_f32_16x16x32_bf16.
//   * operand contiguous along its rows ([K, rows] in memory: the forward weights, both operands of a weight
//     gradient): tile K-row t is 512 bytes = 8 segments of 32 rows; segment s sits at segment position
//     s ^ (t & 3), and K-rows whose index has bit 3 set keep the two 16-row halves of every segment swapped (the
//     sixteen-lane groups of one fragment read then fall on different banks in both pipelines below).  Fragments
//     are read with ds_read_b64_tr_b16, which transposes 4 x 4 halfword blocks across each group of 16 lanes: when
//     lane 4e+q of a group points at rows 4q..4q+3 of K-row T(e), lane i receives row i of K-rows T(0..3).  Two such
//     reads (K-rows 8h+0..3 and 8h+4..7) build the same 8-deep fragment a K-contiguous operand gives, so any mix of
//     the two kinds multiplies correctly.
// No operand passes through registers on its way to LDS, which leaves room for the 256 x 256 accumulator at two
// waves per SIMD and lets loads run up to three K tiles ahead.
//
// Two pipelines share all of this and the epilogues: gemm_dlds_wave16 on v_mfma_f32_16x16x32_bf16, the default (the
// chip sustains about 15 % more of that shape at its power limit), and gemm_dlds_wave on v_mfma_f32_32x32x16_bf16,
// kept as a tested option.  Pipeline of one K tile in the latter (one barrier): [fragments of the tile's second half
// are read under the MFMAs of its first half] -> own loads of the next tile have landed (s_waitcnt vmcnt) -> barrier
// (everybody's have, and everybody is done reading this stage) -> [this stage is refilled with the tile one ring
// ahead and the next tile's first fragments are read, both under the MFMAs of the second half]; the former is
// described at its function.  The loads are inline assembly: written with the builtin, the compiler puts a full
// vmcnt(0) in front of every later LDS read, which serialises the ring.
#include <algorithm>
#include <cmath>
#include <type_traits>

#include "gemm_common.h"
#include "kernels.h"

namespace dipaco {

namespace {

constexpr int DL_BK_MIN = 32;                               // K tiles are 32 or 64 deep

typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;

__device__ __forceinline__ void load16_to_lds(const bf16* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}
// the same with a wave-uniform base address (scalar registers) and a 32-bit per-lane byte offset
__device__ __forceinline__ void load16_to_lds_at(const char* base, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {   // vmcnt only: expcnt and lgkmcnt fields at maximum
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Load plan of one wave: wave-level load j of a stage fills LDS bytes [1024 j, 1024 j + 1024) of it; j < NLA: A tile, else
// B tile.  Load i of this wave is j = wave + NW i: its lane's source at K tile 0 (gp), the source's advance per K tile
// (gstep) and the LDS address in stage 0 (ldst).  Rows (columns) beyond the operand re-read its last ones: they only
// feed outputs that are never stored.
template <bool A_KC, bool B_KC, int DL_BM, int DL_BN, int NW, int DL_BK, int LPS>
__device__ __forceinline__ void dlds_load_plan(const GemmDev& g, const char* smem, int lane, int wave, int m0, int n0,
                                               int k_begin, const bf16* (&gp)[LPS], long (&gstep)[LPS],
                                               uint32_t (&ldst)[LPS]) {
  constexpr int DL_ROWB = DL_BK * 2;
  constexpr int NLA = DL_BM * DL_ROWB / 1024;
  const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
#pragma unroll
  for (int i = 0; i < LPS; ++i) {
    const int j = wave + NW * i;
    const bool is_a = j < NLA;
    const int jj = is_a ? j : j - NLA;
    const bf16* base = static_cast<const bf16*>(is_a ? g.A : g.B);
    const long ld = is_a ? g.lda : g.ldb;
    const int r0 = is_a ? m0 : n0, rtot = is_a ? g.M : g.N;
    if (is_a ? A_KC : B_KC) {
      // a wave-level load covers 16 rows of 64 bytes or 8 rows of 128 bytes (whole cache lines: half the requests)
      constexpr int LPR = DL_ROWB / 16, RPL = 64 / LPR;     // lanes per row, rows per load
      const int trow = RPL * jj + lane / LPR;               // row within the tile
      const int row = min(r0 + trow, rtot - 1);
      const int chunk = DL_BK == 32 ? (lane & 3) ^ ((trow >> 2) & 3) : (lane & 7) ^ ((trow >> 1) & 7);
      gp[i] = base + (long)row * ld + k_begin + chunk * 8;
      gstep[i] = DL_BK;
    } else {
      // log2 of the 16-byte chunks per K-row: 4, 5, 6 for tiles 128, 256, 512 wide
      constexpr int SH_A = DL_BM == 512 ? 6 : (DL_BM == 256 ? 5 : 4), SH_B = DL_BN == 512 ? 6 : (DL_BN == 256 ? 5 : 4);
      static_assert((DL_BM == 128 || DL_BM == 256 || DL_BM == 512) && (DL_BN == 128 || DL_BN == 256 || DL_BN == 512),
                    "tile sides of 128, 256 or 512");
      const int sh = is_a ? SH_A : SH_B;
      const int t = (64 >> sh) * jj + (lane >> sh);
      const int cp = lane & ((1 << sh) - 1);
      const int seg = (cp >> 2) ^ (t & 3);
      const int c4 = (cp & 3) ^ (((t >> 3) & 1) << 1);       // K-rows 8..15 (mod 16) keep their 16-row halves swapped
      const int col = min(r0 + (seg * 4 + c4) * 8, rtot - 8);
      gp[i] = base + (long)(k_begin + t) * ld + col;
      gstep[i] = (long)DL_BK * ld;
    }
    ldst[i] = smem_base + j * 1024;
  }
}

// The same plan with wave-uniform bases: a lane keeps one 32-bit byte offset per load (its place inside the operand, K
// tile 0), the operand's base and its advance per K tile are scalars, so a load costs no vector address arithmetic.
// Offsets stay below 2^32: rows x row stride x 2 of a K-contiguous operand is checked on the host.
struct DldsBases {
  const char* a;      // operand A at this product's first K position
  const char* b;
  long adv_a, adv_b;  // bytes per K tile
};
template <bool A_KC, bool B_KC, int DL_BM, int DL_BN, int NW, int DL_BK, int LPS>
__device__ __forceinline__ DldsBases dlds_load_plan_s(const GemmDev& g, const char* smem, int lane, int wave, int m0, int n0,
                                                      int k_begin, uint32_t (&off)[LPS], uint32_t (&ldst)[LPS]) {
  constexpr int DL_ROWB = DL_BK * 2;
  constexpr int NLA = DL_BM * DL_ROWB / 1024;
  const uint32_t smem_base = (uint32_t)(uintptr_t)smem;
  DldsBases o;
  o.a = static_cast<const char*>(g.A) + (A_KC ? (long)k_begin : (long)k_begin * g.lda) * 2;
  o.b = static_cast<const char*>(g.B) + (B_KC ? (long)k_begin : (long)k_begin * g.ldb) * 2;
  o.adv_a = A_KC ? DL_ROWB : (long)DL_BK * g.lda * 2;
  o.adv_b = B_KC ? DL_ROWB : (long)DL_BK * g.ldb * 2;
#pragma unroll
  for (int i = 0; i < LPS; ++i) {
    const int j = wave + NW * i;
    const bool is_a = j < NLA;
    const int jj = is_a ? j : j - NLA;
    const uint32_t ld = (uint32_t)(is_a ? g.lda : g.ldb);
    const int r0 = is_a ? m0 : n0, rtot = is_a ? g.M : g.N;
    if (is_a ? A_KC : B_KC) {
      constexpr int LPR = DL_ROWB / 16, RPL = 64 / LPR;
      const int trow = RPL * jj + lane / LPR;
      const int row = min(r0 + trow, rtot - 1);
      const int chunk = DL_BK == 32 ? (lane & 3) ^ ((trow >> 2) & 3) : (lane & 7) ^ ((trow >> 1) & 7);
      off[i] = ((uint32_t)row * ld + (uint32_t)chunk * 8u) * 2u;
    } else {
      constexpr int SH_A = DL_BM == 512 ? 6 : (DL_BM == 256 ? 5 : 4), SH_B = DL_BN == 512 ? 6 : (DL_BN == 256 ? 5 : 4);
      const int sh = is_a ? SH_A : SH_B;
      const int t = (64 >> sh) * jj + (lane >> sh);
      const int cp = lane & ((1 << sh) - 1);
      const int seg = (cp >> 2) ^ (t & 3);
      const int c4 = (cp & 3) ^ (((t >> 3) & 1) << 1);
      const int col = min(r0 + (seg * 4 + c4) * 8, rtot - 8);
      off[i] = ((uint32_t)t * ld + (uint32_t)col) * 2u;
    }
    ldst[i] = smem_base + j * 1024;
  }
  return o;
}

// A_KC: A is [M, K] (contiguous along K), else [K, M].  B_KC: B is [N, K], else [K, N].
// Shapes built: 256 x 256 tiles, 2 x 4 waves, 4 stages (one workgroup per compute unit; least operand traffic, for
// long K); 256 x 128 tiles, 2 x 2 waves, 3 stages (two workgroups per compute unit); 128 x 512 and 512 x 128 for
// weight gradients.  In all of these a wave owns 128 x 64 outputs and two waves share a SIMD.
// N_STEP = 224 (with DL_BN = 256), an option: the tile is staged exactly like a 256 x 256 one, but tile columns start
// every 224 columns and only the first 224 are computed and stored.  The path's widths (896, 2688, 3584) are
// multiples of 224 = 7 x 32 and not of 256: 896 columns are 4 such tiles instead of 3.5, so a launch is a whole
// number of equal workgroups.  The 7 x 8 blocks of 32 x 32 are dealt so that every SIMD gets 14: waves 0..3 take
// 64 rows x 128 columns, waves 4..7 the same rows x the last 96.
template <typename TC, bool A_KC, bool B_KC, int DL_BM, int DL_BN, int WGM, int WGN, int DL_STAGES, int N_STEP, int DL_BK,
          int TM, int TN>
__device__ __forceinline__ void gemm_dlds_wave(const GemmDev& g, char* smem, int lane, int wave, int rb0, int cb0, int m0,
                                               int n0, int k_begin, int nkt, int split) {
  constexpr int NW = WGM * WGN;
  constexpr int DL_ROWB = DL_BK * 2;                        // bytes of a K-contiguous tile row: 64 or 128
  constexpr int KS = DL_BK / 16;                            // 16-deep matrix-core steps per K tile
  static_assert(DL_BK == 32 || DL_BK == 64, "K tiles of 32 or 64");
  constexpr int DL_TILE_A = DL_BM * DL_ROWB, DL_TILE_B = DL_BN * DL_ROWB;   // bytes of an operand tile (either kind)
  constexpr int DL_STAGE = DL_TILE_A + DL_TILE_B;
  constexpr int KROW_A = DL_BM * 2, KROW_B = DL_BN * 2;     // bytes of a K-row of a row-contiguous tile
  constexpr int NLA = DL_TILE_A / 1024;                     // wave-level loads of the A tile
  constexpr int LPS = DL_STAGE / 1024 / NW;                 // wave-level loads per wave and stage
  constexpr int NM = TM * TN, NR = TM + TN;
  const bool active = m0 + rb0 * 32 < g.M && n0 + cb0 * 32 < g.N;   // wave-uniform
  const bf16* gp[LPS];
  long gstep[LPS];
  uint32_t ldst[LPS];
  dlds_load_plan<A_KC, B_KC, DL_BM, DL_BN, NW, DL_BK, LPS>(g, smem, lane, wave, m0, n0, k_begin, gp, gstep, ldst);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // ---- fragment addresses ----
  const int r = lane & 31, h = lane >> 5;
  const int sw = DL_BK == 32 ? (r >> 2) & 3 : (r >> 1) & 7;
  int foff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) foff[ks] = r * DL_ROWB + ((2 * ks + h) ^ sw) * 16;
  const int g4 = lane >> 4, ep = (lane & 15) >> 2, qp = lane & 3;
  int toffa[TM], toffb[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
    toffa[i] = (8 * (g4 >> 1) + ep) * KROW_A + (((rb0 + i) ^ ep) * 64) + 32 * ((g4 & 1) ^ (g4 >> 1)) + 8 * qp;
#pragma unroll
  for (int j = 0; j < TN; ++j)
    toffb[j] = (8 * (g4 >> 1) + ep) * KROW_B + (((cb0 + j) ^ ep) * 64) + 32 * ((g4 & 1) ^ (g4 >> 1)) + 8 * qp;
  const char* a_base = smem + (A_KC ? rb0 * 32 * DL_ROWB : 0);
  const char* b_base = smem + DL_TILE_A + (B_KC ? cb0 * 32 * DL_ROWB : 0);
  uint4 fa[2][TM], fb[2][TN];
  auto tr_read = [&](const char* p, int krow) {
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)(uint32_t)(uintptr_t)p);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)(uint32_t)(uintptr_t)(p + 4 * krow));
    uint4 o;
    o.x = (uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
    o.y = (uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
    o.z = (uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
    o.w = (uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
    return o;
  };
  auto read_frag = [&](int set, int q, const char* as, const char* bs, int ks) {   // q-th of the NR fragments
    if (q < TM) {
      if (A_KC) fa[set][q] = *reinterpret_cast<const uint4*>(as + q * 32 * DL_ROWB + foff[ks]);
      else fa[set][q] = tr_read(as + toffa[q] + ks * 16 * KROW_A, KROW_A);
    } else {
      if (B_KC) fb[set][q - TM] = *reinterpret_cast<const uint4*>(bs + (q - TM) * 32 * DL_ROWB + foff[ks]);
      else fb[set][q - TM] = tr_read(bs + toffb[q - TM] + ks * 16 * KROW_B, KROW_B);
    }
  };
  auto mfma = [&](int set, int m) {
    const int i = m / TN, j = m % TN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[set][i]),
                                                        __builtin_bit_cast(bf16x8, fb[set][j]), acc[i][j], 0, 0, 0);
  };
  // own loads of every tile but the n newest have landed
  auto wait_newer = [&](int n) {
    if (DL_STAGES > 3 && n >= 3) wait_vmcnt<3 * LPS>();
    else if (n >= 2) wait_vmcnt<2 * LPS>();
    else if (n == 1) wait_vmcnt<LPS>();
    else wait_vmcnt<0>();
  };
  static_assert(DL_STAGES >= 2 && DL_STAGES <= 4, "wait_newer handles rings of two to four");
  static_assert(3 * LPS < 64, "the counter of outstanding loads has six bits");
  static_assert(LPS <= NM, "a stage's loads are dealt over the MFMAs of one step");

  // prologue: the first DL_STAGES tiles, one per stage
#pragma unroll
  for (int s = 0; s < DL_STAGES; ++s)
    if (s < nkt) {
#pragma unroll
      for (int i = 0; i < LPS; ++i) load16_to_lds(gp[i] + s * gstep[i], ldst[i] + s * DL_STAGE);
    }
  wait_newer(min(nkt, DL_STAGES) - 1);
  __syncthreads();
  if (active) {
#pragma unroll
    for (int q = 0; q < NR; ++q) read_frag(0, q, a_base, b_base, 0);
  }

  // One K tile of KS matrix-core steps.  FULL: tile kt + DL_STAGES exists (steady state: no conditions).  Fragment sets
  // alternate (KS is even, so the first step of every tile uses set 0); the fragments of step ks + 1 are read under the
  // MFMAs of step ks; the barrier stands in front of the tile's last step, whose MFMAs cover the refill of this stage
  // and the first fragments of the next.
  auto step = [&](auto FULL, int kt, int stage) {
    constexpr bool full = decltype(FULL)::value;
    const char* as = a_base + stage * DL_STAGE;
    const char* bs = b_base + stage * DL_STAGE;
    const int nst = stage + 1 == DL_STAGES ? 0 : stage + 1;
    const char* as2 = a_base + nst * DL_STAGE;
    const char* bs2 = b_base + nst * DL_STAGE;
    const bool have_next = full || kt + 1 < nkt;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      if (ks + 1 < KS) {
        if (active) {
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            if ((m * NR) % NM < NR && (m * NR) / NM < NR) read_frag(nxt, (m * NR) / NM, as, bs, ks + 1);
            mfma(cur, m);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      } else {
        if (full) wait_vmcnt<(DL_STAGES - 2) * LPS>();
        else wait_newer(max(nkt - 2 - kt, 0));
        __syncthreads();
        if (active) {
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            if (full && (m * LPS) % NM < LPS && (m * LPS) / NM < LPS) {
              const int q = (m * LPS) / NM;
              load16_to_lds(gp[q] + (kt + DL_STAGES) * gstep[q], ldst[q] + stage * DL_STAGE);
            }
            if (have_next && (m * NR) % NM < NR && (m * NR) / NM < NR) read_frag(nxt, (m * NR) / NM, as2, bs2, 0);
            mfma(cur, m);
            __builtin_amdgcn_sched_barrier(0);
          }
        } else if (full) {   // a wave without output still loads its share of the tiles
#pragma unroll
          for (int q = 0; q < LPS; ++q) load16_to_lds(gp[q] + (kt + DL_STAGES) * gstep[q], ldst[q] + stage * DL_STAGE);
        }
      }
    }
  };
  int stage = 0, kt = 0;
  for (; kt + DL_STAGES < nkt; ++kt) {
    step(std::true_type{}, kt, stage);
    stage = stage + 1 == DL_STAGES ? 0 : stage + 1;
  }
  for (; kt < nkt; ++kt) {
    step(std::false_type{}, kt, stage);
    stage = stage + 1 == DL_STAGES ? 0 : stage + 1;
  }

  // every load has landed (the last steps waited for vmcnt 0); all waves are done with the ring before it is reused
  wait_vmcnt<0>();
  __syncthreads();
  if (!active) return;
  // the epilogue takes column blocks of two (or one) 32-wide tiles at a time through the wave's staging region
  float* const stg = reinterpret_cast<float*>(smem) + wave * (32 * (64 + 4));
  const int row0 = m0 + rb0 * 32;
  // (column blocks by compile-time index: a run-time loop over acc would move the accumulators to scratch memory)
  auto block = [&](auto J0) {
    constexpr int j0 = decltype(J0)::value;
    if constexpr (j0 + 1 == TN) {
      f32x16 part[TM][1];
#pragma unroll
      for (int i = 0; i < TM; ++i) part[i][0] = acc[i][j0];
      gemm_epilogue_dispatch<TC, TM, 1, 32>(part, stg, lane, row0, n0 + (cb0 + j0) * 32, split, g);
    } else {
      f32x16 part[TM][2];
#pragma unroll
      for (int i = 0; i < TM; ++i) { part[i][0] = acc[i][j0]; part[i][1] = acc[i][j0 + 1]; }
      gemm_epilogue_dispatch<TC, TM, 2, 64>(part, stg, lane, row0, n0 + (cb0 + j0) * 32, split, g);
    }
  };
  static_assert(TN >= 1 && TN <= 4, "one or two column blocks per wave");
  block(std::integral_constant<int, 0>{});
  if constexpr (TN > 2) {
    if (n0 + (cb0 + 2) * 32 < g.N) block(std::integral_constant<int, 2>{});   // wave-uniform
  }
}

// The same tile pipeline on v_mfma_f32_16x16x32_bf16 (a wave's 128 x 64 outputs are 8 x 4 tiles of 16 x 16; one
// matrix-core step is 32 deep).  On operands that are not all zero the chip sustains about 15 % more of these than of
// the 32 x 32 x 16 shape at its power limit: half the accumulator traffic per flop.
//   fragments: lane l holds row (column) l % 16 and K positions 8 (l / 16) .. + 7 of the step: in a K-contiguous tile
//   that is one ds_read_b128 (chunk 4 s + l / 16 of the row, at its swizzled position); in a row-contiguous tile two
//   transposing reads of K-rows 32 s + 8 (l / 16) + 0..3 and + 4..7.
// Registers: the four B fragments of a step are double-buffered (the next step's are read under rows 4..7 of this
// one); the eight A fragments pass through a window of four slots, each read three rows of MFMAs ahead of its use.
// The barrier of a K tile stands in row 4 of its last step, behind the read of the tile's last A fragment: after it
// the stage is refilled and every read goes to the next stage.
template <typename TC, bool A_KC, bool B_KC, int DL_BM, int DL_BN, int WGM, int WGN, int DL_STAGES, int DL_BK>
__device__ __forceinline__ void gemm_dlds_wave16(const GemmDev& g, char* smem, int lane, int wave, int rb0, int cb0, int m0,
                                                 int n0, int k_begin, int nkt, int split) {
  constexpr int NW = WGM * WGN;
  constexpr int DL_ROWB = DL_BK * 2;
  constexpr int KS = DL_BK / 32;                            // 32-deep matrix-core steps per K tile
  static_assert(DL_BK == 32 || DL_BK == 64, "K tiles of 32 or 64");
  constexpr int DL_TILE_A = DL_BM * DL_ROWB, DL_TILE_B = DL_BN * DL_ROWB;
  constexpr int DL_STAGE = DL_TILE_A + DL_TILE_B;
  constexpr int KROW_A = DL_BM * 2, KROW_B = DL_BN * 2;
  constexpr int LPS = DL_STAGE / 1024 / NW;
  constexpr int NA = 8, NB = 4, AHEAD = 3, SLOTS = 4;
  static_assert(LPS <= 16, "a stage's loads are dealt over the sixteen MFMAs behind the barrier");
  static_assert(DL_STAGES >= 2 && DL_STAGES <= 4 && 3 * LPS < 64, "ring of two to four stages; six-bit load counter");
  const bool active = m0 + rb0 * 32 < g.M && n0 + cb0 * 32 < g.N;   // wave-uniform
  constexpr int NLA = DL_TILE_A / 1024;
  uint32_t off[LPS], ldst[LPS];
  const DldsBases bases = dlds_load_plan_s<A_KC, B_KC, DL_BM, DL_BN, NW, DL_BK, LPS>(g, smem, lane, wave, m0, n0, k_begin, off, ldst);
  // load q of this wave for K tile kt into `stage` (which operand it belongs to is wave-uniform)
  auto issue = [&](int q, int kt, int stage) {
    const bool is_a = wave + NW * q < NLA;
    const char* base = (is_a ? bases.a : bases.b) + (long)kt * (is_a ? bases.adv_a : bases.adv_b);
    load16_to_lds_at(base, off[q], ldst[q] + stage * DL_STAGE);
  };

  f32x4 acc[NA][NB];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // ---- fragment addresses (byte offsets within a stage's A or B tile) ----
  const int m16 = lane & 15, g4 = lane >> 4, ep = (lane & 15) >> 2, qp = lane & 3;
  const int sw = DL_BK == 32 ? (m16 >> 2) & 3 : (m16 >> 1) & 7;
  int koff[KS];                                             // K-contiguous tile: chunk of step s in this lane's row
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) koff[ks] = m16 * DL_ROWB + ((4 * ks + g4) ^ sw) * 16;
  int toffa[NA], toffb[NB];                                 // row-contiguous tile: this lane's 8 bytes of K-row 8 g4 + ep
#pragma unroll
  for (int q = 0; q < NA; ++q) {
    const int blk = 2 * rb0 + q;                            // 16-row block within the tile
    toffa[q] = (8 * g4 + ep) * KROW_A + (((blk >> 1) ^ ep) * 64) + 32 * ((blk ^ g4) & 1) + 8 * qp;
  }
#pragma unroll
  for (int q = 0; q < NB; ++q) {
    const int blk = 2 * cb0 + q;
    toffb[q] = (8 * g4 + ep) * KROW_B + (((blk >> 1) ^ ep) * 64) + 32 * ((blk ^ g4) & 1) + 8 * qp;
  }
  const char* a_base = smem + (A_KC ? rb0 * 32 * DL_ROWB : 0);
  const char* b_base = smem + DL_TILE_A + (B_KC ? cb0 * 32 * DL_ROWB : 0);
  auto tr_read = [&](const char* p, int krow) {
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)(uint32_t)(uintptr_t)p);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)(uint32_t)(uintptr_t)(p + 4 * krow));
    uint4 o;
    o.x = (uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
    o.y = (uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
    o.z = (uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
    o.w = (uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
    return o;
  };
  uint4 aw[SLOTS], bf[2][NB];
  auto read_a = [&](int q, const char* as, int ks) {        // A fragment q of step ks of the stage at `as`
    if (A_KC) aw[q % SLOTS] = *reinterpret_cast<const uint4*>(as + q * 16 * DL_ROWB + koff[ks]);
    else aw[q % SLOTS] = tr_read(as + toffa[q] + ks * 32 * KROW_A, KROW_A);
  };
  auto read_b = [&](int set, int q, const char* bs, int ks) {
    if (B_KC) bf[set][q] = *reinterpret_cast<const uint4*>(bs + q * 16 * DL_ROWB + koff[ks]);
    else bf[set][q] = tr_read(bs + toffb[q] + ks * 32 * KROW_B, KROW_B);
  };
  // own loads of every tile but the n newest have landed
  auto wait_newer = [&](int n) {
    if (DL_STAGES > 3 && n >= 2) wait_vmcnt<2 * LPS>();
    else if (DL_STAGES > 2 && n == 1) wait_vmcnt<LPS>();
    else wait_vmcnt<0>();
  };

  // prologue: the first DL_STAGES tiles, one per stage
#pragma unroll
  for (int s = 0; s < DL_STAGES; ++s)
    if (s < nkt) {
#pragma unroll
      for (int i = 0; i < LPS; ++i) issue(i, s, s);
    }
  // tile 0 has landed when at most the loads of the tiles behind it are outstanding
  if (nkt >= 4 && DL_STAGES >= 4) wait_vmcnt<3 * LPS>();
  else if (nkt >= 3 && DL_STAGES >= 3) wait_vmcnt<2 * LPS>();
  else if (nkt >= 2) wait_vmcnt<LPS>();
  else wait_vmcnt<0>();
  __syncthreads();
  if (active) {
#pragma unroll
    for (int q = 0; q < NB; ++q) read_b(0, q, b_base, 0);
#pragma unroll
    for (int q = 0; q < AHEAD; ++q) read_a(q, a_base, 0);
  }

  // One matrix-core step (32 deep).  SET: which B buffer it multiplies with (steps alternate).  STEADY: tile
  // kt + DL_STAGES exists, so the refill and every prefetch are unconditional.  ks: the step within its K tile.
  auto kstep = [&](auto SETc, auto STEADYc, auto KSc, int kt, int stage) {
    constexpr int set = decltype(SETc)::value, ks = decltype(KSc)::value;
    constexpr bool steady = decltype(STEADYc)::value;
    constexpr bool last = ks == KS - 1;                      // the tile's last step: barrier, refill, on to the next stage
    const char* as = a_base + stage * DL_STAGE;
    const char* bs = b_base + stage * DL_STAGE;
    const int nst = stage + 1 == DL_STAGES ? 0 : stage + 1;
    const char* as2 = last ? a_base + nst * DL_STAGE : as;   // where the next step's fragments are
    const char* bs2 = last ? b_base + nst * DL_STAGE : bs;
    constexpr int ks2 = last ? 0 : ks + 1;
    const bool have_next = steady || !last || kt + 1 < nkt;
    const bool refill = steady || kt + DL_STAGES < nkt;
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      if (active) {
        if (i + AHEAD < NA) read_a(i + AHEAD, as, ks);
        else if (have_next) read_a(i + AHEAD - NA, as2, ks2);
      }
      if (last && i == 4) {
        // own loads of tile kt + 1 have landed: all but those of the tiles behind it that are already requested
        if (steady) wait_vmcnt<(DL_STAGES - 2) * LPS>();
        else wait_newer(min(DL_STAGES - 2, max(nkt - 2 - kt, 0)));
        __syncthreads();
      }
      if (active) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          if (last && i >= 4) {
            const int mm = (i - 4) * NB + j;                 // 0..15: the MFMAs behind the barrier
            if (refill && (mm * LPS) % 16 < LPS && (mm * LPS) / 16 < LPS) {
              const int q = (mm * LPS) / 16;
              issue(q, kt + DL_STAGES, stage);
            }
          }
          if (i >= 4 && j == 0 && have_next) read_b(set ^ 1, i - 4, bs2, ks2);
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, aw[i % SLOTS]),
                                                              __builtin_bit_cast(bf16x8, bf[set][j]), acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else if (last && i == 4 && refill) {   // a wave without output still loads its share of the tiles
#pragma unroll
        for (int q = 0; q < LPS; ++q) issue(q, kt + DL_STAGES, stage);
      }
    }
  };
  using C0 = std::integral_constant<int, 0>;
  using C1 = std::integral_constant<int, 1>;
  int stage = 0, kt = 0;
  auto next_stage = [&] { stage = stage + 1 == DL_STAGES ? 0 : stage + 1; };
  if constexpr (KS == 2) {
    for (; kt + DL_STAGES < nkt; ++kt) {
      kstep(C0{}, std::true_type{}, C0{}, kt, stage);
      kstep(C1{}, std::true_type{}, C1{}, kt, stage);
      next_stage();
    }
    for (; kt < nkt; ++kt) {
      kstep(C0{}, std::false_type{}, C0{}, kt, stage);
      kstep(C1{}, std::false_type{}, C1{}, kt, stage);
      next_stage();
    }
  } else {
    for (; kt + 1 + DL_STAGES < nkt; kt += 2) {
      kstep(C0{}, std::true_type{}, C0{}, kt, stage);
      next_stage();
      kstep(C1{}, std::true_type{}, C0{}, kt + 1, stage);
      next_stage();
    }
    for (; kt < nkt; kt += 2) {
      kstep(C0{}, std::false_type{}, C0{}, kt, stage);
      next_stage();
      if (kt + 1 < nkt) {
        kstep(C1{}, std::false_type{}, C0{}, kt + 1, stage);
        next_stage();
      }
    }
  }

  // every load has landed (the last steps waited for vmcnt 0); all waves are done with the ring before it is reused
  wait_vmcnt<0>();
  __syncthreads();
  if (!active) return;
  float* const stg = reinterpret_cast<float*>(smem) + wave * (32 * (64 + 4));
  gemm_epilogue_dispatch<TC, 4, 2, 64>(acc, stg, lane, m0 + rb0 * 32, n0 + cb0 * 32, split, g);
}

template <typename TC, bool A_KC, bool B_KC, int DL_BM, int DL_BN, int WGM, int WGN, int DL_STAGES, int N_STEP, int DL_BK,
          int MI>
__global__ void __launch_bounds__(64 * WGM * WGN, 2)
gemm_dlds_kernel(const GemmDev g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int split, tile_m, tile_n, k_begin, nkt;
  if (g.uneven) {
    int nsplit;
    gemm_uneven_of_block(g, blockIdx.x, split, nsplit, tile_m, tile_n);
    const long ktiles = g.K / DL_BK;
    const int kt0 = (int)(split * ktiles / nsplit), kt1 = (int)((split + 1) * ktiles / nsplit);
    k_begin = kt0 * DL_BK;
    nkt = kt1 - kt0;
  } else if (g.fast_map) {
    gemm_tile_of_block_fast(g, blockIdx.x, tile_m, tile_n);
    split = 0;
    k_begin = 0;
    nkt = g.K / DL_BK;
  } else {
    gemm_tile_of_block(g, blockIdx.x, split, tile_m, tile_n);
    k_begin = split * g.k_per_split;
    nkt = (min(g.K, k_begin + g.k_per_split) - k_begin) / DL_BK;
  }
  const int m0 = tile_m * DL_BM, n0 = tile_n * N_STEP;
  if constexpr (N_STEP == 224) {
    static_assert(DL_BM == 256 && DL_BN == 256 && WGM == 2 && WGN == 4, "the 224-column tile is staged as 256 x 256");
    // waves w and w + 4 share a SIMD: 2 x 4 + 2 x 3 = 14 blocks of 32 x 32 each
    if (wave < 4)
      gemm_dlds_wave<TC, A_KC, B_KC, DL_BM, DL_BN, WGM, WGN, DL_STAGES, N_STEP, DL_BK, 2, 4>(g, smem, lane, wave, 2 * wave, 0, m0,
                                                                                      n0, k_begin, nkt, split);
    else
      gemm_dlds_wave<TC, A_KC, B_KC, DL_BM, DL_BN, WGM, WGN, DL_STAGES, N_STEP, DL_BK, 2, 3>(g, smem, lane, wave, 2 * (wave - 4), 4,
                                                                                      m0, n0, k_begin, nkt, split);
  } else {
    static_assert(N_STEP == DL_BN, "tiles tile C");
    // Waves w and w + 4 share a SIMD.  They are given different halves of the tile's rows AND of its columns, so
    // that in a tile that sticks out of C by half (896 = 3.5 x 256 is the path's width) every SIMD keeps exactly
    // one wave with work, which then has the matrix core to itself.  (Letting the idle wave of the SIMD take half of
    // every K tile of its partner's outputs was measured: no gain, the launch is not bound by that wave's latencies.)
    static_assert((WGM == 2 && (WGN == 4 || WGN == 2)) || (WGM == 1 && WGN == 8) || (WGM == 4 && WGN == 2),
                  "wave placement below is written for 2 x 4, 2 x 2, 1 x 8 and 4 x 2 waves");
    constexpr int TNW = DL_BN / (32 * WGN);
    static_assert(DL_BM / (32 * WGM) == 4 && TNW == 2, "a wave owns 128 x 64 outputs");
    const int wm = WGM == 1 ? 0 : WGM == 4 ? (wave & 3) : (WGN == 4 ? (wave & 1) ^ (wave >> 2) : wave >> 1);
    const int wn = WGM == 1 ? wave : WGM == 4 ? (wave >> 2) : (WGN == 4 ? 2 * (wave >> 2) + ((wave >> 1) & 1) : wave & 1);
    if constexpr (MI == 16) {
      static_assert(TNW == 2, "the 16 x 16 x 32 pipeline is written for 128 x 64 outputs per wave");
      gemm_dlds_wave16<TC, A_KC, B_KC, DL_BM, DL_BN, WGM, WGN, DL_STAGES, DL_BK>(g, smem, lane, wave, 4 * wm, 2 * wn, m0, n0,
                                                                                k_begin, nkt, split);
    } else {
      gemm_dlds_wave<TC, A_KC, B_KC, DL_BM, DL_BN, WGM, WGN, DL_STAGES, N_STEP, DL_BK, 4, TNW>(g, smem, lane, wave, 4 * wm,
                                                                                        TNW * wn, m0, n0, k_begin, nkt, split);
    }
  }
}

// ---- uneven split-K ----------------------------------------------------------------------------------------
// Cost of one K step of a tile in which only the fraction `frac` of the waves has work, relative to a full tile
// (measured: 0.73 for half a tile -- the operand loads are the same, the matrix-core work halves).
double partial_tile_cost(double frac) { return 0.5 + 0.5 * frac; }

struct UnevenPlan {
  int s[4];          // K slices per class; s[0] = the largest
  int n[4];          // tiles per class
  double cost[4];    // cost of a K step of a tile of the class, a full tile = 1
  int full_m, full_n;
};

// The largest slice count <= max_slices such that every tile class c, cut into ceil(cost_c * s) slices, still
// gives at most one workgroup per compute unit.  False if there is no such plan with at least two slices.
bool plan_uneven(int M, int N, int K, int BM, int BN, int WGM, int WGN, int max_slices, UnevenPlan& p) {
  constexpr int CUS = 256;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  if ((long)tiles_m * tiles_n > CUS / 2) return false;
  const int rm = M - (tiles_m - 1) * BM, rn = N - (tiles_n - 1) * BN;
  const int WM = BM / WGM, WN = BN / WGN;
  const double am = (double)((rm + WM - 1) / WM) / WGM, an = (double)((rn + WN - 1) / WN) / WGN;
  p.full_m = tiles_m - (am < 1.0 ? 1 : 0);
  p.full_n = tiles_n - (an < 1.0 ? 1 : 0);
  p.n[0] = p.full_m * p.full_n;
  p.n[1] = (tiles_m - p.full_m) * p.full_n;
  p.n[2] = p.full_m * (tiles_n - p.full_n);
  p.n[3] = (tiles_m - p.full_m) * (tiles_n - p.full_n);
  const double w[4] = {1.0, partial_tile_cost(am), partial_tile_cost(an), partial_tile_cost(am * an)};
  for (int c = 0; c < 4; ++c) p.cost[c] = w[c];
  const int ktiles = K / DL_BK_MIN;
  for (int sf = std::min(max_slices, ktiles); sf >= 2; --sf) {
    long total = 0;
    for (int c = 0; c < 4; ++c) {
      p.s[c] = std::min(sf, std::max(1, (int)std::ceil(w[c] * sf - 1e-9)));
      total += (long)p.n[c] * p.s[c];
    }
    if (total <= CUS) return true;
  }
  return false;
}

// Length of the longest workgroup of a plan, in K steps of a full tile per unit of K
double plan_makespan(const UnevenPlan& p) {
  double worst = 0.0;
  for (int c = 0; c < 4; ++c)
    if (p.n[c] > 0) worst = std::max(worst, p.cost[c] / p.s[c]);
  return worst;
}

template <typename TC, bool A_KC, bool B_KC, int DL_BM, int BN, int WGM, int WGN, int STAGES, int N_STEP = BN, int DL_BK = 32,
          int MI = 32>
dipaco_status run_dlds(const GemmArgs& a, hipStream_t s) {
  constexpr size_t smem = (size_t)STAGES * (DL_BM + BN) * DL_BK * 2;
  static_assert((size_t)WGM * WGN * 32 * (64 + 4) * sizeof(float) <= smem, "epilogue staging fits in the ring");
  auto kern = gemm_dlds_kernel<TC, A_KC, B_KC, DL_BM, BN, WGM, WGN, STAGES, N_STEP, DL_BK, MI>;
  static std::atomic<unsigned long long> lds_set{0};   // per instantiation
  if (dipaco_status e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return e;
  GemmDev g;
  g.A = a.A; g.B = a.B; g.C = a.C; g.M = a.M; g.N = a.N; g.K = a.K;
  g.lda = a.lda; g.ldb = a.ldb; g.ldc = a.ldc;
  g.bias = a.bias; g.resid = a.resid; g.aux_out = a.aux_out; g.aux_in = a.aux_in; g.act = a.act;
  g.partial = a.partial;
  g.tiles_m = (a.M + DL_BM - 1) / DL_BM;
  g.tiles_n = (a.N + N_STEP - 1) / N_STEP;
  const int ktiles = a.K / DL_BK;
  UnevenPlan up;
  if (N_STEP != BN && (a.splits > 1 || a.N % N_STEP)) return fail(DIPACO_EUNSUPPORTED, "gemm: 224-column tiles need N % 224 == 0 and no split-K");
  if (a.splits > 1 && plan_uneven(a.M, a.N, a.K, DL_BM, BN, WGM, WGN, a.splits, up)) {
    g.uneven = 1;
    g.splits = up.s[0];
    g.k_per_split = 0;
    g.full_m = up.full_m; g.full_n = up.full_n;
    g.cls_base[0] = 0;
    for (int c = 0; c < 4; ++c) { g.cls_s[c] = up.s[c]; g.cls_base[c + 1] = g.cls_base[c] + up.n[c] * up.s[c]; }
    kern<<<(unsigned)g.cls_base[4], 64 * WGM * WGN, smem, s>>>(g);
    DIPACO_LAUNCH_CHECK();
    return launch_splitk_reduce_classes(a.partial, static_cast<float*>(a.C), a.M, a.N, a.ldc, up.full_m * DL_BM,
                                        up.full_n * BN, up.s, s);
  }
  int splits = a.splits < 1 ? 1 : a.splits;
  if (splits > ktiles) splits = ktiles;
  g.k_per_split = ((ktiles + splits - 1) / splits) * DL_BK;
  g.splits = (a.K + g.k_per_split - 1) / g.k_per_split;
  const long blocks = (long)g.tiles_m * g.tiles_n * g.splits;
  if (blocks > 0x7fffffffL) return fail(DIPACO_ESHAPE, "gemm: too many tiles");
  g.colsum_partial = a.colsum ? a.colsum_partial : nullptr;
  gemm_fast_map(g);
  kern<<<(unsigned)blocks, 64 * WGM * WGN, smem, s>>>(g);
  DIPACO_LAUNCH_CHECK();
  if (g.splits > 1) return launch_splitk_reduce(a.partial, static_cast<float*>(a.C), a.M, a.N, a.ldc, g.splits, s);
  constexpr int WAVE_ROWS = N_STEP != BN ? 64 : DL_BM / WGM;   // rows whose column sums one wave leaves
  if (a.colsum) return launch_sum_rows(a.colsum_partial, a.colsum, (a.M + WAVE_ROWS - 1) / WAVE_ROWS, a.N, s, a.sum_batch);
  return DIPACO_OK;
}

// 0 = automatic (the 16 x 16 x 32 pipeline), 1 = 256 x 256 and 2 = 256 x 128 on the 32 x 32 x 16 pipeline, 3 / 4 = 128 x 512 /
// 512 x 128 forced for weight gradients, 5 = 224-column tiles wherever N is a multiple of 224, 6 = K tiles of 64 on the
// 32 x 32 x 16 pipeline, 7 / 8 = the 16 x 16 x 32 pipeline with K tiles of 32 only / of 64 where K allows.  A process-wide
// test and tuning hook.
std::atomic<int> g_dlds_shape{0};

// Weight gradients with a side that is not a multiple of 256 (896 = 7 x 128): 128 x 512 tiles of 1 x 8 waves, or
// 512 x 128 tiles of 4 x 2 waves, cut C into whole tiles only, so that five K slices fit on the chip where the
// 256 x 256 shape, whose last tile row (column) is half empty but costs 0.75, gets four.  An oblong tile moves
// 1.25 x the operand bytes per flop and has three stages: it is taken when its plan's longest workgroup is at
// least 8 % shorter.
// Returns 0 (keep 256 x 256), 1 (128 x 512) or 2 (512 x 128).
int oblong_plan_wins(const GemmArgs& a) {
  if (g_dlds_shape == 3) return 1;
  if (g_dlds_shape == 4) return 2;
  if (g_dlds_shape != 0 || a.splits <= 1) return 0;
  UnevenPlan sq, ob;
  const bool have_sq = plan_uneven(a.M, a.N, a.K, 256, 256, 2, 4, a.splits, sq);
  double best = have_sq ? 0.92 * plan_makespan(sq) : 1e30;
  int pick = 0;
  if (plan_uneven(a.M, a.N, a.K, 128, 512, 1, 8, a.splits, ob) && plan_makespan(ob) < best) { best = plan_makespan(ob); pick = 1; }
  if (plan_uneven(a.M, a.N, a.K, 512, 128, 4, 2, a.splits, ob) && plan_makespan(ob) < best) { best = plan_makespan(ob); pick = 2; }
  return pick;
}

// Tile columns every 224 instead of 256 (N a multiple of 224; see the kernel): one workgroup per compute unit either
// way, 7/8 of the matrix-core work per tile, whole rounds of 256 workgroups.  Measured on the step's products at
// equal flops: within +-2 % of the 256-column tiles where it removes a half-empty tile column or a quarter-full last
// round (N = 896, 2688), 8-10 % behind where it does not (N = 3584: one more tile column).  A tile's time follows the
// operand bytes it stages, not its matrix-core work, and the launch as a whole follows the power limit, so the
// saved work is not seen.  Kept as a tested option (tile setting 10); the automatic choice stays 256 x 256.

// Measured on the step's products (K = 896 .. 32768), the two-workgroup shape gains what it hides of a tile's ends
// and loses more to its extra barriers and operand traffic: level with the 256 x 256 shape on the GELU product, whose
// epilogue is the longest, 3-15 % behind on all others.  It is kept as a tested option; the automatic choice is the
// 256 x 256 shape.
template <typename TC, bool A_KC, bool B_KC>
dipaco_status run_dlds_shape(const GemmArgs& a, hipStream_t s) {
  const int shape = g_dlds_shape;
  // forced shapes of the 32 x 32 x 16 pipeline (tests and comparisons)
  if (shape == 1) return run_dlds<TC, A_KC, B_KC, 256, 256, 2, 4, 4>(a, s);
  if (shape == 2) return run_dlds<TC, A_KC, B_KC, 256, 128, 2, 2, 3>(a, s);
  if constexpr (std::is_same<TC, bf16>::value) {
    if (shape == 5 && a.splits <= 1 && a.N % 224 == 0 && gemm_epilogue_is_fixed(a.act, a.bias, a.resid, a.colsum))
      return run_dlds<TC, A_KC, B_KC, 256, 256, 2, 4, 4, 224>(a, s);
    if (shape == 6 && a.splits <= 1 && a.K % 64 == 0) return run_dlds<TC, A_KC, B_KC, 256, 256, 2, 4, 2, 256, 64>(a, s);
  }
  // the 16 x 16 x 32 pipeline: oblong tiles for the weight gradients whose plan they shorten; else K tiles of 64 in a ring
  // of two wherever K allows (whole cache lines per request, half the barriers; measured 2-5 % ahead of the ring of four
  // K tiles of 32 on every product of the step), else K tiles of 32 in a ring of four.  Measured on this pipeline and left
  // out: the 256 x 128 tile with two workgroups per compute unit (3-20 % behind on every product), and four waves of
  // 128 x 128 outputs, one per SIMD, which read a third less from LDS (5-20 % behind, the smaller figure with the
  // accumulators pinned to the accumulation registers: one wave per SIMD does not cover its own LDS and barrier latencies)
  if constexpr (std::is_same<TC, float>::value) {
    const int oblong = oblong_plan_wins(a);
    if (oblong == 1) return run_dlds<TC, A_KC, B_KC, 128, 512, 1, 8, 3, 512, 32, 16>(a, s);
    if (oblong == 2) return run_dlds<TC, A_KC, B_KC, 512, 128, 4, 2, 3, 128, 32, 16>(a, s);
  }
  if (shape != 7 && a.K % 64 == 0) return run_dlds<TC, A_KC, B_KC, 256, 256, 2, 4, 2, 256, 64, 16>(a, s);
  return run_dlds<TC, A_KC, B_KC, 256, 256, 2, 4, 4, 256, 32, 16>(a, s);
}

}  // namespace

// The shapes this kernel takes: whole K tiles of 32, 16-byte rows, and at least 8 rows (columns) where the
// operand is read along them.
bool gemm_dlds_eligible(const GemmArgs& a) {
  if (a.K < DL_BK_MIN || a.K % DL_BK_MIN || a.lda % 8 || a.ldb % 8) return false;
  if (a.trans_a && (a.M % 8 || a.M < 8)) return false;
  if (!a.trans_b && (a.N % 8 || a.N < 8)) return false;
  if (a.out_f32 ? !(a.trans_a && !a.trans_b) : a.trans_a) return false;
  // 32-bit per-lane offsets into an operand: (rows - 1) x row stride + K tile of a K-contiguous one, 64 K-rows of a
  // row-contiguous one
  const long span_a = a.trans_a ? 64 * a.lda + a.M : (long)a.M * a.lda;
  const long span_b = a.trans_b ? (long)a.N * a.ldb : 64 * a.ldb + a.N;
  if (span_a >= (1L << 31) || span_b >= (1L << 31)) return false;
  return true;
}

void set_gemm_dlds_shape(int shape) { g_dlds_shape = shape; }

int gemm_dlds_plan_slices(int M, int N, int K, int max_slices, bool any_shape) {
  UnevenPlan up;
  const int square = plan_uneven(M, N, K, 256, 256, 2, 4, max_slices, up) ? up.s[0] : 0;
  const int narrow = plan_uneven(M, N, K, 256, 128, 2, 2, max_slices, up) ? up.s[0] : 0;
  const int wide = plan_uneven(M, N, K, 128, 512, 1, 8, max_slices, up) ? up.s[0] : 0;
  const int tall = plan_uneven(M, N, K, 512, 128, 4, 2, max_slices, up) ? up.s[0] : 0;
  if (any_shape) return std::max(std::max(square, narrow), std::max(wide, tall));
  GemmArgs a{};
  a.M = M; a.N = N; a.K = K; a.splits = max_slices;
  const int oblong = oblong_plan_wins(a);
  if (oblong) return oblong == 1 ? wide : tall;
  return g_dlds_shape == 2 ? narrow : square;
}

// Host-only view of the split-K plan a weight gradient X^T dY of these sizes would be launched with, for tests:
// out[0] = tile rows, out[1] = tile columns of the shape taken (0, 0: no uneven plan, the launch uses equal slices);
// out[2], out[3] = tile rows / columns of the class "inside C"; out[4..7] = tiles per class; out[8..11] = K slices
// per class (classes: inside C, over its last rows, over its last columns, over both).
void gemm_dlds_plan_info(int M, int N, int K, int max_slices, int* out) {
  GemmArgs a{};
  a.M = M; a.N = N; a.K = K; a.splits = max_slices;
  const int oblong = oblong_plan_wins(a);
  const int BM = oblong == 1 ? 128 : oblong == 2 ? 512 : 256;
  const int BN = oblong == 1 ? 512 : oblong == 2 ? 128 : (g_dlds_shape == 2 ? 128 : 256);
  const int WGM = oblong == 1 ? 1 : oblong == 2 ? 4 : 2;
  const int WGN = oblong == 1 ? 8 : oblong == 2 ? 2 : (g_dlds_shape == 2 ? 2 : 4);
  UnevenPlan up;
  for (int i = 0; i < 12; ++i) out[i] = 0;
  if (max_slices <= 1 || !plan_uneven(M, N, K, BM, BN, WGM, WGN, max_slices, up)) return;
  out[0] = BM; out[1] = BN; out[2] = up.full_m; out[3] = up.full_n;
  for (int c = 0; c < 4; ++c) { out[4 + c] = up.n[c]; out[8 + c] = up.s[c]; }
}

dipaco_status launch_gemm_dlds(const GemmArgs& a, hipStream_t s) {
  if (!gemm_dlds_eligible(a)) return fail(DIPACO_EUNSUPPORTED, "gemm: shape not supported by the direct-to-LDS kernel");
  if (a.out_f32) return run_dlds_shape<float, false, false>(a, s);
  if (!a.trans_b) return run_dlds_shape<bf16, true, false>(a, s);
  return run_dlds_shape<bf16, true, true>(a, s);
}

}  // namespace dipaco
