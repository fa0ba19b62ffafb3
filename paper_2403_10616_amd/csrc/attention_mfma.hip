// Causal attention on the matrix cores (bf16 operands, fp32 softmax and accumulation), head size 64.
//
// Everything is arranged so that the probabilities never leave registers.  A 32x32 MFMA leaves its result with
// lane l holding column l%32 and rows 8*(e/4) + 4*(l/32) + e%4 (e = 0..15); the B operand of the next MFMA wants
// lane l to hold column l%32 and eight contraction indices.  So whatever must be contracted next is made the
// ROW index of the score tile:
//   forward, dQ:   S^T = K.Q^T  (rows = keys, columns = queries)  ->  O^T += V^T.P^T,   dQ^T += K^T.dS^T
//   dK, dV:        S   = Q.K^T  (rows = queries, columns = keys)  ->  dV^T += dO^T.P,   dK^T += Q^T.dS
// Softmax state (running max, sum, log-sum-exp, D = rowsum(dO*O)) is per query: per lane in the first family, per
// accumulator row in the second.  Exponentials are base 2 with log2(e) folded into the score scale.
// On this chip matrix-core and vector-ALU instructions of the waves of one SIMD do not run side by side (measured:
// 16 MFMAs + 256 FMAs take the sum of their times at two or more waves per SIMD), so every vector instruction of the
// inner loops is paid in full: the forward kernel adds its row sums two bf16 values per instruction on the packed
// probabilities, walks its two stages with compile-time LDS offsets, and leaves the sum over a lane pair to the end.
//
// One workgroup = 4 waves, each wave owns 32 queries (or 32 keys).  K / V (or Q / dO) tiles of 64 rows x 64
// columns go from global memory straight into LDS (16-byte global_load_lds: lane l of a wave-level load writes
// LDS bytes [16 l, 16 l + 16), so the swizzle is applied by choosing which 16 bytes a lane fetches) into a ring
// of stages that runs two or three tiles ahead of the arithmetic, one barrier per tile.  A tile is stored once,
// row-major, and read in both orientations:
//   * rows as the MFMA row index, contraction along the 64 columns: one ds_read_b128 per fragment;
//   * columns as the MFMA row index, contraction along the tile's rows (the V^T, K^T, dO^T, Q^T operands):
//     ds_read_b64_tr_b16, which transposes 4x4 halfword blocks across each group of 16 lanes.  Lane 4e+q of a
//     group points at columns 4q..4q+3 of tile row T(e); lane i then receives column i of rows T(0..3).  The
//     rows T are chosen in the order in which an accumulator holds them (4h + 0..3, then 8 + 4h + 0..3 of each
//     group of 16), so that accumulator elements 8g..8g+7, packed to bf16, are the matching B operand.
// Chunk c (16 bytes) of tile row r sits at chunk position c ^ swz(r), swz(r) = 4*bit1(r) + bits3:2(r): both kinds
// of read are then free of bank conflicts (rows two apart land in different 64-byte groups for the transposing
// read; the lane groups that a ds_read_b128 serves together see eight different swizzles per row parity).
// No atomics: every output element has exactly one writer and a fixed summation order.
#include <type_traits>

#include "kernels.h"
#include "mma_tile.h"

namespace dipaco {

namespace {

constexpr int AT_THREADS = 256;
constexpr int DH = 64;
constexpr int TILE_BYTES = 64 * TILE_ROW_BYTES;   // 64 rows x 128 B
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;

__device__ __forceinline__ f32x16 mfma16(const uint4& a, const uint4& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ void zero(f32x16& v) {
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] = 0.f;
}
// accumulator elements E0..E0+7 as a bf16 B fragment (contraction slots in accumulator order)
template <int E0> __device__ __forceinline__ uint4 pack8(const f32x16& v) {
  bf16x8 o = {(bf16)v[E0 + 0], (bf16)v[E0 + 1], (bf16)v[E0 + 2], (bf16)v[E0 + 3],
              (bf16)v[E0 + 4], (bf16)v[E0 + 5], (bf16)v[E0 + 6], (bf16)v[E0 + 7]};
  return __builtin_bit_cast(uint4, o);
}

__device__ __forceinline__ int swz64(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }

// ---- global memory -> LDS -----------------------------------------------------------------------------------
__device__ __forceinline__ void load16_to_lds(const bf16* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ void load4_to_lds(const float* gptr, uint32_t lds_addr) {   // lane l writes bytes [4 l, 4 l + 4)
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {   // vmcnt only: expcnt and lgkmcnt fields at maximum
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
// This wave's loads of every stage but the n newest have landed; LPW = loads per wave and stage.  (The loads are
// invisible to the compiler, so the count is kept by hand; loads the compiler issues itself only ever make these
// waits longer, never shorter, because the counter is decremented in issue order.)
template <int LPW> __device__ __forceinline__ void wait_stages_but(int n) {
  if (n >= 3) wait_vmcnt<3 * LPW>();
  else if (n == 2) wait_vmcnt<2 * LPW>();
  else if (n == 1) wait_vmcnt<LPW>();
  else wait_vmcnt<0>();
}

// global -> LDS with a wave-uniform base address and a 32-bit per-lane byte offset
__device__ __forceinline__ void load16_to_lds_at(const bf16* base, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory");
}

// This wave's share of the loads of a stage made of two 64x64 tiles: 4 of the 16 wave-level loads (each fills 8
// tile rows = 1024 LDS bytes).  Load i of wave w is number j = w + 4i: tile j / 8, rows 8 (j % 8) .. + 7.
// A lane keeps one 32-bit byte offset per load (its row and 16-byte chunk inside a tile that starts at the operand's
// row 0); the tile's first row is added to the wave-uniform base address, so a stage costs four vector registers.
struct StageLoader {
  uint32_t off[4];      // per lane: (row inside the tile) * row bytes + chunk * 16
  uint32_t chunk[4];    // per lane: chunk * 16 alone (ragged last tile)
};
__device__ __forceinline__ int loader_row(int i, int wave, int lane) { return 8 * ((wave + 4 * i) & 7) + (lane >> 3); }
__device__ __forceinline__ StageLoader make_loader(long ld0, long ld1, int wave, int lane) {
  StageLoader L;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = wave + 4 * i;
    const int rit = loader_row(i, wave, lane);
    L.chunk[i] = (uint32_t)(((lane & 7) ^ swz64(rit)) * 16);
    L.off[i] = (uint32_t)(rit * (j < 8 ? ld0 : ld1) * 2) + L.chunk[i];
  }
  return L;
}
// tile0 / tile1: the two operands (row 0 of this sequence and head), ld0 / ld1 their row strides in elements.
// Rows at or beyond rows_total re-read the last valid row: callers give such rows zero weight (masked
// probabilities, -inf statistics), so any finite value will do, and no branch surrounds a load.  Only the last
// tile of an operand can stick out; every other tile only moves the wave-uniform base.
// Byte offsets are 32-bit: rows_total * row stride * 2 stays below 2^32 (checked by the launchers).
__device__ __forceinline__ void issue_stage(const StageLoader& L, const bf16* tile0, const bf16* tile1, int row0,
                                            int rows_total, long ld0, long ld1, int wave, int lane, uint32_t stage_addr) {
  if (row0 + 64 <= rows_total) {   // wave-uniform
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool first = (wave + 4 * i) < 8;   // wave-uniform
      const int j = wave + 4 * i;
      load16_to_lds_at((first ? tile0 : tile1) + (long)row0 * (first ? ld0 : ld1), L.off[i],
                       stage_addr + (uint32_t)((j >> 3) * TILE_BYTES + (j & 7) * 1024));
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool first = (wave + 4 * i) < 8;
      const int j = wave + 4 * i;
      const int r = min(row0 + loader_row(i, wave, lane), rows_total - 1);
      load16_to_lds_at(first ? tile0 : tile1, (uint32_t)r * (uint32_t)((first ? ld0 : ld1) * 2) + L.chunk[i],
                       stage_addr + (uint32_t)((j >> 3) * TILE_BYTES + (j & 7) * 1024));
    }
  }
}

// ---- fragment reads -----------------------------------------------------------------------------------------
// Row-index reads.  Lane l reads row 32*t + r (r = l%32), chunk (2*ks + h) ^ swz(row), h = l/32; swz does not
// depend on t (it uses bits 1..3 of the row).  b[ks]: byte offset for t = 0; add 4096*t.
struct FragOff { int b[4]; };
__device__ __forceinline__ FragOff frag_offsets(int lane) {
  const int r = lane & 31, h = lane >> 5, s = swz64(r);
  FragOff f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) f.b[ks] = r * TILE_ROW_BYTES + (((2 * ks + h) ^ s) << 4);
  return f;
}
__device__ __forceinline__ uint4 ld16(const char* p) { return *reinterpret_cast<const uint4*>(p); }

// Column-index (transposing) reads.  For output columns 32*dt .. + 31 and the 16 tile rows 32*t + 16*g2 .. + 15,
// read p (0 / 1) of lane l = 16*g4 + 4*e + q fetches columns 32*dt + 16*(g4 & 1) + 4q .. + 3 of tile row
// 32*t + 16*g2 + 8p + 4*(g4 >> 1) + e, and the two reads together give the lane its column's values in tile rows
// 4h + 0..3, 8 + 4h + 0..3 of the group (h = l/32): the order of accumulator elements 8*g2 .. 8*g2 + 7.
// b[dt][p]: byte offset for t = g2 = 0; add (32*t + 16*g2) * 128.
struct TrOff { int b[2][2]; };
__device__ __forceinline__ TrOff tr_offsets(int lane) {
  const int g4 = lane >> 4, e = (lane & 15) >> 2, q = lane & 3, h = g4 >> 1;
  TrOff t;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int row = 8 * p + 4 * h + e;
      const int chunk = (4 * dt + 2 * (g4 & 1) + (q >> 1)) ^ swz64(row);
      t.b[dt][p] = row * TILE_ROW_BYTES + (chunk << 4) + ((q & 1) << 3);
    }
  return t;
}
__device__ __forceinline__ uint4 tr_read(const char* tile, const TrOff& to, int dt, int rows16) {
  const char* base = tile + rows16 * 16 * TILE_ROW_BYTES;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)(uint32_t)(uintptr_t)(base + to.b[dt][0]));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)(uint32_t)(uintptr_t)(base + to.b[dt][1]));
  uint4 o;
  o.x = (uint16_t)lo[0] | ((uint32_t)(uint16_t)lo[1] << 16);
  o.y = (uint16_t)lo[2] | ((uint32_t)(uint16_t)lo[3] << 16);
  o.z = (uint16_t)hi[0] | ((uint32_t)(uint16_t)hi[1] << 16);
  o.w = (uint16_t)hi[2] | ((uint32_t)(uint16_t)hi[3] << 16);
  return o;
}
// acc^T[dt] += (tile^T)[columns 32 dt.., rows 32 t..] . src[t]   for a 64-row tile and two accumulator tiles src
__device__ __forceinline__ void mma_transposed(f32x16 (&acc)[2], const char* tile, const TrOff& to, const f32x16 (&src)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const uint4 p0 = pack8<0>(src[t]), p1 = pack8<8>(src[t]);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
      acc[dt] = mfma16(tr_read(tile, to, dt, 2 * t), p0, acc[dt]);
      acc[dt] = mfma16(tr_read(tile, to, dt, 2 * t + 1), p1, acc[dt]);
    }
  }
}

// The same with the probabilities already packed to bf16: pk[t][0 / 1] = pack8<0 / 8>(src[t]).
__device__ __forceinline__ void mma_transposed_packed(f32x16 (&acc)[2], const char* tile, const TrOff& to,
                                                      const uint4 (&pk)[2][2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) {
      acc[dt] = mfma16(tr_read(tile, to, dt, 2 * t), pk[t][0], acc[dt]);
      acc[dt] = mfma16(tr_read(tile, to, dt, 2 * t + 1), pk[t][1], acc[dt]);
    }
}
// acc + the eight bf16 values of v, two per instruction (v_dot2c_f32_bf16 with a vector of ones: products with 1 and
// the fp32 additions are exact operations on the rounded values, the ones the matrix core then multiplies)
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float add8_bf16(float acc, const uint4& v) {
  const bf16x2 ones = {(bf16)1.0f, (bf16)1.0f};
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.x), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.y), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.z), ones, acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, v.w), ones, acc, false);
  return acc;
}

// store 4 consecutive head columns (accumulator elements 4g..4g+3 of a transposed-output tile) as bf16
__device__ __forceinline__ void store4(bf16* dst, const f32x16& v, int g, float scale) {
  bf16x4 o = {(bf16)(v[4 * g + 0] * scale), (bf16)(v[4 * g + 1] * scale), (bf16)(v[4 * g + 2] * scale),
              (bf16)(v[4 * g + 3] * scale)};
  *reinterpret_cast<bf16x4*>(dst) = o;
}
// out^T tiles ot[dt] hold head column 32*dt + 8*g + 4*h + (0..3) for this lane's row
__device__ __forceinline__ void store_transposed_out(bf16* row_ptr, const f32x16 (&ot)[2], int h, float scale) {
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) store4(row_ptr + 32 * dt + 8 * g + 4 * h, ot[dt], g, scale);
}

// v + (v of the lane that the DPP control selects); rows outside row_mask add 0.  Pure VALU: no LDS traffic.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_add(float v) {
  const int t = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false);
  return v + __builtin_bit_cast(float, t);
}
// Sum over each half of the wave (lanes 0..31, lanes 32..63); the result is valid in lanes 16..31 and 48..63.
__device__ __forceinline__ float half_wave_sum(float v) {
  v = dpp_add<0xb1, 0xf>(v);    // quad_perm [1,0,3,2]
  v = dpp_add<0x4e, 0xf>(v);    // quad_perm [2,3,0,1]: every lane holds its quad's sum
  v = dpp_add<0x141, 0xf>(v);   // row_half_mirror: sums of 8
  v = dpp_add<0x140, 0xf>(v);   // row_mirror: sums of 16
  v = dpp_add<0x142, 0xa>(v);   // row_bcast15 into rows 1 and 3: sums of 32
  return v;
}

// Column sums of a block's 128 rows of a transposed-output tile pair (the bias gradient of the projection whose
// output gradient the block is): every lane adds scale * its values over the 32 rows of its wave, the four waves'
// sums are added in wave order, and the 64 sums go to out[0..64).
// red: LDS [4][64].  All four waves call it; rows with valid = false count as zero.
__device__ __forceinline__ void block_column_sums(const f32x16 (&ot)[2], float scale, bool valid, float (*red)[DH],
                                                  float* __restrict__ out, int wave, int lane) {
  const int h = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float v = half_wave_sum(valid ? ot[dt][k] * scale : 0.f);
      if ((lane & 31) == 31) red[wave][32 * dt + 8 * (k >> 2) + 4 * h + (k & 3)] = v;
    }
  __syncthreads();
  if (threadIdx.x < DH) {
    const int c = threadIdx.x;
    out[c] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
  }
  __syncthreads();   // red is reused by the workgroup's next block
}

// ---- forward ---------------------------------------------------------------------------------------------------
constexpr int FWD_STAGES = 2, DQ_STAGES = 2, DKV_STAGES = 2;   // three stages measured: forward level, backward 4 % slower

__global__ void __launch_bounds__(AT_THREADS, 3) attn_fwd_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                               float* __restrict__ lse, int S, int H, int single) {
  constexpr int NS = FWD_STAGES;
  __shared__ __attribute__((aligned(16))) char smem[NS][2][TILE_BYTES];   // [stage][K | V]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int bh = single ? blockIdx.x : blockIdx.y, b = bh / H, hd = bh % H;
  const int n_bh = single ? gridDim.x : gridDim.y;
  const int bx = single ? (int)blockIdx.y : (int)blockIdx.x;   // single: one block per workgroup, longest first
  const int A = H * DH;
  const long ld = 3L * A;
  const bf16* base = qkv + (long)b * S * ld + hd * DH;
  const FragOff fo = frag_offsets(lane);
  const TrOff to = tr_offsets(lane);
  const uint32_t smem_addr = (uint32_t)(uintptr_t)&smem[0][0][0];
  const StageLoader L = make_loader(ld, ld, wave, lane);
  const bf16* const ktile = base + A;
  const bf16* const vtile = base + 2 * A;
  // A workgroup takes a long and a short query block (block x from the end, then block x from the start), so that
  // every workgroup walks the same number of tiles whatever the causal triangle gives its blocks.
  const int nqb = (S + 127) / 128;
  for (int pass = 0; pass < 2; ++pass) {
  const int qb = pass == 0 ? nqb - 1 - bx : bx;
  if (pass == 1) {
    if (single || qb >= nqb - 1 - bx) break;      // the middle block of an odd count was done in the first pass
    __syncthreads();                              // the stages are reused
  }
  const int q0 = qb * 128, qw0 = q0 + 32 * wave, q = qw0 + r;

  uint4 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    qf[ks] = q < S ? *reinterpret_cast<const uint4*>(base + (long)q * ld + 8 * (2 * ks + h)) : make_uint4(0, 0, 0, 0);

  const int kv_end = min(S, q0 + 128);
  const int ntiles = (kv_end + 63) / 64;
  f32x16 ot[2];
  zero(ot[0]); zero(ot[1]);
  float m = -INFINITY, l = 0.f;
  const float sc = 0.125f * LOG2E;   // 1/sqrt(64), base-2 exponentials

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < ntiles) issue_stage(L, ktile, vtile, s * 64, S, ld, ld, wave, lane, smem_addr + s * 2 * TILE_BYTES);
  static_assert(NS == 2 || NS == 3, "the tile loop below is unrolled over the stages, so that every LDS offset is a constant");
  // one key / value tile; CUR: the stage it sits in
  auto tile = [&](auto CUR, int kt) {
    constexpr int cur = decltype(CUR)::value;
    wait_stages_but<4>(min(NS - 2, ntiles - 1 - kt));
    __syncthreads();   // tile kt is in LDS; nobody still reads the stage of tile kt - 1, which is refilled now
    if (kt + NS - 1 < ntiles)
      issue_stage(L, ktile, vtile, (kt + NS - 1) * 64, S, ld, ld, wave, lane, smem_addr + (cur == 0 ? NS - 1 : cur - 1) * 2 * TILE_BYTES);
    const int kv0 = kt * 64;
    if (kv0 <= qw0 + 31) {   // wave-uniform: at least one query of this wave sees this tile
      const char* k_ = smem[cur][0];
      const char* v_ = smem[cur][1];
      f32x16 st[2];
      zero(st[0]); zero(st[1]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) st[t] = mfma16(ld16(k_ + fo.b[ks] + 4096 * t), qf[ks], st[t]);
      if (kv0 + 63 > qw0) {   // wave-uniform: the tile crosses the diagonal of some query
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (kv0 + 32 * t + acc_row(e, lane) > q) st[t][e] = -INFINITY;
      }
      float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(fmaxf(mx, st[0][e]), st[1][e]);   // one three-input maximum each
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      // The reference exponent m only has to stay within 2^8 of the true running maximum (probabilities then stay
      // below 256, harmless in fp32 sums and in bf16 operands, and the final O / l and lse do not depend on the
      // reference): the accumulators are rescaled only when some query's maximum outgrows it by more than that.
      const float mn = fmaxf(m, mx * sc);   // finite: key 0 is visible to every query
      if (__builtin_amdgcn_ballot_w64(mn > m + 8.0f) != 0) {   // wave-uniform
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        l *= corr;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) ot[dt][e] *= corr;
        m = mn;
      }
      // probabilities, rounded to bf16 once: the rounded values are both what the matrix core multiplies with V and
      // what the row sum adds up (two per instruction), so numerator and denominator of the softmax agree exactly.
      // l is this lane's half of the row (keys 4h + 0..3 of every eight); the halves meet after the last tile.
      uint4 pk[2][2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
#pragma unroll
        for (int e = 0; e < 16; ++e) st[t][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[t][e], sc, -m));
        pk[t][0] = pack8<0>(st[t]);
        pk[t][1] = pack8<8>(st[t]);
        l = add8_bf16(add8_bf16(l, pk[t][0]), pk[t][1]);
      }
      mma_transposed_packed(ot, v_, to, pk);
    }
  };
  for (int kt = 0; kt < ntiles; kt += NS) {
    tile(std::integral_constant<int, 0>{}, kt);
    if (kt + 1 < ntiles) tile(std::integral_constant<int, 1>{}, kt + 1);
    if (NS > 2 && kt + 2 < ntiles) tile(std::integral_constant<int, NS - 1>{}, kt + 2);
  }
  l += __shfl_xor(l, 32, WAVE);
  // the output addresses are formed from here on (an opaque copy of the row index: formed before the loop they would
  // sit in sixteen registers through it)
  int q_out = q;
  asm volatile("" : "+v"(q_out));
  if (q_out < S) {
    store_transposed_out(o + ((long)b * S + q_out) * A + hd * DH, ot, h, 1.0f / l);
    if (h == 0) lse[(long)bh * S + q_out] = (m + __builtin_amdgcn_logf(l)) * LN2;   // v_log_f32 is log2
  }
  }
}

// ---- backward, dQ (also writes D = rowsum(dO * O)) --------------------------------------------------------------
__global__ void __launch_bounds__(AT_THREADS, 2) attn_bwd_dq_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                                  const bf16* __restrict__ d_o,
                                                                  const float* __restrict__ lse, bf16* __restrict__ dqkv,
                                                                  float* __restrict__ dsum, float* __restrict__ colsum, int S, int H, int single) {
  constexpr int NS = DQ_STAGES;
  __shared__ float cs_red[4][DH];
  extern __shared__ __attribute__((aligned(16))) char dq_smem[];   // [stage][K | V]
  char (*smem)[2][TILE_BYTES] = reinterpret_cast<char (*)[2][TILE_BYTES]>(dq_smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int bh = single ? blockIdx.x : blockIdx.y, b = bh / H, hd = bh % H;
  const int n_bh = single ? gridDim.x : gridDim.y;
  const int bx = single ? (int)blockIdx.y : (int)blockIdx.x;   // single: one block per workgroup, longest first
  const int A = H * DH;
  const long ld = 3L * A;
  const bf16* base = qkv + (long)b * S * ld + hd * DH;
  const FragOff fo = frag_offsets(lane);
  const TrOff to = tr_offsets(lane);
  const uint32_t smem_addr = (uint32_t)(uintptr_t)dq_smem;
  const StageLoader L = make_loader(ld, ld, wave, lane);
  const bf16* const ktile = base + A;
  const bf16* const vtile = base + 2 * A;
  const int nqb = (S + 127) / 128;
  for (int pass = 0; pass < 2; ++pass) {   // a long and a short query block per workgroup (see the forward kernel)
  const int qb = pass == 0 ? nqb - 1 - bx : bx;
  if (pass == 1) {
    if (single || qb >= nqb - 1 - bx) break;
    __syncthreads();
  }
  const int q0 = qb * 128, qw0 = q0 + 32 * wave, q = qw0 + r;

  uint4 qf[4], gf[4];
  float D = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int c = 8 * (2 * ks + h);
    if (q < S) {
      qf[ks] = *reinterpret_cast<const uint4*>(base + (long)q * ld + c);
      gf[ks] = *reinterpret_cast<const uint4*>(d_o + ((long)b * S + q) * A + hd * DH + c);
      const uint4 ov = *reinterpret_cast<const uint4*>(o + ((long)b * S + q) * A + hd * DH + c);
      const bf16* gp = reinterpret_cast<const bf16*>(&gf[ks]);
      const bf16* op = reinterpret_cast<const bf16*>(&ov);
#pragma unroll
      for (int i = 0; i < 8; ++i) D += (float)gp[i] * (float)op[i];
    } else {
      qf[ks] = make_uint4(0, 0, 0, 0);
      gf[ks] = make_uint4(0, 0, 0, 0);
    }
  }
  D += __shfl_xor(D, 32, WAVE);
  const float nlse2 = q < S ? -lse[(long)bh * S + q] * LOG2E : -INFINITY;
  // per-query statistics for the dK / dV kernel, in rows padded to whole query blocks: D (0 beyond S) and
  // -lse * log2(e) (-inf beyond S: probability 0), so that kernel needs neither a bounds check nor a rescale
  if (h == 0) {
    const long Sp = (long)nqb * 128;
    dsum[bh * Sp + q] = q < S ? D : 0.f;
    dsum[(long)n_bh * Sp + bh * Sp + q] = nlse2;
  }

  const int kv_end = min(S, q0 + 128);
  const int ntiles = (kv_end + 63) / 64;
  f32x16 dqt[2];
  zero(dqt[0]); zero(dqt[1]);
  const float sc = 0.125f * LOG2E;

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < ntiles) issue_stage(L, ktile, vtile, s * 64, S, ld, ld, wave, lane, smem_addr + s * 2 * TILE_BYTES);
  int cur = 0;
  for (int kt = 0; kt < ntiles; ++kt, cur = cur + 1 == NS ? 0 : cur + 1) {
    wait_stages_but<4>(min(NS - 2, ntiles - 1 - kt));
    __syncthreads();   // tile kt is in LDS; nobody still reads the stage of tile kt - 1, which is refilled now
    if (kt + NS - 1 < ntiles)
      issue_stage(L, ktile, vtile, (kt + NS - 1) * 64, S, ld, ld, wave, lane, smem_addr + (cur == 0 ? NS - 1 : cur - 1) * 2 * TILE_BYTES);
    const int kv0 = kt * 64;
    if (kv0 <= qw0 + 31) {
      const char* k_ = smem[cur][0];
      const char* v_ = smem[cur][1];
      f32x16 st[2], dp[2];
      zero(st[0]); zero(st[1]); zero(dp[0]); zero(dp[1]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          st[t] = mfma16(ld16(k_ + fo.b[ks] + 4096 * t), qf[ks], st[t]);
          dp[t] = mfma16(ld16(v_ + fo.b[ks] + 4096 * t), gf[ks], dp[t]);
        }
      // dS^T without the 1/sqrt(d_head) factor (applied once when dQ is stored)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          st[t][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[t][e], sc, nlse2)) * (dp[t][e] - D);
      if (kv0 + 63 > qw0) {   // wave-uniform: the tile crosses the diagonal
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (kv0 + 32 * t + acc_row(e, lane) > q) st[t][e] = 0.f;
      }
      mma_transposed(dqt, k_, to, st);
    }
  }
  if (q < S) store_transposed_out(dqkv + ((long)b * S + q) * ld + hd * DH, dqt, h, 0.125f);
  // one row of partial column sums per (document, query block): [b * nqb + qb][3 A], this head's 64 dQ columns
  if (colsum) block_column_sums(dqt, 0.125f, q < S, cs_red, colsum + ((long)b * nqb + qb) * ld + hd * DH, wave, lane);
  }
}

// ---- backward, dK and dV ------------------------------------------------------------------------------------------
constexpr int DKV_STAGE = 2 * TILE_BYTES + 2 * 64 * (int)sizeof(float);   // Q | dO | -lse2 | D

__global__ void __launch_bounds__(AT_THREADS, 2) attn_bwd_dkv_mfma(const bf16* __restrict__ qkv,
                                                                   const bf16* __restrict__ d_o,
                                                                   const float* __restrict__ dsum,
                                                                   bf16* __restrict__ dqkv, float* __restrict__ colsum, int S, int H, int single) {
  constexpr int NS = DKV_STAGES;
  __shared__ float cs_red[4][DH];
  extern __shared__ __attribute__((aligned(16))) char dkv_smem[];   // NS stages of DKV_STAGE bytes
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int bh = single ? blockIdx.x : blockIdx.y, b = bh / H, hd = bh % H;
  const int n_bh = single ? gridDim.x : gridDim.y;
  const int bx = single ? (int)blockIdx.y : (int)blockIdx.x;   // single: one block per workgroup, longest first
  const int A = H * DH;
  const long ld = 3L * A;
  const bf16* base = qkv + (long)b * S * ld + hd * DH;
  const bf16* gbase = d_o + (long)b * S * A + hd * DH;
  const FragOff fo = frag_offsets(lane);
  const TrOff to = tr_offsets(lane);
  const uint32_t smem_addr = (uint32_t)(uintptr_t)dkv_smem;
  const int nkb = (S + 127) / 128;
  const int ntiles = (S + 63) / 64;
  // Statistics of a tile's 64 queries (written by the dQ kernel into rows padded to whole query blocks): waves 0
  // and 2 fetch -lse*log2(e), waves 1 and 3 fetch D, one float per lane; the duplicates keep every wave's count of
  // outstanding loads the same.
  const long Sp = (long)nkb * 128;
  const float* stat_src = dsum + ((wave & 1) ? 0 : (long)n_bh * Sp) + bh * Sp + lane;
  const uint32_t stat_dst = 2 * TILE_BYTES + ((wave & 1) ? 256 : 0);
  const StageLoader L = make_loader(ld, A, wave, lane);
  auto issue = [&](int qt, int stage) {
    issue_stage(L, base, gbase, qt * 64, S, ld, A, wave, lane, smem_addr + stage * DKV_STAGE);
    load4_to_lds(stat_src + qt * 64, smem_addr + stage * DKV_STAGE + stat_dst);
  };
  for (int pass = 0; pass < 2; ++pass) {   // an early (long) and a late (short) key block per workgroup
  const int kb = pass == 0 ? bx : nkb - 1 - bx;
  if (pass == 1) {
    if (single || kb <= bx) break;
    __syncthreads();
  }
  const int k0 = kb * 128, kw0 = k0 + 32 * wave, key = kw0 + r;

  uint4 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int c = 8 * (2 * ks + h);
    kf[ks] = key < S ? *reinterpret_cast<const uint4*>(base + (long)key * ld + A + c) : make_uint4(0, 0, 0, 0);
    vf[ks] = key < S ? *reinterpret_cast<const uint4*>(base + (long)key * ld + 2 * A + c) : make_uint4(0, 0, 0, 0);
  }
  f32x16 dkt[2], dvt[2];
  zero(dkt[0]); zero(dkt[1]); zero(dvt[0]); zero(dvt[1]);
  const float sc = 0.125f * LOG2E;

  const int first = k0 / 64;               // first query tile that can see a key of this block
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (first + s < ntiles) issue(first + s, s);
  int cur = 0;
  for (int qt = first; qt < ntiles; ++qt, cur = cur + 1 == NS ? 0 : cur + 1) {
    wait_stages_but<5>(min(NS - 2, ntiles - 1 - qt));
    __syncthreads();
    if (qt + NS - 1 < ntiles) issue(qt + NS - 1, cur == 0 ? NS - 1 : cur - 1);
    const int q0 = qt * 64;
    if (q0 + 63 >= kw0) {   // wave-uniform: some query of this tile sees a key of this wave
      const char* q_ = dkv_smem + cur * DKV_STAGE;
      const char* g_ = q_ + TILE_BYTES;
      const float* nlse2s = reinterpret_cast<const float*>(q_ + 2 * TILE_BYTES);
      const float* Ds = nlse2s + 64;
      f32x16 st[2], dp[2];
      zero(st[0]); zero(st[1]); zero(dp[0]); zero(dp[1]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          st[t] = mfma16(ld16(q_ + fo.b[ks] + 4096 * t), kf[ks], st[t]);
          dp[t] = mfma16(ld16(g_ + fo.b[ks] + 4096 * t), vf[ks], dp[t]);
        }
      // accumulator elements 4g..4g+3 are queries 32t + 8g + 4h + (0..3): their statistics are 16 contiguous bytes
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 Lq = *reinterpret_cast<const float4*>(nlse2s + 32 * t + 8 * g + 4 * h);
          const float4 Dv = *reinterpret_cast<const float4*>(Ds + 32 * t + 8 * g + 4 * h);
          const float Ls[4] = {Lq.x, Lq.y, Lq.z, Lq.w}, Dd[4] = {Dv.x, Dv.y, Dv.z, Dv.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int e = 4 * g + i;
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[t][e], sc, Ls[i]));
            st[t][e] = p;
            dp[t][e] = p * (dp[t][e] - Dd[i]);   // dS without 1/sqrt(d_head) (applied when dK is stored)
          }
        }
      if (q0 < kw0 + 31) {   // wave-uniform: the tile crosses the diagonal of some key
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (q0 + 32 * t + acc_row(e, lane) < key) { st[t][e] = 0.f; dp[t][e] = 0.f; }
      }
      mma_transposed(dvt, g_, to, st);
      mma_transposed(dkt, q_, to, dp);
    }
  }
  if (key < S) {
    bf16* out = dqkv + ((long)b * S + key) * ld + hd * DH;
    store_transposed_out(out + A, dkt, h, 0.125f);
    store_transposed_out(out + 2 * A, dvt, h, 1.0f);
  }
  if (colsum) {
    float* cs = colsum + ((long)b * nkb + kb) * ld + hd * DH;
    block_column_sums(dkt, 0.125f, key < S, cs_red, cs + A, wave, lane);
    block_column_sums(dvt, 1.0f, key < S, cs_red, cs + 2 * A, wave, lane);
  }
  }
}

}  // namespace

std::atomic<int> g_attn_single_block{1};   // test / tuning hook; measured 3-5 % faster than pairing a long with a short block
void set_attention_single_block(int on) { g_attn_single_block = on ? 1 : 0; }

dipaco_status launch_attention_fwd_mfma(const bf16* qkv, bf16* o, float* lse, int B, int S, int H, hipStream_t s) {
  const int single = g_attn_single_block;
  const int nqb = (S + 127) / 128;
  dim3 grid = single ? dim3(B * H, nqb) : dim3((nqb + 1) / 2, B * H);   // one or two query blocks per workgroup
  attn_fwd_mfma<<<grid, AT_THREADS, 0, s>>>(qkv, o, lse, S, H, single);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

size_t attention_colsum_partial_floats(int B, int S, int H) { return (size_t)B * ((S + 127) / 128) * 3 * H * DH; }

dipaco_status launch_attention_bwd_mfma(const bf16* qkv, const bf16* o, const bf16* d_o, const float* lse, bf16* dqkv,
                                        float* dsum, float* colsum_out, float* colsum_partial, int B, int S, int H,
                                        hipStream_t s, SumBatch* batch) {
  const int single = g_attn_single_block;
  const int nqb = (S + 127) / 128;
  dim3 grid = single ? dim3(B * H, nqb) : dim3((nqb + 1) / 2, B * H);   // one or two query (key) blocks per workgroup
  static std::atomic<unsigned long long> dq_lds{0}, dkv_lds{0};
  if (dipaco_status st = ensure_dynamic_lds(reinterpret_cast<const void*>(attn_bwd_dq_mfma), DQ_STAGES * 2 * TILE_BYTES, dq_lds)) return st;
  if (dipaco_status st = ensure_dynamic_lds(reinterpret_cast<const void*>(attn_bwd_dkv_mfma), DKV_STAGES * DKV_STAGE, dkv_lds)) return st;
  attn_bwd_dq_mfma<<<grid, AT_THREADS, DQ_STAGES * 2 * TILE_BYTES, s>>>(qkv, o, d_o, lse, dqkv, dsum, colsum_out ? colsum_partial : nullptr, S, H, single);
  DIPACO_LAUNCH_CHECK();
  attn_bwd_dkv_mfma<<<grid, AT_THREADS, DKV_STAGES * DKV_STAGE, s>>>(qkv, d_o, dsum, dqkv, colsum_out ? colsum_partial : nullptr, S, H, single);
  DIPACO_LAUNCH_CHECK();
  if (colsum_out) return launch_sum_rows(colsum_partial, colsum_out, B * nqb, 3 * H * DH, s, batch);
  return DIPACO_OK;
}

}  // namespace dipaco
