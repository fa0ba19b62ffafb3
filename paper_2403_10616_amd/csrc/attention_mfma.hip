// Causal attention on the matrix cores (bf16 operands, fp32 softmax and accumulation), head size 64.
//
// Everything is arranged so that the probabilities never leave registers.  A 32x32 MFMA leaves its result with
// lane l holding column l%32 and rows 8*(e/4) + 4*(l/32) + e%4 (e = 0..15); the B operand of the next MFMA wants
// lane l to hold column l%32 and eight contraction indices.  So whatever must be contracted next is made the
// ROW index of the score tile:
//   forward, dQ:   S^T = K.Q^T  (rows = keys, columns = queries)  ->  O^T += V^T.P^T,   dQ^T += K^T.dS^T
//   dK, dV:        S   = Q.K^T  (rows = queries, columns = keys)  ->  dV^T += dO^T.P,   dK^T += Q^T.dS
// and the left operands V^T, K^T, dO^T, Q^T are written to LDS transposed, with their 8-byte granules (four
// consecutive contraction indices) placed in the order in which the accumulator holds them.  Softmax state
// (running max, sum, log-sum-exp, D = rowsum(dO*O)) is per query: per lane in the first family, per accumulator
// row in the second.  Exponentials are base 2 with log2(e) folded into the score scale.
//
// One workgroup = 4 waves, each wave owns 32 queries (or 32 keys); K/V (or Q/dO) tiles of 64 rows are staged
// in LDS, double-buffered, loaded by 128 threads each as 4x8 blocks that are stored row-major and/or transposed
// from the same registers.  No atomics: every output element has exactly one writer and a fixed summation order.
#include "kernels.h"
#include "mma_tile.h"

namespace dipaco {

namespace {

constexpr int AT_THREADS = 256;
constexpr int DH = 64;
constexpr int TILE_BYTES = 64 * TILE_ROW_BYTES;   // 64 rows x 128 B
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

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

// ---- 64 x 64 bf16 tile, loaded by 128 threads as 4 (rows) x 8 (columns) blocks -----------------------------
struct SubBlock { uint4 r[4]; };
// lane l of loader wave w2: 8-column block mq = (l&1) + 2*((l>>4)&3), 4-row block kq = ((l>>1)&7) + 8*w2.  A load
// instruction reads 128 contiguous bytes of 8 rows; 16 consecutive lanes of a transposed 8-byte store write 8
// row-granules of two LDS rows whose swizzles differ by 4 (no bank conflicts, see mma_tile.h).
__device__ __forceinline__ void sb_coords(int t128, int& kq, int& mq) {
  const int l = t128 & 63;
  mq = (l & 1) + 2 * ((l >> 4) & 3);
  kq = ((l >> 1) & 7) + 8 * (t128 >> 6);
}
// src points at the tile's first row and column; rows at or beyond rows_valid (>= 1) re-read the last valid row:
// callers give such rows zero weight (masked probabilities), so any finite value will do, and no branch
// surrounds the loads
__device__ __forceinline__ void sb_load(SubBlock& s, const bf16* __restrict__ src, long ld, int rows_valid, int t128) {
  int kq, mq;
  sb_coords(t128, kq, mq);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = min(4 * kq + j, rows_valid - 1);
    s.r[j] = *reinterpret_cast<const uint4*>(src + (long)row * ld + 8 * mq);
  }
}
// LDS tile[row][column]: operand whose contraction index is the column
__device__ __forceinline__ void sb_store_rows(const SubBlock& s, char* tile, int t128) {
  int kq, mq;
  sb_coords(t128, kq, mq);
#pragma unroll
  for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4*>(tile_chunk(tile, 4 * kq + j, mq)) = s.r[j];
}
// LDS tile[column][row], rows (the contraction index) in accumulator order: the granule of rows 4*kq..4*kq+3,
// kq = (t, g2, gh, h) in bits 3..0, goes to chunk (t, g2, h), half gh; a lane of half h then finds, in chunk
// 4t + 2*g2 + h, the eight rows that accumulator elements 8*g2..8*g2+7 of score tile t hold.
__device__ __forceinline__ void sb_store_transposed(const SubBlock& s, char* tile, int t128) {
  int kq, mq;
  sb_coords(t128, kq, mq);
  const int chunk = ((kq >> 2) << 1) | (kq & 1);
  const int half = (kq >> 1) & 1;
  const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&s.r[0]);
  const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&s.r[1]);
  const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&s.r[2]);
  const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&s.r[3]);
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int j = c >> 1;
    uint2 out;
    if ((c & 1) == 0) {
      out.x = (w0[j] & 0xffffu) | (w1[j] << 16);
      out.y = (w2[j] & 0xffffu) | (w3[j] << 16);
    } else {
      out.x = (w0[j] >> 16) | (w1[j] & 0xffff0000u);
      out.y = (w2[j] >> 16) | (w3[j] & 0xffff0000u);
    }
    *reinterpret_cast<uint2*>(tile_chunk(tile, 8 * mq + c, chunk) + (half << 3)) = out;
  }
}

// Byte offsets of this lane's fragments inside a 64-row tile.  Lane l reads row 32*t + r (r = l%32) and chunk
// c ^ swz(row); swz does not depend on t (32*t >> 1 is a multiple of 8) and every chunk index used here is an even
// number plus h = l/32, so chunk ^ swz = even ^ (h ^ swz(r)): four values per lane, b[k] for even = 2k.  A fragment
// read is then tile + b[k] + 4096*t with t a compile-time constant: no address arithmetic in the loops.
struct FragOff { int b[4]; };
__device__ __forceinline__ FragOff frag_offsets(int lane) {
  const int r = lane & 31, u = (lane >> 5) ^ swz(r);
  FragOff f;
#pragma unroll
  for (int k = 0; k < 4; ++k) f.b[k] = r * TILE_ROW_BYTES + ((u ^ (2 * k)) << 4);
  return f;
}
__device__ __forceinline__ uint4 ld16(const char* p) { return *reinterpret_cast<const uint4*>(p); }

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

// ---- forward ---------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(AT_THREADS, 3) attn_fwd_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                            float* __restrict__ lse, int S, int H) {
  __shared__ __attribute__((aligned(16))) char smem[2][2][TILE_BYTES];   // [stage][K rows | V^T]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x;   // long blocks first
  const int bh = blockIdx.y, b = bh / H, hd = bh % H;
  const int A = H * DH;
  const long ld = 3L * A;
  const bf16* base = qkv + (long)b * S * ld + hd * DH;
  const int q0 = qb * 128, qw0 = q0 + 32 * wave, q = qw0 + r;
  const FragOff fo = frag_offsets(lane);

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

  const int t128 = tid & 127;
  const bool load_v = tid >= 128;
  SubBlock sb;
  auto gload = [&](int kt) {
    sb_load(sb, base + (load_v ? 2 * A : A) + (long)(kt * 64) * ld, ld, S - kt * 64, t128);
  };
  auto sstore = [&](int stage) {
    if (load_v) sb_store_transposed(sb, smem[stage][1], t128);
    else sb_store_rows(sb, smem[stage][0], t128);
  };
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < ntiles;
    if (more) gload(kt + 1);
    const int kv0 = kt * 64;
    if (kv0 <= qw0 + 31) {   // wave-uniform: at least one query of this wave sees this tile
      const char* kt_ = smem[cur][0];
      const char* vt_ = smem[cur][1];
      f32x16 st[2];
      zero(st[0]); zero(st[1]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) st[t] = mfma16(ld16(kt_ + fo.b[ks] + 4096 * t), qf[ks], st[t]);
      if (kv0 + 63 > qw0) {   // wave-uniform: the tile crosses the diagonal of some query
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (kv0 + 32 * t + acc_row(e, lane) > q) st[t][e] = -INFINITY;
      }
      float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fmaxf(st[0][e], st[1][e]));
      mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
      const float mn = fmaxf(m, mx * sc);   // finite: key 0 is visible to every query
      float rs = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[t][e], sc, -mn));
          st[t][e] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, WAVE);
      if (__builtin_amdgcn_ballot_w64(mn != m) != 0) {   // wave-uniform: somebody's running maximum moved
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        l *= corr;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int e = 0; e < 16; ++e) ot[dt][e] *= corr;
        m = mn;
      }
      l += rs;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4 p0 = pack8<0>(st[t]), p1 = pack8<8>(st[t]);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          ot[dt] = mfma16(ld16(vt_ + fo.b[2 * t] + 4096 * dt), p0, ot[dt]);
          ot[dt] = mfma16(ld16(vt_ + fo.b[2 * t + 1] + 4096 * dt), p1, ot[dt]);
        }
      }
    }
    if (more) sstore(cur ^ 1);
    __syncthreads();
  }
  if (q < S) {
    store_transposed_out(o + ((long)b * S + q) * A + hd * DH, ot, h, 1.0f / l);
    if (h == 0) lse[(long)bh * S + q] = (m + __builtin_amdgcn_logf(l)) * LN2;   // v_log_f32 is log2
  }
}

// ---- backward, dQ (also writes D = rowsum(dO * O)) --------------------------------------------------------------
__global__ void __launch_bounds__(AT_THREADS, 2) attn_bwd_dq_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                               const bf16* __restrict__ d_o,
                                                               const float* __restrict__ lse, bf16* __restrict__ dqkv,
                                                               float* __restrict__ dsum, int S, int H) {
  __shared__ __attribute__((aligned(16))) char smem[2][3][TILE_BYTES];   // [stage][K rows | V rows | K^T]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int qb = gridDim.x - 1 - blockIdx.x;
  const int bh = blockIdx.y, b = bh / H, hd = bh % H;
  const int A = H * DH;
  const long ld = 3L * A;
  const bf16* base = qkv + (long)b * S * ld + hd * DH;
  const int q0 = qb * 128, qw0 = q0 + 32 * wave, q = qw0 + r;
  const FragOff fo = frag_offsets(lane);

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
  if (q < S && h == 0) dsum[(long)bh * S + q] = D;
  const float nlse2 = q < S ? -lse[(long)bh * S + q] * LOG2E : -INFINITY;

  const int kv_end = min(S, q0 + 128);
  const int ntiles = (kv_end + 63) / 64;
  f32x16 dqt[2];
  zero(dqt[0]); zero(dqt[1]);
  const float sc = 0.125f * LOG2E;

  const int t128 = tid & 127;
  const bool load_v = tid >= 128;
  SubBlock sb;
  auto gload = [&](int kt) {
    sb_load(sb, base + (load_v ? 2 * A : A) + (long)(kt * 64) * ld, ld, S - kt * 64, t128);
  };
  auto sstore = [&](int stage) {
    if (load_v) sb_store_rows(sb, smem[stage][1], t128);
    else { sb_store_rows(sb, smem[stage][0], t128); sb_store_transposed(sb, smem[stage][2], t128); }
  };
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < ntiles;
    if (more) gload(kt + 1);
    const int kv0 = kt * 64;
    if (kv0 <= qw0 + 31) {
      const char* k_rows = smem[cur][0];
      const char* v_rows = smem[cur][1];
      const char* k_t = smem[cur][2];
      f32x16 st[2], dp[2];
      zero(st[0]); zero(st[1]); zero(dp[0]); zero(dp[1]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          st[t] = mfma16(ld16(k_rows + fo.b[ks] + 4096 * t), qf[ks], st[t]);
          dp[t] = mfma16(ld16(v_rows + fo.b[ks] + 4096 * t), gf[ks], dp[t]);
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
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4 s0 = pack8<0>(st[t]), s1 = pack8<8>(st[t]);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          dqt[dt] = mfma16(ld16(k_t + fo.b[2 * t] + 4096 * dt), s0, dqt[dt]);
          dqt[dt] = mfma16(ld16(k_t + fo.b[2 * t + 1] + 4096 * dt), s1, dqt[dt]);
        }
      }
    }
    if (more) sstore(cur ^ 1);
    __syncthreads();
  }
  if (q < S) store_transposed_out(dqkv + ((long)b * S + q) * ld + hd * DH, dqt, h, 0.125f);
}

// ---- backward, dK and dV ------------------------------------------------------------------------------------------
constexpr int DKV_STAGE = 4 * TILE_BYTES + 2 * 64 * (int)sizeof(float);   // Q rows | Q^T | dO rows | dO^T | -lse2 | D

__global__ void __launch_bounds__(AT_THREADS, 2) attn_bwd_dkv_mfma(const bf16* __restrict__ qkv,
                                                                const bf16* __restrict__ d_o,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ dsum,
                                                                bf16* __restrict__ dqkv, int S, int H) {
  extern __shared__ __attribute__((aligned(16))) char dsmem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int kb = blockIdx.x;
  const int bh = blockIdx.y, b = bh / H, hd = bh % H;
  const int A = H * DH;
  const long ld = 3L * A;
  const bf16* base = qkv + (long)b * S * ld + hd * DH;
  const bf16* gbase = d_o + (long)b * S * A + hd * DH;
  const int k0 = kb * 128, kw0 = k0 + 32 * wave, key = kw0 + r;
  const FragOff fo = frag_offsets(lane);

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
  const int ntiles = (S + 63) / 64;
  const int t128 = tid & 127;
  const bool load_g = tid >= 128;
  SubBlock sb;
  float stat = 0.f;
  // per-query statistics of the tile: threads 0-63 fetch -lse*log2(e) (-inf beyond S: probability 0), threads
  // 64-127 fetch D (0 beyond S).  The index is clamped and the override is bitwise, so the load stays unconditional.
  const float* stat_src = (tid & 64) ? dsum + (long)bh * S : lse + (long)bh * S;
  const float stat_mul = (tid & 64) ? 1.0f : -LOG2E;
  const uint32_t stat_fill = (tid & 64) ? 0u : 0xff800000u;
  auto gload = [&](int qt) {
    const int row0 = qt * 64;
    if (load_g) sb_load(sb, gbase + (long)row0 * A, A, S - row0, t128);
    else sb_load(sb, base + (long)row0 * ld, ld, S - row0, t128);
    const int qi = row0 + (tid & 63);
    const float v = stat_src[min(qi, S - 1)] * stat_mul;
    const uint32_t keep = qi < S ? 0xffffffffu : 0u;
    stat = __uint_as_float((__float_as_uint(v) & keep) | (stat_fill & ~keep));
  };
  auto sstore = [&](int stage) {
    char* st = dsmem + stage * DKV_STAGE;
    char* rows = st + (load_g ? 2 : 0) * TILE_BYTES;
    sb_store_rows(sb, rows, t128);
    sb_store_transposed(sb, rows + TILE_BYTES, t128);
    if (tid < 128) reinterpret_cast<float*>(st + 4 * TILE_BYTES)[tid] = stat;
  };
  if (first < ntiles) {
    gload(first);
    sstore(0);
  }
  __syncthreads();
  for (int qt = first; qt < ntiles; ++qt) {
    const int cur = (qt - first) & 1;
    const bool more = qt + 1 < ntiles;
    if (more) gload(qt + 1);
    const int q0 = qt * 64;
    if (q0 + 63 >= kw0) {   // wave-uniform: some query of this tile sees a key of this wave
      const char* stg = dsmem + cur * DKV_STAGE;
      const char* q_rows = stg;
      const char* q_t = stg + TILE_BYTES;
      const char* g_rows = stg + 2 * TILE_BYTES;
      const char* g_t = stg + 3 * TILE_BYTES;
      const float* nlse2s = reinterpret_cast<const float*>(stg + 4 * TILE_BYTES);
      const float* Ds = nlse2s + 64;
      f32x16 st[2], dp[2];
      zero(st[0]); zero(st[1]); zero(dp[0]); zero(dp[1]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          st[t] = mfma16(ld16(q_rows + fo.b[ks] + 4096 * t), kf[ks], st[t]);
          dp[t] = mfma16(ld16(g_rows + fo.b[ks] + 4096 * t), vf[ks], dp[t]);
        }
      // accumulator elements 4g..4g+3 are queries 32t + 8g + 4h + (0..3): their statistics are 16 contiguous bytes
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 L = *reinterpret_cast<const float4*>(nlse2s + 32 * t + 8 * g + 4 * h);
          const float4 Dv = *reinterpret_cast<const float4*>(Ds + 32 * t + 8 * g + 4 * h);
          const float Ls[4] = {L.x, L.y, L.z, L.w}, Dd[4] = {Dv.x, Dv.y, Dv.z, Dv.w};
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
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4 p0 = pack8<0>(st[t]), p1 = pack8<8>(st[t]);
        const uint4 s0 = pack8<0>(dp[t]), s1 = pack8<8>(dp[t]);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          dvt[dt] = mfma16(ld16(g_t + fo.b[2 * t] + 4096 * dt), p0, dvt[dt]);
          dvt[dt] = mfma16(ld16(g_t + fo.b[2 * t + 1] + 4096 * dt), p1, dvt[dt]);
          dkt[dt] = mfma16(ld16(q_t + fo.b[2 * t] + 4096 * dt), s0, dkt[dt]);
          dkt[dt] = mfma16(ld16(q_t + fo.b[2 * t + 1] + 4096 * dt), s1, dkt[dt]);
        }
      }
    }
    if (more) sstore(cur ^ 1);
    __syncthreads();
  }
  if (key < S) {
    bf16* out = dqkv + ((long)b * S + key) * ld + hd * DH;
    store_transposed_out(out + A, dkt, h, 0.125f);
    store_transposed_out(out + 2 * A, dvt, h, 1.0f);
  }
}

}  // namespace

dipaco_status launch_attention_fwd_mfma(const bf16* qkv, bf16* o, float* lse, int B, int S, int H, hipStream_t s) {
  dim3 grid((S + 127) / 128, B * H);
  attn_fwd_mfma<<<grid, AT_THREADS, 0, s>>>(qkv, o, lse, S, H);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_attention_bwd_mfma(const bf16* qkv, const bf16* o, const bf16* d_o, const float* lse, bf16* dqkv,
                                        float* dsum, int B, int S, int H, hipStream_t s) {
  dim3 grid((S + 127) / 128, B * H);
  attn_bwd_dq_mfma<<<grid, AT_THREADS, 0, s>>>(qkv, o, d_o, lse, dqkv, dsum, S, H);
  DIPACO_LAUNCH_CHECK();
  static bool attr_set = false;
  if (!attr_set) {
    DIPACO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_dkv_mfma),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 2 * DKV_STAGE));
    attr_set = true;
  }
  attn_bwd_dkv_mfma<<<grid, AT_THREADS, 2 * DKV_STAGE, s>>>(qkv, d_o, lse, dsum, dqkv, S, H);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace dipaco
