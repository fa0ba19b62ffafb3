// LDS operand tiles for the gfx950 matrix cores and the loaders that fill them.
//
// An operand tile is ROWS rows (the M or N index) by 128 bytes of the contraction index K (64 bf16 or 32
// fp32), K-contiguous: that is the order in which v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32 want both
// operands (lane l supplies row l%32, K-group l/32).  A row is 8 chunks of 16 bytes; chunk c of row r lives at
// chunk position c ^ swz(r).  With swz(r) = ((r&7) + (r>>3)) & 7 the three access patterns used here are free
// of bank conflicts: 16-byte fragment reads by 8 consecutive rows, 16-byte row-major stores, and the 8-byte
// (bf16) / 16-byte (fp32) stores of the transposing loader, whose lanes walk rows 8 (or 4) apart.
//
// Loaders move global memory -> registers (so the next tiles' loads are in flight during the MFMAs of the
// current one) and registers -> LDS.  Loads are unconditional: a tile row beyond the operand is read from the
// operand's last row (it only feeds output rows / columns that are never stored), a K index beyond the range is
// read from the last valid one and replaced by zero.  No branch surrounds a load, so the loads of a tile issue
// back to back and the compiler can wait for exactly the tile it needs.  The direct loader takes a K-contiguous source.  The transposing loader
// takes a source whose rows are K and whose contiguous index is the tile's row: each thread reads a 4 (K) x
// 16-byte block, transposes it in registers and writes K-contiguous pieces.
#pragma once
#include "common.h"

namespace dipaco {

constexpr int TILE_ROW_BYTES = 128;
constexpr int GEMM_THREADS = 256;

template <typename T> struct MmaTraits;
template <> struct MmaTraits<bf16> { static constexpr int VEC = 8; static constexpr int BK = 64; };
template <> struct MmaTraits<float> { static constexpr int VEC = 4; static constexpr int BK = 32; };

// v if keep, else zero -- as a bitwise AND, so that the compiler cannot turn the load of v into a conditional one
__device__ __forceinline__ uint4 keep_or_zero(const uint4& v, bool keep) {
  const uint32_t m = keep ? 0xffffffffu : 0u;
  return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m);
}

__device__ __forceinline__ int swz(int row) { return ((row & 7) + (row >> 3)) & 7; }

__device__ __forceinline__ char* tile_chunk(char* tile, int row, int chunk) {
  return tile + row * TILE_ROW_BYTES + ((chunk ^ swz(row)) << 4);
}

// One K-group step of a 32x32 MFMA tile.  a, b: this lane's 16-byte fragments (row l%32 of the A / B tile,
// chunk 2*ks + l/32).  bf16: one 32x32x16 MFMA.  fp32: four 32x32x2 MFMAs; MFMA s contracts element s of the
// two lane halves' chunks (the same K on both operands, so the order of K inside the step does not matter).
template <typename T> __device__ __forceinline__ void mma_step(f32x16& acc, const uint4& a, const uint4& b);
template <> __device__ __forceinline__ void mma_step<bf16>(f32x16& acc, const uint4& a, const uint4& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0,
                                                0, 0);
}
template <> __device__ __forceinline__ void mma_step<float>(f32x16& acc, const uint4& a, const uint4& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}

// Accumulator element e (0..15) of a 32x32 tile held by lane l: row 8*(e/4) + 4*(l/32) + e%4, column l%32.
__device__ __forceinline__ int acc_row(int e, int lane) { return 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3); }

// ---------------------------------------------------------------------------------------------------------
template <typename T, int ROWS, bool TRANS> struct TileLoader;

// K-contiguous source: element (row, k) at src[row * ld + k].
template <typename T, int ROWS> struct TileLoader<T, ROWS, false> {
  static constexpr int NLD = ROWS / 32;
  static constexpr int VEC = MmaTraits<T>::VEC;
  __device__ static __forceinline__ void load(uint4 (&r)[NLD], const T* __restrict__ src, long ld, int row0,
                                              int rows_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      int idx = tid + GEMM_THREADS * i;
      int row = min(row0 + (idx >> 3), rows_total - 1);
      int k = k0 + (idx & 7) * VEC;
      r[i] = *reinterpret_cast<const uint4*>(src + (long)row * ld + min(k, k_end - VEC));
    }
  }
  // k0, k_end: those of the load that filled r
  __device__ static __forceinline__ void store(const uint4 (&r)[NLD], char* tile, int tid, int k0, int k_end) {
    if (k0 + MmaTraits<T>::BK <= k_end) {   // whole tile inside the K range (uniform branch)
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        int idx = tid + GEMM_THREADS * i;
        *reinterpret_cast<uint4*>(tile_chunk(tile, idx >> 3, idx & 7)) = r[i];
      }
    } else {
      const bool keep = k0 + (tid & 7) * VEC < k_end;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        int idx = tid + GEMM_THREADS * i;
        *reinterpret_cast<uint4*>(tile_chunk(tile, idx >> 3, idx & 7)) = keep_or_zero(r[i], keep);
      }
    }
  }
};

// Row-contiguous bf16 source: element (row, k) at src[k * ld + row].  rows_total % 8 == 0.
template <int ROWS> struct TileLoader<bf16, ROWS, true> {
  static constexpr int NLD = ROWS / 32;
  static constexpr int NSB = ROWS / 128;
  __device__ static __forceinline__ void coords(int tid, int sb, int& kq, int& mq) {
    int w = tid >> 6, l = tid & 63, a = l >> 3;
    kq = 4 * w + (a & 3);                  // block of 4 K rows, 0..15
    mq = (l & 7) + 8 * (a >> 2) + 16 * sb;  // block of 8 tile rows
  }
  __device__ static __forceinline__ void load(uint4 (&r)[NLD], const bf16* __restrict__ src, long ld, int row0,
                                              int rows_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      int row = min(row0 + 8 * mq, rows_total - 8);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int k = k0 + 4 * kq + j;
        r[4 * sb + j] = *reinterpret_cast<const uint4*>(src + (long)min(k, k_end - 1) * ld + row);
      }
    }
  }
  __device__ static __forceinline__ void store(const uint4 (&r)[NLD], char* tile, int tid, int k0, int k_end) {
    if (k0 + MmaTraits<bf16>::BK <= k_end) store_impl<false>(r, tile, tid, k0, k_end);   // uniform branch
    else store_impl<true>(r, tile, tid, k0, k_end);
  }
  template <bool TAIL>
  __device__ static __forceinline__ void store_impl(const uint4 (&r)[NLD], char* tile, int tid, int k0, int k_end) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      const int kk = k0 + 4 * kq;
      const uint4 m0 = keep_or_zero(r[4 * sb + 0], !TAIL || kk + 0 < k_end), m1 = keep_or_zero(r[4 * sb + 1], !TAIL || kk + 1 < k_end);
      const uint4 m2 = keep_or_zero(r[4 * sb + 2], !TAIL || kk + 2 < k_end), m3 = keep_or_zero(r[4 * sb + 3], !TAIL || kk + 3 < k_end);
      const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&m0);
      const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&m1);
      const uint32_t* w2 = reinterpret_cast<const uint32_t*>(&m2);
      const uint32_t* w3 = reinterpret_cast<const uint32_t*>(&m3);
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        int j = c >> 1;
        uint2 out;
        if ((c & 1) == 0) {
          out.x = (w0[j] & 0xffffu) | (w1[j] << 16);
          out.y = (w2[j] & 0xffffu) | (w3[j] << 16);
        } else {
          out.x = (w0[j] >> 16) | (w1[j] & 0xffff0000u);
          out.y = (w2[j] >> 16) | (w3[j] & 0xffff0000u);
        }
        int row = 8 * mq + c;
        *reinterpret_cast<uint2*>(tile_chunk(tile, row, kq >> 1) + ((kq & 1) << 3)) = out;
      }
    }
  }
};

// Row-contiguous fp32 source: element (row, k) at src[k * ld + row].  rows_total % 4 == 0.
template <int ROWS> struct TileLoader<float, ROWS, true> {
  static constexpr int NLD = ROWS / 32;
  static constexpr int NSB = ROWS / 128;
  __device__ static __forceinline__ void coords(int tid, int sb, int& kq, int& mq) {
    int w = tid >> 6, l = tid & 63;
    kq = 2 * w + (l >> 5);     // block of 4 K rows, 0..7
    mq = (l & 31) + 32 * sb;   // block of 4 tile rows
  }
  __device__ static __forceinline__ void load(uint4 (&r)[NLD], const float* __restrict__ src, long ld, int row0,
                                              int rows_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      int row = min(row0 + 4 * mq, rows_total - 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int k = k0 + 4 * kq + j;
        r[4 * sb + j] = *reinterpret_cast<const uint4*>(src + (long)min(k, k_end - 1) * ld + row);
      }
    }
  }
  __device__ static __forceinline__ void store(const uint4 (&r)[NLD], char* tile, int tid, int k0, int k_end) {
    if (k0 + MmaTraits<float>::BK <= k_end) store_impl<false>(r, tile, tid, k0, k_end);   // uniform branch
    else store_impl<true>(r, tile, tid, k0, k_end);
  }
  template <bool TAIL>
  __device__ static __forceinline__ void store_impl(const uint4 (&r)[NLD], char* tile, int tid, int k0, int k_end) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      const int kk = k0 + 4 * kq;
      const uint4 a = keep_or_zero(r[4 * sb + 0], !TAIL || kk + 0 < k_end), b = keep_or_zero(r[4 * sb + 1], !TAIL || kk + 1 < k_end);
      const uint4 c = keep_or_zero(r[4 * sb + 2], !TAIL || kk + 2 < k_end), d = keep_or_zero(r[4 * sb + 3], !TAIL || kk + 3 < k_end);
      *reinterpret_cast<uint4*>(tile_chunk(tile, 4 * mq + 0, kq)) = make_uint4(a.x, b.x, c.x, d.x);
      *reinterpret_cast<uint4*>(tile_chunk(tile, 4 * mq + 1, kq)) = make_uint4(a.y, b.y, c.y, d.y);
      *reinterpret_cast<uint4*>(tile_chunk(tile, 4 * mq + 2, kq)) = make_uint4(a.z, b.z, c.z, d.z);
      *reinterpret_cast<uint4*>(tile_chunk(tile, 4 * mq + 3, kq)) = make_uint4(a.w, b.w, c.w, d.w);
    }
  }
};

// All MFMAs of one K tile for a wave that owns TM x TN 32x32 tiles starting at rows a_row0 / b_row0.
template <typename T, int TM, int TN>
__device__ __forceinline__ void mma_ktile(f32x16 (&acc)[TM][TN], char* a_tile, char* b_tile, int a_row0, int b_row0,
                                          int lane) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    uint4 af[TM], bfr[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const uint4*>(tile_chunk(a_tile, a_row0 + 32 * i + r, 2 * ks + h));
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const uint4*>(tile_chunk(b_tile, b_row0 + 32 * j + r, 2 * ks + h));
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) mma_step<T>(acc[i][j], af[i], bfr[j]);
  }
}

}  // namespace dipaco
