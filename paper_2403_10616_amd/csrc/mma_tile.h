// LDS operand tiles for the gfx950 matrix cores and the loaders that fill them.
//
// An operand tile is ROWS rows (the M or N index) by 128 bytes of the contraction index K (64 bf16 or 32
// fp32), K-contiguous: that is the order in which v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32 want both
// operands (lane l supplies row l%32, K-group l/32).  A row is 8 chunks of 16 bytes; chunk c of row r lives at
// chunk position c ^ swz(r), swz(r) = (r >> 1) & 7.
//
// Why this swizzle.  LDS has 64 banks of 4 bytes (addresses 256 bytes apart share a bank).  Measured on gfx950
// with two-lane probes and the SQ_LDS_BANK_CONFLICT counter, the lanes of a wave are served together in these
// sets:  ds_read_b128: {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31} and the same +32;  ds_read_b64: 32 consecutive
// lanes;  ds_write_b128: 8 consecutive lanes;  ds_write_b64: 16 consecutive lanes.  An access is free of conflicts
// when the lanes of a set touch different 16-byte (8-byte) slots of the 256-byte bank space.  A fragment read has
// lane l on row l%32: the rows of either read set, split by parity (odd rows sit 128 bytes higher), take every
// value of (r >> 1) & 7 once, so XOR-ing it into the chunk spreads them over the 8 chunk positions.  Row-major
// 16-byte stores put 8 consecutive lanes on the 8 chunks of one row.  The transposing loader assigns lanes so
// that 16 consecutive lanes write 8 K-granules of two rows of different swizzle (see its coords()).
//
// Loaders move global memory -> registers -> LDS, so that loads of later tiles are in flight during the MFMAs
// of the current one.  Every thread's element offsets inside the operand are fixed for the whole K loop and
// kept as 32-bit values; a tile is addressed as (operand + K offset, uniform) + offset.  Loads are unconditional:
// a tile row beyond the operand reads the operand's last rows (it only feeds output rows / columns that are
// never stored).  A K tile that sticks out of the K range takes a slower path (chosen by a uniform branch) that
// reads the last valid K index instead and zeroes the excess when the tile is written to LDS.
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

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

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
// TileLoader<T, ROWS, TRANS>:
//   offsets(off, ld, row0, rows_total, tid)   this thread's element offsets, relative to K offset 0
//   k_step(ld)                                elements to advance the operand pointer per unit of K
//   load_full(r, src_k, off)                  tile completely inside the K range; src_k = operand + k0 * k_step
//   load_tail(r, src, ld, row0, rows_total, k0, k_end, tid)    any tile (K indices clamped to the last valid one)
//   store(r, tile, tid, k0, k_end)            registers -> LDS (zeroing K >= k_end)
template <typename T, int ROWS, bool TRANS, int NT = GEMM_THREADS> struct TileLoader;   // NT threads fill a tile

// K-contiguous source: element (row, k) at src[row * ld + k].
template <typename T, int ROWS, int NT> struct TileLoader<T, ROWS, false, NT> {
  static constexpr int NLD = ROWS * 8 / NT;
  static constexpr int VEC = MmaTraits<T>::VEC;
  __device__ static __forceinline__ long k_step(long) { return 1; }
  __device__ static __forceinline__ void offsets(uint32_t (&off)[NLD], long ld, int row0, int rows_total, int tid) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + NT * i;
      const int row = min(row0 + (idx >> 3), rows_total - 1);
      off[i] = (uint32_t)((long)row * ld + (idx & 7) * VEC);
    }
  }
  __device__ static __forceinline__ void load_full(uint4 (&r)[NLD], const T* __restrict__ src_k,
                                                   const uint32_t (&off)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) r[i] = *reinterpret_cast<const uint4*>(src_k + off[i]);
  }
  __device__ static __forceinline__ void load_tail(uint4 (&r)[NLD], const T* __restrict__ src, long ld, int row0,
                                                   int rows_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + NT * i;
      const int row = min(row0 + (idx >> 3), rows_total - 1);
      const int k = min(k0 + (idx & 7) * VEC, k_end - VEC);
      r[i] = *reinterpret_cast<const uint4*>(src + (long)row * ld + k);
    }
  }
  __device__ static __forceinline__ void store_full(const uint4 (&r)[NLD], char* tile, int tid) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int idx = tid + NT * i;
      *reinterpret_cast<uint4*>(tile_chunk(tile, idx >> 3, idx & 7)) = r[i];
    }
  }
  __device__ static __forceinline__ void store(const uint4 (&r)[NLD], char* tile, int tid, int k0, int k_end) {
    if (k0 + MmaTraits<T>::BK <= k_end) {   // whole tile inside the K range (uniform branch)
      store_full(r, tile, tid);
    } else {
      const bool keep = k0 + (tid & 7) * VEC < k_end;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int idx = tid + NT * i;
        *reinterpret_cast<uint4*>(tile_chunk(tile, idx >> 3, idx & 7)) = keep_or_zero(r[i], keep);
      }
    }
  }
};

// Row-contiguous bf16 source: element (row, k) at src[k * ld + row].  rows_total % 8 == 0.
// A thread owns 4 (K) x 8 (rows) blocks.  Lane l of wave w: 8-row block mq = (l&1) + 2*((l>>4)&3) + 8*(w>>1),
// 4-K block kq = ((l>>1)&7) + 8*(w&1).  One load instruction then reads, per K row, 128 contiguous bytes; one
// 8-byte LDS store instruction has each run of 16 consecutive lanes write 8 K-granules of two rows whose swizzles
// differ by 4: sixteen different 8-byte slots.
template <int ROWS, int NT> struct TileLoader<bf16, ROWS, true, NT> {
  static constexpr int NLD = ROWS * 8 / NT;
  static constexpr int NSB = NLD / 4;          // 4 x 8 blocks per thread; NT threads cover NT/2 rows per pass
  __device__ static __forceinline__ long k_step(long ld) { return ld; }
  __device__ static __forceinline__ void coords(int tid, int sb, int& kq, int& mq) {
    const int w = tid >> 6, l = tid & 63;
    kq = ((l >> 1) & 7) + 8 * (w & 1);
    mq = (l & 1) + 2 * ((l >> 4) & 3) + 8 * (w >> 1) + (NT / 16) * sb;
  }
  __device__ static __forceinline__ void offsets(uint32_t (&off)[NLD], long ld, int row0, int rows_total, int tid) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      const int row = min(row0 + 8 * mq, rows_total - 8);
#pragma unroll
      for (int j = 0; j < 4; ++j) off[4 * sb + j] = (uint32_t)((long)(4 * kq + j) * ld + row);
    }
  }
  __device__ static __forceinline__ void load_full(uint4 (&r)[NLD], const bf16* __restrict__ src_k,
                                                   const uint32_t (&off)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) r[i] = *reinterpret_cast<const uint4*>(src_k + off[i]);
  }
  __device__ static __forceinline__ void load_tail(uint4 (&r)[NLD], const bf16* __restrict__ src, long ld, int row0,
                                                   int rows_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      const int row = min(row0 + 8 * mq, rows_total - 8);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = min(k0 + 4 * kq + j, k_end - 1);
        r[4 * sb + j] = *reinterpret_cast<const uint4*>(src + (long)k * ld + row);
      }
    }
  }
  __device__ static __forceinline__ void store_full(const uint4 (&r)[NLD], char* tile, int tid) {
    store_impl<false>(r, tile, tid, 0, 0);
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
        const int j = c >> 1;
        uint2 out;
        if ((c & 1) == 0) {
          out.x = (w0[j] & 0xffffu) | (w1[j] << 16);
          out.y = (w2[j] & 0xffffu) | (w3[j] << 16);
        } else {
          out.x = (w0[j] >> 16) | (w1[j] & 0xffff0000u);
          out.y = (w2[j] >> 16) | (w3[j] & 0xffff0000u);
        }
        const int row = 8 * mq + c;
        *reinterpret_cast<uint2*>(tile_chunk(tile, row, kq >> 1) + ((kq & 1) << 3)) = out;
      }
    }
  }
};

// Row-contiguous fp32 source: element (row, k) at src[k * ld + row].  rows_total % 4 == 0.
// A thread owns 4 (K) x 4 (rows) blocks: lane l of wave w has 4-row block mq = (l&3) + 4*((l>>3)&7) and 4-K block
// kq = ((l>>2)&1) + 2*w, so that 8 consecutive lanes write 8 different 16-byte slots.
template <int ROWS, int NT> struct TileLoader<float, ROWS, true, NT> {
  static constexpr int NLD = ROWS * 8 / NT;
  static constexpr int NSB = NLD / 4;
  __device__ static __forceinline__ long k_step(long ld) { return ld; }
  __device__ static __forceinline__ void coords(int tid, int sb, int& kq, int& mq) {
    const int w = tid >> 6, l = tid & 63;
    kq = ((l >> 2) & 1) + 2 * (w & 3);
    mq = (l & 3) + 4 * ((l >> 3) & 7) + 32 * (w >> 2) + (NT / 8) * sb;
  }
  __device__ static __forceinline__ void offsets(uint32_t (&off)[NLD], long ld, int row0, int rows_total, int tid) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      const int row = min(row0 + 4 * mq, rows_total - 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) off[4 * sb + j] = (uint32_t)((long)(4 * kq + j) * ld + row);
    }
  }
  __device__ static __forceinline__ void load_full(uint4 (&r)[NLD], const float* __restrict__ src_k,
                                                   const uint32_t (&off)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) r[i] = *reinterpret_cast<const uint4*>(src_k + off[i]);
  }
  __device__ static __forceinline__ void load_tail(uint4 (&r)[NLD], const float* __restrict__ src, long ld, int row0,
                                                   int rows_total, int k0, int k_end, int tid) {
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
      int kq, mq;
      coords(tid, sb, kq, mq);
      const int row = min(row0 + 4 * mq, rows_total - 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = min(k0 + 4 * kq + j, k_end - 1);
        r[4 * sb + j] = *reinterpret_cast<const uint4*>(src + (long)k * ld + row);
      }
    }
  }
  __device__ static __forceinline__ void store_full(const uint4 (&r)[NLD], char* tile, int tid) {
    store_impl<false>(r, tile, tid, 0, 0);
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

// Fragments of K group ks (chunk 2*ks + l/32) for a wave that owns TM x TN 32x32 tiles starting at rows
// a_row0 / b_row0 of the A / B tile.
template <int TM, int TN>
__device__ __forceinline__ void load_frags(uint4 (&af)[TM], uint4 (&bfr)[TN], char* a_tile, char* b_tile, int a_row0,
                                           int b_row0, int lane, int ks) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const uint4*>(tile_chunk(a_tile, a_row0 + 32 * i + r, 2 * ks + h));
#pragma unroll
  for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const uint4*>(tile_chunk(b_tile, b_row0 + 32 * j + r, 2 * ks + h));
}
template <typename T, int TM, int TN>
__device__ __forceinline__ void mma_group(f32x16 (&acc)[TM][TN], const uint4 (&af)[TM], const uint4 (&bfr)[TN]) {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) mma_step<T>(acc[i][j], af[i], bfr[j]);
}
// Ask the scheduler to issue the NR fragment reads and NM MFMAs just emitted interleaved (reads spread under
// the MFMAs) instead of all reads first.
template <int NR, int NM> __device__ __forceinline__ void interleave_reads_with_mfma() {
  constexpr int Q = NM / NR > 0 ? NM / NR : 1;
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
    __builtin_amdgcn_sched_group_barrier(0x008, Q, 0);   // Q MFMAs
  }
  if (NM > Q * NR) __builtin_amdgcn_sched_group_barrier(0x008, NM - Q * NR, 0);
}

// All MFMAs of one K tile (fragments of group ks+1 are read while the MFMAs of group ks run).
template <typename T, int TM, int TN>
__device__ __forceinline__ void mma_ktile(f32x16 (&acc)[TM][TN], char* a_tile, char* b_tile, int a_row0, int b_row0,
                                          int lane) {
  uint4 af[2][TM], bfr[2][TN];
  load_frags<TM, TN>(af[0], bfr[0], a_tile, b_tile, a_row0, b_row0, lane, 0);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    if (ks < 3) load_frags<TM, TN>(af[(ks + 1) & 1], bfr[(ks + 1) & 1], a_tile, b_tile, a_row0, b_row0, lane, ks + 1);
    mma_group<T, TM, TN>(acc, af[ks & 1], bfr[ks & 1]);
  }
}

}  // namespace dipaco
