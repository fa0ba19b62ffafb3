// Pieces shared by the matrix-core GEMM kernels: the kernel argument block, the workgroup -> tile mapping and
// the epilogue that turns a wave's accumulators into 16-byte row-contiguous stores.
#pragma once
#include "common.h"
#include "mma_tile.h"

namespace dipaco {

struct GemmDev {
  const void* A; const void* B; void* C;
  int M, N, K;
  long lda, ldb, ldc;
  const void* bias; const void* resid; void* aux_out; const void* aux_in;
  int act;
  int splits;
  int k_per_split;   // multiple of BK
  float* partial;
  float* colsum_partial = nullptr;   // [ceil(M / rows of a wave)][N]: column sums of each wave's rows of C
  int tiles_m, tiles_n;
  // Uneven split-K (weight gradients, one workgroup per compute unit): tiles fall into four classes -- inside C,
  // sticking out over its last rows, over its last columns, over both -- and a class whose tiles cost less per K
  // step is cut into fewer K slices, so that all workgroups of the launch end together.  Class c owns workgroup
  // ids [cls_base[c], cls_base[c + 1]), slice-major; full_m / full_n = tile rows / columns of the first class.
  int uneven = 0;
  int cls_s[4];
  int cls_base[5];
  int full_m, full_n;
};

constexpr int N_XCD = 8;

template <typename T> struct OutVec;   // 8 consecutive output elements
template <> struct OutVec<float> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
};
template <> struct OutVec<bf16> {
  static __device__ __forceinline__ void load(const bf16* p, float (&v)[8]) { load_vec16<bf16>(p, v); }
  static __device__ __forceinline__ void store(bf16* p, const float (&v)[8]) { store_vec16<bf16>(p, v); }
};


// Workgroup ids are dealt to the 8 XCDs round-robin and every XCD owns a private L2: XCD x gets the contiguous
// range of tile ids [x * per, ...), walked in groups of 8 tile rows that share their B panels.
__device__ __forceinline__ void gemm_tile_of_block(const GemmDev& g, int bid, int& split, int& tile_m, int& tile_n) {
  const int tiles = g.tiles_m * g.tiles_n;
  split = bid / tiles;
  bid -= split * tiles;
  {
    const int per = tiles / N_XCD, rem = tiles % N_XCD;
    const int x = bid % N_XCD, i = bid / N_XCD;
    bid = x * per + min(x, rem) + i;
  }
  const int group = 8;
  const int per_group = group * g.tiles_n;
  const int gidx = bid / per_group;
  const int first_m = gidx * group;
  const int gsize = min(group, g.tiles_m - first_m);
  const int in_group = bid - gidx * per_group;
  tile_m = first_m + in_group % gsize;
  tile_n = in_group / gsize;
}

// XCD x gets the contiguous range [x * per, ...) of `total` work items
__device__ __forceinline__ int xcd_contiguous(int bid, int total) {
  const int per = total / N_XCD, rem = total % N_XCD;
  const int x = bid % N_XCD, i = bid / N_XCD;
  return x * per + min(x, rem) + i;
}

// Uneven split-K: workgroup id -> tile, K slice and the number of slices its tile is cut into.
__device__ __forceinline__ void gemm_uneven_of_block(const GemmDev& g, int bid, int& split, int& nsplit, int& tile_m,
                                                     int& tile_n) {
  const int v = xcd_contiguous(bid, g.cls_base[4]);
  const int c = (v >= g.cls_base[1]) + (v >= g.cls_base[2]) + (v >= g.cls_base[3]);
  const int local = v - g.cls_base[c];
  nsplit = g.cls_s[c];
  const int n_tiles = (g.cls_base[c + 1] - g.cls_base[c]) / nsplit;
  split = local / n_tiles;
  const int t = local - split * n_tiles;
  if (c == 0) { tile_m = t % g.full_m; tile_n = t / g.full_m; }
  else if (c == 1) { tile_m = g.full_m; tile_n = t; }
  else if (c == 2) { tile_m = t; tile_n = g.full_n; }
  else { tile_m = g.full_m; tile_n = g.full_n; }
}

// Eight consecutive elements of T as raw 16-byte vectors (loaded early, converted when used).
template <typename T> struct Raw8 { uint4 v[sizeof(T) / 2]; };
template <typename T> __device__ __forceinline__ Raw8<T> raw8_load(const T* p) {
  Raw8<T> r;
#pragma unroll
  for (int k = 0; k < (int)sizeof(T) / 2; ++k) r.v[k] = reinterpret_cast<const uint4*>(p)[k];
  return r;
}
template <typename T> __device__ __forceinline__ void raw8_unpack(const Raw8<T>& r, float (&out)[8]) {
  const T* e = reinterpret_cast<const T*>(&r);
#pragma unroll
  for (int c = 0; c < 8; ++c) out[c] = to_f32(e[c]);
}

// Epilogue of one wave: its TM x TN accumulator tiles (32 x 32 each, rows from row0, columns from col0) go
// through stg, a wave-private LDS region of 32 x (WN + 4) floats, 32 rows at a time, so that bias / GELU /
// residual are applied on, and C is written with, 16-byte row-contiguous accesses.  N is a multiple of 8 (checked
// on the host), so an 8-column group is either inside C or outside.  The residual / auxiliary input vectors of a
// block of 32 rows are requested one block ahead (two register buffers), so that their latency hides behind the
// staging, arithmetic and stores of the block before.
template <typename T, typename TC, int TM, int TN, int WN>
__device__ __forceinline__ void gemm_epilogue(const f32x16 (&acc)[TM][TN], float* stg, int lane, int row0, int col0,
                                              int split, const GemmDev& g) {
  constexpr int LDW = WN + 4;
  const int col_l = lane & 31;
  constexpr int GROUPS = WN / 8;                 // 8-column groups per row
  constexpr int ITERS = 32 * GROUPS / WAVE;
  const T* bias = static_cast<const T*>(g.bias);
  const T* resid = static_cast<const T*>(g.resid);
  const T* aux_in = static_cast<const T*>(g.aux_in);
  T* aux_out = static_cast<T*>(g.aux_out);
  const bool to_partial = g.splits > 1;
  float* P = to_partial ? g.partial + (size_t)split * g.M * g.N : nullptr;
  const bool want_aux = g.act == 2 || g.act == 4;
  // one operand stream is requested ahead: the saved operand if there is one, else the residual (a product that
  // takes both loads its residual where it is used)
  const T* ahead = want_aux ? aux_in : resid;
  const bool resid_late = want_aux && resid;
  Raw8<T> rin[2][ITERS];
  // requests the vectors of 32-row block i into buffer i & 1
  auto prefetch = [&](int i) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int item = lane + WAVE * it;
      const int row = row0 + 32 * i + item / GROUPS, col = col0 + 8 * (item % GROUPS);
      if (ahead && row < g.M && col < g.N) rin[i & 1][it] = raw8_load(ahead + (size_t)row * g.ldc + col);
    }
  };
  prefetch(0);
  static_assert(WAVE % GROUPS == 0, "a lane keeps its column group over the items");
  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // column sums over this lane's rows
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i + 1 < TM) prefetch(i + 1);   // in flight while block i is staged, combined and stored
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) stg[acc_row(e, lane) * LDW + 32 * j + col_l] = acc[i][j][e];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int item = lane + WAVE * it;
      const int rr = item / GROUPS, cg = item % GROUPS;
      const int row = row0 + 32 * i + rr;
      const int col = col0 + 8 * cg;
      const float4 lo = *reinterpret_cast<const float4*>(stg + rr * LDW + 8 * cg);
      const float4 hi = *reinterpret_cast<const float4*>(stg + rr * LDW + 8 * cg + 4);
      float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      if (row >= g.M || col >= g.N) continue;
      if (to_partial) {
        OutVec<float>::store(P + (size_t)row * g.N + col, v);
        continue;
      }
      const size_t off = (size_t)row * g.ldc + col;
      if (bias) {
        float b[8];
        OutVec<T>::load(bias + col, b);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] += b[c];
      }
      if (g.act == 1) {
        // the saved pre-activation is what backward differentiates at: GELU is applied to the stored value
        OutVec<T>::store(aux_out + off, v);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = gelu_t<T>(to_f32(from_f32<T>(v[c])));
      } else if (g.act == 3) {
        float dv[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = gelu_with_grad_t<T>(v[c], dv[c]);
        OutVec<T>::store(aux_out + off, dv);
      } else if (want_aux) {
        float u[8];
        raw8_unpack(rin[i & 1][it], u);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] *= g.act == 2 ? gelu_grad_t<T>(u[c]) : u[c];
      }
      if (resid) {
        float rv[8];
        raw8_unpack(resid_late ? raw8_load(resid + off) : rin[i & 1][it], rv);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] += rv[c];
      }
      OutVec<TC>::store(static_cast<TC*>(g.C) + off, v);
      if (g.colsum_partial) {
#pragma unroll
        for (int c = 0; c < 8; ++c) cs[c] += v[c];
      }
    }
  }
  if (g.colsum_partial && !to_partial) {
    // lanes l, l + GROUPS, ... hold the same columns: fixed butterfly, then one row of partial sums per wave
#pragma unroll
    for (int m = GROUPS; m < WAVE; m <<= 1)
#pragma unroll
      for (int c = 0; c < 8; ++c) cs[c] += __shfl_xor(cs[c], m, WAVE);
    const int col = col0 + 8 * lane;
    if (lane < GROUPS && col < g.N && row0 < g.M)
      OutVec<float>::store(g.colsum_partial + (size_t)(row0 / (32 * TM)) * g.N + col, cs);
  }
}

}  // namespace dipaco
