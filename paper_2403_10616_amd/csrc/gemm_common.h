// Pieces shared by the matrix-core GEMM kernels: the kernel argument block, the workgroup -> tile mapping and
// the epilogue that turns a wave's accumulators into 16-byte row-contiguous stores.
#pragma once
#include <type_traits>
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
  // tile mapping without run-time divisions (filled by the host when the sizes allow, see gemm_fast_map):
  // tiles per XCD and their remainder, and ceil(2^32 / (8 tiles_n))
  int fast_map = 0, xcd_per = 0, xcd_rem = 0;
  unsigned group_mul = 0;
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

// The same mapping for one K range per tile (splits == 1), with the divisions done on the host: a workgroup issues
// its first loads some hundred instructions earlier.  Valid when g.fast_map is set.
__device__ __forceinline__ void gemm_tile_of_block_fast(const GemmDev& g, int bid, int& tile_m, int& tile_n) {
  const int x = bid & (N_XCD - 1), i = bid >> 3;
  const int vt = x * g.xcd_per + min(x, g.xcd_rem) + i;
  const int per_group = 8 * g.tiles_n;
  const int gidx = (int)__umulhi((unsigned)vt, g.group_mul);   // vt / per_group, exact for vt * per_group < 2^32
  const int first_m = gidx * 8;
  const int in_group = vt - gidx * per_group;
  const int gsize = g.tiles_m - first_m;
  if (gsize >= 8) {
    tile_m = first_m + (in_group & 7);
    tile_n = in_group >> 3;
  } else {   // the last, shorter group of tile rows
    tile_m = first_m + in_group % gsize;
    tile_n = in_group / gsize;
  }
}
// host side of the above
inline void gemm_fast_map(GemmDev& g) {
  static_assert(N_XCD == 8, "the fast mapping is written for 8 XCDs");
  const long tiles = (long)g.tiles_m * g.tiles_n, per_group = 8L * g.tiles_n;
  g.fast_map = g.splits == 1 && !g.uneven && tiles * per_group < (1L << 32) && per_group > 1;
  if (!g.fast_map) return;
  g.xcd_per = (int)(tiles / N_XCD);
  g.xcd_rem = (int)(tiles % N_XCD);
  g.group_mul = (unsigned)(((1ULL << 32) + per_group - 1) / per_group);
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

// Rows 32 i .. 32 i + 31 of a wave's accumulators into its staging region (row stride LDW floats), for the two
// accumulator layouts: 32 x 32 tiles of v_mfma_f32_32x32x16 (lane: column l % 32, rows acc_row(e, l)) and 16 x 16 tiles
// of v_mfma_f32_16x16x32 (lane: column l % 16, rows 4 (l / 16) + e); the latter come as [2 TM][2 TN] tiles.
template <int LDW, int TM, int TN>
__device__ __forceinline__ void stage_block(const f32x16 (&acc)[TM][TN], int i, float* stg, int lane) {
  const int col_l = lane & 31;
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) stg[acc_row(e, lane) * LDW + 32 * j + col_l] = acc[i][j][e];
}
template <int LDW, int TM2, int TN2>
__device__ __forceinline__ void stage_block(const f32x4 (&acc)[TM2][TN2], int i, float* stg, int lane) {
  const int col_l = lane & 15, row_l = 4 * (lane >> 4);
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int j = 0; j < TN2; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) stg[(16 * a + row_l + e) * LDW + 16 * j + col_l] = acc[2 * i + a][j][e];
}

// Epilogue of one wave: its TM x TN accumulator tiles (32 x 32 each, rows from row0, columns from col0) go
// through stg, a wave-private LDS region of 32 x (WN + 4) floats, 32 rows at a time, so that bias / GELU /
// residual are applied on, and C is written with, 16-byte row-contiguous accesses.  N is a multiple of 8 (checked
// on the host), so an 8-column group is either inside C or outside.  The residual / auxiliary input vectors of a
// block of 32 rows are requested one block ahead (two register buffers), so that their latency hides behind the
// staging, arithmetic and stores of the block before.
template <typename T, typename TC, int TM, int TN, int WN, typename ACC>
__device__ __forceinline__ void gemm_epilogue(const ACC& acc, float* stg, int lane, int row0, int col0,
                                              int split, const GemmDev& g) {
  // The argument block lives in kernel-argument memory: every field the loops below use is read once, here, so
  // that no scalar load (and the wait for it, which also stalls the LDS traffic) is left inside them.
  const int gM = g.M, gN = g.N, g_act = g.act;
  const long g_ldc = g.ldc;
  TC* const gC = static_cast<TC*>(g.C);
  float* const g_cs = g.colsum_partial;

  constexpr int LDW = WN + 4;
  constexpr int GROUPS = WN / 8;                 // 8-column groups per row
  constexpr int ITERS = 32 * GROUPS / WAVE;
  const T* bias = static_cast<const T*>(g.bias);
  const T* resid = static_cast<const T*>(g.resid);
  const T* aux_in = static_cast<const T*>(g.aux_in);
  T* aux_out = static_cast<T*>(g.aux_out);
  const bool to_partial = g.splits > 1;
  float* P = to_partial ? g.partial + (size_t)split * gM * gN : nullptr;
  const bool want_aux = g_act == 2 || g_act == 4;
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
      if (ahead && row < gM && col < gN) rin[i & 1][it] = raw8_load(ahead + (size_t)row * g_ldc + col);
    }
  };
  prefetch(0);
  static_assert(WAVE % GROUPS == 0, "a lane keeps its column group over the items");
  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // column sums over this lane's rows
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (i + 1 < TM) prefetch(i + 1);   // in flight while block i is staged, combined and stored
    __builtin_amdgcn_wave_barrier();
    stage_block<LDW>(acc, i, stg, lane);
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
      if (row >= gM || col >= gN) continue;
      if (to_partial) {
        OutVec<float>::store(P + (size_t)row * gN + col, v);
        continue;
      }
      const size_t off = (size_t)row * g_ldc + col;
      if (bias) {
        float b[8];
        OutVec<T>::load(bias + col, b);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] += b[c];
      }
      if (g_act == 1) {
        // the saved pre-activation is what backward differentiates at: GELU is applied to the stored value
        OutVec<T>::store(aux_out + off, v);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = gelu_t<T>(to_f32(from_f32<T>(v[c])));
      } else if (g_act == 3) {
        float dv[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] = gelu_with_grad_t<T>(v[c], dv[c]);
        OutVec<T>::store(aux_out + off, dv);
      } else if (want_aux) {
        float u[8];
        raw8_unpack(rin[i & 1][it], u);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] *= g_act == 2 ? gelu_grad_t<T>(u[c]) : u[c];
      }
      if (resid) {
        float rv[8];
        raw8_unpack(resid_late ? raw8_load(resid + off) : rin[i & 1][it], rv);
#pragma unroll
        for (int c = 0; c < 8; ++c) v[c] += rv[c];
      }
      OutVec<TC>::store(gC + off, v);
      if (g_cs) {
#pragma unroll
        for (int c = 0; c < 8; ++c) cs[c] += v[c];
      }
    }
  }
  if (g_cs && !to_partial) {
    // lanes l, l + GROUPS, ... hold the same columns: fixed butterfly, then one row of partial sums per wave
#pragma unroll
    for (int m = GROUPS; m < WAVE; m <<= 1)
#pragma unroll
      for (int c = 0; c < 8; ++c) cs[c] += __shfl_xor(cs[c], m, WAVE);
    const int col = col0 + 8 * lane;
    if (lane < GROUPS && col < gN && row0 < gM)
      OutVec<float>::store(g_cs + (size_t)(row0 / (32 * TM)) * gN + col, cs);
  }
}

// The same epilogue with everything that does not depend on the data fixed at compile time -- the activation, which
// of bias / residual / column sums / split-K partial output are present -- for the bf16 direct-to-LDS kernel.  The
// general function above decides all of that per 16-byte item with wave-uniform branches; a wave spends about 2000
// instruction issues there (7 us of a 32 us tile at two waves per SIMD).  Here an item is straight-line code: the
// bias vector is loaded once (a lane keeps its eight columns over all items), addresses advance by constants, and
// the operand prefetch is fenced so that the conversion of the loaded values is not scheduled next to the load.
template <typename TC, int TM, int TN, int WN, int ACT, bool BIAS, bool RESID, bool CS, bool PARTIAL, typename ACC>
__device__ __forceinline__ void gemm_epilogue_fixed(const ACC& acc, float* stg, int lane, int row0,
                                                    int col0, int split, const GemmDev& g) {
  using T = bf16;
  constexpr int LDW = WN + 4;
  constexpr int GROUPS = WN / 8;
  constexpr int ITERS = 32 * GROUPS / WAVE;
  constexpr int ROWS_PER_IT = WAVE / GROUPS;
  constexpr bool AUX_IN = ACT == 2 || ACT == 4, AUX_OUT = ACT == 1 || ACT == 3;
  static_assert(WAVE % GROUPS == 0, "a lane keeps its column group over the items");
  static_assert(!PARTIAL || (ACT == 0 && !BIAS && !RESID && !CS), "split-K partial planes take no epilogue");
  const int gM = g.M, gN = g.N;
  const long ld = PARTIAL ? (long)gN : g.ldc;
  const int rr0 = lane / GROUPS, cg = lane % GROUPS;
  const int col = col0 + 8 * cg;
  const bool col_ok = col < gN;
  const long off0 = (long)(row0 + rr0) * ld + col;                      // element offset of this lane's first item
  using TO = typename std::conditional<PARTIAL, float, TC>::type;
  TO* const out = PARTIAL ? reinterpret_cast<TO*>(g.partial + (size_t)split * gM * gN) : static_cast<TO*>(g.C);
  const T* const ahead = AUX_IN ? static_cast<const T*>(g.aux_in) : static_cast<const T*>(g.resid);
  constexpr bool AHEAD = AUX_IN || RESID;
  constexpr bool RESID_LATE = AUX_IN && RESID;
  float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (BIAS && col_ok) OutVec<T>::load(static_cast<const T*>(g.bias) + col, bv);
  Raw8<T> rin[2][ITERS];
  auto prefetch = [&](int i) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int row = row0 + 32 * i + ROWS_PER_IT * it + rr0;
      if (row < gM && col_ok) rin[i & 1][it] = raw8_load(ahead + off0 + (long)(32 * i + ROWS_PER_IT * it) * ld);
    }
  };
  if (AHEAD) prefetch(0);
  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    if (AHEAD && i + 1 < TM) prefetch(i + 1);
    __builtin_amdgcn_sched_barrier(0);   // the loads above are issued here; what uses them stays below
    __builtin_amdgcn_wave_barrier();
    stage_block<LDW>(acc, i, stg, lane);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int rr = ROWS_PER_IT * it + rr0;
      const int row = row0 + 32 * i + rr;
      const float4 lo = *reinterpret_cast<const float4*>(stg + rr * LDW + 8 * cg);
      const float4 hi = *reinterpret_cast<const float4*>(stg + rr * LDW + 8 * cg + 4);
      float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const long off = off0 + (long)(32 * i + ROWS_PER_IT * it) * ld;
      if (row < gM && col_ok) {
        if (BIAS) {
#pragma unroll
          for (int c = 0; c < 8; ++c) v[c] += bv[c];
        }
        if (ACT == 1) {
          OutVec<T>::store(static_cast<T*>(g.aux_out) + off, v);
#pragma unroll
          for (int c = 0; c < 8; ++c) v[c] = gelu_t<T>(to_f32(from_f32<T>(v[c])));
        } else if (ACT == 3) {
          float dv[8];
#pragma unroll
          for (int c = 0; c < 8; ++c) v[c] = gelu_with_grad_t<T>(v[c], dv[c]);
          OutVec<T>::store(static_cast<T*>(g.aux_out) + off, dv);
        } else if (AUX_IN) {
          float u[8];
          raw8_unpack(rin[i & 1][it], u);
#pragma unroll
          for (int c = 0; c < 8; ++c) v[c] *= ACT == 2 ? gelu_grad_t<T>(u[c]) : u[c];
        }
        if (RESID) {
          float rv[8];
          raw8_unpack(RESID_LATE ? raw8_load(static_cast<const T*>(g.resid) + off) : rin[i & 1][it], rv);
#pragma unroll
          for (int c = 0; c < 8; ++c) v[c] += rv[c];
        }
        OutVec<TO>::store(out + off, v);
        if (CS) {
#pragma unroll
          for (int c = 0; c < 8; ++c) cs[c] += v[c];
        }
      }
    }
  }
  if (CS) {
#pragma unroll
    for (int m = GROUPS; m < WAVE; m <<= 1)
#pragma unroll
      for (int c = 0; c < 8; ++c) cs[c] += __shfl_xor(cs[c], m, WAVE);
    if (lane < GROUPS && col_ok && row0 < gM)
      OutVec<float>::store(g.colsum_partial + (size_t)(row0 / (32 * TM)) * gN + col, cs);
  }
  (void)AUX_OUT;
}

// Picks the fixed epilogue for the combinations the training step uses; everything else takes the general one.
template <typename TC, int TM, int TN, int WN, typename ACC>
__device__ __forceinline__ void gemm_epilogue_dispatch(const ACC& acc, float* stg, int lane, int row0,
                                                       int col0, int split, const GemmDev& g) {
  const bool bias = g.bias != nullptr, resid = g.resid != nullptr, cs = g.colsum_partial != nullptr;
  const int act = g.act;
#define DIPACO_EPI(ACT, B, R, C, P) \
  gemm_epilogue_fixed<TC, TM, TN, WN, ACT, B, R, C, P>(acc, stg, lane, row0, col0, split, g)
  if constexpr (std::is_same<TC, float>::value) {
    // fp32 outputs (weight gradients) take no bias / activation / residual (checked on the host): a split-K plane or
    // C itself, nothing else, so the general function is not instantiated for them at all
    if (g.splits > 1) DIPACO_EPI(0, false, false, false, true);
    else DIPACO_EPI(0, false, false, false, false);
    return;
  }
  if constexpr (std::is_same<TC, bf16>::value) {
    if (act == 0 && !cs) {
      if (!bias && !resid) { DIPACO_EPI(0, false, false, false, false); return; }
      if (bias && !resid) { DIPACO_EPI(0, true, false, false, false); return; }
      if (bias && resid) { DIPACO_EPI(0, true, true, false, false); return; }
    }
    if (act == 3 && bias && !resid && !cs) { DIPACO_EPI(3, true, false, false, false); return; }
    if (act == 4 && !bias && !resid) {
      if (cs) { DIPACO_EPI(4, false, false, true, false); return; }
      DIPACO_EPI(4, false, false, false, false);
      return;
    }
  }
#undef DIPACO_EPI
  // the general function only where a wave owns four row blocks (the kernels' standard shapes); launches of other
  // shapes are restricted on the host to the combinations above (gemm_epilogue_is_fixed)
  if constexpr (std::is_same<TC, bf16>::value && TM == 4) gemm_epilogue<bf16, TC, TM, TN, WN>(acc, stg, lane, row0, col0, split, g);
}

// host: does a bf16-output product with these epilogue options take one of the compile-time epilogues above?
inline bool gemm_epilogue_is_fixed(int act, bool bias, bool resid, bool colsum) {
  if (act == 0 && !colsum) return (!bias && !resid) || bias;
  if (act == 3) return bias && !resid && !colsum;
  if (act == 4) return !bias && !resid;
  return false;
}

}  // namespace dipaco
