// Matrix-core GEMM for the path's linear layers: projections, MLP, vocabulary head, and their input / weight
// gradients.  bf16 or fp32 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32).
//
// One workgroup of 4 waves (2 x 2) computes a BM x BN tile of C; each wave owns (BM/64) x (BN/64) MFMA tiles of
// 32x32.  Both operands are staged in LDS K-contiguous (mma_tile.h); the next K tile is fetched into registers
// while the current one is multiplied, LDS is double-buffered, one barrier per K tile.
#include <algorithm>

#include "kernels.h"
#include "mma_tile.h"

namespace dipaco {

namespace {

struct GemmDev {
  const void* A; const void* B; void* C;
  int M, N, K;
  long lda, ldb, ldc;
  const void* bias; const void* resid; void* aux_out; const void* aux_in;
  int act;
  int splits;
  int k_per_split;   // multiple of BK
  float* partial;
  int tiles_m, tiles_n;
};

template <typename T, typename TC, bool TA, bool TB, int BM, int BN>
__global__ void __launch_bounds__(GEMM_THREADS) gemm_kernel(const GemmDev g) {
  constexpr int BK = MmaTraits<T>::BK;
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int STAGE = (BM + BN) * TILE_ROW_BYTES;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  int bid = blockIdx.x;
  const int tiles = g.tiles_m * g.tiles_n;
  const int split = bid / tiles;
  bid -= split * tiles;
  // tile order: N fastest inside groups of 8 M-tiles, so that concurrently running workgroups share operand panels
  const int group = 8;
  const int per_group = group * g.tiles_n;
  const int gidx = bid / per_group;
  const int first_m = gidx * group;
  const int gsize = min(group, g.tiles_m - first_m);
  const int in_group = bid - gidx * per_group;
  const int tile_m = first_m + in_group % gsize;
  const int tile_n = in_group / gsize;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int k_begin = split * g.k_per_split;
  const int k_end = min(g.K, k_begin + g.k_per_split);
  const int nkt = (k_end - k_begin + BK - 1) / BK;

  const T* A = static_cast<const T*>(g.A);
  const T* B = static_cast<const T*>(g.B);
  using LA = TileLoader<T, BM, TA>;
  using LB = TileLoader<T, BN, !TB>;   // B as stored [K,N] is row(N)-contiguous: needs the transposing loader

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[LA::NLD], rb[LB::NLD];
  if (nkt > 0) {
    LA::load(ra, A, g.lda, m0, g.M, k_begin, k_end, tid);
    LB::load(rb, B, g.ldb, n0, g.N, k_begin, k_end, tid);
    LA::store(ra, smem, tid);
    LB::store(rb, smem + BM * TILE_ROW_BYTES, tid);
  }
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    char* cur = smem + (kt & 1) * STAGE;
    char* nxt = smem + ((kt + 1) & 1) * STAGE;
    const bool more = kt + 1 < nkt;
    if (more) {
      const int k0 = k_begin + (kt + 1) * BK;
      LA::load(ra, A, g.lda, m0, g.M, k0, k_end, tid);
      LB::load(rb, B, g.ldb, n0, g.N, k0, k_end, tid);
    }
    mma_ktile<T, TM, TN>(acc, cur, cur + BM * TILE_ROW_BYTES, wm * (BM / 2), wn * (BN / 2), lane);
    if (more) {
      LA::store(ra, nxt, tid);
      LB::store(rb, nxt + BM * TILE_ROW_BYTES, tid);
    }
    __syncthreads();
  }

  // ---- epilogue ----
  const int col_l = lane & 31;
  if (g.splits > 1) {
    float* P = g.partial + (size_t)split * g.M * g.N;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * (BN / 2) + 32 * j + col_l;
        if (col >= g.N) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + wm * (BM / 2) + 32 * i + acc_row(e, lane);
          if (row < g.M) P[(size_t)row * g.N + col] = acc[i][j][e];
        }
      }
    return;
  }
  const T* bias = static_cast<const T*>(g.bias);
  const T* resid = static_cast<const T*>(g.resid);
  const T* aux_in = static_cast<const T*>(g.aux_in);
  T* aux_out = static_cast<T*>(g.aux_out);
  TC* C = static_cast<TC*>(g.C);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * (BN / 2) + 32 * j + col_l;
      if (col >= g.N) continue;
      const float bv = bias ? to_f32(bias[col]) : 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm * (BM / 2) + 32 * i + acc_row(e, lane);
        if (row >= g.M) continue;
        const size_t off = (size_t)row * g.ldc + col;
        float v = acc[i][j][e] + bv;
        if (g.act == 1) {
          // the saved pre-activation is what backward differentiates at: apply GELU to the stored value
          T pre = from_f32<T>(v);
          aux_out[off] = pre;
          v = gelu_f(to_f32(pre));
        } else if (g.act == 2) {
          v *= gelu_grad_f(to_f32(aux_in[off]));
        }
        if (resid) v += to_f32(resid[off]);
        C[off] = from_f32<TC>(v);
      }
    }
}

__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float* __restrict__ partial, float* __restrict__ C,
                                                            int M, int N, long ldc, int splits) {
  const size_t total = (size_t)M * N;
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
    float s = partial[i];
    for (int z = 1; z < splits; ++z) s += partial[(size_t)z * total + i];
    const size_t row = i / N, col = i - row * N;
    C[row * ldc + col] = s;
  }
}

template <typename T, typename TC, bool TA, bool TB, int BM, int BN>
dipaco_status run(const GemmArgs& a, hipStream_t s) {
  constexpr int BK = MmaTraits<T>::BK;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * TILE_ROW_BYTES;
  auto kern = gemm_kernel<T, TC, TA, TB, BM, BN>;
  static bool attr_set = false;   // one attribute call per instantiation and process
  if (!attr_set) {
    DIPACO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)smem));
    attr_set = true;
  }
  GemmDev g;
  g.A = a.A; g.B = a.B; g.C = a.C; g.M = a.M; g.N = a.N; g.K = a.K;
  g.lda = a.lda; g.ldb = a.ldb; g.ldc = a.ldc;
  g.bias = a.bias; g.resid = a.resid; g.aux_out = a.aux_out; g.aux_in = a.aux_in; g.act = a.act;
  g.splits = a.splits < 1 ? 1 : a.splits;
  g.partial = a.partial;
  g.tiles_m = (a.M + BM - 1) / BM;
  g.tiles_n = (a.N + BN - 1) / BN;
  const int ktiles = (a.K + BK - 1) / BK;
  if (g.splits > ktiles) g.splits = ktiles > 0 ? ktiles : 1;
  g.k_per_split = ((ktiles + g.splits - 1) / g.splits) * BK;
  g.splits = (a.K + g.k_per_split - 1) / g.k_per_split;
  if (g.splits < 1) g.splits = 1;
  const long blocks = (long)g.tiles_m * g.tiles_n * g.splits;
  if (blocks > 0x7fffffffL) return fail(DIPACO_ESHAPE, "gemm: too many tiles");
  kern<<<(unsigned)blocks, GEMM_THREADS, smem, s>>>(g);
  DIPACO_LAUNCH_CHECK();
  if (g.splits > 1) {
    size_t total = (size_t)a.M * a.N;
    int rb = (int)std::min<size_t>((total + 255) / 256, 256 * 32);
    splitk_reduce_kernel<<<rb, 256, 0, s>>>(a.partial, static_cast<float*>(a.C), a.M, a.N, a.ldc, g.splits);
    DIPACO_LAUNCH_CHECK();
  }
  return DIPACO_OK;
}

}  // namespace

template <typename T> dipaco_status launch_gemm(const GemmArgs& a, hipStream_t s) {
  constexpr int VEC = MmaTraits<T>::VEC;
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(DIPACO_ESHAPE, "gemm: empty operand");
  // 16-byte vectors run along the contiguous index of each operand
  if ((a.trans_a ? a.M : a.K) % VEC || (a.trans_b ? a.K : a.N) % VEC || a.lda % VEC || a.ldb % VEC)
    return fail(DIPACO_ESHAPE, "gemm: contiguous extents and leading dimensions must be multiples of 16 bytes");
  if (!aligned16(a.A) || !aligned16(a.B)) return fail(DIPACO_EALIGN, "gemm: operand not 16-byte aligned");
  if (a.splits > 1 && (!a.out_f32 || a.bias || a.resid || a.act || !a.partial))
    return fail(DIPACO_EINVAL, "gemm: split-K needs fp32 output, a partial buffer and no epilogue");
  if (a.out_f32) {
    if (a.trans_a && !a.trans_b) return run<T, float, true, false, 128, 128>(a, s);
    return fail(DIPACO_EUNSUPPORTED, "gemm: fp32 output only for A^T.B");
  }
  if (!a.trans_a && !a.trans_b) return run<T, T, false, false, 128, 128>(a, s);
  if (!a.trans_a && a.trans_b) return run<T, T, false, true, 128, 128>(a, s);
  return fail(DIPACO_EUNSUPPORTED, "gemm: operand layout not instantiated");
}

template dipaco_status launch_gemm<float>(const GemmArgs&, hipStream_t);
template dipaco_status launch_gemm<bf16>(const GemmArgs&, hipStream_t);

}  // namespace dipaco
