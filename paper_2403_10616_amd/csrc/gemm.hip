// Matrix-core GEMM for the path's linear layers: projections, MLP, vocabulary head, and their input / weight
// gradients.  bf16 or fp32 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32).
//
// One workgroup of 4 waves (2 x 2) computes a BM x BN tile of C; each wave owns (BM/64) x (BN/64) MFMA tiles of
// 32x32.  Both operands are staged in LDS K-contiguous (mma_tile.h), double-buffered.  Global loads run three K
// tiles ahead of the MFMAs: two tiles are in flight in registers (two register sets, used alternately) and one
// waits in the second LDS buffer, so a round trip to memory is covered by two full K steps of matrix work.
// The result goes back through LDS, 32 rows of the wave's tile at a time, so that bias / GELU / residual are
// applied on, and C is written with, 16-byte row-contiguous accesses.
// Workgroup ids are remapped so that each of the 8 XCDs (which receive consecutive ids round-robin and own a
// private L2) works on one contiguous range of tiles, walked in groups of 8 tile rows sharing the B panels.
#include <algorithm>
#include <type_traits>

#include "gemm_common.h"
#include "kernels.h"
#include "mma_tile.h"

namespace dipaco {

namespace {

// BM x BN tile, WGM x WGN waves, NS register sets of K tiles in flight
template <typename T, typename TC, bool TA, bool TB, int BM, int BN, int WGM, int WGN, int NS>
__global__ void __launch_bounds__(64 * WGM * WGN) gemm_kernel(const GemmDev g) {
  constexpr int BK = MmaTraits<T>::BK;
  constexpr int NT = 64 * WGM * WGN;
  constexpr int TM = BM / (32 * WGM), TN = BN / (32 * WGN);
  constexpr int STAGE = (BM + BN) * TILE_ROW_BYTES;
  constexpr int WN = BN / WGN;          // columns per wave
  constexpr int LDW = WN + 4;           // padded row of the epilogue staging buffer (floats)
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  int split, tile_m, tile_n;
  gemm_tile_of_block(g, blockIdx.x, split, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int k_begin = split * g.k_per_split;
  const int k_end = min(g.K, k_begin + g.k_per_split);
  const int nkt = (k_end - k_begin + BK - 1) / BK;

  const T* A = static_cast<const T*>(g.A);
  const T* B = static_cast<const T*>(g.B);
  using LA = TileLoader<T, BM, TA, NT>;
  using LB = TileLoader<T, BN, !TB, NT>;   // B as stored [K,N] is row(N)-contiguous: needs the transposing loader

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[NS][LA::NLD], rb[NS][LB::NLD];   // NS register sets of tiles in flight
  uint32_t offa[LA::NLD], offb[LB::NLD];
  LA::offsets(offa, g.lda, m0, g.M, tid);
  LB::offsets(offb, g.ldb, n0, g.N, tid);
  const long ka = LA::k_step(g.lda), kb = LB::k_step(g.ldb);
  const int nfull = (k_end - k_begin) / BK;   // K tiles completely inside the range; nkt - nfull is 0 or 1
  const int a_row0 = wm * (BM / WGM), b_row0 = wn * (BN / WGN);

  auto stage_a = [&](int st) { return smem + st * STAGE; };
  auto stage_b = [&](int st) { return smem + st * STAGE + BM * TILE_ROW_BYTES; };
  auto gload = [&](auto R, auto FULL, int kt) {
    constexpr int r = decltype(R)::value;
    const int k0 = k_begin + kt * BK;
    if (decltype(FULL)::value || k0 + BK <= k_end) {
      LA::load_full(ra[r], A + k0 * ka, offa);
      LB::load_full(rb[r], B + k0 * kb, offb);
    } else {
      LA::load_tail(ra[r], A, g.lda, m0, g.M, k0, k_end, tid);
      LB::load_tail(rb[r], B, g.ldb, n0, g.N, k0, k_end, tid);
    }
  };
  auto sstore = [&](auto R, auto BUF, auto FULL, int kt) {   // register set R -> LDS buffer BUF (= kt & 1)
    constexpr int r = decltype(R)::value, buf = decltype(BUF)::value;
    if (decltype(FULL)::value) {
      LA::store_full(ra[r], stage_a(buf), tid);
      LB::store_full(rb[r], stage_b(buf), tid);
    } else {
      const int k0 = k_begin + kt * BK;
      LA::store(ra[r], stage_a(buf), tid, k0, k_end);
      LB::store(rb[r], stage_b(buf), tid, k0, k_end);
    }
  };

  // Fragment double buffer.  At the top of a step, f*[0] holds K group 0 of the tile about to be multiplied.
  constexpr bool PIPE = WGM * WGN == 4;   // one wave per SIMD: software-pipeline the fragments
  uint4 fa[PIPE ? 2 : 1][TM], fb[PIPE ? 2 : 1][TN];
  using R0 = std::integral_constant<int, 0>;
  using R1 = std::integral_constant<int, 1>;
  using Full = std::true_type;
  using Any = std::false_type;
  // One K tile.  Tile t sits in LDS buffer t&1 (= r).  Tile t+1 waits in a register set; it goes to the other
  // LDS buffer and its register set is refilled with tile t+1+NS while K groups 0-1 of tile t are multiplied (so
  // NS tiles are in flight in registers).  After the first barrier the other buffer is complete, so group 0 of
  // tile t+1 is fetched under the MFMAs of group 3 and the matrix cores never wait for a tile's first fragments.
  // The second barrier keeps buffer r from being overwritten (next step) while a wave still reads it.
  auto step = [&](auto R, auto FULL, int t) {
    constexpr int r = decltype(R)::value;
    constexpr bool full = decltype(FULL)::value;
    using Set = std::integral_constant<int, NS == 2 ? 1 - r : 0>;   // register set of tile t+1
    using Buf = std::integral_constant<int, 1 - r>;
    const bool have_next = full || t + 1 < nkt;
    if (have_next) sstore(Set{}, Buf{}, FULL, t + 1);
    if (full || t + 1 + NS < nkt) gload(Set{}, FULL, t + 1 + NS);
    if constexpr (PIPE) {
      load_frags<TM, TN>(fa[1], fb[1], stage_a(r), stage_b(r), a_row0, b_row0, lane, 1);
      mma_group<T, TM, TN>(acc, fa[0], fb[0]);
      load_frags<TM, TN>(fa[0], fb[0], stage_a(r), stage_b(r), a_row0, b_row0, lane, 2);
      mma_group<T, TM, TN>(acc, fa[1], fb[1]);
      __syncthreads();
      load_frags<TM, TN>(fa[1], fb[1], stage_a(r), stage_b(r), a_row0, b_row0, lane, 3);
      mma_group<T, TM, TN>(acc, fa[0], fb[0]);
      if (have_next) load_frags<TM, TN>(fa[0], fb[0], stage_a(1 - r), stage_b(1 - r), a_row0, b_row0, lane, 0);
      mma_group<T, TM, TN>(acc, fa[1], fb[1]);
      __syncthreads();
    } else {
      // two waves per SIMD hide each other's LDS latency: one fragment set, one barrier per K tile
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        load_frags<TM, TN>(fa[0], fb[0], stage_a(r), stage_b(r), a_row0, b_row0, lane, ks);
        mma_group<T, TM, TN>(acc, fa[0], fb[0]);
      }
      __syncthreads();
    }
  };

  gload(R0{}, Any{}, 0);
  if (NS == 2 && nkt > 1) gload(R1{}, Any{}, 1);
  sstore(R0{}, R0{}, Any{}, 0);
  if (nkt > NS) gload(R0{}, Any{}, NS);
  __syncthreads();
  if constexpr (PIPE) load_frags<TM, TN>(fa[0], fb[0], stage_a(0), stage_b(0), a_row0, b_row0, lane, 0);
  int t = 0;
  for (; t + 2 + NS < nfull; t += 2) {   // steady state: every tile touched is complete, no conditions
    step(R0{}, Full{}, t);
    step(R1{}, Full{}, t + 1);
  }
  for (; t < nkt; t += 2) {              // drain (and short K): same steps with existence / tail checks
    step(R0{}, Any{}, t);
    if (t + 1 < nkt) step(R1{}, Any{}, t + 1);
  }

  gemm_epilogue<T, TC, TM, TN, WN>(acc, reinterpret_cast<float*>(smem) + wave * (32 * LDW), lane,
                                   m0 + wm * (BM / WGM), n0 + wn * WN, split, g);
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

}  // namespace

namespace {
// As splitk_reduce_kernel, for partial planes in which the number of K slices depends on where the element lies:
// n_slices[(row >= row_edge) + 2 * (col >= col_edge)]
__global__ void __launch_bounds__(128) splitk_reduce_classes_kernel(const float* __restrict__ partial,
                                                                    float* __restrict__ C, int M, int N, long ldc,
                                                                    int row_edge, int col_edge, int s0, int s1, int s2,
                                                                    int s3) {
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  const size_t total = (size_t)M * N, quads = total / 4;
  const size_t stride = (size_t)gridDim.x * 128;
  // one 16-byte vector per thread in the usual launch; a plane is read once (streaming loads), the first eight
  // slices are requested together and added in slice order
  for (size_t q = (size_t)blockIdx.x * 128 + threadIdx.x; q < quads; q += stride) {
    const size_t i = 4 * q;
    const size_t row = i / N, col = i - row * N;   // N is a multiple of 8: the four elements share a row
    const bool er = (int)row >= row_edge, ec = (int)col >= col_edge;
    const int n = er ? (ec ? s3 : s1) : (ec ? s2 : s0);
    f32x4_t v[8];
#pragma unroll
    for (int z = 0; z < 8; ++z)
      if (z < n) v[z] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(partial + (size_t)z * total + i));
    f32x4_t acc = v[0];
#pragma unroll
    for (int z = 1; z < 8; ++z)
      if (z < n) acc += v[z];
    for (int z = 8; z < n; ++z) acc += __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(partial + (size_t)z * total + i));
    *reinterpret_cast<f32x4_t*>(C + row * ldc + col) = acc;
  }
}
}  // namespace

dipaco_status launch_splitk_reduce_classes(const float* partial, float* C, int M, int N, long ldc, int row_edge,
                                           int col_edge, const int (&n_slices)[4], hipStream_t s) {
  if (N % 8 || ldc % 4 || col_edge % 4) return fail(DIPACO_ESHAPE, "split-K reduce: N, ldc, col_edge must be multiples of 8, 4, 4");
  const size_t quads = (size_t)M * N / 4;
  const unsigned rb = (unsigned)std::min<size_t>((quads + 127) / 128, 0x7fffffffu);
  splitk_reduce_classes_kernel<<<rb, 128, 0, s>>>(partial, C, M, N, ldc, row_edge, col_edge, n_slices[0], n_slices[1],
                                                  n_slices[2], n_slices[3]);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_splitk_reduce(const float* partial, float* C, int M, int N, long ldc, int splits, hipStream_t s) {
  const size_t total = (size_t)M * N;
  const int rb = (int)std::min<size_t>((total + 255) / 256, 256 * 32);
  splitk_reduce_kernel<<<rb, 256, 0, s>>>(partial, C, M, N, ldc, splits);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

namespace {

template <typename T, typename TC, bool TA, bool TB, int BM, int BN, int WGM, int WGN, int NS>
dipaco_status run(const GemmArgs& a, hipStream_t s) {
  constexpr int BK = MmaTraits<T>::BK;
  constexpr size_t smem_loop = 2 * (size_t)(BM + BN) * TILE_ROW_BYTES;
  constexpr size_t smem_epi = (size_t)WGM * WGN * 32 * (size_t)(BN / WGN + 4) * sizeof(float);
  constexpr size_t smem = smem_loop > smem_epi ? smem_loop : smem_epi;
  auto kern = gemm_kernel<T, TC, TA, TB, BM, BN, WGM, WGN, NS>;
  static std::atomic<unsigned long long> lds_set{0};   // per instantiation
  if (dipaco_status e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_set)) return e;
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
  g.colsum_partial = a.colsum ? a.colsum_partial : nullptr;
  kern<<<(unsigned)blocks, 64 * WGM * WGN, smem, s>>>(g);
  DIPACO_LAUNCH_CHECK();
  if (g.splits > 1) return launch_splitk_reduce(a.partial, static_cast<float*>(a.C), a.M, a.N, a.ldc, g.splits, s);
  constexpr int WAVE_ROWS = BM / WGM;
  if (a.colsum) return launch_sum_rows(a.colsum_partial, a.colsum, (a.M + WAVE_ROWS - 1) / WAVE_ROWS, a.N, s, a.sum_batch);
  return DIPACO_OK;
}

std::atomic<int> g_forced_tile{0};   // test / tuning hook (dipaco_k_set_gemm_tile), not a per-call setting

// Measured on the training step's shapes: the eight-wave 256 x 256 tile is the fastest wherever its workgroups
// can fill most of the chip's 256 compute units; below that the 128 x 128 tile (two workgroups per unit) wins.
int pick_tile(int M, int N, int K, int splits) {
  if (g_forced_tile && g_forced_tile != 5) return g_forced_tile;
  const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256) * (splits < 1 ? 1 : splits);
  return (K >= 256 && t256 >= 160) ? 4 : 1;
}

template <typename T, typename TC, bool TA, bool TB>
dipaco_status run_tiled(const GemmArgs& a, hipStream_t s) {
  switch (pick_tile(a.M, a.N, a.K, a.splits)) {
    case 4: return run<T, TC, TA, TB, 256, 256, 2, 4, 1>(a, s);
    case 3: return run<T, TC, TA, TB, 256, 256, 2, 2, 1>(a, s);
    case 2: return run<T, TC, TA, TB, 256, 128, 2, 2, 2>(a, s);
    default: return run<T, TC, TA, TB, 128, 128, 2, 2, 2>(a, s);
  }
}

}  // namespace

void set_gemm_tile(int t) {
  g_forced_tile = t > 5 ? 5 : t;
  set_gemm_dlds_shape(t > 5 ? t - 5 : 0);
}

// Split count for a long-K product (a weight gradient: K = tokens).  With 256 x 256 tiles the cost of one
// candidate, in units of one K step of one tile, is rounds * (K / s + fixed) + s * (traffic of one partial
// plane), where rounds = workgroups / 256 rounded up; the constants are fitted to measured launches.
static int splits_tile256(int M, int N, int K, int smax) {
  const long t256 = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (t256 * smax < 160) return 0;   // cannot fill the chip: not a 256 x 256 case
  const double plane = (double)M * N * 6e-5;
  double best = 0;
  int best_s = 1;
  for (int s = 1; s <= smax; ++s) {
    const long rounds = (t256 * s + 255) / 256;
    const double cost = rounds * ((double)K / s + 600.0) + (s > 1 ? s * plane : 0.0);
    if (s == 1 || cost < best) { best = cost; best_s = s; }
  }
  return best_s;
}

static int splits_tile128(int M, int N, int smax) {
  const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  const long s = std::min<long>((512 + t128 - 1) / t128, smax);
  return (int)std::max<long>(s, 1);
}

size_t gemm_colsum_partial_floats(int M, int N) { return (size_t)((M + 31) / 32) * N; }

// Most slices a long-K product is cut into by the register-staged kernels: a slice keeps at least 256 of K, and a
// small output under a very long contraction (the router's 256 x 768 gradient over 2^20 documents) may still put a
// workgroup on every compute unit.  The cost model below decides how many are actually taken.
constexpr int GEMM_SLICE_CAP_STAGED = 128;

int gemm_plan_splits(int M, int N, int K, bool bf16_operands) {
  const int smax = (int)std::min<long>(GEMM_SLICE_CAP_STAGED, std::max(1, K / 256));
  if (bf16_operands && (g_forced_tile == 0 || g_forced_tile >= 5)) {
    // direct-to-LDS kernel, one workgroup per compute unit, fewer slices for tiles that stick out of C
    const int s = gemm_dlds_plan_slices(M, N, K, (int)std::min<long>(GEMM_SLICE_CAP, std::max(1, K / 256)), false);
    if (s) return s;
  }
  if (g_forced_tile == 0 || g_forced_tile >= 4) {
    const int s = splits_tile256(M, N, K, smax);
    if (s) return s;
  }
  return splits_tile128(M, N, smax);
}

// Upper bound of gemm_plan_splits over every tile setting: sizes the partial-product workspace.
int gemm_max_splits(int M, int N, int K) {
  const int smax = (int)std::min<long>(GEMM_SLICE_CAP_STAGED, std::max(1, K / 256));
  const int cap = (int)std::min<long>(GEMM_SLICE_CAP, std::max(1, K / 256));
  return std::max(std::max(splits_tile256(M, N, K, smax), splits_tile128(M, N, smax)),
                  gemm_dlds_plan_slices(M, N, K, cap, true));
}

template <typename T> dipaco_status launch_gemm(const GemmArgs& a, hipStream_t s) {
  constexpr int VEC = MmaTraits<T>::VEC;
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(DIPACO_ESHAPE, "gemm: empty operand");
  // 16-byte vectors run along the contiguous index of each operand and along the rows of C
  if ((a.trans_a ? a.M : a.K) % VEC || (a.trans_b ? a.K : a.N) % VEC || a.lda % VEC || a.ldb % VEC)
    return fail(DIPACO_ESHAPE, "gemm: contiguous extents and leading dimensions must be multiples of 16 bytes");
  if (a.ldc % 8 || a.N % 8) return fail(DIPACO_ESHAPE, "gemm: N and ldc must be multiples of 8");
  // per-thread element offsets are 32-bit
  const long ext_a = (a.trans_a ? 64 : (long)a.M) * a.lda + a.M, ext_b = (a.trans_b ? (long)a.N : 64) * a.ldb + a.N;
  if (ext_a >= (1L << 32) || ext_b >= (1L << 32)) return fail(DIPACO_ESHAPE, "gemm: operand above 2^32 elements");
  if (!aligned16(a.A) || !aligned16(a.B) || !aligned16(a.C) || !aligned16(a.bias) || !aligned16(a.resid) ||
      !aligned16(a.aux_in) || !aligned16(a.aux_out) || !aligned16(a.partial))
    return fail(DIPACO_EALIGN, "gemm: operand not 16-byte aligned");
  if (a.act < 0 || a.act > 4) return fail(DIPACO_EINVAL, "gemm: act must be 0..4");
  if ((a.act == 1 || a.act == 3) && !a.aux_out) return fail(DIPACO_EINVAL, "gemm: act 1 / 3 need aux_out");
  if ((a.act == 2 || a.act == 4) && !a.aux_in) return fail(DIPACO_EINVAL, "gemm: act 2 / 4 need aux_in");
  if (a.out_f32 && (a.bias || a.resid || a.act)) return fail(DIPACO_EINVAL, "gemm: fp32 output takes no epilogue");
  if (a.colsum && (!a.colsum_partial || a.splits > 1 || a.out_f32 || !aligned16(a.colsum_partial)))
    return fail(DIPACO_EINVAL, "gemm: column sums need their scratch, no split-K and an output of the operands' type");
  if (a.splits > 1 && (!a.out_f32 || a.bias || a.resid || a.act || !a.partial))
    return fail(DIPACO_EINVAL, "gemm: split-K needs fp32 output, a partial buffer and no epilogue");
  if constexpr (std::is_same<T, bf16>::value) {
    // bf16 products that fill the chip with 256 x 256 tiles go to the direct-to-LDS kernel when their shape allows
    const bool big = pick_tile(a.M, a.N, a.K, a.splits) == 4;
    if ((g_forced_tile == 5 || (g_forced_tile == 0 && big)) && gemm_dlds_eligible(a)) return launch_gemm_dlds(a, s);
  }
  if (a.out_f32) {
    if (a.trans_a && !a.trans_b) return run_tiled<T, float, true, false>(a, s);
    return fail(DIPACO_EUNSUPPORTED, "gemm: fp32 output only for A^T.B");
  }
  if (!a.trans_a && !a.trans_b) return run_tiled<T, T, false, false>(a, s);
  if (!a.trans_a && a.trans_b) return run_tiled<T, T, false, true>(a, s);
  return fail(DIPACO_EUNSUPPORTED, "gemm: operand layout not instantiated");
}

template dipaco_status launch_gemm<float>(const GemmArgs&, hipStream_t);
template dipaco_status launch_gemm<bf16>(const GemmArgs&, hipStream_t);

}  // namespace dipaco
