// k-means prefix routing: idx[n] = argmin_k ||z_n - c_k||^2, per-centroid histogram, and the gap between the
// two best scores.  The argmin is taken over s(n,k) = ||c_k||^2 - 2 z_n.c_k (||z_n||^2 is common to all k), so
// the work is one fp32 contraction z.C^T on the matrix cores (v_mfma_f32_32x32x2_f32) with the reduction over
// centroids done in the epilogue: scores never reach memory.
//
// One workgroup (8 waves, 2 x 4: two per SIMD, so that one wave's staging, barriers and reductions run under the
// other's matrix instructions) owns 256 points and walks the centroids in tiles of 256; every wave holds a 128 x 64
// block of scores in accumulators.  ||c_k||^2 is accumulated by the threads that stage the centroid
// tile, from the very values they put into LDS.
#include <type_traits>

#include "kernels.h"
#include "mma_tile.h"

namespace dipaco {

namespace {

constexpr int RBM = 256;   // points per workgroup
constexpr int RBN = 256;   // centroids per tile
constexpr int RBK = 32;    // fp32 K tile
constexpr int R_THREADS = 512;
constexpr int R_WN = 4;    // waves along the centroids, 64 columns each
constexpr int R_STAGE = (RBM + RBN) * TILE_ROW_BYTES;
constexpr int R_MAX_K_LDS_HIST = 4096;
constexpr int R_TM = RBM / 64;   // 32-row score tiles per wave (two waves along the points)

// Best and second-best (score, index) of a row, ordered lexicographically: exact ties go to the lower index.
// TOP2 = false: the second index is not tracked (only its score, for the margin).
struct Best {
  float s1; int i1; float s2; int i2;
};
constexpr int NO_INDEX = 0x7fffffff;

// (s, i) before (t, j) in the lexicographic order
__device__ __forceinline__ bool lex_less(float s, int i, float t, int j) { return s < t || (s == t && i < j); }

// Candidate (s, k) whose index k is larger than every index the entry has seen: a tie keeps the earlier entry, so
// plain < decides.  Written as selects: no branch, a NaN score never enters.
template <bool TOP2> __device__ __forceinline__ void best_push_ascending(Best& b, float s, int k) {
  const bool lt1 = s < b.s1, lt2 = s < b.s2;
  if (TOP2) b.i2 = lt1 ? b.i1 : (lt2 ? k : b.i2);
  b.s2 = lt1 ? b.s1 : (lt2 ? s : b.s2);
  b.i1 = lt1 ? k : b.i1;
  b.s1 = lt1 ? s : b.s1;
}
// The two best of the union of two entries over disjoint index sets.  A selection, not arithmetic: the result does
// not depend on the order in which entries are merged.
template <bool TOP2> __device__ __forceinline__ Best best_merge(const Best& a, const Best& b) {
  const bool lt = lex_less(b.s1, b.i1, a.s1, a.i1);
  Best o;
  o.s1 = lt ? b.s1 : a.s1;
  o.i1 = lt ? b.i1 : a.i1;
  const float xs = lt ? a.s1 : b.s1, ys = lt ? b.s2 : a.s2;   // the first that lost, the second of the one that won
  if (TOP2) {
    const int xi = lt ? a.i1 : b.i1, yi = lt ? b.i2 : a.i2;
    const bool ly = lex_less(ys, yi, xs, xi);
    o.s2 = ly ? ys : xs;
    o.i2 = ly ? yi : xi;
  } else {
    o.s2 = ys < xs ? ys : xs;
    o.i2 = NO_INDEX;
  }
  return o;
}

// The value of lane l ^ MASK (MASK < 32): quad permutes on the vector ALU for 1 and 2, the LDS crossbar (no LDS
// memory) for 4, 8, 16.
template <int MASK> __device__ __forceinline__ int lane_xor(int v) {
  if constexpr (MASK == 1) return __builtin_amdgcn_update_dpp(v, v, 0xb1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
  else if constexpr (MASK == 2) return __builtin_amdgcn_update_dpp(v, v, 0x4e, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  else return __builtin_amdgcn_ds_swizzle(v, (MASK << 10) | 0x1f);   // bit mode: and 0x1f, or 0, xor MASK
}
template <int MASK> __device__ __forceinline__ float lane_xor(float v) {
  return __builtin_bit_cast(float, lane_xor<MASK>(__builtin_bit_cast(int, v)));
}

// Reduction over the 32 lanes that share rows: the entries of 2^LEVEL rows (BASE .. BASE + 2^LEVEL - 1 of the lane's
// 32), reduced over lane bits 0 .. LEVEL-1, as ONE entry per lane.  Two halves are reduced first; then the lane whose
// bit LEVEL-1 is clear keeps the entry of the lower half and hands the other to its partner lane ^ 2^(LEVEL-1), the
// partner the other way round, and each merges what it keeps with what it receives.  At LEVEL 5 every lane holds one
// row (number l & 31) reduced over all 32 lanes: 31 merges per lane instead of the 160 of a butterfly on every row,
// and, walked depth-first, never more than LEVEL + 1 entries alive (leaf(r) builds row r's entry when it is needed).
template <bool TOP2, int LEVEL, int BASE, typename Leaf>
__device__ __forceinline__ Best best_reduce_rows(const Leaf& leaf, int lane) {
  if constexpr (LEVEL == 0) {
    return leaf(std::integral_constant<int, BASE>{});
  } else {
    constexpr int MASK = 1 << (LEVEL - 1);
    const Best lo = best_reduce_rows<TOP2, LEVEL - 1, BASE>(leaf, lane);
    const Best hi = best_reduce_rows<TOP2, LEVEL - 1, BASE + MASK>(leaf, lane);
    const bool up = (lane & MASK) != 0;
    Best mine, theirs, got;
    mine.s1 = up ? hi.s1 : lo.s1; mine.i1 = up ? hi.i1 : lo.i1; mine.s2 = up ? hi.s2 : lo.s2;
    theirs.s1 = up ? lo.s1 : hi.s1; theirs.i1 = up ? lo.i1 : hi.i1; theirs.s2 = up ? lo.s2 : hi.s2;
    mine.i2 = TOP2 ? (up ? hi.i2 : lo.i2) : NO_INDEX;
    theirs.i2 = TOP2 ? (up ? lo.i2 : hi.i2) : NO_INDEX;
    got.s1 = lane_xor<MASK>(theirs.s1); got.i1 = lane_xor<MASK>(theirs.i1); got.s2 = lane_xor<MASK>(theirs.s2);
    got.i2 = TOP2 ? lane_xor<MASK>(theirs.i2) : NO_INDEX;
    return best_merge<TOP2>(mine, got);
  }
}

// z: row n at z + n * ldz.  TOP2: idx is [N, 2] (second entry -1 when K = 1) and hist counts both memberships.
template <bool TOP2>
__global__ void __launch_bounds__(R_THREADS) route_kernel(const float* __restrict__ z, long ldz,
                                                             const float* __restrict__ c,
                                                             const float* __restrict__ lin_bias, long N, int D, int K,
                                                             int* __restrict__ idx,
                                                             unsigned long long* __restrict__ hist,
                                                             float* __restrict__ margin) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ float cnorm[RBN];
  __shared__ unsigned int lhist[R_MAX_K_LDS_HIST];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / R_WN, wn = wave % R_WN;
  const long m0 = (long)blockIdx.x * RBM;
  const int rows_left = (int)min((long)RBM, N - m0);
  const float* zb = z + m0 * ldz;
  const bool use_lhist = K <= R_MAX_K_LDS_HIST;
  const float dot_mul = lin_bias ? 1.0f : 2.0f;
  if (use_lhist) for (int k = tid; k < K; k += R_THREADS) lhist[k] = 0;

  using LZ = TileLoader<float, RBM, false, R_THREADS>;
  using LC = TileLoader<float, RBN, false, R_THREADS>;
  const int nkt = (D + RBK - 1) / RBK;

  // Running best / second best of one row per lane and pair of row tiles: after the reduction at the end of a
  // centroid tile lane l holds, of pair hb, row tile 2 hb + ((l & 31) >> 4), accumulator element e = l & 15.
  Best run[R_TM / 2];
#pragma unroll
  for (int hb = 0; hb < R_TM / 2; ++hb) { run[hb].s1 = INFINITY; run[hb].i1 = NO_INDEX; run[hb].s2 = INFINITY; run[hb].i2 = NO_INDEX; }

  for (int n0 = 0; n0 < K; n0 += RBN) {
    f32x16 acc[R_TM][2];
#pragma unroll
    for (int i = 0; i < R_TM; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    float nrm[LC::NLD];
#pragma unroll
    for (int i = 0; i < LC::NLD; ++i) nrm[i] = 0.f;

    uint4 rz[LZ::NLD], rc[LC::NLD];
    const float* cb = c + (long)n0 * D;
    const int crow_left = min(RBN, K - n0);
    LZ::load_tail(rz, zb, ldz, 0, rows_left, 0, D, tid);
    LC::load_tail(rc, cb, D, 0, crow_left, 0, D, tid);
    __syncthreads();   // previous centroid tile's readers of LDS and of cnorm are done
    LZ::store(rz, smem, tid, 0, D);
    LC::store(rc, smem + RBM * TILE_ROW_BYTES, tid, 0, D);
    const bool keep0 = (tid & 7) * 4 < D;
#pragma unroll
    for (int i = 0; i < LC::NLD; ++i) {
      float4 v = *reinterpret_cast<float4*>(&rc[i]);
      if (keep0) nrm[i] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
      char* cur = smem + (kt & 1) * R_STAGE;
      char* nxt = smem + ((kt + 1) & 1) * R_STAGE;
      const bool more = kt + 1 < nkt;
      if (more) {
        LZ::load_tail(rz, zb, ldz, 0, rows_left, (kt + 1) * RBK, D, tid);
        LC::load_tail(rc, cb, D, 0, crow_left, (kt + 1) * RBK, D, tid);
      }
      mma_ktile<float, R_TM, 2>(acc, cur, cur + RBM * TILE_ROW_BYTES, wm * (RBM / 2), wn * 64, lane);
      if (more) {
        const int k0n = (kt + 1) * RBK;
        LZ::store(rz, nxt, tid, k0n, D);
        LC::store(rc, nxt + RBM * TILE_ROW_BYTES, tid, k0n, D);
        const bool keep = k0n + (tid & 7) * 4 < D;
#pragma unroll
        for (int i = 0; i < LC::NLD; ++i) {
          float4 v = *reinterpret_cast<float4*>(&rc[i]);
          if (keep) nrm[i] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
      }
      __syncthreads();
    }
    // ||c||^2: thread tid staged chunk (tid & 7) of centroid rows (tid >> 3) + 64 i
#pragma unroll
    for (int i = 0; i < LC::NLD; ++i) {
      float v = nrm[i];
      v += __shfl_xor(v, 1, WAVE);
      v += __shfl_xor(v, 2, WAVE);
      v += __shfl_xor(v, 4, WAVE);
      if ((tid & 7) == 0) {
        const int col = (tid >> 3) + (R_THREADS / 8) * i;
        // linear router: the score to minimise is -(w_k.z + b_k), so -b_k takes the place of ||c_k||^2
        // a column beyond K scores +inf: it never enters a best entry
        cnorm[col] = n0 + col < K ? (lin_bias ? -lin_bias[n0 + col] : v) : INFINITY;
      }
    }
    __syncthreads();
    // this centroid tile: for each pair of row tiles (32 rows of the lane) the best entries over the lane's 2 columns
    // (ascending index), reduced over the 32 lanes of the half (they hold the other columns of the same rows) to one
    // row per lane, and folded into the running entry of that row
    float cn[2];
    int kk[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = wn * 64 + 32 * j + (lane & 31);
      kk[j] = n0 + col;
      cn[j] = cnorm[col];
    }
#pragma unroll
    for (int hb = 0; hb < R_TM / 2; ++hb) {
      auto leaf = [&](auto R) {
        constexpr int r = decltype(R)::value;
        Best b;
        b.s1 = INFINITY; b.i1 = NO_INDEX; b.s2 = INFINITY; b.i2 = NO_INDEX;
#pragma unroll
        for (int j = 0; j < 2; ++j)
          best_push_ascending<TOP2>(b, __builtin_fmaf(-dot_mul, acc[2 * hb + r / 16][j][r % 16], cn[j]), kk[j]);
        return b;
      };
      run[hb] = best_merge<TOP2>(run[hb], best_reduce_rows<TOP2, 5, 0>(leaf, lane));
    }
  }

  // Row of a lane's entry: step t of the reduction kept the entries whose bit t equals lane bit t, so the entry left
  // is number l & 31 = 16 i + e of its pair.  Then the four waves along N are merged through LDS (the operand stages
  // are free: every wave has passed the barriers that end the last centroid tile).
  float* const red_s1 = reinterpret_cast<float*>(smem);
  float* const red_s2 = red_s1 + R_WN * RBM;
  int* const red_i1 = reinterpret_cast<int*>(red_s2 + R_WN * RBM);
  int* const red_i2 = red_i1 + R_WN * RBM;
  static_assert(4 * R_WN * RBM * sizeof(float) <= 2 * (size_t)R_STAGE, "the merge arrays fit in the operand stages");
#pragma unroll
  for (int hb = 0; hb < R_TM / 2; ++hb) {
    const int r = lane & 31;
    const int row = wm * (RBM / 2) + 64 * hb + 32 * (r >> 4) + acc_row(r & 15, lane);
    red_s1[wn * RBM + row] = run[hb].s1; red_i1[wn * RBM + row] = run[hb].i1; red_s2[wn * RBM + row] = run[hb].s2;
    if (TOP2) red_i2[wn * RBM + row] = run[hb].i2;
  }
  __syncthreads();
  if (tid < RBM && tid < rows_left) {
    Best b;
    b.s1 = red_s1[tid]; b.i1 = red_i1[tid]; b.s2 = red_s2[tid]; b.i2 = TOP2 ? red_i2[tid] : NO_INDEX;
#pragma unroll
    for (int w = 1; w < R_WN; ++w) {
      Best o;
      o.s1 = red_s1[w * RBM + tid]; o.i1 = red_i1[w * RBM + tid]; o.s2 = red_s2[w * RBM + tid];
      o.i2 = TOP2 ? red_i2[w * RBM + tid] : NO_INDEX;
      b = best_merge<TOP2>(b, o);
    }
    // A row none of whose scores compares below +inf (NaN or infinite features: a diverged path) never entered an
    // entry.  It is given the first centroid (the first two with TOP2) and a NaN margin, which is what the plain
    // definition's argmin over a row of NaN distances yields; it must not reach the histogram with an unset index.
    if (b.i1 == NO_INDEX) {
      b.i1 = 0;
      b.i2 = K > 1 ? 1 : NO_INDEX;
      b.s1 = b.s2 = __builtin_nanf("");
    }
    if (TOP2) {
      const bool has2 = b.i2 != NO_INDEX;
      idx[2 * (m0 + tid)] = b.i1;
      idx[2 * (m0 + tid) + 1] = has2 ? b.i2 : -1;
      if (has2) {
        if (use_lhist) atomicAdd(&lhist[b.i2], 1u);
        else atomicAdd(&hist[b.i2], 1ull);
      }
    } else {
      idx[m0 + tid] = b.i1;
    }
    if (margin) margin[m0 + tid] = b.s2 - b.s1;
    if (use_lhist) atomicAdd(&lhist[b.i1], 1u);
    else atomicAdd(&hist[b.i1], 1ull);
  }
  if (use_lhist) {
    __syncthreads();
    for (int k = tid; k < K; k += R_THREADS) {
      unsigned int v = lhist[k];
      if (v) atomicAdd(&hist[k], (unsigned long long)v);
    }
  }
}

// ---- K-class logistic regression: per-row softmax cross-entropy --------------------------------------------------
// One wave per row of logits [rows, K] (K a multiple of 4, at most LOGIT_MAX_K): nll[row] = logsumexp - logit[label],
// and in place logits <- (softmax - onehot(label)) * inv_n.  A row whose label is outside [0, K) gives 0 and zeros.
constexpr int LOGIT_MAX_VEC = 16;                 // float4 per lane
constexpr int LOGIT_MAX_K = 64 * 4 * LOGIT_MAX_VEC;
__global__ void __launch_bounds__(256) logistic_rows_kernel(float* __restrict__ logits, const int* __restrict__ labels,
                                                            long rows, int K, float inv_n, float* __restrict__ nll) {
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const int nvec = K >> 2;
  float4* lr = reinterpret_cast<float4*>(logits + row * K);
  float4 v[LOGIT_MAX_VEC];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < LOGIT_MAX_VEC; ++i) {
    const int c = lane + 64 * i;
    if (c < nvec) {
      v[i] = lr[c];
      mx = fmaxf(mx, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
    }
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  const int label = labels[row];
  const bool valid = label >= 0 && label < K;
  float sum = 0.f, at_label = 0.f;   // at_label: logit[label] - max, held by one lane
#pragma unroll
  for (int i = 0; i < LOGIT_MAX_VEC; ++i) {
    const int c = lane + 64 * i;
    if (c < nvec) {
      float x[4] = {v[i].x - mx, v[i].y - mx, v[i].z - mx, v[i].w - mx};
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (valid && 4 * c + q == label) at_label = x[q];
      v[i].x = expf(x[0]); v[i].y = expf(x[1]); v[i].z = expf(x[2]); v[i].w = expf(x[3]);
      sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) sum += __shfl_xor(sum, o, 64);
  const float scale = valid ? inv_n / sum : 0.f;
#pragma unroll
  for (int i = 0; i < LOGIT_MAX_VEC; ++i) {
    const int c = lane + 64 * i;
    if (c < nvec) {
      float e[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
      float o[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q] = e[q] * scale - ((valid && 4 * c + q == label) ? inv_n : 0.f);
      lr[c] = make_float4(o[0], o[1], o[2], o[3]);
    }
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) at_label += __shfl_xor(at_label, o, 64);
  if (lane == 0) nll[row] = valid ? logf(sum) - at_label : 0.f;
}

// The same for K <= 256, where a row is at most one 16-byte vector per lane: a wave takes ROWS rows at once, so that
// ROWS loads are in flight per lane instead of one (a million one-kilobyte rows are latency-bound otherwise), and the
// reductions run on the DPP lanes.
constexpr int LOGIT_SMALL_ROWS = 8;
__global__ void __launch_bounds__(256) logistic_rows_small_kernel(float* __restrict__ logits,
                                                                  const int* __restrict__ labels, long rows, int K,
                                                                  float inv_n, float* __restrict__ nll) {
  constexpr int ROWS = LOGIT_SMALL_ROWS;
  const long row0 = ((long)blockIdx.x * 4 + (threadIdx.x >> 6)) * ROWS;
  if (row0 >= rows) return;   // whole waves leave: the reductions below see all 64 lanes
  const int lane = threadIdx.x & 63;
  const bool on = lane < (K >> 2);
  float4 v[ROWS];
  float at[ROWS];
  int label[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    const long row = row0 + r;
    const bool ok = row < rows;   // wave-uniform
    v[r] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    label[r] = -1;
    at[r] = 0.f;
    if (ok) {
      if (on) v[r] = reinterpret_cast<const float4*>(logits + row * K)[lane];
      const int l = labels[row];
      if (l >= 0 && l < K) { label[r] = l; at[r] = logits[row * K + l]; }   // read before the row is overwritten
    }
  }
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    const long row = row0 + r;
    if (row >= rows) break;
    const bool valid = label[r] >= 0;
    const float mx = wave_max(fmaxf(fmaxf(v[r].x, v[r].y), fmaxf(v[r].z, v[r].w)));
    float e[4] = {expf(v[r].x - mx), expf(v[r].y - mx), expf(v[r].z - mx), expf(v[r].w - mx)};   // exp(-inf) = 0 off the row
    const float sum = wave_sum((e[0] + e[1]) + (e[2] + e[3]));
    const float scale = valid ? inv_n / sum : 0.f;
    if (on) {
      float o[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q] = e[q] * scale - ((valid && 4 * lane + q == label[r]) ? inv_n : 0.f);
      reinterpret_cast<float4*>(logits + row * K)[lane] = make_float4(o[0], o[1], o[2], o[3]);
    }
    if (lane == 0) nll[row] = valid ? logf(sum) - (at[r] - mx) : 0.f;
  }
}

}  // namespace

dipaco_status launch_logistic_rows(float* logits, const int* labels, int64_t rows, int K, float inv_n, float* nll,
                                   hipStream_t s) {
  if (K < 4 || K % 4 || K > LOGIT_MAX_K) return fail(DIPACO_ESHAPE, "logistic rows: K must be a multiple of 4 in [4, 4096]");
  if (rows == 0) return DIPACO_OK;
  const bool small = K <= 256;
  const int64_t rows_per_block = small ? 4 * LOGIT_SMALL_ROWS : 4;
  const int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
  if (blocks > 0x7fffffffLL) return fail(DIPACO_ESHAPE, "logistic rows: too many rows");
  if (small) logistic_rows_small_kernel<<<(unsigned)blocks, 256, 0, s>>>(logits, labels, (long)rows, K, inv_n, nll);
  else logistic_rows_kernel<<<(unsigned)blocks, 256, 0, s>>>(logits, labels, (long)rows, K, inv_n, nll);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_route(const float* z, int64_t ldz, const float* c, const float* lin_bias, int64_t N, int D, int K,
                           int n_best, int* idx, long long* hist, float* margin, hipStream_t s) {
  dipaco_status st = launch_fill_i64(hist, 0, (size_t)K, s);
  if (st != DIPACO_OK) return st;
  if (N == 0) return DIPACO_OK;
  constexpr size_t smem = 2 * (size_t)R_STAGE;
  static std::atomic<unsigned long long> lds_one{0}, lds_two{0};
  if (dipaco_status e = ensure_dynamic_lds(reinterpret_cast<const void*>(route_kernel<false>), (int)smem, lds_one)) return e;
  if (dipaco_status e = ensure_dynamic_lds(reinterpret_cast<const void*>(route_kernel<true>), (int)smem, lds_two)) return e;
  const int64_t blocks = (N + RBM - 1) / RBM;
  if (blocks > 0x7fffffffLL) return fail(DIPACO_ESHAPE, "route: N too large");
  auto* h = reinterpret_cast<unsigned long long*>(hist);
  if (n_best == 2) route_kernel<true><<<(unsigned)blocks, R_THREADS, smem, s>>>(z, (long)ldz, c, lin_bias, (long)N, D, K, idx, h, margin);
  else route_kernel<false><<<(unsigned)blocks, R_THREADS, smem, s>>>(z, (long)ldz, c, lin_bias, (long)N, D, K, idx, h, margin);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace dipaco
