// Row-wise kernels of the path transformer: embedding gather, LayerNorm forward/backward, column sums (bias
// gradients), softmax cross-entropy over the vocabulary, and the deterministic embedding gradient.
// All are HBM-bound: I/O in the activation type T (fp32 or bf16), arithmetic in fp32, 16-byte accesses.
#include <algorithm>

#include <type_traits>

#include "kernels.h"

namespace dipaco {

namespace {

constexpr int ROW_THREADS = 256;
constexpr int ROWS_PER_BLOCK = ROW_THREADS / WAVE;  // one wave per row

// ---- embedding -------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(ROW_THREADS) embed_kernel(const T* __restrict__ E, const T* __restrict__ P,
                                                            const int* __restrict__ tok, T* __restrict__ x, int rows,
                                                            int S, int d, int vocab) {
  constexpr int VEC = Vec16<T>::N;
  const int row = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  int t = tok[row];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const T* e = E + (size_t)t * d;
  const T* p = P + (size_t)(row % S) * d;
  T* o = x + (size_t)row * d;
  for (int c = lane * VEC; c < d; c += WAVE * VEC) {
    float a[VEC], b[VEC];
    load_vec16(e + c, a);
    load_vec16(p + c, b);
#pragma unroll
    for (int i = 0; i < VEC; ++i) a[i] += b[i];
    store_vec16(o + c, a);
  }
}

// ---- LayerNorm forward: one wave per row ------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(ROW_THREADS) ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                             const T* __restrict__ b, T* __restrict__ y,
                                                             float* __restrict__ mean, float* __restrict__ rstd,
                                                             int rows, int d, float eps) {
  constexpr int VEC = Vec16<T>::N;
  const int row = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const T* xr = x + (size_t)row * d;
  float s = 0.f;
  for (int c = lane * VEC; c < d; c += WAVE * VEC) {
    float a[VEC];
    load_vec16(xr + c, a);
#pragma unroll
    for (int i = 0; i < VEC; ++i) s += a[i];
  }
  const float mu = wave_sum(s) / d;
  float q = 0.f;
  for (int c = lane * VEC; c < d; c += WAVE * VEC) {
    float a[VEC];
    load_vec16(xr + c, a);
#pragma unroll
    for (int i = 0; i < VEC; ++i) { float t = a[i] - mu; q += t * t; }
  }
  const float rs = 1.0f / sqrtf(wave_sum(q) / d + eps);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  T* yr = y + (size_t)row * d;
  for (int c = lane * VEC; c < d; c += WAVE * VEC) {
    float a[VEC], gg[VEC], bb[VEC];
    load_vec16(xr + c, a);
    load_vec16(g + c, gg);
    load_vec16(b + c, bb);
#pragma unroll
    for (int i = 0; i < VEC; ++i) a[i] = (a[i] - mu) * rs * gg[i] + bb[i];
    store_vec16(yr + c, a);
  }
}

// The same with the row held in registers (NIT chunks of 16 bytes per lane, d <= 64 * VEC * NIT): x is read once, and
// the gain and bias vectors are requested before the reductions, so that a row costs one trip to memory instead of
// three dependent ones.  Same order of additions as the kernel above: identical results.
template <typename T, int NIT>
__global__ void __launch_bounds__(ROW_THREADS) ln_fwd_reg_kernel(const T* __restrict__ x, const T* __restrict__ g,
                                                                 const T* __restrict__ b, T* __restrict__ y,
                                                                 float* __restrict__ mean, float* __restrict__ rstd,
                                                                 int rows, int d, float eps) {
  constexpr int VEC = Vec16<T>::N;
  const int row = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int lane = threadIdx.x & 63;
  const T* xr = x + (size_t)row * d;
  float a[NIT][VEC], gg[NIT][VEC], bb[NIT][VEC];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = (lane + WAVE * it) * VEC;
    if (c < d) {
      load_vec16(xr + c, a[it]);
      load_vec16(g + c, gg[it]);
      load_vec16(b + c, bb[it]);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if ((lane + WAVE * it) * VEC < d) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) s += a[it][i];
    }
  const float mu = wave_sum(s) / d;
  float q = 0.f;
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if ((lane + WAVE * it) * VEC < d) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) { float t = a[it][i] - mu; q += t * t; }
    }
  const float rs = 1.0f / sqrtf(wave_sum(q) / d + eps);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  T* yr = y + (size_t)row * d;
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = (lane + WAVE * it) * VEC;
    if (c < d) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) a[it][i] = (a[it][i] - mu) * rs * gg[it][i] + bb[it][i];
      store_vec16(yr + c, a[it]);
    }
  }
}

// ---- LayerNorm backward -----------------------------------------------------------------------------------
// Each workgroup owns LN_BWD_ROWS consecutive rows (one wave per row at a time), writes dx for them and one
// partial row of dg / db / column sums of dx; a second kernel sums the partial rows in block order.  The column
// sums of dx (of the values as stored, i.e. rounded to T) are the bias gradient of the linear layer whose output
// gradient dx is.
constexpr int LN_BWD_ROWS = 32;
constexpr int LN_MAX_IT = 4;   // column chunks per lane: d <= 64 * VEC * LN_MAX_IT

template <typename T, int NIT>   // NIT column chunks of 16 bytes per lane: d <= 64 * VEC * NIT
__global__ void __launch_bounds__(ROW_THREADS) ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                             const T* __restrict__ g, const float* __restrict__ mean,
                                                             const float* __restrict__ rstd,
                                                             const T* __restrict__ resid_grad, T* __restrict__ dx,
                                                             float* __restrict__ partial, int rows, int d,
                                                             int rows_per_block) {
  constexpr int VEC = Vec16<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row0 = blockIdx.x * rows_per_block;
  float ag[NIT][VEC], ab[NIT][VEC], ac[NIT][VEC], gv[NIT][VEC];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = (lane + WAVE * it) * VEC;
#pragma unroll
    for (int i = 0; i < VEC; ++i) { ag[it][i] = 0.f; ab[it][i] = 0.f; ac[it][i] = 0.f; gv[it][i] = 0.f; }
    if (c < d) load_vec16(g + c, gv[it]);
  }

  // The rows of a wave are pipelined by hand: the 16-byte vectors of the next row (and its statistics) are requested
  // before the current row is reduced, so that a row does not wait out a whole trip to memory.
  uint4 nx[NIT], ndy[NIT], nres[NIT];
  float nmu = 0.f, nrs = 0.f;
  auto fetch = [&](int row) {
    nmu = mean[row];
    nrs = rstd[row];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = (lane + WAVE * it) * VEC;
      if (c < d) {
        nx[it] = *reinterpret_cast<const uint4*>(x + (size_t)row * d + c);
        ndy[it] = *reinterpret_cast<const uint4*>(dy + (size_t)row * d + c);
        if (resid_grad) nres[it] = *reinterpret_cast<const uint4*>(resid_grad + (size_t)row * d + c);
      }
    }
  };
  auto unpack = [](const uint4& raw, float (&out)[VEC]) {
    const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
    for (int i = 0; i < VEC; ++i) out[i] = to_f32(e[i]);
  };
  int r = wave;
  bool have = r < rows_per_block && row0 + r < rows;
  if (have) fetch(row0 + r);
  while (have) {
    const int row = row0 + r;
    const float mu = nmu, rs = nrs;
    float xh[NIT][VEC], dv[NIT][VEC], out[NIT][VEC];   // the row stays in registers between the two passes
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = (lane + WAVE * it) * VEC;
      if (c < d) {
        unpack(nx[it], xh[it]);
        unpack(ndy[it], dv[it]);
        if (resid_grad) unpack(nres[it], out[it]);
        else {
#pragma unroll
          for (int i = 0; i < VEC; ++i) out[it][i] = 0.f;
        }
      }
    }
    r += ROWS_PER_BLOCK;
    have = r < rows_per_block && row0 + r < rows;
    if (have) fetch(row0 + r);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = (lane + WAVE * it) * VEC;
      if (c < d) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          xh[it][i] = (xh[it][i] - mu) * rs;
          const float dxh = dv[it][i] * gv[it][i];
          s1 += dxh;
          s2 += dxh * xh[it][i];
          ag[it][i] += dv[it][i] * xh[it][i];
          ab[it][i] += dv[it][i];
        }
      }
    }
    const float c1 = wave_sum(s1) / d, c2 = wave_sum(s2) / d;
    T* dxr = dx + (size_t)row * d;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = (lane + WAVE * it) * VEC;
      if (c < d) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          out[it][i] += rs * (dv[it][i] * gv[it][i] - c1 - xh[it][i] * c2);
          ac[it][i] += to_f32(from_f32<T>(out[it][i]));
        }
        store_vec16(dxr + c, out[it]);
      }
    }
  }
  // combine the four waves' column sums in wave order: each wave in turn adds into a [3][d] LDS row
  extern __shared__ float cols[];
  for (int w = 0; w < ROWS_PER_BLOCK; ++w) {
    if (wave == w) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int c = (lane + WAVE * it) * VEC;
        if (c < d) {
#pragma unroll
          for (int i = 0; i < VEC; ++i) {
            if (w == 0) { cols[c + i] = ag[it][i]; cols[d + c + i] = ab[it][i]; cols[2 * d + c + i] = ac[it][i]; }
            else { cols[c + i] += ag[it][i]; cols[d + c + i] += ab[it][i]; cols[2 * d + c + i] += ac[it][i]; }
          }
        }
      }
    }
    __syncthreads();
  }
  float* out = partial + (size_t)blockIdx.x * 3 * d;
  for (int c = threadIdx.x; c < 3 * d; c += ROW_THREADS) out[c] = cols[c];
}

// out[c] = sum over p of partial[p * stride + c].  32 columns x 32 partial phases per workgroup: phase y adds
// partials y, y+32, ... in order (four loads in flight), then the phase sums are added in phase order (a fixed tree).
// Column c goes to out0 / out1 / out2 by c / d (a null output is skipped).
constexpr int SP_COLS = 32, SP_PHASES = 32;
__global__ void __launch_bounds__(SP_COLS * SP_PHASES) sum_partials_kernel(const float* __restrict__ partial,
                                                                           float* __restrict__ out0,
                                                                           float* __restrict__ out1,
                                                                           float* __restrict__ out2, int n_partials,
                                                                           int stride, int d) {
  __shared__ float red[SP_PHASES][SP_COLS + 1];
  const int x = threadIdx.x % SP_COLS, y = threadIdx.x / SP_COLS;
  const int c = blockIdx.x * SP_COLS + x;
  float s = 0.f;
  if (c < stride) {
    int p = y;
    for (; p + 3 * SP_PHASES < n_partials; p += 4 * SP_PHASES) {
      const float a0 = partial[(size_t)p * stride + c], a1 = partial[(size_t)(p + SP_PHASES) * stride + c];
      const float a2 = partial[(size_t)(p + 2 * SP_PHASES) * stride + c];
      const float a3 = partial[(size_t)(p + 3 * SP_PHASES) * stride + c];
      s += a0; s += a1; s += a2; s += a3;
    }
    for (; p < n_partials; p += SP_PHASES) s += partial[(size_t)p * stride + c];
  }
  red[y][x] = s;
  __syncthreads();
  if (y == 0 && c < stride) {
    float t = red[0][x];
#pragma unroll
    for (int q = 1; q < SP_PHASES; ++q) t += red[q][x];
    if (c < d) out0[c] = t;
    else if (c < 2 * d) out1[c - d] = t;
    else if (out2) out2[c - 2 * d] = t;
  }
}

// The same for a batch of jobs: blockIdx.y is the job, blockIdx.x its block of 32 columns.
struct SumBatchArgs { SumJob job[SUM_BATCH_MAX]; };
__global__ void __launch_bounds__(SP_COLS * SP_PHASES) sum_partials_batch_kernel(const SumBatchArgs a) {
  __shared__ float red[SP_PHASES][SP_COLS + 1];
  const SumJob& j = a.job[blockIdx.y];
  const int n_partials = j.n_partials, stride = j.stride, d = j.d;
  if ((int)blockIdx.x * SP_COLS >= stride) return;   // workgroup-uniform: this job has fewer columns than the widest
  const float* __restrict__ partial = j.partial;
  const int x = threadIdx.x % SP_COLS, y = threadIdx.x / SP_COLS;
  const int c = blockIdx.x * SP_COLS + x;
  float s = 0.f;
  if (c < stride) {
    int p = y;
    for (; p + 3 * SP_PHASES < n_partials; p += 4 * SP_PHASES) {
      const float a0 = partial[(size_t)p * stride + c], a1 = partial[(size_t)(p + SP_PHASES) * stride + c];
      const float a2 = partial[(size_t)(p + 2 * SP_PHASES) * stride + c];
      const float a3 = partial[(size_t)(p + 3 * SP_PHASES) * stride + c];
      s += a0; s += a1; s += a2; s += a3;
    }
    for (; p < n_partials; p += SP_PHASES) s += partial[(size_t)p * stride + c];
  }
  red[y][x] = s;
  __syncthreads();
  if (y == 0 && c < stride) {
    float t = red[0][x];
#pragma unroll
    for (int q = 1; q < SP_PHASES; ++q) t += red[q][x];
    if (c < d) j.out0[c] = t;
    else if (c < 2 * d) j.out1[c - d] = t;
    else if (j.out2) j.out2[c - 2 * d] = t;
  }
}

// ---- column sums -----------------------------------------------------------------------------------------
constexpr int CS_ROWS = 256;   // rows per workgroup
template <typename T>
__global__ void __launch_bounds__(ROW_THREADS) colsum_kernel(const T* __restrict__ x, float* __restrict__ partial,
                                                             int rows, int cols) {
  constexpr int VEC = Vec16<T>::N;
  // workgroup: 64 column chunks (16 B each) x 4 row phases
  __shared__ float red[ROWS_PER_BLOCK][WAVE * VEC];
  const int lane = threadIdx.x & 63, phase = threadIdx.x >> 6;
  const int c = (blockIdx.x * WAVE + lane) * VEC;
  const int row0 = blockIdx.y * CS_ROWS;
  const int row1 = min(rows, row0 + CS_ROWS);
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  if (c < cols) {
    for (int r = row0 + phase; r < row1; r += ROWS_PER_BLOCK) {
      float v[VEC];
      load_vec16(x + (size_t)r * cols + c, v);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += v[i];
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) red[phase][lane * VEC + i] = acc[i];
  __syncthreads();
  if (phase == 0 && c < cols) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float s = red[0][lane * VEC + i];
      for (int p = 1; p < ROWS_PER_BLOCK; ++p) s += red[p][lane * VEC + i];
      partial[(size_t)blockIdx.y * cols + c + i] = s;
    }
  }
}

// ---- loss ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) count_valid_kernel(const int* __restrict__ targets, int n,
                                                           int* __restrict__ n_valid) {
  __shared__ int red[16];
  int c = 0;
  for (int i = threadIdx.x; i < n; i += 1024) c += targets[i] >= 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, WAVE);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int s = 0;
    for (int i = 0; i < 16; ++i) s += red[i];
    n_valid[0] = s;
  }
}

__device__ __forceinline__ float block_reduce(float v, float* red, bool is_max) {
  v = is_max ? wave_max(v) : wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  return r;
}

// one workgroup per row of logits
// One workgroup per row.  NV > 0: XENT_THREADS threads keep the whole row in registers (NV 16-byte vectors each,
// V <= NV * XENT_THREADS * 16 / sizeof(T)), so the logits cross the memory interface once in each direction.
// NV == 0: any V, three passes over memory.
constexpr int XENT_THREADS = 1024;
// exp for the softmax: logits held in bf16 carry 8 significant bits, so the hardware base-2 exponential (relative
// error about 1e-6 over the range used here) is exact enough; fp32 runs keep the library routine
template <typename T> __device__ __forceinline__ float softmax_exp(float x);
template <> __device__ __forceinline__ float softmax_exp<float>(float x) { return expf(x); }
template <> __device__ __forceinline__ float softmax_exp<bf16>(float x) {
  return __builtin_amdgcn_exp2f(x * 1.4426950408889634f);
}
// GRAD = false: the negative log-likelihood alone (scoring passes); the logits are left as they are.
template <typename T, int NV, bool GRAD>
__global__ void __launch_bounds__(NV > 0 ? XENT_THREADS : ROW_THREADS)
softmax_xent_kernel(T* __restrict__ logits, const int* __restrict__ targets, const int* __restrict__ n_valid,
                    float* __restrict__ nll, int V) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int NTH = NV > 0 ? XENT_THREADS : ROW_THREADS;
  constexpr int NKEEP = NV > 0 ? NV : 1;
  __shared__ float red[NTH / WAVE];
  const int row = blockIdx.x;
  T* lr = logits + (size_t)row * V;
  const int tgt = targets[row];
  if (tgt < 0) {   // ignored position: no loss, no gradient (uniform branch: tgt is per workgroup)
    float zero[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) zero[i] = 0.f;
    if (GRAD)
      for (int c = threadIdx.x * VEC; c < V; c += NTH * VEC) store_vec16(lr + c, zero);
    if (threadIdx.x == 0) nll[row] = 0.f;
    return;
  }
  uint4 keep[NKEEP];
  auto vec_at = [&](int k, int c, float (&v)[VEC]) {   // k-th vector of this thread, at column c
    if (NV > 0) {
      const T* e = reinterpret_cast<const T*>(&keep[k]);
#pragma unroll
      for (int i = 0; i < VEC; ++i) v[i] = to_f32(e[i]);
    } else {
      load_vec16(lr + c, v);
    }
  };
  auto for_each_vec = [&](auto&& f) {   // f(k, c): this thread's k-th vector, at column c
    if constexpr (NV > 0) {
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        const int c = (threadIdx.x + k * NTH) * VEC;
        if (c < V) f(k, c);
      }
    } else {
      for (int c = threadIdx.x * VEC; c < V; c += NTH * VEC) f(0, c);
    }
  };
  float mx = -INFINITY;
  if constexpr (NV > 0) for_each_vec([&](int k, int c) { keep[k] = *reinterpret_cast<const uint4*>(lr + c); });
  for_each_vec([&](int k, int c) {
    float v[VEC];
    vec_at(k, c, v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) mx = fmaxf(mx, v[i]);
  });
  mx = block_reduce(mx, red, true);
  float se = 0.f;
  for_each_vec([&](int k, int c) {
    float v[VEC];
    vec_at(k, c, v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) se += softmax_exp<T>(v[i] - mx);
  });
  se = block_reduce(se, red, false);
  const int t = tgt >= V ? V - 1 : tgt;
  if (threadIdx.x == 0) nll[row] = logf(se) - (to_f32(lr[t]) - mx);
  if (!GRAD) return;
  __syncthreads();   // lr[t] is read before anyone overwrites it
  const float inv = 1.0f / se;
  const float scale = 1.0f / (float)n_valid[0];
  for_each_vec([&](int k, int c) {
    float v[VEC];
    vec_at(k, c, v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float p = softmax_exp<T>(v[i] - mx) * inv;
      if (c + i == t) p -= 1.0f;
      v[i] = p * scale;
    }
    store_vec16(lr + c, v);
  });
}

// loss = (sum of nll in a fixed tree order) / n_valid; one workgroup
__global__ void __launch_bounds__(1024) mean_loss_kernel(const float* __restrict__ nll, const int* __restrict__ n_valid,
                                                         float* __restrict__ loss, int rows) {
  __shared__ float red[16];
  // 16-byte loads, four in flight per thread (one workgroup has to pull a million values for the router's loss);
  // the order of the additions is fixed by the indices alone
  const float4* __restrict__ nll4 = reinterpret_cast<const float4*>(nll);
  const int n4 = (reinterpret_cast<uintptr_t>(nll) & 15) == 0 ? rows >> 2 : 0;   // unaligned: the scalar loop takes all
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int i = threadIdx.x;
  for (; i + 3 * 1024 < n4; i += 4 * 1024) {
    const float4 a = nll4[i], b = nll4[i + 1024], c = nll4[i + 2048], d = nll4[i + 3072];
    s0 += (a.x + a.y) + (a.z + a.w);
    s1 += (b.x + b.y) + (b.z + b.w);
    s2 += (c.x + c.y) + (c.z + c.w);
    s3 += (d.x + d.y) + (d.z + d.w);
  }
  for (; i < n4; i += 1024) {
    const float4 a = nll4[i];
    s0 += (a.x + a.y) + (a.z + a.w);
  }
  for (int j = 4 * n4 + threadIdx.x; j < rows; j += 1024) s1 += nll[j];
  float s = (s0 + s1) + (s2 + s3);
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < 16; ++i) t += red[i];
    loss[0] = t / (float)n_valid[0];
  }
}

// ---- embedding gradient ----------------------------------------------------------------------------------
// d_tok[v] = sum of dx rows whose token is v, added in increasing position order (no float atomics): positions are
// grouped by token with a stable sort (kmeans.hip), then one workgroup per vocabulary row adds its positions.
// One workgroup (16 waves) per vocabulary row.  Wave w adds the row's positions w, w+16, ... in order (lanes over
// 16-byte column chunks, eight row loads in flight), then the wave sums are added in wave order: a fixed tree, so the frequent tokens
// of a Zipf batch (thousands of positions) are spread over the workgroup without any atomics.
constexpr int TG_WAVES = 16;
constexpr int TG_UNROLL = 8;   // row loads in flight per wave
constexpr int TG_MAX_D = 2048;   // widest model: 16 partial rows of 2048 floats = 128 KB of the 160 KB of LDS
template <typename T>
__global__ void __launch_bounds__(TG_WAVES * WAVE) tok_grad_kernel(const T* __restrict__ dx,
                                                                   const int* __restrict__ offsets,
                                                                   const int* __restrict__ order,
                                                                   float* __restrict__ d_tok, int d) {
  constexpr int VEC = Vec16<T>::N;
  extern __shared__ float tg_red[];   // [TG_WAVES][d]
  const int v = blockIdx.x;
  const int lo = offsets[v], hi = offsets[v + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* o = d_tok + (size_t)v * d;
  if (hi - lo <= 1) {   // most of the vocabulary: nothing to add
    for (int c = threadIdx.x * VEC; c < d; c += TG_WAVES * WAVE * VEC) {
      float a[VEC];
      if (hi > lo) load_vec16(dx + (size_t)order[lo] * d + c, a);
      else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) a[i] = 0.f;
      }
#pragma unroll
      for (int i = 0; i < VEC; ++i) o[c + i] = a[i];
    }
    return;
  }
  for (int c = lane * VEC; c < d; c += WAVE * VEC) {
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    int j = lo + wave;
    for (; j + (TG_UNROLL - 1) * TG_WAVES < hi; j += TG_UNROLL * TG_WAVES) {
      float a[TG_UNROLL][VEC];
#pragma unroll
      for (int u = 0; u < TG_UNROLL; ++u) load_vec16(dx + (size_t)order[j + u * TG_WAVES] * d + c, a[u]);
#pragma unroll
      for (int u = 0; u < TG_UNROLL; ++u)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += a[u][i];
    }
    for (; j < hi; j += TG_WAVES) {
      float a[VEC];
      load_vec16(dx + (size_t)order[j] * d + c, a);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += a[i];
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) tg_red[wave * d + c + i] = acc[i];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += TG_WAVES * WAVE) {
    float t = tg_red[c];
#pragma unroll
    for (int w = 1; w < TG_WAVES; ++w) t += tg_red[w * d + c];
    o[c] = t;
  }
}

// d_pos[s] = sum_b dx[b*S + s] for s < S, 0 for S <= s < max_seq
template <typename T>
__global__ void __launch_bounds__(128) pos_grad_kernel(const T* __restrict__ dx, float* __restrict__ d_pos, int B, int S,
                                                       int d) {
  constexpr int VEC = Vec16<T>::N;
  const int s = blockIdx.x;
  for (int c = threadIdx.x * VEC; c < d; c += 128 * VEC) {
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    if (s < S) {
      for (int b = 0; b < B; ++b) {
        float a[VEC];
        load_vec16(dx + ((size_t)b * S + s) * d + c, a);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += a[i];
      }
    }
    float* o = d_pos + (size_t)s * d + c;
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[i] = acc[i];
  }
}

inline int row_blocks(int rows) { return (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK; }

}  // namespace

template <typename T>
dipaco_status launch_embed(const T* E, const T* P, const int* tokens, T* x, int B, int S, int d, int vocab,
                           hipStream_t s) {
  const int rows = B * S;
  embed_kernel<T><<<row_blocks(rows), ROW_THREADS, 0, s>>>(E, P, tokens, x, rows, S, d, vocab);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

template <typename T>
dipaco_status launch_layernorm_fwd(const T* x, const T* g, const T* b, T* y, float* mean, float* rstd, int rows,
                                   int d, float eps, hipStream_t s) {
  constexpr int VEC = Vec16<T>::N;
  const int chunks = (d + WAVE * VEC - 1) / (WAVE * VEC);   // 16-byte chunks per lane
  if (chunks <= 1) ln_fwd_reg_kernel<T, 1><<<row_blocks(rows), ROW_THREADS, 0, s>>>(x, g, b, y, mean, rstd, rows, d, eps);
  else if (chunks <= 2) ln_fwd_reg_kernel<T, 2><<<row_blocks(rows), ROW_THREADS, 0, s>>>(x, g, b, y, mean, rstd, rows, d, eps);
  else if (chunks <= 4) ln_fwd_reg_kernel<T, 4><<<row_blocks(rows), ROW_THREADS, 0, s>>>(x, g, b, y, mean, rstd, rows, d, eps);
  else ln_fwd_kernel<T><<<row_blocks(rows), ROW_THREADS, 0, s>>>(x, g, b, y, mean, rstd, rows, d, eps);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

size_t ln_bwd_partial_floats(int rows, int d) {
  return (size_t)((rows + LN_BWD_ROWS - 1) / LN_BWD_ROWS) * 3 * d;
}

template <typename T>
dipaco_status launch_layernorm_bwd(const T* dy, const T* x, const T* g, const float* mean, const float* rstd,
                                   const T* resid_grad, T* dx, float* dg, float* db, float* dcol, float* partial,
                                   int rows, int d, hipStream_t s, SumBatch* batch) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int NIT = (sizeof(T) == 4) ? 2 * LN_MAX_IT : LN_MAX_IT;
  if (d > WAVE * VEC * NIT) return fail(DIPACO_ESHAPE, "layernorm backward: d_model above 2048");
  const size_t lds = 3 * d * sizeof(float);
  // the kernel keeps NIT chunks per lane of seven row-shaped quantities in registers: narrow models take the
  // instantiation with half (a quarter) of them and twice (four times) the waves per SIMD
  int n_blocks = 0;
  // resident workgroups per compute unit of each instantiation, remembered with the LDS size they were asked for
  // (packed lds << 8 | resident; a host thread that loses a race merely asks again)
  static std::atomic<unsigned long long> occupancy[3];
  auto run = [&](auto kern, int variant) -> dipaco_status {
    // Rows per workgroup: LN_BWD_ROWS, unless that gives a little more than a whole number of rounds of resident
    // workgroups (1024 workgroups over 768 slots run as two rounds): then as many rows as fill the slots once.
    const unsigned long long seen = occupancy[variant].load(std::memory_order_relaxed);
    int resident = (seen >> 8) == lds ? (int)(seen & 255) : 0;
    if (resident == 0) {
      int nb = 0;
      DIPACO_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, ROW_THREADS, lds));
      resident = nb > 0 ? (nb < 255 ? nb : 255) : 1;
      occupancy[variant].store(((unsigned long long)lds << 8) | (unsigned)resident, std::memory_order_relaxed);
    }
    const long slots = 256L * resident;
    int rpb = LN_BWD_ROWS;
    const long base_blocks = (rows + LN_BWD_ROWS - 1) / LN_BWD_ROWS;
    if (base_blocks > slots && base_blocks < 2 * slots) {
      rpb = (int)((rows + slots - 1) / slots);
      rpb = (rpb + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK * ROWS_PER_BLOCK;
    }
    n_blocks = (rows + rpb - 1) / rpb;
    kern<<<n_blocks, ROW_THREADS, lds, s>>>(dy, x, g, mean, rstd, resid_grad, dx, partial, rows, d, rpb);
    return DIPACO_OK;
  };
  dipaco_status st;
  if (d <= WAVE * VEC * NIT / 4) st = run(ln_bwd_kernel<T, NIT / 4>, 0);
  else if (d <= WAVE * VEC * NIT / 2) st = run(ln_bwd_kernel<T, NIT / 2>, 1);
  else st = run(ln_bwd_kernel<T, NIT>, 2);
  if (st != DIPACO_OK) return st;
  DIPACO_LAUNCH_CHECK();
  return sum_partials(partial, dg, db, dcol, n_blocks, 3 * d, d, batch, s);
}

dipaco_status sum_partials(const float* partial, float* out0, float* out1, float* out2, int n_partials, int stride,
                           int d, SumBatch* batch, hipStream_t s) {
  if (batch) {
    if (batch->count == SUM_BATCH_MAX) {
      const dipaco_status st = flush_sum_batch(*batch, s);
      if (st != DIPACO_OK) return st;
    }
    batch->job[batch->count++] = SumJob{partial, out0, out1, out2, n_partials, stride, d};
    return DIPACO_OK;
  }
  // columns of a null third output are not computed
  const int ncols = (!out2 && stride > 2 * d) ? 2 * d : stride;
  sum_partials_kernel<<<(ncols + SP_COLS - 1) / SP_COLS, SP_COLS * SP_PHASES, 0, s>>>(partial, out0, out1, out2, n_partials, stride, d);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status flush_sum_batch(SumBatch& batch, hipStream_t s) {
  if (batch.count == 0) return DIPACO_OK;
  SumBatchArgs a;
  int widest = 0;
  for (int i = 0; i < batch.count; ++i) {
    a.job[i] = batch.job[i];
    widest = std::max(widest, batch.job[i].stride);
  }
  dim3 grid((widest + SP_COLS - 1) / SP_COLS, batch.count);
  sum_partials_batch_kernel<<<grid, SP_COLS * SP_PHASES, 0, s>>>(a);
  batch.count = 0;
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

size_t colsum_partial_floats(int rows, int cols) { return (size_t)((rows + CS_ROWS - 1) / CS_ROWS) * cols; }

template <typename T>
dipaco_status launch_colsum(const T* x, float* out, float* partial, int rows, int cols, hipStream_t s) {
  constexpr int VEC = Vec16<T>::N;
  const int chunks = (rows + CS_ROWS - 1) / CS_ROWS;
  dim3 grid((cols + WAVE * VEC - 1) / (WAVE * VEC), chunks);
  colsum_kernel<T><<<grid, ROW_THREADS, 0, s>>>(x, partial, rows, cols);
  DIPACO_LAUNCH_CHECK();
  sum_partials_kernel<<<(cols + SP_COLS - 1) / SP_COLS, SP_COLS * SP_PHASES, 0, s>>>(partial, out, out, nullptr, chunks, cols, cols);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_sum_rows(const float* partial, float* out, int n_partials, int cols, hipStream_t s, SumBatch* batch) {
  return sum_partials(partial, out, out, nullptr, n_partials, cols, cols, batch, s);
}

dipaco_status launch_count_valid(const int* targets, int n, int* n_valid, hipStream_t s) {
  count_valid_kernel<<<1, 1024, 0, s>>>(targets, n, n_valid);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

template <typename T>
dipaco_status launch_softmax_xent(T* logits, const int* targets, const int* n_valid, float* nll, int rows, int V,
                                  bool want_grad, hipStream_t s) {
  const size_t vectors = ((size_t)V * sizeof(T) + 15) / 16;
  auto go = [&](auto grad) {
    constexpr bool G = decltype(grad)::value;
    if (vectors <= 4 * (size_t)XENT_THREADS) softmax_xent_kernel<T, 4, G><<<rows, XENT_THREADS, 0, s>>>(logits, targets, n_valid, nll, V);
    else if (vectors <= 8 * (size_t)XENT_THREADS) softmax_xent_kernel<T, 8, G><<<rows, XENT_THREADS, 0, s>>>(logits, targets, n_valid, nll, V);
    else softmax_xent_kernel<T, 0, G><<<rows, ROW_THREADS, 0, s>>>(logits, targets, n_valid, nll, V);
  };
  if (want_grad) go(std::true_type{});
  else go(std::false_type{});
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_mean_loss(const float* nll, const int* n_valid, float* loss, int rows, hipStream_t s) {
  mean_loss_kernel<<<1, 1024, 0, s>>>(nll, n_valid, loss, rows);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

size_t embed_bwd_scratch_ints(int rows, int vocab) {
  return (size_t)vocab + (size_t)vocab + 1 + (size_t)rows + sort_scratch_ints(rows, vocab);
}

template <typename T>
dipaco_status launch_embed_bwd(const T* dx, const int* tokens, float* d_tok, float* d_pos, int* scratch, int B,
                               int S, int d, int vocab, int max_seq, hipStream_t s) {
  const int rows = B * S;
  int* count = scratch;
  int* offsets = scratch + vocab;
  int* order = offsets + vocab + 1;
  int* sort_scratch = order + rows;
  // positions grouped by token id, earlier positions first (stable sort: integer work only), so that every
  // vocabulary row is summed in a fixed order
  dipaco_status st = launch_key_offsets(tokens, rows, vocab, count, offsets, nullptr, s);
  if (st != DIPACO_OK) return st;
  st = launch_stable_sort_indices(tokens, rows, vocab, order, sort_scratch, s);
  if (st != DIPACO_OK) return st;
  // 16 partial rows of d floats: above 64 KB (d_model > 1024) the kernel's dynamic-LDS limit has to be raised
  static std::atomic<unsigned long long> tg_lds{0};
  st = ensure_dynamic_lds(reinterpret_cast<const void*>(tok_grad_kernel<T>), TG_WAVES * TG_MAX_D * (int)sizeof(float), tg_lds);
  if (st != DIPACO_OK) return st;
  if (d > TG_MAX_D) return fail(DIPACO_ESHAPE, "embedding gradient: d_model above 2048");
  tok_grad_kernel<T><<<vocab, TG_WAVES * WAVE, TG_WAVES * d * sizeof(float), s>>>(dx, offsets, order, d_tok, d);
  DIPACO_LAUNCH_CHECK();
  pos_grad_kernel<T><<<max_seq, 128, 0, s>>>(dx, d_pos, B, S, d);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

// out[b, :] = mean over the S positions of x[b*S + p, :]  (fp32, positions added in order)
template <typename T>
__global__ void __launch_bounds__(256) mean_pool_kernel(const T* __restrict__ x, float* __restrict__ out, int S, int d) {
  const int b = blockIdx.x;
  for (int c = threadIdx.x; c < d; c += 256) {
    float s = 0.f;
    for (int p = 0; p < S; ++p) s += to_f32(x[((size_t)b * S + p) * d + c]);
    out[(size_t)b * d + c] = s / (float)S;
  }
}

// out[b] = -(sum over the S positions of nll[b*S + p]), positions added in a fixed tree order
__global__ void __launch_bounds__(256) doc_score_kernel(const float* __restrict__ nll, float* __restrict__ out, int S) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  float s = 0.f;
  for (int p = threadIdx.x; p < S; p += 256) s += nll[(size_t)b * S + p];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) out[b] = -(((red[0] + red[1]) + red[2]) + red[3]);
}

dipaco_status launch_doc_score(const float* nll, float* out, int B, int S, hipStream_t s) {
  doc_score_kernel<<<B, 256, 0, s>>>(nll, out, S);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

template <typename T>
dipaco_status launch_mean_pool(const T* x, float* out, int B, int S, int d, hipStream_t s) {
  mean_pool_kernel<T><<<B, 256, 0, s>>>(x, out, S, d);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

#define INSTANTIATE(T)                                                                                              \
  template dipaco_status launch_embed<T>(const T*, const T*, const int*, T*, int, int, int, int, hipStream_t);       \
  template dipaco_status launch_layernorm_fwd<T>(const T*, const T*, const T*, T*, float*, float*, int, int, float,  \
                                                 hipStream_t);                                                      \
  template dipaco_status launch_layernorm_bwd<T>(const T*, const T*, const T*, const float*, const float*, const T*, \
                                                 T*, float*, float*, float*, float*, int, int, hipStream_t,         \
                                                 SumBatch*);                                                        \
  template dipaco_status launch_colsum<T>(const T*, float*, float*, int, int, hipStream_t);                          \
  template dipaco_status launch_mean_pool<T>(const T*, float*, int, int, int, hipStream_t);                          \
  template dipaco_status launch_softmax_xent<T>(T*, const int*, const int*, float*, int, int, bool, hipStream_t);          \
  template dipaco_status launch_embed_bwd<T>(const T*, const int*, float*, float*, int*, int, int, int, int, int,    \
                                             hipStream_t);
INSTANTIATE(float)
INSTANTIATE(bf16)

}  // namespace dipaco
