// Bandwidth-bound kernels: path composition (copy + bf16 image), AdamW, the module outer step, fills.
// All are one-pass float4 streams: every parameter byte is read once and written once.
#include "kernels.h"

namespace dipaco {

namespace {

// Launch shape of the streaming kernels: workgroups of 128 threads and one 16-byte vector per thread and stream, i.e.
// as many workgroups as the buffer has 2 KB pieces.  Measured on the 18-stream outer step (57.9 M elements x 16 inputs)
// and on the 7.5-stream AdamW pattern (174 M elements): 6.1 / 5.8 TB/s, against 5.4 / 4.9 TB/s for 16384 workgroups of
// 256 threads walking the buffer with a grid stride, 5.1 TB/s for 1024-4096 persistent workgroups and 5.0-5.6 TB/s for
// workgroup-contiguous chunks of 16-256 KB.  Short-lived workgroups let the dispatcher keep every compute unit's
// request queues full; a thread that loops issues its next loads only after its stores.  (The grid-stride loops
// remain for buffers beyond 2^31 workgroups' worth.)
constexpr int EW_THREADS = 128;
constexpr int TABLE_THREADS = 256;   // the table-driven kernel walks chunks of OUTER_CHUNK elements per workgroup

inline unsigned ew_blocks(size_t n_vec) {
  size_t b = (n_vec + EW_THREADS - 1) / EW_THREADS;
  if (b < 1) b = 1;
  if (b > 0x7fffffffu) b = 0x7fffffffu;
  return (unsigned)b;
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float* p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void stream_store4(float* p, float4 v) {
  const f32x4_t o = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(p));
}

__device__ __forceinline__ void store_bf16x4(bf16* dst, float4 v) {
  bf16x4 o = {(bf16)v.x, (bf16)v.y, (bf16)v.z, (bf16)v.w};
  *reinterpret_cast<bf16x4*>(dst) = o;
}

// ---- compose: dst[i] = src[i], lowp[i] = bf16(src[i]) ------------------------------------------------
__global__ void __launch_bounds__(EW_THREADS) copy_cast_kernel(const float* __restrict__ src,
                                                                float* __restrict__ dst, bf16* __restrict__ lowp,
                                                                size_t n) {
  size_t nv = n >> 2;
  size_t stride = (size_t)gridDim.x * EW_THREADS;
  for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < nv; i += stride) {
    float4 v = reinterpret_cast<const float4*>(src)[i];
    reinterpret_cast<float4*>(dst)[i] = v;
    if (lowp) store_bf16x4(lowp + 4 * i, v);
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {  // tail
    size_t i = (nv << 2) + threadIdx.x;
    float v = src[i];
    dst[i] = v;
    if (lowp) lowp[i] = (bf16)v;
  }
}

// ---- AdamW ---------------------------------------------------------------------------------------------
// Which elements are weight-decayed follows from the flat layout: the stem (embeddings) entirely, inside every
// decoder block the four matrices (between in-block edges 0-1, 2-3, 4-5, 6-7), in the head only w_head.
struct AdamArgs {
  float* theta;
  const float* grad;
  float* m;
  float* v;
  bf16* lowp;
  size_t n;
  unsigned long long stem_end, blocks_end, block_size, head_matrix;
  unsigned int edge[8];
  float lr, beta1, beta2, eps, wd, inv_bc1, inv_bc2;
};

__device__ __forceinline__ bool adam_decayed(const AdamArgs& a, unsigned long long pos) {
  if (pos < a.stem_end) return true;
  if (pos >= a.blocks_end) return pos >= a.head_matrix;
  const unsigned int off = (unsigned int)(pos - a.stem_end) % (unsigned int)a.block_size;   // block region < 2^32 elements
  int c = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) c += off >= a.edge[i];
  return c & 1;
}

__device__ __forceinline__ float adam_one(float th, float g, float& m, float& v, const AdamArgs& a, float decay) {
  m = a.beta1 * m + (1.0f - a.beta1) * g;
  v = a.beta2 * v + (1.0f - a.beta2) * g * g;
  float mhat = m * a.inv_bc1;
  float vhat = v * a.inv_bc2;
  return th - a.lr * (mhat / (sqrtf(vhat) + a.eps) + decay * th);
}

__device__ __forceinline__ void adam_apply4(const AdamArgs& a, size_t i, float4 th, float4 g, float4 m, float4 v) {
  const float decay = adam_decayed(a, (unsigned long long)i << 2) ? a.wd : 0.0f;
  th.x = adam_one(th.x, g.x, m.x, v.x, a, decay);
  th.y = adam_one(th.y, g.y, m.y, v.y, a, decay);
  th.z = adam_one(th.z, g.z, m.z, v.z, a, decay);
  th.w = adam_one(th.w, g.w, m.w, v.w, a, decay);
  stream_store4(a.theta + 4 * i, th);
  stream_store4(a.m + 4 * i, m);
  stream_store4(a.v + 4 * i, v);
  if (a.lowp) store_bf16x4(a.lowp + 4 * i, th);
}

__global__ void __launch_bounds__(EW_THREADS) adamw_kernel(const AdamArgs a) {
  size_t nv = a.n >> 2;  // every tensor starts and ends on a multiple of 4 elements (checked at create)
  size_t stride = (size_t)gridDim.x * EW_THREADS;
  // every value is touched once per step: streaming (non-temporal) loads and stores keep them out of the caches' way
  for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < nv; i += stride) {
    const float4 th = stream_load4(a.theta + 4 * i), g = stream_load4(a.grad + 4 * i);
    const float4 m = stream_load4(a.m + 4 * i), v = stream_load4(a.v + 4 * i);
    adam_apply4(a, i, th, g, m, v);
  }
}

// ---- outer step ----------------------------------------------------------------------------------------
struct OuterArgs {
  const float* in[DIPACO_MAX_PATHS_PER_MODULE];
  float alpha[DIPACO_MAX_PATHS_PER_MODULE];
  float* theta;
  float* buf;
  size_t n;
  int n_paths;
  int is_delta;
  float lr, mu;
};

__device__ __forceinline__ float4 outer_one(float4 th, float4 d, float4& b, float lr, float mu) {
  b.x = mu * b.x + d.x; b.y = mu * b.y + d.y; b.z = mu * b.z + d.z; b.w = mu * b.w + d.w;
  th.x -= lr * (d.x + mu * b.x); th.y -= lr * (d.y + mu * b.y);
  th.z -= lr * (d.z + mu * b.z); th.w -= lr * (d.w + mu * b.w);
  return th;
}

// NP > 0: path count known at compile time (loads of all inputs are issued together); NP = 0: runtime loop.
template <int NP>
__global__ void __launch_bounds__(EW_THREADS) outer_kernel(const OuterArgs a) {
  size_t nv = a.n >> 2;
  size_t stride = (size_t)gridDim.x * EW_THREADS;
  const int np = NP > 0 ? NP : a.n_paths;
  for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < nv; i += stride) {
    float4 th = stream_load4(a.theta + 4 * i);
    float4 b = stream_load4(a.buf + 4 * i);
    float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
    if (NP > 0) {
      float4 x[NP > 0 ? NP : 1];
#pragma unroll
      for (int p = 0; p < NP; ++p) x[p] = stream_load4(a.in[p] + 4 * i);
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        float al = a.alpha[p];
        if (a.is_delta) { d.x += al * x[p].x; d.y += al * x[p].y; d.z += al * x[p].z; d.w += al * x[p].w; }
        else { d.x += al * (th.x - x[p].x); d.y += al * (th.y - x[p].y); d.z += al * (th.z - x[p].z); d.w += al * (th.w - x[p].w); }
      }
    } else {
      for (int p = 0; p < np; ++p) {
        float4 x = stream_load4(a.in[p] + 4 * i);
        float al = a.alpha[p];
        if (a.is_delta) { d.x += al * x.x; d.y += al * x.y; d.z += al * x.z; d.w += al * x.w; }
        else { d.x += al * (th.x - x.x); d.y += al * (th.y - x.y); d.z += al * (th.z - x.z); d.w += al * (th.w - x.w); }
      }
    }
    th = outer_one(th, d, b, a.lr, a.mu);
    stream_store4(a.theta + 4 * i, th);
    stream_store4(a.buf + 4 * i, b);
  }
  if (blockIdx.x == 0 && threadIdx.x < (a.n & 3)) {  // tail elements
    size_t i = (nv << 2) + threadIdx.x;
    float th = a.theta[i], b = a.buf[i], d = 0.f;
    for (int p = 0; p < np; ++p) {
      float x = a.in[p][i];
      d += a.alpha[p] * (a.is_delta ? x : (th - x));
    }
    b = a.mu * b + d;
    a.theta[i] = th - a.lr * (d + a.mu * b);
    a.buf[i] = b;
  }
}

// ---- outer step of a table of modules ---------------------------------------------------------------------
// One workgroup takes chunks of OUTER_CHUNK elements; the module a chunk belongs to is found by bisection over
// the entries' first_chunk (workgroup-uniform).  Per thread four 16-byte vectors are in flight per input.
__global__ void __launch_bounds__(TABLE_THREADS) outer_table_kernel(const OuterTableEntry* __restrict__ entries,
                                                                 const float* const* __restrict__ inputs,
                                                                 const float* __restrict__ alpha, int n_modules,
                                                                 unsigned long long total_chunks, float lr, float mu) {
  constexpr int IT = OUTER_CHUNK / 4 / TABLE_THREADS;
  for (unsigned long long chunk = blockIdx.x; chunk < total_chunks; chunk += gridDim.x) {
    int lo = 0, hi = n_modules - 1;   // largest m with first_chunk[m] <= chunk
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (entries[mid].first_chunk <= chunk) lo = mid; else hi = mid - 1;
    }
    const OuterTableEntry e = entries[lo];
    const size_t local = chunk - e.first_chunk;
    const size_t nv = e.n_elems >> 2;
    const size_t i0 = local * (OUTER_CHUNK / 4) + threadIdx.x;
    const float* const* in = inputs + e.path_begin;
    const float* al = alpha + e.path_begin;
    float4 th[IT], b[IT], d[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const size_t i = i0 + (size_t)it * TABLE_THREADS;
      d[it] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < nv) {
        th[it] = stream_load4(e.theta + 4 * i);
        b[it] = stream_load4(e.momentum + 4 * i);
      }
    }
    for (int p = 0; p < e.n_paths; ++p) {
      const float* src = in[p];
      const float a = al[p];
      float4 x[IT];
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const size_t i = i0 + (size_t)it * TABLE_THREADS;
        x[it] = i < nv ? stream_load4(src + 4 * i) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        if (e.is_delta) {
          d[it].x += a * x[it].x; d[it].y += a * x[it].y; d[it].z += a * x[it].z; d[it].w += a * x[it].w;
        } else {
          d[it].x += a * (th[it].x - x[it].x); d[it].y += a * (th[it].y - x[it].y);
          d[it].z += a * (th[it].z - x[it].z); d[it].w += a * (th[it].w - x[it].w);
        }
      }
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const size_t i = i0 + (size_t)it * TABLE_THREADS;
      if (i < nv) {
        stream_store4(e.theta + 4 * i, outer_one(th[it], d[it], b[it], lr, mu));
        stream_store4(e.momentum + 4 * i, b[it]);
      }
    }
    // the up to three elements after the last whole vector belong to the module's last chunk
    const size_t last_chunk = (e.n_elems + OUTER_CHUNK - 1) / OUTER_CHUNK - 1;
    if (local == last_chunk && threadIdx.x < (e.n_elems & 3)) {
      const size_t i = (nv << 2) + threadIdx.x;
      const float t = e.theta[i];
      float bb = e.momentum[i], dd = 0.f;
      for (int p = 0; p < e.n_paths; ++p) dd += al[p] * (e.is_delta ? in[p][i] : (t - in[p][i]));
      bb = mu * bb + dd;
      e.theta[i] = t - lr * (dd + mu * bb);
      e.momentum[i] = bb;
    }
  }
}

// Streaming form of the outer step: sum <- (first ? 0 : sum) + w * (is_delta ? in : theta_prev - in), one path at a
// time as its result arrives; then the Nesterov update from the finished sum.
__global__ void __launch_bounds__(EW_THREADS) delta_accumulate_kernel(float* __restrict__ sum,
                                                                      const float* __restrict__ theta_prev,
                                                                      const float* __restrict__ in, float w, size_t n,
                                                                      int is_delta, int first) {
  const size_t nv = n >> 2;
  const size_t stride = (size_t)gridDim.x * EW_THREADS;
  for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < nv; i += stride) {
    float4 x = stream_load4(in + 4 * i);   // read once; the running sum is read again by the next call and stays cacheable
    if (!is_delta) {
      const float4 t = reinterpret_cast<const float4*>(theta_prev)[i];
      x = make_float4(t.x - x.x, t.y - x.y, t.z - x.z, t.w - x.w);
    }
    float4 a = first ? make_float4(0.f, 0.f, 0.f, 0.f) : reinterpret_cast<const float4*>(sum)[i];
    a.x += w * x.x; a.y += w * x.y; a.z += w * x.z; a.w += w * x.w;
    reinterpret_cast<float4*>(sum)[i] = a;
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const size_t i = (nv << 2) + threadIdx.x;
    const float x = is_delta ? in[i] : theta_prev[i] - in[i];
    sum[i] = (first ? 0.f : sum[i]) + w * x;
  }
}

// Delta = scale * sum;  buf <- mu buf + Delta;  theta <- theta - lr (Delta + mu buf)
__global__ void __launch_bounds__(EW_THREADS) outer_apply_kernel(float* __restrict__ theta, float* __restrict__ buf,
                                                                 const float* __restrict__ sum, float scale, size_t n,
                                                                 float lr, float mu) {
  const size_t nv = n >> 2;
  const size_t stride = (size_t)gridDim.x * EW_THREADS;
  for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < nv; i += stride) {
    float4 d = reinterpret_cast<const float4*>(sum)[i];
    d.x *= scale; d.y *= scale; d.z *= scale; d.w *= scale;
    float4 b = reinterpret_cast<const float4*>(buf)[i];
    const float4 th = outer_one(reinterpret_cast<const float4*>(theta)[i], d, b, lr, mu);
    reinterpret_cast<float4*>(theta)[i] = th;
    reinterpret_cast<float4*>(buf)[i] = b;
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const size_t i = (nv << 2) + threadIdx.x;
    const float d = scale * sum[i];
    const float b = mu * buf[i] + d;
    theta[i] = theta[i] - lr * (d + mu * b);
    buf[i] = b;
  }
}

template <typename T>
__global__ void __launch_bounds__(EW_THREADS) fill_kernel(T* p, T value, size_t n) {
  size_t stride = (size_t)gridDim.x * EW_THREADS;
  for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) p[i] = value;
}

}  // namespace

dipaco_status launch_copy_cast(const float* src, float* dst, bf16* lowp, size_t n, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  copy_cast_kernel<<<ew_blocks(n >> 2), EW_THREADS, 0, s>>>(src, dst, lowp, n);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_adamw(float* theta, const float* grad, float* m, float* v, bf16* lowp, const AdamLayout& lay,
                           size_t n, int64_t step, float lr, float beta1, float beta2, float eps, float wd,
                           hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  AdamArgs a;
  a.theta = theta; a.grad = grad; a.m = m; a.v = v; a.lowp = lowp; a.n = n;
  a.stem_end = lay.stem_end; a.blocks_end = lay.blocks_end; a.block_size = lay.block_size ? lay.block_size : 1;
  a.head_matrix = lay.head_matrix;
  for (int i = 0; i < 8; ++i) a.edge[i] = lay.edge[i];
  a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps; a.wd = wd;
  a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  adamw_kernel<<<ew_blocks(n >> 2), EW_THREADS, 0, s>>>(a);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_outer(float* theta, float* momentum, const float* const* inputs, const float* alpha,
                           int n_paths, size_t n, int is_delta, float lr, float mu, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  OuterArgs a;
  for (int p = 0; p < n_paths; ++p) { a.in[p] = inputs[p]; a.alpha[p] = alpha[p]; }
  for (int p = n_paths; p < DIPACO_MAX_PATHS_PER_MODULE; ++p) { a.in[p] = nullptr; a.alpha[p] = 0.f; }
  a.theta = theta; a.buf = momentum; a.n = n; a.n_paths = n_paths; a.is_delta = is_delta; a.lr = lr; a.mu = mu;
  const unsigned blocks = ew_blocks(n >> 2);
  switch (n_paths) {
    case 1: outer_kernel<1><<<blocks, EW_THREADS, 0, s>>>(a); break;
    case 2: outer_kernel<2><<<blocks, EW_THREADS, 0, s>>>(a); break;
    case 4: outer_kernel<4><<<blocks, EW_THREADS, 0, s>>>(a); break;
    case 8: outer_kernel<8><<<blocks, EW_THREADS, 0, s>>>(a); break;
    case 16: outer_kernel<16><<<blocks, EW_THREADS, 0, s>>>(a); break;
    default: outer_kernel<0><<<blocks, EW_THREADS, 0, s>>>(a); break;
  }
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_outer_table(const OuterTableEntry* entries, const float* const* inputs, const float* alpha,
                                 int n_modules, unsigned long long total_chunks, float lr, float mu, hipStream_t s) {
  if (n_modules <= 0 || total_chunks == 0) return DIPACO_OK;
  const unsigned blocks = (unsigned)std::min<unsigned long long>(total_chunks, 0x7fffffffull);   // one chunk per workgroup
  outer_table_kernel<<<blocks, TABLE_THREADS, 0, s>>>(entries, inputs, alpha, n_modules, total_chunks, lr, mu);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_delta_accumulate(float* sum, const float* theta_prev, const float* in, float w, size_t n,
                                      int is_delta, int first, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  delta_accumulate_kernel<<<ew_blocks((n >> 2) + 1), EW_THREADS, 0, s>>>(sum, theta_prev, in, w, n, is_delta, first);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_outer_apply(float* theta, float* momentum, const float* sum, float scale, size_t n, float lr,
                                 float mu, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  outer_apply_kernel<<<ew_blocks((n >> 2) + 1), EW_THREADS, 0, s>>>(theta, momentum, sum, scale, n, lr, mu);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_fill_f32(float* p, float value, size_t n, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  fill_kernel<float><<<ew_blocks(n), EW_THREADS, 0, s>>>(p, value, n);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_fill_i32(int* p, int value, size_t n, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  fill_kernel<int><<<ew_blocks(n), EW_THREADS, 0, s>>>(p, value, n);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_fill_i64(long long* p, long long value, size_t n, hipStream_t s) {
  if (n == 0) return DIPACO_OK;
  fill_kernel<long long><<<ew_blocks(n), EW_THREADS, 0, s>>>(p, value, n);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace dipaco
