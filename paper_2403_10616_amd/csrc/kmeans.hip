// k-means update step (the "fit" half of generative routing): every centroid becomes the mean of the points
// assigned to it; a centroid without points keeps its value.  Sums are formed in a fixed order, so the result is
// bit-reproducible: points are first put in cluster order by a stable counting sort (integer work only), then each
// cluster's rows are added in chunks of KM_CHUNK rows whose partial sums are added in chunk order.
//
// Also here: the stable sort itself (least-significant-digit radix sort on 8-bit digits of an int key, carrying the
// element's index), which the token-embedding gradient uses to group positions by token id.
#include "kernels.h"

namespace dipaco {

namespace {

constexpr int SORT_BLOCK = 2048;   // keys per workgroup
constexpr int KM_CHUNK = 512;      // rows per partial sum
constexpr int KM_COLS = 1024;      // columns per workgroup (4 float4 per lane)

__device__ __forceinline__ int clamp_key(int k, int n_keys) { return k < 0 ? 0 : (k >= n_keys ? n_keys - 1 : k); }

// block_hist[b][d] = number of keys of block b whose digit is d
__global__ void __launch_bounds__(256) sort_hist_kernel(const int* __restrict__ keys, int n, int n_keys, int shift,
                                                        int* __restrict__ block_hist) {
  __shared__ int h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int base = blockIdx.x * SORT_BLOCK;
  for (int i = threadIdx.x; i < SORT_BLOCK; i += 256) {
    const int j = base + i;
    if (j < n) atomicAdd(&h[(clamp_key(keys[j], n_keys) >> shift) & 255], 1);
  }
  __syncthreads();
  block_hist[blockIdx.x * 256 + threadIdx.x] = h[threadIdx.x];
}

// block_hist[b][d] <- first output slot of block b's keys with digit d (digits in order, blocks in order inside a digit)
__global__ void __launch_bounds__(256) sort_scan_kernel(int* __restrict__ block_hist, int nblocks) {
  __shared__ int total[256];
  const int d = threadIdx.x;
  int run = 0;
  for (int b0 = 0; b0 < nblocks; b0 += 16) {   // 16 independent loads in flight, then the running sum
    int t[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) t[i] = b0 + i < nblocks ? block_hist[(b0 + i) * 256 + d] : 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (b0 + i < nblocks) block_hist[(b0 + i) * 256 + d] = run;
      run += t[i];
    }
  }
  total[d] = run;
  __syncthreads();
  int start = 0;
  for (int e = 0; e < d; ++e) start += total[e];
  if (start)
    for (int b = 0; b < nblocks; ++b) block_hist[b * 256 + d] += start;
}

// One wave per block walks its keys 64 at a time, in order.  Lanes holding the same digit find each other with eight
// ballots; a lane's slot is the digit's running counter plus the number of such lanes below it: a stable order.
__global__ void __launch_bounds__(64) sort_scatter_kernel(const int* __restrict__ keys_in, const int* __restrict__ vals_in,
                                                          int n, int n_keys, int shift, const int* __restrict__ block_base,
                                                          int* __restrict__ keys_out, int* __restrict__ vals_out) {
  __shared__ int cnt[256];
  const int lane = threadIdx.x;
  for (int d = lane; d < 256; d += 64) cnt[d] = block_base[blockIdx.x * 256 + d];
  __syncthreads();
  const int base = blockIdx.x * SORT_BLOCK;
  for (int i = 0; i < SORT_BLOCK; i += 64) {
    const int j = base + i + lane;
    const bool live = j < n;
    const int key = live ? clamp_key(keys_in[j], n_keys) : 0;
    const int digit = (key >> shift) & 255;
    unsigned long long same = __builtin_amdgcn_ballot_w64(live);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const unsigned long long set = __builtin_amdgcn_ballot_w64(live && ((digit >> b) & 1));
      same &= ((digit >> b) & 1) ? set : ~set;
    }
    if (live) {
      const int below = __builtin_popcountll(same & ((1ull << lane) - 1ull));
      const int slot = cnt[digit] + below;
      if (keys_out) keys_out[slot] = key;
      vals_out[slot] = vals_in ? vals_in[j] : j;
    }
    __syncthreads();   // everybody has read the counters
    if (live && (same >> lane) == 1ull) cnt[digit] += __builtin_popcountll(same);   // the highest lane of each group
    __syncthreads();
  }
}

// count[k] = number of keys equal to k (integer atomics: the result does not depend on their order)
// LDS: a workgroup counts KC_BLOCK keys in LDS first (n_keys <= KC_MAX_LDS) and adds only its non-zero bins.
constexpr int KC_BLOCK = 8192, KC_MAX_LDS = 36864;   // 144 KB of counters at most
template <bool LDS>
__global__ void __launch_bounds__(256) key_count_kernel(const int* __restrict__ keys, long n, int n_keys,
                                                        int* __restrict__ count) {
  extern __shared__ int h[];   // LDS: n_keys counters
  if (LDS) {
    for (int k = threadIdx.x; k < n_keys; k += 256) h[k] = 0;
    __syncthreads();
  }
  const long base = (long)blockIdx.x * KC_BLOCK;
  for (int i = threadIdx.x; i < KC_BLOCK; i += 256) {
    const long j = base + i;
    if (j < n) atomicAdd(LDS ? &h[clamp_key(keys[j], n_keys)] : &count[clamp_key(keys[j], n_keys)], 1);
  }
  if (LDS) {
    __syncthreads();
    for (int k = threadIdx.x; k < n_keys; k += 256)
      if (h[k]) atomicAdd(&count[k], h[k]);
  }
}

// start[k] = sum of count[0..k), k = 0..n_keys; chunk_start[k] = sum over k' < k of ceil(count[k'] / KM_CHUNK).
// One workgroup: every thread sums a run of consecutive keys, the 1024 run totals are scanned in LDS, then every
// thread walks its run again.
__global__ void __launch_bounds__(1024) key_scan_kernel(const int* __restrict__ count, int n_keys, int* __restrict__ start,
                                                        int* __restrict__ chunk_start) {
  __shared__ int run_sum[1024], run_chunks[1024];
  const int per = (n_keys + 1023) / 1024;
  const int k0 = min(threadIdx.x * per, n_keys), k1 = min(k0 + per, n_keys);
  int s = 0, ch = 0;
  for (int k = k0; k < k1; ++k) { const int c = count[k]; s += c; ch += (c + KM_CHUNK - 1) / KM_CHUNK; }
  run_sum[threadIdx.x] = s;
  run_chunks[threadIdx.x] = ch;
  __syncthreads();
  if (threadIdx.x < 64) {   // exclusive scan of the 1024 run totals: 16 per lane, then across the wave
    const int lane = threadIdx.x;
    int a[16], b[16], ta = 0, tb = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) { a[i] = run_sum[16 * lane + i]; b[i] = run_chunks[16 * lane + i]; ta += a[i]; tb += b[i]; }
    int ia = ta, ib = tb;   // inclusive scan over the lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int ua = __shfl_up(ia, o, 64), ub = __shfl_up(ib, o, 64);
      if (lane >= o) { ia += ua; ib += ub; }
    }
    int ea = ia - ta, eb = ib - tb;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      run_sum[16 * lane + i] = ea; run_chunks[16 * lane + i] = eb;
      ea += a[i]; eb += b[i];
    }
    if (lane == 63) {
      start[n_keys] = ia;
      if (chunk_start) chunk_start[n_keys] = ib;
    }
  }
  __syncthreads();
  s = run_sum[threadIdx.x];
  ch = run_chunks[threadIdx.x];
  for (int k = k0; k < k1; ++k) {
    start[k] = s;
    if (chunk_start) chunk_start[k] = ch;
    const int c = count[k];
    s += c;
    ch += (c + KM_CHUNK - 1) / KM_CHUNK;
  }
}

__global__ void __launch_bounds__(256) fill_int_kernel2(int* p, int v, long n) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// partial[chunk][col] = sum of the chunk's rows, rows in sorted order: wave w adds rows w, w+4, ...; the four wave
// sums are added in wave order.  Workgroup (x, y): chunk x, columns [KM_COLS y, KM_COLS (y+1)).
__global__ void __launch_bounds__(256) kmeans_partial_kernel(const float* __restrict__ z, long ldz,
                                                             const int* __restrict__ order, const int* __restrict__ start,
                                                             const int* __restrict__ chunk_start, int K, int D,
                                                             float* __restrict__ partial) {
  __shared__ float red[4][KM_COLS];
  const int chunk = blockIdx.x;
  if (chunk >= chunk_start[K]) return;   // uniform
  int lo = 0, hi = K;                    // last k with chunk_start[k] <= chunk
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (chunk_start[mid] <= chunk) lo = mid; else hi = mid;
  }
  const int k = lo;
  const int r0 = start[k] + (chunk - chunk_start[k]) * KM_CHUNK;
  const int r1 = min(r0 + KM_CHUNK, start[k + 1]);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = blockIdx.y * KM_COLS;
  float4 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) acc[t] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int r = r0 + wave; r < r1; r += 4) {
    const float* row = z + (long)order[r] * ldz;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int c = c0 + 4 * (lane + 64 * t);
      if (c < D) {
        const float4 v = *reinterpret_cast<const float4*>(row + c);
        acc[t].x += v.x; acc[t].y += v.y; acc[t].z += v.z; acc[t].w += v.w;
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) *reinterpret_cast<float4*>(&red[wave][4 * (lane + 64 * t)]) = acc[t];
  __syncthreads();
  for (int c = threadIdx.x; c < KM_COLS && c0 + c < D; c += 256)
    partial[(long)chunk * D + c0 + c] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
}

// centroid k <- (sum of its chunks' partial sums, in chunk order) / count; untouched when the count is 0
__global__ void __launch_bounds__(256) kmeans_finish_kernel(const float* __restrict__ partial,
                                                            const int* __restrict__ start,
                                                            const int* __restrict__ chunk_start, int D,
                                                            float* __restrict__ centroids, long long* __restrict__ counts) {
  const int k = blockIdx.x;
  const int n = start[k + 1] - start[k];
  if (threadIdx.x == 0 && blockIdx.y == 0 && counts) counts[k] = n;
  if (n == 0) return;
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c >= D) return;
  float s = 0.f;
  for (int ch = chunk_start[k]; ch < chunk_start[k + 1]; ++ch) s += partial[(long)ch * D + c];
  centroids[(long)k * D + c] = (float)((double)s / (double)n);
}

}  // namespace

size_t sort_scratch_ints(long n, int n_keys) {
  const long nblocks = (n + SORT_BLOCK - 1) / SORT_BLOCK;
  const size_t two_pass = n_keys > 256 ? 2 * (size_t)n : 0;   // keys and indices after the first pass
  return (size_t)nblocks * 256 + two_pass;
}

// order[0..n): the indices 0..n-1, stably sorted by keys[i] clamped to [0, n_keys); n_keys <= 65536.
dipaco_status launch_stable_sort_indices(const int* keys, long n, int n_keys, int* order, int* scratch, hipStream_t s) {
  if (n <= 0) return DIPACO_OK;
  if (n > 0x7fffffffL - SORT_BLOCK) return fail(DIPACO_ESHAPE, "sort: too many elements");
  if (n_keys < 1 || n_keys > 65536) return fail(DIPACO_ESHAPE, "sort: key range must be 1..65536");
  const int nblocks = (int)((n + SORT_BLOCK - 1) / SORT_BLOCK);
  int* block_hist = scratch;
  int* keys_a = scratch + (size_t)nblocks * 256;
  int* vals_a = keys_a + n;
  const bool two = n_keys > 256;
  sort_hist_kernel<<<nblocks, 256, 0, s>>>(keys, (int)n, n_keys, 0, block_hist);
  DIPACO_LAUNCH_CHECK();
  sort_scan_kernel<<<1, 256, 0, s>>>(block_hist, nblocks);
  DIPACO_LAUNCH_CHECK();
  sort_scatter_kernel<<<nblocks, 64, 0, s>>>(keys, nullptr, (int)n, n_keys, 0, block_hist, two ? keys_a : nullptr,
                                             two ? vals_a : order);
  DIPACO_LAUNCH_CHECK();
  if (two) {
    sort_hist_kernel<<<nblocks, 256, 0, s>>>(keys_a, (int)n, n_keys, 8, block_hist);
    DIPACO_LAUNCH_CHECK();
    sort_scan_kernel<<<1, 256, 0, s>>>(block_hist, nblocks);
    DIPACO_LAUNCH_CHECK();
    sort_scatter_kernel<<<nblocks, 64, 0, s>>>(keys_a, vals_a, (int)n, n_keys, 8, block_hist, nullptr, order);
    DIPACO_LAUNCH_CHECK();
  }
  return DIPACO_OK;
}

// start[k] = number of keys below k (k = 0..n_keys); chunk_start (nullable): see key_scan_kernel; count: [n_keys] scratch
dipaco_status launch_key_offsets(const int* keys, long n, int n_keys, int* count, int* start, int* chunk_start,
                                 hipStream_t s) {
  fill_int_kernel2<<<(n_keys + 255) / 256, 256, 0, s>>>(count, 0, n_keys);
  DIPACO_LAUNCH_CHECK();
  if (n > 0) {
    const unsigned blocks = (unsigned)((n + KC_BLOCK - 1) / KC_BLOCK);
    if (n_keys <= KC_MAX_LDS) {
      static std::atomic<unsigned long long> lds_set{0};
      if (dipaco_status st = ensure_dynamic_lds(reinterpret_cast<const void*>(key_count_kernel<true>), KC_MAX_LDS * (int)sizeof(int), lds_set)) return st;
      key_count_kernel<true><<<blocks, 256, (size_t)n_keys * sizeof(int), s>>>(keys, n, n_keys, count);
    } else {
      key_count_kernel<false><<<blocks, 256, 0, s>>>(keys, n, n_keys, count);
    }
    DIPACO_LAUNCH_CHECK();
  }
  key_scan_kernel<<<1, 1024, 0, s>>>(count, n_keys, start, chunk_start);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

static size_t km_max_chunks(long N, int K) { return (size_t)(N / KM_CHUNK) + (size_t)K; }

size_t kmeans_workspace_bytes(long N, int D, int K) {
  const size_t ints = (size_t)N /*order*/ + sort_scratch_ints(N, K) + (size_t)K /*count*/ + 2 * ((size_t)K + 1);
  const size_t ints_padded = (ints + 3) / 4 * 4;   // keep the float part 16-byte aligned
  return ints_padded * 4 + km_max_chunks(N, K) * (size_t)D * 4;
}

dipaco_status launch_kmeans_update(const float* z, long ldz, const int* idx, long N, int D, int K, float* centroids,
                                   long long* counts, void* workspace, hipStream_t s) {
  int* order = static_cast<int*>(workspace);
  int* sort_scratch = order + N;
  int* count = sort_scratch + sort_scratch_ints(N, K);
  int* start = count + K;
  int* chunk_start = start + K + 1;
  const size_t ints = (size_t)N + sort_scratch_ints(N, K) + (size_t)K + 2 * ((size_t)K + 1);
  float* partial = reinterpret_cast<float*>(static_cast<int*>(workspace) + (ints + 3) / 4 * 4);
  dipaco_status st = launch_key_offsets(idx, N, K, count, start, chunk_start, s);
  if (st != DIPACO_OK) return st;
  st = launch_stable_sort_indices(idx, N, K, order, sort_scratch, s);
  if (st != DIPACO_OK) return st;
  if (N > 0) {
    dim3 grid((unsigned)km_max_chunks(N, K), (unsigned)((D + KM_COLS - 1) / KM_COLS));
    kmeans_partial_kernel<<<grid, 256, 0, s>>>(z, ldz, order, start, chunk_start, K, D, partial);
    DIPACO_LAUNCH_CHECK();
  }
  dim3 fgrid((unsigned)K, (unsigned)((D + 255) / 256));
  kmeans_finish_kernel<<<fgrid, 256, 0, s>>>(partial, start, chunk_start, D, centroids, counts);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace dipaco
