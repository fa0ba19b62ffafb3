// Routing more often than once per document at evaluation (Section 2.4.3; appendix, "More frequent routing during
// evaluation").  Everything here works on the score array S_ijp = -nll[p][i][j] that the forward-only scoring pass
// leaves per path: running sums over the positions (fp64, so that window sums are differences of two of them), the
// window labels T_ij = argmax_p sum_{j..j+L-1} S_ijp that the token-level router is trained on, and the
// log-likelihood of documents whose chunks of W tokens are each scored by the path chosen for that chunk.
#include "common.h"
#include "kernels.h"

namespace dipaco {

namespace {

constexpr int SCAN_THREADS = 256;

// prefix[(p * B + b) * (S + 1) + j] = sum of nll[p][b][0 .. j), one workgroup per (p, b) row; positions are added in
// index order inside a thread's run and runs are combined left to right.
__global__ void __launch_bounds__(SCAN_THREADS) nll_prefix_kernel(const float* __restrict__ nll,
                                                                  double* __restrict__ prefix, int S) {
  __shared__ double run_sum[SCAN_THREADS];
  const size_t row = blockIdx.x;
  const float* src = nll + row * S;
  double* dst = prefix + row * (size_t)(S + 1);
  const int per = (S + SCAN_THREADS - 1) / SCAN_THREADS;
  const int lo = min(S, (int)threadIdx.x * per), hi = min(S, lo + per);
  double s = 0.0;
  for (int j = lo; j < hi; ++j) s += (double)src[j];
  run_sum[threadIdx.x] = s;
  __syncthreads();
  double before = 0.0;
  for (int t = 0; t < (int)threadIdx.x; ++t) before += run_sum[t];
  if (threadIdx.x == 0) dst[0] = 0.0;
  s = before;
  for (int j = lo; j < hi; ++j) {
    s += (double)src[j];
    dst[j + 1] = s;
  }
}

// targets[b][j] = argmin_p (prefix[p][b][min(S, j + L)] - prefix[p][b][j]), lowest p on ties
__global__ void __launch_bounds__(256) window_targets_kernel(const double* __restrict__ prefix, int* __restrict__ targets,
                                                             int P, int B, int S, int L) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long)B * S) return;
  const int b = (int)(i / S), j = (int)(i - (long)b * S);
  const int e = (int)min((long)S, (long)j + L);
  double best = 0.0;
  int arg = 0;
  for (int p = 0; p < P; ++p) {
    const double* row = prefix + ((size_t)p * B + b) * (size_t)(S + 1);
    const double w = row[e] - row[j];
    if (p == 0 || w < best) { best = w; arg = p; }
  }
  targets[i] = arg;
}

// out[b] = -sum over chunks c of (prefix[choice[b][c]][b][end_c] - prefix[choice[b][c]][b][c W]); one thread per document
__global__ void __launch_bounds__(256) chunk_score_kernel(const double* __restrict__ prefix, const int* __restrict__ choice,
                                                          float* __restrict__ out, int P, int B, int S, int W) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= B) return;
  const int n_chunks = (S + W - 1) / W;
  double s = 0.0;
  for (int c = 0; c < n_chunks; ++c) {
    int p = choice[(size_t)b * n_chunks + c];
    p = min(max(p, 0), P - 1);
    const double* row = prefix + ((size_t)p * B + b) * (size_t)(S + 1);
    s += row[min(S, (c + 1) * W)] - row[c * W];
  }
  out[b] = (float)(-s);
}

}  // namespace

size_t reroute_prefix_doubles(int P, int B, int S) { return (size_t)P * B * (size_t)(S + 1); }

dipaco_status launch_window_targets(const float* nll, int P, int B, int S, int L, int* targets, double* prefix,
                                    hipStream_t s) {
  nll_prefix_kernel<<<(unsigned)(P * B), SCAN_THREADS, 0, s>>>(nll, prefix, S);
  DIPACO_LAUNCH_CHECK();
  const long n = (long)B * S;
  window_targets_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(prefix, targets, P, B, S, L);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

dipaco_status launch_chunk_score(const float* nll, const int* choice, int P, int B, int S, int W, float* out,
                                 double* prefix, hipStream_t s) {
  nll_prefix_kernel<<<(unsigned)(P * B), SCAN_THREADS, 0, s>>>(nll, prefix, S);
  DIPACO_LAUNCH_CHECK();
  chunk_score_kernel<<<(unsigned)((B + 255) / 256), 256, 0, s>>>(prefix, choice, out, P, B, S, W);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace dipaco
