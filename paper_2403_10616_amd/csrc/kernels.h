// Host-side launchers of every kernel in libdipaco (one per .hip file group).  All enqueue on `s` and return.
#pragma once
#include "common.h"

namespace dipaco {

struct SumBatch;   // deferred fixed-order reductions, see transformer.hip below

// ---- elementwise.hip ---------------------------------------------------------------------------------
dipaco_status launch_copy_cast(const float* src, float* dst, bf16* lowp, size_t n, hipStream_t s);
// where weight decay applies in the flat path buffer: [0, stem_end) all; blocks of block_size elements up to
// blocks_end, decayed between in-block edges 0-1, 2-3, 4-5, 6-7; in the head from head_matrix on.
struct AdamLayout {
  unsigned long long stem_end, blocks_end, block_size, head_matrix;
  unsigned int edge[8];
};
dipaco_status launch_adamw(float* theta, const float* grad, float* m, float* v, bf16* lowp, const AdamLayout& lay,
                           size_t n, int64_t step, float lr, float beta1, float beta2, float eps, float wd,
                           hipStream_t s);
dipaco_status launch_outer(float* theta, float* momentum, const float* const* inputs, const float* alpha,
                           int n_paths, size_t n, int is_delta, float lr, float mu, hipStream_t s);
// streaming outer step: sum <- (first ? 0 : sum) + w * (is_delta ? in : theta_prev - in);  then
// Delta = scale * sum, momentum <- mu momentum + Delta, theta <- theta - lr (Delta + mu momentum)
dipaco_status launch_delta_accumulate(float* sum, const float* theta_prev, const float* in, float w, size_t n,
                                      int is_delta, int first, hipStream_t s);
dipaco_status launch_outer_apply(float* theta, float* momentum, const float* sum, float scale, size_t n, float lr,
                                 float mu, hipStream_t s);
// One entry of the device-resident module table of the table-driven outer step; chunks of OUTER_CHUNK elements
// are the unit of work, first_chunk the running sum of the chunk counts of the entries before.
constexpr size_t OUTER_CHUNK = 4096;
struct OuterTableEntry {
  float* theta;
  float* momentum;
  unsigned long long n_elems;
  unsigned long long first_chunk;
  unsigned long long path_begin;   // index of the module's first input pointer / weight in the table's flat arrays
  int n_paths;
  int is_delta;
};
dipaco_status launch_outer_table(const OuterTableEntry* entries, const float* const* inputs, const float* alpha,
                                 int n_modules, unsigned long long total_chunks, float lr, float mu, hipStream_t s);
dipaco_status launch_fill_f32(float* p, float value, size_t n, hipStream_t s);
dipaco_status launch_fill_i32(int* p, int value, size_t n, hipStream_t s);
dipaco_status launch_fill_i64(long long* p, long long value, size_t n, hipStream_t s);

// ---- route.hip ---------------------------------------------------------------------------------------
// z row n at z + n * ldz;  n_best = 1: idx [N];  n_best = 2: idx [N, 2] (best, second best; -1 if K = 1), hist
// counts both memberships
// lin_bias (nullable): linear router -- c holds the K weight rows and the score minimised is -(c_k.z_n + lin_bias[k])
dipaco_status launch_route(const float* z, int64_t ldz, const float* c, const float* lin_bias, int64_t N, int D, int K,
                           int n_best, int* idx, long long* hist, float* margin, hipStream_t s);
// logits [rows, K] fp32 -> nll[rows] and, in place, (softmax - onehot(label)) * inv_n; labels outside [0, K): zeros
dipaco_status launch_logistic_rows(float* logits, const int* labels, int64_t rows, int K, float inv_n, float* nll,
                                   hipStream_t s);

// ---- reroute.hip -------------------------------------------------------------------------------------
// nll: [P, B, S] per-position negative log-likelihoods of B documents under P paths; prefix: scratch of
// reroute_prefix_doubles(P, B, S) doubles.
size_t reroute_prefix_doubles(int P, int B, int S);
// targets[b, j] = argmin_p sum of nll[p, b, j .. min(S, j + L) - 1], lowest p on ties
dipaco_status launch_window_targets(const float* nll, int P, int B, int S, int L, int* targets, double* prefix,
                                    hipStream_t s);
// out[b] = -sum over chunks c of W positions of the nll of path choice[b, c] on that chunk (choice clamped to [0, P))
dipaco_status launch_chunk_score(const float* nll, const int* choice, int P, int B, int S, int W, float* out,
                                 double* prefix, hipStream_t s);

// ---- kmeans.hip --------------------------------------------------------------------------------------
// order[0..n) = the indices 0..n-1 stably sorted by keys[i] (clamped to [0, n_keys), n_keys <= 65536);
// scratch: sort_scratch_ints(n, n_keys) ints
size_t sort_scratch_ints(long n, int n_keys);
dipaco_status launch_stable_sort_indices(const int* keys, long n, int n_keys, int* order, int* scratch, hipStream_t s);
// start[k] = number of keys below k, k = 0..n_keys (count: [n_keys] scratch; chunk_start: nullable, [n_keys + 1])
dipaco_status launch_key_offsets(const int* keys, long n, int n_keys, int* count, int* start, int* chunk_start,
                                 hipStream_t s);
// centroids[k] <- mean of the rows z[n] (row stride ldz) with idx[n] = k, in a fixed summation order; clusters
// without rows keep their centroid.  counts (nullable): rows per cluster.
size_t kmeans_workspace_bytes(long N, int D, int K);
dipaco_status launch_kmeans_update(const float* z, long ldz, const int* idx, long N, int D, int K, float* centroids,
                                   long long* counts, void* workspace, hipStream_t s);

// ---- gemm.hip ----------------------------------------------------------------------------------------
// C[M,N] = opA(A) . opB(B)  (+ epilogue), fp32 accumulation on the matrix cores.
//   trans_a = 0: A is [M,K] row-major (lda);  1: A is [K,M] row-major (lda)
//   trans_b = 0: B is [K,N] row-major (ldb);  1: B is [N,K] row-major (ldb)
// Epilogue (all optional, applied in this order): + bias[n];  act = 1: aux_out = value, value = GELU(value);
// act = 2: value *= GELU'(aux_in);  act = 3: aux_out = GELU'(value), value = GELU(value);  act = 4: value *= aux_in;
// + resid[m,n].  aux and resid have row stride ldc.  (The path step uses the pair 3 / 4: the forward pass leaves the
// derivative itself, which it gets almost for free beside GELU, and the backward epilogue is one multiplication.)
// out_f32 = 1 writes fp32 (used for weight gradients), else T.
// splits > 1 (only with out_f32 and no epilogue): K is cut into `splits` ranges whose partial products go to
// `partial` ([splits, M, N] fp32) and are then summed in index order.
struct GemmArgs {
  const void* A; const void* B; void* C;
  int M, N, K;
  long lda, ldb, ldc;
  const void* bias;
  const void* resid;
  void* aux_out;
  const void* aux_in;
  int act;
  int trans_a, trans_b;
  int out_f32;
  int splits;
  float* partial;
  // optional: colsum[n] = sum over m of the values written to C (before rounding to C's type), fp32, fixed order;
  // colsum_partial = gemm_colsum_partial_floats(M, N) floats of scratch.  Not with split-K.
  float* colsum = nullptr;
  float* colsum_partial = nullptr;
  SumBatch* sum_batch = nullptr;   // where the final sum of colsum_partial is deferred to (nullptr: summed at once)
};
size_t gemm_colsum_partial_floats(int M, int N);
template <typename T> dipaco_status launch_gemm(const GemmArgs& g, hipStream_t s);
// gemm_dlds.hip: bf16, 256x256 tiles loaded from global memory straight into LDS; takes the shapes for which
// gemm_dlds_eligible holds (whole K tiles of 32, 16-byte rows); launch_gemm routes to it by itself
bool gemm_dlds_eligible(const GemmArgs& g);
dipaco_status launch_gemm_dlds(const GemmArgs& g, hipStream_t s);
void set_gemm_dlds_shape(int shape);   // 0 = automatic, 1 = 256 x 256, 2 = 256 x 128, 3 / 4 = 128 x 512 / 512 x 128 for weight gradients, 5 = 224-column tiles where N % 224 == 0
// C[m, n] = sum over z < splits of partial[z, m, n], in index order
dipaco_status launch_splitk_reduce(const float* partial, float* C, int M, int N, long ldc, int splits, hipStream_t s);
// 0 = automatic; 1 = 128x128, 2 = 256x128, 3 / 4 = 256x256 workgroup tiles with four / eight waves, 5 = the
// direct-to-LDS kernel wherever the shape allows, 6 / 7 / 8 / 9 / 10 = the same with its 256x256 / 256x128 / 128x512 / 512x128 (these two: weight gradients) / 224-column shape forced
// (tuning and tests)
void set_gemm_tile(int t);
// the same where the number of slices depends on the tile class of the element:
// n_slices[(row >= row_edge) + 2 * (col >= col_edge)]
dipaco_status launch_splitk_reduce_classes(const float* partial, float* C, int M, int N, long ldc, int row_edge,
                                           int col_edge, const int (&n_slices)[4], hipStream_t s);
// direct-to-LDS kernel: slices of a full tile in its uneven split-K plan with at most max_slices, 0 if it has none
// (for the tile shape in force, or the larger count over both shapes)
int gemm_dlds_plan_slices(int M, int N, int K, int max_slices, bool any_shape);
void gemm_dlds_plan_info(int M, int N, int K, int max_slices, int* out);   // host-only, for tests: see gemm_dlds.hip
constexpr int GEMM_SLICE_CAP = 32;
// split count the weight-gradient products are launched with
int gemm_plan_splits(int M, int N, int K, bool bf16_operands);
int gemm_max_splits(int M, int N, int K);    // its upper bound over tile settings (workspace sizing)

// ---- transformer.hip ---------------------------------------------------------------------------------
template <typename T>
dipaco_status launch_embed(const T* tok_emb, const T* pos_emb, const int* tokens, T* x, int B, int S, int d,
                           int vocab, hipStream_t s);
template <typename T>
dipaco_status launch_layernorm_fwd(const T* x, const T* g, const T* b, T* y, float* mean, float* rstd, int rows,
                                   int d, float eps, hipStream_t s);
// dx = resid_grad (nullable) + LN backward of dy;  dg/db fp32 via `partial` ([ln_bwd_partial_floats] scratch);
// dcol (nullable) = column sums of dx as stored: the bias gradient of the linear layer that dx is the output gradient of.
template <typename T>
dipaco_status launch_layernorm_bwd(const T* dy, const T* x, const T* g, const float* mean, const float* rstd,
                                   const T* resid_grad, T* dx, float* dg, float* db, float* dcol, float* partial,
                                   int rows, int d, hipStream_t s, SumBatch* batch = nullptr);
size_t ln_bwd_partial_floats(int rows, int d);
// Fixed-order sums of rows of partial results (column sums of a product's output, LayerNorm parameter gradients):
//   column c of sum over p < n_partials of partial[p * stride + c] goes to out0 / out1 / out2 by c / d (a null output
//   is skipped).
// A producer hands its reduction to a SumBatch when the caller gives it one: the path step collects the 49
// reductions of its backward pass and runs them as one launch at the end (each on a partial buffer of its own)
// instead of 49 launches of a few microseconds between the big kernels.
struct SumJob {
  const float* partial;
  float* out0; float* out1; float* out2;
  int n_partials, stride, d;
};
constexpr int SUM_BATCH_MAX = 64;   // 64 jobs of 48 bytes travel as kernel arguments
struct SumBatch {
  SumJob job[SUM_BATCH_MAX];
  int count = 0;
};
// runs the reduction now (batch == nullptr) or appends it to the batch (a full batch is flushed first)
dipaco_status sum_partials(const float* partial, float* out0, float* out1, float* out2, int n_partials, int stride,
                           int d, SumBatch* batch, hipStream_t s);
dipaco_status flush_sum_batch(SumBatch& batch, hipStream_t s);
// out[c] = sum over p < n_partials of partial[p * cols + c], fixed order
dipaco_status launch_sum_rows(const float* partial, float* out, int n_partials, int cols, hipStream_t s,
                              SumBatch* batch = nullptr);
// out[n] = sum_m x[m,n] (fp32, fixed order);  partial: colsum_partial_floats scratch
template <typename T>
dipaco_status launch_colsum(const T* x, float* out, float* partial, int rows, int cols, hipStream_t s);
size_t colsum_partial_floats(int rows, int cols);
// out[b, :] (fp32) = mean over positions of x[b*S + p, :]
template <typename T> dipaco_status launch_mean_pool(const T* x, float* out, int B, int S, int d, hipStream_t s);
// out[b] = -sum_p nll[b*S + p]
dipaco_status launch_doc_score(const float* nll, float* out, int B, int S, hipStream_t s);
// n_valid[0] = #targets >= 0
dipaco_status launch_count_valid(const int* targets, int n, int* n_valid, hipStream_t s);
// logits [rows, V] (T) -> nll[rows] fp32 and, when want_grad, in place dlogits = (softmax - onehot)/n_valid (0 on
// ignored rows); without want_grad the logits are only read (n_valid is then not used)
template <typename T>
dipaco_status launch_softmax_xent(T* logits, const int* targets, const int* n_valid, float* nll, int rows, int V,
                                  bool want_grad, hipStream_t s);
// loss = sum(nll) / n_valid, fixed-order tree
dipaco_status launch_mean_loss(const float* nll, const int* n_valid, float* loss, int rows, hipStream_t s);
// token/position embedding gradients (deterministic).  ints: embed_bwd_scratch_ints(rows, vocab) scratch.
template <typename T>
dipaco_status launch_embed_bwd(const T* dx, const int* tokens, float* d_tok, float* d_pos, int* scratch, int B,
                               int S, int d, int vocab, int max_seq, hipStream_t s);
size_t embed_bwd_scratch_ints(int rows, int vocab);

// ---- attention.hip -----------------------------------------------------------------------------------
// qkv: [B*S, 3A] (q | k | v, head h at columns h*dh), o: [B*S, A], lse: [B, H, S] fp32.
template <typename T>
dipaco_status launch_attention_fwd(const T* qkv, T* o, float* lse, int B, int S, int H, int dh, hipStream_t s);
// dqkv: [B*S, 3A];  dscratch: fp32 scratch of 2 * B * H * roundup(S, 128) floats (per-query statistics);
// colsum_out (nullable): fp32 [3A] = column sums of dqkv in a fixed order, with colsum_partial =
// attention_bwd_colsum_floats(B, S, H, dh) floats of scratch
template <typename T>
dipaco_status launch_attention_bwd(const T* qkv, const T* o, const T* d_o, const float* lse, T* dqkv,
                                   float* dscratch, float* colsum_out, float* colsum_partial, int B, int S, int H,
                                   int dh, hipStream_t s, SumBatch* batch = nullptr);
size_t attention_bwd_colsum_floats(int B, int S, int H, int dh);

// ---- probe.hip: register-only instruction-issue loops (measurement aid) --------------------------------
constexpr int ISSUE_PROBE_BLOCKS = 256;   // one workgroup per compute unit
// out: ISSUE_PROBE_BLOCKS * 256 * waves_per_simd floats
dipaco_status launch_issue_probe(int mode, int waves_per_simd, int iters, float* out, hipStream_t s);

// ---- attention_mfma.hip: bf16, head size 64, matrix cores ---------------------------------------------
dipaco_status launch_attention_fwd_mfma(const bf16* qkv, bf16* o, float* lse, int B, int S, int H, hipStream_t s);
// colsum_out (nullable): fp32 [3 H 64], the column sums of dqkv (the bias gradient of the QKV projection), from the
// kernels' epilogues; colsum_partial: attention_colsum_partial_floats(B, S, H) floats of scratch
dipaco_status launch_attention_bwd_mfma(const bf16* qkv, const bf16* o, const bf16* d_o, const float* lse, bf16* dqkv,
                                        float* dsum, float* colsum_out, float* colsum_partial, int B, int S, int H,
                                        hipStream_t s, SumBatch* batch = nullptr);
size_t attention_colsum_partial_floats(int B, int S, int H);
// 0: a workgroup takes a long and a short block of the causal triangle; 1: one block per workgroup, longest first
void set_attention_single_block(int on);

}  // namespace dipaco
