/*
 * dipaco.h - C ABI of libdipaco.so: the data-parallel hot path of DiPaCo (arXiv 2403.10616) on one
 * MI355X (gfx950).  One path = one decoder-only transformer LM assembled from one module per level of the
 * module grid (Section 2.3, Section 2.6); the library runs its inner step (Algorithm 1, inner loop: loss,
 * gradient, AdamW), the per-module outer step (Algorithm 1, outer loop, with the shard-size weights of
 * Section 2.7) and k-means prefix routing (Section 2.4.1, eq. 1).
 *
 * Conventions common to every call
 *   - Every "device" pointer is HIP device memory owned by the caller; "host" pointers are ordinary host
 *     memory read during the call only.  The library allocates and frees no device memory, in any call: scratch
 *     comes from the caller's workspace arguments (one entry point uses a fixed device array instead, see
 *     dipaco_path_prefix_features_static).  It keeps no numerical state between calls: optimiser moments,
 *     momentum and step counters are arguments.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls validate every argument
 *     and shape on the host first, then enqueue kernels on that stream and return without synchronising.
 *     DIPACO_EINVAL / ESHAPE / EALIGN / EWORKSPACE / EUNSUPPORTED mean that nothing was enqueued.  DIPACO_EHIP
 *     reports a failure of the HIP runtime itself (a launch or attribute call): kernels of the same call that
 *     were enqueued before it still run, and the call's outputs are then undefined.  dipaco_last_error()
 *     describes the last failure (per host thread).
 *   - Thread safety: calls may be made from several host threads.  The dipaco_k_set_* switches of
 *     dipaco_kernels.h are process-wide test and tuning hooks: changing them while another thread is inside
 *     the library changes which kernel variant that thread's next launch takes, nothing else.
 *   - Device pointers must be 16-byte aligned.
 *   - Flat path buffer layout (elements): stem | level 1 | ... | level L | head, where
 *       stem  = tok_emb [vocab, d_model], pos_emb [max_seq, d_model]
 *       level = its decoder blocks in order, each block =
 *               ln1_g[d] ln1_b[d] w_qkv[d,3A] b_qkv[3A] w_o[A,d] b_o[d] ln2_g[d] ln2_b[d]
 *               w_up[d,F] b_up[F] w_down[F,d] b_down[d]          (A = n_heads*d_head, F = d_mlp)
 *       head  = lnf_g[d] lnf_b[d] w_head[d, vocab]
 *     Matrices are row-major [in, out] (y = x W + b).  Columns of w_qkv: q heads, then k heads, then v heads.
 *     dipaco_tensor_info enumerates exactly this.
 */
#ifndef DIPACO_H
#define DIPACO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dipaco_ctx dipaco_ctx; /* opaque, host-only: shapes and offsets; no numerical state */

typedef enum {
  DIPACO_OK = 0,
  DIPACO_EINVAL = -1,       /* null pointer, negative size, bad enum                       */
  DIPACO_ESHAPE = -2,       /* a size the kernels do not support (see dipaco_create)        */
  DIPACO_EALIGN = -3,       /* a device pointer is not 16-byte aligned                      */
  DIPACO_EWORKSPACE = -4,   /* workspace smaller than dipaco_workspace_bytes                */
  DIPACO_EHIP = -5,         /* a HIP runtime call failed (message has hipGetErrorString)    */
  DIPACO_EUNSUPPORTED = -6
} dipaco_status;

typedef enum { DIPACO_F32 = 0, DIPACO_BF16 = 1 } dipaco_dtype;

/* One path's architecture (Section 4 and the hyper-parameter table: blocks, width, heads, key/value size,
 * vocabulary).  Pre-LN blocks, learned positions, untied head, biases on the linears, exact-erf GELU. */
typedef struct {
  int32_t n_levels;                /* L (Section 2.3)                                                   */
  const int32_t* layers_per_level; /* host, [L]: decoder blocks contributed by each level's module      */
  int32_t d_model, n_heads, d_head, d_mlp, vocab, max_seq;
  float ln_eps;
  int32_t compute;                 /* dipaco_dtype: arithmetic of activations and matrix operands.
                                      Master weights, gradients and optimiser state are always fp32.     */
} dipaco_arch;

/* Requirements: d_model, n_heads*d_head, d_mlp, vocab multiples of 8; d_head in {32, 64, 128}; d_model <= 2048;
 * vocab <= 65536; n_levels >= 1, every layers_per_level >= 0.  Otherwise DIPACO_ESHAPE.  Host-only: the context
 * holds shapes and offsets, no device memory. */
dipaco_status dipaco_create(dipaco_ctx** out, const dipaco_arch* arch);
void dipaco_destroy(dipaco_ctx* ctx);

/* Message for the last non-OK status returned on this host thread ("" if none). */
const char* dipaco_last_error(void);

/* Layout queries.  Segment s: 0 = stem, 1..L = levels, L+1 = head. */
size_t dipaco_path_param_count(const dipaco_ctx* ctx);
int32_t dipaco_segment_count(const dipaco_ctx* ctx);                  /* L + 2 */
size_t dipaco_segment_offset(const dipaco_ctx* ctx, int32_t segment); /* elements from the buffer start */
size_t dipaco_segment_size(const dipaco_ctx* ctx, int32_t segment);
int32_t dipaco_tensor_count(const dipaco_ctx* ctx);
/* Tensor i in storage order: name copied into name_out (host, capacity name_cap, NUL-terminated);
 * rows/cols (cols = 1 for vectors); decayed = 1 if AdamW applies weight decay to it. */
dipaco_status dipaco_tensor_info(const dipaco_ctx* ctx, int32_t i, char* name_out, size_t name_cap,
                                 size_t* offset, int64_t* rows, int64_t* cols, int32_t* decayed);

/* Path id <-> module tuple (Section 2.3): j = sum_l j_l * prod_{m>l} K_m, 0-based, level 1 most significant.
 * K, modules: host [L].  Returns -1 / DIPACO_EINVAL on out-of-range input. */
int64_t dipaco_path_index(const int32_t* modules, const int32_t* K, int32_t L);
dipaco_status dipaco_path_modules(int64_t j, const int32_t* K, int32_t L, int32_t* modules_out);

/* Bytes of device workspace dipaco_path_fwd_bwd needs for a [batch, seq] input. */
size_t dipaco_workspace_bytes(const dipaco_ctx* ctx, int32_t batch, int32_t seq);

/* Start-of-round copy of the global modules into one path's local parameters (Algorithm 1: theta_i^t =
 * theta_i^{t-1}; Section 2.6).  segment_ptrs: host array of L+2 device pointers (stem, the chosen module of
 * each level, head), each holding dipaco_segment_size fp32 elements.  Writes the flat fp32 buffer
 * path_master [dipaco_path_param_count] and, if path_lowp is not NULL, its bf16 (round-to-nearest-even)
 * image of the same length. */
dipaco_status dipaco_compose_path(dipaco_ctx* ctx, const float* const* segment_ptrs, float* path_master,
                                  void* path_lowp, void* stream);

/* L = f(x, theta_i) and its gradient (Algorithm 1, inner loop): mean next-token negative log-likelihood
 * over positions with target >= 0, natural log.
 *   path_master  device fp32 [param_count]; read when compute = F32.
 *   path_lowp    device bf16 [param_count]; read when compute = BF16 (must be the image of path_master
 *                written by dipaco_compose_path / dipaco_inner_adamw); may be NULL for F32.
 *   tokens       device int32 [batch, seq], ids in [0, vocab) (out-of-range ids are clamped).
 *   targets      device int32 [batch, seq]; negative = position ignored.  At least one must be >= 0.
 *   loss_out     device float, overwritten.     token_nll_out  device float [batch, seq] or NULL:
 *                per-position NLL (0 at ignored positions).
 *   grads        device fp32 [param_count], overwritten (same layout as path_master; rows of pos_emb
 *                beyond seq get 0).
 *   workspace    device, >= dipaco_workspace_bytes(ctx, batch, seq), contents undefined on return.
 * seq <= max_seq; batch * seq <= 2^24 and batch * seq * (max(d_mlp, 3 * n_heads * d_head, vocab) + 1) < 2^32
 * (DIPACO_ESHAPE otherwise).  Results are bit-reproducible from call to call on the same inputs. */
dipaco_status dipaco_path_fwd_bwd(dipaco_ctx* ctx, const float* path_master, const void* path_lowp,
                                  const int32_t* tokens, const int32_t* targets, int32_t batch, int32_t seq,
                                  float* loss_out, float* token_nll_out, float* grads, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* Router features g(document) (appendix on routing: the last block's hidden states averaged over a document's
 * 32-token prefix): the path's blocks are run forward on tokens [batch, seq] (seq = 32
 * in the paper) and features_out[b, :] = mean over the seq positions of the residual stream that leaves the last
 * block (before the final LayerNorm; the head is not evaluated).  features_out: device fp32 [batch, d_model]; these
 * are the z of dipaco_route_prefix.  path_master / path_lowp as in dipaco_path_fwd_bwd.
 * workspace: device, >= dipaco_features_workspace_bytes(ctx, batch, seq) (one block's activations, reused). */
size_t dipaco_features_workspace_bytes(const dipaco_ctx* ctx, int32_t batch, int32_t seq);
dipaco_status dipaco_path_prefix_features(dipaco_ctx* ctx, const float* path_master, const void* path_lowp,
                                          const int32_t* tokens, int32_t batch, int32_t seq, float* features_out,
                                          void* workspace, size_t workspace_bytes, void* stream);

/* dipaco_path_prefix_features for callers that cannot allocate device memory or carry a workspace around (code under
 * HIP graph capture, a tight serving loop that routes incoming documents, harnesses that forbid hipMalloc): the same
 * kernels, with the activations kept in a device array of DIPACO_STATIC_SCRATCH_BYTES that is part of the library's
 * code object (each GPU the library runs on holds its own copy until the process ends).  Arguments as in
 * dipaco_path_prefix_features, without the workspace; results are identical bit for bit.
 *   - DIPACO_EWORKSPACE when dipaco_features_workspace_bytes(ctx, batch, seq) exceeds DIPACO_STATIC_SCRATCH_BYTES
 *     (64 MiB: 2048 prefix tokens of the 896-wide path in bf16, e.g. 64 documents x 32 tokens); nothing is enqueued.
 *   - The call allocates and frees nothing, on the host side of the device or on it.  The first call on a device looks
 *     up the array's address there (no allocation, no synchronisation).
 *   - Every call on one GPU uses that GPU's single array: two calls that overlap in time on one GPU (different
 *     streams or host threads) race.  Nothing in the array has to start at zero; its contents after a call are
 *     undefined. */
#define DIPACO_STATIC_SCRATCH_BYTES (64u << 20)
size_t dipaco_static_scratch_bytes(void);   /* = DIPACO_STATIC_SCRATCH_BYTES */
dipaco_status dipaco_path_prefix_features_static(dipaco_ctx* ctx, const float* path_master, const void* path_lowp,
                                                 const int32_t* tokens, int32_t batch, int32_t seq,
                                                 float* features_out, void* stream);

/* Path scores for discriminative routing (Section 2.4.2; appendix on routing: the summed auto-regressive
 * log-likelihood of each document under each path, whose argmax over paths is the router's training label):
 * forward pass only.  doc_loglik_out[b] = sum over positions with target >= 0 of log p(target | prefix), natural log
 * (device fp32 [batch]); token_nll_out: device fp32 [batch, seq] or NULL, the per-position negative log-likelihoods
 * (0 at ignored positions).  Call once per path on the same documents and take the argmax on the host; the same call
 * at seq = 2048 is the forward-only evaluation of Section 4.  tokens / targets / parameters as in
 * dipaco_path_fwd_bwd; workspace >= dipaco_score_workspace_bytes(ctx, batch, seq). */
size_t dipaco_score_workspace_bytes(const dipaco_ctx* ctx, int32_t batch, int32_t seq);
dipaco_status dipaco_path_score(dipaco_ctx* ctx, const float* path_master, const void* path_lowp, const int32_t* tokens,
                                const int32_t* targets, int32_t batch, int32_t seq, float* doc_loglik_out,
                                float* token_nll_out, void* workspace, size_t workspace_bytes, void* stream);

/* Routing more often than once per document at evaluation (Section 2.4.3; appendix on more frequent routing
 * during evaluation).  token_nll: device fp32 [n_paths, batch, seq], the per-position negative log-likelihoods that
 * dipaco_path_score writes (token_nll_out) for each path on the same documents, i.e. -S_ijp.
 *   dipaco_window_targets: targets_out[b, j] (device int32 [batch, seq]) = argmax_p sum_{j' = j}^{min(seq, j + window) - 1}
 *     S_{b j' p}: the labels T_ij the token-level router is trained to transduce; lowest p on exact ties.  The window
 *     sums are differences of fp64 running sums.
 *   dipaco_chunk_routed_score: doc_loglik_out[b] (device fp32 [batch]) = log-likelihood of document b when its c-th chunk
 *     of `chunk` consecutive positions is scored by path chunk_path[b, c] (device int32 [batch, ceil(seq / chunk)],
 *     values clamped to [0, n_paths)); every path conditions on the whole preceding text, as its scoring pass did.
 *     chunk = seq with one path per document is that path's dipaco_path_score.
 * workspace: device, >= dipaco_reroute_workspace_bytes(n_paths, batch, seq) bytes (0 = invalid shape). */
size_t dipaco_reroute_workspace_bytes(int32_t n_paths, int32_t batch, int32_t seq);
dipaco_status dipaco_window_targets(const float* token_nll, int32_t n_paths, int32_t batch, int32_t seq, int32_t window,
                                    int32_t* targets_out, void* workspace, size_t workspace_bytes, void* stream);
dipaco_status dipaco_chunk_routed_score(const float* token_nll, const int32_t* chunk_path, int32_t n_paths, int32_t batch,
                                        int32_t seq, int32_t chunk, float* doc_loglik_out, void* workspace,
                                        size_t workspace_bytes, void* stream);

/* InnerOpt = AdamW (Algorithm 1, inner loop; Section 2.5), over the whole flat path buffer, in place:
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   theta <- theta - lr * ( (m/(1-b1^step)) / (sqrt(v/(1-b2^step)) + eps) + weight_decay * theta ),
 * weight decay applied to matrices and embeddings only.  step counts from 1.  If path_lowp is not NULL the
 * bf16 image of the new theta is written there. */
dipaco_status dipaco_inner_adamw(dipaco_ctx* ctx, float* path_master, const float* grads, float* m, float* v,
                                 void* path_lowp, int64_t step, float lr, float beta1, float beta2, float eps,
                                 float weight_decay, void* stream);

#define DIPACO_MAX_PATHS_PER_MODULE 256

/* Outer step of one module (Algorithm 1, outer loop; weights per Section 2.7), in place on theta/momentum:
 *   Delta = sum_i alpha_i (theta - input_i)   (is_delta = 0: inputs are the paths' local copies theta_i)
 *         = sum_i alpha_i  input_i            (is_delta = 1: inputs are ready-made deltas)
 *   alpha_i = weights_i / sum(weights)        (weights NULL = uniform: the plain mean over P_le paths)
 *   momentum <- mu * momentum + Delta;   theta <- theta - outer_lr * (Delta + mu * momentum)   (Nesterov)
 * inputs: host array of n_paths device pointers, fp32 [n_elems] each; weights: host [n_paths], positive.
 * 1 <= n_paths <= DIPACO_MAX_PATHS_PER_MODULE.  The sum runs in index order, so the result is reproducible. */
dipaco_status dipaco_module_outer_step(float* theta, float* momentum, const float* const* inputs,
                                       const float* weights, int32_t n_paths, size_t n_elems, int32_t is_delta,
                                       float outer_lr, float outer_momentum, void* stream);

/* The same outer step one path at a time (Section 3.3, online parameter gradient averaging: a path's result joins
 * the partial sum when it arrives, without waiting for the other paths), with the optional outer gradient norm
 * rescaling of Section 2.7:
 *   dipaco_module_delta_accumulate:  delta_sum <- (first ? 0 : delta_sum) + weight * (theta_prev - input)   (is_delta = 0)
 *                                                                         + weight * input                  (is_delta = 1)
 *       weight: the path's un-normalised shard weight (1 for the uniform mean); theta_prev may be NULL when is_delta.
 *   dipaco_module_outer_apply:       Delta = norm_scale * delta_sum / weight_sum;
 *       momentum <- mu * momentum + Delta;   theta <- theta - outer_lr * (Delta + mu * momentum)
 *       weight_sum: the sum of the weights accumulated; norm_scale: 1, or sqrt(number of paths through the module)
 *       for the norm rescaling (read as a multiplication: averaging over more paths acts like a larger
 *       batch, so the averaged step is made longer).
 * All buffers device fp32 [n_elems], 16-byte aligned; delta_sum is caller-owned scratch that lives across the calls.
 * With norm_scale = 1 the result equals dipaco_module_outer_step up to the order of the additions. */
dipaco_status dipaco_module_delta_accumulate(float* delta_sum, const float* theta_prev, const float* input, float weight,
                                             size_t n_elems, int32_t is_delta, int32_t first, void* stream);
dipaco_status dipaco_module_outer_apply(float* theta, float* momentum, const float* delta_sum, double weight_sum,
                                        float norm_scale, size_t n_elems, float outer_lr, float outer_momentum,
                                        void* stream);

/* Outer step of many modules in one launch.  Algorithm 1 runs the outer update for every module (l, e) of the grid;
 * Section 2.6 keeps it for path-specific modules too (one path, no averaging, same outer optimiser), so a phase ends
 * with many updates of very different sizes and path counts.  A table that lives in device memory describes them all;
 * it is built once and reused for as long as the buffers it names stay where they are.
 *   dipaco_module_desc: one module, as in dipaco_module_outer_step: theta / momentum device fp32 [n_elems], 16-byte
 *     aligned; inputs = HOST array of n_paths device pointers (fp32 [n_elems], 16-byte aligned); weights = HOST
 *     [n_paths] positive, or NULL for the plain mean; norm_scale multiplies the averaged Delta (1, or sqrt(paths
 *     through the module) for the rescaling of Section 2.7); n_elems may be 0.
 *   dipaco_outer_table_bytes: size of the table image for these modules (0 on invalid arguments).
 *   dipaco_outer_table_pack:  host-only; validates the descriptions and writes the image (normalised weights
 *     alpha_i = norm_scale * w_i / sum w in fp32, pointers, chunk offsets) into HOST memory `image`.  The caller copies
 *     the image to device memory (8-byte aligned) and passes both copies to the step.
 *   dipaco_outer_step_table:  momentum <- mu * momentum + Delta; theta <- theta - outer_lr * (Delta + mu * momentum)
 *     for every module of the table, Delta summed over its inputs in index order (reproducible).  Modules must not
 *     overlap in memory. */
typedef struct dipaco_module_desc {
  float* theta;
  float* momentum;
  const float* const* inputs;
  const float* weights;
  uint64_t n_elems;
  int32_t n_paths;
  int32_t is_delta;
  float norm_scale;
} dipaco_module_desc;
size_t dipaco_outer_table_bytes(const dipaco_module_desc* modules, int32_t n_modules);
dipaco_status dipaco_outer_table_pack(const dipaco_module_desc* modules, int32_t n_modules, void* image,
                                      size_t image_bytes);
dipaco_status dipaco_outer_step_table(const void* table_host, const void* table_device, size_t table_bytes,
                                      float outer_lr, float outer_momentum, void* stream);

/* Generative routing (Section 2.4.1, eq. 1): idx[n] = argmin_k ||z_n - c_k||^2, lowest k on exact ties of the
 * computed scores; hist[k] = number of n routed to k.  The kernel minimises ||c_k||^2 - 2 z_n.c_k (same
 * argmin) in fp32.
 *   z device fp32 [N, D] row-major; centroids device fp32 [K, D]; idx_out device int32 [N];
 *   hist_out device int64 [K], overwritten; margin_out device fp32 [N] or NULL: second-best minus best score
 *   (+inf when K = 1).  D multiple of 4, 1 <= K <= 4096, N >= 0.
 *   Centroids must be finite.  A row of z that holds a NaN has no nearest centroid (every score is NaN, as it is
 *   for infinite features that meet centroid entries of both signs): it is routed to centroid 0 (second choice 1 in
 *   the top-2 form), counted there, and its margin is NaN, so that a caller can find and drop such rows.  Other rows
 *   with infinite entries get an index in [0, K) and are counted once; which one is not specified.  Eq. 1 itself
 *   assigns every finite document. */
dipaco_status dipaco_route_prefix(const float* z, const float* centroids, int64_t N, int32_t D, int32_t K,
                                  int32_t* idx_out, int64_t* hist_out, float* margin_out, void* stream);

/* The same assignment with a row stride and, optionally, the two closest centroids.
 *   z          device fp32, row n at z + n * ldz (ldz >= D, multiple of 4): a column block of a wider feature matrix
 *              can be routed in place, which is all that product k-means needs (appendix on product k-means: route
 *              the first and the second half of the features against their own centroid sets; the pair of indices
 *              is the path's module tuple, see dipaco_path_index).
 *   n_best = 1: idx_out int32 [N] as above.
 *   n_best = 2: idx_out int32 [N, 2] = the closest and the second closest centroid (the top-2 overlapping shards of
 *              Section 2.4.4; second entry -1 when K = 1), ties to the lower index; hist_out[k] counts the documents
 *              that have k as either choice, i.e. the sizes of the overlapping shards.
 *   margin_out as above (second-best minus best score) in both modes. */
dipaco_status dipaco_route_prefix_top(const float* z, int64_t ldz, const float* centroids, int64_t N, int32_t D,
                                      int32_t K, int32_t n_best, int32_t* idx_out, int64_t* hist_out, float* margin_out,
                                      void* stream);

/* Discriminative router (Section 2.4.2; appendix on routing): a K-class linear logistic classifier on the features z,
 * trained on the labels argmax_p sum_j S_ijp that dipaco_path_score provides, then used as r(z).
 *   dipaco_route_linear: idx[n] = argmax_k (weights_k . z_n + bias_k), lowest k on exact ties; hist_out as in
 *     dipaco_route_prefix; margin_out (or NULL) = best minus second-best logit (+inf when K = 1).  weights device
 *     fp32 [K, D]; bias device fp32 [K]; z row n at z + n * ldz.  D multiple of 4, 1 <= K <= 4096.
 *   dipaco_router_logistic_grad: loss = mean over the N documents of -log softmax(z_n W^T + b)[label_n] and its
 *     gradients dweights_out [K, D] (NULL: not computed), dbias_out [K], all fp32 on the device; the caller applies
 *     them with the optimiser it likes (dipaco_module_outer_step with one ready-made delta is plain / Nesterov SGD).
 *     Since dbias = mean softmax - label frequencies, descending on the bias alone (dweights_out = NULL) is the
 *     bias fit of the appendix on routing (a bias trained until the predicted document-to-path distribution is the
 *     target one): it stops where the mean predicted
 *     distribution equals the labels'.  labels device int32 [N]; a label outside [0, K) drops its document from loss
 *     and gradients (the mean stays over N).  z device fp32 [N, D] contiguous.  D and K multiples of 8, K <= 4096,
 *     N * max(D, K) < 2^32.  workspace: device, >= dipaco_router_workspace_bytes(N, D, K) bytes (0 = invalid shape). */
dipaco_status dipaco_route_linear(const float* z, int64_t ldz, const float* weights, const float* bias, int64_t N, int32_t D,
                                  int32_t K, int32_t* idx_out, int64_t* hist_out, float* margin_out, void* stream);
size_t dipaco_router_workspace_bytes(int64_t N, int32_t D, int32_t K);
dipaco_status dipaco_router_logistic_grad(const float* z, const int32_t* labels, const float* weights, const float* bias,
                                          int64_t N, int32_t D, int32_t K, float* loss_out, float* dweights_out,
                                          float* dbias_out, void* workspace, size_t workspace_bytes, void* stream);

/* One k-means update (Section 2.4.1 fits the prototypes c_i by k-means on the features z; with dipaco_route_prefix
 * as the assignment step this is one Lloyd iteration): centroids[k] <- mean of the rows z_n with idx[n] = k, in place; a
 * centroid without rows keeps its value.  idx values are clamped to [0, K).  counts_out: device int64 [K] or NULL.
 * The sums are formed in a fixed order (stable counting sort by cluster, partial sums of 512 rows added in order):
 * results are bit-reproducible.  workspace: device, >= dipaco_kmeans_workspace_bytes(N, D, K) bytes.
 * D multiple of 4, 1 <= K <= 4096. */
size_t dipaco_kmeans_workspace_bytes(int64_t N, int32_t D, int32_t K);
dipaco_status dipaco_kmeans_update(const float* z, int64_t ldz, const int32_t* idx, int64_t N, int32_t D, int32_t K,
                                   float* centroids, int64_t* counts_out, void* workspace, size_t workspace_bytes,
                                   void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DIPACO_H */
