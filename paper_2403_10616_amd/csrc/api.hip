// C ABI of libdipaco: argument validation, parameter layout, workspace planning and the launch order of the
// path step.  All arithmetic lives in the kernels; this file only decides which kernel runs on which buffer.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/dipaco_kernels.h"
#include "kernels.h"

namespace dipaco {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }
dipaco_status fail(dipaco_status st, const std::string& msg) {
  g_last_error = msg;
  return st;
}
dipaco_status check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return DIPACO_OK;
  return fail(DIPACO_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

struct TensorInfo {
  std::string name;
  size_t off;
  int64_t rows, cols;
  bool decay;
};

struct BlockOff {
  size_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_up, b_up, w_down, b_down;
};

}  // namespace dipaco

using namespace dipaco;

struct dipaco_ctx {
  dipaco_arch arch;
  std::vector<int32_t> layers_per_level;
  int n_layers = 0;
  int A = 0;   // n_heads * d_head
  std::vector<TensorInfo> tensors;
  std::vector<BlockOff> blocks;
  size_t tok_emb = 0, pos_emb = 0, lnf_g = 0, lnf_b = 0, w_head = 0;
  std::vector<size_t> seg_off, seg_size;
  size_t n_params = 0;
  AdamLayout adam;
};

namespace dipaco {

// ---- workspace plan --------------------------------------------------------------------------------------
struct LayerBufs {
  size_t x_in, h1, mean1, rstd1, qkv, o, lse, x_mid, h2, mean2, rstd2, u, act;
};
struct Plan {
  std::vector<LayerBufs> layers;
  size_t x_final, meanf, rstdf, y, logits, nll, n_valid;
  size_t dxa, dxb, dh, du, dqkv, d_o, dsum;
  size_t ln_partial, cs_partial, splitk_partial, embed_ints;
  size_t ln_partial_stride, cs_partial_stride;   // bytes between the buffers of consecutive producers
  size_t total;
};

template <typename T> static int dw_splits(int M, int N, int K) { return gemm_plan_splits(M, N, K, sizeof(T) == 2); }

static Plan make_plan(const dipaco_ctx* c, int B, int S) {
  const dipaco_arch& a = c->arch;
  const size_t T = (size_t)B * S, d = a.d_model, A = c->A, F = a.d_mlp, V = a.vocab;
  const size_t es = a.compute == DIPACO_BF16 ? 2 : 4;
  size_t pos = 0;
  auto take = [&](size_t bytes) {
    size_t at = pos;
    pos += (bytes + 255) & ~(size_t)255;
    return at;
  };
  Plan p;
  p.layers.resize(c->n_layers);
  for (auto& L : p.layers) {
    L.x_in = take(T * d * es); L.h1 = take(T * d * es); L.mean1 = take(T * 4); L.rstd1 = take(T * 4);
    L.qkv = take(T * 3 * A * es); L.o = take(T * A * es); L.lse = take((size_t)B * a.n_heads * S * 4);
    L.x_mid = take(T * d * es); L.h2 = take(T * d * es); L.mean2 = take(T * 4); L.rstd2 = take(T * 4);
    L.u = take(T * F * es); L.act = take(T * F * es);
  }
  p.x_final = take(T * d * es); p.meanf = take(T * 4); p.rstdf = take(T * 4); p.y = take(T * d * es);
  p.logits = take(T * V * es); p.nll = take(T * 4); p.n_valid = take(256);
  p.dxa = take(T * d * es); p.dxb = take(T * d * es); p.dh = take(T * d * es); p.du = take(T * F * es);
  p.dqkv = take(T * 3 * A * es); p.d_o = take(T * A * es); p.dsum = take(2 * (size_t)B * a.n_heads * ((S + 127) / 128 * 128) * 4);
  // Partial rows of the backward pass's fixed-order sums.  Their final reductions run as one launch at the end of the
  // step, so every producer keeps a buffer of its own: one per LayerNorm, two per block (the column sums of dU and
  // of dqkv).
  p.ln_partial_stride = (ln_bwd_partial_floats((int)T, (int)d) * 4 + 255) & ~(size_t)255;
  p.ln_partial = take(p.ln_partial_stride * (2 * (size_t)c->n_layers + 1));
  const size_t widest = std::max(std::max(F, 3 * A), d);
  p.cs_partial_stride = (std::max(std::max(colsum_partial_floats((int)T, (int)widest), gemm_colsum_partial_floats((int)T, (int)F)),
                                  attention_bwd_colsum_floats((int)B, (int)S, a.n_heads, a.d_head)) * 4 + 255) & ~(size_t)255;
  p.cs_partial = take(p.cs_partial_stride * std::max<size_t>(1, 2 * (size_t)c->n_layers));
  size_t sk = 0;
  auto need = [&](size_t M, size_t N) { sk = std::max(sk, (size_t)gemm_max_splits((int)M, (int)N, (int)T) * M * N); };
  need(d, 3 * A); need(A, d); need(d, F); need(F, d); need(d, V);
  p.splitk_partial = take(sk * 4);
  p.embed_ints = take(embed_bwd_scratch_ints((int)T, (int)V) * 4);
  p.total = pos;
  return p;
}

// ---- the path step ---------------------------------------------------------------------------------------
template <typename T>
static dipaco_status gemm(const T* A, const T* B, void* C, int M, int N, int K, long lda, long ldb, long ldc,
                          bool ta, bool tb, const T* bias, const T* resid, T* aux_out, const T* aux_in, int act,
                          bool out_f32, int splits, float* partial, hipStream_t s, float* colsum = nullptr,
                          float* colsum_partial = nullptr, SumBatch* sum_batch = nullptr) {
  GemmArgs g;
  g.colsum = colsum; g.colsum_partial = colsum_partial; g.sum_batch = sum_batch;
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.bias = bias; g.resid = resid; g.aux_out = aux_out; g.aux_in = aux_in; g.act = act;
  g.trans_a = ta; g.trans_b = tb; g.out_f32 = out_f32; g.splits = splits; g.partial = partial;
  return launch_gemm<T>(g, s);
}

#define TRY(expr)                          \
  do {                                     \
    dipaco_status _s = (expr);             \
    if (_s != DIPACO_OK) return _s;        \
  } while (0)

template <typename T>
static dipaco_status run_fwd_bwd(const dipaco_ctx* c, const T* W, const int* tokens, const int* targets, int B, int S,
                                 float* loss_out, float* nll_out, float* G, char* ws, hipStream_t st) {
  const dipaco_arch& a = c->arch;
  const int T_ = B * S, d = a.d_model, A = c->A, F = a.d_mlp, V = a.vocab, H = a.n_heads, dh = a.d_head;
  const Plan p = make_plan(c, B, S);
  auto buf = [&](size_t off) { return reinterpret_cast<T*>(ws + off); };
  auto fbuf = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  float* skp = fbuf(p.splitk_partial);
  SumBatch sums;            // the backward pass's final reductions, run as one launch at the end
  int ln_jobs = 0, cs_jobs = 0;
  auto next_lnp = [&]() { return fbuf(p.ln_partial + p.ln_partial_stride * (size_t)ln_jobs++); };
  auto next_csp = [&]() { return fbuf(p.cs_partial + p.cs_partial_stride * (size_t)cs_jobs++); };
  int* n_valid = reinterpret_cast<int*>(ws + p.n_valid);
  float* nll = nll_out ? nll_out : fbuf(p.nll);
  const int NL = c->n_layers;

  // weight gradient dW[K_in, N_out] = X^T . dY (contraction over the tokens), fp32 into the gradient buffer
  auto dweight = [&](const T* X, const T* dY, size_t w_off, int K_in, int N_out) {
    return gemm<T>(X, dY, G + w_off, K_in, N_out, T_, K_in, N_out, N_out, true, false, nullptr, nullptr, nullptr, nullptr,
                   0, true, dw_splits<T>(K_in, N_out, T_), skp, st);
  };

  // ---------------- forward ----------------
  T* x0 = NL > 0 ? buf(p.layers[0].x_in) : buf(p.x_final);
  TRY(launch_embed<T>(W + c->tok_emb, W + c->pos_emb, tokens, x0, B, S, d, V, st));
  for (int l = 0; l < NL; ++l) {
    const LayerBufs& L = p.layers[l];
    const BlockOff& o = c->blocks[l];
    T* x_next = l + 1 < NL ? buf(p.layers[l + 1].x_in) : buf(p.x_final);
    TRY(launch_layernorm_fwd<T>(buf(L.x_in), W + o.ln1_g, W + o.ln1_b, buf(L.h1), fbuf(L.mean1), fbuf(L.rstd1), T_, d,
                                a.ln_eps, st));
    TRY(gemm<T>(buf(L.h1), W + o.w_qkv, buf(L.qkv), T_, 3 * A, d, d, 3 * A, 3 * A, false, false, W + o.b_qkv, nullptr,
                nullptr, nullptr, 0, false, 1, nullptr, st));
    TRY(launch_attention_fwd<T>(buf(L.qkv), buf(L.o), fbuf(L.lse), B, S, H, dh, st));
    TRY(gemm<T>(buf(L.o), W + o.w_o, buf(L.x_mid), T_, d, A, A, d, d, false, false, W + o.b_o, buf(L.x_in), nullptr,
                nullptr, 0, false, 1, nullptr, st));
    TRY(launch_layernorm_fwd<T>(buf(L.x_mid), W + o.ln2_g, W + o.ln2_b, buf(L.h2), fbuf(L.mean2), fbuf(L.rstd2), T_, d,
                                a.ln_eps, st));
    // L.u receives GELU'(pre-activation), the only thing the backward pass needs of it
    TRY(gemm<T>(buf(L.h2), W + o.w_up, buf(L.act), T_, F, d, d, F, F, false, false, W + o.b_up, nullptr, buf(L.u),
                nullptr, 3, false, 1, nullptr, st));
    TRY(gemm<T>(buf(L.act), W + o.w_down, x_next, T_, d, F, F, d, d, false, false, W + o.b_down, buf(L.x_mid), nullptr,
                nullptr, 0, false, 1, nullptr, st));
  }
  TRY(launch_layernorm_fwd<T>(buf(p.x_final), W + c->lnf_g, W + c->lnf_b, buf(p.y), fbuf(p.meanf), fbuf(p.rstdf), T_, d,
                              a.ln_eps, st));
  TRY(gemm<T>(buf(p.y), W + c->w_head, buf(p.logits), T_, V, d, d, V, V, false, false, nullptr, nullptr, nullptr,
              nullptr, 0, false, 1, nullptr, st));
  TRY(launch_count_valid(targets, T_, n_valid, st));
  TRY(launch_softmax_xent<T>(buf(p.logits), targets, n_valid, nll, T_, V, true, st));
  TRY(launch_mean_loss(nll, n_valid, loss_out, T_, st));

  // ---------------- backward ----------------
  T* dlogits = buf(p.logits);
  TRY(dweight(buf(p.y), dlogits, c->w_head, d, V));
  TRY(gemm<T>(dlogits, W + c->w_head, buf(p.dh), T_, d, V, V, V, d, false, true, nullptr, nullptr, nullptr, nullptr, 0,
              false, 1, nullptr, st));
  T* dx = buf(p.dxa);
  T* dx_other = buf(p.dxb);
  // every LayerNorm backward also leaves the column sums of the dx it writes: the bias gradient of the linear
  // layer below it in the residual stream (W_down of the block before, W_o of its own block)
  TRY(launch_layernorm_bwd<T>(buf(p.dh), buf(p.x_final), W + c->lnf_g, fbuf(p.meanf), fbuf(p.rstdf), nullptr, dx,
                              G + c->lnf_g, G + c->lnf_b, NL > 0 ? G + c->blocks[NL - 1].b_down : nullptr, next_lnp(), T_, d,
                              st, &sums));
  for (int l = NL - 1; l >= 0; --l) {
    const LayerBufs& L = p.layers[l];
    const BlockOff& o = c->blocks[l];
    // x_next = x_mid + gelu(u) W_down + b_down
    TRY(dweight(buf(L.act), dx, o.w_down, F, d));
    // du = (dx W_down^T) * GELU'(u); its column sums, the gradient of b_up, come out of the same product
    TRY(gemm<T>(dx, W + o.w_down, buf(p.du), T_, F, d, d, d, F, false, true, nullptr, nullptr, nullptr, buf(L.u), 4,
                false, 1, nullptr, st, G + o.b_up, next_csp(), &sums));
    TRY(dweight(buf(L.h2), buf(p.du), o.w_up, d, F));
    TRY(gemm<T>(buf(p.du), W + o.w_up, buf(p.dh), T_, d, F, F, F, d, false, true, nullptr, nullptr, nullptr, nullptr, 0,
                false, 1, nullptr, st));
    TRY(launch_layernorm_bwd<T>(buf(p.dh), buf(L.x_mid), W + o.ln2_g, fbuf(L.mean2), fbuf(L.rstd2), dx, dx_other,
                                G + o.ln2_g, G + o.ln2_b, G + o.b_o, next_lnp(), T_, d, st, &sums));
    // x_mid = x_in + attn(...) W_o + b_o          (dx_other = gradient at x_mid)
    TRY(dweight(buf(L.o), dx_other, o.w_o, A, d));
    TRY(gemm<T>(dx_other, W + o.w_o, buf(p.d_o), T_, A, d, d, d, A, false, true, nullptr, nullptr, nullptr, nullptr, 0,
                false, 1, nullptr, st));
    // dqkv and its column sums, the gradient of b_qkv
    TRY(launch_attention_bwd<T>(buf(L.qkv), buf(L.o), buf(p.d_o), fbuf(L.lse), buf(p.dqkv), fbuf(p.dsum), G + o.b_qkv,
                                next_csp(), B, S, H, dh, st, &sums));
    TRY(dweight(buf(L.h1), buf(p.dqkv), o.w_qkv, d, 3 * A));
    TRY(gemm<T>(buf(p.dqkv), W + o.w_qkv, buf(p.dh), T_, d, 3 * A, 3 * A, 3 * A, d, false, true, nullptr, nullptr,
                nullptr, nullptr, 0, false, 1, nullptr, st));
    TRY(launch_layernorm_bwd<T>(buf(p.dh), buf(L.x_in), W + o.ln1_g, fbuf(L.mean1), fbuf(L.rstd1), dx_other, dx,
                                G + o.ln1_g, G + o.ln1_b, l > 0 ? G + c->blocks[l - 1].b_down : nullptr, next_lnp(), T_, d, st,
                                &sums));
  }
  TRY(flush_sum_batch(sums, st));
  TRY(launch_embed_bwd<T>(dx, tokens, G + c->tok_emb, G + c->pos_emb, reinterpret_cast<int*>(ws + p.embed_ints), B, S,
                          d, V, a.max_seq, st));
  return DIPACO_OK;
}

// ---- prefix features: forward through the blocks only, one set of layer buffers reused by every block -------
struct FeaturePlan {
  size_t x_a, x_b, h, mean, rstd, qkv, o, lse, x_mid, u, act, logits, nll, n_valid, total;
};
static FeaturePlan make_feature_plan(const dipaco_ctx* c, int B, int S, bool with_head = false) {
  const dipaco_arch& a = c->arch;
  const size_t T = (size_t)B * S, d = a.d_model, A = c->A, F = a.d_mlp;
  const size_t es = a.compute == DIPACO_BF16 ? 2 : 4;
  size_t pos = 0;
  auto take = [&](size_t bytes) { size_t at = pos; pos += (bytes + 255) & ~(size_t)255; return at; };
  FeaturePlan p;
  p.x_a = take(T * d * es); p.x_b = take(T * d * es); p.h = take(T * d * es); p.mean = take(T * 4); p.rstd = take(T * 4);
  p.qkv = take(T * 3 * A * es); p.o = take(T * A * es); p.lse = take((size_t)B * a.n_heads * S * 4);
  p.x_mid = take(T * d * es); p.u = take(T * F * es); p.act = take(T * F * es);
  p.logits = p.nll = p.n_valid = 0;
  if (with_head) { p.logits = take(T * (size_t)a.vocab * es); p.nll = take(T * 4); p.n_valid = take(256); }
  p.total = pos;
  return p;
}

// out: router features [B, d] (targets == nullptr), or per-document log-likelihood [B] (+ nll_out [B, S], nullable)
template <typename T>
static dipaco_status run_features(const dipaco_ctx* c, const T* W, const int* tokens, const int* targets, int B, int S,
                                  float* out, float* nll_out, char* ws, hipStream_t st) {
  const dipaco_arch& a = c->arch;
  const int T_ = B * S, d = a.d_model, A = c->A, F = a.d_mlp, V = a.vocab, H = a.n_heads, dh = a.d_head;
  const FeaturePlan p = make_feature_plan(c, B, S, targets != nullptr);
  auto buf = [&](size_t off) { return reinterpret_cast<T*>(ws + off); };
  auto fbuf = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  T* x = buf(p.x_a);
  T* x_other = buf(p.x_b);
  TRY(launch_embed<T>(W + c->tok_emb, W + c->pos_emb, tokens, x, B, S, d, V, st));
  for (int l = 0; l < c->n_layers; ++l) {
    const BlockOff& o = c->blocks[l];
    TRY(launch_layernorm_fwd<T>(x, W + o.ln1_g, W + o.ln1_b, buf(p.h), fbuf(p.mean), fbuf(p.rstd), T_, d, a.ln_eps, st));
    TRY(gemm<T>(buf(p.h), W + o.w_qkv, buf(p.qkv), T_, 3 * A, d, d, 3 * A, 3 * A, false, false, W + o.b_qkv, nullptr,
                nullptr, nullptr, 0, false, 1, nullptr, st));
    TRY(launch_attention_fwd<T>(buf(p.qkv), buf(p.o), fbuf(p.lse), B, S, H, dh, st));
    TRY(gemm<T>(buf(p.o), W + o.w_o, buf(p.x_mid), T_, d, A, A, d, d, false, false, W + o.b_o, x, nullptr, nullptr, 0,
                false, 1, nullptr, st));
    TRY(launch_layernorm_fwd<T>(buf(p.x_mid), W + o.ln2_g, W + o.ln2_b, buf(p.h), fbuf(p.mean), fbuf(p.rstd), T_, d,
                                a.ln_eps, st));
    TRY(gemm<T>(buf(p.h), W + o.w_up, buf(p.act), T_, F, d, d, F, F, false, false, W + o.b_up, nullptr, buf(p.u), nullptr,
                3, false, 1, nullptr, st));
    TRY(gemm<T>(buf(p.act), W + o.w_down, x_other, T_, d, F, F, d, d, false, false, W + o.b_down, buf(p.x_mid), nullptr,
                nullptr, 0, false, 1, nullptr, st));
    std::swap(x, x_other);
  }
  if (!targets) return launch_mean_pool<T>(x, out, B, S, d, st);
  // scoring: final LayerNorm, head, per-token negative log-likelihood, summed per document
  TRY(launch_layernorm_fwd<T>(x, W + c->lnf_g, W + c->lnf_b, buf(p.h), fbuf(p.mean), fbuf(p.rstd), T_, d, a.ln_eps, st));
  TRY(gemm<T>(buf(p.h), W + c->w_head, buf(p.logits), T_, V, d, d, V, V, false, false, nullptr, nullptr, nullptr, nullptr,
              0, false, 1, nullptr, st));
  float* nll = nll_out ? nll_out : fbuf(p.nll);
  TRY(launch_softmax_xent<T>(buf(p.logits), targets, nullptr, nll, T_, V, false, st));   // no gradient: logits are only read
  return launch_doc_score(nll, out, B, S, st);
}

// Everything about a [batch, seq] input that a kernel of the path would refuse, checked before the first launch: the
// kernels index their operands with 32-bit element offsets, so tokens x (widest activation row) stays below 2^32.
static dipaco_status check_batch_shape(const dipaco_ctx* c, int B, int S, bool with_head) {
  if (B < 1 || S < 1 || S > c->arch.max_seq) return fail(DIPACO_ESHAPE, "batch >= 1 and 1 <= seq <= max_seq required");
  if ((int64_t)B * S > (1 << 24)) return fail(DIPACO_ESHAPE, "batch*seq above 2^24 is not supported");
  const int64_t widest = std::max<int64_t>(std::max<int64_t>(c->arch.d_mlp, 3 * (int64_t)c->A),
                                           std::max<int64_t>(c->arch.d_model, with_head ? c->arch.vocab : 0));
  if ((int64_t)S * 3 * c->A * 2 >= (1LL << 32))   // the attention kernels address one sequence's q | k | v rows with 32-bit byte offsets
    return fail(DIPACO_ESHAPE, "seq * 3 * heads * d_head * 2 bytes must stay below 2^32");
  if ((int64_t)B * S * (widest + 1) >= (1LL << 32))
    return fail(DIPACO_ESHAPE, "batch*seq times the widest activation row (d_mlp, 3*heads*d_head, vocab) must stay below 2^32");
  return DIPACO_OK;
}

static dipaco_status check_ptr(const void* p, const char* name) {
  if (!p) return fail(DIPACO_EINVAL, std::string(name) + " is NULL");
  if (!aligned16(p)) return fail(DIPACO_EALIGN, std::string(name) + " is not 16-byte aligned");
  return DIPACO_OK;
}

}  // namespace dipaco

// ==========================================================================================================
extern "C" {

const char* dipaco_last_error(void) { return g_last_error.c_str(); }

dipaco_status dipaco_create(dipaco_ctx** out, const dipaco_arch* arch) {
  if (!out || !arch || !arch->layers_per_level) return fail(DIPACO_EINVAL, "dipaco_create: NULL argument");
  *out = nullptr;
  const dipaco_arch& a = *arch;
  if (a.n_levels < 1) return fail(DIPACO_ESHAPE, "n_levels must be >= 1");
  if (a.compute != DIPACO_F32 && a.compute != DIPACO_BF16) return fail(DIPACO_EINVAL, "unknown compute dtype");
  if (a.d_model <= 0 || a.n_heads <= 0 || a.d_mlp <= 0 || a.vocab <= 0 || a.max_seq <= 0)
    return fail(DIPACO_ESHAPE, "sizes must be positive");
  if (a.d_head != 32 && a.d_head != 64 && a.d_head != 128) return fail(DIPACO_ESHAPE, "d_head must be 32, 64 or 128");
  if (a.d_model % 8 || a.d_mlp % 8 || a.vocab % 8) return fail(DIPACO_ESHAPE, "d_model, d_mlp and vocab must be multiples of 8");
  if (a.d_model > 2048) return fail(DIPACO_ESHAPE, "d_model above 2048 is not supported");
  if (a.vocab > 65536) return fail(DIPACO_ESHAPE, "vocab above 65536 is not supported");
  if ((int64_t)a.vocab * a.d_model >= (1LL << 31) || (int64_t)a.d_mlp * a.d_model >= (1LL << 31))
    return fail(DIPACO_ESHAPE, "a weight matrix above 2^31 elements is not supported");
  if (!(a.ln_eps > 0.f)) return fail(DIPACO_EINVAL, "ln_eps must be positive");
  dipaco_ctx* c = new dipaco_ctx();
  c->arch = a;
  c->layers_per_level.assign(a.layers_per_level, a.layers_per_level + a.n_levels);
  c->arch.layers_per_level = c->layers_per_level.data();
  for (int v : c->layers_per_level) {
    if (v < 0) { delete c; return fail(DIPACO_ESHAPE, "layers_per_level must be >= 0"); }
    c->n_layers += v;
  }
  c->A = a.n_heads * a.d_head;
  const size_t d = a.d_model, A = c->A, F = a.d_mlp, V = a.vocab;
  size_t off = 0;
  auto put = [&](const std::string& name, int64_t rows, int64_t cols, bool decay) {
    c->tensors.push_back({name, off, rows, cols, decay});
    size_t at = off;
    off += (size_t)rows * cols;
    return at;
  };
  c->seg_off.push_back(0);
  c->tok_emb = put("tok_emb", V, d, true);
  c->pos_emb = put("pos_emb", a.max_seq, d, true);
  c->seg_size.push_back(off);
  int layer = 0;
  for (int lv = 0; lv < a.n_levels; ++lv) {
    c->seg_off.push_back(off);
    for (int i = 0; i < c->layers_per_level[lv]; ++i, ++layer) {
      const std::string p = "blk" + std::to_string(layer) + ".";
      BlockOff b;
      b.ln1_g = put(p + "ln1_g", d, 1, false); b.ln1_b = put(p + "ln1_b", d, 1, false);
      b.w_qkv = put(p + "w_qkv", d, 3 * A, true); b.b_qkv = put(p + "b_qkv", 3 * A, 1, false);
      b.w_o = put(p + "w_o", A, d, true); b.b_o = put(p + "b_o", d, 1, false);
      b.ln2_g = put(p + "ln2_g", d, 1, false); b.ln2_b = put(p + "ln2_b", d, 1, false);
      b.w_up = put(p + "w_up", d, F, true); b.b_up = put(p + "b_up", F, 1, false);
      b.w_down = put(p + "w_down", F, d, true); b.b_down = put(p + "b_down", d, 1, false);
      c->blocks.push_back(b);
    }
    c->seg_size.push_back(off - c->seg_off.back());
  }
  c->seg_off.push_back(off);
  c->lnf_g = put("lnf_g", d, 1, false);
  c->lnf_b = put("lnf_b", d, 1, false);
  c->w_head = put("w_head", d, V, true);
  c->seg_size.push_back(off - c->seg_off.back());
  c->n_params = off;

  c->adam.stem_end = c->seg_off[1];
  c->adam.blocks_end = c->lnf_g;
  c->adam.head_matrix = c->w_head;
  c->adam.block_size = 0;
  for (int i = 0; i < 8; ++i) c->adam.edge[i] = 0;
  if (c->n_layers > 0) {
    const BlockOff& b0 = c->blocks[0];
    const size_t base = b0.ln1_g;
    c->adam.block_size = b0.b_down + d - base;
    const size_t e[8] = {b0.w_qkv, b0.b_qkv, b0.w_o, b0.b_o, b0.w_up, b0.b_up, b0.w_down, b0.b_down};
    for (int i = 0; i < 8; ++i) c->adam.edge[i] = (unsigned int)(e[i] - base);
    if (c->adam.blocks_end - c->adam.stem_end >= (1ull << 32)) {
      delete c;
      return fail(DIPACO_ESHAPE, "decoder blocks above 2^32 elements in total");
    }
  }
  *out = c;
  return DIPACO_OK;
}

void dipaco_destroy(dipaco_ctx* c) { delete c; }

size_t dipaco_path_param_count(const dipaco_ctx* c) { return c ? c->n_params : 0; }
int32_t dipaco_segment_count(const dipaco_ctx* c) { return c ? (int32_t)c->seg_off.size() : 0; }
size_t dipaco_segment_offset(const dipaco_ctx* c, int32_t s) {
  return (c && s >= 0 && s < (int32_t)c->seg_off.size()) ? c->seg_off[s] : 0;
}
size_t dipaco_segment_size(const dipaco_ctx* c, int32_t s) {
  return (c && s >= 0 && s < (int32_t)c->seg_size.size()) ? c->seg_size[s] : 0;
}
int32_t dipaco_tensor_count(const dipaco_ctx* c) { return c ? (int32_t)c->tensors.size() : 0; }

dipaco_status dipaco_tensor_info(const dipaco_ctx* c, int32_t i, char* name_out, size_t name_cap, size_t* offset,
                                 int64_t* rows, int64_t* cols, int32_t* decayed) {
  if (!c || i < 0 || i >= (int32_t)c->tensors.size()) return fail(DIPACO_EINVAL, "dipaco_tensor_info: bad index");
  const TensorInfo& t = c->tensors[i];
  if (name_out && name_cap) {
    std::strncpy(name_out, t.name.c_str(), name_cap - 1);
    name_out[name_cap - 1] = 0;
  }
  if (offset) *offset = t.off;
  if (rows) *rows = t.rows;
  if (cols) *cols = t.cols;
  if (decayed) *decayed = t.decay ? 1 : 0;
  return DIPACO_OK;
}

int64_t dipaco_path_index(const int32_t* modules, const int32_t* K, int32_t L) {
  if (!modules || !K || L < 1) return -1;
  int64_t j = 0;
  for (int l = 0; l < L; ++l) {
    if (K[l] < 1 || modules[l] < 0 || modules[l] >= K[l]) return -1;
    j = j * K[l] + modules[l];
  }
  return j;
}

dipaco_status dipaco_path_modules(int64_t j, const int32_t* K, int32_t L, int32_t* out) {
  if (!K || !out || L < 1 || j < 0) return fail(DIPACO_EINVAL, "dipaco_path_modules: bad argument");
  for (int l = L - 1; l >= 0; --l) {
    if (K[l] < 1) return fail(DIPACO_EINVAL, "dipaco_path_modules: K must be >= 1");
    out[l] = (int32_t)(j % K[l]);
    j /= K[l];
  }
  if (j != 0) return fail(DIPACO_EINVAL, "dipaco_path_modules: path index out of range");
  return DIPACO_OK;
}

size_t dipaco_workspace_bytes(const dipaco_ctx* c, int32_t batch, int32_t seq) {
  if (!c || batch < 1 || seq < 1) return 0;
  return make_plan(c, batch, seq).total;
}

dipaco_status dipaco_compose_path(dipaco_ctx* c, const float* const* segs, float* master, void* lowp, void* stream) {
  if (!c || !segs) return fail(DIPACO_EINVAL, "dipaco_compose_path: NULL argument");
  TRY(check_ptr(master, "path_master"));
  if (lowp && !aligned16(lowp)) return fail(DIPACO_EALIGN, "path_lowp is not 16-byte aligned");
  const int n = (int)c->seg_off.size();
  for (int s = 0; s < n; ++s)
    if (c->seg_size[s]) TRY(check_ptr(segs[s], "segment pointer"));
  for (int s = 0; s < n; ++s) {
    bf16* lp = lowp ? static_cast<bf16*>(lowp) + c->seg_off[s] : nullptr;
    TRY(launch_copy_cast(segs[s], master + c->seg_off[s], lp, c->seg_size[s], static_cast<hipStream_t>(stream)));
  }
  return DIPACO_OK;
}

dipaco_status dipaco_path_fwd_bwd(dipaco_ctx* c, const float* master, const void* lowp, const int32_t* tokens,
                                  const int32_t* targets, int32_t B, int32_t S, float* loss_out, float* nll_out,
                                  float* grads, void* ws, size_t ws_bytes, void* stream) {
  if (!c) return fail(DIPACO_EINVAL, "dipaco_path_fwd_bwd: NULL context");
  TRY(check_batch_shape(c, B, S, true));
  const bool lowprec = c->arch.compute == DIPACO_BF16;
  TRY(check_ptr(lowprec ? lowp : static_cast<const void*>(master), lowprec ? "path_lowp" : "path_master"));
  TRY(check_ptr(tokens, "tokens"));
  TRY(check_ptr(targets, "targets"));
  TRY(check_ptr(grads, "grads"));
  TRY(check_ptr(ws, "workspace"));
  if (!loss_out) return fail(DIPACO_EINVAL, "loss_out is NULL");
  if (ws_bytes < make_plan(c, B, S).total) return fail(DIPACO_EWORKSPACE, "workspace too small");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (lowprec)
    return run_fwd_bwd<bf16>(c, static_cast<const bf16*>(lowp), tokens, targets, B, S, loss_out, nll_out, grads,
                             static_cast<char*>(ws), st);
  return run_fwd_bwd<float>(c, master, tokens, targets, B, S, loss_out, nll_out, grads, static_cast<char*>(ws), st);
}

size_t dipaco_features_workspace_bytes(const dipaco_ctx* c, int32_t batch, int32_t seq) {
  if (!c || batch < 1 || seq < 1) return 0;
  return make_feature_plan(c, batch, seq).total;
}

dipaco_status dipaco_path_prefix_features(dipaco_ctx* c, const float* master, const void* lowp, const int32_t* tokens,
                                          int32_t B, int32_t S, float* features_out, void* ws, size_t ws_bytes,
                                          void* stream) {
  if (!c) return fail(DIPACO_EINVAL, "dipaco_path_prefix_features: NULL context");
  TRY(check_batch_shape(c, B, S, false));
  const bool lowprec = c->arch.compute == DIPACO_BF16;
  TRY(check_ptr(lowprec ? lowp : static_cast<const void*>(master), lowprec ? "path_lowp" : "path_master"));
  TRY(check_ptr(tokens, "tokens"));
  TRY(check_ptr(features_out, "features_out"));
  TRY(check_ptr(ws, "workspace"));
  if (ws_bytes < make_feature_plan(c, B, S).total) return fail(DIPACO_EWORKSPACE, "workspace too small");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (lowprec) return run_features<bf16>(c, static_cast<const bf16*>(lowp), tokens, nullptr, B, S, features_out, nullptr, static_cast<char*>(ws), st);
  return run_features<float>(c, master, tokens, nullptr, B, S, features_out, nullptr, static_cast<char*>(ws), st);
}

// ---- router features for callers that cannot allocate ------------------------------------------------------
// The activations of dipaco_path_prefix_features live in one file-scope device array instead of a caller's
// workspace.  Every GPU holds its own copy of the array at its own address: the address is looked up once per device
// (with that device current) and only that pointer is ever handed to kernels.
namespace {
constexpr size_t STATIC_SCRATCH_BYTES = DIPACO_STATIC_SCRATCH_BYTES;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
std::mutex g_scratch_mutex;
char* g_scratch_ptr[STATIC_MAX_DEVICES] = {};

dipaco_status static_scratch(char** out) {
  int device = -1;
  DIPACO_HIP(hipGetDevice(&device));
  if (device < 0 || device >= STATIC_MAX_DEVICES) return dipaco::fail(DIPACO_EUNSUPPORTED, "device ordinal above 63");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    DIPACO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return dipaco::fail(DIPACO_EHIP, "static scratch has no usable device address");
    g_scratch_ptr[device] = static_cast<char*>(p);
  }
  *out = g_scratch_ptr[device];
  return DIPACO_OK;
}
}  // namespace

size_t dipaco_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

dipaco_status dipaco_path_prefix_features_static(dipaco_ctx* c, const float* master, const void* lowp,
                                                 const int32_t* tokens, int32_t B, int32_t S, float* features_out,
                                                 void* stream) {
  if (!c) return fail(DIPACO_EINVAL, "dipaco_path_prefix_features_static: NULL context");
  TRY(check_batch_shape(c, B, S, false));
  const size_t need = make_feature_plan(c, B, S).total;
  if (need > STATIC_SCRATCH_BYTES)
    return fail(DIPACO_EWORKSPACE, "dipaco_path_prefix_features_static: this batch x seq needs " + std::to_string(need) +
                                       " bytes of activations, the static scratch holds " +
                                       std::to_string(STATIC_SCRATCH_BYTES) + "; use dipaco_path_prefix_features");
  const bool lowprec = c->arch.compute == DIPACO_BF16;
  TRY(check_ptr(lowprec ? lowp : static_cast<const void*>(master), lowprec ? "path_lowp" : "path_master"));
  TRY(check_ptr(tokens, "tokens"));
  TRY(check_ptr(features_out, "features_out"));
  char* ws = nullptr;
  TRY(static_scratch(&ws));
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (lowprec) return run_features<bf16>(c, static_cast<const bf16*>(lowp), tokens, nullptr, B, S, features_out, nullptr, ws, st);
  return run_features<float>(c, master, tokens, nullptr, B, S, features_out, nullptr, ws, st);
}

size_t dipaco_score_workspace_bytes(const dipaco_ctx* c, int32_t batch, int32_t seq) {
  if (!c || batch < 1 || seq < 1) return 0;
  return make_feature_plan(c, batch, seq, true).total;
}

dipaco_status dipaco_path_score(dipaco_ctx* c, const float* master, const void* lowp, const int32_t* tokens,
                                const int32_t* targets, int32_t B, int32_t S, float* doc_loglik_out, float* nll_out,
                                void* ws, size_t ws_bytes, void* stream) {
  if (!c) return fail(DIPACO_EINVAL, "dipaco_path_score: NULL context");
  TRY(check_batch_shape(c, B, S, true));
  const bool lowprec = c->arch.compute == DIPACO_BF16;
  TRY(check_ptr(lowprec ? lowp : static_cast<const void*>(master), lowprec ? "path_lowp" : "path_master"));
  TRY(check_ptr(tokens, "tokens"));
  TRY(check_ptr(targets, "targets"));
  TRY(check_ptr(doc_loglik_out, "doc_loglik_out"));
  TRY(check_ptr(ws, "workspace"));
  if (ws_bytes < make_feature_plan(c, B, S, true).total) return fail(DIPACO_EWORKSPACE, "workspace too small");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (lowprec) return run_features<bf16>(c, static_cast<const bf16*>(lowp), tokens, targets, B, S, doc_loglik_out, nll_out, static_cast<char*>(ws), st);
  return run_features<float>(c, master, tokens, targets, B, S, doc_loglik_out, nll_out, static_cast<char*>(ws), st);
}

dipaco_status dipaco_inner_adamw(dipaco_ctx* c, float* master, const float* grads, float* m, float* v, void* lowp,
                                 int64_t step, float lr, float beta1, float beta2, float eps, float wd, void* stream) {
  if (!c) return fail(DIPACO_EINVAL, "dipaco_inner_adamw: NULL context");
  if (step < 1) return fail(DIPACO_EINVAL, "step counts from 1");
  if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f)) return fail(DIPACO_EINVAL, "betas must be in [0,1)");
  TRY(check_ptr(master, "path_master"));
  TRY(check_ptr(grads, "grads"));
  TRY(check_ptr(m, "m"));
  TRY(check_ptr(v, "v"));
  if (lowp && !aligned16(lowp)) return fail(DIPACO_EALIGN, "path_lowp is not 16-byte aligned");
  return launch_adamw(master, grads, m, v, static_cast<bf16*>(lowp), c->adam, c->n_params, step, lr, beta1, beta2, eps, wd, static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_module_outer_step(float* theta, float* momentum, const float* const* inputs, const float* weights,
                                       int32_t n_paths, size_t n_elems, int32_t is_delta, float outer_lr,
                                       float outer_momentum, void* stream) {
  if (!inputs) return fail(DIPACO_EINVAL, "inputs is NULL");
  if (n_paths < 1 || n_paths > DIPACO_MAX_PATHS_PER_MODULE)
    return fail(DIPACO_ESHAPE, "n_paths must be in [1, DIPACO_MAX_PATHS_PER_MODULE]");
  TRY(check_ptr(theta, "theta"));
  TRY(check_ptr(momentum, "momentum"));
  for (int i = 0; i < n_paths; ++i) TRY(check_ptr(inputs[i], "input pointer"));
  float alpha[DIPACO_MAX_PATHS_PER_MODULE];
  double sum = 0.0;
  for (int i = 0; i < n_paths; ++i) {
    const double w = weights ? (double)weights[i] : 1.0;
    if (!(w > 0.0) || !std::isfinite(w)) return fail(DIPACO_EINVAL, "weights must be positive and finite");
    sum += w;
  }
  for (int i = 0; i < n_paths; ++i) alpha[i] = (float)((weights ? (double)weights[i] : 1.0) / sum);
  return launch_outer(theta, momentum, inputs, alpha, n_paths, n_elems, is_delta ? 1 : 0, outer_lr, outer_momentum,
                      static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_module_delta_accumulate(float* delta_sum, const float* theta_prev, const float* input, float weight,
                                             size_t n_elems, int32_t is_delta, int32_t first, void* stream) {
  if (!(weight > 0.0f) || !std::isfinite(weight)) return fail(DIPACO_EINVAL, "weight must be positive and finite");
  TRY(check_ptr(delta_sum, "delta_sum"));
  TRY(check_ptr(input, "input"));
  if (!is_delta) TRY(check_ptr(theta_prev, "theta_prev"));
  return launch_delta_accumulate(delta_sum, theta_prev, input, weight, n_elems, is_delta ? 1 : 0, first ? 1 : 0,
                                 static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_module_outer_apply(float* theta, float* momentum, const float* delta_sum, double weight_sum,
                                        float norm_scale, size_t n_elems, float outer_lr, float outer_momentum,
                                        void* stream) {
  if (!(weight_sum > 0.0) || !std::isfinite(weight_sum)) return fail(DIPACO_EINVAL, "weight_sum must be positive and finite");
  if (!(norm_scale > 0.0f) || !std::isfinite(norm_scale)) return fail(DIPACO_EINVAL, "norm_scale must be positive and finite");
  TRY(check_ptr(theta, "theta"));
  TRY(check_ptr(momentum, "momentum"));
  TRY(check_ptr(delta_sum, "delta_sum"));
  return launch_outer_apply(theta, momentum, delta_sum, (float)((double)norm_scale / weight_sum), n_elems, outer_lr,
                            outer_momentum, static_cast<hipStream_t>(stream));
}

// ---- table-driven outer step: image = header | entries | input pointers | alpha ----------------------------
namespace {
struct OuterTableHeader {
  unsigned long long magic, n_modules, total_chunks, total_paths;
};
constexpr unsigned long long OUTER_TABLE_MAGIC = 0x64697061636f5442ull;

size_t outer_table_layout(unsigned long long n_modules, unsigned long long total_paths, size_t& off_inputs,
                          size_t& off_alpha) {
  off_inputs = sizeof(OuterTableHeader) + n_modules * sizeof(dipaco::OuterTableEntry);
  off_alpha = off_inputs + total_paths * sizeof(const float*);
  return (off_alpha + total_paths * sizeof(float) + 15) & ~(size_t)15;
}
}  // namespace

size_t dipaco_outer_table_bytes(const dipaco_module_desc* modules, int32_t n_modules) {
  if (!modules || n_modules < 1) return 0;
  unsigned long long paths = 0;
  for (int m = 0; m < n_modules; ++m) {
    if (modules[m].n_paths < 1 || modules[m].n_paths > DIPACO_MAX_PATHS_PER_MODULE) return 0;
    paths += (unsigned long long)modules[m].n_paths;
  }
  size_t a, b;
  return outer_table_layout((unsigned long long)n_modules, paths, a, b);
}

dipaco_status dipaco_outer_table_pack(const dipaco_module_desc* modules, int32_t n_modules, void* image,
                                      size_t image_bytes) {
  using namespace dipaco;
  if (!modules || !image) return fail(DIPACO_EINVAL, "modules / image is NULL");
  if (n_modules < 1) return fail(DIPACO_EINVAL, "n_modules must be >= 1");
  const size_t need = dipaco_outer_table_bytes(modules, n_modules);
  if (need == 0) return fail(DIPACO_ESHAPE, "n_paths must be in [1, DIPACO_MAX_PATHS_PER_MODULE]");
  if (image_bytes < need) return fail(DIPACO_EWORKSPACE, "table image too small");
  unsigned long long paths = 0;
  for (int m = 0; m < n_modules; ++m) paths += (unsigned long long)modules[m].n_paths;
  size_t off_inputs, off_alpha;
  outer_table_layout((unsigned long long)n_modules, paths, off_inputs, off_alpha);
  char* base = static_cast<char*>(image);
  std::memset(base, 0, need);
  OuterTableEntry* entries = reinterpret_cast<OuterTableEntry*>(base + sizeof(OuterTableHeader));
  const float** inputs = reinterpret_cast<const float**>(base + off_inputs);
  float* alpha = reinterpret_cast<float*>(base + off_alpha);
  unsigned long long chunk = 0, pb = 0;
  for (int m = 0; m < n_modules; ++m) {
    const dipaco_module_desc& d = modules[m];
    if (!d.inputs) return fail(DIPACO_EINVAL, "inputs is NULL");
    TRY(check_ptr(d.theta, "theta"));
    TRY(check_ptr(d.momentum, "momentum"));
    if (!(d.norm_scale > 0.0f) || !std::isfinite(d.norm_scale))
      return fail(DIPACO_EINVAL, "norm_scale must be positive and finite");
    double sum = 0.0;
    for (int i = 0; i < d.n_paths; ++i) {
      TRY(check_ptr(d.inputs[i], "input pointer"));
      const double w = d.weights ? (double)d.weights[i] : 1.0;
      if (!(w > 0.0) || !std::isfinite(w)) return fail(DIPACO_EINVAL, "weights must be positive and finite");
      sum += w;
    }
    for (int i = 0; i < d.n_paths; ++i) {
      inputs[pb + i] = d.inputs[i];
      alpha[pb + i] = (float)((double)d.norm_scale * (d.weights ? (double)d.weights[i] : 1.0) / sum);
    }
    OuterTableEntry& e = entries[m];
    e.theta = d.theta; e.momentum = d.momentum; e.n_elems = d.n_elems; e.first_chunk = chunk; e.path_begin = pb;
    e.n_paths = d.n_paths; e.is_delta = d.is_delta ? 1 : 0;
    chunk += (d.n_elems + OUTER_CHUNK - 1) / OUTER_CHUNK;
    pb += (unsigned long long)d.n_paths;
  }
  OuterTableHeader* h = reinterpret_cast<OuterTableHeader*>(base);
  h->magic = OUTER_TABLE_MAGIC; h->n_modules = (unsigned long long)n_modules; h->total_chunks = chunk; h->total_paths = paths;
  return DIPACO_OK;
}

dipaco_status dipaco_outer_step_table(const void* table_host, const void* table_device, size_t table_bytes,
                                      float outer_lr, float outer_momentum, void* stream) {
  using namespace dipaco;
  if (!table_host || !table_device) return fail(DIPACO_EINVAL, "table is NULL");
  if ((uintptr_t)table_device % 8) return fail(DIPACO_EALIGN, "device table is not 8-byte aligned");
  if (table_bytes < sizeof(OuterTableHeader)) return fail(DIPACO_EINVAL, "table image too small");
  const OuterTableHeader* h = static_cast<const OuterTableHeader*>(table_host);
  if (h->magic != OUTER_TABLE_MAGIC) return fail(DIPACO_EINVAL, "not a table image written by dipaco_outer_table_pack");
  size_t off_inputs, off_alpha;
  if (h->n_modules > 0x7fffffffull || outer_table_layout(h->n_modules, h->total_paths, off_inputs, off_alpha) > table_bytes)
    return fail(DIPACO_EINVAL, "table image does not match its size");
  const char* dev = static_cast<const char*>(table_device);
  return launch_outer_table(reinterpret_cast<const OuterTableEntry*>(dev + sizeof(OuterTableHeader)),
                            reinterpret_cast<const float* const*>(dev + off_inputs),
                            reinterpret_cast<const float*>(dev + off_alpha), (int)h->n_modules, h->total_chunks, outer_lr,
                            outer_momentum, static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_route_prefix(const float* z, const float* centroids, int64_t N, int32_t D, int32_t K,
                                  int32_t* idx_out, int64_t* hist_out, float* margin_out, void* stream) {
  if (N < 0) return fail(DIPACO_EINVAL, "N must be >= 0");
  if (D < 4 || D % 4) return fail(DIPACO_ESHAPE, "D must be a positive multiple of 4");
  if (K < 1 || K > 4096) return fail(DIPACO_ESHAPE, "K must be in [1, 4096]");
  TRY(check_ptr(centroids, "centroids"));
  TRY(check_ptr(hist_out, "hist_out"));
  if (N > 0) {
    TRY(check_ptr(z, "z"));
    TRY(check_ptr(idx_out, "idx_out"));
  }
  return launch_route(z, D, centroids, nullptr, N, D, K, 1, idx_out, reinterpret_cast<long long*>(hist_out), margin_out,
                      static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_route_prefix_top(const float* z, int64_t ldz, const float* centroids, int64_t N, int32_t D,
                                      int32_t K, int32_t n_best, int32_t* idx_out, int64_t* hist_out, float* margin_out,
                                      void* stream) {
  if (N < 0) return fail(DIPACO_EINVAL, "N must be >= 0");
  if (D < 4 || D % 4) return fail(DIPACO_ESHAPE, "D must be a positive multiple of 4");
  if (ldz < D || ldz % 4) return fail(DIPACO_ESHAPE, "ldz must be a multiple of 4, at least D");
  if (K < 1 || K > 4096) return fail(DIPACO_ESHAPE, "K must be in [1, 4096]");
  if (n_best != 1 && n_best != 2) return fail(DIPACO_EINVAL, "n_best must be 1 or 2");
  TRY(check_ptr(centroids, "centroids"));
  TRY(check_ptr(hist_out, "hist_out"));
  if (N > 0) {
    TRY(check_ptr(z, "z"));
    TRY(check_ptr(idx_out, "idx_out"));
  }
  return launch_route(z, ldz, centroids, nullptr, N, D, K, n_best, idx_out, reinterpret_cast<long long*>(hist_out),
                      margin_out, static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_route_linear(const float* z, int64_t ldz, const float* weights, const float* bias, int64_t N, int32_t D,
                                  int32_t K, int32_t* idx_out, int64_t* hist_out, float* margin_out, void* stream) {
  if (N < 0) return fail(DIPACO_EINVAL, "N must be >= 0");
  if (D < 4 || D % 4) return fail(DIPACO_ESHAPE, "D must be a positive multiple of 4");
  if (ldz < D || ldz % 4) return fail(DIPACO_ESHAPE, "ldz must be a multiple of 4, at least D");
  if (K < 1 || K > 4096) return fail(DIPACO_ESHAPE, "K must be in [1, 4096]");
  TRY(check_ptr(weights, "weights"));
  TRY(check_ptr(bias, "bias"));
  TRY(check_ptr(hist_out, "hist_out"));
  if (N > 0) {
    TRY(check_ptr(z, "z"));
    TRY(check_ptr(idx_out, "idx_out"));
  }
  return launch_route(z, ldz, weights, bias, N, D, K, 1, idx_out, reinterpret_cast<long long*>(hist_out), margin_out,
                      static_cast<hipStream_t>(stream));
}

namespace {
struct RouterPlan { size_t logits, nll, n_valid, cs_partial, sk_partial, total; };
RouterPlan make_router_plan(int64_t N, int D, int K) {
  RouterPlan p;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
  p.logits = take((size_t)N * K * 4);
  p.nll = take((size_t)N * 4);
  p.n_valid = take(256);
  p.cs_partial = take(dipaco::colsum_partial_floats((int)N, K) * 4);
  p.sk_partial = take((size_t)dipaco::gemm_max_splits(K, D, (int)N) * K * D * 4);
  p.total = off;
  return p;
}
dipaco_status check_router_shape(int64_t N, int D, int K) {
  using namespace dipaco;
  if (N < 1 || N > 0x7fffffffLL) return fail(DIPACO_ESHAPE, "N must be in [1, 2^31)");
  if (D < 8 || D % 8) return fail(DIPACO_ESHAPE, "D must be a positive multiple of 8");
  if (K < 8 || K % 8 || K > 4096) return fail(DIPACO_ESHAPE, "K must be a multiple of 8 in [8, 4096]");
  if ((int64_t)N * std::max(D, K) >= (1LL << 32)) return fail(DIPACO_ESHAPE, "N * max(D, K) must stay below 2^32");
  return DIPACO_OK;
}
}  // namespace

size_t dipaco_router_workspace_bytes(int64_t N, int32_t D, int32_t K) {
  if (check_router_shape(N, D, K) != DIPACO_OK) return 0;
  return make_router_plan(N, D, K).total;
}

dipaco_status dipaco_router_logistic_grad(const float* z, const int32_t* labels, const float* weights, const float* bias,
                                          int64_t N, int32_t D, int32_t K, float* loss_out, float* dweights_out,
                                          float* dbias_out, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace dipaco;
  TRY(check_router_shape(N, D, K));
  TRY(check_ptr(z, "z"));
  TRY(check_ptr(labels, "labels"));
  TRY(check_ptr(weights, "weights"));
  TRY(check_ptr(bias, "bias"));
  TRY(check_ptr(loss_out, "loss_out"));
  TRY(check_ptr(dbias_out, "dbias_out"));
  if (dweights_out) TRY(check_ptr(dweights_out, "dweights_out"));
  TRY(check_ptr(workspace, "workspace"));
  const RouterPlan p = make_router_plan(N, D, K);
  if (workspace_bytes < p.total) return fail(DIPACO_EWORKSPACE, "workspace smaller than dipaco_router_workspace_bytes");
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  float* logits = reinterpret_cast<float*>(ws + p.logits);
  float* nll = reinterpret_cast<float*>(ws + p.nll);
  int* n_valid = reinterpret_cast<int*>(ws + p.n_valid);
  // logits = z W^T + b;  then per row the loss and (softmax - onehot) / N in place
  TRY(gemm<float>(z, weights, logits, (int)N, K, D, D, D, K, false, true, bias, nullptr, nullptr, nullptr, 0, false, 1,
                  nullptr, st));
  TRY(launch_logistic_rows(logits, labels, N, K, (float)(1.0 / (double)N), nll, st));
  TRY(launch_fill_i32(n_valid, (int)N, 1, st));
  TRY(launch_mean_loss(nll, n_valid, loss_out, (int)N, st));
  // db = column sums;  dW = dlogits^T z (contraction over the documents)
  TRY(launch_colsum<float>(logits, dbias_out, reinterpret_cast<float*>(ws + p.cs_partial), (int)N, K, st));
  if (dweights_out)
    TRY(gemm<float>(logits, z, dweights_out, K, D, (int)N, K, D, D, true, false, nullptr, nullptr, nullptr, nullptr, 0,
                    true, gemm_plan_splits(K, D, (int)N, false), reinterpret_cast<float*>(ws + p.sk_partial), st));
  return DIPACO_OK;
}

namespace {
dipaco_status check_reroute_shape(int32_t P, int32_t B, int32_t S) {
  using namespace dipaco;
  if (P < 1 || P > 4096) return fail(DIPACO_ESHAPE, "n_paths must be in [1, 4096]");
  if (B < 1 || S < 1) return fail(DIPACO_ESHAPE, "batch and seq must be positive");
  if ((int64_t)P * B > 0x7fffffffLL || (int64_t)B * S > 0x7fffffffLL * 128)
    return fail(DIPACO_ESHAPE, "n_paths * batch and batch * seq are too large");
  return DIPACO_OK;
}
}  // namespace

size_t dipaco_reroute_workspace_bytes(int32_t n_paths, int32_t batch, int32_t seq) {
  if (check_reroute_shape(n_paths, batch, seq) != DIPACO_OK) return 0;
  return dipaco::reroute_prefix_doubles(n_paths, batch, seq) * sizeof(double);
}

dipaco_status dipaco_window_targets(const float* token_nll, int32_t n_paths, int32_t batch, int32_t seq, int32_t window,
                                    int32_t* targets_out, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace dipaco;
  TRY(check_reroute_shape(n_paths, batch, seq));
  if (window < 1) return fail(DIPACO_EINVAL, "window must be >= 1");
  TRY(check_ptr(token_nll, "token_nll"));
  TRY(check_ptr(targets_out, "targets_out"));
  TRY(check_ptr(workspace, "workspace"));
  if (workspace_bytes < dipaco_reroute_workspace_bytes(n_paths, batch, seq))
    return fail(DIPACO_EWORKSPACE, "workspace smaller than dipaco_reroute_workspace_bytes");
  return launch_window_targets(token_nll, n_paths, batch, seq, window, targets_out, static_cast<double*>(workspace),
                               static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_chunk_routed_score(const float* token_nll, const int32_t* chunk_path, int32_t n_paths, int32_t batch,
                                        int32_t seq, int32_t chunk, float* doc_loglik_out, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  using namespace dipaco;
  TRY(check_reroute_shape(n_paths, batch, seq));
  if (chunk < 1) return fail(DIPACO_EINVAL, "chunk must be >= 1");
  TRY(check_ptr(token_nll, "token_nll"));
  TRY(check_ptr(chunk_path, "chunk_path"));
  TRY(check_ptr(doc_loglik_out, "doc_loglik_out"));
  TRY(check_ptr(workspace, "workspace"));
  if (workspace_bytes < dipaco_reroute_workspace_bytes(n_paths, batch, seq))
    return fail(DIPACO_EWORKSPACE, "workspace smaller than dipaco_reroute_workspace_bytes");
  return launch_chunk_score(token_nll, chunk_path, n_paths, batch, seq, chunk, doc_loglik_out,
                            static_cast<double*>(workspace), static_cast<hipStream_t>(stream));
}

size_t dipaco_kmeans_workspace_bytes(int64_t N, int32_t D, int32_t K) {
  if (N < 0 || D < 1 || K < 1) return 0;
  return kmeans_workspace_bytes((long)N, D, K);
}

dipaco_status dipaco_kmeans_update(const float* z, int64_t ldz, const int32_t* idx, int64_t N, int32_t D, int32_t K,
                                   float* centroids, int64_t* counts_out, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  if (N < 0 || N > 0x7fff0000LL) return fail(DIPACO_EINVAL, "N must be in [0, 2^31 - 65536]");
  if (D < 4 || D % 4) return fail(DIPACO_ESHAPE, "D must be a positive multiple of 4");
  if (ldz < D || ldz % 4) return fail(DIPACO_ESHAPE, "ldz must be a multiple of 4, at least D");
  if (K < 1 || K > 4096) return fail(DIPACO_ESHAPE, "K must be in [1, 4096]");
  TRY(check_ptr(centroids, "centroids"));
  TRY(check_ptr(workspace, "workspace"));
  if (workspace_bytes < kmeans_workspace_bytes((long)N, D, K)) return fail(DIPACO_EWORKSPACE, "workspace too small");
  if (N > 0) {
    TRY(check_ptr(z, "z"));
    TRY(check_ptr(idx, "idx"));
  }
  return launch_kmeans_update(z, (long)ldz, idx, (long)N, D, K, centroids, reinterpret_cast<long long*>(counts_out),
                              workspace, static_cast<hipStream_t>(stream));
}

// ---- kernel-level entry points (include/dipaco_kernels.h) -------------------------------------------------
dipaco_status dipaco_k_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t out_f32, int32_t M, int32_t N,
                            int32_t K, const void* A, const void* B, void* C, const void* bias, const void* resid,
                            void* aux_out, const void* aux_in, int32_t act, int32_t splits, float* partial,
                            void* stream) {
  GemmArgs g;
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K;
  g.lda = trans_a ? M : K; g.ldb = trans_b ? K : N; g.ldc = N;
  g.bias = bias; g.resid = resid; g.aux_out = aux_out; g.aux_in = aux_in; g.act = act;
  g.trans_a = trans_a; g.trans_b = trans_b; g.out_f32 = out_f32; g.splits = splits; g.partial = partial;
  if (!A || !B || !C) return fail(DIPACO_EINVAL, "dipaco_k_gemm: NULL operand");
  hipStream_t st = static_cast<hipStream_t>(stream);
  return dtype == DIPACO_BF16 ? launch_gemm<bf16>(g, st) : launch_gemm<float>(g, st);
}

dipaco_status dipaco_k_gemm_colsum(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                                   const void* A, const void* B, void* C, const void* bias, const void* resid,
                                   void* aux_out, const void* aux_in, int32_t act, float* colsum_out,
                                   float* colsum_scratch, void* stream) {
  GemmArgs g;
  g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K;
  g.lda = trans_a ? M : K; g.ldb = trans_b ? K : N; g.ldc = N;
  g.bias = bias; g.resid = resid; g.aux_out = aux_out; g.aux_in = aux_in; g.act = act;
  g.trans_a = trans_a; g.trans_b = trans_b; g.out_f32 = 0; g.splits = 1; g.partial = nullptr;
  g.colsum = colsum_out; g.colsum_partial = colsum_scratch;
  if (!A || !B || !C || !colsum_out || !colsum_scratch) return fail(DIPACO_EINVAL, "dipaco_k_gemm_colsum: NULL argument");
  hipStream_t st = static_cast<hipStream_t>(stream);
  return dtype == DIPACO_BF16 ? launch_gemm<bf16>(g, st) : launch_gemm<float>(g, st);
}

dipaco_status dipaco_k_set_gemm_tile(int32_t tile) {
  if (tile < 0 || tile > 13) return fail(DIPACO_EINVAL, "dipaco_k_set_gemm_tile: tile must be 0..13");
  set_gemm_tile(tile);
  return DIPACO_OK;
}

dipaco_status dipaco_k_gemm_split_plan(int32_t M, int32_t N, int32_t K, int32_t max_slices, int32_t* out) {
  if (!out || M < 1 || N < 1 || K < 32 || K % 32) return fail(DIPACO_EINVAL, "dipaco_k_gemm_split_plan: bad argument");
  gemm_dlds_plan_info(M, N, K, max_slices, out);
  return DIPACO_OK;
}

dipaco_status dipaco_k_set_attention_blocks(int32_t single_block) {
  if (single_block != 0 && single_block != 1) return fail(DIPACO_EINVAL, "dipaco_k_set_attention_blocks: 0 or 1");
  set_attention_single_block(single_block);
  return DIPACO_OK;
}

dipaco_status dipaco_k_issue_probe(int32_t mode, int32_t waves_per_simd, int32_t iters, float* out, void* stream) {
  if (mode < 0 || mode > 8 || waves_per_simd < 1 || waves_per_simd > 4 || iters < 1 || !out)
    return fail(DIPACO_EINVAL, "dipaco_k_issue_probe: mode 0..8, waves_per_simd 1..4, iters >= 1, out not NULL");
  return launch_issue_probe(mode, waves_per_simd, iters, out, static_cast<hipStream_t>(stream));
}

dipaco_status dipaco_k_attention_fwd(int32_t dtype, const void* qkv, void* o, float* lse, int32_t B, int32_t S,
                                     int32_t H, int32_t dh, void* stream) {
  if (!qkv || !o || !lse || B < 1 || S < 1 || H < 1) return fail(DIPACO_EINVAL, "dipaco_k_attention_fwd: bad argument");
  if ((int64_t)S * 3 * H * dh * 2 >= (1LL << 32) || (int64_t)B * S * 3 * H * dh >= (1LL << 32))
    return fail(DIPACO_ESHAPE, "dipaco_k_attention_fwd: sequence or batch too large for 32-bit offsets");
  hipStream_t st = static_cast<hipStream_t>(stream);
  return dtype == DIPACO_BF16
             ? launch_attention_fwd<bf16>(static_cast<const bf16*>(qkv), static_cast<bf16*>(o), lse, B, S, H, dh, st)
             : launch_attention_fwd<float>(static_cast<const float*>(qkv), static_cast<float*>(o), lse, B, S, H, dh, st);
}

dipaco_status dipaco_k_attention_bwd(int32_t dtype, const void* qkv, const void* o, const void* d_o, const float* lse,
                                     void* dqkv, float* dsum, float* colsum_out, float* colsum_scratch, int32_t B,
                                     int32_t S, int32_t H, int32_t dh, void* stream) {
  if (!qkv || !o || !d_o || !lse || !dqkv || !dsum || B < 1 || S < 1 || H < 1 || (colsum_out && !colsum_scratch))
    return fail(DIPACO_EINVAL, "dipaco_k_attention_bwd: bad argument");
  if ((int64_t)S * 3 * H * dh * 2 >= (1LL << 32) || (int64_t)B * S * 3 * H * dh >= (1LL << 32))
    return fail(DIPACO_ESHAPE, "dipaco_k_attention_bwd: sequence or batch too large for 32-bit offsets");
  hipStream_t st = static_cast<hipStream_t>(stream);
  return dtype == DIPACO_BF16
             ? launch_attention_bwd<bf16>(static_cast<const bf16*>(qkv), static_cast<const bf16*>(o),
                                          static_cast<const bf16*>(d_o), lse, static_cast<bf16*>(dqkv), dsum, colsum_out,
                                          colsum_scratch, B, S, H, dh, st)
             : launch_attention_bwd<float>(static_cast<const float*>(qkv), static_cast<const float*>(o),
                                           static_cast<const float*>(d_o), lse, static_cast<float*>(dqkv), dsum, colsum_out,
                                           colsum_scratch, B, S, H, dh, st);
}

}  // extern "C"
