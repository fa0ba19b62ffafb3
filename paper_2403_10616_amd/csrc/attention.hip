// Causal self-attention, forward and backward, on the packed QKV buffer.
//
// Layout: qkv is [B*S, 3A] with A = H*dh; row t holds q (columns 0..A), k (A..2A), v (2A..3A); head h owns
// columns h*dh..(h+1)*dh of each third.  o and d_o are [B*S, A].  lse[b,h,i] = log sum_j exp(s_ij).
//
// Reference kernels ("scalar" path): one thread per query row (forward, dQ) or per key row (dK, dV), fp32
// arithmetic, online softmax, no atomics, so every output element is produced by one thread in a fixed order.
// They serve fp32 runs and head sizes 32 / 128; bf16 with head size 64 runs on the matrix cores
// (attention_mfma.hip).
#include "kernels.h"

namespace dipaco {

namespace {

constexpr int ATT_THREADS = 64;

template <typename T, int DH>
__global__ void __launch_bounds__(ATT_THREADS) attn_fwd_scalar(const T* __restrict__ qkv, T* __restrict__ o,
                                                               float* __restrict__ lse, int S, int H) {
  constexpr int VEC = Vec16<T>::N;
  const int bh = blockIdx.x, b = bh / H, h = bh % H;
  const int i = blockIdx.y * ATT_THREADS + threadIdx.x;
  if (i >= S) return;
  const int A = H * DH;
  const size_t ld = 3 * (size_t)A;
  const T* base = qkv + (size_t)b * S * ld + h * DH;
  const float scale = rsqrtf((float)DH);
  float q[DH], acc[DH];
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    float t[VEC];
    load_vec16(base + (size_t)i * ld + c, t);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { q[c + e] = t[e] * scale; acc[c + e] = 0.f; }
  }
  float m = -INFINITY, l = 0.f;
  for (int j = 0; j <= i; ++j) {
    const T* kr = base + (size_t)j * ld + A;
    const T* vr = kr + A;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
      float t[VEC];
      load_vec16(kr + c, t);
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += q[c + e] * t[e];
    }
    const float mn = fmaxf(m, s);
    const float corr = expf(m - mn);   // exp(-inf) = 0 on the first key
    const float p = expf(s - mn);
    l = l * corr + p;
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
      float t[VEC];
      load_vec16(vr + c, t);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[c + e] = acc[c + e] * corr + p * t[e];
    }
    m = mn;
  }
  const float inv = 1.0f / l;
  T* orow = o + ((size_t)b * S + i) * A + h * DH;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    float t[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) t[e] = acc[c + e] * inv;
    store_vec16(orow + c, t);
  }
  lse[((size_t)b * H + h) * S + i] = m + logf(l);
}

// dQ_i = scale * sum_{j<=i} p_ij (dO_i.v_j - D_i) k_j, with D_i = dO_i.o_i (also stored for the dK/dV kernel)
template <typename T, int DH>
__global__ void __launch_bounds__(ATT_THREADS) attn_bwd_dq_scalar(const T* __restrict__ qkv, const T* __restrict__ o,
                                                                  const T* __restrict__ d_o,
                                                                  const float* __restrict__ lse, T* __restrict__ dqkv,
                                                                  float* __restrict__ dsum, int S, int H) {
  constexpr int VEC = Vec16<T>::N;
  const int bh = blockIdx.x, b = bh / H, h = bh % H;
  const int i = blockIdx.y * ATT_THREADS + threadIdx.x;
  if (i >= S) return;
  const int A = H * DH;
  const size_t ld = 3 * (size_t)A;
  const T* base = qkv + (size_t)b * S * ld + h * DH;
  const float scale = rsqrtf((float)DH);
  float q[DH], go[DH], acc[DH];
  float D = 0.f;
  const T* orow = o + ((size_t)b * S + i) * A + h * DH;
  const T* gorow = d_o + ((size_t)b * S + i) * A + h * DH;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    float t[VEC], u[VEC], w[VEC];
    load_vec16(base + (size_t)i * ld + c, t);
    load_vec16(gorow + c, u);
    load_vec16(orow + c, w);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { q[c + e] = t[e] * scale; go[c + e] = u[e]; D += u[e] * w[e]; acc[c + e] = 0.f; }
  }
  const float L = lse[((size_t)b * H + h) * S + i];
  dsum[((size_t)b * H + h) * S + i] = D;
  for (int j = 0; j <= i; ++j) {
    const T* kr = base + (size_t)j * ld + A;
    const T* vr = kr + A;
    float s = 0.f, dp = 0.f;
    float kk[DH];
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
      float t[VEC], u[VEC];
      load_vec16(kr + c, t);
      load_vec16(vr + c, u);
#pragma unroll
      for (int e = 0; e < VEC; ++e) { kk[c + e] = t[e]; s += q[c + e] * t[e]; dp += go[c + e] * u[e]; }
    }
    const float ds = expf(s - L) * (dp - D) * scale;
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] += ds * kk[c];
  }
  T* out = dqkv + ((size_t)b * S + i) * ld + h * DH;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    float t[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) t[e] = acc[c + e];
    store_vec16(out + c, t);
  }
}

// dV_j = sum_{i>=j} p_ij dO_i;  dK_j = scale * sum_{i>=j} p_ij (dO_i.v_j - D_i) q_i
template <typename T, int DH>
__global__ void __launch_bounds__(ATT_THREADS) attn_bwd_dkv_scalar(const T* __restrict__ qkv, const T* __restrict__ d_o,
                                                                   const float* __restrict__ lse,
                                                                   const float* __restrict__ dsum, T* __restrict__ dqkv,
                                                                   int S, int H) {
  constexpr int VEC = Vec16<T>::N;
  const int bh = blockIdx.x, b = bh / H, h = bh % H;
  const int j = blockIdx.y * ATT_THREADS + threadIdx.x;
  if (j >= S) return;
  const int A = H * DH;
  const size_t ld = 3 * (size_t)A;
  const T* base = qkv + (size_t)b * S * ld + h * DH;
  const float scale = rsqrtf((float)DH);
  float k[DH], v[DH], dk[DH], dv[DH];
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    float t[VEC], u[VEC];
    load_vec16(base + (size_t)j * ld + A + c, t);
    load_vec16(base + (size_t)j * ld + 2 * A + c, u);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { k[c + e] = t[e]; v[c + e] = u[e]; dk[c + e] = 0.f; dv[c + e] = 0.f; }
  }
  const float* Lrow = lse + ((size_t)b * H + h) * S;
  const float* Drow = dsum + ((size_t)b * H + h) * S;
  for (int i = j; i < S; ++i) {
    const T* qr = base + (size_t)i * ld;
    const T* gor = d_o + ((size_t)b * S + i) * A + h * DH;
    float qq[DH], gg[DH];
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
      float t[VEC], u[VEC];
      load_vec16(qr + c, t);
      load_vec16(gor + c, u);
#pragma unroll
      for (int e = 0; e < VEC; ++e) { qq[c + e] = t[e]; gg[c + e] = u[e]; s += t[e] * k[c + e]; dp += u[e] * v[c + e]; }
    }
    const float p = expf(s * scale - Lrow[i]);
    const float ds = p * (dp - Drow[i]) * scale;
#pragma unroll
    for (int c = 0; c < DH; ++c) { dv[c] += p * gg[c]; dk[c] += ds * qq[c]; }
  }
  T* outk = dqkv + ((size_t)b * S + j) * ld + A + h * DH;
  T* outv = outk + A;
#pragma unroll
  for (int c = 0; c < DH; c += VEC) {
    float t[VEC], u[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { t[e] = dk[c + e]; u[e] = dv[c + e]; }
    store_vec16(outk + c, t);
    store_vec16(outv + c, u);
  }
}

template <typename T, int DH>
dipaco_status fwd_scalar(const T* qkv, T* o, float* lse, int B, int S, int H, hipStream_t s) {
  dim3 grid(B * H, (S + ATT_THREADS - 1) / ATT_THREADS);
  attn_fwd_scalar<T, DH><<<grid, ATT_THREADS, 0, s>>>(qkv, o, lse, S, H);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}
template <typename T, int DH>
dipaco_status bwd_scalar(const T* qkv, const T* o, const T* d_o, const float* lse, T* dqkv, float* dsum, int B, int S,
                         int H, hipStream_t s) {
  dim3 grid(B * H, (S + ATT_THREADS - 1) / ATT_THREADS);
  attn_bwd_dq_scalar<T, DH><<<grid, ATT_THREADS, 0, s>>>(qkv, o, d_o, lse, dqkv, dsum, S, H);
  DIPACO_LAUNCH_CHECK();
  attn_bwd_dkv_scalar<T, DH><<<grid, ATT_THREADS, 0, s>>>(qkv, d_o, lse, dsum, dqkv, S, H);
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace

template <typename T> constexpr bool is_bf16() { return sizeof(T) == 2; }

template <typename T>
dipaco_status launch_attention_fwd(const T* qkv, T* o, float* lse, int B, int S, int H, int dh, hipStream_t s) {
  if (is_bf16<T>() && dh == 64)
    return launch_attention_fwd_mfma(reinterpret_cast<const bf16*>(qkv), reinterpret_cast<bf16*>(o), lse, B, S, H, s);
  switch (dh) {
    case 32: return fwd_scalar<T, 32>(qkv, o, lse, B, S, H, s);
    case 64: return fwd_scalar<T, 64>(qkv, o, lse, B, S, H, s);
    case 128: return fwd_scalar<T, 128>(qkv, o, lse, B, S, H, s);
  }
  return fail(DIPACO_ESHAPE, "attention: d_head must be 32, 64 or 128");
}

size_t attention_bwd_colsum_floats(int B, int S, int H, int dh) {
  return std::max(colsum_partial_floats(B * S, 3 * H * dh), dh == 64 ? attention_colsum_partial_floats(B, S, H) : 0);
}

template <typename T>
dipaco_status launch_attention_bwd(const T* qkv, const T* o, const T* d_o, const float* lse, T* dqkv, float* dsum,
                                   float* colsum_out, float* colsum_partial, int B, int S, int H, int dh,
                                   hipStream_t s, SumBatch* batch) {
  if (is_bf16<T>() && dh == 64)   // the matrix-core kernels take the column sums in their epilogues
    return launch_attention_bwd_mfma(reinterpret_cast<const bf16*>(qkv), reinterpret_cast<const bf16*>(o),
                                     reinterpret_cast<const bf16*>(d_o), lse, reinterpret_cast<bf16*>(dqkv), dsum,
                                     colsum_out, colsum_partial, B, S, H, s, batch);
  dipaco_status st;
  switch (dh) {
    case 32: st = bwd_scalar<T, 32>(qkv, o, d_o, lse, dqkv, dsum, B, S, H, s); break;
    case 64: st = bwd_scalar<T, 64>(qkv, o, d_o, lse, dqkv, dsum, B, S, H, s); break;
    case 128: st = bwd_scalar<T, 128>(qkv, o, d_o, lse, dqkv, dsum, B, S, H, s); break;
    default: return fail(DIPACO_ESHAPE, "attention: d_head must be 32, 64 or 128");
  }
  if (st != DIPACO_OK || !colsum_out) return st;
  return launch_colsum<T>(dqkv, colsum_out, colsum_partial, B * S, 3 * H * dh, s);
}

template dipaco_status launch_attention_fwd<float>(const float*, float*, float*, int, int, int, int, hipStream_t);
template dipaco_status launch_attention_fwd<bf16>(const bf16*, bf16*, float*, int, int, int, int, hipStream_t);
template dipaco_status launch_attention_bwd<float>(const float*, const float*, const float*, const float*, float*,
                                                   float*, float*, float*, int, int, int, int, hipStream_t, SumBatch*);
template dipaco_status launch_attention_bwd<bf16>(const bf16*, const bf16*, const bf16*, const float*, bf16*, float*,
                                                  float*, float*, int, int, int, int, hipStream_t, SumBatch*);

}  // namespace dipaco
