// Shared device/host helpers for the gfx950 kernels of libdipaco.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <string>

#include "../../include/dipaco.h"

namespace dipaco {

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int WAVE = 64;

// ---- error plumbing (host) -------------------------------------------------------------------------
void set_error(const std::string& msg);
dipaco_status fail(dipaco_status st, const std::string& msg);
dipaco_status check_hip(hipError_t e, const char* what);
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define DIPACO_HIP(call)                                              \
  do {                                                                \
    dipaco_status _st = ::dipaco::check_hip((call), #call);           \
    if (_st != DIPACO_OK) return _st;                                 \
  } while (0)
#define DIPACO_LAUNCH_CHECK() DIPACO_HIP(hipGetLastError())

// Raises a kernel's dynamic-LDS limit to `bytes`, once per device: `done` is a call site's own bit mask of the
// devices already served.  Host threads may race here; the worst case is a repeated, identical attribute call.
inline dipaco_status ensure_dynamic_lds(const void* kernel, int bytes, std::atomic<unsigned long long>& done) {
  int device = 0;
  DIPACO_HIP(hipGetDevice(&device));
  const unsigned long long bit = 1ull << (device & 63);
  if (done.load(std::memory_order_acquire) & bit) return DIPACO_OK;
  DIPACO_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  done.fetch_or(bit, std::memory_order_release);
  return DIPACO_OK;
}

// ---- scalar conversions (device) -------------------------------------------------------------------
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return static_cast<float>(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return static_cast<bf16>(x); }  // RNE

// 16-byte vector of T: 4 floats or 8 bf16
template <typename T> struct Vec16;
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16> { static constexpr int N = 8; };

template <typename T>
__device__ __forceinline__ void load_vec16(const T* p, float (&out)[Vec16<T>::N]) {
  uint4 raw = *reinterpret_cast<const uint4*>(p);
  const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
  for (int i = 0; i < Vec16<T>::N; ++i) out[i] = to_f32(e[i]);
}
template <typename T>
__device__ __forceinline__ void store_vec16(T* p, const float (&in)[Vec16<T>::N]) {
  uint4 raw;
  T* e = reinterpret_cast<T*>(&raw);
#pragma unroll
  for (int i = 0; i < Vec16<T>::N; ++i) e[i] = from_f32<T>(in[i]);
  *reinterpret_cast<uint4*>(p) = raw;
}

// exact GELU and its derivative
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752f));
  float pdf = 0.39894228040143268f * __expf(-0.5f * u * u);
  return cdf + u * pdf;
}

// The same two functions for kernels whose result is rounded to bf16.  erf comes from the rational approximation
// 7.1.26 of Abramowitz & Stegun, erfc(z) = (a1 t + ... + a5 t^5) exp(-z^2), t = 1 / (1 + p z), z >= 0, whose
// absolute error is below 1.5e-7 (fp32 rounding of a value near 1, 1/10000 of a bf16 rounding step); it costs one
// reciprocal and one exponential, and the exponential exp(-u^2 / 2) is the one the derivative's density term needs.
// The lower tail is formed as 0.5 erfc(z) directly, without cancellation.
__device__ __forceinline__ void normal_cdf_fast(float u, float& cdf, float& gauss) {
  // constants folded: t = 1 / (1 + p |u| / sqrt 2); the polynomial carries the factor 0.5; exp(-u^2 / 2) = 2^(-w^2) with
  // w = u sqrt(log2(e) / 2)
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(fabsf(u), 0.3275911f * 0.70710678118654752f, 1.0f));
  float poly = __builtin_fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
  poly = __builtin_fmaf(poly, t, 0.5f * 1.421413741f);
  poly = __builtin_fmaf(poly, t, 0.5f * -0.284496736f);
  poly = __builtin_fmaf(poly, t, 0.5f * 0.254829592f);
  const float w = u * 0.84932180028801904f;                       // sqrt(log2(e) / 2)
  gauss = __builtin_amdgcn_exp2f(-(w * w));                       // exp(-u^2 / 2)
  const float q = poly * t * gauss;                               // 0.5 erfc(|u| / sqrt 2)
  cdf = u >= 0.f ? 1.0f - q : q;
}
template <typename T> __device__ __forceinline__ float gelu_t(float u);
template <> __device__ __forceinline__ float gelu_t<float>(float u) { return gelu_f(u); }
template <> __device__ __forceinline__ float gelu_t<bf16>(float u) {
  float cdf, gauss;
  normal_cdf_fast(u, cdf, gauss);
  return u * cdf;
}
// GELU(u) and GELU'(u) together (they share the normal distribution function and density)
template <typename T> __device__ __forceinline__ float gelu_with_grad_t(float u, float& grad);
template <> __device__ __forceinline__ float gelu_with_grad_t<float>(float u, float& grad) {
  const float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752f));
  grad = cdf + u * 0.39894228040143268f * __expf(-0.5f * u * u);
  return u * cdf;
}
template <> __device__ __forceinline__ float gelu_with_grad_t<bf16>(float u, float& grad) {
  float cdf, gauss;
  normal_cdf_fast(u, cdf, gauss);
  grad = __builtin_fmaf(u * 0.39894228040143268f, gauss, cdf);
  return u * cdf;
}
template <typename T> __device__ __forceinline__ float gelu_grad_t(float u);
template <> __device__ __forceinline__ float gelu_grad_t<float>(float u) { return gelu_grad_f(u); }
template <> __device__ __forceinline__ float gelu_grad_t<bf16>(float u) {
  float cdf, gauss;
  normal_cdf_fast(u, cdf, gauss);
  return __builtin_fmaf(u * 0.39894228040143268f, gauss, cdf);
}

// ---- wave / block reductions -----------------------------------------------------------------------
// Wave reductions on the DPP lanes of the vector ALU (no LDS traffic): quad swaps, mirrors within rows of 16, then
// the last lane of a row broadcast into the next rows; lane 63 ends up with the result, which is then read out as
// a wave-uniform value.  The order of the additions is fixed.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_fetch(float v, float identity) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity),
                                                               __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_fetch<0xb1, 0xf>(v, 0.f);    // quad_perm [1,0,3,2]
  v += dpp_fetch<0x4e, 0xf>(v, 0.f);    // quad_perm [2,3,0,1]
  v += dpp_fetch<0x141, 0xf>(v, 0.f);   // row_half_mirror
  v += dpp_fetch<0x140, 0xf>(v, 0.f);   // row_mirror: every lane holds the sum of its row of 16
  v += dpp_fetch<0x142, 0xa>(v, 0.f);   // row_bcast15 into rows 1 and 3
  v += dpp_fetch<0x143, 0xc>(v, 0.f);   // row_bcast31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  const float lowest = -INFINITY;
  v = fmaxf(v, dpp_fetch<0xb1, 0xf>(v, lowest));
  v = fmaxf(v, dpp_fetch<0x4e, 0xf>(v, lowest));
  v = fmaxf(v, dpp_fetch<0x141, 0xf>(v, lowest));
  v = fmaxf(v, dpp_fetch<0x140, 0xf>(v, lowest));
  v = fmaxf(v, dpp_fetch<0x142, 0xa>(v, lowest));
  v = fmaxf(v, dpp_fetch<0x143, 0xc>(v, lowest));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

}  // namespace dipaco
