// Measurement aid (include/dipaco_kernels.h: dipaco_k_issue_probe): register-only loops that show how matrix-core and
// vector-ALU instructions share a SIMD.  No memory traffic inside the loops; one workgroup per compute unit.
#include "kernels.h"

namespace dipaco {

namespace {

// MODE 0: 16 MFMA (four independent accumulators) per iteration;  1: 256 independent FMA;  2: the 16 MFMA, then the
// 256 FMA;  3: sixteen times (1 MFMA, 16 FMA) in program order;  4: 256 times (exp2, multiply, add).
template <int MODE> __global__ void __launch_bounds__(1024) issue_probe_kernel(float* out, int iters) {
  f32x16 acc[4];
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (bf16)(1.0f + threadIdx.x * 0.001f); b[e] = (bf16)0.5f; }
  float v[16];
  for (int e = 0; e < 16; ++e) v[e] = threadIdx.x * 0.01f + e;
  const float c1 = 1.0001f, c2 = 0.0001f;
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0 || MODE == 2) {
#pragma unroll
      for (int m = 0; m < 16; ++m) acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m & 3], 0, 0, 0);
    }
    if (MODE == 1 || MODE == 2) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = __builtin_fmaf(v[e], c1, c2);
    }
    if (MODE == 3) {
#pragma unroll
      for (int m = 0; m < 16; ++m) {
        acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m & 3], 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = __builtin_fmaf(v[e], c1, c2);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (MODE == 4) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = __builtin_amdgcn_exp2f(v[e]) * 0.0f + v[e];
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  float s = 0.f;
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  for (int e = 0; e < 16; ++e) s += v[e];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace

dipaco_status launch_issue_probe(int mode, int waves_per_simd, int iters, float* out, hipStream_t s) {
  const int threads = 256 * waves_per_simd, blocks = ISSUE_PROBE_BLOCKS;
  switch (mode) {
    case 0: issue_probe_kernel<0><<<blocks, threads, 0, s>>>(out, iters); break;
    case 1: issue_probe_kernel<1><<<blocks, threads, 0, s>>>(out, iters); break;
    case 2: issue_probe_kernel<2><<<blocks, threads, 0, s>>>(out, iters); break;
    case 3: issue_probe_kernel<3><<<blocks, threads, 0, s>>>(out, iters); break;
    default: issue_probe_kernel<4><<<blocks, threads, 0, s>>>(out, iters); break;
  }
  DIPACO_LAUNCH_CHECK();
  return DIPACO_OK;
}

}  // namespace dipaco
