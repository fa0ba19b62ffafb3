// Measurement aid (include/dipaco_kernels.h: dipaco_k_issue_probe): register-only loops that show how matrix-core and
// vector-ALU instructions share a SIMD, and what the chip sustains of the two bf16 matrix-core shapes.  No memory traffic inside the loops; one workgroup per compute unit.
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

// What the chip sustains of the two bf16 matrix-core shapes at its power limit: a wave's 128 x 64 outputs as 4 x 2 tiles of
// v_mfma_f32_32x32x16 (SHAPE 0) or 8 x 4 tiles of v_mfma_f32_16x16x32 (SHAPE 1), 32 deep per iteration either way
// (524,288 flop per wave), operands held in registers: pseudo-random bf16 in [-2, 2) or all zero.
__device__ inline unsigned probe_hash(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
__device__ inline unsigned probe_pair(unsigned seed, bool random) {   // two bf16 in one dword
  if (!random) return 0u;
  const unsigned h = probe_hash(seed);
  auto one = [](unsigned b) { return ((b & 1u) << 15) | ((125u + ((b >> 1) % 3u)) << 7) | ((b >> 3) & 0x7fu); };
  return one(h & 0xffffu) | (one(h >> 16) << 16);
}
template <int SHAPE> __global__ void __launch_bounds__(512, 2) mfma_shape_probe_kernel(float* out, int iters, int random) {
  const unsigned tid = blockIdx.x * blockDim.x + threadIdx.x;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  float sum = 0.f;
  if (SHAPE == 0) {
    u32x4 a[2][4], b[2][2];
    for (int k = 0; k < 2; ++k) {
      for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 4; ++e) a[k][i][e] = probe_pair(tid * 977u + (k * 4 + i) * 13u + e, random);
      for (int j = 0; j < 2; ++j)
        for (int e = 0; e < 4; ++e) b[k][j][e] = probe_pair(tid * 613u + (k * 2 + j) * 29u + e + 7777u, random);
    }
    f32x16 acc[4][2];
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 2; ++j)
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[k][i]),
                                                                __builtin_bit_cast(bf16x8, b[k][j]), acc[i][j], 0, 0, 0);
      if ((it & 63) == 63)   // keep the sums finite
        for (int i = 0; i < 4; ++i)
          for (int j = 0; j < 2; ++j) { sum += acc[i][j][0]; for (int e = 0; e < 16; ++e) acc[i][j][e] *= 1e-3f; }
    }
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 2; ++j)
        for (int e = 0; e < 16; ++e) sum += acc[i][j][e];
  } else {
    u32x4 a[8], b[4];
    for (int i = 0; i < 8; ++i)
      for (int e = 0; e < 4; ++e) a[i][e] = probe_pair(tid * 977u + i * 13u + e, random);
    for (int j = 0; j < 4; ++j)
      for (int e = 0; e < 4; ++e) b[j][e] = probe_pair(tid * 613u + j * 29u + e + 7777u, random);
    f32x4 acc[8][4];
    for (int i = 0; i < 8; ++i)
      for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[j]),
                                                              acc[i][j], 0, 0, 0);
      if ((it & 63) == 63)
        for (int i = 0; i < 8; ++i)
          for (int j = 0; j < 4; ++j) { sum += acc[i][j][0]; for (int e = 0; e < 4; ++e) acc[i][j][e] *= 1e-3f; }
    }
    for (int i = 0; i < 8; ++i)
      for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 4; ++e) sum += acc[i][j][e];
  }
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

}  // namespace

dipaco_status launch_issue_probe(int mode, int waves_per_simd, int iters, float* out, hipStream_t s) {
  const int threads = 256 * waves_per_simd, blocks = ISSUE_PROBE_BLOCKS;
  if (mode >= 5) {   // matrix-core shapes at two waves per SIMD: 5 / 6 = 32x32x16 on zeros / random, 7 / 8 = 16x16x32
    if (mode < 7) mfma_shape_probe_kernel<0><<<blocks, 512, 0, s>>>(out, iters, mode == 6);
    else mfma_shape_probe_kernel<1><<<blocks, 512, 0, s>>>(out, iters, mode == 8);
    DIPACO_LAUNCH_CHECK();
    return DIPACO_OK;
  }
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
