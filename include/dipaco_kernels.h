/*
 * dipaco_kernels.h - kernel-level entry points of libdipaco.so.
 *
 * These expose single kernels of the path step (Algorithm 1 inner loop of arXiv 2403.10616: the pieces of
 * f(x, theta_i) and its gradient) so that each can be checked against its plain definition and timed against
 * its own roofline.  They follow the conventions of dipaco.h: caller-owned device pointers, 16-byte aligned,
 * work enqueued on `stream`, non-zero status = nothing enqueued.  dtype is a dipaco_dtype: the element type of
 * every `void*` operand (fp32 or bf16); accumulation is always fp32.
 */
#ifndef DIPACO_KERNELS_H
#define DIPACO_KERNELS_H

#include "dipaco.h"

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] = opA(A) . opB(B) on the matrix cores.
 *   trans_a = 0: A is [M,K] row-major; 1: A is [K,M] row-major.   trans_b = 0: B is [K,N]; 1: B is [N,K].
 *   Supported: (0,0) forward, (0,1) input gradient, (1,0) with out_f32 = 1 weight gradient.
 * Epilogue in this order, each optional: + bias[N];  act = 1: aux_out[M,N] = value, value = GELU(value);
 * act = 2: value *= GELU'(aux_in[M,N]);  act = 3: aux_out[M,N] = GELU'(value), value = GELU(value);
 * act = 4: value *= aux_in[M,N];  + resid[M,N].  out_f32 = 1: C is fp32, else dtype.
 * splits > 1 (needs out_f32, no epilogue): K is cut into ranges whose partial products are written to
 * partial ([splits, M, N] fp32) and summed in index order.  The contiguous extent of each operand must be a
 * multiple of 16 bytes and N a multiple of 8. */
dipaco_status dipaco_k_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t out_f32, int32_t M, int32_t N,
                            int32_t K, const void* A, const void* B, void* C, const void* bias, const void* resid,
                            void* aux_out, const void* aux_in, int32_t act, int32_t splits, float* partial,
                            void* stream);

/* dipaco_k_gemm without split-K that also returns colsum_out[n] (device fp32 [N]) = sum over m of the values written
 * to C[m, n] (after the epilogue, before rounding to C's type), added in a fixed order: the bias gradient of a linear
 * layer when C is its output gradient.  colsum_scratch: device fp32, at least ceil(M / 32) * N elements. */
dipaco_status dipaco_k_gemm_colsum(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                                   const void* A, const void* B, void* C, const void* bias, const void* resid,
                                   void* aux_out, const void* aux_in, int32_t act, float* colsum_out,
                                   float* colsum_scratch, void* stream);

/* Force the GEMM workgroup tile for every later call in this process: 0 = automatic (default), 1 = 128x128,
 * 2 = 256x128, 3 = 256x256 with four waves, 4 = 256x256 with eight waves, 5 = the bf16 kernel that loads its
 * 256x256 tiles from global memory straight into LDS, for every shape it takes (K a multiple of 32, 16-byte rows;
 * other shapes and fp32 keep the automatic choice), 6 / 7 = the same kernel with its 256x256 / 256x128 tile forced,
 * 8 / 9 = the same with 128x512 / 512x128 tiles for weight gradients (fp32 output) and 256x256 for the rest,
 * 10 = the same with tile columns every 224 wherever N is a multiple of 224 (bf16 output), 11 = its eight-wave 256x256
 * tile with K tiles of 64 in a ring of two (K a multiple of 64, no split-K), 12 / 13 = the 256x256 tile computed with
 * 16x16x32 matrix-core instructions, K tiles of 32 in a ring of four / of 64 in a ring of two.
 * For tests (every tile shape must give the same parity) and tuning: a process-wide switch, not a per-call setting. */
dipaco_status dipaco_k_set_gemm_tile(int32_t tile);

/* Host-only (no GPU needed): the uneven split-K plan that the weight gradient C[M, N] = X^T dY with K = tokens is
 * launched with when at most max_slices K slices are allowed (dipaco_k_gemm with trans_a = 1, out_f32 = 1, bf16).
 * out (host int32 [12]): tile height and width of the shape taken (0, 0 when there is no such plan and the launch
 * cuts K into equal slices); tile rows / columns of the class of tiles inside C; tiles per class; K slices per class.
 * Classes: inside C, over its last rows, over its last columns, over both.  One workgroup per (tile, slice): their
 * total never exceeds the 256 compute units. */
dipaco_status dipaco_k_gemm_split_plan(int32_t M, int32_t N, int32_t K, int32_t max_slices, int32_t* out);

/* How the bf16 attention kernels deal the blocks of the causal triangle to workgroups, for every later call in this
 * process (tuning and tests): 0 = a long and a short block per workgroup, 1 = one block per workgroup, launched
 * longest first.  Results are identical. */
dipaco_status dipaco_k_set_attention_blocks(int32_t single_block);

/* Causal softmax attention.  qkv: [B*S, 3*H*dh], row = q | k | v, head h at columns h*dh of each third;
 * o: [B*S, H*dh];  lse: fp32 [B, H, S] = log sum_j exp(q_i.k_j / sqrt(dh)), j <= i.  dh in {32, 64, 128}. */
dipaco_status dipaco_k_attention_fwd(int32_t dtype, const void* qkv, void* o, float* lse, int32_t B, int32_t S,
                                     int32_t H, int32_t dh, void* stream);

/* Gradient of the above: d_o [B*S, H*dh] -> dqkv [B*S, 3*H*dh].  dsum: fp32 scratch of 2 * B * H * S128 floats,
 * S128 = S rounded up to a multiple of 128 (per-query statistics passed between the two backward kernels).
 * colsum_out: NULL, or fp32 [3*H*dh] = the column sums of dqkv (the bias gradient of the QKV projection), added in a
 * fixed order; then colsum_scratch: fp32, at least max(ceil(B*S / 256), B * ceil(S / 128)) * 3*H*dh elements. */
dipaco_status dipaco_k_attention_bwd(int32_t dtype, const void* qkv, const void* o, const void* d_o, const float* lse,
                                     void* dqkv, float* dsum, float* colsum_out, float* colsum_scratch, int32_t B,
                                     int32_t S, int32_t H, int32_t dh, void* stream);

/* Measurement aid, no part of the method: register-only loops that show how the matrix cores and the vector ALU of a
 * SIMD share instruction issue (the inner loops of the attention kernels are priced with it).  One workgroup of
 * 256 * waves_per_simd threads per compute unit (256 workgroups) runs `iters` iterations of
 *   mode 0: 16 v_mfma_f32_32x32x16_bf16 on four independent accumulators;   mode 1: 256 independent v_fma_f32;
 *   mode 2: the 16 MFMA, then the 256 FMA;   mode 3: sixteen times (1 MFMA, 16 FMA) in program order;
 *   mode 4: 256 times (v_exp_f32, multiply, add);
 *   modes 5..8 (always 512 threads per workgroup, two waves per SIMD; waves_per_simd is ignored): what the chip sustains
 *   of the two bf16 matrix-core shapes, a wave's 128 x 64 outputs computed 32 deep per iteration (524,288 flop per wave
 *   and iteration) from operands held in registers: 5 / 6 = v_mfma_f32_32x32x16_bf16 on all-zero / pseudo-random
 *   operands, 7 / 8 = v_mfma_f32_16x16x32_bf16 likewise (the GEMM kernel's choice of shape rests on 6 against 8).
 * The caller times the launch.  out: device fp32, 256 * 256 * waves_per_simd elements (at least 256 * 512 for modes
 * 5..8), overwritten (keeps the loops alive).  mode in 0..8, waves_per_simd in 1..4, iters >= 1, else DIPACO_EINVAL. */
dipaco_status dipaco_k_issue_probe(int32_t mode, int32_t waves_per_simd, int32_t iters, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DIPACO_KERNELS_H */
