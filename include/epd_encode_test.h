/*
 * epd_encode_test.h  --  measurement and test hooks of the encode-stage library.
 *
 * Not needed to serve: single kernels in isolation (parity tests hold them
 * against the CPU oracle step by step), per-kernel-family timing (the
 * benchmark's roofline figures) and a read-back of the residual stream.  Same
 * conventions as epd_encode.h.  These calls may allocate and synchronise.
 */
#ifndef EPD_ENCODE_TEST_H
#define EPD_ENCODE_TEST_H

#include "epd_encode.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Copy the residual stream (float32 [rows, D], the encoder state after the
 * last layer of the last micro-batch of the previous call) to host memory.
 * Synchronises the device.  rows * D * 4 must be <= dst_bytes. */
epd_status epd_debug_read_stream(epd_ctx* ctx, void* dst /*host*/, int64_t rows, int64_t dst_bytes);

/* Time the dominant kernel family in isolation: runs `iters` launches of the
 * bf16 MFMA GEMM  C[M,N] = A[M,K] * W[N,K]^T  (+ bias) on dev buffers the
 * caller provides, bracketed by HIP events on `hip_stream`; returns the mean
 * milliseconds per launch in *ms_per_launch.  A [M,K] bf16, W [N,K] bf16,
 * bias [N] fp32 (may be null), C [M,N] bf16.  M % 256 == 0, N % 128 == 0,
 * K % 128 == 0. */
epd_status epd_op_gemm_bf16(const void* A, const void* W, const float* bias, void* C, int32_t M,
                            int32_t N, int32_t K, int32_t iters, float* ms_per_launch,
                            void* hip_stream);

/* One launch of the bf16 MFMA GEMM in a chosen form, for tests that hold the forms against each
 * other: epi 0 bias, 1 bias + GELU(erf), 2 bias + GELU(tanh) -> C [M,N] bf16; epi 3 -> R [M,N]
 * fp32 += A W^T + bias (C unused).  form 0 = what the library would pick, 1 = 256x128 tile,
 * 2 = 128x128 tile, 3 = 128x128 tile with the loads four slabs ahead (K % 256 == 0), 6 = 256x256 tile with the plain loop, 7 = pipelined loop, 8 = pipelined loop with both operand slabs
 * loaded straight into LDS, 9 = persistent kernel (not epi 3), 10 = persistent kernel of the residual product (epi 3 only),
 * 11 = 64x64 tiles with both operand slabs in an LDS ring (what the library picks for launches of a slice or two).
 * 12 = the persistent residual product on 256x192 tiles (epi 3 only, N % 192 == 0: what the library picks for a
 * width like 1152, which is six such tile columns and four and a half 256-wide ones).
 * M >= 1 (any), N % 128 == 0 (N % 256 == 0 for forms 6 to 10), K % 128 == 0; bias [N] fp32.
 * A [M,K], C [M,N] and R [M,N] hold exactly M rows; no row past M is written.  (The kernels read whole
 * 256-row tiles; for a ragged M, and for R, the call runs on padded copies it allocates, and synchronises.) */
epd_status epd_op_gemm_bf16_form(const void* A, const void* W, const float* bias, void* C, float* R,
                                 int32_t M, int32_t N, int32_t K, int32_t epi, int32_t form,
                                 void* hip_stream);

/* The pre-norms of a layer have no kernel of their own in bf16 mode: the residual epilogue that updates a row
 * x also stores bf16(x) and the row's statistics, and the product that follows the norm runs on bf16(x) against
 * weights that carry the norm's gain, applying mean and 1 / sqrt(variance + eps) in its epilogue.  Statistics of
 * a row: one pair (mean, sum of squared deviations from that mean) per group of 128 columns, stats
 * [rows][ceil(dim / 128)][2] fp32.
 * epd_op_row_stats: xb [rows, dim] bf16 = x [rows, dim] fp32 and the pairs of every row (dim % 4 == 0).
 * epd_op_gemm_residual_stats: R [M,N] fp32 += A [M,K] W [N,K]^T + bias as epd_op_gemm_bf16_form's epi 3 (forms
 *   0, 1, 2, 3, 6, 7, 8), and xb [M,N] = bf16 of the updated R with its pairs in stats [M][N / 128][2];
 *   M % 256 == 0 here, and R must hold 256 floats behind its last row.
 * epd_op_norm_gemm_bf16: C [M,N] bf16 = act(norm(x) W^T + bias) the folded way: x [M,D] fp32, gamma / beta [D]
 *   fp32 (beta null: RMSNorm), W [N,D] bf16, bias [N] fp32; epi 0 none, 1 GELU(erf), 2 GELU(tanh); form as
 *   epd_op_gemm_bf16_form; M % 256 == 0, N % 128 == 0, D % 128 == 0.  Allocates and synchronises. */
epd_status epd_op_row_stats(const float* x, int64_t rows, int32_t dim, void* xb, float* stats, void* hip_stream);
epd_status epd_op_gemm_residual_stats(const void* A, const void* W, const float* bias, float* R, void* xb, float* stats,
                                      int32_t M, int32_t N, int32_t K, int32_t form, void* hip_stream);
epd_status epd_op_norm_gemm_bf16(const float* x, const float* gamma, const float* beta, const void* W, const float* bias,
                                 void* C, int32_t M, int32_t N, int32_t D, float eps, int32_t epi, int32_t form,
                                 void* hip_stream);

/* Tile-local non-causal attention on packed slices, bf16:  for every slice t
 * and head h, O = softmax(Q K^T / sqrt(hd)) V over the slice's own n_tokens
 * keys.  The kernel takes the logits in the log2 domain straight from the product: the caller's q must
 * carry the factor log2(e) / sqrt(hd) (the library folds it into the q projection), i.e. the weight of
 * key j for query i is 2^(q_i . k_j) / sum_j' 2^(q_i . k_j').  q, k dev bf16 [T * n_tokens, H * hd_pad]
 * with row stride ld_qk elements; vt dev bf16 [T, H, hd_pad, n_tokens] (values transposed); o dev
 * bf16 [T * n_tokens, H * hd_pad].  hd_pad in {64, 72, 96, 128}, n_tokens % 64 == 0.
 * Only the first n_keys (1 .. n_tokens) rows of a slice are tokens:
 * the others are left out of every softmax as keys, and their rows of o hold unused values. */
epd_status epd_op_attention_bf16(const void* q, const void* k, const void* vt, void* o,
                                 int32_t n_slices, int32_t n_tokens, int32_t n_keys, int32_t heads,
                                 int32_t hd_pad, int32_t ld_qk, void* hip_stream);

/* The same attention with its output leaving as MXFP8 (the out-projection's operand under epd_model_desc::mx_fp8),
 * converted from the kernel's fp32 accumulators: codes dev uint8 [T * n_tokens, H * hd_pad], scales dev uint32
 * [H * hd_pad / 128, T * n_tokens] (layout of epd_op_mx_rows).  hd_pad % 32 == 0, H * hd_pad % 128 == 0. */
epd_status epd_op_attention_mx(const void* q, const void* k, const void* vt, void* codes, void* scales, int32_t n_slices,
                               int32_t n_tokens, int32_t n_keys, int32_t heads, int32_t hd_pad, int32_t ld_qk, void* hip_stream);

/* Check of the MFMA operand / result lane layout the kernels assume:
 * D[32,32] (fp32, row-major) = A[32,16] * B[16,32] (bf16, row-major), one
 * v_mfma_f32_32x32x16_bf16.  All pointers dev. */
epd_status epd_op_mfma_probe(const void* A, const void* B, float* D, void* hip_stream);

/* MXFP8 operands (epd_model_desc::mx_fp8): element format OCP FP8 E4M3, one power-of-two scale byte
 * (value 2^(byte - 127)) per block of 32 consecutive elements of the contraction dimension (OCP Microscaling
 * Formats specification v1.0).  Device layout: codes [rows, K] bytes; scales uint32 [K / 128, rows], word (s, r)
 * = the scale bytes of blocks 4 s .. 4 s + 3 of row r, block 4 s + b in byte b.
 * epd_op_mx_rows: conversion of `rows` rows of `dim` elements (dim % 128 == 0; fp32, or bf16 if in_bf16), after
 *   a LayerNorm (kind 0, gamma / beta [dim] fp32), an RMSNorm (kind 1, gamma) or as they are (kind 2).
 * epd_op_mx_gemm: out = (A W^T) * cscale[n] + bias[n] on such operands (A [M, K], W [N, K]; M % 256 == 0,
 *   N % 256 == 0, K % 128 == 0; cscale may be null); epi 0 -> C bf16 [M, N]; epi 5 -> C bf16 transposed per
 *   slice and head, [M / n_tok, heads, hd_pad, n_tok] with N = heads * hd_pad; epi 1 / 2 -> GELU (erf / tanh form),
 *   then converted: codes Cq [M, N], scales SC [N / 128, M]; epi 3 -> R fp32 [M, N] += out.
 * epd_op_mx_mfma_probe: one v_mfma_scale_f32_32x32x64_f8f6f4 on caller-supplied registers (a, b: int32 [64][8],
 *   sa, sb: int32 [64], scale byte 0 used; d: fp32 [64][16]), for the operand-layout test.  All pointers dev. */
epd_status epd_op_mx_rows(const void* in, int32_t in_bf16, int64_t rows, int32_t dim, int32_t kind, const float* gamma,
                          const float* beta, float eps, void* codes, void* scales, void* hip_stream);
epd_status epd_op_mx_gemm(int32_t epi, const void* A, const void* SA, const void* W, const void* SW, const float* bias,
                          const float* cscale, int32_t M, int32_t N, int32_t K, void* C, float* R, void* Cq, void* SC,
                          int32_t n_tok, int32_t heads, int32_t hd_pad, void* hip_stream);
epd_status epd_op_mx_mfma_probe(const void* a, const void* b, const void* sa, const void* sb, float* d, void* hip_stream);

/* Per-kernel-family timing of the previous epd_encode / epd_encode_range
 * call on this context, measured with HIP events on the call's stream.
 * epd_profile_enable(ctx, 1) makes subsequent calls bracket every launch
 * with two event records; epd_profile_read synchronises the device and fills
 * ms[family] (summed) and launches[family] (kernels launched: a product that
 * the library cuts into two launches counts twice).  Families: 0 im2col + patch-embed
 * GEMM, 1 pre-norms, 2 QKV GEMM, 3 attention, 4 q/k norm, 5 projector input
 * (shuffle / norm / convert), 6 out-proj GEMM, 7 FC1 GEMM, 8 FC2 GEMM,
 * 9 projector GEMMs. */
enum { EPD_PROF_FAMILIES = 10 };
epd_status epd_profile_enable(epd_ctx* ctx, int32_t on);
epd_status epd_profile_read(epd_ctx* ctx, float* ms /*host [10]*/, int32_t* launches /*host [10]*/);

/* Measured ceilings next to the nominal ones (the roofline figures of the benchmark).
 * epd_op_mfma_peak: a register-resident loop of v_mfma_f32_32x32x16_bf16 on every CU (two waves per SIMD,
 * eight independent accumulators, eight rotating operand fragment pairs, no LDS or memory traffic inside
 * the loop); *tflops = dense bf16 rate over `reps` launches of `iters` loop trips.  operands: dev, 16 KiB of
 * bf16 the fragments are loaded from (random values: the operand buses toggle as in a real product), or
 * null for constant ones (the chip clocks higher on those).  sink: dev, 4 bytes per launched thread
 * (2 * CUs * 256 floats), keeps the loop alive.
 * epd_op_copy_peak: dst = src, `bytes` (multiple of 16) in 16-byte pieces; *gbps = read + write rate.
 * epd_op_coissue: how matrix and vector instructions of two waves of one SIMD share its issue port (what bounds the
 * attention kernel, whose step is a matrix product, exponentials, a matrix product).  One workgroup of eight waves
 * per CU: four waves (one per SIMD) issue iters_mfma x 16 v_mfma_f32_32x32x16_bf16 on independent accumulators, the
 * other four iters_valu x 32 pairs of v_exp_f32 + fma; which = 1 the matrix waves alone, 2 the vector waves alone,
 * 3 both together.  *ms_per_launch over `reps` launches.  operands: dev, 8 KiB of bf16; sink: dev, 4 bytes per
 * launched thread (CUs * 512 floats). */
epd_status epd_op_mfma_peak(const void* operands, int32_t iters, int32_t reps, float* sink, float* tflops,
                            void* hip_stream);
epd_status epd_op_copy_peak(const void* src, void* dst, int64_t bytes, int32_t reps, float* gbps, void* hip_stream);
epd_status epd_op_coissue(const void* operands, int32_t iters_mfma, int32_t iters_valu, int32_t which, int32_t reps,
                          float* sink, float* ms_per_launch, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EPD_ENCODE_TEST_H */
