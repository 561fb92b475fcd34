// Internal launcher interface between the C boundary (epd_api.hip) and the
// gfx950 kernels.  Not part of the public boundary.
#pragma once
#include "common.h"

namespace epd {

// Where the patch tokens of a slice sit in the residual stream: slice t owns `stride` rows and its
// patch token i is row t * stride + off + i (off = 1 behind a class token; stride > off + n when a
// slice's rows are padded to a multiple of 8).  n == 0: the rows are contiguous.
struct SliceRows {
  int n, stride, off;
  __host__ __device__ long row(long r) const { return n ? (r / n) * stride + off + r % n : r; }
};

// ---- fp32 mode (simple_f32.hip) -------------------------------------------
void f32_im2col(const float* tiles, float* A, int T, int S, int p, hipStream_t st);
void f32_gemm(int epi, const float* A, int lda, const float* W, const float* bias, float* C, int ldc,
              const float* pos, int n_pos, int M, int N, int K, hipStream_t st,
              const int* row_map = nullptr, int block_tokens = 1, SliceRows xrows = SliceRows{0, 0, 0});
void f32_norm(int kind, const float* in, long ld_in, float* out, long ld_out, const float* gamma,
              const float* beta, long rows, int dim, int groups, float eps, hipStream_t st);
// Slice t: keys / values rows t*N .. t*N+N-1 (row stride ld).  Encoder layers: n_q = N queries from the
// slice's own rows.  q_shared: the n_q query rows (stride ld_q) are the same for every slice (resampler).
// Output row t*n_q + i.
void f32_attention(const float* q, long ld_q, int n_q, int q_shared, const float* k, const float* v, long ld,
                   float* o, long ldo, int T, int N, int H, int hd, float scale, hipStream_t st);
// out[r][c] = in[r][c] + add[r % add_rows][c], rows of dim floats
void f32_add_rows(const float* in, const float* add, int add_rows, float* out, long rows, int dim, hipStream_t st);
void f32_shuffle(const float* in, SliceRows src, float* out, int T, int g, int D, hipStream_t st);
// out[r] = in[src.row(r)], rows of D floats
void f32_take_rows(const float* in, SliceRows src, float* out, long rows, int D, hipStream_t st);

// ---- bf16 mode -------------------------------------------------------------
// GEMM  C[M,N] = A[M,K] * W[N,K]^T with fused epilogue (gemm_bf16.hip).
// A must be readable for round_up(M,256) rows, W for Npad rows (zero rows
// beyond N); K % 128 == 0; N % 4 == 0 (N % 8 == 0 for bf16 outputs); Npad % 128 == 0.
struct GemmParams {
  int epi;
  int cfg;                    // 0: chosen by shape and epilogue; tests / timing: 1 = 256x128 tile, 2 / 3 = 128x128 tile (loads two / four slabs ahead), 6 = 256x256 plain loop,
                              // 7 = 256x256 pipelined loop, 8 = the same with both operands straight into LDS,
                              // 9 = 256x256 persistent (bf16-output epilogues), 10 = persistent residual product, 11 = 64x64 tiles (small launches),
                              // 12 = persistent residual product on 256x192 tiles (N % 192 == 0)
  int band;                   // 0: automatic; else tile columns per L2 band (must divide Npad / BN)
  const bf16_t* A; long lda;
  const bf16_t* W;            // packed [Npad, K]
  const float* bias;          // [Npad]
  int M, N, K, Npad;
  bf16_t* C; long ldc;        // bf16 output (BIAS, GELU_*)
  const int* row_map;         // optional paged output: row r -> row_map[r / block_tokens] * block_tokens + r % block_tokens
  int block_tokens;
  float* R; long ldr;         // fp32 residual stream (RESIDUAL, POS); RESIDUAL reads whole tiles: R must hold
                              // round_up(M, 256) rows plus (Npad - N) floats behind the last one
  const float* pos; int n_pos;   // POS: product row r gets pos[r % n_pos] and lands in row xrows.row(r) of R
  SliceRows xrows;
  bf16_t* VT;                 // EPI_VT: values, transposed per (slice, head): [T, H, hd_pad, n_tok]
  int hd_pad, heads, n_tok;   // EPI_VT: column c = h * hd_pad + d, row r = t * n_tok + n
  // Pre-norm folded into the product (bf16-output epilogues; null `stats`: off).  A holds bf16(x) of the
  // residual stream, W the weights times the norm gain, bias the bias plus W beta, and
  //   out[r][n] = rstd_r * (acc[r][n] - mean_r * colsum[n]) + bias[n]
  // with mean_r / rstd_r from the row's statistics pairs (common.h: one pair per 128 columns of x).
  const float* stats;         // [M][n_part][2], n_part <= STAT_REGS
  const float* colsum;        // [Npad]: sum over k of the packed (gain-scaled, rounded) weights
  int n_part, stat_group;     // pairs per row and the columns a pair covers (128 as emitted; the whole row once combined)
  int norm_dim, norm_rms;     // columns of x; 1: RMSNorm (no mean)
  float norm_eps;
  // Residual epilogue (RESIDUAL; null `xb`: off): also stores bf16 of the updated rows to xb [M, ldxb] and
  // their statistics pairs to stats_out [M][n_part_out][2] (pair index = column / 128).
  bf16_t* xb; long ldxb;
  float* stats_out; int n_part_out;
  // A second product over the same A in the same launch (epi EPI_BIAS, small launches only: bf16_gemm_pair_fits):
  // the value projection next to the q/k projection.  Its packed weights and bias follow the first product's
  // directly (rows Npad .. Npad + n2_pad of W, entries Npad .. of bias); its n2 columns leave through the
  // EPI_VT store (VT, hd_pad, heads, n_tok).  n2_pad == 0: off.
  int n2, n2_pad;
};
hipError_t bf16_gemm(const GemmParams& p, hipStream_t st);
// true: bf16_gemm runs p with its second product (n2_pad > 0) as one launch; false: the caller issues two products
bool bf16_gemm_pair_fits(const GemmParams& p);
long bf16_gemm_kernel_launches();   // kernels launched by bf16_gemm on the calling host thread so far (a figure for the profiling hooks)
hipError_t bf16_gemm_init();  // raises the dynamic-LDS limit of the kernels (idempotent: safe from any thread, any number of times)

// A_pe[row][e] = bf16(pixel) for e < 3*p*p, 0 for the K padding up to lda.
void bf16_im2col(const float* tiles, bf16_t* A, int lda, int T, int S, int p, hipStream_t st);

// LayerNorm (kind 0) / RMSNorm (1) of bf16 rows in place: x [rows, dim] bf16 (row stride ld, dim % 8 == 0, rows
// 16-byte aligned), statistics in fp32.  The rows are bf16 copies of the residual stream left by the residual epilogues.
void bf16_norm_rows(bf16_t* x, long ld, const float* gamma, const float* beta, long rows, int dim, int kind, float eps,
                    hipStream_t st);

// bf16(x) and the statistics pairs of every row of the residual stream x [rows, dim] (dim % 4 == 0): what the
// residual epilogue emits for the rows it updates, for rows that come from elsewhere (embedding, class token).
void bf16_row_stats(const float* x, long ldx, long rows, int dim, bf16_t* xb, long ldxb, float* stats, int n_part,
                    hipStream_t st);

// Rows of more than STAT_REGS pairs: one pair (mean, squared deviations) over the whole row from the n_part pairs
// over 128 columns each.  out [rows][2].
void bf16_combine_stats(const float* stats, long rows, int n_part, int dim, float* out, hipStream_t st);

// Fold a pre-norm into a packed Linear in place: bias[n] += sum_k W[n][k] beta[k] (beta null: RMSNorm),
// W[n][k] = bf16(W[n][k] gamma[k]), colsum[n] = sum_k W[n][k] over the rounded products.  rows x cols of the
// packed matrix (row stride ld); gamma / beta hold `dim` <= cols values, columns past dim are left alone.
void fold_norm_into_linear(bf16_t* W, int rows, int cols, long ld, const float* gamma, const float* beta, int dim,
                           float* bias, float* colsum, hipStream_t st);

// Row operation fp32 -> bf16 (rowop_bf16.hip): optional pixel-shuffle gather
// of the source rows, then LayerNorm (kind 0), RMSNorm (1) or plain convert (2).
struct RowOpParams {
  int kind;
  const float* in; long ld_in;   // residual stream [.., D]
  bf16_t* out; long ld_out;
  const float* gamma; const float* beta;
  long rows;                      // output rows
  int dim;                        // output row length (D, or 4D with shuffle)
  int shuffle;                    // 1: gather 2x2 grid neighbours, dim == 4*D
  int g, D;                       // grid side and source row length (shuffle only)
  float eps;
  SliceRows src;                  // source row of patch token r (shuffle: of grid cell r) = src.row(r)
};
void bf16_rowop(const RowOpParams& p, hipStream_t st);

// In-place RMSNorm of the q rows and the k rows of the QK buffer in one launch (k = q + k_off elements,
// its own gain).  Logical row R of `dim` (padded) elements at buf + (R / groups) * ld + (R % groups) * dim;
// `count` = number of real elements the mean runs over.
void bf16_qknorm(bf16_t* buf, long ld, long k_off, const float* gamma_q, const float* gamma_k, long rows, int dim,
                 int groups, int count, float eps, hipStream_t st);

// Slice t owns rows t * n_tok .. of q, k, o and columns 0 .. n_tok of its V^T rows (n_tok % 8 == 0);
// only its first n_keys rows are real tokens: later keys are masked out, later queries give unused rows.
// Keys are read in blocks of 64: when n_tok % 64 != 0 the last block reaches up to 63 rows of q / k and
// 63 elements of v^T past the slice (the next slice's, or slack the caller keeps behind the buffers).
// n_q queries per slice (n_tok unless q_shared); q_shared: the query rows are rows 0 .. n_q-1 of q
// for every slice (learned queries of the resampler; q must be readable for round_up(n_q, 32) rows) instead
// of the slice's own rows.  Row t * n_q + i of o is query i of slice t.
// The queries carry the logit scale: weight of key j for query i = 2^(q_i . k_j) / sum_j' 2^(q_i . k_j').
// oq != null (hd_pad % 32 == 0 only): the output leaves as MXFP8 instead of bf16, converted from the fp32
// accumulators: codes oq [rows][ld_o bytes] (column h * hd_pad + d), scale words so [column / 128][ld_so]
// (ld_so >= rows; layout of gemm_mxfp8.hip); o is not written then.
hipError_t bf16_attention(const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* o, int n_slices,
                          int n_tok, int n_keys, int n_q, int q_shared, int heads, int hd_pad, long ld_qk,
                          long ld_o, hipStream_t st, unsigned char* oq = nullptr, unsigned* so = nullptr, long ld_so = 0);

// W[r][0..cols) *= c (rounded to bf16 again) and b[r] *= c for r < rows: a constant factor of a product's
// output folded into the rows of its packed weights
void scale_rows_by(bf16_t* W, int rows, int cols, long ld, float* b, float c, hipStream_t st);
// v[i] *= c for i < n (fp32)
void scale_vector(float* v, int n, float c, hipStream_t st);

// LayerNorm of bf16 rows (statistics in fp32 over `dim` elements, dim % 4 == 0): out = LN(in) and, when
// out_plus is set, out_plus = LN(in) + add[row % add_rows] (fp32 table [add_rows, dim]).
void bf16_ln_rows(const bf16_t* in, long ld_in, const float* gamma, const float* beta, float eps, bf16_t* out,
                  long ld_out, bf16_t* out_plus, const float* add, int add_rows, long rows, int dim, hipStream_t st);

// Rows of the residual stream no product writes: the class token's row of every slice
// (cls + pos[0]; cls null = no class token) and the padding rows n_real .. stride - 1 (zeros).
void fill_slice_rows(float* X, int D, int T, int stride, int n_real, const float* cls, const float* pos0,
                     hipStream_t st);

// Weight packing (pack.hip): dst[r][c] for r < rows_pad, c < cols_pad, zero
// outside the source.  row_hd/col_hd > 0: the packed index runs over heads
// padded from hd to hd_pad (index = blk*H*hd_pad + h*hd_pad + d -> blk*H*hd + h*hd + d).
struct PackMap { int hd, hd_pad, heads; };  // hd == 0: identity
void pack_matrix_bf16(const bf16_t* src, int rows, int cols, bf16_t* dst, int rows_pad, int cols_pad,
                      PackMap rmap, PackMap cmap, hipStream_t st);
void pack_vector_f32(const void* src, int src_is_bf16, int n, float* dst, int n_pad, PackMap map,
                     hipStream_t st);

// Layer scale folded into a packed Linear: W[r][0..cols) *= s[r] for r < rows (row stride ld), and
// b[r] *= s[r].  W is bf16 or fp32, s and b fp32.
void scale_rows(void* W, int w_is_bf16, int rows, int cols, long ld, float* b, const float* s, hipStream_t st);

// Paged multimodal-token cache: copy `n_blocks` blocks of `block_bytes` (multiple of 16) from
// src_pool[src_ids[i]] to dst_pool[dst_ids[i]]; a null id array means block i (contiguous side).
void mm_copy_blocks(const void* src_pool, const int* src_ids, void* dst_pool, const int* dst_ids,
                    int n_blocks, long block_bytes, hipStream_t st);

// fp32 residual-stream rows <-> rows of a paged cache of fp32 or bf16 tokens of the same width.
// Patch token r (stream row xr.row(r)) is token r % block_tokens of block row_map[r / block_tokens].
void stream_to_blocks(const float* X, long ldx, SliceRows xr, void* pool, int pool_is_bf16, int dim, const int* row_map,
                      int block_tokens, long rows, hipStream_t st);
void blocks_to_stream(const void* pool, int pool_is_bf16, int dim, const int* row_map, int block_tokens,
                      float* X, long ldx, SliceRows xr, long rows, hipStream_t st);

// ---- MXFP8 operands (gemm_mxfp8.hip) -----------------------------------------------------------------------
// codes [rows][K] bytes (E4M3), K contiguous; scales [K / 128][ld] 32-bit words: word (s, r) = the scale bytes
// of row r's four 32-element blocks of K slab s (byte b = block 4 s + b, value 2^(byte - 127)).
//
// Rows -> MXFP8, optionally behind a norm: kind 0 LayerNorm, 1 RMSNorm, 2 plain conversion; input fp32 or
// bf16 rows of `dim` elements (dim % 128 == 0), statistics and normalised values in fp32, converted from fp32.
struct MxRowParams {
  int kind;
  const void* in; long ld_in; int in_bf16;
  const float* gamma; const float* beta; float eps;
  long rows; int dim;
  unsigned char* codes; long ld_codes;     // bytes per row, >= dim, % 4 == 0
  unsigned* scales; long ld_scales;        // words per K slab, >= rows
};
hipError_t mx_rows(const MxRowParams& p, hipStream_t st);

// C[M,N] = A[M,K] W[N,K]^T on MXFP8 operands, fp32 accumulation, out = acc * cscale[n] + bias[n], then:
//   EPI_BIAS            bf16 C [M, ldc];
//   EPI_VT              bf16, transposed per (slice, head) as in GemmParams;
//   EPI_BIAS_GELU_*     activation, then MXFP8 along the output features: codes Cq [M, ldcq] (the first ncq
//                       columns are written, ncq % 128 == 0, zeros past N) and scale words SC [ncq / 128][sc_ld]
//                       (the operand of the next product);
//   EPI_BIAS_RESIDUAL   R[M, ldr] (fp32) += out.
// A and SA must be readable for round_up(M, 256) rows, W / SW / bias / cscale for Npad rows (Npad % 256 == 0,
// zero rows past N); K % 128 == 0.  cscale may be null (all ones).
struct MxGemmParams {
  int epi;
  const unsigned char* A; long lda;
  const unsigned* SA; long sa_ld;
  const unsigned char* W;
  const unsigned* SW;          // [K / 128][Npad]
  const float* bias;
  const float* cscale;
  int M, N, K, Npad;
  bf16_t* C; long ldc;
  float* R; long ldr;
  bf16_t* VT; int hd_pad, heads, n_tok;
  unsigned char* Cq; long ldcq; int ncq;
  unsigned* SC; long sc_ld;
};
hipError_t mx_gemm(const MxGemmParams& p, hipStream_t st);
hipError_t mx_gemm_init();   // raises the dynamic-LDS limit of the kernels (idempotent)
// one v_mfma_scale_f32_32x32x64_f8f6f4 on caller-supplied registers (operand-layout test): a, b [64][8], sa, sb [64], d [64][16]
void mx_mfma_probe(const int* a, const int* b, const int* sa, const int* sb, float* d, hipStream_t st);

// MFMA lane-layout check: D[32,32] = A[32,16] * B[16,32] with operands loaded
// and the result stored under the layout the kernels assume.
void mfma_probe(const bf16_t* A, const bf16_t* B, float* D, hipStream_t st);

}  // namespace epd
