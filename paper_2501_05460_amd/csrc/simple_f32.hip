// fp32 mode of the encode stage: plain, bounds-checked kernels with fp32
// storage and fp32 accumulation.  This mode exists for the small fp32
// configuration (launch-latency bound) and as the on-device numerical
// reference of the bf16 MFMA path; it is not tuned.
#include "kernels.h"

namespace epd {

// ---------------------------------------------------------------- im2col ----
// A[t*N + y*g + x][(c*p + dy)*p + dx] = tiles[t][c][p*y + dy][p*x + dx]
__global__ void k_f32_im2col(const float* __restrict__ tiles, float* __restrict__ A, int S, int p,
                             int g, int Kp, long total) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int e = (int)(i % Kp);
  long row = i / Kp;
  int N = g * g;
  long t = row / N;
  int n = (int)(row % N);
  int y = n / g, x = n % g;
  int c = e / (p * p), r = e % (p * p);
  int dy = r / p, dx = r % p;
  A[i] = tiles[((t * 3 + c) * S + (p * y + dy)) * (long)S + (p * x + dx)];
}

void f32_im2col(const float* tiles, float* A, int T, int S, int p, hipStream_t st) {
  int g = S / p, Kp = 3 * p * p;
  long total = (long)T * g * g * Kp;
  if (total == 0) return;
  int bs = 256;
  k_f32_im2col<<<dim3((unsigned)((total + bs - 1) / bs)), dim3(bs), 0, st>>>(tiles, A, S, p, g, Kp, total);
}

// ------------------------------------------------------------------ GEMM ----
// C[M,N] = A[M,K] * W[N,K]^T, TS x TS block tile (64: 4x4 outputs per thread, 32: 2x2), 64-deep k slab, 256 threads.
// The launches of this mode are small: with 64 x 64 tiles the tiny configuration has a dozen workgroups on 256
// CUs and its time is one thread's chain of 16 K multiply-adds, so launches that would leave most CUs idle take
// 32 x 32 tiles (a quarter of the chain, four times the workgroups).  A thread adds the k-steps of an element in
// ascending order whatever the tile or slab shape: same bits.
constexpr int F32_BK = 64;
template <int EPI, int TS>
__global__ __launch_bounds__(256) void k_f32_gemm(const float* __restrict__ A, int lda,
                                                  const float* __restrict__ W,
                                                  const float* __restrict__ bias, float* C, int ldc,
                                                  const float* __restrict__ pos, int n_pos, int M,
                                                  int N, int K, const int* __restrict__ row_map,
                                                  int block_tokens, SliceRows xrows) {
  constexpr int R = TS / 16;   // outputs per thread in each direction
  __shared__ float sA[F32_BK][TS + 1];
  __shared__ float sW[F32_BK][TS + 1];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  float acc[R][R] = {};
  // the slab after the current one waits in registers, so its memory latency passes under the current slab's
  // arithmetic instead of in front of every slab
  constexpr int PER_T = TS * F32_BK / 256;
  float ra[PER_T], rw[PER_T];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int u = 0; u < PER_T; ++u) {
      const int i = tid + 256 * u;
      const int r = i / F32_BK, kk = i % F32_BK;
      const int gm = m0 + r, gn = n0 + r, gk = k0 + kk;
      ra[u] = (gm < M && gk < K) ? A[(long)gm * lda + gk] : 0.f;
      rw[u] = (gn < N && gk < K) ? W[(long)gn * K + gk] : 0.f;
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += F32_BK) {
#pragma unroll
    for (int u = 0; u < PER_T; ++u) {
      const int i = tid + 256 * u;
      sA[i % F32_BK][i / F32_BK] = ra[u];
      sW[i % F32_BK][i / F32_BK] = rw[u];
    }
    __syncthreads();
    if (k0 + F32_BK < K) fetch(k0 + F32_BK);
#pragma unroll 16
    for (int kk = 0; kk < F32_BK; ++kk) {
      float a[R], w[R];
#pragma unroll
      for (int i = 0; i < R; ++i) a[i] = sA[kk][ty * R + i];
#pragma unroll
      for (int j = 0; j < R; ++j) w[j] = sW[kk][tx * R + j];
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int j = 0; j < R; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < R; ++i) {
    int r = m0 + ty * R + i;
    if (r >= M) continue;
#pragma unroll
    for (int j = 0; j < R; ++j) {
      int c = n0 + tx * R + j;
      if (c >= N) continue;
      float v = acc[i][j] + (bias ? bias[c] : 0.f);
      // paged output: row r of the product lives in block row_map[r / block_tokens]
      const long orow = row_map ? (long)row_map[r / block_tokens] * block_tokens + r % block_tokens : r;
      long o = orow * ldc + c;
      if (EPI == EPI_BIAS_RESIDUAL) {
        C[o] += v;
      } else if (EPI == EPI_BIAS_POS) {
        C[xrows.row(r) * ldc + c] = v + pos[(long)(r % n_pos) * N + c];   // patch embedding: through the slice layout
      } else {
        C[o] = apply_act<EPI>(v);
      }
    }
  }
}

static int f32_cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    n = (hipGetDevice(&dev) == hipSuccess &&
         hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
  }
  return n;
}

template <int TS>
static void f32_gemm_ts(int epi, const float* A, int lda, const float* W, const float* bias, float* C, int ldc,
                        const float* pos, int n_pos, int M, int N, int K, hipStream_t st, const int* row_map,
                        int block_tokens, SliceRows xrows) {
  dim3 grid((N + TS - 1) / TS, (M + TS - 1) / TS), block(256);
  switch (epi) {
    case EPI_BIAS: k_f32_gemm<EPI_BIAS, TS><<<grid, block, 0, st>>>(A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, row_map, block_tokens, xrows); break;
    case EPI_BIAS_GELU_ERF: k_f32_gemm<EPI_BIAS_GELU_ERF, TS><<<grid, block, 0, st>>>(A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, row_map, block_tokens, xrows); break;
    case EPI_BIAS_GELU_TANH: k_f32_gemm<EPI_BIAS_GELU_TANH, TS><<<grid, block, 0, st>>>(A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, row_map, block_tokens, xrows); break;
    case EPI_BIAS_RESIDUAL: k_f32_gemm<EPI_BIAS_RESIDUAL, TS><<<grid, block, 0, st>>>(A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, row_map, block_tokens, xrows); break;
    default: k_f32_gemm<EPI_BIAS_POS, TS><<<grid, block, 0, st>>>(A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, row_map, block_tokens, xrows); break;
  }
}

void f32_gemm(int epi, const float* A, int lda, const float* W, const float* bias, float* C, int ldc,
              const float* pos, int n_pos, int M, int N, int K, hipStream_t st, const int* row_map,
              int block_tokens, SliceRows xrows) {
  if (M == 0 || N == 0) return;
  const long tiles64 = (long)((N + 63) / 64) * ((M + 63) / 64);
  if (tiles64 * 2 <= f32_cu_count()) f32_gemm_ts<32>(epi, A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, st, row_map, block_tokens, xrows);
  else f32_gemm_ts<64>(epi, A, lda, W, bias, C, ldc, pos, n_pos, M, N, K, st, row_map, block_tokens, xrows);
}

// ------------------------------------------------------------------ norm ----
// Logical row R of `dim` elements lives at in + (R / groups) * ld_in + (R % groups) * dim
// (groups > 1: per-head norm inside a wider row).  One wave per row.
__global__ __launch_bounds__(256) void k_f32_norm(int kind, const float* in, long ld_in, float* out,
                                                  long ld_out, const float* __restrict__ gamma,
                                                  const float* __restrict__ beta, long rows, int dim,
                                                  int groups, float eps) {
  long R = (long)blockIdx.x * 4 + threadIdx.x / 64;
  if (R >= rows) return;
  int lane = threadIdx.x % 64;
  const float* x = in + (R / groups) * ld_in + (R % groups) * (long)dim;
  float* y = out + (R / groups) * ld_out + (R % groups) * (long)dim;
  float s = 0.f;
  float mean = 0.f;
  if (kind == 0) {
    for (int i = lane; i < dim; i += 64) s += x[i];
    mean = wave_sum(s) / dim;
  }
  float q = 0.f;
  for (int i = lane; i < dim; i += 64) {
    float d = x[i] - mean;
    q += d * d;
  }
  float rstd = 1.0f / sqrtf(wave_sum(q) / dim + eps);
  for (int i = lane; i < dim; i += 64) {
    float v = (x[i] - mean) * rstd * gamma[i];
    if (kind == 0) v += beta[i];
    y[i] = v;
  }
}

void f32_norm(int kind, const float* in, long ld_in, float* out, long ld_out, const float* gamma,
              const float* beta, long rows, int dim, int groups, float eps, hipStream_t st) {
  if (rows == 0) return;
  k_f32_norm<<<dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st>>>(kind, in, ld_in, out, ld_out, gamma,
                                                                    beta, rows, dim, groups, eps);
}

// ------------------------------------------------------------- attention ----
// One block per (query, head, slice): logits of the slice's N keys in LDS,
// block-wide max and sum, then one thread per output channel.
__global__ __launch_bounds__(128) void k_f32_attention(const float* __restrict__ q, long ld_q, int q_shared,
                                                       const float* __restrict__ k,
                                                       const float* __restrict__ v, long ld,
                                                       float* __restrict__ o, long ldo, int N, int hd,
                                                       float scale) {
  extern __shared__ float sm[];
  float* sc = sm;          // [N]
  float* sq = sm + N;      // [hd]
  __shared__ float red[2];
  const int tid = threadIdx.x;
  const int qi = blockIdx.x, h = blockIdx.y, t = blockIdx.z;
  const long row0 = (long)t * N;
  const long qrow = q_shared ? qi : row0 + qi;
  const long orow = (long)t * gridDim.x + qi;
  for (int d = tid; d < hd; d += 128) sq[d] = q[qrow * ld_q + h * hd + d];
  __syncthreads();
  float mx = -INFINITY;
  for (int j = tid; j < N; j += 128) {
    const float* kr = k + (row0 + j) * ld + h * hd;
    float acc = 0.f;
    for (int d = 0; d < hd; ++d) acc = fmaf(sq[d], kr[d], acc);
    acc *= scale;
    sc[j] = acc;
    mx = fmaxf(mx, acc);
  }
  mx = wave_max(mx);
  if (tid % 64 == 0) red[tid / 64] = mx;
  __syncthreads();
  mx = fmaxf(red[0], red[1]);
  __syncthreads();
  float sum = 0.f;
  for (int j = tid; j < N; j += 128) {
    float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  if (tid % 64 == 0) red[tid / 64] = sum;
  __syncthreads();
  float inv = 1.0f / (red[0] + red[1]);
  for (int d = tid; d < hd; d += 128) {
    float acc = 0.f;
    for (int j = 0; j < N; ++j) acc = fmaf(sc[j], v[(row0 + j) * ld + h * hd + d], acc);
    o[orow * ldo + h * hd + d] = acc * inv;
  }
}

void f32_attention(const float* q, long ld_q, int n_q, int q_shared, const float* k, const float* v, long ld,
                   float* o, long ldo, int T, int N, int H, int hd, float scale, hipStream_t st) {
  if (T == 0) return;
  size_t smem = (size_t)(N + hd) * sizeof(float);
  k_f32_attention<<<dim3(n_q, H, T), dim3(128), smem, st>>>(q, ld_q, q_shared, k, v, ld, o, ldo, N, hd, scale);
}

__global__ void k_f32_add_rows(const float* __restrict__ in, const float* __restrict__ add, int add_rows,
                               float* __restrict__ out, int dim, long total) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  out[i] = in[i] + add[((i / dim) % add_rows) * dim + i % dim];
}

void f32_add_rows(const float* in, const float* add, int add_rows, float* out, long rows, int dim, hipStream_t st) {
  long total = rows * dim;
  if (total == 0) return;
  k_f32_add_rows<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(in, add, add_rows, out, dim, total);
}

// --------------------------------------------------------- pixel shuffle ----
// out[t*N/4 + Y*(g/2) + X][(dy*2 + dx)*D + c] = in[row of patch t*N + (2Y+dy)*g + (2X+dx)][c]
__global__ void k_f32_shuffle(const float* __restrict__ in, SliceRows srows, float* __restrict__ out, int g, int D,
                              long total) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int D4 = 4 * D;
  int e = (int)(i % D4);
  long m = i / D4;
  int h = g / 2;
  long t = m / (h * h);
  int mm = (int)(m % (h * h));
  int Y = mm / h, X = mm % h;
  int blk = e / D, c = e % D;
  int dy = blk / 2, dx = blk % 2;
  long src = srows.row(t * g * g + (long)(2 * Y + dy) * g + (2 * X + dx));
  out[i] = in[src * D + c];
}

void f32_shuffle(const float* in, SliceRows src, float* out, int T, int g, int D, hipStream_t st) {
  long total = (long)T * (g * g / 4) * 4 * D;
  if (total == 0) return;
  k_f32_shuffle<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(in, src, out, g, D, total);
}

__global__ void k_f32_take_rows(const float* __restrict__ in, SliceRows srows, float* __restrict__ out, int D, long total) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  out[i] = in[srows.row(i / D) * D + i % D];
}

void f32_take_rows(const float* in, SliceRows src, float* out, long rows, int D, hipStream_t st) {
  long total = rows * D;
  if (total == 0) return;
  k_f32_take_rows<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(in, src, out, D, total);
}

}  // namespace epd
