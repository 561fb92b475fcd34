// HBM-bound row kernels of the bf16 path: im2col of the pixels, the
// fp32 -> bf16 pre-norms (with the optional pixel-shuffle gather in front of
// the projector), the in-place q/k RMSNorm, weight packing, and the MFMA
// layout probe.
#include "kernels.h"

namespace epd {

// ---------------------------------------------------------------- im2col ----
// One thread per 16-byte chunk of the output: 8 consecutive elements of a patch
// vector (order channel, dy, dx), zeros in the K padding; lda % 8 == 0.
__global__ __launch_bounds__(256) void k_bf16_im2col(const float* __restrict__ tiles,
                                                     bf16_t* __restrict__ A, int lda, int S, int p,
                                                     int g, long total) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int per_row = lda >> 3;
  const int e0 = (int)(i % per_row) << 3;
  const long row = i / per_row;
  const int N = g * g, pp = p * p, kp = 3 * pp;
  const long t = row / N;
  const int n = (int)(row % N);
  const int y = n / g, x = n % g;
  const float* base = tiles + (t * 3 * S + (long)p * y) * S + p * x;   // channel 0, dy 0, dx 0 of the patch
  bf16x8 out;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int e = e0 + k;
    const int c = e / pp, r = e % pp;
    out[k] = (bf16_t)(e < kp ? base[((long)c * S + r / p) * S + r % p] : 0.f);
  }
  *reinterpret_cast<bf16x8*>(A + row * (long)lda + e0) = out;
}

void bf16_im2col(const float* tiles, bf16_t* A, int lda, int T, int S, int p, hipStream_t st) {
  const int g = S / p;
  const long total = (long)T * g * g * (lda >> 3);
  if (total == 0) return;
  k_bf16_im2col<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(tiles, A, lda, S, p, g, total);
}

// ------------------------------------------------------------- row norms ----
// One wave per output row, rows of `dim` floats (dim % 4 == 0) held in
// registers when they fit (NV float4 per lane), otherwise re-read.
template <int NV>
__global__ __launch_bounds__(256) void k_bf16_rowop(const RowOpParams p) {
  const long R = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (R >= p.rows) return;
  const int lane = threadIdx.x & 63;
  const int nchunk = p.dim >> 2;

  // source address of float4 chunk c of output row R
  long base_t = 0;
  int Y = 0, X = 0;
  if (p.shuffle) {
    const int hgrid = p.g >> 1;
    const long tok_per = (long)hgrid * hgrid;
    const long t = R / tok_per;
    const int m = (int)(R % tok_per);
    Y = m / hgrid;
    X = m % hgrid;
    base_t = p.src.row(t * p.g * p.g);   // stream row of the slice's patch 0; a slice's patch rows are consecutive
  }
  const long plain_row = p.shuffle ? 0 : p.src.row(R);
  auto src = [&](int c) -> const float4* {
    if (!p.shuffle) return reinterpret_cast<const float4*>(p.in + plain_row * p.ld_in) + c;
    const int e = c << 2;
    const int blk = e / p.D, ch = e % p.D;
    const long srow = base_t + (long)(2 * Y + (blk >> 1)) * p.g + (2 * X + (blk & 1));
    return reinterpret_cast<const float4*>(p.in + srow * p.ld_in + ch);
  };

  float4 v[NV > 0 ? NV : 1];
  float s = 0.f;
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(src(c)));
        v[i] = make_float4(t[0], t[1], t[2], t[3]);
      } else {
        v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
      s += v[i].x + v[i].y + v[i].z + v[i].w;
    }
  } else {
    for (int c = lane; c < nchunk; c += 64) {
      const float4 a = *src(c);
      s += a.x + a.y + a.z + a.w;
    }
  }
  float mean = 0.f, rstd = 1.f;
  if (p.kind != 2) {
    if (p.kind == 0) mean = wave_sum(s) / p.dim;
    float qs = 0.f;
    if (NV > 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        if (c < nchunk) {
          const float a = v[i].x - mean, b = v[i].y - mean, cc = v[i].z - mean, d = v[i].w - mean;
          qs += a * a + b * b + cc * cc + d * d;
        }
      }
    } else {
      for (int c = lane; c < nchunk; c += 64) {
        const float4 t4 = *src(c);
        const float a = t4.x - mean, b = t4.y - mean, cc = t4.z - mean, d = t4.w - mean;
        qs += a * a + b * b + cc * cc + d * d;
      }
    }
    rstd = 1.0f / sqrtf(wave_sum(qs) / p.dim + p.eps);
  }
  bf16_t* out = p.out + R * p.ld_out;
  auto emit = [&](int c, float4 a) {
    float r[4] = {a.x, a.y, a.z, a.w};
    if (p.kind != 2) {
      const float4 gm = *(reinterpret_cast<const float4*>(p.gamma) + c);
      r[0] = (r[0] - mean) * rstd * gm.x;
      r[1] = (r[1] - mean) * rstd * gm.y;
      r[2] = (r[2] - mean) * rstd * gm.z;
      r[3] = (r[3] - mean) * rstd * gm.w;
      if (p.kind == 0) {
        const float4 bt = *(reinterpret_cast<const float4*>(p.beta) + c);
        r[0] += bt.x; r[1] += bt.y; r[2] += bt.z; r[3] += bt.w;
      }
    }
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16_t)r[e];
    *(reinterpret_cast<bf16x4*>(out) + c) = o;
  };
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) emit(c, v[i]);
    }
  } else {
    for (int c = lane; c < nchunk; c += 64) emit(c, *src(c));
  }
}

void bf16_rowop(const RowOpParams& p, hipStream_t st) {
  if (p.rows == 0) return;
  dim3 grid((unsigned)((p.rows + 3) / 4)), block(256);
  const int per_lane = (p.dim / 4 + 63) / 64;
  if (per_lane <= 4) k_bf16_rowop<4><<<grid, block, 0, st>>>(p);
  else if (per_lane <= 8) k_bf16_rowop<8><<<grid, block, 0, st>>>(p);
  else if (per_lane <= 16) k_bf16_rowop<16><<<grid, block, 0, st>>>(p);
  else k_bf16_rowop<0><<<grid, block, 0, st>>>(p);
}

// ---------------------------------------- pre-norm of bf16 rows, in place ----
// The residual epilogues leave bf16(x) of the rows they update; this kernel turns such rows into the normalised
// operand of the next product in place: a third less traffic than reading the fp32 stream (2 + 2 instead of
// 4 + 2 bytes per element).  One wave per row, the row held in registers (NV chunks of 8 elements per lane;
// NV = 0: read twice), statistics in fp32 over the rounded values.  dim % 8 == 0, rows 16-byte aligned.
template <int NV>
__global__ __launch_bounds__(256) void k_bf16_norm_rows(bf16_t* __restrict__ x, long ld, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, long rows, int dim, int kind,
                                                        float eps) {
  const long R = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (R >= rows) return;
  const int lane = threadIdx.x & 63;
  bf16x8* row = reinterpret_cast<bf16x8*>(x + R * ld);
  const int nchunk = dim >> 3;
  bf16x8 v[NV > 0 ? NV : 1];
  float s = 0.f;
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        v[i] = row[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) s += (float)v[i][e];
      }
    }
  } else {
    for (int c = lane; c < nchunk; c += 64) {
      const bf16x8 a = row[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) s += (float)a[e];
    }
  }
  const float mean = kind == 0 ? wave_sum(s) / dim : 0.f;
  float qs = 0.f;
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nchunk) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float d = (float)v[i][e] - mean; qs = __builtin_fmaf(d, d, qs); }
      }
  } else {
    for (int c = lane; c < nchunk; c += 64) {
      const bf16x8 a = row[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = (float)a[e] - mean; qs = __builtin_fmaf(d, d, qs); }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(qs) / dim + eps);
  auto emit = [&](int c, bf16x8 a) {
    bf16x8 o;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float4 gm = *(reinterpret_cast<const float4*>(gamma) + 2 * c + h);
      float r[4] = {((float)a[4 * h + 0] - mean) * rstd * gm.x, ((float)a[4 * h + 1] - mean) * rstd * gm.y,
                    ((float)a[4 * h + 2] - mean) * rstd * gm.z, ((float)a[4 * h + 3] - mean) * rstd * gm.w};
      if (kind == 0) {
        const float4 bt = *(reinterpret_cast<const float4*>(beta) + 2 * c + h);
        r[0] += bt.x; r[1] += bt.y; r[2] += bt.z; r[3] += bt.w;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) o[4 * h + e] = (bf16_t)r[e];
    }
    row[c] = o;
  };
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nchunk) emit(lane + 64 * i, v[i]);
  } else {
    for (int c = lane; c < nchunk; c += 64) emit(c, row[c]);
  }
}

void bf16_norm_rows(bf16_t* x, long ld, const float* gamma, const float* beta, long rows, int dim, int kind, float eps,
                    hipStream_t st) {
  if (rows == 0) return;
  const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
  const int per_lane = (dim / 8 + 63) / 64;
  if (per_lane <= 2) k_bf16_norm_rows<2><<<grid, block, 0, st>>>(x, ld, gamma, beta, rows, dim, kind, eps);
  else if (per_lane <= 4) k_bf16_norm_rows<4><<<grid, block, 0, st>>>(x, ld, gamma, beta, rows, dim, kind, eps);
  else if (per_lane <= 8) k_bf16_norm_rows<8><<<grid, block, 0, st>>>(x, ld, gamma, beta, rows, dim, kind, eps);
  else k_bf16_norm_rows<0><<<grid, block, 0, st>>>(x, ld, gamma, beta, rows, dim, kind, eps);
}

// ------------------------------------------------------- row statistics ----
// One wave per row: lane l holds columns 4 (l + 64 j) .. + 3 in round j, so the lower half of the wave covers
// group 2 j of 128 columns and the upper half group 2 j + 1: the lane layout of the residual epilogue.
__global__ __launch_bounds__(256) void k_bf16_row_stats(const float* __restrict__ x, long ldx, long rows, int dim,
                                                        bf16_t* __restrict__ xb, long ldxb, float* __restrict__ stats,
                                                        int n_part) {
  const long R = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (R >= rows) return;
  const int lane = threadIdx.x & 63;
  for (int j = 0; j * 256 < dim; ++j) {
    const int col = 4 * (lane + 64 * j), g = col / STAT_GROUP;
    const bool valid = col < dim;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (valid) {
      v = *reinterpret_cast<const f32x4*>(x + R * ldx + col);
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16_t)v[e];
      *reinterpret_cast<bf16x4*>(xb + R * ldxb + col) = o;
    }
    const int cnt = dim - g * STAT_GROUP < STAT_GROUP ? dim - g * STAT_GROUP : STAT_GROUP;
    float mean, m2;
    group_mean_m2(v, valid, cnt > 0 ? 1.0f / (float)cnt : 0.f, mean, m2);
    if ((lane & 31) == 0 && g < n_part) *reinterpret_cast<float2*>(stats + (R * n_part + g) * 2) = make_float2(mean, m2);
  }
}

void bf16_row_stats(const float* x, long ldx, long rows, int dim, bf16_t* xb, long ldxb, float* stats, int n_part,
                    hipStream_t st) {
  if (rows == 0) return;
  k_bf16_row_stats<<<dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st>>>(x, ldx, rows, dim, xb, ldxb, stats, n_part);
}

__global__ __launch_bounds__(256) void k_combine_stats(const float* __restrict__ stats, long rows, int n_part, int dim,
                                                       float* __restrict__ out) {
  const long r = (long)blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  const float* pairs = stats + r * n_part * 2;
  const float2 c = combine_pairs([&](int g) { return *reinterpret_cast<const float2*>(pairs + 2 * g); }, n_part, STAT_GROUP, dim);
  *reinterpret_cast<float2*>(out + 2 * r) = c;
}

void bf16_combine_stats(const float* stats, long rows, int n_part, int dim, float* out, hipStream_t st) {
  if (rows == 0) return;
  k_combine_stats<<<dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st>>>(stats, rows, n_part, dim, out);
}

// One wave per row of the packed matrix.  The sums run lane-strided over k and end in a wave reduction: a
// fixed order, so a context built twice holds the same bits.
__global__ __launch_bounds__(256) void k_fold_norm(bf16_t* __restrict__ W, int rows, int cols, long ld,
                                                   const float* __restrict__ gamma, const float* __restrict__ beta,
                                                   int dim, float* __restrict__ bias, float* __restrict__ colsum) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  bf16_t* w = W + (long)r * ld;
  float dot = 0.f, cs = 0.f;
  for (int k = lane; k < cols; k += 64) {
    float v = (float)w[k];
    if (k < dim) {
      if (beta) dot = __builtin_fmaf(v, beta[k], dot);
      const bf16_t scaled = (bf16_t)(v * gamma[k]);
      w[k] = scaled;
      v = (float)scaled;
    }
    cs += v;
  }
  dot = wave_sum(dot);
  cs = wave_sum(cs);
  if (lane == 0) {
    if (beta) bias[r] += dot;
    colsum[r] = cs;
  }
}

void fold_norm_into_linear(bf16_t* W, int rows, int cols, long ld, const float* gamma, const float* beta, int dim,
                           float* bias, float* colsum, hipStream_t st) {
  if (rows == 0) return;
  k_fold_norm<<<dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st>>>(W, rows, cols, ld, gamma, beta, dim, bias, colsum);
}

// --------------------------------------------------------- q/k RMSNorm ------
// One wave per logical row, q rows first, then k rows (k = q + k_off elements, its own gain).  The
// row waits in registers between the sum of squares and the scaling when it fits (NV chunks per
// lane), otherwise it is read twice.
template <int NV, int W>   // W = elements per chunk: 8 (16-byte accesses) when the row length allows, else 4
__global__ __launch_bounds__(256) void k_bf16_qknorm(bf16_t* buf, long ld, long k_off,
                                                     const float* __restrict__ gamma_q,
                                                     const float* __restrict__ gamma_k, long rows,
                                                     int dim, int groups, int count, float eps) {
  typedef __bf16 vec_t __attribute__((ext_vector_type(W)));
  long R = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (R >= 2 * rows) return;
  const bool is_k = R >= rows;
  if (is_k) R -= rows;
  const float* gamma = is_k ? gamma_k : gamma_q;
  const int lane = threadIdx.x & 63;
  vec_t* x = reinterpret_cast<vec_t*>(buf + (is_k ? k_off : 0) + (R / groups) * ld + (R % groups) * (long)dim);
  const int nchunk = dim / W;
  vec_t v[NV > 0 ? NV : 1];
  float qs = 0.f;
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) {
        v[i] = x[c];
#pragma unroll
        for (int e = 0; e < W; ++e) qs += (float)v[i][e] * (float)v[i][e];
      }
    }
  } else {
    for (int c = lane; c < nchunk; c += 64) {
      const vec_t a = x[c];
#pragma unroll
      for (int e = 0; e < W; ++e) qs += (float)a[e] * (float)a[e];
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(qs) / count + eps);
  auto emit = [&](int c, vec_t a) {
    vec_t o;
#pragma unroll
    for (int h = 0; h < W / 4; ++h) {
      const float4 gm = *(reinterpret_cast<const float4*>(gamma) + c * (W / 4) + h);
      o[4 * h + 0] = (bf16_t)((float)a[4 * h + 0] * rstd * gm.x);
      o[4 * h + 1] = (bf16_t)((float)a[4 * h + 1] * rstd * gm.y);
      o[4 * h + 2] = (bf16_t)((float)a[4 * h + 2] * rstd * gm.z);
      o[4 * h + 3] = (bf16_t)((float)a[4 * h + 3] * rstd * gm.w);
    }
    x[c] = o;
  };
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunk) emit(c, v[i]);
    }
  } else {
    for (int c = lane; c < nchunk; c += 64) emit(c, x[c]);
  }
}

template <int W>
static void bf16_qknorm_w(bf16_t* buf, long ld, long k_off, const float* gamma_q, const float* gamma_k, long rows,
                          int dim, int groups, int count, float eps, hipStream_t st) {
  const dim3 grid((unsigned)((2 * rows + 3) / 4)), block(256);
  const int per_lane = (dim / W + 63) / 64;
  if (per_lane <= 2) k_bf16_qknorm<2, W><<<grid, block, 0, st>>>(buf, ld, k_off, gamma_q, gamma_k, rows, dim, groups, count, eps);
  else if (per_lane <= 8) k_bf16_qknorm<8, W><<<grid, block, 0, st>>>(buf, ld, k_off, gamma_q, gamma_k, rows, dim, groups, count, eps);
  else if (per_lane <= 16 && W == 4) k_bf16_qknorm<16, W><<<grid, block, 0, st>>>(buf, ld, k_off, gamma_q, gamma_k, rows, dim, groups, count, eps);
  else k_bf16_qknorm<0, W><<<grid, block, 0, st>>>(buf, ld, k_off, gamma_q, gamma_k, rows, dim, groups, count, eps);
}

void bf16_qknorm(bf16_t* buf, long ld, long k_off, const float* gamma_q, const float* gamma_k, long rows, int dim,
                 int groups, int count, float eps, hipStream_t st) {
  if (rows == 0) return;
  // 16-byte chunks when every row starts on a 16-byte boundary and holds whole chunks
  const bool wide = dim % 8 == 0 && ld % 8 == 0 && k_off % 8 == 0 && (reinterpret_cast<uintptr_t>(buf) & 15) == 0;
  if (wide) bf16_qknorm_w<8>(buf, ld, k_off, gamma_q, gamma_k, rows, dim, groups, count, eps, st);
  else bf16_qknorm_w<4>(buf, ld, k_off, gamma_q, gamma_k, rows, dim, groups, count, eps, st);
}

// ---------------------------------------------- LayerNorm of bf16 rows ------
// One wave per row; the row is read twice (statistics, then output).
__global__ __launch_bounds__(256) void k_bf16_ln_rows(const bf16_t* __restrict__ in, long ld_in,
                                                      const float* __restrict__ gamma,
                                                      const float* __restrict__ beta, float eps,
                                                      bf16_t* __restrict__ out, long ld_out,
                                                      bf16_t* __restrict__ out_plus,
                                                      const float* __restrict__ add, int add_rows, long rows,
                                                      int dim) {
  const long R = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (R >= rows) return;
  const int lane = threadIdx.x & 63;
  const bf16x4* x = reinterpret_cast<const bf16x4*>(in + R * ld_in);
  const int nchunk = dim >> 2;
  float s = 0.f;
  for (int c = lane; c < nchunk; c += 64) {
    const bf16x4 a = x[c];
    s += (float)a[0] + (float)a[1] + (float)a[2] + (float)a[3];
  }
  const float mean = wave_sum(s) / dim;
  float qs = 0.f;
  for (int c = lane; c < nchunk; c += 64) {
    const bf16x4 a = x[c];
#pragma unroll
    for (int e = 0; e < 4; ++e) { const float d = (float)a[e] - mean; qs += d * d; }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(qs) / dim + eps);
  const float* arow = out_plus ? add + (R % add_rows) * (long)dim : nullptr;
  for (int c = lane; c < nchunk; c += 64) {
    const bf16x4 a = x[c];
    const float4 gm = reinterpret_cast<const float4*>(gamma)[c], bt = reinterpret_cast<const float4*>(beta)[c];
    const float r[4] = {((float)a[0] - mean) * rstd * gm.x + bt.x, ((float)a[1] - mean) * rstd * gm.y + bt.y,
                        ((float)a[2] - mean) * rstd * gm.z + bt.z, ((float)a[3] - mean) * rstd * gm.w + bt.w};
    bf16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16_t)r[e];
    reinterpret_cast<bf16x4*>(out + R * ld_out)[c] = o;
    if (out_plus) {
      const float4 ad = reinterpret_cast<const float4*>(arow)[c];
      bf16x4 p;
      p[0] = (bf16_t)(r[0] + ad.x); p[1] = (bf16_t)(r[1] + ad.y); p[2] = (bf16_t)(r[2] + ad.z); p[3] = (bf16_t)(r[3] + ad.w);
      reinterpret_cast<bf16x4*>(out_plus + R * ld_out)[c] = p;
    }
  }
}

void bf16_ln_rows(const bf16_t* in, long ld_in, const float* gamma, const float* beta, float eps, bf16_t* out,
                  long ld_out, bf16_t* out_plus, const float* add, int add_rows, long rows, int dim, hipStream_t st) {
  if (rows == 0) return;
  k_bf16_ln_rows<<<dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st>>>(in, ld_in, gamma, beta, eps, out, ld_out,
                                                                        out_plus, add, add_rows, rows, dim);
}

// --------------------------------------------------------------- packing ----
__device__ __forceinline__ int unpad_index(int i, PackMap m, int limit) {
  if (m.hd == 0) return i < limit ? i : -1;
  const int per = m.heads * m.hd_pad;
  const int blk = i / per, w = i % per;
  const int h = w / m.hd_pad, d = w % m.hd_pad;
  if (d >= m.hd) return -1;
  const int s = blk * m.heads * m.hd + h * m.hd + d;
  return s < limit ? s : -1;
}

__global__ void k_pack_matrix(const bf16_t* __restrict__ src, int rows, int cols, bf16_t* __restrict__ dst,
                              int rows_pad, int cols_pad, PackMap rmap, PackMap cmap) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)rows_pad * cols_pad) return;
  const int r = (int)(i / cols_pad), c = (int)(i % cols_pad);
  const int sr = unpad_index(r, rmap, rows), sc = unpad_index(c, cmap, cols);
  dst[i] = (sr >= 0 && sc >= 0) ? src[(long)sr * cols + sc] : (bf16_t)0.f;
}

void pack_matrix_bf16(const bf16_t* src, int rows, int cols, bf16_t* dst, int rows_pad, int cols_pad,
                      PackMap rmap, PackMap cmap, hipStream_t st) {
  const long total = (long)rows_pad * cols_pad;
  if (total == 0) return;
  k_pack_matrix<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(src, rows, cols, dst, rows_pad,
                                                                            cols_pad, rmap, cmap);
}

__global__ void k_pack_vector(const void* __restrict__ src, int src_is_bf16, int n, float* __restrict__ dst,
                              int n_pad, PackMap map) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pad) return;
  const int s = unpad_index(i, map, n);
  float v = 0.f;
  if (s >= 0) v = src_is_bf16 ? (float)reinterpret_cast<const bf16_t*>(src)[s] : reinterpret_cast<const float*>(src)[s];
  dst[i] = v;
}

void pack_vector_f32(const void* src, int src_is_bf16, int n, float* dst, int n_pad, PackMap map,
                     hipStream_t st) {
  if (n_pad == 0) return;
  k_pack_vector<<<dim3((n_pad + 255) / 256), dim3(256), 0, st>>>(src, src_is_bf16, n, dst, n_pad, map);
}

template <typename T>
__global__ void k_scale_rows(T* __restrict__ W, int rows, int cols, long ld, float* __restrict__ b,
                             const float* __restrict__ s) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)rows * cols) return;
  const int r = (int)(i / cols), c = (int)(i % cols);
  W[(long)r * ld + c] = (T)((float)W[(long)r * ld + c] * s[r]);
  if (c == 0) b[r] *= s[r];
}

void scale_rows(void* W, int w_is_bf16, int rows, int cols, long ld, float* b, const float* s, hipStream_t st) {
  const long total = (long)rows * cols;
  if (total == 0) return;
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (w_is_bf16) k_scale_rows<bf16_t><<<grid, block, 0, st>>>((bf16_t*)W, rows, cols, ld, b, s);
  else k_scale_rows<float><<<grid, block, 0, st>>>((float*)W, rows, cols, ld, b, s);
}

// W[r][0..cols) *= c and b[r] *= c for r < rows (bf16 matrix, fp32 bias)
__global__ void k_scale_rows_by(bf16_t* __restrict__ W, int rows, int cols, long ld, float* __restrict__ b, float c) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)rows * cols) return;
  const int r = (int)(i / cols), k = (int)(i % cols);
  W[(long)r * ld + k] = (bf16_t)((float)W[(long)r * ld + k] * c);
  if (k == 0) b[r] *= c;
}

void scale_rows_by(bf16_t* W, int rows, int cols, long ld, float* b, float c, hipStream_t st) {
  const long total = (long)rows * cols;
  if (total == 0) return;
  k_scale_rows_by<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(W, rows, cols, ld, b, c);
}

__global__ void k_scale_vector(float* __restrict__ v, int n, float c) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) v[i] *= c;
}

void scale_vector(float* v, int n, float c, hipStream_t st) {
  if (n <= 0) return;
  k_scale_vector<<<dim3((n + 255) / 256), dim3(256), 0, st>>>(v, n, c);
}

// ------------------------------------------------- paged cache block copy ----
// `per_block` consecutive workgroups share one cache block, each moving chunks
// of 16 KiB: a thread issues four 16-byte loads before the four stores, so a
// wave keeps 4 KiB in flight.  Streaming (nontemporal) on both sides: nothing
// is read twice.  HBM-bound: every byte is read once and written once.
__global__ __launch_bounds__(256) void k_mm_copy_blocks(const unsigned char* __restrict__ src_pool,
                                                        const int* __restrict__ src_ids,
                                                        unsigned char* __restrict__ dst_pool,
                                                        const int* __restrict__ dst_ids, long block_bytes,
                                                        int per_block) {
  const int b = blockIdx.x / per_block, part = blockIdx.x % per_block;
  const long sb = src_ids ? src_ids[b] : b, db = dst_ids ? dst_ids[b] : b;
  const u32x4* s = reinterpret_cast<const u32x4*>(src_pool + sb * block_bytes);
  u32x4* d = reinterpret_cast<u32x4*>(dst_pool + db * block_bytes);
  const long n16 = block_bytes >> 4;
  for (long base = (long)part * 1024; base < n16; base += (long)per_block * 1024) {
    const long i = base + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i + j * 256 < n16) v[j] = __builtin_nontemporal_load(s + i + j * 256);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (i + j * 256 < n16) __builtin_nontemporal_store(v[j], d + i + j * 256);
  }
}

void mm_copy_blocks(const void* src_pool, const int* src_ids, void* dst_pool, const int* dst_ids,
                    int n_blocks, long block_bytes, hipStream_t st) {
  if (n_blocks <= 0 || block_bytes <= 0) return;
  const long n16 = block_bytes >> 4;
  int per_block = (int)((n16 + 1023) / 1024);  // one 16 KiB chunk per workgroup while the grid stays modest
  if (per_block < 1) per_block = 1;
  if (per_block > 8) per_block = 8;
  k_mm_copy_blocks<<<dim3((unsigned)n_blocks * per_block), dim3(256), 0, st>>>(
      (const unsigned char*)src_pool, src_ids, (unsigned char*)dst_pool, dst_ids, block_bytes, per_block);
}

// ------------------------------------- residual stream <-> paged cache rows ----
// One thread per element; consecutive threads walk one row, so both sides are
// coalesced.  TO_POOL: stream -> cache (rounding to the cache's type), else the
// reverse (exact widening).
template <typename T, bool TO_POOL>
__global__ __launch_bounds__(256) void k_stream_blocks(float* X, long ldx, SliceRows xr, T* pool, int dim,
                                                       const int* __restrict__ row_map, int block_tokens,
                                                       long total) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long)gridDim.x * 256) {
    const long r = i / dim;
    const int c = (int)(i % dim);
    const long prow = (long)row_map[r / block_tokens] * block_tokens + r % block_tokens;
    const long xrow = xr.row(r);
    if (TO_POOL) pool[prow * dim + c] = (T)X[xrow * ldx + c];
    else X[xrow * ldx + c] = (float)pool[prow * dim + c];
  }
}

// ------------------------------- class-token and padding rows of the stream ----
// One thread per element of a row that no product writes.
__global__ __launch_bounds__(256) void k_fill_slice_rows(float* X, int D, int stride, int n_real, int extra,
                                                         const float* __restrict__ cls,
                                                         const float* __restrict__ pos0, long total) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % D);
  const long rr = i / D;
  const long t = rr / extra;
  const int e = (int)(rr % extra);       // 0: class row (when there is one), then the padding rows
  const bool is_cls = cls && e == 0;
  const int row = is_cls ? 0 : n_real + e - (cls ? 1 : 0);
  X[(t * stride + row) * (long)D + c] = is_cls ? cls[c] + pos0[c] : 0.f;
}

void fill_slice_rows(float* X, int D, int T, int stride, int n_real, const float* cls, const float* pos0,
                     hipStream_t st) {
  const int extra = (cls ? 1 : 0) + (stride - n_real);
  const long total = (long)T * extra * D;
  if (total <= 0) return;
  k_fill_slice_rows<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(X, D, stride, n_real, extra, cls, pos0, total);
}

static unsigned stream_blocks_grid(long total) {
  long g = (total + 255) / 256;
  return (unsigned)(g > 65536 ? 65536 : g);
}

void stream_to_blocks(const float* X, long ldx, SliceRows xr, void* pool, int pool_is_bf16, int dim, const int* row_map,
                      int block_tokens, long rows, hipStream_t st) {
  const long total = rows * dim;
  if (total <= 0) return;
  const dim3 grid(stream_blocks_grid(total)), block(256);
  if (pool_is_bf16)
    k_stream_blocks<bf16_t, true><<<grid, block, 0, st>>>(const_cast<float*>(X), ldx, xr, (bf16_t*)pool, dim, row_map, block_tokens, total);
  else
    k_stream_blocks<float, true><<<grid, block, 0, st>>>(const_cast<float*>(X), ldx, xr, (float*)pool, dim, row_map, block_tokens, total);
}

void blocks_to_stream(const void* pool, int pool_is_bf16, int dim, const int* row_map, int block_tokens,
                      float* X, long ldx, SliceRows xr, long rows, hipStream_t st) {
  const long total = rows * dim;
  if (total <= 0) return;
  const dim3 grid(stream_blocks_grid(total)), block(256);
  if (pool_is_bf16)
    k_stream_blocks<bf16_t, false><<<grid, block, 0, st>>>(X, ldx, xr, (bf16_t*)pool, dim, row_map, block_tokens, total);
  else
    k_stream_blocks<float, false><<<grid, block, 0, st>>>(X, ldx, xr, (float*)pool, dim, row_map, block_tokens, total);
}

// ------------------------------------------------------------ MFMA probe ----
__global__ __launch_bounds__(64) void k_mfma_probe(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                   float* __restrict__ D) {
  const int l = threadIdx.x, l32 = l & 31, lh = l >> 5;
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a[j] = A[l32 * 16 + lh * 8 + j];          // A[m][k], row-major 32 x 16
    b[j] = B[(lh * 8 + j) * 32 + l32];        // B[k][n], row-major 16 x 32
  }
  f32x16 c;
#pragma unroll
  for (int e = 0; e < 16; ++e) c[e] = 0.f;
  c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#pragma unroll
  for (int i = 0; i < 16; ++i) D[(8 * (i / 4) + 4 * lh + (i % 4)) * 32 + l32] = c[i];
}

void mfma_probe(const bf16_t* A, const bf16_t* B, float* D, hipStream_t st) {
  k_mfma_probe<<<dim3(1), dim3(64), 0, st>>>(A, B, D);
}

}  // namespace epd
