// Shared device-side helpers of the gfx950 encode kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define EPD_WAVE 64

// Epilogue kinds shared by the fp32 and the bf16 GEMMs.
enum EpiKind : int {
  EPI_BIAS = 0,           // out = acc + bias
  EPI_BIAS_GELU_ERF = 1,  // out = gelu_erf(acc + bias)
  EPI_BIAS_GELU_TANH = 2, // out = gelu_tanh(acc + bias)
  EPI_BIAS_RESIDUAL = 3,  // res[r][c] += acc + bias   (fp32 residual stream, in place)
  EPI_BIAS_POS = 4,       // res[r][c]  = acc + bias + pos[r % n_pos][c]
  EPI_VT = 5              // out = acc + bias, written transposed per (slice, head): VT[t][h][d][n]
};

// Exact-form and tanh-form GELU for the fp32 path.
__device__ __forceinline__ float gelu_erf_f(float x) {
  return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float c = 0.79788456080286535588f;  // sqrt(2/pi)
  return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}

// GELU for the bf16 epilogues: branch-free, one exp and one reciprocal each.
// erf form: x * Phi(x) with Phi(x) ~= 1 / (1 + exp(-x (a + b x^2))), the logistic
// shape of the tanh form with both coefficients fitted (minimax over |x| <= 7)
// to x * Phi(x) itself: |error| <= 2.7e-4 (the tanh form's own coefficients
// give 4.7e-4), the size of a bf16 rounding step at |y| = 0.07 and below the
// rounding of any larger output.  b > 0, so the exponent is monotonic and needs
// no clamp: it overflows to +inf / underflows to 0 exactly where Phi is 0 / 1.
// A third term (c x^4, with the argument clamped to +-7) brought the error to
// 2.6e-5 and cost 3 % of the FC1 product's time.  The coefficients carry the
// factor -log2(e) of exp2.
__device__ __forceinline__ float gelu_erf_fast(float x) {
  const float e = __builtin_amdgcn_exp2f(x * fmaf(x * x, -1.001257265e-01f, -2.308765046e+00f));
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}
// tanh form: 0.5 x (1 + tanh u) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3);
// -2 log2(e) sqrt(2/pi) is folded into the two coefficients of exp2's argument.
__device__ __forceinline__ float gelu_tanh_fast(float x) {
  const float e = __builtin_amdgcn_exp2f(x * fmaf(x * x, -1.029432396e-01f, -2.302208198e+00f));
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int EPI>
__device__ __forceinline__ float apply_act(float v) {
  if (EPI == EPI_BIAS_GELU_ERF) return gelu_erf_f(v);
  if (EPI == EPI_BIAS_GELU_TANH) return gelu_tanh_f(v);
  return v;
}
template <int EPI>
__device__ __forceinline__ float apply_act_fast(float v) {
  if (EPI == EPI_BIAS_GELU_ERF) return gelu_erf_fast(v);
  if (EPI == EPI_BIAS_GELU_TANH) return gelu_tanh_fast(v);
  return v;
}

// ---- MXFP8 conversion (OCP Microscaling Formats v1.0: E4M3 elements, one power-of-two scale per block of 32) ----
// Scale byte of a block whose largest magnitude is amax (finite fp32): floor(log2(amax)) - 8 + 127 is the
// biased fp32 exponent minus 8; clamped at 0 (zero blocks, and magnitudes below 2^-119).
__device__ __forceinline__ unsigned mx_scale_byte(float amax) {
  const int b = (int)((__float_as_uint(amax) >> 23) & 0xffu) - 8;
  return (unsigned)(b > 0 ? b : 0);
}
// 2^(127 - byte): the factor that brings a block's elements into E4M3's range (exact: a power of two)
__device__ __forceinline__ float mx_inv_scale(unsigned byte) { return __uint_as_float((254u - byte) << 23); }

// four scaled values -> four E4M3 bytes (element 0 in the low byte); saturation by the clamp, rounding to
// nearest even by the conversion instruction
__device__ __forceinline__ unsigned mx_pack4(float a, float b, float c, float d) {
  a = __builtin_amdgcn_fmed3f(a, -448.f, 448.f);
  b = __builtin_amdgcn_fmed3f(b, -448.f, 448.f);
  c = __builtin_amdgcn_fmed3f(c, -448.f, 448.f);
  d = __builtin_amdgcn_fmed3f(d, -448.f, 448.f);
  int r = 0;
  r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, r, false);
  r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
  return (unsigned)r;
}


__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Sum over the 32 lanes of each half of a wave (lanes 0-31 and 32-63 apart); every lane of a half gets its
// half's sum.  Four DPP exchanges inside the rows of 16 lanes (xor 1, xor 2, mirror inside 8, mirror inside
// 16), then the two rows of a half are added through the row swap.  The additions of a step are the same
// pair in both lanes that take part (a + b and b + a), so all lanes hold the same bits, and the order of
// the additions depends on nothing but the lane numbers.
__device__ __forceinline__ float half_wave_sum(float v) {
  auto dpp = [](float x, auto ctrl) {
    constexpr int C = decltype(ctrl)::value;
    return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), C, 0xf, 0xf, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1, 0, 3, 2]
  v += dpp(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2, 3, 0, 1]
  v += dpp(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v += dpp(v, std::integral_constant<int, 0x140>{});   // row_mirror
  const unsigned b = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(b, b, false, false);   // r[0]: even rows in both rows of a pair, r[1]: odd rows
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Pre-norm statistics of a row of the residual stream, kept as one (mean, sum of squared deviations from that
// mean) pair per group of 128 columns: each pair is exact to rounding whatever the row's offset, and the pairs
// combine without cancellation (pairwise update of means and squared deviations).  STAT_GROUP columns per pair.
#define STAT_GROUP 128

// One group's pair from the four values a lane of the half-wave holds (lanes whose columns lie past the row
// pass valid = false and contribute nothing); inv_cnt = 1 / (columns of the group inside the row).
__device__ __forceinline__ void group_mean_m2(const f32x4 v, bool valid, float inv_cnt, float& mean, float& m2) {
  const float s = valid ? (v[0] + v[1]) + (v[2] + v[3]) : 0.f;
  mean = half_wave_sum(s) * inv_cnt;
  float q = 0.f;
  if (valid) {
    const float a = v[0] - mean, b = v[1] - mean, c = v[2] - mean, d = v[3] - mean;
    q = __builtin_fmaf(d, d, __builtin_fmaf(c, c, __builtin_fmaf(b, b, a * a)));
  }
  m2 = half_wave_sum(q);
}

// Mean and sum of squared deviations of a whole row of `dim` columns from its n_part pairs over groups of
// `group` columns (the last group may be shorter), combined pairwise: no difference of large sums anywhere.
// get(g) returns pair g as a float2.
template <typename Get>
__device__ __forceinline__ float2 combine_pairs(Get get, int n_part, int group, int dim) {
  float ms = 0.f;
  for (int g = 0; g < n_part; ++g) {
    const int cnt = dim - g * group < group ? dim - g * group : group;
    ms = __builtin_fmaf((float)cnt, get(g).x, ms);
  }
  const float mu = ms / (float)dim;
  float m2 = 0.f;
  for (int g = 0; g < n_part; ++g) {
    const int cnt = dim - g * group < group ? dim - g * group : group;
    const float2 pr = get(g);
    const float d = pr.x - mu;
    m2 += __builtin_fmaf((float)cnt * d, d, pr.y);
  }
  return make_float2(mu, m2);
}

// The pairs of one row held in registers: loaded in one batch (the loads are independent, so their latency
// is paid once and can pass under other work), combined later into the row's mean and 1 / sqrt(variance + eps)
// (rms: 1 / sqrt(mean square + eps), and the mean returned as 0: nothing is subtracted).  At most STAT_REGS
// pairs per row: wider rows are first combined into a single pair per row by a kernel of their own.
#define STAT_REGS 10
struct RowPairs {
  float2 pr[STAT_REGS];
  __device__ __forceinline__ void load(const float* __restrict__ pairs, int n_part) {
#pragma unroll
    for (int g = 0; g < STAT_REGS; ++g)
      pr[g] = g < n_part ? *reinterpret_cast<const float2*>(pairs + 2 * g) : make_float2(0.f, 0.f);
  }
  __device__ __forceinline__ void finish(int n_part, int group, int dim, int rms, float eps, float& mean, float& rstd) const {
    float ms = 0.f;
#pragma unroll
    for (int g = 0; g < STAT_REGS; ++g)
      if (g < n_part) {
        const int cnt = dim - g * group < group ? dim - g * group : group;
        ms = __builtin_fmaf((float)cnt, pr[g].x, ms);
      }
    const float mu = ms / (float)dim;
    float m2 = 0.f;
#pragma unroll
    for (int g = 0; g < STAT_REGS; ++g)
      if (g < n_part) {
        const int cnt = dim - g * group < group ? dim - g * group : group;
        const float d = pr[g].x - mu;
        m2 += __builtin_fmaf((float)cnt * d, d, pr[g].y);
      }
    float var = m2 / (float)dim;
    if (rms) var = __builtin_fmaf(mu, mu, var);
    mean = rms ? 0.f : mu;
    rstd = 1.0f / sqrtf(var + eps);
  }
};
