// Shared device-side helpers of the gfx950 encode kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
