// Shared device-side helpers of the gfx950 encode kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
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
// erf form: x * Phi(x) with erfc(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2),
// t = 1 / (1 + p z), z >= 0 (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7, far
// below one bf16 ulp of the result).
__device__ __forceinline__ float gelu_erf_fast(float x) {
  const float z = fabsf(x) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float poly = fmaf(t, 1.061405429f, -1.453152027f);
  poly = fmaf(t, poly, 1.421413741f);
  poly = fmaf(t, poly, -0.284496736f);
  poly = fmaf(t, poly, 0.254829592f);
  const float erfc_z = poly * t * __builtin_amdgcn_exp2f(-1.4426950408889634f * z * z);  // erfc(|x|/sqrt 2)
  const float phi_neg = 0.5f * erfc_z;                   // Phi(-|x|)
  return x >= 0.f ? x - x * phi_neg : x * phi_neg;       // x Phi(x)
}
// tanh form: 0.5 x (1 + tanh u) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3)
__device__ __forceinline__ float gelu_tanh_fast(float x) {
  const float u = 0.79788456080286535588f * fmaf(0.044715f * x * x, x, x);
  const float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);
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
