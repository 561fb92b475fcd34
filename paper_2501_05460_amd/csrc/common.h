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

__device__ __forceinline__ float gelu_erf_f(float x) {
  return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_tanh_f(float x) {
  const float c = 0.79788456080286535588f;  // sqrt(2/pi)
  return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}

template <int EPI>
__device__ __forceinline__ float apply_act(float v) {
  if (EPI == EPI_BIAS_GELU_ERF) return gelu_erf_f(v);
  if (EPI == EPI_BIAS_GELU_TANH) return gelu_tanh_f(v);
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
