// Measured ceilings of the chip, for the benchmark's roofline figures (test / measurement hooks, not on
// the encode path): a register-resident MFMA loop and a plain streaming copy.  See include/epd_encode_test.h.
#include "../../include/epd_encode_test.h"

#include "common.h"

namespace {

// Every wave keeps NACC independent 32 x 32 accumulators and NFRAG operand fragment pairs in registers and
// issues v_mfma_f32_32x32x16_bf16 back to back: no LDS, no memory traffic inside the loop.  The fragment
// pairs rotate, so with random operands the operand buses toggle from one instruction to the next as they
// do in a real product; with constant operands (all ones) they do not, and the chip clocks higher.
constexpr int NACC = 8, NFRAG = 8;

__global__ __launch_bounds__(256, 2) void k_mfma_loop(const bf16_t* __restrict__ operands, int iters,
                                                      float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[NFRAG], b[NFRAG];
#pragma unroll
  for (int f = 0; f < NFRAG; ++f) {
    if (operands) {
      // 2 * NFRAG fragments of 64 lanes x 8 values each, the same for every wave
      a[f] = *reinterpret_cast<const bf16x8*>(operands + ((2 * f) * 64 + lane) * 8);
      b[f] = *reinterpret_cast<const bf16x8*>(operands + ((2 * f + 1) * 64 + lane) * 8);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) { a[f][e] = (bf16_t)1.0f; b[f][e] = (bf16_t)1.0f; }
    }
  }
  f32x16 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int f = 0; f < NFRAG; ++f)
#pragma unroll
      for (int i = 0; i < NACC; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(f + i) % NFRAG], b[f], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NACC; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Do matrix and vector instructions of two waves on one SIMD issue side by side?  A workgroup of eight waves per CU:
// waves 0-3 (one per SIMD) issue v_mfma_f32_32x32x16_bf16 on four independent accumulators, waves 4-7 (the second
// wave of each SIMD) pairs of v_exp_f32 + fma on eight independent registers (the softmax step's mix).  which: 1 the
// matrix waves only, 2 the vector waves only, 3 both.
__global__ __launch_bounds__(512, 1) void k_coissue(const bf16_t* __restrict__ operands, int iters_m, int iters_v, int which,
                                                    float* __restrict__ sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float out = 0.f;
  if (wave < 4) {
    if (!(which & 1)) return;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      a[f] = *reinterpret_cast<const bf16x8*>(operands + ((2 * f) * 64 + lane) * 8);
      b[f] = *reinterpret_cast<const bf16x8*>(operands + ((2 * f + 1) * 64 + lane) * 8);
    }
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters_m; ++it) {
#pragma unroll
      for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(f + i) & 3], b[f], acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) out += acc[i][e];
  } else {
    if (!(which & 2)) return;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = -0.001f * (lane + i);
    for (int it = 0; it < iters_v; ++it) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(__builtin_amdgcn_exp2f(v[i]), -0.5f, -0.25f);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) out += v[i];
  }
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = out;
}

// dst[i] = src[i], 16 bytes per thread and step, grid-stride
__global__ __launch_bounds__(256) void k_stream_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, long n16) {
  const long stride = (long)gridDim.x * blockDim.x;
  for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

template <typename F>
float time_launches(hipStream_t st, int reps, const F& launch) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.f;
  launch();   // warm-up
  (void)hipEventRecord(e0, st);
  for (int i = 0; i < reps; ++i) launch();
  (void)hipEventRecord(e1, st);
  float ms = -1.f;
  if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) ms = -1.f;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return ms < 0.f ? ms : ms / reps;
}

}  // namespace

extern "C" {

epd_status epd_op_mfma_peak(const void* operands, int32_t iters, int32_t reps, float* sink, float* tflops,
                            void* hip_stream) {
  if (!sink || !tflops || iters < 1 || reps < 1) return EPD_ERR_INVALID_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return EPD_ERR_HIP;
  hipStream_t st = (hipStream_t)hip_stream;
  const int grid = cus * 2;   // two workgroups of four waves per CU: two waves per SIMD
  const float ms = time_launches(st, reps, [&] {
    k_mfma_loop<<<dim3(grid), dim3(256), 0, st>>>((const bf16_t*)operands, iters, sink);
  });
  if (ms <= 0.f || hipGetLastError() != hipSuccess) return EPD_ERR_HIP;
  const double flops = (double)grid * 4 * iters * NFRAG * NACC * 2.0 * 32 * 32 * 16;
  *tflops = (float)(flops / (ms * 1e-3) / 1e12);
  return EPD_OK;
}

epd_status epd_op_coissue(const void* operands, int32_t iters_mfma, int32_t iters_valu, int32_t which, int32_t reps,
                          float* sink, float* ms_per_launch, void* hip_stream) {
  if (!operands || !sink || !ms_per_launch || iters_mfma < 0 || iters_valu < 0 || which < 1 || which > 3 || reps < 1 ||
      iters_mfma > (1 << 20) || iters_valu > (1 << 20))
    return EPD_ERR_INVALID_ARG;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return EPD_ERR_HIP;
  hipStream_t st = (hipStream_t)hip_stream;
  const float ms = time_launches(st, reps, [&] {
    k_coissue<<<dim3(cus), dim3(512), 0, st>>>((const bf16_t*)operands, iters_mfma, iters_valu, which, sink);
  });
  if (ms <= 0.f || hipGetLastError() != hipSuccess) return EPD_ERR_HIP;
  *ms_per_launch = ms;
  return EPD_OK;
}

epd_status epd_op_copy_peak(const void* src, void* dst, int64_t bytes, int32_t reps, float* gbps, void* hip_stream) {
  if (!src || !dst || !gbps || bytes < 16 || bytes % 16 || reps < 1 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
    return EPD_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)hip_stream;
  const long n16 = bytes / 16;
  const long want = (n16 + 255) / 256;
  const unsigned grid = (unsigned)(want < 256L * 64 ? want : 256L * 64);
  const float ms = time_launches(st, reps, [&] {
    k_stream_copy<<<dim3(grid), dim3(256), 0, st>>>((const u32x4*)src, (u32x4*)dst, n16);
  });
  if (ms <= 0.f || hipGetLastError() != hipSuccess) return EPD_ERR_HIP;
  *gbps = (float)(2.0 * (double)bytes / (ms * 1e-3) / 1e9);   // read + write
  return EPD_OK;
}

}  // extern "C"
