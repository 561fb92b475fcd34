// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T, fp32 accumulate,
// fused epilogues (bias, GELU, residual add into the fp32 stream, position
// embedding, transposed store of the attention values).
//
// Block tile 256 x BN x 64 (BN = 256 or 128), 8 waves of 64 lanes.  Both
// operands are K-contiguous, staged through LDS as [row][64] bf16 with the
// 16-byte chunks of a row XOR-swizzled by (row & 7) so that the 32 rows a
// wave reads for one MFMA operand fall into different banks.  Global loads of
// k-slab kt+1 are issued before the MFMAs of slab kt and written to the other
// LDS buffer after them: one barrier per slab.
//
// v_mfma_f32_32x32x16_bf16 operand layout (checked on the device by
// mfma_probe): lane l supplies row (l % 32) of the 32 x 16 left operand /
// column (l % 32) of the 16 x 32 right operand, k = 8*(l / 32) + 0..7;
// result register i of lane l is D[8*(i/4) + 4*(l/32) + i%4][l % 32].
// The weight fragment is fed as the LEFT operand, so a lane owns one token
// and four consecutive output features per register group: 8-byte bf16 /
// 16-byte fp32 accesses in the epilogue.  For the attention values (EPI_VT)
// the roles are swapped, so a lane owns four consecutive tokens of one
// feature, which is what the transposed value layout wants.
#include "kernels.h"

namespace epd {

namespace {

constexpr int BM = 256;
constexpr int BK = 64;
constexpr int NTHREADS = 512;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

template <int BN, int EPI>
__global__ __launch_bounds__(NTHREADS, 1) void k_gemm_bf16(const GemmParams p) {
  constexpr int WAVES_N = BN / 64;      // 4 | 2
  constexpr int WAVES_M = 8 / WAVES_N;  // 2 | 4
  constexpr int WM = BM / WAVES_M;      // 128 | 64
  constexpr int TM = WM / 32;           // 4 | 2
  constexpr int TN = 2;
  constexpr int A_LD = BM * 8 / NTHREADS;  // 16-byte chunks per thread per slab
  constexpr int B_LD = BN * 8 / NTHREADS;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem);  // [2][BM][64]
  bf16_t* sB = sA + 2 * BM * BK;                 // [2][BN][64]

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a
  // contiguous run of output tiles (N fastest) so its L2 sees whole panels.
  const int gn = p.Npad / BN;
  const int nb = gridDim.x;
  int id = blockIdx.x;
  {
    const int x = id & 7, slot = id >> 3;
    const int q = nb >> 3, r = nb & 7;
    id = x * q + (x < r ? x : r) + slot;
  }
  const int m0 = (id / gn) * BM;
  const int n0 = (id % gn) * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;

  const int ld_row = tid >> 3, ld_c = tid & 7;
  const int st_off = ld_row * BK + ((ld_c ^ (ld_row & 7)) * 8);
  const bf16_t* gA = p.A + (long)(m0 + ld_row) * p.lda + ld_c * 8;
  const bf16_t* gB = p.W + (long)(n0 + ld_row) * p.K + ld_c * 8;

  u32x4 ra[A_LD], rb[B_LD];
  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      ra[i] = *reinterpret_cast<const u32x4*>(gA + (long)(64 * i) * p.lda + kt * BK);
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
      rb[i] = *reinterpret_cast<const u32x4*>(gB + (long)(64 * i) * p.K + kt * BK);
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      *reinterpret_cast<u32x4*>(sA + buf * BM * BK + 64 * i * BK + st_off) = ra[i];
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
      *reinterpret_cast<u32x4*>(sB + buf * BN * BK + 64 * i * BK + st_off) = rb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // attention values: token-major MFMA result, stored transposed
  constexpr bool tok_major = (EPI == EPI_VT);

  const int KT = p.K / BK;
  gload(0);
  sstore(0);
  __syncthreads();

  const int frag_sw = l32 & 7;
  for (int kt = 0; kt < KT; ++kt) {
    // always issue the next slab's loads (the last iteration re-reads the
    // final slab into the idle buffer): keeps the staging registers free of
    // control flow
    gload(kt + 1 < KT ? kt + 1 : kt);
    const bf16_t* a_s = sA + (kt & 1) * BM * BK + (wm * WM + l32) * BK;
    const bf16_t* b_s = sB + (kt & 1) * BN * BK + (wn * 64 + l32) * BK;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int coff = (((2 * kk + lh) ^ frag_sw) * 8);
      bf16x8 xf[TM], wf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) xf[i] = *reinterpret_cast<const bf16x8*>(a_s + i * 32 * BK + coff);
#pragma unroll
      for (int j = 0; j < TN; ++j) wf[j] = *reinterpret_cast<const bf16x8*>(b_s + j * 32 * BK + coff);
      if (tok_major) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(xf[i], wf[j], acc[i][j]);
      } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(wf[j], xf[i], acc[i][j]);
      }
    }
    sstore((kt + 1) & 1);
    __syncthreads();
  }

  // ------------------------------------------------------------ epilogue ----
  if (tok_major) {
    // lane = feature, register group = 4 consecutive tokens
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int c = n0 + wn * 64 + j * 32 + l32;
      const int fv = c;
      if (fv >= p.N) continue;
      const float bv = p.bias[c];
      const int h = fv / p.hd_pad, d = fv % p.hd_pad;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) {
          const int r0 = m0 + wm * WM + i * 32 + gi * 8 + lh * 4;
          if (r0 >= p.M) continue;
          const int t = r0 / p.n_tok, n = r0 % p.n_tok;
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(acc[i][j][gi * 4 + e] + bv);
          *reinterpret_cast<bf16x4*>(p.VT + (((long)t * p.heads + h) * p.hd_pad + d) * p.n_tok + n) = o;
        }
      }
    }
    return;
  }

  // lane = token, register group = 4 consecutive features
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int r = m0 + wm * WM + i * 32 + l32;
    if (r >= p.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) {
        const int c0 = n0 + wn * 64 + j * 32 + gi * 8 + lh * 4;
        if (c0 >= p.N) continue;
        const float4 b4 = *reinterpret_cast<const float4*>(p.bias + c0);
        float v[4] = {acc[i][j][gi * 4 + 0] + b4.x, acc[i][j][gi * 4 + 1] + b4.y,
                      acc[i][j][gi * 4 + 2] + b4.z, acc[i][j][gi * 4 + 3] + b4.w};
        if (EPI == EPI_BIAS_RESIDUAL) {
          float4* dst = reinterpret_cast<float4*>(p.R + (long)r * p.ldr + c0);
          float4 x = *dst;
          x.x += v[0]; x.y += v[1]; x.z += v[2]; x.w += v[3];
          *dst = x;
        } else if (EPI == EPI_BIAS_POS) {
          const float4 ps = *reinterpret_cast<const float4*>(p.pos + (long)(r % p.n_pos) * p.N + c0);
          float4 x = {v[0] + ps.x, v[1] + ps.y, v[2] + ps.z, v[3] + ps.w};
          *reinterpret_cast<float4*>(p.R + (long)r * p.ldr + c0) = x;
        } else {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16_t)apply_act<EPI>(v[e]);
          *reinterpret_cast<bf16x4*>(p.C + (long)r * p.ldc + c0) = o;
        }
      }
    }
  }
}

template <int BN>
constexpr size_t smem_bytes() { return (size_t)2 * (BM + BN) * BK * sizeof(bf16_t); }

template <int BN, int EPI>
hipError_t launch(const GemmParams& p, hipStream_t st) {
  const int gm = (p.M + BM - 1) / BM, gn = p.Npad / BN;
  if (gm == 0 || gn == 0) return hipSuccess;
  k_gemm_bf16<BN, EPI><<<dim3(gm * gn), dim3(NTHREADS), smem_bytes<BN>(), st>>>(p);
  return hipGetLastError();
}

template <int BN>
hipError_t dispatch(const GemmParams& p, hipStream_t st) {
  switch (p.epi) {
    case EPI_BIAS: return launch<BN, EPI_BIAS>(p, st);
    case EPI_BIAS_GELU_ERF: return launch<BN, EPI_BIAS_GELU_ERF>(p, st);
    case EPI_BIAS_GELU_TANH: return launch<BN, EPI_BIAS_GELU_TANH>(p, st);
    case EPI_BIAS_RESIDUAL: return launch<BN, EPI_BIAS_RESIDUAL>(p, st);
    case EPI_BIAS_POS: return launch<BN, EPI_BIAS_POS>(p, st);
    case EPI_VT: return launch<BN, EPI_VT>(p, st);
  }
  return hipErrorInvalidValue;
}

template <int BN, int EPI>
hipError_t set_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16<BN, EPI>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<BN>());
}

template <int BN>
hipError_t set_attr_all() {
  hipError_t e;
  if ((e = set_attr<BN, EPI_BIAS>()) != hipSuccess) return e;
  if ((e = set_attr<BN, EPI_BIAS_GELU_ERF>()) != hipSuccess) return e;
  if ((e = set_attr<BN, EPI_BIAS_GELU_TANH>()) != hipSuccess) return e;
  if ((e = set_attr<BN, EPI_BIAS_RESIDUAL>()) != hipSuccess) return e;
  if ((e = set_attr<BN, EPI_BIAS_POS>()) != hipSuccess) return e;
  return set_attr<BN, EPI_VT>();
}

}  // namespace

hipError_t bf16_gemm_init() {
  hipError_t e = set_attr_all<256>();
  if (e != hipSuccess) return e;
  return set_attr_all<128>();
}

hipError_t bf16_gemm(const GemmParams& p, hipStream_t st) {
  if (p.K % BK != 0 || p.Npad % 128 != 0 || p.N % 4 != 0) return hipErrorInvalidValue;
  return (p.Npad % 256 == 0) ? dispatch<256>(p, st) : dispatch<128>(p, st);
}

}  // namespace epd
