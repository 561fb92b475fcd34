// MXFP8 operands for the large products of an encoder layer on gfx950.
//
// Format (OCP Microscaling Formats specification v1.0, MXFP8 with E4M3 elements): along the contraction
// dimension K, 32 consecutive elements form a block that shares one power-of-two scale (one byte, value
// 2^(byte - 127)); an element is an OCP FP8 E4M3 number.  Conversion of a block: shared exponent =
// floor(log2(max |v|)) - 8, element = nearest E4M3 value of v / scale (ties to even), saturated to +-448.
//
// Layout in HBM: codes [rows][K] bytes, K contiguous; scales [K / 128][rows] 32-bit words, word (s, r) holding
// the four scale bytes of row r's blocks 4 s .. 4 s + 3 (byte b = block 4 s + b): one K slab of 128 elements
// of a 256-row tile reads 256 consecutive words.
//
// Product: C[M,N] = A[M,K] W[N,K]^T with v_mfma_scale_f32_32x32x64_f8f6f4, which takes the block scales as
// operands and applies them inside the instruction: lane l supplies row l % 32 of its 32 x 64 operand; its
// registers 0-3 hold k = 16 (l / 32) .. + 15 and its registers 4-7 hold k = 32 + 16 (l / 32) .. + 15, so a block
// (k 0..31 or 32..63) is shared by lanes l and l + 32, and the scale register of lanes 0-31 carries the scale
// byte of the row's first block, that of lanes 32-63 the second's; result register i of lane l is
// D[8 (i / 4) + 4 (l / 32) + i % 4][l % 32] (the layout of the 32x32 bf16 instruction).  All of this is what
// the operand-layout test holds on the device.  Block tile 256 x 256 x 128, 8 waves of 128 x 64, both operand
// slabs and their scale words go from global memory straight into LDS one slab ahead (LDS-DMA); LDS rows of
// 128 bytes with the 16-byte chunks XOR-swizzled by (row >> 1) & 7, as in the bf16 kernel.
#include <cstring>
#include <type_traits>

#include "kernels.h"

namespace epd {

namespace {

typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef unsigned char u8;

constexpr int BM = 256, BN = 256;
constexpr int BKB = 128;               // K elements (= bytes) per slab
constexpr int WM = 128, WN = 64;       // wave tile
constexpr int TM = WM / 32, TN = WN / 32;
constexpr int NT = 512;
constexpr size_t SMEM_OPERANDS = (size_t)2 * (BM + BN) * BKB;           // 128 KiB: two slab buffers per operand
constexpr size_t SMEM_SCALES = (size_t)2 * (BM + BN) * sizeof(unsigned);  // per buffer: 256 words of A rows, 256 of W rows
constexpr size_t SMEM_TOTAL = SMEM_OPERANDS + SMEM_SCALES + 2 * BN * sizeof(float);

#define SWZ(row) (((row) >> 1) & 7)

// ---- conversion: mx_scale_byte / mx_inv_scale / mx_pack4 live in common.h (the attention kernel converts its output too) ----
template <typename C>
__device__ __forceinline__ float dpp_f(float x, C) {
  return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), C::value, 0xf, 0xf, true));
}

__device__ __forceinline__ float max4abs(float a, float b, float c, float d) {
  return fmaxf(fmaxf(fabsf(a), fabsf(b)), fmaxf(fabsf(c), fabsf(d)));
}

// ---- rows -> MXFP8 (optionally behind a LayerNorm / RMSNorm) ----------------------------------------------
// One wave per row; lane l owns the 4-element chunks l + 64 i, so a block of 32 elements is 8 neighbouring
// lanes and a slab of 128 elements the 32 lanes of a half-wave.  The row stays in registers (NV chunks per
// lane; NV = 0: read again for every pass).
template <bool IN_BF16, int NV>
__global__ __launch_bounds__(256) void k_mx_rows(const MxRowParams p) {
  const long R = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (R >= p.rows) return;
  const int lane = threadIdx.x & 63;
  const int nchunk = p.dim >> 2;
  auto load = [&](int c) -> float4 {
    if (IN_BF16) {
      const bf16x4 t = *(reinterpret_cast<const bf16x4*>(reinterpret_cast<const bf16_t*>(p.in) + R * p.ld_in) + c);
      return make_float4((float)t[0], (float)t[1], (float)t[2], (float)t[3]);
    }
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(p.in) + R * p.ld_in) + c);
    return make_float4(t[0], t[1], t[2], t[3]);
  };
  constexpr int NVR = NV > 0 ? NV : 1;
  float4 v[NVR];
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = lane + 64 * i < nchunk ? load(lane + 64 * i) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float mean = 0.f, rstd = 1.f;
  if (p.kind != 2) {
    float s = 0.f;
    if (p.kind == 0) {
      if (NV > 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) s += v[i].x + v[i].y + v[i].z + v[i].w;
      } else {
        for (int c = lane; c < nchunk; c += 64) { const float4 a = load(c); s += a.x + a.y + a.z + a.w; }
      }
      mean = wave_sum(s) / p.dim;
    }
    float qs = 0.f;
    auto sq = [&](float4 t) {
      const float a = t.x - mean, b = t.y - mean, cc = t.z - mean, d = t.w - mean;
      qs += a * a + b * b + cc * cc + d * d;
    };
    if (NV > 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i)
        if (lane + 64 * i < nchunk) sq(v[i]);
    } else {
      for (int c = lane; c < nchunk; c += 64) sq(load(c));
    }
    rstd = 1.0f / sqrtf(wave_sum(qs) / p.dim + p.eps);
  }
  unsigned* codes = reinterpret_cast<unsigned*>(p.codes + R * p.ld_codes);
  // every lane of the wave takes part (the exchanges below are wave-wide); lanes past the row carry zeros
  auto emit = [&](int c, float4 a, bool in_row) {
    float r[4] = {a.x, a.y, a.z, a.w};
    if (p.kind != 2 && in_row) {
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
    // largest magnitude of the block's eight lanes: three exchanges inside a row of 16 lanes (no LDS traffic)
    float amax = max4abs(r[0], r[1], r[2], r[3]);
    amax = fmaxf(amax, dpp_f(amax, std::integral_constant<int, 0xB1>{}));    // quad_perm [1, 0, 3, 2]
    amax = fmaxf(amax, dpp_f(amax, std::integral_constant<int, 0x4E>{}));    // quad_perm [2, 3, 0, 1]
    amax = fmaxf(amax, dpp_f(amax, std::integral_constant<int, 0x141>{}));   // row_half_mirror: the other quad of the eight
    const unsigned byte = mx_scale_byte(amax);
    const float inv = mx_inv_scale(byte);
    const unsigned word = mx_pack4(r[0] * inv, r[1] * inv, r[2] * inv, r[3] * inv);
    if (in_row) {
      codes[c] = word;
      // block c / 8 of the row = byte (c / 8) % 4 of scale word (c / 32, R): the block's first lane stores it
      if ((lane & 7) == 0) reinterpret_cast<unsigned char*>(p.scales + (long)(c >> 5) * p.ld_scales + R)[(c >> 3) & 3] = (unsigned char)byte;
    }
  };
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (64 * i < nchunk) emit(lane + 64 * i, v[i], lane + 64 * i < nchunk);
  } else {
    for (int c0 = 0; c0 < nchunk; c0 += 64) {
      const bool in_row = c0 + lane < nchunk;
      emit(c0 + lane, in_row ? load(c0 + lane) : make_float4(0.f, 0.f, 0.f, 0.f), in_row);
    }
  }
}

// ---- product ------------------------------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(NT, 1) void k_gemm_mxfp8(const MxGemmParams p, const int gm_, const int gw) {
  constexpr bool tok_major = EPI == EPI_VT;
  constexpr bool MX_OUT = EPI == EPI_BIAS_GELU_ERF || EPI == EPI_BIAS_GELU_TANH;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u8* sB = smem;                            // [2][BN][128]
  u8* sA = smem + 2 * BN * BKB;             // [2][BM][128]
  unsigned* sS = reinterpret_cast<unsigned*>(smem + SMEM_OPERANDS);   // [2][A rows 0..255 | W rows 0..255]
  float* sBias = reinterpret_cast<float*>(smem + SMEM_OPERANDS + SMEM_SCALES);   // [BN]
  float* sCs = sBias + BN;                                                        // [BN] per-column factor

  // Workgroups are dealt round-robin to the 8 XCDs; XCD x takes a contiguous run of the tile sequence, which
  // walks a band of gw tile columns top to bottom before the next band (weight panel of the band L2-resident).
  const int gn = p.Npad / BN;
  int id = blockIdx.x;
  {
    const int nb = gridDim.x;
    const int x = id & 7, slot = id >> 3;
    const int q = nb >> 3, r = nb & 7;
    id = x * q + (x < r ? x : r) + slot;
  }
  const int band_tiles = gm_ * gw;
  const int full_bands = gn / gw;
  int band = id / band_tiles, in_band = id % band_tiles, bw = gw;
  if (band >= full_bands) { band = full_bands; in_band = id - full_bands * band_tiles; bw = gn - full_bands * gw; }
  const int m0 = (in_band / bw) * BM;
  const int n0 = (band * gw + in_band % bw) * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave >> 2, wn = wave & 3;
  const int l32 = lane & 31, lh = lane >> 5;
  const int KT = p.K / BKB;

  if (tid < BN) {
    sBias[tid] = p.bias[n0 + tid];
    sCs[tid] = p.cscale ? p.cscale[n0 + tid] : 1.0f;
  }

  // LDS-DMA: lane l of a wave lands on 16 bytes at (wave-uniform LDS base) + 16 l, i.e. a wave fills 8 slab rows
  // linearly; the swizzle is applied on the global side: the lane that lands on physical chunk c of its row
  // fetches logical chunk c ^ SWZ(row).
  const int ld_row = tid >> 3, ld_c = tid & 7;
  const unsigned a_voff = (unsigned)ld_row * (unsigned)p.lda + (unsigned)((ld_c ^ SWZ(ld_row)) * 16);
  const unsigned b_voff = (unsigned)ld_row * (unsigned)p.K + (unsigned)((ld_c ^ SWZ(ld_row)) * 16);
  const unsigned s_voff = (unsigned)lane * 4u;
  auto issue = [&](int buf, int kt) {
#pragma unroll
    for (int i = 0; i < BN * 8 / NT; ++i) {
      const u8* g = p.W + (long)(n0 + 64 * i) * p.K + (long)kt * BKB;   // uniform
      const unsigned lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(sB + buf * BN * BKB + (wave_u * 64 + NT * i) * 16);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(b_voff), "s"(g), "s"(lds) : "memory", "m0");
    }
#pragma unroll
    for (int i = 0; i < BM * 8 / NT; ++i) {
      const u8* g = p.A + (long)(m0 + 64 * i) * p.lda + (long)kt * BKB;
      const unsigned lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(sA + buf * BM * BKB + (wave_u * 64 + NT * i) * 16);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(a_voff), "s"(g), "s"(lds) : "memory", "m0");
    }
    {
      // scale words of the slab: waves 0-3 fetch the tile's 256 A rows, waves 4-7 its 256 W rows, 64 words each
      const unsigned* g = wave_u < 4 ? p.SA + (long)kt * p.sa_ld + m0 + 64 * wave_u
                                     : p.SW + (long)kt * p.Npad + n0 + 64 * (wave_u - 4);
      const unsigned lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(sS + buf * (BM + BN) + 64 * wave_u);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" :: "v"(s_voff), "s"(g), "s"(lds) : "memory", "m0");
    }
  };
  auto wait_all_vm = [&]() { __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xf << 8)); };   // vmcnt(0), other counters untouched

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int frag_sw = SWZ(l32);
  auto compute = [&](int buf) {
    const u8* a_s = sA + buf * BM * BKB + (wm * WM + l32) * BKB;
    const u8* b_s = sB + buf * BN * BKB + (wn * WN + l32) * BKB;
    const unsigned* s_a = sS + buf * (BM + BN) + wm * WM + l32;
    const unsigned* s_b = sS + buf * (BM + BN) + BM + wn * WN + l32;
    // a lane carries the scale of block 2 kk + lh of the slab into k-step kk: that byte is brought to byte 2 kk of
    // the register once (shift by 8 lh), and the instruction's byte select (0 or 2) does the rest
    int sa[TM], sb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) sa[i] = (int)(s_a[i * 32] >> (8 * lh));
#pragma unroll
    for (int j = 0; j < TN; ++j) sb[j] = (int)(s_b[j * 32] >> (8 * lh));
#pragma unroll
    for (int kk = 0; kk < BKB / 64; ++kk) {
      // 16-byte chunks lh and 2 + lh of the k-step's four: k = 16 lh .. + 15 and 32 + 16 lh .. + 15
      const int c0 = 4 * kk + lh;
      const int o0 = ((c0 ^ frag_sw) * 16), o1 = (((c0 + 2) ^ frag_sw) * 16);
      i32x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const u32x4 lo = *reinterpret_cast<const u32x4*>(a_s + i * 32 * BKB + o0);
        const u32x4 hi = *reinterpret_cast<const u32x4*>(a_s + i * 32 * BKB + o1);
        fa[i] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const u32x4 lo = *reinterpret_cast<const u32x4*>(b_s + j * 32 * BKB + o0);
        const u32x4 hi = *reinterpret_cast<const u32x4*>(b_s + j * 32 * BKB + o1);
        fb[j] = i32x8{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          // the weight fragment is the LEFT operand (a lane then owns one token and four consecutive features
          // per register group), except for the transposed value store
          if (kk == 0)
            acc[i][j] = tok_major ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], acc[i][j], 0, 0, 0, sa[i], 0, sb[j])
                                  : __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], acc[i][j], 0, 0, 0, sb[j], 0, sa[i]);
          else
            acc[i][j] = tok_major ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], acc[i][j], 0, 0, 2, sa[i], 2, sb[j])
                                  : __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], acc[i][j], 0, 0, 2, sb[j], 2, sa[i]);
        }
    }
  };

  issue(0, 0);
  wait_all_vm();
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) issue(buf ^ 1, kt + 1);   // the other buffer is free since the barrier that ended slab kt - 1
    compute(buf);
    wait_all_vm();        // this wave's share of slab kt + 1 has landed
    __syncthreads();      // ... everyone's has, and everyone is done reading slab kt
  }

  // ------------------------------------------------------------------ epilogue ----
  // through LDS (the operand buffers are idle), so that global memory sees 16-byte chunks of whole rows
  u8* stage = smem;
  if constexpr (EPI == EPI_BIAS_RESIDUAL) {
    // R[row][col] += acc * cscale + bias on the fp32 stream, four passes of 64 token rows: [64][BN] floats.  The
    // stream rows of a pass wait in registers, fetched two passes ahead (those of the first two passes in one batch
    // in front of the first staging), through a buffer descriptor: one lane offset for all of a thread's chunks, the
    // row part of the address in scalar registers, so the 16 loads in flight cost 64 data registers and no more.
    // (The descriptor's range check covers the lane offset only: R holds round_up(M, 256) rows, rows past M are
    // read like any other and never written.)
    constexpr int XROWS = 64, ROWB = BN * 4, XNCH = ROWB / 16, PER_T = XROWS * XNCH / NT, XSTEP = NT / XNCH;
    int et = tid;
    asm volatile("" : "+v"(et));   // opaque copy: what the epilogue derives from it is not hoisted above the main loop
    const int x_r0 = et / XNCH, x_c = et % XNCH;
    const int x_col = n0 + x_c * 4;
    const bool col_ok = x_col < p.N;
    __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(p.R, 0, (int)0x7fffffff, 0x00020000);
    const unsigned x_voff = ((unsigned)x_r0 * (unsigned)p.ldr + (unsigned)x_col) * 4u;
    f32x4 xr[2][PER_T];
    auto xload = [&](auto set, int pass) {
      constexpr int S = decltype(set)::value;
#pragma unroll
      for (int i = 0; i < PER_T; ++i)
        xr[S][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
            rsrc_x, x_voff, (unsigned)(m0 + pass * XROWS + XSTEP * i) * (unsigned)p.ldr * 4u, 2));
    };
    auto one_pass = [&](auto set, int pass) {
      constexpr int S = decltype(set)::value;
      if (pass > 0) __syncthreads();
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int base = wm * WM + i * 32;
        if (base / XROWS != pass) continue;   // wave-uniform
        const int r = base % XROWS + l32;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int gi = 0; gi < 4; ++gi) {
            const int cl = wn * WN + j * 32 + gi * 8 + lh * 4;
            const f32x4 b4 = *reinterpret_cast<const f32x4*>(sBias + cl), c4 = *reinterpret_cast<const f32x4*>(sCs + cl);
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaf(acc[i][j][gi * 4 + e], c4[e], b4[e]);
            *reinterpret_cast<f32x4*>(stage + r * ROWB + (((cl >> 2) ^ (r & 15)) << 4)) = v;
          }
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < PER_T; ++i) {
        const int r = x_r0 + XSTEP * i;
        const int row = m0 + pass * XROWS + r;
        if (row < p.M && col_ok) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(stage + r * ROWB + ((x_c ^ (r & 15)) << 4));
          __builtin_nontemporal_store(xr[S][i] + v, reinterpret_cast<f32x4*>(p.R + (long)row * p.ldr + x_col));
        }
      }
      if (pass + 2 < BM / XROWS) xload(set, pass + 2);
    };
    using X0 = std::integral_constant<int, 0>;
    using X1 = std::integral_constant<int, 1>;
    xload(X0{}, 0);
    xload(X1{}, 1);
    one_pass(X0{}, 0);
    one_pass(X1{}, 1);
    one_pass(X0{}, 2);
    one_pass(X1{}, 3);
  } else if constexpr (MX_OUT) {
    // act(acc * cscale + bias) converted to MXFP8 along the output features (the contraction dimension of the
    // next product).  A lane and its partner lane ^ 32 together hold the 32 features of one block of one token:
    // 16 each (register group gi -> features 8 gi + 4 lh .. + 3).  Codes are staged as [256 rows][256 bytes]
    // (16-byte chunk c of row r at chunk c ^ (r & 15)), scale bytes as [256 rows][8].
    u8* sScale = smem + BM * BN;   // behind the code tile
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int r = wm * WM + i * 32 + l32;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float v[16];
        float amax = 0.f;
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) {
          const int cl = wn * WN + j * 32 + gi * 8 + lh * 4;
          const f32x4 b4 = *reinterpret_cast<const f32x4*>(sBias + cl), c4 = *reinterpret_cast<const f32x4*>(sCs + cl);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[gi * 4 + e] = apply_act_fast<EPI>(__builtin_fmaf(acc[i][j][gi * 4 + e], c4[e], b4[e]));
            amax = fmaxf(amax, fabsf(v[gi * 4 + e]));
          }
        }
        amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
        const unsigned byte = mx_scale_byte(amax);
        const float inv = mx_inv_scale(byte);
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) {
          const int cb = wn * WN + j * 32 + gi * 8 + lh * 4;   // byte column inside the tile
          *reinterpret_cast<unsigned*>(stage + r * BN + (((cb >> 4) ^ (r & 15)) << 4) + (cb & 15)) =
              mx_pack4(v[gi * 4] * inv, v[gi * 4 + 1] * inv, v[gi * 4 + 2] * inv, v[gi * 4 + 3] * inv);
        }
        if (lh == 0) sScale[r * 8 + wn * 2 + j] = (u8)byte;
      }
    }
    __syncthreads();
    constexpr int NCH = BN / 16, PER_T = BM * NCH / NT;
#pragma unroll
    for (int i = 0; i < PER_T; ++i) {
      const int q = tid + NT * i;
      const int r = q / NCH, c = q % NCH;
      const int row = m0 + r, col = n0 + c * 16;
      if (row < p.M && col < p.ncq)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(stage + r * BN + ((c ^ (r & 15)) << 4)),
                                    reinterpret_cast<u32x4*>(p.Cq + (long)row * p.ldcq + col));
    }
    {
      const int r = tid & (BM - 1), half = tid >> 8;    // 256 rows x 2 slabs of 128 features
      const int slab = n0 / BKB + half;
      if (m0 + r < p.M && slab * BKB < p.ncq)
        p.SC[(long)slab * p.sc_ld + m0 + r] = *reinterpret_cast<const unsigned*>(sScale + r * 8 + half * 4);
    }
  } else {
    // bf16 staging of the whole tile: rows = the MFMA lane dimension (tokens; features for the transposed store)
    constexpr int SROWS = tok_major ? BN : BM, SCOLS = tok_major ? BM : BN;
    constexpr int ROWB = SCOLS * 2, NCH = ROWB / 16, PER_T = SROWS * NCH / NT;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = tok_major ? (wn * WN + j * 32 + l32) : (wm * WM + i * 32 + l32);
        const float bl = tok_major ? sBias[r] : 0.f, cs = tok_major ? sCs[r] : 1.f;
#pragma unroll
        for (int gi = 0; gi < 4; ++gi) {
          const int cl = (tok_major ? (wm * WM + i * 32) : (wn * WN + j * 32)) + gi * 8 + lh * 4;
          bf16x4 o;
          if (tok_major) {
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16_t)__builtin_fmaf(acc[i][j][gi * 4 + e], cs, bl);
          } else {
            const f32x4 b4 = *reinterpret_cast<const f32x4*>(sBias + cl), c4 = *reinterpret_cast<const f32x4*>(sCs + cl);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16_t)__builtin_fmaf(acc[i][j][gi * 4 + e], c4[e], b4[e]);
          }
          *reinterpret_cast<bf16x4*>(stage + r * ROWB + (((cl >> 3) ^ (r & 15)) << 4) + ((cl & 4) << 1)) = o;
        }
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PER_T; ++i) {
      const int q = tid + NT * i;
      const int r = q / NCH, c = q % NCH;
      const u32x4 v = *reinterpret_cast<const u32x4*>(stage + r * ROWB + ((c ^ (r & 15)) << 4));
      if (tok_major) {
        const int f = n0 + r, tok = m0 + c * 8;
        if (f < p.N && tok < p.M) {
          const int h = f / p.hd_pad, d = f % p.hd_pad;
          const int t = tok / p.n_tok, n = tok % p.n_tok;
          __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p.VT + (((long)t * p.heads + h) * p.hd_pad + d) * p.n_tok + n));
        }
      } else {
        const int row = m0 + r, col = n0 + c * 8;
        if (row < p.M && col < p.N) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p.C + (long)row * p.ldc + col));
      }
    }
  }
}

// One instruction on caller-supplied registers: lane l gets a[l][0..7], b[l][0..7] and the scale registers
// sa[l], sb[l] (byte 0 is used) and leaves its 16 result registers in d[l][0..15].
__global__ __launch_bounds__(64) void k_mx_mfma_probe(const int* a, const int* b, const int* sa, const int* sb, float* d) {
  const int l = threadIdx.x;
  i32x8 fa, fb;
#pragma unroll
  for (int e = 0; e < 8; ++e) { fa[e] = a[l * 8 + e]; fb[e] = b[l * 8 + e]; }
  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa, fb, acc, 0, 0, 0, sa[l], 0, sb[l]);
#pragma unroll
  for (int e = 0; e < 16; ++e) d[l * 16 + e] = acc[e];
}

template <int EPI>
hipError_t launch(const MxGemmParams& p, hipStream_t st) {
  const int gm = (p.M + BM - 1) / BM, gn = p.Npad / BN;
  const int gw = gn <= 4 ? gn : 4;
  k_gemm_mxfp8<EPI><<<dim3((unsigned)(gm * gn)), dim3(NT), SMEM_TOTAL, st>>>(p, gm, gw);
  return hipGetLastError();
}

template <int EPI>
hipError_t set_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_mxfp8<EPI>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)SMEM_TOTAL);
}

}  // namespace

hipError_t mx_gemm_init() {
  static const hipError_t once = [] {
    hipError_t e;
    if ((e = set_attr<EPI_BIAS>()) != hipSuccess) return e;
    if ((e = set_attr<EPI_VT>()) != hipSuccess) return e;
    if ((e = set_attr<EPI_BIAS_GELU_ERF>()) != hipSuccess) return e;
    if ((e = set_attr<EPI_BIAS_GELU_TANH>()) != hipSuccess) return e;
    return set_attr<EPI_BIAS_RESIDUAL>();
  }();
  return once;
}

hipError_t mx_gemm(const MxGemmParams& p, hipStream_t st) {
  // what the kernel assumes, checked where the launch is made
  const long a_extent = ((long)(p.M + BM - 1) / BM * BM) * p.lda;
  if (p.M <= 0 || p.K <= 0 || p.K % BKB || p.Npad <= 0 || p.Npad % BN || p.N > p.Npad || p.lda < p.K || p.lda % 16 ||
      p.sa_ld < (long)(p.M + BM - 1) / BM * BM || a_extent >= (1L << 32) || (long)p.Npad * p.K >= (1L << 32) ||
      !p.A || !p.SA || !p.W || !p.SW || !p.bias)
    return hipErrorInvalidValue;
  switch (p.epi) {
    case EPI_BIAS: return p.C && p.N % 8 == 0 ? launch<EPI_BIAS>(p, st) : hipErrorInvalidValue;
    case EPI_VT: return p.VT && p.n_tok % 8 == 0 && p.hd_pad > 0 ? launch<EPI_VT>(p, st) : hipErrorInvalidValue;
    case EPI_BIAS_GELU_ERF:
    case EPI_BIAS_GELU_TANH:
      if (!p.Cq || !p.SC || p.ncq <= 0 || p.ncq % BKB || p.ldcq < p.ncq || p.ldcq % 16 || p.sc_ld < (long)(p.M + BM - 1) / BM * BM) return hipErrorInvalidValue;
      return p.epi == EPI_BIAS_GELU_ERF ? launch<EPI_BIAS_GELU_ERF>(p, st) : launch<EPI_BIAS_GELU_TANH>(p, st);
    case EPI_BIAS_RESIDUAL:   // the stream rows are addressed through 32-bit offsets
      if (!p.R || p.N % 4 || p.ldr < p.N || ((long)(p.M + BM - 1) / BM * BM) * p.ldr * 4 >= (1L << 32)) return hipErrorInvalidValue;
      return launch<EPI_BIAS_RESIDUAL>(p, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t mx_rows(const MxRowParams& p, hipStream_t st) {
  if (p.rows == 0) return hipSuccess;
  if (p.dim <= 0 || p.dim % 128 || p.ld_codes < p.dim || p.ld_codes % 4 || p.ld_scales < p.rows || !p.in || !p.codes ||
      !p.scales || (p.kind != 2 && !p.gamma) || (p.kind == 0 && !p.beta) || p.kind < 0 || p.kind > 2)
    return hipErrorInvalidValue;
  const dim3 grid((unsigned)((p.rows + 3) / 4)), block(256);
  const int per_lane = (p.dim / 4 + 63) / 64;
#define MX_ROWS(BF, NV) k_mx_rows<BF, NV><<<grid, block, 0, st>>>(p)
  if (p.in_bf16) {
    if (per_lane <= 4) MX_ROWS(true, 4); else if (per_lane <= 8) MX_ROWS(true, 8); else if (per_lane <= 16) MX_ROWS(true, 16); else MX_ROWS(true, 0);
  } else {
    if (per_lane <= 4) MX_ROWS(false, 4); else if (per_lane <= 8) MX_ROWS(false, 8); else if (per_lane <= 16) MX_ROWS(false, 16); else MX_ROWS(false, 0);
  }
#undef MX_ROWS
  return hipGetLastError();
}

void mx_mfma_probe(const int* a, const int* b, const int* sa, const int* sb, float* d, hipStream_t st) {
  k_mx_mfma_probe<<<dim3(1), dim3(64), 0, st>>>(a, b, sa, sb, d);
}

}  // namespace epd
