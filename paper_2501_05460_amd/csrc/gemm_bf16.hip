// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] * W[N,K]^T, fp32 accumulate,
// fused epilogues (bias, GELU, residual add into the fp32 stream, position
// embedding, transposed store of the attention values).
//
// Block tile 256 x BN x 64 (BN = 256 or 128; 128 x 128 x 64 for small launches), 8 waves of 64 lanes.  Both
// operands are K-contiguous, staged through LDS as [row][64] bf16 with the
// 16-byte chunks of a row XOR-swizzled by the row so that the 32 rows a
// wave reads for one MFMA operand fall into different banks (64 banks, 16
// lanes per 128-bit access phase: rows r and r+1 share a chunk column, so the
// XOR key is (row >> 1) & 7).  One barrier per slab, two LDS buffers.
//
// Main loop of the default shape (PIPE = 1): the activation slab is read two
// slabs ahead into registers through a buffer descriptor (L2 / Infinity-Cache
// latency is longer than one slab of MFMA work) and stored to the other LDS
// buffer a slab later; the weight slab, which sits in L2, goes from global
// memory straight into the other LDS buffer one slab ahead (global_load_lds,
// no staging registers).  The MFMA operand fragments of k-step kk+1 are read
// from LDS into a second register set while the MFMAs of k-step kk issue back
// to back.  PIPE = 0 is the plain form (both operands staged in registers,
// fragment reads left to the compiler), kept for the other tile shapes.
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
#include <cstdlib>
#include <type_traits>

#include "kernels.h"

namespace epd {

namespace {

constexpr int BM = 256;
constexpr int BK = 64;

// XOR swizzle of the 16-byte chunk index by the row
#define SWZ(row) (((row) >> 1) & 7)

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Configurations (BN, 512 threads, 64-wide wave tiles), one workgroup per CU, two LDS buffers:
//   BN = 256  256x256 tile, 128x64 per wave (PIPE = 1: pipelined loop, the default; PIPE = 0:
//             both operands two slabs ahead in two register sets, fragment reads left to the
//             compiler: the reference the pipelined loop is checked against bit for bit);
//   BN = 128  256x128 tile, 64x64 per wave, PIPE = 0: outputs narrower than 256 columns;
//   BN = 128, BM = 128  128x128 tile, 32x64 per wave, PIPE = 0, two workgroups per CU: launches of
//             a few slices, whose time is a sum of single-tile latencies.
// (Tried and dropped, none faster on the six workloads: 4 waves of 128x128 with AGPR
// accumulators, 256x128 tiles with two 4-wave workgroups per CU, 32-deep slabs.)
template <int BN, int NT, int BM_ = BM>
constexpr size_t smem_main_bytes() {
  // operand slabs, or the epilogue staging tile (BM x BN bf16 / 64 x BN fp32), whichever is larger
  constexpr size_t operands = (size_t)2 * (BM_ + BN) * BK * sizeof(bf16_t);
  constexpr size_t staging = (size_t)BM_ * BN * sizeof(bf16_t);
  return operands > staging ? operands : staging;
}

// FOLD (compiled apart so that the plain kernels keep their code and registers).  bf16-output epilogues: 2 = apply a
// folded pre-norm (GemmParams::stats).  Residual epilogue: 1 = also store the updated rows as bf16
// (GemmParams::xb), 2 = and their statistics pairs (GemmParams::stats_out).
template <int BN, int NTHREADS, int WN, int EPI, int PIPE, int BM_ = 256, int FOLD = 0>
__global__ __launch_bounds__(NTHREADS, BM_ == 128 && PIPE == 0 ? 2 : 1) void k_gemm_bf16(const GemmParams p, const int gm_, const int gw) {
  constexpr int BM = BM_;   // token rows of the tile: 256, or 128 for launches of a few slices
  static_assert(BM_ == 256 ? (PIPE <= 1 || PIPE == 3) : (BM_ == 128 && BN == 128 && (PIPE == 0 || PIPE == 2)), "tile shapes compiled");
  constexpr int NWAVES = NTHREADS / 64;
  constexpr int WAVES_N = BN / WN;           // 4 | 2
  constexpr int WAVES_M = NWAVES / WAVES_N;  // 2 | 4 | 2
  constexpr int WM = BM / WAVES_M;           // 128 | 64 | 128
  constexpr int TM = WM / 32;                // 4 | 2 | 4
  constexpr int TN = WN / 32;                // 2 | 4
  constexpr int A_LD = BM * 8 / NTHREADS;    // 16-byte chunks per thread per slab
  constexpr int B_LD = BN * 8 / NTHREADS;
  constexpr int NBUF = 2;  // LDS slab buffers
  // register sets the global loads land in = slabs they run ahead of the MFMAs.  PIPE = 2 (128 x 128
  // tiles of launches with at most one tile per CU): four, because such a launch is bound by the bytes
  // it keeps in flight, not by the matrix cores
  constexpr int NSET = PIPE == 2 ? 4 : 2;
  constexpr int ROWS_PER_LD = NTHREADS / 8;      // rows covered by one 16-byte load per thread

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // weight slabs first: their LDS addresses (<= 64 KiB) also serve as the 16-bit base of the
  // direct global-to-LDS loads
  bf16_t* sB = reinterpret_cast<bf16_t*>(smem);  // [NBUF][BN][64]
  bf16_t* sA = sB + NBUF * BN * BK;              // [NBUF][BM][64]
  float* sBias = reinterpret_cast<float*>(smem + smem_main_bytes<BN, NTHREADS, BM>());  // [BN]
  float* sCol = sBias + BN;   // [BN] column sums of the weights (folded pre-norm)
  float* sMu = sCol + BN;     // [BM] mean of the tile's rows
  float* sRs = sMu + BM;      // [BM] 1 / sqrt(variance + eps)
  constexpr bool BF16_OUT = !(EPI == EPI_BIAS_RESIDUAL || EPI == EPI_BIAS_POS);
  constexpr bool fold = BF16_OUT && FOLD == 2;
  constexpr bool emit = EPI == EPI_BIAS_RESIDUAL && FOLD >= 1;        // bf16 rows
  constexpr bool emit_stats = EPI == EPI_BIAS_RESIDUAL && FOLD == 2;  // and their statistics

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.
  // XCD x takes a contiguous run of the tile sequence, and the sequence walks
  // a band of `gw` tile columns top to bottom before moving to the next
  // band: the band's weight panel (gw * BN rows) stays L2-resident while the
  // activation panels stream through once per band.
  const int gn = p.Npad / BN;
  int id = blockIdx.x;
  {
    const int nb = gridDim.x;
    const int x = id & 7, slot = id >> 3;
    const int q = nb >> 3, r = nb & 7;
    id = x * q + (x < r ? x : r) + slot;
  }
  const int band_tiles = gm_ * gw;
  const int full_bands = gn / gw;                 // the last band may be narrower
  int band = id / band_tiles, in_band = id % band_tiles, bw = gw;
  if (band >= full_bands) { band = full_bands; in_band = id - full_bands * band_tiles; bw = gn - full_bands * gw; }
  const int m0 = (in_band / bw) * BM;
  const int n0 = (band * gw + in_band % bw) * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  (void)NWAVES;
  const int l32 = lane & 31, lh = lane >> 5;

  const int KT_ = p.K / BK;  // even (K % 128 == 0)
  // the tile's bias values wait in LDS for the epilogue (a global load there
  // would sit exposed between the last MFMA and the first store)
  if (tid < BN) sBias[tid] = p.bias[n0 + tid];
  if (fold) {   // read by the epilogue, many barriers from here
    if (tid < BN) sCol[tid] = p.colsum[n0 + tid];
    if (tid < BM) {
      const float* pairs = p.stats + (long)(m0 + tid < p.M ? m0 + tid : p.M - 1) * p.n_part * 2;   // rows past M: any valid row, never stored
      RowPairs rp;
      rp.load(pairs, p.n_part);
      float mu, rs;
      rp.finish(p.n_part, p.stat_group, p.norm_dim, p.norm_rms, p.norm_eps, mu, rs);
      sMu[tid] = mu;
      sRs[tid] = rs;
    }
  }
  const int ld_row = tid >> 3, ld_c = tid & 7;
  const int st_off = ld_row * BK + ((ld_c ^ SWZ(ld_row)) * 8);

  // global addresses = wave-uniform base (scalar registers) + one 32-bit lane offset per operand
  const unsigned a_voff = ((unsigned)ld_row * (unsigned)p.lda + ld_c * 8) * 2;   // bytes
  const unsigned b_voff = ((unsigned)ld_row * (unsigned)p.K + ld_c * 8) * 2;

  // Residual epilogue: the tile's fp32 rows are added in passes of 64 token
  // rows; the rows of pass p wait in register set p % 2, loaded two passes
  // ahead (the first two while the last slabs are multiplied), so the
  // read-modify-write never waits for memory with the MFMA pipe idle.
  constexpr int XROWS = 64;                          // token rows per fp32 epilogue pass
  constexpr int XNCH = BN * 4 / 16;                  // 16-byte chunks per staging row
  constexpr int XPER_T = XROWS * XNCH / NTHREADS;    // chunks per thread and pass
  constexpr int XSTEP = NTHREADS / XNCH;             // rows between a thread's consecutive chunks
  static_assert(NTHREADS % XNCH == 0, "a thread keeps one chunk column");
  // chunk i of a thread: tile row tid / XNCH + XSTEP * i (the same for a whole
  // wave), column chunk tid % XNCH: one lane offset serves every access, the
  // row part of the address is wave-uniform
  const int x_r0 = XNCH % 64 == 0 ? __builtin_amdgcn_readfirstlane(tid / XNCH) : tid / XNCH;  // wave-uniform when a row is >= 64 chunks
  const int x_col = n0 + (tid % XNCH) * 4;
  const bool x_col_ok = x_col < p.N;
  const unsigned x_voff = (unsigned)x_r0 * (unsigned)p.ldr + (unsigned)x_col;
  // PIPE == 1: the weight slab goes from global memory straight into LDS (no
  // staging registers), one slab ahead; only the activation slab is staged in
  // registers, two slabs ahead.
  constexpr bool B_DIRECT = PIPE == 1 || PIPE == 3;
  // PIPE == 3: the activation slab goes straight into LDS as well, one slab ahead (no staging registers at all)
  constexpr bool A_DIRECT = PIPE == 3;
  // the operand register sets can carry residual rows of the first passes when the counts match:
  // both sets = passes 0 and 1 (A and B staged), or both sets = the two halves of pass 0 (A staged only)
  constexpr bool X_IN_LOOP = EPI == EPI_BIAS_RESIDUAL &&
                             (A_DIRECT || (B_DIRECT ? XPER_T == 2 * A_LD : XPER_T == A_LD + B_LD));
  f32x4 xr[2][X_IN_LOOP ? XPER_T : 1];
  auto xload = [&](auto set, int pass) {
    if constexpr (X_IN_LOOP) {
      constexpr int S = decltype(set)::value;
      if (x_col_ok) {
#pragma unroll
        for (int i = 0; i < XPER_T; ++i) {
          const int row0 = m0 + pass * XROWS + XSTEP * i;            // uniform
          if (row0 + x_r0 < p.M) xr[S][i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p.R + (long)row0 * p.ldr + x_voff));
        }
      }
    }
  };


  // Global operands are read through buffer descriptors: descriptor + scalar offset + one lane
  // offset per operand, so no per-load address arithmetic touches vector registers.  The range
  // check of a descriptor covers the lane offset only, not the scalar one: the rows of a ragged
  // last tile past M are read like any other (A and R hold round_up(M, 256) rows) and their
  // results never stored.  The host launcher checks that every extent fits 32 bits.
  __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(p.A), 0, (int)(unsigned)(((long)(p.M - 1) * p.lda + p.K) * 2), 0x00020000);
  __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(p.W), 0, (int)(unsigned)((long)p.Npad * p.K * 2), 0x00020000);
  __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
      p.R, 0, EPI == EPI_BIAS_RESIDUAL ? (int)(unsigned)(((long)(p.M - 1) * p.ldr + p.N) * 4) : 0, 0x00020000);

  // Two register sets: the loads of slab k+2 are in flight while slab k is
  // multiplied and slab k+1 (loaded one iteration earlier) moves to LDS.
  u32x4 ra[NSET][A_LD], rb[NSET][B_DIRECT ? 1 : B_LD];
  auto gload = [&](auto set, int kt) {
    constexpr int S = decltype(set)::value;
    // Residual epilogue: the two loads past the last slab (kt == KT_ into set
    // 0, KT_ + 1 into set 1) fetch fp32 rows of the first epilogue passes into
    // the same registers instead of re-reading operands.  Chunk c of a pass =
    // rows XSTEP * c + x_r0 of the pass, this lane's 16-byte column chunk.
    // Staged A and B: set s holds pass s, chunks 0 .. XPER_T-1; staged A only:
    // set s holds chunks s * A_LD .. of pass 0.
    const bool past = kt >= KT_;
    const int xpass = kt - KT_;
    kt = past ? KT_ - 1 : kt;  // past the end (other epilogues): re-read the last slab, result unused
    if (X_IN_LOOP && past && xpass >= 2) return;   // four register sets: only two of them carry residual rows
    if (X_IN_LOOP && past) {   // one uniform branch per slab, taken for the last two slabs of a tile
      auto so_x = [&](int c) {
        const int pass = B_DIRECT ? 0 : xpass, ci = B_DIRECT ? xpass * A_LD + c : c;
        return (unsigned)(m0 + pass * XROWS + XSTEP * ci) * (unsigned)p.ldr * 4u;
      };
#pragma unroll
      for (int i = 0; i < A_LD; ++i) ra[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, x_voff * 4u, so_x(i), 2);
      if constexpr (!B_DIRECT) {
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
          rb[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_x, x_voff * 4u, so_x(A_LD + i), 2);
      }
    } else {
#pragma unroll
      for (int i = 0; i < A_LD; ++i) {
        const unsigned so = ((unsigned)(m0 + ROWS_PER_LD * i) * (unsigned)p.lda + (unsigned)(kt * BK)) * 2u;
        ra[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, a_voff, so, 0);
      }
      if constexpr (!B_DIRECT) {
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
          const unsigned so = ((unsigned)(n0 + ROWS_PER_LD * i) * (unsigned)p.K + (unsigned)(kt * BK)) * 2u;
          rb[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_b, b_voff, so, 0);
        }
      }
    }
  };
  // Weight slab kt -> LDS buffer buf without passing through registers.  The
  // hardware puts lane l's 16 bytes at (wave-uniform LDS base) + 16 l, so a
  // wave fills 1 KiB = 8 slab rows linearly; the swizzle is applied on the
  // global side instead: the lane that lands on physical chunk ld_c of its row
  // fetches logical chunk ld_c ^ SWZ(row).
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const unsigned bd_voff = ((unsigned)ld_row * (unsigned)p.K + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  auto bload = [&](int buf, int kt) {
    if constexpr (B_DIRECT) {
#pragma unroll
      for (int i = 0; i < B_LD; ++i) {
        const bf16_t* g = p.W + (long)(n0 + ROWS_PER_LD * i) * p.K + kt * BK;   // uniform
        bf16_t* l = sB + buf * BN * BK + (wave_u * 64 + NTHREADS * i) * 8;
        // Written as assembly on purpose: for the builtin form the compiler makes every later
        // LDS read wait for ALL outstanding vector-memory loads (it cannot tell the two LDS
        // buffers apart), which would serialise the pipeline.  Completion is awaited
        // explicitly (wait_vm) in front of the barrier that publishes the buffer.
        const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)l;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(bd_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
      }
    }
  };
  // PIPE == 3: activation slab kt -> LDS buffer buf, same scheme (LDS-DMA reaches the whole LDS through M0 on gfx950)
  const unsigned ad_voff = ((unsigned)ld_row * (unsigned)p.lda + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  auto aload = [&](int buf, int kt) {
    if constexpr (A_DIRECT) {
#pragma unroll
      for (int i = 0; i < A_LD; ++i) {
        const bf16_t* g = p.A + (long)(m0 + ROWS_PER_LD * i) * p.lda + kt * BK;   // uniform
        bf16_t* l = sA + buf * BM * BK + (wave_u * 64 + NTHREADS * i) * 8;
        const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)l;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(ad_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
      }
    }
  };
  // wait until at most n of this wave's vector-memory loads are outstanding (they complete in order)
  auto wait_vm = [&](auto n) {
    constexpr int N = decltype(n)::value;
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
  };
  auto sstore = [&](auto set, int buf) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      *reinterpret_cast<u32x4*>(sA + buf * BM * BK + ROWS_PER_LD * i * BK + st_off) = ra[S][i];
    if constexpr (!B_DIRECT) {
#pragma unroll
      for (int i = 0; i < B_LD; ++i)
        *reinterpret_cast<u32x4*>(sB + buf * BN * BK + ROWS_PER_LD * i * BK + st_off) = rb[S][i];
    }
  };

  // attention values: token-major MFMA result, stored transposed
  constexpr bool tok_major = (EPI == EPI_VT);

  f32x16 acc[TM][TN];
  const int frag_sw = SWZ(l32);
  auto compute = [&](int buf) {
    const bf16_t* a_s = sA + buf * BM * BK + (wm * WM + l32) * BK;
    const bf16_t* b_s = sB + buf * BN * BK + (wn * WN + l32) * BK;
    if constexpr (TM * TN <= 2) {
      // Small tiles run alone on their CU and their time is the chain LDS read -> MFMA of one wave:
      // all fragments of the slab are read first (two k-steps' worth per batch of registers), so the
      // LDS latency is paid once per half slab instead of once per k-step.  The k-steps of an element
      // are still added in order.
#pragma unroll
      for (int k2 = 0; k2 < BK / 16; k2 += 2) {
        bf16x8 xf[2][TM], wf[2][TN];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int coff = (((2 * (k2 + q) + lh) ^ frag_sw) * 8);
#pragma unroll
          for (int i = 0; i < TM; ++i) xf[q][i] = *reinterpret_cast<const bf16x8*>(a_s + i * 32 * BK + coff);
#pragma unroll
          for (int j = 0; j < TN; ++j) wf[q][j] = *reinterpret_cast<const bf16x8*>(b_s + j * 32 * BK + coff);
        }
        __builtin_amdgcn_sched_barrier(0);   // the scheduler would otherwise sink each read to its MFMA
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = tok_major ? mfma32(xf[q][i], wf[q][j], acc[i][j]) : mfma32(wf[q][j], xf[q][i], acc[i][j]);
      }
      return;
    }
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
  };

  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  if constexpr (PIPE == 1 || PIPE == 3) {
    // The operand fragments run one k-step ahead of the MFMAs in a second
    // register set, so a wave issues its MFMAs back to back instead of
    // waiting for LDS in front of every k-step; the slab hand-over (LDS
    // stores of the next slab + barrier) sits in front of the LAST k-step,
    // whose MFMAs cover the first fragment reads from the other buffer.
    bf16x8 fa[2][TM], fb[2][TN];
    auto ldfrag = [&](auto set, int buf, int kk) {
      constexpr int S = decltype(set)::value;
      const bf16_t* a_s = sA + buf * BM * BK + (wm * WM + l32) * BK;
      const bf16_t* b_s = sB + buf * BN * BK + (wn * WN + l32) * BK;
      const int coff = (((2 * kk + lh) ^ frag_sw) * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[S][i] = *reinterpret_cast<const bf16x8*>(a_s + i * 32 * BK + coff);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[S][j] = *reinterpret_cast<const bf16x8*>(b_s + j * 32 * BK + coff);
    };
    auto mma = [&](auto set) {
      constexpr int S = decltype(set)::value;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = tok_major ? mfma32(fa[S][i], fb[S][j], acc[i][j]) : mfma32(fb[S][j], fa[S][i], acc[i][j]);
    };
    // scheduling hint: spread the TM + TN LDS reads of the next k-step over the TM * TN MFMAs of this one
    auto interleave = [&]() {
      constexpr int PER = (TM * TN) / (TM + TN) > 0 ? (TM * TN) / (TM + TN) : 1;
#pragma unroll
      for (int i = 0; i < TM + TN; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // DS read
      }
    };
    // The hand-over is unconditional so that a slab is straight-line code: behind the last slab it
    // re-reads the last weight slab and parks stale registers in the idle buffer, nobody reads them.
    auto slab = [&](auto lset, auto sset, int buf, int kt) {
      bload(buf ^ 1, kt + 1 < KT_ ? kt + 1 : KT_ - 1);  // the other buffer is free since the last barrier
      gload(lset, kt + 2);   // past the last slab: residual rows of the first epilogue passes (see gload)
      // the loads stay in front of the slab's arithmetic: moved down by the scheduler they would
      // share registers with the fragments and lose half of their head start
      __builtin_amdgcn_sched_barrier(0);
      ldfrag(S1{}, buf, 1); mma(S0{}); interleave();
      ldfrag(S0{}, buf, 2); mma(S1{}); interleave();
      ldfrag(S1{}, buf, 3); mma(S0{}); interleave();
      __builtin_amdgcn_sched_barrier(0);   // the LDS stores wait for loads issued a slab ago: keep them late
      sstore(sset, buf ^ 1);
      if constexpr (B_DIRECT) wait_vm(std::integral_constant<int, A_LD>{});  // all but the newest A loads: the weight slab has landed
      __syncthreads();
      ldfrag(S0{}, buf ^ 1, 0); mma(S1{}); interleave();
    };
    // PIPE == 3: both slabs of step kt + 1 are in flight towards the other buffer while step kt is multiplied.
    // The last two steps also start the residual rows of the first two epilogue passes (PHASE 1: the step
    // before the last, whose wait leaves those newest loads in flight; PHASE 2: the last step, which has
    // nothing to fetch for the product).
    // residual rows of an epilogue pass through the buffer descriptor: every lane of every wave issues exactly
    // XPER_T loads whatever the tile's position (rows past M are read like any other, columns past N come back
    // as zero), so the wait below can count them
    auto xload_all = [&](auto set, int pass) {
      if constexpr (X_IN_LOOP) {
        constexpr int S = decltype(set)::value;
#pragma unroll
        for (int i = 0; i < XPER_T; ++i)
          xr[S][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
              rsrc_x, x_voff * 4u, (unsigned)(m0 + pass * XROWS + XSTEP * i) * (unsigned)p.ldr * 4u, 2));
      }
    };
    auto slab_direct = [&](int buf, int kt, auto phase) {
      constexpr int PHASE = decltype(phase)::value;
      if constexpr (PHASE < 2) { bload(buf ^ 1, kt + 1); aload(buf ^ 1, kt + 1); }
      if constexpr (PHASE == 1) xload_all(S0{}, 0);
      if constexpr (PHASE == 2) xload_all(S1{}, 1);
      __builtin_amdgcn_sched_barrier(0);
      ldfrag(S1{}, buf, 1); mma(S0{}); interleave();
      ldfrag(S0{}, buf, 2); mma(S1{}); interleave();
      ldfrag(S1{}, buf, 3); mma(S0{}); interleave();
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (PHASE < 2) {
        // both slabs have landed in the other buffer (loads complete in order: the residual rows are newer)
        wait_vm(std::integral_constant<int, (PHASE == 1 && X_IN_LOOP) ? XPER_T : 0>{});
        __syncthreads();
        ldfrag(S0{}, buf ^ 1, 0);
      }
      mma(S1{});
      if constexpr (PHASE < 2) interleave();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using P2 = std::integral_constant<int, 2>;
    if constexpr (A_DIRECT) {
      bload(0, 0);
      aload(0, 0);
      wait_vm(std::integral_constant<int, 0>{});
      __syncthreads();
      ldfrag(S0{}, 0, 0);
      for (int kt = 0; kt < KT_ - 2; kt += 2) {
        slab_direct(0, kt, P0{});
        slab_direct(1, kt + 1, P0{});
      }
      slab_direct(0, KT_ - 2, P1{});
      slab_direct(1, KT_ - 1, P2{});
    } else {
    bload(0, 0);
    gload(S0{}, 0);
    gload(S1{}, 1);
    sstore(S0{}, 0);
    // loads complete in order: once all but the newest A_LD (slab 1's) are done, weight slab 0 has landed
    if constexpr (B_DIRECT) wait_vm(std::integral_constant<int, A_LD>{});
    __syncthreads();
    ldfrag(S0{}, 0, 0);
    for (int kt = 0; kt < KT_; kt += 2) {
      slab(S0{}, S1{}, 0, kt);
      slab(S1{}, S0{}, 1, kt + 1);
    }
    }
    if constexpr (X_IN_LOOP && B_DIRECT && !A_DIRECT) {
#pragma unroll
      for (int i = 0; i < XPER_T; ++i) xr[0][i] = __builtin_bit_cast(f32x4, ra[i / A_LD][i % A_LD]);
      xload(S1{}, 1);   // into the registers the operand fragments have left
    } else if constexpr (X_IN_LOOP && !A_DIRECT) {
#pragma unroll
      for (int i = 0; i < XPER_T; ++i) {
        xr[0][i] = __builtin_bit_cast(f32x4, i < A_LD ? ra[0][i < A_LD ? i : 0] : rb[0][i < A_LD ? 0 : i - A_LD]);
        xr[1][i] = __builtin_bit_cast(f32x4, i < A_LD ? ra[1][i < A_LD ? i : 0] : rb[1][i < A_LD ? 0 : i - A_LD]);
      }
    }
  } else if constexpr (PIPE == 2) {
    // four slabs ahead (the launcher takes this form only for K % 256 == 0)
    using S2 = std::integral_constant<int, 2>;
    using S3 = std::integral_constant<int, 3>;
    gload(S0{}, 0);
    gload(S1{}, 1);
    gload(S2{}, 2);
    gload(S3{}, 3);
    sstore(S0{}, 0);
    __syncthreads();
    for (int kt = 0; kt < KT_; kt += 4) {
      gload(S0{}, kt + 4);   // past the last slab: residual rows of epilogue pass 0 (see gload)
      compute(0);
      sstore(S1{}, 1);
      __syncthreads();
      gload(S1{}, kt + 5);   // ... and of pass 1
      compute(1);
      sstore(S2{}, 0);
      __syncthreads();
      gload(S2{}, kt + 6);
      compute(0);
      sstore(S3{}, 1);
      __syncthreads();
      gload(S3{}, kt + 7);
      compute(1);
      if (X_IN_LOOP && kt + 4 >= KT_) break;   // nothing left to hand over
      sstore(S0{}, 0);
      __syncthreads();
    }
    if constexpr (X_IN_LOOP) {
#pragma unroll
      for (int i = 0; i < XPER_T; ++i) {
        xr[0][i] = __builtin_bit_cast(f32x4, i < A_LD ? ra[0][i < A_LD ? i : 0] : rb[0][i < A_LD ? 0 : i - A_LD]);
        xr[1][i] = __builtin_bit_cast(f32x4, i < A_LD ? ra[1][i < A_LD ? i : 0] : rb[1][i < A_LD ? 0 : i - A_LD]);
      }
    }
  } else {
    gload(S0{}, 0);
    gload(S1{}, 1);
    sstore(S0{}, 0);
    __syncthreads();
    for (int kt = 0; kt < KT_; kt += 2) {
      gload(S0{}, kt + 2);   // past the last slab: residual rows of epilogue pass 0 (see gload)
      compute(0);
      sstore(S1{}, 1);
      __syncthreads();
      gload(S1{}, kt + 3);   // ... and of pass 1
      compute(1);
      if (X_IN_LOOP && kt + 2 >= KT_) break;   // nothing left to hand over
      sstore(S0{}, 0);
      __syncthreads();
    }
    if constexpr (X_IN_LOOP) {
#pragma unroll
      for (int i = 0; i < XPER_T; ++i) {
        xr[0][i] = __builtin_bit_cast(f32x4, i < A_LD ? ra[0][i < A_LD ? i : 0] : rb[0][i < A_LD ? 0 : i - A_LD]);
        xr[1][i] = __builtin_bit_cast(f32x4, i < A_LD ? ra[1][i < A_LD ? i : 0] : rb[1][i < A_LD ? 0 : i - A_LD]);
      }
    }
  }

  // ------------------------------------------------------------ epilogue ----
  // The accumulators go through LDS (the operand buffers are idle now) so
  // that global memory sees whole 16-byte chunks of consecutive rows: a lane
  // owns one staging row (l32) and four consecutive columns per register
  // group; chunk c of staging row r sits at physical chunk c ^ (r & 15), which
  // spreads the 16 rows of an access phase over all banks.
  __syncthreads();  // every wave is done reading the operand buffers
  unsigned char* stage = smem;

  if (EPI == EPI_BIAS_RESIDUAL || EPI == EPI_BIAS_POS) {
    // fp32 staging, XROWS token rows per pass: [XROWS][BN] floats
    constexpr int ROWB = BN * 4;          // bytes per staging row
    constexpr int PASSES = BM / XROWS;
    auto fp32_pass = [&](auto set, int pass) {
      constexpr int S = decltype(set)::value;
      if (pass > 0) __syncthreads();
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int base = wm * WM + i * 32;            // first tile row of this 32-row group
        if (base / XROWS != pass) continue;            // wave-uniform
        const int r = base % XROWS + l32;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int gi = 0; gi < 4; ++gi) {
            const int cl = wn * WN + j * 32 + gi * 8 + lh * 4;  // column inside the tile
            const float4 b4 = *reinterpret_cast<const float4*>(sBias + cl);
            f32x4 v = {acc[i][j][gi * 4 + 0] + b4.x, acc[i][j][gi * 4 + 1] + b4.y,
                       acc[i][j][gi * 4 + 2] + b4.z, acc[i][j][gi * 4 + 3] + b4.w};
            *reinterpret_cast<f32x4*>(stage + r * ROWB + (((cl >> 2) ^ (r & 15)) << 4)) = v;
          }
      }
      __syncthreads();
      // The sums leave through global stores.  The 128-bit buffer store with a scalar offset is no
      // alternative here: the compiler puts no wait state behind that form, and with the next chunk's
      // additions rewriting its data registers in the following cycle a stored row was wrong once in
      // about 1e8 stores on gfx950 (gone with one s_nop behind each store, no faster than this form).
      if constexpr (emit) {
        // The updated rows also leave as bf16 (the operand of the next product, whose pre-norm is folded into
        // its weights) together with their statistics pairs.  A half-wave holds one row's 128-column group,
        // four values per lane, whatever the tile shape, so the pairs carry the same bits for every shape.
        const int c = tid % XNCH;
        const int grp = x_col / STAT_GROUP;
        const int left = p.N - grp * STAT_GROUP;
        const float inv_cnt = left <= 0 ? 0.f : 1.0f / (float)(left < STAT_GROUP ? left : STAT_GROUP);
#pragma unroll
        for (int i = 0; i < XPER_T; ++i) {
          const int r = x_r0 + XSTEP * i;
          const int row = m0 + pass * XROWS + XSTEP * i + x_r0;
          const bool ok = x_col_ok && row < p.M;
          f32x4 sum = {0.f, 0.f, 0.f, 0.f};
          if (ok) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(stage + r * ROWB + ((c ^ (r & 15)) << 4));
            f32x4* dst = reinterpret_cast<f32x4*>(p.R + (long)(row - x_r0) * p.ldr + x_voff);
            if constexpr (X_IN_LOOP) { sum = xr[S][i] + v; __builtin_nontemporal_store(sum, dst); }
            else { sum = *dst + v; *dst = sum; }
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16_t)sum[e];
            *reinterpret_cast<bf16x4*>(p.xb + (long)row * p.ldxb + x_col) = o;
          }
          if constexpr (emit_stats) {
            float mean, m2;
            group_mean_m2(sum, ok, inv_cnt, mean, m2);
            if ((tid & 31) == 0 && row < p.M && grp < p.n_part_out)
              *reinterpret_cast<float2*>(p.stats_out + ((long)row * p.n_part_out + grp) * 2) = make_float2(mean, m2);
          }
        }
      } else if (x_col_ok) {
        const int c = tid % XNCH;
#pragma unroll
        for (int i = 0; i < XPER_T; ++i) {
          const int r = x_r0 + XSTEP * i;
          const int row0 = m0 + pass * XROWS + XSTEP * i;              // uniform
          if (row0 + x_r0 < p.M) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(stage + r * ROWB + ((c ^ (r & 15)) << 4));
            f32x4* dst = reinterpret_cast<f32x4*>(p.R + (long)row0 * p.ldr + x_voff);
            if (EPI == EPI_BIAS_RESIDUAL) {
              if constexpr (X_IN_LOOP) __builtin_nontemporal_store(xr[S][i] + v, dst);   // streamed: read next by a row kernel, not by this launch
              else *dst = *dst + v;      // other tile shapes: plain read-modify-write
            } else {   // patch embedding: position row by patch index, output row through the slice layout
              const int row = row0 + x_r0;
              *reinterpret_cast<f32x4*>(p.R + p.xrows.row(row) * p.ldr + x_col) =
                  v + *reinterpret_cast<const f32x4*>(p.pos + (long)(row % p.n_pos) * p.N + x_col);
            }
          }
        }
      }
      if (pass + 2 < PASSES) xload(set, pass + 2);
    };
#pragma unroll
    for (int pass = 0; pass < PASSES; pass += 2) {
      fp32_pass(S0{}, pass);
      fp32_pass(S1{}, pass + 1);
    }
  } else {
  // bf16 staging of the whole tile: rows = MFMA lane dimension
  constexpr int SROWS = tok_major ? BN : BM;   // staging rows
  constexpr int SCOLS = tok_major ? BM : BN;   // staging columns
  constexpr int ROWB = SCOLS * 2;
  constexpr int NCH = ROWB / 16;
  constexpr int PER_T = SROWS * NCH / NTHREADS;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      // lane dimension: feature (tok_major) or token; register dimension: the other one
      const int r = tok_major ? (wn * WN + j * 32 + l32) : (wm * WM + i * 32 + l32);
      // the lane's own scalars: bias and column sum of its feature (tok_major), or mean / rstd of its token
      float bl = 0.f, cs = 0.f, mu = 0.f, rs = 1.f;
      if (tok_major) { bl = sBias[r]; if (fold) cs = sCol[r]; }
      else if (fold) { mu = sMu[r]; rs = sRs[r]; }
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) {
        const int cl = (tok_major ? (wm * WM + i * 32) : (wn * WN + j * 32)) + gi * 8 + lh * 4;
        float v[4];
        if (tok_major) {
          if (fold) {   // rstd_t (acc - mean_t colsum) + bias over four consecutive tokens t
            const f32x4 m4 = *reinterpret_cast<const f32x4*>(sMu + cl), r4 = *reinterpret_cast<const f32x4*>(sRs + cl);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaf(r4[e], __builtin_fmaf(-m4[e], cs, acc[i][j][gi * 4 + e]), bl);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][gi * 4 + e] + bl;
          }
        } else {
          const f32x4 b4 = *reinterpret_cast<const f32x4*>(sBias + cl);
          if (fold) {
            const f32x4 c4 = *reinterpret_cast<const f32x4*>(sCol + cl);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaf(rs, __builtin_fmaf(-mu, c4[e], acc[i][j][gi * 4 + e]), b4[e]);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][gi * 4 + e] + b4[e];
          }
        }
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16_t)apply_act_fast<EPI>(v[e]);
        *reinterpret_cast<bf16x4*>(stage + r * ROWB + (((cl >> 3) ^ (r & 15)) << 4) + ((cl & 4) << 1)) = o;
      }
    }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < PER_T; ++i) {
    const int q = tid + NTHREADS * i;
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
      if (row < p.M && col < p.N) {
        const long orow = p.row_map ? (long)p.row_map[row / p.block_tokens] * p.block_tokens + row % p.block_tokens : row;
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p.C + orow * p.ldc + col));
      }
    }
  }
  }  // staging kind
}


// ---------------------------------------------------------------------------
// Persistent form of the default shape (256 x 256 x 64 tile, 8 waves, pipelined
// loop) for the epilogues with bf16 output.  One workgroup per CU walks the
// tile sequence with stride gridDim.x.  The loads that would run past the last
// slab of a tile fetch the first two slabs of the workgroup's NEXT tile instead
// (slab 0 into LDS buffer 0, slab 1 into a register set), and the epilogue
// stages the finished tile through LDS buffer 1 only, in two passes of 128
// rows: the next tile's main loop starts right behind the last store, without
// the launch gap and the exposed first-slab latency a fresh workgroup pays.
// ---------------------------------------------------------------------------
// ADIR: the activation slab also goes from global memory straight into LDS (one slab ahead, like the weight
// slab) instead of through registers two slabs ahead.
template <int EPI, bool FOLD, bool ADIR = false>
__global__ __launch_bounds__(512, 1) void k_gemm_bf16_persist(const GemmParams p, const int gm_, const int gw,
                                                              const int n_tiles) {
  constexpr int BN = 256, NTHREADS = 512, WN = 64, WAVES_N = 4, WM = 128, TM = 4, TN = 2;
  constexpr int A_LD = 4, B_LD = 4, ROWS_PER_LD = 64;
  constexpr bool tok_major = (EPI == EPI_VT);
  static_assert(EPI != EPI_BIAS_RESIDUAL && EPI != EPI_BIAS_POS, "bf16-output epilogues only");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* sB = reinterpret_cast<bf16_t*>(smem);  // [2][BN][64]: bytes 0 .. 64 Ki
  bf16_t* sA = sB + 2 * BN * BK;                 // [2][BM][64]: bytes 64 Ki .. 128 Ki
  float* sBias = reinterpret_cast<float*>(smem + smem_main_bytes<BN, NTHREADS>());
  float* sCol = sBias + BN;   // column sums of the weights, mean and rstd of the tile's rows (folded pre-norm)
  float* sMu = sCol + BN;
  float* sRs = sMu + BM;
  constexpr bool fold = FOLD;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  const int KT_ = p.K / BK;  // even
  const int gn = p.Npad / BN;
  // Per-tile scalars of the epilogue: bias and, with a folded pre-norm, the column sums of the weights and
  // mean / rstd of the tile's rows.  The statistics pairs of the NEXT tile's rows are loaded into registers at
  // the start of a tile's epilogue (one thread per row, one batch of independent loads whose latency passes
  // under the epilogue) and combined at its end, when nobody reads the current tile's scalars any more.
  // (The register copy of the pairs lives inside one epilogue: a variable carried around the tile loop would
  // occupy its registers through the main loop as well.)
  // (t: the calling thread's index, handed in so that the epilogue can pass its opaque copy, see there)
  auto pairs_of = [&](int t, int mrow0) {
    return p.stats + (long)(mrow0 + t < p.M ? mrow0 + t : p.M - 1) * p.n_part * 2;   // rows past M: any valid row, never stored
  };
  auto stats_load = [&](int t, RowPairs& rp, int mrow0) { if (fold && t < BM) rp.load(pairs_of(t, mrow0), p.n_part); };
  auto tile_scalars = [&](int t, const RowPairs& rp, int mrow0, int ncol0) {
    if (t < BN) sBias[t] = p.bias[ncol0 + t];
    if (fold) {
      if (t < BN) sCol[t] = p.colsum[ncol0 + t];
      if (t < BM) {
        float mu, rs;
        rp.finish(p.n_part, p.stat_group, p.norm_dim, p.norm_rms, p.norm_eps, mu, rs);
        sMu[t] = mu;
        sRs[t] = rs;
      }
    }
  };

  // position in the launch order -> tile (same XCD-aware band order as the one-tile kernel; a
  // persistent workgroup keeps pos % 8, i.e. its XCD)
  auto tile_of = [&](int pos, int& m0, int& n0) {
    const int x = pos & 7, slot = pos >> 3;
    const int q = n_tiles >> 3, r = n_tiles & 7;
    const int id = x * q + (x < r ? x : r) + slot;
    const int band_tiles = gm_ * gw;
    const int full_bands = gn / gw;
    int band = id / band_tiles, in_band = id % band_tiles, bw = gw;
    if (band >= full_bands) { band = full_bands; in_band = id - full_bands * band_tiles; bw = gn - full_bands * gw; }
    m0 = (in_band / bw) * BM;
    n0 = (band * gw + in_band % bw) * BN;
  };

  const int ld_row = tid >> 3, ld_c = tid & 7;
  const int st_off = ld_row * BK + ((ld_c ^ SWZ(ld_row)) * 8);
  const unsigned a_voff = ((unsigned)ld_row * (unsigned)p.lda + ld_c * 8) * 2;
  const unsigned bd_voff = ((unsigned)ld_row * (unsigned)p.K + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(p.A), 0, (int)(unsigned)(((long)(p.M - 1) * p.lda + p.K) * 2), 0x00020000);

  __amdgpu_buffer_rsrc_t rsrc_c = __builtin_amdgcn_make_buffer_rsrc(
      p.C, 0, (tok_major || !p.C) ? 0 : (int)(unsigned)(((long)(p.M - 1) * p.ldc + p.N) * 2), 0x00020000);

  u32x4 ra[2][A_LD];
  auto gload = [&](auto set, int mrow0, int kt) {   // activation slab kt of the tile rows mrow0 ..
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
      const unsigned so = ((unsigned)(mrow0 + ROWS_PER_LD * i) * (unsigned)p.lda + (unsigned)(kt * BK)) * 2u;
      ra[S][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, a_voff, so, 0);
    }
  };
  auto bload = [&](int buf, int ncol0, int kt) {    // weight slab kt of the tile columns ncol0 .. -> LDS
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
      const bf16_t* g = p.W + (long)(ncol0 + ROWS_PER_LD * i) * p.K + kt * BK;   // uniform
      bf16_t* l = sB + buf * BN * BK + (wave_u * 64 + NTHREADS * i) * 8;
      const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)l;
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                   :: "v"(bd_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
    }
  };
  auto sstore = [&](auto set, int buf) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      *reinterpret_cast<u32x4*>(sA + buf * BM * BK + ROWS_PER_LD * i * BK + st_off) = ra[S][i];
  };
  // ADIR: activation slab kt of the tile rows mrow0 .. -> LDS, the swizzle applied on the global side as for the
  // weights (LDS-DMA reaches the whole LDS through M0 on gfx950, so the activation buffers above 64 KiB are fine)
  const unsigned ad_voff = ((unsigned)ld_row * (unsigned)p.lda + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  auto aload = [&](int buf, int mrow0, int kt) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
      const bf16_t* g = p.A + (long)(mrow0 + ROWS_PER_LD * i) * p.lda + kt * BK;   // uniform
      bf16_t* l = sA + buf * BM * BK + (wave_u * 64 + NTHREADS * i) * 8;
      const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)l;
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                   :: "v"(ad_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
    }
  };
  auto wait_vm = [&](auto n) {
    constexpr int N = decltype(n)::value;
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
  };

  f32x16 acc[TM][TN];
  bf16x8 fa[2][TM], fb[2][TN];
  const int frag_sw = SWZ(l32);
  auto ldfrag = [&](auto set, int buf, int kk) {
    constexpr int S = decltype(set)::value;
    const bf16_t* a_s = sA + buf * BM * BK + (wm * WM + l32) * BK;
    const bf16_t* b_s = sB + buf * BN * BK + (wn * WN + l32) * BK;
    const int coff = (((2 * kk + lh) ^ frag_sw) * 8);
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[S][i] = *reinterpret_cast<const bf16x8*>(a_s + i * 32 * BK + coff);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[S][j] = *reinterpret_cast<const bf16x8*>(b_s + j * 32 * BK + coff);
  };
  auto mma = [&](auto set) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = tok_major ? mfma32(fa[S][i], fb[S][j], acc[i][j]) : mfma32(fb[S][j], fa[S][i], acc[i][j]);
  };
  auto interleave = [&]() {
#pragma unroll
    for (int i = 0; i < TM + TN; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  using VM_A = std::integral_constant<int, A_LD>;

  int pos = blockIdx.x, m0, n0, m0n, n0n;
  tile_of(pos, m0, n0);
  {
    RowPairs rp0;
    stats_load(tid, rp0, m0);
    tile_scalars(tid, rp0, m0, n0);
  }
  using VM_0 = std::integral_constant<int, 0>;
  bload(0, n0, 0);
  if constexpr (ADIR) {
    aload(0, m0, 0);
    wait_vm(VM_0{});
  } else {
    gload(S0{}, m0, 0);
    gload(S1{}, m0, 1);
    sstore(S0{}, 0);
    wait_vm(VM_A{});   // loads complete in order: all but slab 1's are done, weight slab 0 has landed
  }
  __syncthreads();

  for (;;) {
    ldfrag(S0{}, 0, 0);   // (the copy the last hand-over of the previous tile read is not kept across the epilogue)
    const int nxt = pos + (int)gridDim.x;
    const bool has_next = nxt < n_tiles;
    if (has_next) tile_of(nxt, m0n, n0n); else { m0n = m0; n0n = n0; }   // no next tile: harmless re-reads
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // slab kt sits in LDS buffer `buf` with its first fragments in set 0; slab kt+1 in the register
    // set `sset`.  Slab indices past the tile's end name the first slabs of the next tile.
    auto slab = [&](auto lset, auto sset, int buf, int kt) {
      const bool w_own = kt + 1 < KT_, a_own = kt + 2 < KT_;
      bload(buf ^ 1, w_own ? n0 : n0n, w_own ? kt + 1 : kt + 1 - KT_);
      if constexpr (ADIR) aload(buf ^ 1, w_own ? m0 : m0n, w_own ? kt + 1 : kt + 1 - KT_);
      else gload(lset, a_own ? m0 : m0n, a_own ? kt + 2 : kt + 2 - KT_);
      __builtin_amdgcn_sched_barrier(0);
      ldfrag(S1{}, buf, 1); mma(S0{}); interleave();
      ldfrag(S0{}, buf, 2); mma(S1{}); interleave();
      ldfrag(S1{}, buf, 3); mma(S0{}); interleave();
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (ADIR) {
        wait_vm(VM_0{});        // both slabs have landed in the other buffer
      } else {
        sstore(sset, buf ^ 1);
        wait_vm(VM_A{});
      }
      __syncthreads();
      ldfrag(S0{}, buf ^ 1, 0); mma(S1{}); interleave();
    };
    for (int kt = 0; kt < KT_; kt += 2) {
      slab(S0{}, S1{}, 0, kt);
      slab(S1{}, S0{}, 1, kt + 1);
    }
    // Here LDS buffer 0 holds slab 0 of the next tile and register set 1 holds its slab 1; nobody reads buffer 1 any more (the reads of the last slab were
    // complete at the barrier inside its hand-over).

    // ---- epilogue through LDS buffer 1: staging rows 0..63 of a pass in sB[1], 64..127 in sA[1] ----
    {
    // The epilogue's addresses derive from the thread index through an opaque copy, made anew for every tile:
    // computed once in front of the tile loop (they are loop invariants) they would sit in registers, that is
    // in scratch memory, through the main loop, and every tile would wait for their reloads before its
    // epilogue; recomputing them is a few dozen integer operations.
    int tid_opaque = threadIdx.x;
    asm volatile("" : "+v"(tid_opaque));
    const int tid = tid_opaque, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int l32 = lane & 31, lh = lane >> 5;
    constexpr int ROWB = 512, NCH = 32;
    auto stage_row = [&](int r) -> unsigned char* {   // r = 0..127 inside the pass
      return reinterpret_cast<unsigned char*>(r < 64 ? sB + BN * BK : sA + BM * BK) + (r & 63) * ROWB;
    };
    // Every wave stages half of its own sub-tiles per pass (token-major result: its 32-row group
    // j == pass of both halves i; otherwise its groups i = 2 pass, 2 pass + 1), so a pass holds 128
    // staging rows: slot (r / G) * G + r % G  <->  tile row (slot / G) * 2G + pass * G + slot % G,
    // G = 32 (token-major) or 64.
    constexpr int G = tok_major ? 32 : 64;
    RowPairs rp;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      if (pass > 0) {
        __syncthreads();       // pass 0 has been read out
        if constexpr (fold) stats_load(tid, rp, m0n);   // half of the accumulators are gone: room for the next tile's pairs (no next tile: m0n = m0, harmless re-read)
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if ((tok_major ? j : i / 2) != pass) continue;
          // lane dimension: feature (tok_major) or token; register dimension: the other one
          const int rg = tok_major ? (wn * WN + j * 32 + l32) : (wm * WM + i * 32 + l32);
          const int r = (rg / (2 * G)) * G + rg % G;
          float bl = 0.f, cs = 0.f, mu = 0.f, rs = 1.f;
          if (tok_major) { bl = sBias[rg]; if (fold) cs = sCol[rg]; }
          else if (fold) { mu = sMu[rg]; rs = sRs[rg]; }
          unsigned char* srow = stage_row(r);
#pragma unroll
          for (int gi = 0; gi < 4; ++gi) {
            const int cl = (tok_major ? (wm * WM + i * 32) : (wn * WN + j * 32)) + gi * 8 + lh * 4;
            float v[4];
            if (tok_major) {
              if (fold) {
                const f32x4 m4 = *reinterpret_cast<const f32x4*>(sMu + cl), r4 = *reinterpret_cast<const f32x4*>(sRs + cl);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaf(r4[e], __builtin_fmaf(-m4[e], cs, acc[i][j][gi * 4 + e]), bl);
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][gi * 4 + e] + bl;
              }
            } else {
              const f32x4 b4 = *reinterpret_cast<const f32x4*>(sBias + cl);
              if (fold) {
                const f32x4 c4 = *reinterpret_cast<const f32x4*>(sCol + cl);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaf(rs, __builtin_fmaf(-mu, c4[e], acc[i][j][gi * 4 + e]), b4[e]);
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][gi * 4 + e] + b4[e];
              }
            }
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16_t)apply_act_fast<EPI>(v[e]);
            *reinterpret_cast<bf16x4*>(srow + (((cl >> 3) ^ (r & 15)) << 4) + ((cl & 4) << 1)) = o;
          }
        }
      __syncthreads();
      if (pass == 1 && has_next) tile_scalars(tid, rp, m0n, n0n);   // every read of this tile's scalars is behind us
      // read-out: all LDS reads first, then the stores.  Thread tid owns 16-byte chunk tid % 32 of
      // staging rows tid / 32 + 16 i.
      constexpr int PER_T = 128 * NCH / NTHREADS;   // 8
      u32x4 v[PER_T];
      const int c = tid % NCH;
#pragma unroll
      for (int i = 0; i < PER_T; ++i) {
        const int r = tid / NCH + (NTHREADS / NCH) * i;
        v[i] = *reinterpret_cast<const u32x4*>(stage_row(r) + ((c ^ (r & 15)) << 4));
      }
      if (tok_major) {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
          const int r = tid / NCH + (NTHREADS / NCH) * i;
          const int rg = (r / G) * 2 * G + pass * G + r % G;
          const int f = n0 + rg, tok = m0 + c * 8;
          if (f < p.N && tok < p.M) {
            const int h = f / p.hd_pad, d = f % p.hd_pad;
            const int t = tok / p.n_tok, n = tok % p.n_tok;
            __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4*>(p.VT + (((long)t * p.heads + h) * p.hd_pad + d) * p.n_tok + n));
          }
        }
      } else if (p.row_map) {   // paged output: rows go through the block map
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
          const int r = tid / NCH + (NTHREADS / NCH) * i;
          const int row = m0 + (r / G) * 2 * G + pass * G + r % G, col = n0 + c * 8;
          if (row < p.M && col < p.N) {
            const long orow = (long)p.row_map[row / p.block_tokens] * p.block_tokens + row % p.block_tokens;
            __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4*>(p.C + orow * p.ldc + col));
          }
        }
      } else if (n0 + c * 8 < p.N) {
        // buffer stores: the whole byte offset is the lane offset (the only part the descriptor's range
        // check sees; a scalar offset is outside it), so a row past M is dropped by the hardware.  The
        // data registers are not written again before the next barrier.
        const unsigned voff = ((unsigned)(tid / NCH) * (unsigned)p.ldc + (unsigned)(n0 + c * 8)) * 2u;
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
          const int r0 = (NTHREADS / NCH) * i;                                  // staging row of lane row 0
          const int row0 = m0 + (r0 / G) * 2 * G + pass * G + r0 % G;           // uniform (G % 16 == 0)
          __builtin_amdgcn_raw_buffer_store_b128(v[i], rsrc_c, voff + (unsigned)row0 * (unsigned)p.ldc * 2u, 0, 2);   // streamed (nt): read by a later launch
        }
      }
    }
    }
    if (!has_next) break;
    __syncthreads();   // buffer 1 has been read out: the next tile's first hand-over may fill it
    pos = nxt; m0 = m0n; n0 = n0n;
  }
}

// ---------------------------------------------------------------------------
// Persistent form of the residual product, R += A W^T + bias on the fp32 stream: the tile walk and the main loop
// of the persistent kernel above (both operand slabs straight into LDS, the loads past a tile's last slab fetch
// the next tile's first slab into buffer 0), and the four-pass fp32 read-modify-write epilogue staged through
// LDS buffer 1 only.  A pass holds sub-tile row group i = pass of all eight waves (rows wm * 128 + 32 pass ..
// + 31 of both wave rows: staging row r = 32 wm + row), so every wave stages in every pass.  The stream rows of
// the first two passes are fetched while the last two slabs are multiplied, those of pass p + 2 behind pass p.
//
// BN = 192 (tile 256 x 192) is for output widths that are whole multiples of 192 and not of 256 (1152 = 6 x 192
// = 4.5 x 256: every fifth 256-wide tile column would be half empty).  Its waves stand 4 x 2, each on 64 x 96
// (2 x 3 MFMA blocks; the k-steps of an element are summed in the same order, so the bits are those of every
// other form).  The 64 staging rows of a pass then hold sub-tile row group pass / 2 of wave rows 2 (pass % 2)
// and 2 (pass % 2) + 1, so half of the waves stage in a pass, and a staging row's 48 chunks no longer match a
// wave: thread t reads chunks t, t + 512, .. of the 3072 a pass has, row and column per lane.
// ---------------------------------------------------------------------------
template <int BN>
__global__ __launch_bounds__(512, 1) void k_gemm_bf16_persist_res(const GemmParams p, const int gm_, const int gw,
                                                                  const int n_tiles) {
  static_assert(BN == 256 || BN == 192, "tile widths compiled");
  constexpr bool WIDE = BN == 256;
  constexpr int NTHREADS = 512, WAVES_N = WIDE ? 4 : 2, WN = BN / WAVES_N, WM = BM / (8 / WAVES_N), TM = WM / 32, TN = WN / 32;
  constexpr int A_LD = 4, B_LD = BN / 64, ROWS_PER_LD = 64;
  constexpr int XNCH = BN * 4 / 16;                // 16-byte chunks per staging row (BN = 256: one wave reads one row)
  constexpr int XSTEP = NTHREADS / XNCH;           // BN = 256: 8 staging rows between a thread's chunks
  constexpr int XPER_T = 64 * XNCH / NTHREADS;     // 8 (6) chunks per thread and pass
  constexpr int ROWB = BN * 4;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* sB = reinterpret_cast<bf16_t*>(smem);  // [2][BN][64]: bytes 0 .. 64 Ki
  bf16_t* sA = sB + 2 * BN * BK;                 // [2][BM][64]: bytes 64 Ki .. 128 Ki
  float* sBias = reinterpret_cast<float*>(smem + smem_main_bytes<BN, NTHREADS>());

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  const int KT_ = p.K / BK;  // even
  const int gn = WIDE ? p.Npad / BN : p.N / BN;

  auto tile_of = [&](int pos, int& m0, int& n0) {
    const int x = pos & 7, slot = pos >> 3;
    const int q = n_tiles >> 3, r = n_tiles & 7;
    const int id = x * q + (x < r ? x : r) + slot;
    const int band_tiles = gm_ * gw;
    const int full_bands = gn / gw;
    int band = id / band_tiles, in_band = id % band_tiles, bw = gw;
    if (band >= full_bands) { band = full_bands; in_band = id - full_bands * band_tiles; bw = gn - full_bands * gw; }
    m0 = (in_band / bw) * BM;
    n0 = (band * gw + in_band % bw) * BN;
  };

  const int ld_row = tid >> 3, ld_c = tid & 7;
  const unsigned ad_voff = ((unsigned)ld_row * (unsigned)p.lda + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  const unsigned bd_voff = ((unsigned)ld_row * (unsigned)p.K + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma = [&](const bf16_t* g, bf16_t* l, unsigned voff) {
    const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)l;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(g), "s"(lds_addr) : "memory", "m0");
  };
  auto bload = [&](int buf, int ncol0, int kt) {
#pragma unroll
    for (int i = 0; i < B_LD; ++i)
      dma(p.W + (long)(ncol0 + ROWS_PER_LD * i) * p.K + kt * BK, sB + buf * BN * BK + (wave_u * 64 + NTHREADS * i) * 8, bd_voff);
  };
  auto aload = [&](int buf, int mrow0, int kt) {
#pragma unroll
    for (int i = 0; i < A_LD; ++i)
      dma(p.A + (long)(mrow0 + ROWS_PER_LD * i) * p.lda + kt * BK, sA + buf * BM * BK + (wave_u * 64 + NTHREADS * i) * 8, ad_voff);
  };
  auto wait_vm = [&](auto n) {
    constexpr int N = decltype(n)::value;
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
  };

  f32x16 acc[TM][TN];
  bf16x8 fa[2][TM], fb[2][TN];
  const int frag_sw = SWZ(l32);
  auto ldfrag = [&](auto set, int buf, int kk) {
    constexpr int S = decltype(set)::value;
    const bf16_t* a_s = sA + buf * BM * BK + (wm * WM + l32) * BK;
    const bf16_t* b_s = sB + buf * BN * BK + (wn * WN + l32) * BK;
    const int coff = (((2 * kk + lh) ^ frag_sw) * 8);
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[S][i] = *reinterpret_cast<const bf16x8*>(a_s + i * 32 * BK + coff);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[S][j] = *reinterpret_cast<const bf16x8*>(b_s + j * 32 * BK + coff);
  };
  auto mma = [&](auto set) {
    constexpr int S = decltype(set)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(fb[S][j], fa[S][i], acc[i][j]);
  };
  auto interleave = [&]() {
#pragma unroll
    for (int i = 0; i < TM + TN; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  using VM_0 = std::integral_constant<int, 0>;
  using VM_X = std::integral_constant<int, XPER_T>;

  // Stream rows of an epilogue pass through a buffer descriptor: every lane of every wave issues exactly XPER_T
  // loads whatever the tile's position, so a wait can count them.  BN = 256: the row is a scalar offset, outside
  // the descriptor's range check (rows past M are read like any other: R holds whole tiles); columns past N fall
  // outside the range and come back as zero.  BN = 192: row and column are the lane offset; a row past M comes
  // back as zero.
  __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc(
      p.R, 0, (int)(unsigned)(((long)(p.M - 1) * p.ldr + p.N) * 4), 0x00020000);
  f32x4 xr[2][XPER_T];
  // staging row r of a pass <-> tile row: BN = 256: (r / 32) * 128 + 32 pass + r % 32;
  // BN = 192: (2 (pass % 2) + r / 32) * 64 + 32 (pass / 2) + r % 32
  auto tile_row = [&](int pass, int r) {
    return WIDE ? (r >> 5) * 128 + pass * 32 + (r & 31) : (2 * (pass & 1) + (r >> 5)) * 64 + (pass >> 1) * 32 + (r & 31);
  };
  // BN = 192: chunk i of this thread in a pass: staging row and chunk column
  auto x_r = [&](int i) { return (tid + NTHREADS * i) / XNCH; };
  auto x_c = [&](int i) { return (tid + NTHREADS * i) % XNCH; };

  int pos = blockIdx.x, m0, n0, m0n, n0n;
  tile_of(pos, m0, n0);
  if (tid < BN) sBias[tid] = p.bias[n0 + tid];
  bload(0, n0, 0);
  aload(0, m0, 0);
  wait_vm(VM_0{});
  __syncthreads();

  for (;;) {
    ldfrag(S0{}, 0, 0);
    const int nxt = pos + (int)gridDim.x;
    const bool has_next = nxt < n_tiles;
    if (has_next) tile_of(nxt, m0n, n0n); else { m0n = m0; n0n = n0; }   // no next tile: harmless re-reads
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // the thread's chunk of the stream: column n0 + 4 (tid % 64), rows given by the pass
    const int x_col = n0 + (tid % XNCH) * 4;
    const bool x_col_ok = x_col < p.N;
    auto xload = [&](auto set, int pass) {
      constexpr int S = decltype(set)::value;
#pragma unroll
      for (int i = 0; i < XPER_T; ++i)
        if constexpr (WIDE)
          xr[S][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
              rsrc_x, (unsigned)x_col * 4u, (unsigned)(m0 + tile_row(pass, wave_u + XSTEP * i)) * (unsigned)p.ldr * 4u, 2));
        else
          xr[S][i] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
              rsrc_x, ((unsigned)(m0 + tile_row(pass, x_r(i))) * (unsigned)p.ldr + (unsigned)(n0 + x_c(i) * 4)) * 4u, 0, 2));
    };
    // PHASE 0: a slab in the middle of the tile; 1: the slab before the last (also starts the stream rows of pass 0,
    // which its wait leaves in flight); 2: the last slab (fetches the next tile's first slab, starts pass 1's rows)
    auto slab = [&](int buf, int kt, auto phase) {
      constexpr int PHASE = decltype(phase)::value;
      const bool own = kt + 1 < KT_;
      bload(buf ^ 1, own ? n0 : n0n, own ? kt + 1 : 0);
      aload(buf ^ 1, own ? m0 : m0n, own ? kt + 1 : 0);
      if constexpr (PHASE == 1) xload(S0{}, 0);
      if constexpr (PHASE == 2) xload(S1{}, 1);
      __builtin_amdgcn_sched_barrier(0);
      ldfrag(S1{}, buf, 1); mma(S0{}); interleave();
      ldfrag(S0{}, buf, 2); mma(S1{}); interleave();
      ldfrag(S1{}, buf, 3); mma(S0{}); interleave();
      __builtin_amdgcn_sched_barrier(0);
      // loads complete in order: everything but the newest stream rows has landed
      if constexpr (PHASE == 0) wait_vm(VM_0{}); else wait_vm(VM_X{});
      __syncthreads();
      if constexpr (PHASE < 2) { ldfrag(S0{}, buf ^ 1, 0); mma(S1{}); interleave(); }
      else mma(S1{});
    };
    for (int kt = 0; kt < KT_ - 2; kt += 2) {
      slab(0, kt, std::integral_constant<int, 0>{});
      slab(1, kt + 1, std::integral_constant<int, 0>{});
    }
    slab(0, KT_ - 2, std::integral_constant<int, 1>{});
    slab(1, KT_ - 1, std::integral_constant<int, 2>{});
    // LDS buffer 0 now holds slab 0 of the next tile; nobody reads buffer 1 any more.

    // ---- epilogue through LDS buffer 1: staging rows 0..31 in sB[1], 32..63 in sA[1], [row][256] floats ----
    {
      // addresses from an opaque copy of the thread index, made anew per tile (see the persistent kernel above)
      int tid_opaque = threadIdx.x;
      asm volatile("" : "+v"(tid_opaque));
      const int tid = tid_opaque, lane = tid & 63, wave = tid >> 6;
      const int wm = wave / WAVES_N, wn = wave % WAVES_N;
      const int l32 = lane & 31, lh = lane >> 5;
      const int wave_u = __builtin_amdgcn_readfirstlane(wave);
      auto stage_row = [&](int r) -> unsigned char* {
        return reinterpret_cast<unsigned char*>(r < 32 ? sB + BN * BK : sA + BM * BK) + (r & 31) * ROWB;
      };
      auto fp32_pass = [&](auto set, auto pass_) {
        constexpr int S = decltype(set)::value;
        constexpr int pass = decltype(pass_)::value;
        constexpr int sub = WIDE ? pass : pass >> 1;     // sub-tile row group of a wave that goes through this pass
        if (pass > 0) __syncthreads();   // the previous pass has been read out
        if (WIDE || (wm >> 1) == (pass & 1)) {           // wave-uniform
          const int r = (WIDE ? wm : wm & 1) * 32 + l32;   // this lane's staging row
          unsigned char* srow = stage_row(r);
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
              const int cl = wn * WN + j * 32 + gi * 8 + lh * 4;
              const f32x4 b4 = *reinterpret_cast<const f32x4*>(sBias + cl);
              f32x4 v;
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = acc[sub][j][gi * 4 + e] + b4[e];
              *reinterpret_cast<f32x4*>(srow + (((cl >> 2) ^ (r & 15)) << 4)) = v;
            }
        }
        __syncthreads();
        if (pass == 3 && has_next && tid < BN) sBias[tid] = p.bias[n0n + tid];   // every bias read is behind us
        if constexpr (WIDE) {
          if (x_col_ok) {
            const int c = tid % XNCH;
#pragma unroll
            for (int i = 0; i < XPER_T; ++i) {
              const int r = wave_u + XSTEP * i;
              const int row = m0 + tile_row(pass, r);              // uniform
              if (row < p.M) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(stage_row(r) + ((c ^ (r & 15)) << 4));
                __builtin_nontemporal_store(xr[S][i] + v, reinterpret_cast<f32x4*>(p.R + (long)row * p.ldr + x_col));
              }
            }
          }
        } else {
#pragma unroll
          for (int i = 0; i < XPER_T; ++i) {
            const int r = x_r(i), c = x_c(i);
            const int row = m0 + tile_row(pass, r), col = n0 + c * 4;
            if (row < p.M && col < p.N) {
              const f32x4 v = *reinterpret_cast<const f32x4*>(stage_row(r) + ((c ^ (r & 15)) << 4));
              __builtin_nontemporal_store(xr[S][i] + v, reinterpret_cast<f32x4*>(p.R + (long)row * p.ldr + col));
            }
          }
        }
        if (pass + 2 < 4) xload(set, pass + 2);
      };
      fp32_pass(S0{}, std::integral_constant<int, 0>{});
      fp32_pass(S1{}, std::integral_constant<int, 1>{});
      fp32_pass(S0{}, std::integral_constant<int, 2>{});
      fp32_pass(S1{}, std::integral_constant<int, 3>{});
    }
    if (!has_next) break;
    __syncthreads();   // buffer 1 has been read out: the next tile's first hand-over may fill it
    pos = nxt; m0 = m0n; n0 = n0n;
  }
}

// ---------------------------------------------------------------------------
// Small-tile form for launches of one or two slices (a worker's share of a request under intra-request
// parallelism, Section 3.2.2).  Such a launch has a handful of 128 x 128 tiles, most CUs idle and the busy ones
// waiting for operand slabs: its time is the latency chain of one tile, not matrix work.  Here a tile is
// 64 x 64 (four times as many workgroups, each asking for a quarter of the bytes), four waves of 32 x 32, and
// both operand slabs go from global memory straight into an LDS ring of RING stages, RING - 1 slabs ahead of
// the MFMAs, one barrier per slab.  An element's k-steps are added in the order of every other form (same
// instruction, k ascending), so the bits are those of the large tiles.  The epilogue writes from registers:
// a lane owns one token and 4 consecutive features per register group (EPI_VT: one feature, 4 tokens).
// ---------------------------------------------------------------------------
constexpr int SM_T = 64, SM_RING = 4;
constexpr int SM_STAGE = 2 * SM_T * BK;   // bf16 elements of a ring stage: activation slab, then weight slab
constexpr size_t SM_LDS = (size_t)SM_RING * SM_STAGE * sizeof(bf16_t);

// DUAL (EPI_BIAS): tile columns from Npad on are a second product over the same activations, the value projection,
// whose tiles run with the operand roles of EPI_VT and leave through its store (GemmParams::n2).
template <int EPI, bool DUAL = false>
__global__ __launch_bounds__(256, 2) void k_gemm_bf16_small(const GemmParams p, const int gm, const int bw_) {
  static_assert(!DUAL || EPI == EPI_BIAS, "the second product rides on the plain bias epilogue");
  constexpr bool tok_major = (EPI == EPI_VT);
  constexpr int LPS = 4;   // direct loads per thread and slab: two 32-row halves of each operand
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* ring = reinterpret_cast<bf16_t*>(smem);

  // XCD x (workgroups are dealt round-robin) takes a contiguous run of the tile sequence; the sequence walks
  // bands of bw_ tile columns top to bottom, so the ~32 tiles an XCD holds at once share few operand panels
  const int gn = (p.Npad + (DUAL ? p.n2_pad : 0)) / SM_T;
  int id = blockIdx.x;
  {
    const int nb = gridDim.x, x = id & 7, slot = id >> 3, q = nb >> 3, r = nb & 7;
    id = x * q + (x < r ? x : r) + slot;
  }
  const int band_tiles = gm * bw_, full_bands = gn / bw_;
  int band = id / band_tiles, in_band = id % band_tiles, bw = bw_;
  if (band >= full_bands) { band = full_bands; in_band = id - full_bands * band_tiles; bw = gn - full_bands * bw_; }
  const int m0 = (in_band / bw) * SM_T;
  const int n0 = (band * bw_ + in_band % bw) * SM_T;
  const bool vt_tile = tok_major || (DUAL && n0 >= p.Npad);   // uniform over the workgroup

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const int ld_row = tid >> 3, ld_c = tid & 7;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // the lane that lands on physical chunk ld_c of its LDS row fetches logical chunk ld_c ^ SWZ(row)
  const unsigned a_voff = ((unsigned)ld_row * (unsigned)p.lda + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  const unsigned b_voff = ((unsigned)ld_row * (unsigned)p.K + ((ld_c ^ SWZ(ld_row)) * 8)) * 2;
  const int KT_ = p.K / BK;

  // slab kt -> ring stage kt % RING (rows of a ragged last tile past M are read like any other: A holds whole
  // 256-row tiles; their results are never stored)
  auto issue = [&](int kt) {
    bf16_t* st = ring + (kt % SM_RING) * SM_STAGE;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const bf16_t* g = p.A + (long)(m0 + 32 * i) * p.lda + kt * BK;   // uniform
      const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(st + (wave_u * 64 + 256 * i) * 8);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                   :: "v"(a_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const bf16_t* g = p.W + (long)(n0 + 32 * i) * p.K + kt * BK;
      const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(st + SM_T * BK + (wave_u * 64 + 256 * i) * 8);
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                   :: "v"(b_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
    }
  };
  auto wait_vm = [&](auto n) {
    constexpr int N = decltype(n)::value;
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
  };

#pragma unroll
  for (int s = 0; s < SM_RING - 1; ++s)
    if (s < KT_) issue(s);

  // what the epilogue reads, fetched under the main loop: bias, and the residual rows it adds to.
  // Register group g of a lane: tile row (token) wm * 32 + l32, tile columns wn * 32 + 8 g + 4 lh .. + 3
  // (EPI_VT: feature wn * 32 + l32, tokens wm * 32 + 8 g + 4 lh .. + 3)
  const int row = m0 + wm * 32 + l32;                 // token of this lane (not EPI_VT)
  const int col0 = n0 + wn * 32 + 4 * lh;             // first feature of register group 0 (not EPI_VT)
  f32x4 b4[4], x4[4];
  float b1 = 0.f;
  if (vt_tile) {
    b1 = p.bias[n0 + wn * 32 + l32];
  } else {
#pragma unroll
    for (int g = 0; g < 4; ++g) b4[g] = *reinterpret_cast<const f32x4*>(p.bias + col0 + 8 * g);
  }
  if constexpr (EPI == EPI_BIAS_RESIDUAL) {
#pragma unroll
    for (int g = 0; g < 4; ++g)
      if (row < p.M && col0 + 8 * g < p.N) x4[g] = *reinterpret_cast<const f32x4*>(p.R + (long)row * p.ldr + col0 + 8 * g);
  } else if constexpr (EPI == EPI_BIAS_POS) {
#pragma unroll
    for (int g = 0; g < 4; ++g)
      if (row < p.M && col0 + 8 * g < p.N) x4[g] = *reinterpret_cast<const f32x4*>(p.pos + (long)(row % p.n_pos) * p.N + col0 + 8 * g);
  }

  f32x16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const int frag_sw = SWZ(l32);
  auto main_loop = [&](auto tm) {
  constexpr bool TOKM = decltype(tm)::value;
  for (int kt = 0; kt < KT_; ++kt) {
    // Loads complete in order: slab kt has landed once at most LPS x (slabs issued behind it) of this
    // thread's loads are outstanding.  (The epilogue's own loads above are older than every slab but the
    // first RING - 1, and counted among the outstanding ones only before those have landed.)
    const int behind = KT_ - 1 - kt;
    if (behind >= SM_RING - 2) wait_vm(std::integral_constant<int, (SM_RING - 2) * LPS>{});
    else if (behind == 1) wait_vm(std::integral_constant<int, LPS>{});
    else wait_vm(std::integral_constant<int, 0>{});
    __syncthreads();   // everyone's part of slab kt is in LDS, and everyone is done reading slab kt - 1
    if (kt + SM_RING - 1 < KT_) issue(kt + SM_RING - 1);   // into the stage slab kt - 1 has left
    const bf16_t* a_s = ring + (kt % SM_RING) * SM_STAGE + (wm * 32 + l32) * BK;
    const bf16_t* b_s = ring + (kt % SM_RING) * SM_STAGE + SM_T * BK + (wn * 32 + l32) * BK;
    bf16x8 xf[BK / 16], wf[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int coff = ((2 * kk + lh) ^ frag_sw) * 8;
      xf[kk] = *reinterpret_cast<const bf16x8*>(a_s + coff);
      wf[kk] = *reinterpret_cast<const bf16x8*>(b_s + coff);
    }
    __builtin_amdgcn_sched_barrier(0);   // all fragment reads of the slab first: their latency is paid once
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) acc = TOKM ? mfma32(xf[kk], wf[kk], acc) : mfma32(wf[kk], xf[kk], acc);
  }
  };
  if (DUAL && vt_tile) main_loop(std::true_type{});
  else main_loop(std::integral_constant<bool, tok_major>{});

  if (vt_tile) {
    const int f = n0 - (DUAL ? p.Npad : 0) + wn * 32 + l32;   // feature of the value projection
    if (f < (DUAL ? p.n2 : p.N)) {
      const int h = f / p.hd_pad, d = f % p.hd_pad;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int tok = m0 + wm * 32 + 8 * g + 4 * lh;   // n_tok % 8 == 0: the four tokens share a slice
        if (tok < p.M) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16_t)(acc[4 * g + e] + b1);
          const int t = tok / p.n_tok, n = tok % p.n_tok;
          *reinterpret_cast<bf16x4*>(p.VT + (((long)t * p.heads + h) * p.hd_pad + d) * p.n_tok + n) = o;
        }
      }
    }
  } else if (row < p.M) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int col = col0 + 8 * g;
      if (col >= p.N) continue;
      const f32x4 v = {acc[4 * g + 0] + b4[g][0], acc[4 * g + 1] + b4[g][1], acc[4 * g + 2] + b4[g][2], acc[4 * g + 3] + b4[g][3]};
      if constexpr (EPI == EPI_BIAS_RESIDUAL) {
        *reinterpret_cast<f32x4*>(p.R + (long)row * p.ldr + col) = x4[g] + v;
      } else if constexpr (EPI == EPI_BIAS_POS) {
        *reinterpret_cast<f32x4*>(p.R + p.xrows.row(row) * p.ldr + col) = v + x4[g];
      } else {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16_t)apply_act_fast<EPI>(v[e]);
        const long orow = p.row_map ? (long)p.row_map[row / p.block_tokens] * p.block_tokens + row % p.block_tokens : row;
        *reinterpret_cast<bf16x4*>(p.C + orow * p.ldc + col) = o;
      }
    }
  }
}

// behind the operand slabs: the tile's bias values, and for a folded pre-norm the column sums of its
// weights and the mean / rstd of its rows
template <int BN, int NT, int BM_ = BM>
constexpr size_t smem_bytes() { return smem_main_bytes<BN, NT, BM_>() + (2 * BN + 2 * BM_) * sizeof(float); }

thread_local long g_kernel_launches = 0;   // kernels launched by bf16_gemm on this host thread so far (a product may be cut into two launches)

template <int BN, int NT, int WN, int EPI, int PIPE, int BM_ = BM, int FOLD = 0>
hipError_t launch(const GemmParams& p, hipStream_t st) {
  const int gm = (p.M + BM_ - 1) / BM_, gn = p.Npad / BN;
  const int n_tiles = gm * gn;
  if (n_tiles == 0) return hipSuccess;
  // Band width.  The ~32 workgroups an XCD runs at once cover (32 / gw) tile rows x gw tile
  // columns and move through K together, so per wave of tiles the L2 pulls 32 / gw activation
  // panels and gw weight panels (256 x K each) over the fabric; the weight panels are not
  // pulled again by later waves while a band's whole weight panel fits the 4 MiB L2.
  const double panel = 256.0 * p.K * sizeof(bf16_t);
  int gw = 1;
  double best = 1e30;
  for (int c = 1; c <= gn && c <= 32; ++c) {
    const bool resident = c * (double)BN * p.K * sizeof(bf16_t) <= 2.5 * (1 << 20);
    const double cost = (32.0 / c) * panel + (resident ? 0.0 : c * panel * (BN / 256.0));
    if (cost < best * 0.999) { best = cost; gw = c; }
  }
  if (p.band > 0 && p.band <= gn) gw = p.band;
  k_gemm_bf16<BN, NT, WN, EPI, PIPE, BM_, FOLD><<<dim3(n_tiles), dim3(NT), smem_bytes<BN, NT, BM_>(), st>>>(p, gm, gw);
  ++g_kernel_launches;
  return hipGetLastError();
}

int cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      n = 256;
  }
  return n;
}

template <int EPI, bool DUAL = false>
hipError_t launch_small_e(const GemmParams& p, hipStream_t st) {
  const int gm = (p.M + SM_T - 1) / SM_T, gn = (p.Npad + (DUAL ? p.n2_pad : 0)) / SM_T;
  if (gm * gn == 0) return hipSuccess;
  k_gemm_bf16_small<EPI, DUAL><<<dim3(gm * gn), dim3(256), SM_LDS, st>>>(p, gm, gn < 4 ? gn : 4);
  ++g_kernel_launches;
  return hipGetLastError();
}
// the small-tile form has neither the folded pre-norm nor the bf16 copy of the residual rows
bool small_form_has(const GemmParams& p) { return !p.stats && !p.xb; }
hipError_t launch_small(const GemmParams& p, hipStream_t st) {
  if (p.n2_pad > 0) return p.epi == EPI_BIAS ? launch_small_e<EPI_BIAS, true>(p, st) : hipErrorInvalidValue;
  switch (p.epi) {
    case EPI_BIAS: return launch_small_e<EPI_BIAS>(p, st);
    case EPI_BIAS_GELU_ERF: return launch_small_e<EPI_BIAS_GELU_ERF>(p, st);
    case EPI_BIAS_GELU_TANH: return launch_small_e<EPI_BIAS_GELU_TANH>(p, st);
    case EPI_BIAS_RESIDUAL: return launch_small_e<EPI_BIAS_RESIDUAL>(p, st);
    case EPI_BIAS_POS: return launch_small_e<EPI_BIAS_POS>(p, st);
    case EPI_VT: return launch_small_e<EPI_VT>(p, st);
  }
  return hipErrorInvalidValue;
}
template <int EPI, bool DUAL = false>
hipError_t set_attr_small() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16_small<EPI, DUAL>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)SM_LDS);
}
// EPD_SMALL_TILES=0: launches of a slice or two stay on the 128 x 128 tiles (what the small form was measured against)
bool small_tiles() {
  static const bool on = !(getenv("EPD_SMALL_TILES") && getenv("EPD_SMALL_TILES")[0] == '0');
  return on;
}

// Activation slabs straight into LDS (no register hop): the persistent kernels (-5 % on the q/k, value and FC1
// products of the 104-slice batch) and the residual product when K is long (FC2 -1 %; the short out-projection
// is 1 % faster with its rows staged in registers two slabs ahead).  EPD_A_DIRECT=0 keeps the register-staged
// forms, the ones these were measured against.
bool a_direct() {
  static const bool on = !(getenv("EPD_A_DIRECT") && getenv("EPD_A_DIRECT")[0] == '0');
  return on;
}

template <int EPI, bool FOLD>
hipError_t launch_persist(const GemmParams& p, hipStream_t st) {
  const int gm = (p.M + BM - 1) / BM, gn = p.Npad / 256;
  const int n_tiles = gm * gn;
  if (n_tiles == 0) return hipSuccess;
  const double panel = 256.0 * p.K * sizeof(bf16_t);
  int gw = 1;
  double best = 1e30;
  for (int c = 1; c <= gn && c <= 32; ++c) {
    const bool resident = c * 256.0 * p.K * sizeof(bf16_t) <= 2.5 * (1 << 20);
    const double cost = (32.0 / c) * panel + (resident ? 0.0 : c * panel);
    if (cost < best * 0.999) { best = cost; gw = c; }
  }
  if (p.band > 0 && p.band <= gn) gw = p.band;
  const int grid = n_tiles < cu_count() ? n_tiles : cu_count();
  if (!FOLD && a_direct()) k_gemm_bf16_persist<EPI, false, true><<<dim3(grid), dim3(512), smem_bytes<256, 512>(), st>>>(p, gm, gw, n_tiles);
  else k_gemm_bf16_persist<EPI, FOLD><<<dim3(grid), dim3(512), smem_bytes<256, 512>(), st>>>(p, gm, gw, n_tiles);
  ++g_kernel_launches;
  return hipGetLastError();
}

bool persist_res() {   // EPD_PERSIST_RES=0: the residual products stay on the one-tile-per-workgroup kernels
  static const bool on = !(getenv("EPD_PERSIST_RES") && getenv("EPD_PERSIST_RES")[0] == '0');
  return on;
}

// residual product on the persistent kernel (whole 256 x BN tiles; no bf16 rows / statistics emitted);
// BN = 192 wants N % 192 == 0
template <int BN = 256>
hipError_t launch_persist_res(const GemmParams& p, hipStream_t st) {
  if (BN != 256 && p.N % BN != 0) return hipErrorInvalidValue;
  const int gm = (p.M + BM - 1) / BM, gn = BN == 256 ? p.Npad / 256 : p.N / BN;
  const int n_tiles = gm * gn;
  if (n_tiles == 0) return hipSuccess;
  const double panel = (double)BN * p.K * sizeof(bf16_t);
  int gw = 1;
  double best = 1e30;
  for (int c = 1; c <= gn && c <= 32; ++c) {
    const bool resident = c * panel <= 2.5 * (1 << 20);
    const double cost = (32.0 / c) * panel + (resident ? 0.0 : c * panel);
    if (cost < best * 0.999) { best = cost; gw = c; }
  }
  if (p.band > 0 && p.band <= gn) gw = p.band;
  const int grid = n_tiles < cu_count() ? n_tiles : cu_count();
  k_gemm_bf16_persist_res<BN><<<dim3(grid), dim3(512), smem_bytes<BN, 512>(), st>>>(p, gm, gw, n_tiles);
  ++g_kernel_launches;
  return hipGetLastError();
}

bool tiles_192() {   // EPD_TILES_192=0: widths like 1152 stay on the 256-wide tiles
  static const bool on = !(getenv("EPD_TILES_192") && getenv("EPD_TILES_192")[0] == '0');
  return on;
}

template <bool FOLD>
hipError_t dispatch_persist_f(const GemmParams& p, hipStream_t st) {
  switch (p.epi) {
    case EPI_BIAS: return launch_persist<EPI_BIAS, FOLD>(p, st);
    case EPI_BIAS_GELU_ERF: return launch_persist<EPI_BIAS_GELU_ERF, FOLD>(p, st);
    case EPI_BIAS_GELU_TANH: return launch_persist<EPI_BIAS_GELU_TANH, FOLD>(p, st);
    case EPI_VT: return launch_persist<EPI_VT, FOLD>(p, st);
  }
  return hipErrorInvalidValue;
}
hipError_t dispatch_persist(const GemmParams& p, hipStream_t st) {
  return p.stats ? dispatch_persist_f<true>(p, st) : dispatch_persist_f<false>(p, st);
}

template <int EPI, bool FOLD>
hipError_t set_attr_persist() {
  if (!FOLD) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16_persist<EPI, false, true>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<256, 512>());
    if (e != hipSuccess) return e;
  }
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16_persist<EPI, FOLD>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<256, 512>());
}

template <int BN, int NT, int WN, int PIPE = 0, int BM_ = BM>
hipError_t dispatch(const GemmParams& p, hipStream_t st) {
  if (p.stats) {   // folded pre-norm (bf16-output epilogues)
    switch (p.epi) {
      case EPI_BIAS: return launch<BN, NT, WN, EPI_BIAS, PIPE, BM_, 2>(p, st);
      case EPI_BIAS_GELU_ERF: return launch<BN, NT, WN, EPI_BIAS_GELU_ERF, PIPE, BM_, 2>(p, st);
      case EPI_BIAS_GELU_TANH: return launch<BN, NT, WN, EPI_BIAS_GELU_TANH, PIPE, BM_, 2>(p, st);
      case EPI_VT: return launch<BN, NT, WN, EPI_VT, PIPE, BM_, 2>(p, st);
    }
    return hipErrorInvalidValue;
  }
  if (p.xb) {      // residual epilogue that also stores the rows as bf16, with or without their statistics
    if (p.epi != EPI_BIAS_RESIDUAL) return hipErrorInvalidValue;
    return p.stats_out ? launch<BN, NT, WN, EPI_BIAS_RESIDUAL, PIPE, BM_, 2>(p, st)
                       : launch<BN, NT, WN, EPI_BIAS_RESIDUAL, PIPE, BM_, 1>(p, st);
  }
  switch (p.epi) {
    case EPI_BIAS: return launch<BN, NT, WN, EPI_BIAS, PIPE, BM_>(p, st);
    case EPI_BIAS_GELU_ERF: return launch<BN, NT, WN, EPI_BIAS_GELU_ERF, PIPE, BM_>(p, st);
    case EPI_BIAS_GELU_TANH: return launch<BN, NT, WN, EPI_BIAS_GELU_TANH, PIPE, BM_>(p, st);
    case EPI_BIAS_RESIDUAL: return launch<BN, NT, WN, EPI_BIAS_RESIDUAL, PIPE, BM_>(p, st);
    case EPI_BIAS_POS: return launch<BN, NT, WN, EPI_BIAS_POS, PIPE, BM_>(p, st);
    case EPI_VT: return launch<BN, NT, WN, EPI_VT, PIPE, BM_>(p, st);
  }
  return hipErrorInvalidValue;
}

template <int BN, int NT, int WN, int EPI, int PIPE, int BM_, int FOLD = 0>
hipError_t set_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16<BN, NT, WN, EPI, PIPE, BM_, FOLD>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<BN, NT, BM_>());
}

template <int BN, int NT, int WN, int PIPE = 0, int BM_ = BM>
hipError_t set_attr_all() {
  hipError_t e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS, PIPE, BM_>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_GELU_ERF, PIPE, BM_>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_GELU_TANH, PIPE, BM_>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_RESIDUAL, PIPE, BM_>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_POS, PIPE, BM_>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_VT, PIPE, BM_>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS, PIPE, BM_, 2>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_GELU_ERF, PIPE, BM_, 2>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_GELU_TANH, PIPE, BM_, 2>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_RESIDUAL, PIPE, BM_, 1>()) != hipSuccess) return e;
  if ((e = set_attr<BN, NT, WN, EPI_BIAS_RESIDUAL, PIPE, BM_, 2>()) != hipSuccess) return e;
  return set_attr<BN, NT, WN, EPI_VT, PIPE, BM_, 2>();
}

}  // namespace

long bf16_gemm_kernel_launches() { return g_kernel_launches; }

// The q/k and the value projection of a single slice as one launch of small tiles: three tiles per CU on the
// 300M shape, where two launches of two and one were measured 5 us slower per layer.
bool bf16_gemm_pair_fits(const GemmParams& p) {
  return p.cfg == 0 && p.epi == EPI_BIAS && p.n2_pad > 0 && p.n2_pad % SM_T == 0 && small_tiles() && small_form_has(p) &&
         (long)((p.M + SM_T - 1) / SM_T) * ((p.Npad + p.n2_pad) / SM_T) * 2 <= 7L * cu_count();
}

hipError_t bf16_gemm_init() {
  hipError_t e = set_attr_all<256, 512, 64>();
  if (e != hipSuccess) return e;
  if ((e = set_attr_all<256, 512, 64, 1>()) != hipSuccess) return e;
  if ((e = set_attr_all<256, 512, 64, 3>()) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16_persist_res<256>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<256, 512>())) != hipSuccess) return e;
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_bf16_persist_res<192>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<192, 512>())) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_BIAS, false>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_BIAS_GELU_ERF, false>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_BIAS_GELU_TANH, false>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_VT, false>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_BIAS, true>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_BIAS_GELU_ERF, true>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_BIAS_GELU_TANH, true>()) != hipSuccess) return e;
  if ((e = set_attr_persist<EPI_VT, true>()) != hipSuccess) return e;
  if ((e = set_attr_all<128, 512, 64>()) != hipSuccess) return e;
  if ((e = set_attr_all<128, 512, 64, 0, 128>()) != hipSuccess) return e;
  if ((e = set_attr_all<128, 512, 64, 2, 128>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_BIAS>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_BIAS_GELU_ERF>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_BIAS_GELU_TANH>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_BIAS_RESIDUAL>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_BIAS_POS>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_VT>()) != hipSuccess) return e;
  if ((e = set_attr_small<EPI_BIAS, true>()) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t bf16_gemm(const GemmParams& p, hipStream_t st) {
  if (p.K % (2 * BK) != 0 || p.Npad % 128 != 0 || p.N % 4 != 0) return hipErrorInvalidValue;
  if (p.stats && (p.n_part < 1 || p.n_part > STAT_REGS || p.stat_group < 1 || !p.colsum)) return hipErrorInvalidValue;
  // operands are addressed through 32-bit buffer offsets
  if ((long)p.M * p.lda * 2 >= (1L << 32) || (long)p.Npad * p.K * 2 >= (1L << 32) ||
      (p.R && (long)p.M * p.ldr * 4 >= (1L << 32)) || (p.C && !p.row_map && (long)p.M * p.ldc * 2 >= (1L << 32)))
    return hipErrorInvalidValue;
  const bool f32_out = p.epi == EPI_BIAS_RESIDUAL || p.epi == EPI_BIAS_POS;
  if (!f32_out && p.epi != EPI_VT && (p.N % 8 != 0 || p.ldc % 8 != 0)) return hipErrorInvalidValue;
  if (p.n2_pad > 0) return bf16_gemm_pair_fits(p) ? launch_small(p, st) : hipErrorInvalidValue;
  switch (p.cfg) {
    case 1: return dispatch<128, 512, 64>(p, st);
    case 2: return dispatch<128, 512, 64, 0, 128>(p, st);
    case 3: if (p.K % 256 == 0) return dispatch<128, 512, 64, 2, 128>(p, st); break;
    case 6: if (p.Npad % 256 == 0) return dispatch<256, 512, 64, 0>(p, st); break;
    case 7: if (p.Npad % 256 == 0) return dispatch<256, 512, 64, 1>(p, st); break;
    case 8: if (p.Npad % 256 == 0) return dispatch<256, 512, 64, 3>(p, st); break;
    case 9: if (p.Npad % 256 == 0 && p.epi != EPI_BIAS_RESIDUAL && p.epi != EPI_BIAS_POS) return dispatch_persist(p, st); break;
    case 10: if (p.Npad % 256 == 0 && p.epi == EPI_BIAS_RESIDUAL && !p.xb) return launch_persist_res(p, st); break;
    case 11: if (small_form_has(p)) return launch_small(p, st); break;
    case 12: if (p.N % 192 == 0 && p.epi == EPI_BIAS_RESIDUAL && !p.xb) return launch_persist_res<192>(p, st); break;
  }
  // One or two slices: 64 x 64 tiles while there are at most two of them per CU (measured against the
  // 128 x 128 tiles on 1024 and 2048 rows: ahead up to 512 tiles, behind from 1024 on).  Same bits.
  if (p.cfg == 0 && small_tiles() && small_form_has(p) &&
      (long)((p.M + SM_T - 1) / SM_T) * (p.Npad / SM_T) <= 2L * cu_count())
    return launch_small(p, st);
  // A width of 1152 is four and a half 256-wide tile columns and six 192-wide ones.  The residual product takes
  // 256 x 192 tiles when their rounds, at T192 of a 256 x 256 tile's time each, come to less: the 10-slice
  // SigLIP-shaped request (240 tiles in one round instead of 200: -8 % on both of its residual products), not a
  // micro-batch of 128 slices (12 rounds for 10).  Same bits.
  if (p.cfg == 0 && p.epi == EPI_BIAS_RESIDUAL && !p.xb && persist_res() && tiles_192() && p.N % 192 == 0 && p.N % 256 != 0) {
    const long cus = cu_count(), gm = (p.M + BM - 1) / BM;
    const long t256 = gm * ((p.N + 255) / 256), t192 = gm * (p.N / 192);
    constexpr double T192 = 0.92;   // measured: a 256 x 192 tile takes 0.92 of a 256 x 256 tile's time (more operand bytes per flop)
    if (t256 * 2 > cus && (double)((t192 + cus - 1) / cus) * T192 < (double)((t256 + cus - 1) / cus))
      return launch_persist_res<192>(p, st);
  }
  if (p.Npad % 256 != 0) return dispatch<128, 512, 64>(p, st);
  // A width like 3200 leaves the last 256-wide tile column half used.  When that column is also what
  // spills the launch into a nearly empty last round (at most a quarter of the CUs busy), the residual
  // product is cut by columns: the whole 256-wide tile columns, and the last 128 columns as a launch of
  // 128-wide tiles (weight rows, bias and residual columns are pointer offsets).  Same bits.  A 128-wide
  // tile takes about as long as a 256-wide one, so the cut pays only then: -4 % on the 6B shape's FC2,
  // +1 % on a SigLIP-shaped batch of 480 slices whose 2560 tiles are ten full rounds anyway.
  const long tiles_all = (long)((p.M + BM - 1) / BM) * (p.Npad / 256), cus = cu_count();
  if (p.cfg == 0 && p.epi == EPI_BIAS_RESIDUAL && p.N > 256 && p.N % 256 != 0 && p.N % 256 <= 128 &&
      tiles_all >= cus && tiles_all % cus != 0 && (tiles_all % cus) * 4 <= cus) {
    const int n_a = p.N / 256 * 256;
    GemmParams a = p, b = p;
    a.N = n_a; a.Npad = n_a;
    b.N = p.N - n_a; b.Npad = 128;
    b.W = p.W + (long)n_a * p.K; b.bias = p.bias + n_a; b.R = p.R + n_a;
    if (p.xb) { b.xb = p.xb + n_a; b.stats_out = p.stats_out + (n_a / STAT_GROUP) * 2; }   // n_a % 256 == 0
    const hipError_t e = bf16_gemm(a, st);
    return e != hipSuccess ? e : bf16_gemm(b, st);
  }
  // Small batches: when 256-wide tiles would leave half of the CUs without one, 128 x 128 tiles
  // quadruple the number of workgroups (two of them fit a CU) and shorten the one round there is.  Same
  // bits: a tile shape changes which lane holds an element, never the order in which its k-steps are
  // summed.  With at most one such tile per CU the launch is bound by the bytes it keeps in flight:
  // the loop with four register sets (loads four slabs ahead; K in whole groups of four slabs) takes
  // it.  (Measured and not kept: 256 x 128 tiles for this regime, 17 % slower on one slice; the
  // pipelined loop on them, 8 % slower still.)
  const long tiles256 = (long)((p.M + BM - 1) / BM) * (p.Npad / 256);
  if (tiles256 * 4 <= cu_count() && p.K % 256 == 0) return dispatch<128, 512, 64, 2, 128>(p, st);
  if (tiles256 * 2 <= cu_count()) return dispatch<128, 512, 64, 0, 128>(p, st);   // beyond that the small tiles lose (13 slices: +9 %)
  if (p.epi != EPI_BIAS_RESIDUAL && p.epi != EPI_BIAS_POS) {
    // A batch of a few rounds whose last round fills at most half of the CUs (the SigLIP-shaped request of
    // 10 slices: 360 tiles of its q/k projection = 1.4 rounds) is cut by rows like the long-K residual
    // products below: whole rounds on the persistent kernel, the remaining rows as one round of 256 x 128
    // tiles.  Same bits.  The plain loop of those tiles is slower per flop, so the cut pays only while the
    // last round is a large part of the launch.
    if (p.cfg == 0 && p.epi != EPI_VT && (!p.row_map || p.block_tokens > 0)) {
      const long cu = cu_count(), gn = p.Npad / 256, gm = (p.M + BM - 1) / BM;
      const long rounds = tiles256 / cu, rem = tiles256 % cu;
      const long rows_a = rounds * cu / gn;
      const long tiles_b = (gm - rows_a) * gn;
      if (rounds >= 1 && rounds <= 4 && rem > 0 && rows_a >= 1 && rows_a < gm && tiles_b * 2 <= cu &&
          (!p.row_map || (rows_a * BM) % p.block_tokens == 0)) {
        GemmParams a = p, b = p;
        a.M = (int)(rows_a * BM);
        b.M = p.M - a.M;
        b.A = p.A + (long)a.M * p.lda;
        if (p.stats) b.stats = p.stats + (long)a.M * p.n_part * 2;
        if (p.row_map) b.row_map = p.row_map + a.M / p.block_tokens;
        else b.C = p.C + (long)a.M * p.ldc;
        const hipError_t e = dispatch_persist(a, st);
        return e != hipSuccess ? e : dispatch<128, 512, 64>(b, st);
      }
    }
    return dispatch_persist(p, st);
  }
  // A last round that fills at most half of the CUs costs a whole tile time.  The residual product
  // (rows are independent, all addressing is by pointer) is cut by rows instead: whole rounds of
  // 256-wide tiles, then the remaining rows as one round of 128-wide tiles, half as long.  Same bits.
  // Measured: -4 % on the K = 12800 product of the 6B shape, -1 % at K = 4096, +2 % at K = 1024 (the
  // second launch costs more than the short tiles save; +0.6 % with the persistent kernel), hence the K limit.
  if (p.epi == EPI_BIAS_RESIDUAL && p.K >= 2048) {
    const long cu = cu_count(), gn = p.Npad / 256, gm = (p.M + BM - 1) / BM;
    const long rounds = tiles256 / cu, rem = tiles256 % cu;
    const long rows_a = rounds * cu / gn;                    // tile rows of the whole rounds
    const long tiles_b = (gm - rows_a) * gn;
    if (rounds >= 1 && rem > 0 && rows_a >= 1 && rows_a < gm && tiles_b * 2 <= cu) {
      GemmParams a = p, b = p;
      a.M = (int)(rows_a * BM);
      b.M = p.M - a.M;
      b.A = p.A + (long)a.M * p.lda;
      b.R = p.R + (long)a.M * p.ldr;
      if (p.xb) { b.xb = p.xb + (long)a.M * p.ldxb; b.stats_out = p.stats_out + (long)a.M * p.n_part_out * 2; }
      const hipError_t e = (persist_res() && !a.xb) ? launch_persist_res(a, st)
                           : a_direct() ? dispatch<256, 512, 64, 3>(a, st) : dispatch<256, 512, 64, 1>(a, st);   // K >= 2048 here
      return e != hipSuccess ? e : dispatch<128, 512, 64>(b, st);
    }
  }
  if (p.epi == EPI_BIAS_RESIDUAL && persist_res() && !p.xb) return launch_persist_res(p, st);
  return (a_direct() && p.K >= 2048) ? dispatch<256, 512, 64, 3>(p, st) : dispatch<256, 512, 64, 1>(p, st);
}

}  // namespace epd
