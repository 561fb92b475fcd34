// Tile-local flash attention for gfx950 (bf16 MFMA, fp32 online softmax).
//
// One workgroup = 128 queries of one (slice, head); 4 waves x 32 queries.
// Keys and values of the same slice stream through LDS in blocks of 64 keys
// (double buffered, one barrier per block).  Everything is computed
// transposed so that a lane always owns ONE query:
//     S^T = K Q^T        (left operand: key rows from LDS, right: Q from registers)
//     O^T += V^T P^T     (left operand: V^T rows from LDS, right: P^T from the S^T registers)
// With the 32x32 MFMA result layout (register i of lane l = row
// 8*(i/4) + 4*(l/32) + i%4, column l%32) the softmax row statistics are
// per-lane scalars plus one exchange with lane l^32, and the exponentiated
// S^T registers are already a valid right operand for the second product:
// registers 8j..8j+7 of a lane hold keys {16j + 4h + 0..3, 16j + 8 + 4h + 0..3}
// (h = l/32); the V^T fragment is read from LDS in the same key order.
// Values arrive pre-transposed ([slice, head, hd, token]) from the QKV GEMM.
#include "kernels.h"

namespace epd {

namespace {

constexpr int BQ = 128;   // queries per workgroup
constexpr int BKEY = 64;  // keys per LDS block

template <int HD>
struct AttnSmem {
  static constexpr int K_LD = HD + 8;      // bf16 elements per key row (16 B pad)
  static constexpr int V_LD = BKEY + 8;    // bf16 elements per V^T row
  static constexpr int K_ELEMS = BKEY * K_LD;
  static constexpr int V_ELEMS = HD * V_LD;
  static constexpr size_t BYTES = (size_t)2 * (K_ELEMS + V_ELEMS) * sizeof(bf16_t);
};

template <int HD>
__global__ __launch_bounds__(256) void k_attention_bf16(const bf16_t* __restrict__ q,
                                                        const bf16_t* __restrict__ k,
                                                        const bf16_t* __restrict__ vt,
                                                        bf16_t* __restrict__ o, int n_tok, int heads,
                                                        long ld_qk, long ld_o, float scale_log2e) {
  using SM = AttnSmem<HD>;
  constexpr int KS = HD / 16;   // k-steps of the S^T product
  constexpr int MB = HD / 32;   // 32-row blocks of O^T
  constexpr int KCH = HD / 8;   // 16-byte chunks per key row
  constexpr int K_LOADS = BKEY * KCH / 256;
  constexpr int V_LOADS = HD * (BKEY / 8) / 256;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem);       // [2][BKEY][K_LD]
  bf16_t* sV = sK + 2 * SM::K_ELEMS;                  // [2][HD][V_LD]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int qb = blockIdx.x, h = blockIdx.y, t = blockIdx.z;
  const long row0 = (long)t * n_tok;
  const int q0 = qb * BQ + wave * 32;
  const bool active = q0 < n_tok;   // n_tok is a multiple of 64, so a wave is all in or all out

  const bf16_t* kbase = k + row0 * ld_qk + (long)h * HD;
  const bf16_t* vbase = vt + ((long)t * heads + h) * HD * (long)n_tok;

  // Q fragments: lane = query, 8 consecutive head-dim elements per k-step
  bf16x8 qf[KS];
  if (active) {
    const bf16_t* qp = q + (row0 + q0 + l32) * ld_qk + (long)h * HD + lh * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
  } else {
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[s][e] = (bf16_t)0.f;
  }

  u32x4 rk[K_LOADS], rv[V_LOADS];
  auto gload = [&](int kb) {
#pragma unroll
    for (int i = 0; i < K_LOADS; ++i) {
      const int c = tid + 256 * i;
      const int row = c / KCH, ch = c % KCH;
      rk[i] = *reinterpret_cast<const u32x4*>(kbase + (long)(kb * BKEY + row) * ld_qk + ch * 8);
    }
#pragma unroll
    for (int i = 0; i < V_LOADS; ++i) {
      const int c = tid + 256 * i;
      const int row = c / (BKEY / 8), ch = c % (BKEY / 8);
      rv[i] = *reinterpret_cast<const u32x4*>(vbase + (long)row * n_tok + kb * BKEY + ch * 8);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < K_LOADS; ++i) {
      const int c = tid + 256 * i;
      const int row = c / KCH, ch = c % KCH;
      *reinterpret_cast<u32x4*>(sK + buf * SM::K_ELEMS + row * SM::K_LD + ch * 8) = rk[i];
    }
#pragma unroll
    for (int i = 0; i < V_LOADS; ++i) {
      const int c = tid + 256 * i;
      const int row = c / (BKEY / 8), ch = c % (BKEY / 8);
      *reinterpret_cast<u32x4*>(sV + buf * SM::V_ELEMS + row * SM::V_LD + ch * 8) = rv[i];
    }
  };

  f32x16 oacc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[b][e] = 0.f;
  float m_run = -INFINITY;  // running max of the scaled logits (log2 domain)
  float l_run = 0.f;        // this lane's share of the running sum

  const int NB = n_tok / BKEY;
  gload(0);
  sstore(0);
  __syncthreads();

  for (int kb = 0; kb < NB; ++kb) {
    gload(kb + 1 < NB ? kb + 1 : kb);  // unconditional: staging registers stay out of control flow
    if (active) {
      const bf16_t* ks = sK + (kb & 1) * SM::K_ELEMS;
      const bf16_t* vs = sV + (kb & 1) * SM::V_ELEMS;
      // S^T for the two 32-key halves of the block
      f32x16 s[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[kt][e] = 0.f;
#pragma unroll
        for (int st = 0; st < KS; ++st) {
          const bf16x8 kf =
              *reinterpret_cast<const bf16x8*>(ks + (kt * 32 + l32) * SM::K_LD + st * 16 + lh * 8);
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kt], 0, 0, 0);
        }
      }
      // online softmax, one query per lane (shared with lane ^ 32)
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kt][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx * scale_log2e);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      float psum = 0.f;
      bf16x8 pf[2][2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float pe = __builtin_amdgcn_exp2f(fmaf(s[kt][e], scale_log2e, -m_new));
          psum += pe;
          pf[kt][e >> 3][e & 7] = (bf16_t)pe;
        }
      l_run = l_run * alpha + psum;
#pragma unroll
      for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[b][e] *= alpha;
      // O^T += V^T P^T
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int key = kt * 32 + j * 16 + lh * 4;
#pragma unroll
          for (int b = 0; b < MB; ++b) {
            const bf16_t* vp = vs + (b * 32 + l32) * SM::V_LD + key;
            const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vp);
            const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vp + 8);
            bf16x8 vf;
#pragma unroll
            for (int e = 0; e < 4; ++e) { vf[e] = lo[e]; vf[4 + e] = hi[e]; }
            oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kt][j], oacc[b], 0, 0, 0);
          }
        }
    }
    sstore((kb + 1) & 1);
    __syncthreads();
  }

  if (!active) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l_tot;
  bf16_t* op = o + (row0 + q0 + l32) * ld_o + (long)h * HD;
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
      bf16x4 ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[b][gi * 4 + e] * inv);
      *reinterpret_cast<bf16x4*>(op + b * 32 + gi * 8 + lh * 4) = ov;
    }
}

template <int HD>
hipError_t launch_attn(const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* o, int n_slices,
                       int n_tok, int heads, long ld_qk, long ld_o, float scale, hipStream_t st) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attention_bf16<HD>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)AttnSmem<HD>::BYTES);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid((n_tok + BQ - 1) / BQ, heads, n_slices);
  k_attention_bf16<HD><<<grid, dim3(256), AttnSmem<HD>::BYTES, st>>>(
      q, k, vt, o, n_tok, heads, ld_qk, ld_o, scale * 1.4426950408889634f);
  return hipGetLastError();
}

}  // namespace

hipError_t bf16_attention(const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* o, int n_slices,
                          int n_tok, int heads, int hd_pad, long ld_qk, long ld_o, float scale,
                          hipStream_t st) {
  if (n_slices == 0) return hipSuccess;
  if (n_tok % BKEY != 0 || n_tok <= 0) return hipErrorInvalidValue;
  switch (hd_pad) {
    case 64: return launch_attn<64>(q, k, vt, o, n_slices, n_tok, heads, ld_qk, ld_o, scale, st);
    case 96: return launch_attn<96>(q, k, vt, o, n_slices, n_tok, heads, ld_qk, ld_o, scale, st);
    case 128: return launch_attn<128>(q, k, vt, o, n_slices, n_tok, heads, ld_qk, ld_o, scale, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace epd
