// Tile-local flash attention for gfx950 (bf16 MFMA, fp32 online softmax).
//
// One workgroup = 4 waves, each owning QT sub-tiles of 32 queries of one
// (slice, head).  Keys and values of the same slice stream through LDS in
// blocks of 64 keys (double buffered, one barrier per block); the online
// softmax advances in steps of 32 keys, software-pipelined so that the S^T
// MFMAs of step i+1 run under the exponentials of step i.  Everything is computed transposed so
// that a lane always owns ONE query per sub-tile:
//     S^T = K Q^T        (left operand: key rows from LDS, right: Q from registers)
//     O^T += V^T P^T     (left operand: V^T rows from LDS, right: P^T from the S^T registers)
// With the 32x32 MFMA result layout (register i of lane l = row
// 8*(i/4) + 4*(l/32) + i%4, column l%32) the softmax row statistics are
// per-lane scalars plus one exchange with lane l^32, and the exponentiated
// S^T registers are already a valid right operand for the second product:
// registers 8j..8j+7 of a lane hold keys {16j + 4h + 0..3, 16j + 8 + 4h + 0..3}
// (h = l/32).  The V^T block is stored in LDS with exactly that key order
// inside every group of 16 keys (positions [0-3, 8-11, 4-7, 12-15]), so the
// matching left operand is one 16-byte LDS read.  A K / V^T fragment read
// from LDS feeds all QT sub-tiles of the wave.
// Values arrive pre-transposed ([slice, head, hd, token]) from the value GEMM.
//
// The queries arrive carrying the logit scale: q = (1 / sqrt(hd)) log2(e) x (the projection that makes them has
// the factor folded into its weights), so the S^T registers are the logits in the log2 domain as they stand
// and the weights are exp2 of them with no arithmetic in between.
//
// The reference value m that is subtracted from a query's logits follows the
// running maximum lazily: it moves (and the accumulators are rescaled) only
// when a logit exceeds it by more than RESCALE_LOG2 in the log2 domain, which
// bounds the weights by 2^RESCALE_LOG2 instead of by 1: harmless for bf16
// weights and fp32 sums, and it takes the rescaling out of almost every step
// (with the exact running maximum some query of a wave moves it at most steps).
// The sum of the weights is taken over the rounded values the second product
// uses: two per v_dot2_f32_bf16, or, where the V^T tile has spare rows past
// the head dim (hd = 72 in 96 rows), by a row of ones in V^T, so that the sum
// comes out of the second product itself.  Where the sum is taken on the VALU
// the common step computes no maximum at all: a step whose weights sum to
// more than 2^RESCALE_LOG2 (or overflow) is what triggers the maximum, the
// move of the reference and a second round of exponentials.
#include <cstdlib>

#include "kernels.h"

namespace epd {

namespace {

constexpr int BKEY = 64;  // keys per LDS block
constexpr float RESCALE_LOG2 = 8.0f;   // a logit may exceed the reference by this much (log2 domain)
constexpr float RESCALE_SUM = 256.0f;  // 2^RESCALE_LOG2: what a lane's 16 weights of a step may sum to

// max of two values and the two held by lane ^ 32: the swap leaves the low half's values in both
// halves of one result and the high half's in both halves of the other
__device__ __forceinline__ float max_with_other_half(float x, float y) {
  const unsigned b = __float_as_uint(fmaxf(fmaxf(x, y), y));
  const auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  return fmaxf(fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])), __uint_as_float(b));
}

// HD = head dim as stored in q, k, v^T (a multiple of 8).  The products run
// over HD rounded up to the MFMA shapes (16 for q.k, 32 rows of O^T); the
// extra head-dim positions exist only in LDS and registers, as zeros.
template <int HD>
struct AttnSmem {
  static constexpr int HDK = (HD + 15) / 16 * 16;   // contraction length of S^T
  static constexpr int HDV = (HD + 31) / 32 * 32;   // rows of V^T / O^T
  static constexpr int K_LD = HDK + 8;     // bf16 elements per key row (16 B pad)
  static constexpr int V_LD = BKEY + 8;    // bf16 elements per V^T row
  static constexpr int K_ELEMS = BKEY * K_LD;
  static constexpr int V_ELEMS = HDV * V_LD;
  static constexpr size_t BYTES = (size_t)2 * (K_ELEMS + V_ELEMS) * sizeof(bf16_t);
};

// Registers: with the S^T product of step i + 1 issued ahead of the softmax of step i (two sets of S^T and
// weight registers) head dim 64 takes 140 registers, three workgroups per CU, head dims 72 / 96 three or two,
// 128 two; more waves hide the MFMA -> exp -> MFMA dependency chain better than fragment reuse saves LDS
// reads (two sub-tiles per wave at two workgroups per CU measured slower).
// MASK: the slices carry rows past n_keys (compiled apart: the unmasked kernel keeps its registers and
// its step free of the key-index compare).
// W4: four workgroups per CU (head dim 64, where 128 registers and 37 KiB of LDS per workgroup allow it).  One
// step's S^T registers and weights only, no step issued ahead: 118 registers, and the fourth wave of a SIMD
// covers what the look-ahead covered (-10 % on 104 slices of 1024 tokens, same bits).
template <int HD, int QT, bool MASK, bool W4 = false>
__global__ __launch_bounds__(256, W4 ? 4 : (HD == 64 ? 3 : 2)) void k_attention_bf16(const bf16_t* __restrict__ q,
                                                        const bf16_t* __restrict__ k,
                                                        const bf16_t* __restrict__ vt,
                                                        bf16_t* __restrict__ o, int n_tok, int n_keys, int n_q,
                                                        int q_shared, int heads, int n_pairs, long ld_qk,
                                                        long ld_o, unsigned char* __restrict__ oq,
                                                        unsigned* __restrict__ so, long ld_so) {
  using SM = AttnSmem<HD>;
  constexpr int BQ = 128 * QT;  // queries per workgroup
  constexpr int KS = SM::HDK / 16;   // k-steps of the S^T product
  constexpr int MB = SM::HDV / 32;   // 32-row blocks of O^T
  constexpr int KCH = HD / 8;        // 16-byte chunks per key row in memory
  constexpr int K_TOTAL = BKEY * KCH, V_TOTAL = HD * (BKEY / 8);   // chunks per block
  constexpr int K_LOADS = (K_TOTAL + 255) / 256;
  constexpr int V_LOADS = (V_TOTAL + 255) / 256;
  constexpr bool K_EXACT = K_TOTAL % 256 == 0, V_EXACT = V_TOTAL % 256 == 0;
  // KDMA (four-workgroup form at head dim 64): key blocks go from global memory straight into LDS (no staging
  // registers, no LDS stores by the waves).  A key row is then exactly 128 bytes, rows unpadded, the 16-byte chunks of
  // a row XOR-swizzled by (row >> 1) & 7 like the GEMM's operand slabs (the hardware puts lane l's 16 bytes at a
  // wave-uniform base + 16 l, so the swizzle is applied on the global side).
  constexpr bool KDMA = W4 && HD == 64;
  constexpr int K_ROW = KDMA ? 64 : SM::K_LD;   // bf16 elements per key row in LDS

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* sK = reinterpret_cast<bf16_t*>(smem);       // [2][BKEY][K_LD]
  bf16_t* sV = sK + 2 * SM::K_ELEMS;                  // [2][HD][V_LD]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  // Workgroups are dealt round-robin to the 8 XCDs: keep the q-blocks of one
  // (slice, head) on one XCD so that its K / V^T block is fetched into one L2.
  const int n_qb = (n_q + BQ - 1) / BQ;
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int pair = (seq / n_qb) * 8 + xcd;          // (slice, head) index
  if (pair >= n_pairs) return;                      // whole workgroup leaves before any barrier
  const int qb = seq % n_qb, h = pair % heads, t = pair / heads;
  const long row0 = (long)t * n_tok;
  const int q0 = qb * BQ + wave * 32 * QT;
  // n_tok is a multiple of 64: a 32-query sub-tile is all in or all out (rows past n_keys are computed like
  // any other and never used)
  bool act[QT];
  bool any_act = false;
#pragma unroll
  for (int u = 0; u < QT; ++u) { act[u] = q0 + u * 32 < n_q; any_act = any_act || act[u]; }
  const long q_row0 = q_shared ? 0 : row0;   // learned queries: the same rows for every slice

  const bf16_t* kbase = k + row0 * ld_qk + (long)h * HD;
  const bf16_t* vbase = vt + ((long)t * heads + h) * HD * (long)n_tok;

  // Q fragments: lane = query, 8 consecutive head-dim elements per k-step
  bf16x8 qf[QT][KS];
#pragma unroll
  for (int u = 0; u < QT; ++u) {
    const int qrow = act[u] ? q0 + u * 32 + l32 : 0;  // inactive sub-tiles read a valid row, result unused
    const bf16_t* qp = q + (q_row0 + qrow) * ld_qk + (long)h * HD + lh * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s * 16 + 8 < HD || lh == 0) {
        qf[u][s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
      } else {   // head-dim positions past HD (last k-step of a head dim that is not a multiple of 16)
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[u][s][e] = (bf16_t)0.f;
      }
    }
  }

  // A thread's chunks keep their place inside every key block: 32-bit byte offsets once, the
  // block's base stays in scalar registers.
  u32x4 rk[KDMA ? 1 : K_LOADS], rv[V_LOADS];
  unsigned koff[K_LOADS], voff[V_LOADS];
#pragma unroll
  for (int i = 0; i < K_LOADS; ++i) {
    int c = tid + 256 * i;
    if (!K_EXACT) c = c < K_TOTAL ? c : 0;   // spare threads of the last round re-read chunk 0, never stored
    koff[i] = (unsigned)(((long)(c / KCH) * ld_qk + (c % KCH) * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < V_LOADS; ++i) {
    int c = tid + 256 * i;
    if (!V_EXACT) c = c < V_TOTAL ? c : 0;
    voff[i] = (unsigned)(((long)(c / (BKEY / 8)) * n_tok + (c % (BKEY / 8)) * 8) * 2);
  }
  auto gload = [&](int kb) {
    const char* kblk = reinterpret_cast<const char*>(kbase + (long)kb * BKEY * ld_qk);
    const char* vblk = reinterpret_cast<const char*>(vbase + (long)kb * BKEY);
    if constexpr (!KDMA) {
#pragma unroll
      for (int i = 0; i < K_LOADS; ++i) rk[i] = *reinterpret_cast<const u32x4*>(kblk + koff[i]);
    }
#pragma unroll
    for (int i = 0; i < V_LOADS; ++i) rv[i] = *reinterpret_cast<const u32x4*>(vblk + voff[i]);
  };
  // key block kb -> LDS buffer buf, two instructions of 32 rows each; lane = (row within 8, physical chunk)
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int kd_row = wave * 8 + (lane >> 3);
  const unsigned kd_voff = (unsigned)((kd_row * ld_qk + (((lane & 7) ^ ((kd_row >> 1) & 7)) * 8)) * 2);
  auto kdma = [&](int buf, int kb) {
    if constexpr (KDMA) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const bf16_t* g = kbase + ((long)kb * BKEY + 32 * i) * ld_qk;   // uniform
        bf16_t* l = sK + buf * SM::K_ELEMS + (32 * i + wave_u * 8) * K_ROW;
        const unsigned lds_addr = (unsigned)(size_t)(__attribute__((address_space(3))) void*)l;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :: "v"(kd_voff), "s"(g), "s"(lds_addr) : "memory", "m0");
      }
    }
  };
  auto kdma_wait = [&]() {
    if constexpr (KDMA) __builtin_amdgcn_s_waitcnt(0 | (0x7 << 4) | (0xf << 8));   // vmcnt(0): this thread's part has landed
  };
  // kb: the key block the staged registers hold
  auto sstore = [&](int buf, int kb) {
    if constexpr (!KDMA) {
#pragma unroll
      for (int i = 0; i < K_LOADS; ++i) {
        const int c = tid + 256 * i;
        if (!K_EXACT && c >= K_TOTAL) continue;
        const int row = c / KCH, ch = c % KCH;
        *reinterpret_cast<u32x4*>(sK + buf * SM::K_ELEMS + row * SM::K_LD + ch * 8) = rk[i];
      }
    }
#pragma unroll
    for (int i = 0; i < V_LOADS; ++i) {
      const int c = tid + 256 * i;
      if (!V_EXACT && c >= V_TOTAL) continue;
      const int row = c / (BKEY / 8), ch = c % (BKEY / 8);
      // chunk ch holds keys 8ch..8ch+7; inside a group of 16 keys the LDS order is
      // [0-3, 8-11, 4-7, 12-15]: keys 8ch+0..3 -> position 16(ch/2) + 4(ch%2),
      // keys 8ch+4..7 -> position 16(ch/2) + 8 + 4(ch%2)
      bf16_t* dst = sV + buf * SM::V_ELEMS + row * SM::V_LD + (ch >> 1) * 16 + (ch & 1) * 4;
      if (MASK && (kb + 1) * BKEY > n_keys) {   // uniform: only the last block(s) of a slice whose rows are padded
        // Values of keys past n_keys are no part of the slice (the next slice's, or whatever an earlier call
        // left in the workspace): their weights are exactly zero, but 0 * NaN or 0 * Inf would still poison
        // the sum, so they are cleared on the way into LDS.  Word j of the chunk holds keys key0 + 2j, + 2j + 1.
        const int key0 = kb * BKEY + ch * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          rv[i][j] &= (key0 + 2 * j < n_keys ? 0x0000ffffu : 0u) | (key0 + 2 * j + 1 < n_keys ? 0xffff0000u : 0u);
      }
      u32x2 lo = {rv[i][0], rv[i][1]}, hi = {rv[i][2], rv[i][3]};
      *reinterpret_cast<u32x2*>(dst) = lo;
      *reinterpret_cast<u32x2*>(dst + 8) = hi;
    }
  };

  constexpr bool SUM_MFMA = SM::HDV > HD;   // a spare V^T row of ones makes the second product sum the weights
  constexpr int SUM_B = HD / 32, SUM_I = 4 * ((HD % 32) / 8);   // O^T row HD: block, register (lanes 0..31; HD % 8 == 0)
  f32x16 oacc[QT][MB];
  // m_ref: the reference subtracted from this query's logits (log2 domain);
  // l_run: this lane's share of the running sum of weights (unused with SUM_MFMA)
  float m_ref[QT], l_run[QT];
  // Wave-uniform: some query of the wave has a reference other than 0.  While it is false (the common case:
  // logits of a few units) the exponentials are taken of the S^T registers as they are.
  bool shifted = false;
#pragma unroll
  for (int u = 0; u < QT; ++u) {
    m_ref[u] = 0.f;
    l_run[u] = 0.f;
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[u][b][e] = 0.f;
  }

  // S^T of one 32-key step for all sub-tiles (MFMAs only: they run while the
  // wave goes on with the softmax arithmetic of the previous step)
  auto issue_s = [&](f32x16 (&s)[QT], const bf16_t* ks, int kt) {
#pragma unroll
    for (int u = 0; u < QT; ++u)
#pragma unroll
      for (int e = 0; e < 16; ++e) s[u][e] = 0.f;
    if constexpr (KDMA) {
      // all fragments of the step first, then the products: the LDS latency is paid once per step (the registers
      // the staged key block has left make room for the second pair)
      bf16x8 kf[KS];
#pragma unroll
      for (int st = 0; st < KS; ++st)
        kf[st] = *reinterpret_cast<const bf16x8*>(ks + (kt * 32 + l32) * K_ROW + (((2 * st + lh) ^ ((l32 >> 1) & 7)) * 8));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int st = 0; st < KS; ++st)
#pragma unroll
        for (int u = 0; u < QT; ++u) s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st], qf[u][st], s[u], 0, 0, 0);
      return;
    }
#pragma unroll
    for (int st = 0; st < KS; ++st) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + (kt * 32 + l32) * SM::K_LD + st * 16 + lh * 8);
#pragma unroll
      for (int u = 0; u < QT; ++u) s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[u][st], s[u], 0, 0, 0);
    }
  };
  // weights of one step from its shifted logits, and (unless the second product sums them) their
  // sum over the rounded values that product uses, two per instruction
  auto weights = [&](const f32x16& sv, bf16x8 (&pv)[2], float& psum) {
#pragma unroll
    for (int e = 0; e < 16; ++e) pv[e >> 3][e & 7] = (bf16_t)__builtin_amdgcn_exp2f(sv[e]);
    psum = 0.f;
    if (!SUM_MFMA) {
      const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv[j], pv[j], 0, 1), ones, psum, false);
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv[j], pv[j], 2, 3), ones, psum, false);
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv[j], pv[j], 4, 5), ones, psum, false);
        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv[j], pv[j], 6, 7), ones, psum, false);
      }
    }
  };
  // Online softmax of one step, one query per lane (shared with lane ^ 32).  `force`: the first
  // step of a slice takes its own maximum as the reference, whatever its size.
  auto softmax = [&](f32x16 (&s)[QT], bf16x8 (&pf)[QT][2], int key0, bool force) {
#pragma unroll
    for (int u = 0; u < QT; ++u) {
      if (MASK && key0 + 32 > n_keys) {   // uniform; only the last steps of a slice whose rows are padded
        // rows past n_keys are no tokens: logit -inf, weight 0 (the first step always holds a real key,
        // so the reference is finite by the time a step is masked entirely)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (key0 + 8 * (e >> 2) + 4 * lh + (e & 3) >= n_keys) s[u][e] = -INFINITY;
      }
      // logits relative to the reference as it stands (log2 domain already: q carries the scale)
      if (shifted) {
#pragma unroll
        for (int e = 0; e < 16; ++e) s[u][e] -= m_ref[u];
      }
      float psum = 0.f;
      bool move;
      if (!SUM_MFMA) {
        // No maximum in the common step: the weights are taken against the reference as it stands and
        // their sum tells whether one of them was too large (a logit above RESCALE_LOG2 alone makes the
        // sum exceed 2^RESCALE_LOG2; an overflowed weight makes it infinite).
        weights(s[u], pf[u], psum);
        move = force || __builtin_amdgcn_ballot_w64(!(psum <= RESCALE_SUM)) != 0;
      } else {
        move = true;   // the sum sits in the accumulator of the second product: decide by the maximum
      }
      if (move) {
        // three-input maxima throughout (the two-input form would first quieten its inputs)
        float mx = fmaxf(fmaxf(s[u][0], s[u][1]), s[u][2]);
#pragma unroll
        for (int e = 3; e < 15; e += 2) mx = fmaxf(fmaxf(mx, s[u][e]), s[u][e + 1]);
        mx = max_with_other_half(mx, s[u][15]);
        // Whether THIS query's reference moves depends on its own logits only (the move is entered when any
        // query of the wave asks for it): a query's bits must not depend on which other queries share its
        // wave, which in slices whose rows are padded can be rows of the next slice.
        bool mine;
        if (!SUM_MFMA) {
          const float t = (force || !(psum <= RESCALE_SUM)) ? 1.0f : 0.f;   // this lane's half of the query's keys
          mine = max_with_other_half(t, t) > 0.f;
        } else {
          mine = force || mx > RESCALE_LOG2;
        }
        if (!SUM_MFMA || force || __builtin_amdgcn_ballot_w64(mx > RESCALE_LOG2) != 0) {
          // this query's reference moves by d: to the step's maximum (a sum above 2^RESCALE_LOG2 over 16 weights
          // means a logit above RESCALE_LOG2 - 4).  First step: unless that maximum is within a few units of 0
          // already (then the reference stays 0 and the step's weights stay below 2^4 each)
          const float d = !mine ? 0.f : (force ? (fabsf(mx) > 4.0f ? mx : 0.f) : mx);
          shifted = shifted || __builtin_amdgcn_ballot_w64(d != 0.f) != 0;
          // nothing has been accumulated before the first step (and the factor would overflow for a
          // first maximum below -127)
          const float alpha = force ? 1.0f : __builtin_amdgcn_exp2f(-d);
          l_run[u] *= alpha;
#pragma unroll
          for (int b = 0; b < MB; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[u][b][e] *= alpha;
#pragma unroll
          for (int e = 0; e < 16; ++e) s[u][e] -= d;
          m_ref[u] += d;
          if (!SUM_MFMA) weights(s[u], pf[u], psum);   // again, against the new reference
        }
      }
      if (SUM_MFMA) weights(s[u], pf[u], psum);
      else l_run[u] += psum;
    }
  };
  // O^T += V^T P^T for one step
  auto issue_pv = [&](bf16x8 (&pf)[QT][2], const bf16_t* vs, int kt) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int b = 0; b < MB; ++b) {
        const bf16x8 vf =
            *reinterpret_cast<const bf16x8*>(vs + (b * 32 + l32) * SM::V_LD + kt * 32 + j * 16 + lh * 8);
#pragma unroll
        for (int u = 0; u < QT; ++u)
          oacc[u][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u][j], oacc[u][b], 0, 0, 0);
      }
  };

  const int NB = (n_tok + BKEY - 1) / BKEY;   // a last block may reach past the slice: those keys are masked
  gload(0);
  // head-dim positions that exist only in LDS stay zero for the whole kernel:
  // columns HD .. HDK-1 of every key row, rows HD .. HDV-1 of V^T, both buffers
  if constexpr (SM::HDK > HD) {
    for (int r = tid; r < 2 * BKEY; r += 256) {
      bf16_t* dst = sK + (r / BKEY) * SM::K_ELEMS + (r % BKEY) * SM::K_LD + HD;
#pragma unroll
      for (int e = 0; e < SM::HDK - HD; ++e) dst[e] = (bf16_t)0.f;
    }
  }
  if constexpr (SM::HDV > HD) {
    constexpr int PAD_ELEMS = (SM::HDV - HD) * SM::V_LD;
    for (int e = tid; e < 2 * PAD_ELEMS; e += 256)
      sV[(e / PAD_ELEMS) * SM::V_ELEMS + HD * SM::V_LD + e % PAD_ELEMS] =
          (bf16_t)(e % PAD_ELEMS < SM::V_LD ? 1.0f : 0.f);   // row HD: ones (sums the weights), the rest zero
  }
  kdma(0, 0);
  sstore(0, 0);
  kdma_wait();
  __syncthreads();

  // Software pipeline over the 32-key steps: the S^T MFMAs of the next step
  // are in flight while the VALU does the softmax of the current one.  s0 of a
  // block is issued right after the barrier that published the block.
  if constexpr (W4) {
    f32x16 s0[QT];
    bf16x8 p0[QT][2];
    for (int kb = 0; kb < NB; ++kb) {
      kdma((kb + 1) & 1, kb + 1 < NB ? kb + 1 : kb);   // the other buffer: nobody reads it after the previous barrier
      gload(kb + 1 < NB ? kb + 1 : kb);
      const bf16_t* ks = sK + (kb & 1) * SM::K_ELEMS;
      const bf16_t* vs = sV + (kb & 1) * SM::V_ELEMS;
      if (any_act) {
        issue_s(s0, ks, 0);
        softmax(s0, p0, kb * BKEY, kb == 0);
        // a step whose keys all lie past n_keys (the second half of a padded slice's last block) has weights of
        // exactly zero: left out, same bits
        const bool second = !MASK || kb * BKEY + 32 < n_keys;   // uniform
        if (second) issue_s(s0, ks, 1);   // the weights of step 0 are out of the S^T registers: step 1's product starts
        issue_pv(p0, vs, 0);              // under the second product of step 0
        if (second) {
          softmax(s0, p0, kb * BKEY + 32, false);
          issue_pv(p0, vs, 1);
        }
      }
      sstore((kb + 1) & 1, kb + 1 < NB ? kb + 1 : kb);
      kdma_wait();
      __syncthreads();
    }
  } else {
  f32x16 s0[QT], s1[QT];
  bf16x8 p0[QT][2], p1[QT][2];
  if (any_act) issue_s(s0, sK, 0);
  for (int kb = 0; kb < NB; ++kb) {
    gload(kb + 1 < NB ? kb + 1 : kb);  // unconditional: staging registers stay out of control flow
    const bf16_t* ks = sK + (kb & 1) * SM::K_ELEMS;
    const bf16_t* vs = sV + (kb & 1) * SM::V_ELEMS;
    if (any_act) {
      issue_s(s1, ks, 1);
      softmax(s0, p0, kb * BKEY, kb == 0);
      issue_pv(p0, vs, 0);
      softmax(s1, p1, kb * BKEY + 32, false);
      issue_pv(p1, vs, 1);
    }
    sstore((kb + 1) & 1, kb + 1 < NB ? kb + 1 : kb);   // the other buffer: nobody reads it after the previous barrier
    __syncthreads();
    if (any_act && kb + 1 < NB) issue_s(s0, sK + ((kb + 1) & 1) * SM::K_ELEMS, 0);
  }

  }
#pragma unroll
  for (int u = 0; u < QT; ++u) {
    if (!act[u] || q0 + u * 32 + l32 >= n_q) continue;   // a shared query set need not fill its last 32 rows
    // SUM_MFMA: row HD of O^T holds the sum, in lanes 0..31 (query = lane)
    const float l_tot = SUM_MFMA ? __shfl(oacc[u][SUM_B < MB ? SUM_B : 0][SUM_I], l32, 64)
                                 : l_run[u] + __shfl_xor(l_run[u], 32, 64);
    const float inv = 1.0f / l_tot;
    if constexpr (HD % 32 == 0) {
      if (oq) {
        // MXFP8 output (the out-projection's operand): block b of this head = the 32 head-dim rows of O^T block b,
        // 16 in this lane and 16 in lane ^ 32 (register group gi -> rows 8 gi + 4 lh .. + 3), so the block's
        // largest magnitude is one exchange away; codes [row][ld_o bytes], scale words [column / 128][ld_so].
        const long row = (long)t * n_q + q0 + u * 32 + l32;
#pragma unroll
        for (int b = 0; b < MB; ++b) {
          float v[16];
          float amax = 0.f;
#pragma unroll
          for (int e = 0; e < 16; ++e) { v[e] = oacc[u][b][e] * inv; amax = fmaxf(amax, fabsf(v[e])); }
          amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
          const unsigned byte = mx_scale_byte(amax);
          const float sc = mx_inv_scale(byte);
          const int col0 = h * HD + b * 32;
#pragma unroll
          for (int gi = 0; gi < 4; ++gi)
            *reinterpret_cast<unsigned*>(oq + row * ld_o + col0 + gi * 8 + lh * 4) =
                mx_pack4(v[gi * 4] * sc, v[gi * 4 + 1] * sc, v[gi * 4 + 2] * sc, v[gi * 4 + 3] * sc);
          if (lh == 0) reinterpret_cast<unsigned char*>(so + (long)(col0 >> 7) * ld_so + row)[(col0 >> 5) & 3] = (unsigned char)byte;
        }
        continue;
      }
    }
    bf16_t* op = o + ((long)t * n_q + q0 + u * 32 + l32) * ld_o + (long)h * HD;
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
      for (int gi = 0; gi < 4; ++gi) {
        const int d0 = b * 32 + gi * 8 + lh * 4;
        if (SM::HDV > HD && d0 >= HD) continue;   // rows of O^T past the head dim
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[u][b][gi * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(op + d0) = ov;
      }
  }
}

template <int HD, int QT, bool MASK, bool W4 = false>
hipError_t launch_attn_m(const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* o, int n_slices,
                         int n_tok, int n_keys, int n_q, int q_shared, int heads, long ld_qk, long ld_o,
                         unsigned char* oq, unsigned* so, long ld_so, hipStream_t st) {
  // once per instantiation; the initialisation of a function-local static is safe against concurrent callers
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attention_bf16<HD, QT, MASK, W4>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     (int)AttnSmem<HD>::BYTES);
  if (attr != hipSuccess) return attr;
  constexpr int BQ = 128 * QT;
  const int n_qb = (n_q + BQ - 1) / BQ, n_pairs = n_slices * heads;
  const long n_wg = (long)((n_pairs + 7) / 8) * 8 * n_qb;
  if (n_wg > 0x7fffffffL) return hipErrorInvalidValue;
  k_attention_bf16<HD, QT, MASK, W4><<<dim3((unsigned)n_wg), dim3(256), AttnSmem<HD>::BYTES, st>>>(
      q, k, vt, o, n_tok, n_keys, n_q, q_shared, heads, n_pairs, ld_qk, ld_o, oq, so, ld_so);
  return hipGetLastError();
}

template <int HD, int QT>
hipError_t launch_attn(const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* o, int n_slices,
                       int n_tok, int n_keys, int n_q, int q_shared, int heads, long ld_qk, long ld_o,
                       unsigned char* oq, unsigned* so, long ld_so, hipStream_t st) {
  // head dim 64: the four-workgroup form (EPD_ATTN_W4=0: the three-workgroup form with a step issued ahead, which it
  // was measured against: 660 -> 638 us on 104 slices of 1024 tokens, 16 heads; same bits)
  static const bool w4 = !(getenv("EPD_ATTN_W4") && getenv("EPD_ATTN_W4")[0] == '0');
  if (HD == 64 && w4)
    return (n_keys < n_tok || n_tok % BKEY != 0)
               ? launch_attn_m<HD, QT, true, HD == 64>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st)
               : launch_attn_m<HD, QT, false, HD == 64>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st);
  return (n_keys < n_tok || n_tok % BKEY != 0)
             ? launch_attn_m<HD, QT, true>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st)
             : launch_attn_m<HD, QT, false>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st);
}

}  // namespace

hipError_t bf16_attention(const bf16_t* q, const bf16_t* k, const bf16_t* vt, bf16_t* o, int n_slices,
                          int n_tok, int n_keys, int n_q, int q_shared, int heads, int hd_pad, long ld_qk,
                          long ld_o, hipStream_t st, unsigned char* oq, unsigned* so, long ld_so) {
  if (n_slices == 0) return hipSuccess;
  // MXFP8 output: whole blocks of 32 per head only, rows of at least heads * hd_pad bytes, 4-byte pieces
  if (oq && (hd_pad % 32 != 0 || !so || ld_o % 4 != 0 || ld_o < (long)heads * hd_pad || ld_so < (long)n_slices * n_q)) return hipErrorInvalidValue;
  // n_tok % 8: V^T rows are read in 16-byte chunks.  A slice whose rows are no multiple of the key block is
  // read up to 63 rows (q, k) / 63 elements (v^T) past its end: the caller's buffers must reach that far.
  if (n_tok % 8 != 0 || n_tok <= 0 || n_keys < 1 || n_keys > n_tok || n_q < 1) return hipErrorInvalidValue;
  if (!q_shared && n_q != n_tok) return hipErrorInvalidValue;   // a slice's own rows: one query per row
  switch (hd_pad) {
    case 64: return launch_attn<64, 1>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st);
    case 72: return launch_attn<72, 1>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st);
    case 96: return launch_attn<96, 1>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st);
    case 128: return launch_attn<128, 1>(q, k, vt, o, n_slices, n_tok, n_keys, n_q, q_shared, heads, ld_qk, ld_o, oq, so, ld_so, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace epd
