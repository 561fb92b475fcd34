// C boundary of the encode-stage library: validation, weight packing,
// workspace, and the per-micro-batch launch sequence.  See include/epd_encode.h.
#include "../../include/epd_encode.h"
#include "../../include/epd_encode_test.h"

#include <cstdarg>
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <cmath>
#include <vector>

#include "kernels.h"
#include "mm_cache.h"

using namespace epd;

namespace {

thread_local char g_err[512] = "";

void set_err(char* buf, size_t len, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, len, fmt, ap);
  va_end(ap);
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

// N padding of a weight matrix: the 256-wide block tile is the faster one
// even when it pads (measured: 1152 -> 1280 and 3200 -> 3328 columns both beat
// the 128-wide tile in algorithmic flop/s), so only narrow products use 128.
inline int pad_n(int n) { return n > 128 ? round_up(n, 256) : round_up(n, 128); }

// --------------------------------------------------------------------------
// tensor order of epd_weights
// --------------------------------------------------------------------------
struct TensorSpec { long rows, cols; };  // vectors: rows = 1

struct LayerIdx { int n1_g, n1_b, qkv_w, qkv_b, qn_g, kn_g, o_w, o_b, ls1, n2_g, n2_b, fc1_w, fc1_b, fc2_w, fc2_b, ls2; };

struct WeightIndex {
  int pe_w, pe_b, pos, cls;
  std::vector<LayerIdx> layers;
  int fn_g, fn_b, pn_g, pn_b, pa_w, pa_b, pb_w, pb_b;
  int r_kv_w, r_query, r_pos, r_lnq_g, r_lnq_b, r_lnkv_g, r_lnkv_b, r_in_w, r_in_b, r_out_w, r_out_b, r_lnp_g, r_lnp_b, r_proj_w;
  std::vector<TensorSpec> specs;
};

// N = patches per slice; Nt = tokens per slice inside the encoder (patches + class token); Ns = rows a
// slice owns in the activation buffers (bf16 mode: Nt rounded up to 8, the unit of the transposed value
// store; the extra rows are masked as keys and never read as tokens; fp32 mode: Nt).
struct Dims {
  int S, p, g, N, Kp, D, H, hd, F, L, N_out, Pin, Pmid, Pout, cls, Nt, Ns;
  SliceRows xrows() const { return (Ns == N) ? SliceRows{0, 0, 0} : SliceRows{N, Ns, cls}; }
};

Dims dims_of(const epd_model_desc& d) {
  Dims x;
  x.S = d.tile_size; x.p = d.patch; x.g = d.tile_size / d.patch; x.N = x.g * x.g;
  x.Kp = 3 * d.patch * d.patch; x.D = d.hidden; x.H = d.heads; x.hd = d.hidden / d.heads;
  x.F = d.mlp; x.L = d.layers;
  x.N_out = d.proj_kind == EPD_PROJ_RESAMPLER ? d.proj_mid : (d.pixel_shuffle ? x.N / 4 : x.N);
  x.Pin = d.pixel_shuffle ? 4 * x.D : x.D;
  x.Pmid = d.proj_mid; x.Pout = d.proj_out;
  x.cls = d.class_token ? 1 : 0;
  x.Nt = x.N + x.cls;
  x.Ns = d.dtype == EPD_DTYPE_BF16 ? round_up(x.Nt, 8) : x.Nt;
  return x;
}

WeightIndex build_index(const epd_model_desc& d) {
  const Dims x = dims_of(d);
  WeightIndex w;
  auto add = [&](long r, long c) { w.specs.push_back({r, c}); return (int)w.specs.size() - 1; };
  const bool ln = d.norm == EPD_NORM_LAYERNORM;
  w.pe_w = add(x.D, x.Kp); w.pe_b = add(1, x.D); w.pos = add(x.Nt, x.D);
  w.cls = x.cls ? add(1, x.D) : -1;
  for (int l = 0; l < x.L; ++l) {
    LayerIdx i;
    i.n1_g = add(1, x.D); i.n1_b = ln ? add(1, x.D) : -1;
    i.qkv_w = add(3L * x.D, x.D); i.qkv_b = add(1, 3L * x.D);
    i.qn_g = i.kn_g = -1;
    if (d.qk_norm == EPD_QKNORM_FULL) { i.qn_g = add(1, x.D); i.kn_g = add(1, x.D); }
    if (d.qk_norm == EPD_QKNORM_PER_HEAD) { i.qn_g = add(1, x.hd); i.kn_g = add(1, x.hd); }
    i.o_w = add(x.D, x.D); i.o_b = add(1, x.D);
    i.ls1 = d.layer_scale ? add(1, x.D) : -1;
    i.n2_g = add(1, x.D); i.n2_b = ln ? add(1, x.D) : -1;
    i.fc1_w = add(x.F, x.D); i.fc1_b = add(1, x.F);
    i.fc2_w = add(x.D, x.F); i.fc2_b = add(1, x.D);
    i.ls2 = d.layer_scale ? add(1, x.D) : -1;
    w.layers.push_back(i);
  }
  w.fn_g = w.fn_b = w.pn_g = w.pn_b = w.pa_w = w.pa_b = w.pb_w = w.pb_b = -1;
  if (d.final_norm) { w.fn_g = add(1, x.D); w.fn_b = ln ? add(1, x.D) : -1; }
  if (d.proj_prenorm) { w.pn_g = add(1, x.Pin); w.pn_b = add(1, x.Pin); }
  if (d.proj_kind == EPD_PROJ_RESAMPLER) {
    const long E = x.Pout, Q = x.Pmid;
    w.r_kv_w = add(E, x.D); w.r_query = add(Q, E); w.r_pos = add(x.N, E);
    w.r_lnq_g = add(1, E); w.r_lnq_b = add(1, E); w.r_lnkv_g = add(1, E); w.r_lnkv_b = add(1, E);
    w.r_in_w = add(3 * E, E); w.r_in_b = add(1, 3 * E); w.r_out_w = add(E, E); w.r_out_b = add(1, E);
    w.r_lnp_g = add(1, E); w.r_lnp_b = add(1, E); w.r_proj_w = add(E, E);
  } else if (d.proj_kind == EPD_PROJ_LINEAR) {
    w.pa_w = add(x.Pout, x.Pin); w.pa_b = add(1, x.Pout);
  } else {
    w.pa_w = add(x.Pmid, x.Pin); w.pa_b = add(1, x.Pmid);
    w.pb_w = add(x.Pout, x.Pmid); w.pb_b = add(1, x.Pout);
  }
  return w;
}

epd_status check_desc(const epd_model_desc* d, char* err, size_t len) {
  if (!d) { set_err(err, len, "desc is null"); return EPD_ERR_INVALID_ARG; }
  if (d->dtype != EPD_DTYPE_FP32 && d->dtype != EPD_DTYPE_BF16) { set_err(err, len, "dtype must be 0 (fp32) or 1 (bf16)"); return EPD_ERR_INVALID_ARG; }
  if (d->norm < 0 || d->norm > 1 || d->qk_norm < 0 || d->qk_norm > 2 || d->act < 0 || d->act > 1 ||
      d->final_norm < 0 || d->final_norm > 1 || d->pixel_shuffle < 0 || d->pixel_shuffle > 1 ||
      d->proj_kind < 0 || d->proj_kind > 2 || d->proj_prenorm < 0 || d->proj_prenorm > 1 ||
      d->layer_scale < 0 || d->layer_scale > 1 || d->class_token < 0 || d->class_token > 1 ||
      d->mx_fp8 < 0 || d->mx_fp8 > 1) {
    set_err(err, len, "an enum field of the description is out of range"); return EPD_ERR_INVALID_ARG;
  }
  if (d->tile_size <= 0 || d->patch <= 0 || d->hidden <= 0 || d->heads <= 0 || d->mlp <= 0 ||
      d->layers < 0 || d->proj_out <= 0 || d->max_tiles_per_call <= 0 || !(d->eps > 0.f)) {
    set_err(err, len, "sizes must be positive (layers >= 0, eps > 0, max_tiles_per_call >= 1)"); return EPD_ERR_SHAPE;
  }
  if (d->tile_size % d->patch) { set_err(err, len, "tile_size %d is not a multiple of patch %d", d->tile_size, d->patch); return EPD_ERR_SHAPE; }
  if (d->hidden % d->heads) { set_err(err, len, "hidden %d is not a multiple of heads %d", d->hidden, d->heads); return EPD_ERR_SHAPE; }
  if (d->proj_kind == EPD_PROJ_MLP && d->proj_mid <= 0) { set_err(err, len, "proj_mid must be positive for an MLP projector"); return EPD_ERR_SHAPE; }
  if (d->proj_kind == EPD_PROJ_RESAMPLER) {
    if (d->proj_mid <= 0 || d->proj_heads <= 0 || d->proj_out % d->proj_heads) {
      set_err(err, len, "resampler needs proj_mid (queries) > 0 and proj_heads > 0 dividing proj_out"); return EPD_ERR_SHAPE;
    }
    if (d->pixel_shuffle || d->proj_prenorm) { set_err(err, len, "resampler excludes pixel_shuffle and proj_prenorm"); return EPD_ERR_INVALID_ARG; }
  }
  const Dims x = dims_of(*d);
  if (d->pixel_shuffle && (x.g % 2)) { set_err(err, len, "pixel shuffle needs an even patch grid, got %d", x.g); return EPD_ERR_SHAPE; }
  if ((long)x.Ns * d->max_tiles_per_call > (1L << 30)) { set_err(err, len, "max_tiles_per_call too large"); return EPD_ERR_UNSUPPORTED; }
  if (d->dtype == EPD_DTYPE_BF16) {
    if (x.hd > 128) { set_err(err, len, "bf16 mode supports head dim <= 128, got %d", x.hd); return EPD_ERR_UNSUPPORTED; }
    if (x.D % 4 || x.hd % 4 || x.F % 8 || x.Pout % 8 || (d->proj_kind == EPD_PROJ_MLP && x.Pmid % 8)) {
      set_err(err, len, "bf16 mode needs hidden and head dim %% 4 == 0, mlp and projector widths %% 8 == 0"); return EPD_ERR_UNSUPPORTED;
    }
    if (d->proj_kind == EPD_PROJ_RESAMPLER) {
      const int hdr = d->proj_out / d->proj_heads;
      if (x.N % 64 || hdr > 128 || hdr % 4) {
        set_err(err, len, "bf16 resampler needs patches per slice %% 64 == 0 and a head dim <= 128, %% 4 == 0 (got %d, %d)", x.N, hdr);
        return EPD_ERR_UNSUPPORTED;
      }
    }
  }
  if (d->mx_fp8 && (d->dtype != EPD_DTYPE_BF16 || x.D % 128)) {
    set_err(err, len, "mx_fp8 needs bf16 mode and hidden %% 128 == 0 (blocks of 32 along whole 128-element slabs), got hidden %d", x.D);
    return EPD_ERR_UNSUPPORTED;
  }
  if (x.N > 16384) { set_err(err, len, "more than 16384 patches per slice is not supported"); return EPD_ERR_UNSUPPORTED; }
  if (d->dtype == EPD_DTYPE_FP32) {
    // the fp32 attention kernel keeps one query's logits and the query itself in LDS (64 KiB without opt-in)
    const int hdr = d->proj_kind == EPD_PROJ_RESAMPLER ? d->proj_out / d->proj_heads : 0;
    if (((long)x.Nt + std::max(x.hd, hdr)) * 4 > 65536) {
      set_err(err, len, "fp32 mode supports at most %d tokens per slice at this head dim", 16384 - std::max(x.hd, hdr));
      return EPD_ERR_UNSUPPORTED;
    }
  }
  return EPD_OK;
}

// --------------------------------------------------------------------------
// context
// --------------------------------------------------------------------------
struct Linear {
  const void* W = nullptr;  // fp32 mode: float [N,K]; bf16 mode: packed bf16 [Npad,K]
  const float* b = nullptr; // fp32 (padded to Npad in bf16 mode)
  int N = 0, K = 0, Npad = 0;
};

// Cross-attention resampler projector: weights, the projected learned queries, and its workspace.
struct Resampler {
  Linear kv, k, v, o, proj;     // kv: hidden -> E; k, v: in-projections of keys / values; o: out-projection; proj: last matrix
  const float *lnkv_g = nullptr, *lnkv_b = nullptr, *lnp_g = nullptr, *lnp_b = nullptr;
  const float* pos = nullptr;   // [N, E] fp32
  void* qp = nullptr;           // in-projected LN_q(query): bf16 [>= round_up(Q, 256), Eq_k] / fp32 [Q, E]
  int Q = 0, E = 0, H = 0, hd = 0, hd_pad = 0, Eq = 0, Eq_k = 0, E_k = 0;
  void *xin = nullptr, *kvraw = nullptr, *kin = nullptr, *vin = nullptr, *K = nullptr, *V = nullptr, *O = nullptr,
       *o2 = nullptr, *o3 = nullptr;   // V: bf16 [mb, H, hd_pad, N] (transposed) / fp32 [M, E]
};

// A Linear whose weights are kept as MXFP8 codes and block scales (gemm_mxfp8.hip), rows padded to 256
struct MxLinear {
  const unsigned char* W = nullptr;   // [Npad, K]
  const unsigned* SW = nullptr;       // [K / 128][Npad]
  const float* b = nullptr;           // [Npad]
  const float* cs = nullptr;          // [Npad] factor applied to the product in the epilogue, or null
  int N = 0, K = 0, Npad = 0;
};

struct LayerW {
  const float *n1_g = nullptr, *n1_b = nullptr, *n2_g = nullptr, *n2_b = nullptr, *qn_g = nullptr, *kn_g = nullptr;
  Linear qkv, v, o, fc1, fc2;  // bf16 mode: qkv holds q,k only and v the value projection
  // folded pre-norms (bf16 mode): the weights of qkv, v (first norm) and fc1 (second norm) carry the norm's gain,
  // their biases its shift, and these are the column sums of the packed weights the epilogues subtract the mean with
  const float *qkv_cs = nullptr, *v_cs = nullptr, *fc1_cs = nullptr;
  MxLinear mqkv, mv, mo, mfc1, mfc2;   // epd_model_desc::mx_fp8: the same matrices as MXFP8 operands (mo: only when the heads are stored unpadded)
};

}  // namespace

enum { NORM_CLASSIC = 0, NORM_COPY = 1, NORM_FOLD = 2 };

struct epd_ctx {
  epd_model_desc d;
  Dims x;
  bool bf16;
  std::vector<void*> allocs;
  char err[512];

  // weights
  Linear pe, pa, pb;
  Resampler rs;
  const float* pos = nullptr;   // [Nt, D]; row 0 is the class token's when there is one
  const float* cls = nullptr;   // [D], null without a class token
  const float *fn_g = nullptr, *fn_b = nullptr, *pn_g = nullptr, *pn_b = nullptr;
  std::vector<LayerW> layers;

  // bf16 layout
  int hd_pad = 0, Dq = 0, Dq_k = 0, D_k = 0, F_k = 0, Kp_k = 0, Pin_k = 0, Pmid_k = 0;

  // How the pre-norms of the layers run in bf16 mode (EPD_NORM_MODE = classic | copy | fold at epd_create):
  //   NORM_CLASSIC  a row kernel reads the fp32 stream and writes the normalised bf16 operand (the default: the
  //                 fastest of the three as measured, because the products' epilogues run with the matrix cores
  //                 idle, so every store and every vector operation added there costs more than it saves);
  //   NORM_COPY     the residual epilogues also leave bf16(x) in Xn and a row kernel normalises those rows in
  //                 place: a third less traffic per norm;
  //   NORM_FOLD     no norm kernel at all: the residual epilogues leave bf16(x) and the rows' statistics, the
  //                 products run on bf16(x) against gain-scaled weights and apply mean / rstd in their epilogues.
  int norm_mode = 0;
  bool fold = false;        // norm_mode == NORM_FOLD
  bool mx = false;          // epd_model_desc::mx_fp8: q/k, value, FC1 and FC2 products on MXFP8 operands
  bool mx_o = false;        // ... and the out-projection (head dim stored without padding: the blocks of 32 are the definition's)
  void* OQ = nullptr;       // attention output as MXFP8: codes [Mp, Dq_k], then scale words [Dq_k / 128][Mp]
  std::vector<std::vector<float>> host_keep;   // host vectors with copies to the device in flight (epd_create only)
  float* stats = nullptr;   // [Mp][n_part][2]: one pair per 128 columns, as the residual epilogues emit them
  float* stats1 = nullptr;  // [Mp][2]: one pair per row, made from `stats` when a row has more pairs than the products take (wide models)
  int n_part = 0;

  // workspace (sized for mb slices)
  int mb = 0;
  long Mp = 0, Mp_out = 0;
  float* X = nullptr;      // residual stream fp32 [Mp, D]
  void* Xn = nullptr;      // normalised activations
  void* QKV = nullptr;     // fp32: [M,3D]; bf16: q,k [Mp, 2Dq]
  void* VT = nullptr;      // bf16: [mb, H, hd_pad, N]
  void* O = nullptr;
  void* Hd = nullptr;
  void* Ape = nullptr;
  void* Pin = nullptr;
  void* Pmid = nullptr;
  long last_rows = 0;

  // paged output (epd_encode_paged): device row-block map of the current micro-batch
  int* d_rowmap = nullptr;       // [mb * N] ints (enough for any block size, trunk or projector rows)
  // the caller's (pageable) block table reaches d_rowmap through two pinned staging buffers used in turn,
  // each guarded by an event recorded behind its upload: the copy is truly asynchronous, and the host only
  // waits when a call has more than two micro-batches in flight
  int* h_rowmap[2] = {nullptr, nullptr};
  hipEvent_t ev_rowmap[2] = {nullptr, nullptr};
  bool rowmap_pending[2] = {false, false};
  int rowmap_turn = 0;
  const int* cur_rowmap = nullptr;  // null: contiguous output
  int cur_block_tokens = 1;
  const void* cur_in_pool = nullptr;  // STAGE_PROJECT: cache pool the pre-projection tokens are read from

  // profiling
  bool prof = false;
  std::vector<hipEvent_t> ev;
  std::vector<int> ev_family;
  std::vector<int> ev_kernels;   // kernels launched inside each bracket
  size_t ev_used = 0;
};

namespace {

struct ProfScope {
  epd_ctx* c; hipStream_t st; bool on; long gemm_before;
  ProfScope(epd_ctx* c_, int family, hipStream_t st_) : c(c_), st(st_), on(false), gemm_before(0) {
    if (c->prof && c->ev_used + 2 <= c->ev.size()) {
      on = true;
      c->ev_family.push_back(family);
      gemm_before = bf16_gemm_kernel_launches();
      hipEventRecord(c->ev[c->ev_used], st);
    }
  }
  ~ProfScope() {
    if (on) {
      hipEventRecord(c->ev[c->ev_used + 1], st);
      c->ev_used += 2;
      // a bracket around a product counts the kernels it was cut into; any other bracket holds one kernel
      const long k = bf16_gemm_kernel_launches() - gemm_before;
      c->ev_kernels.push_back(k > 0 ? (int)k : 1);
    }
  }
};

#define HIP_TRY(ctx, expr)                                                                   \
  do {                                                                                       \
    hipError_t e__ = (expr);                                                                 \
    if (e__ != hipSuccess) {                                                                 \
      set_err((ctx)->err, sizeof((ctx)->err), "%s failed: %s", #expr, hipGetErrorString(e__)); \
      return EPD_ERR_HIP;                                                                    \
    }                                                                                        \
  } while (0)

void* dalloc(epd_ctx* c, size_t bytes, bool zero, hipStream_t st) {
  void* p = nullptr;
  if (bytes == 0) bytes = 256;
  if (hipMalloc(&p, bytes) != hipSuccess) return nullptr;
  c->allocs.push_back(p);
  if (zero && hipMemsetAsync(p, 0, bytes, st) != hipSuccess) return nullptr;
  return p;
}

// fp32 copy of a small tensor (bias / gain / position embedding), optionally
// re-indexed over padded heads and zero-padded to n_pad.
const float* make_vec(epd_ctx* c, const epd_weights* w, int idx, long n, int n_pad, PackMap map, hipStream_t st) {
  if (idx < 0) return nullptr;
  float* dst = (float*)dalloc(c, (size_t)n_pad * sizeof(float), false, st);
  if (!dst) return nullptr;
  pack_vector_f32(w->tensors[idx], c->bf16 ? 1 : 0, (int)n, dst, n_pad, map, st);
  return dst;
}

// elements of the weight dtype further into a caller tensor
const void* tensor_at(const epd_ctx* c, const void* base, long elems) {
  return (const char*)base + elems * (c->bf16 ? 2 : 4);
}

// fp32 copy of n values at src (weight dtype), zero-padded / head-reindexed to n_pad; src null: zeros
const float* make_vec_p(epd_ctx* c, const void* src, long n, int n_pad, PackMap map, hipStream_t st) {
  float* dst = (float*)dalloc(c, (size_t)n_pad * sizeof(float), src == nullptr, st);
  if (!dst) return nullptr;
  if (src) pack_vector_f32(src, c->bf16 ? 1 : 0, (int)n, dst, n_pad, map, st);
  return dst;
}

// Linear from a [N, K] matrix at Wsrc and a bias at bsrc (null: no bias, a zero vector is kept)
bool make_linear_p(epd_ctx* c, const void* Wsrc, const void* bsrc, int N, int K, Linear* out, hipStream_t st,
                   int Npad, int Kpad, PackMap rmap, PackMap cmap, int n_packed) {
  out->N = n_packed; out->K = Kpad; out->Npad = Npad;
  if (!c->bf16) {
    const size_t bytes = (size_t)N * K * sizeof(float);
    void* dst = dalloc(c, bytes, false, st);
    if (!dst) return false;
    if (hipMemcpyAsync(dst, Wsrc, bytes, hipMemcpyDeviceToDevice, st) != hipSuccess) return false;
    out->W = dst; out->N = N; out->K = K; out->Npad = N;
    out->b = make_vec_p(c, bsrc, N, N, PackMap{0, 0, 0}, st);
    return out->b != nullptr;
  }
  bf16_t* dst = (bf16_t*)dalloc(c, (size_t)Npad * Kpad * sizeof(bf16_t), false, st);
  if (!dst) return false;
  pack_matrix_bf16((const bf16_t*)Wsrc, N, K, dst, Npad, Kpad, rmap, cmap, st);
  out->W = dst;
  out->b = make_vec_p(c, bsrc, N, Npad, rmap, st);
  return out->b != nullptr;
}

bool make_linear(epd_ctx* c, const epd_weights* w, int wi, int bi, int N, int K, Linear* out, hipStream_t st,
                 int Npad, int Kpad, PackMap rmap, PackMap cmap, int n_packed) {
  return make_linear_p(c, w->tensors[wi], bi >= 0 ? w->tensors[bi] : nullptr, N, K, out, st, Npad, Kpad, rmap, cmap, n_packed);
}

GemmParams gp(int epi, const void* A, long lda, const Linear& lin, int M);

// MXFP8 copy of a packed bf16 Linear: codes and block scales of its rows as they are now (call it before any
// factor is folded into the rows: conversion is not invariant under factors that are not powers of two)
bool mx_make(epd_ctx* c, const Linear& lin, MxLinear* out, hipStream_t st) {
  const int np = round_up(lin.Npad, 256);
  unsigned char* codes = (unsigned char*)dalloc(c, (size_t)np * lin.K, true, st);
  unsigned* sw = (unsigned*)dalloc(c, (size_t)(lin.K / 128) * np * sizeof(unsigned), true, st);
  if (!codes || !sw) return false;
  MxRowParams p;
  memset(&p, 0, sizeof(p));
  p.kind = 2; p.in = lin.W; p.ld_in = lin.K; p.in_bf16 = 1; p.rows = lin.Npad; p.dim = lin.K;
  p.codes = codes; p.ld_codes = lin.K; p.scales = sw; p.ld_scales = np;
  if (mx_rows(p, st) != hipSuccess) return false;
  out->W = codes; out->SW = sw; out->N = lin.N; out->K = lin.K; out->Npad = np;
  return true;
}
// ... and its bias as it is at the end of the layer's set-up (factors folded in), plus the factor of the product:
// `cs_dev` (device, n_cs values) or the constant `cs_const` for the first n_cs columns, 1 elsewhere; n_cs == 0: none
bool mx_finish(epd_ctx* c, const Linear& lin, MxLinear* out, const float* cs_dev, float cs_const, int n_cs, hipStream_t st) {
  float* b = (float*)dalloc(c, (size_t)out->Npad * sizeof(float), true, st);
  if (!b || hipMemcpyAsync(b, lin.b, (size_t)lin.Npad * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return false;
  out->b = b;
  if (n_cs > 0) {
    float* cs = (float*)dalloc(c, (size_t)out->Npad * sizeof(float), false, st);
    if (!cs) return false;
    c->host_keep.emplace_back((size_t)out->Npad, 1.0f);
    std::vector<float>& h = c->host_keep.back();
    if (!cs_dev) for (int i = 0; i < n_cs; ++i) h[i] = cs_const;
    if (hipMemcpyAsync(cs, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice, st) != hipSuccess) return false;
    if (cs_dev && hipMemcpyAsync(cs, cs_dev, (size_t)n_cs * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return false;
    out->cs = cs;
  }
  return true;
}

epd_status build_ctx(epd_ctx* c, const epd_weights* w, hipStream_t st) {
  const epd_model_desc& d = c->d;
  const Dims& x = c->x;
  const WeightIndex wi = build_index(d);
  const PackMap id{0, 0, 0};
  const bool bf = c->bf16;

  if (bf) {
    // head dims the attention kernel is built for; others are zero-padded up to the next one
    c->hd_pad = x.hd <= 64 ? 64 : (x.hd == 72 ? 72 : (x.hd <= 96 ? 96 : 128));
    c->Dq = x.H * c->hd_pad;
    c->Dq_k = round_up(c->Dq, 128);
    c->D_k = round_up(x.D, 128);
    c->Kp_k = round_up(x.Kp, 128);
    c->Pin_k = round_up(x.Pin, 128);
    HIP_TRY(c, bf16_gemm_init());
  }
  const PackMap heads{x.hd, c->hd_pad, x.H};
  if (bf) {
    const char* m = getenv("EPD_NORM_MODE");
    c->norm_mode = NORM_CLASSIC;
    if (m && !strcmp(m, "copy")) c->norm_mode = x.D % 8 == 0 ? NORM_COPY : NORM_CLASSIC;   // the in-place kernel moves 16-byte chunks
    else if (m && !strcmp(m, "fold")) c->norm_mode = NORM_FOLD;
    else if (m && *m && strcmp(m, "classic")) {
      set_err(c->err, sizeof(c->err), "EPD_NORM_MODE must be classic, copy or fold, got '%s'", m);
      return EPD_ERR_INVALID_ARG;
    }
  }
  c->fold = c->norm_mode == NORM_FOLD;
  c->n_part = (x.D + STAT_GROUP - 1) / STAT_GROUP;
  c->mx = bf && d.mx_fp8;
  if (c->mx) {
    if (c->norm_mode != NORM_CLASSIC) {
      set_err(c->err, sizeof(c->err), "mx_fp8 converts in the pre-norm kernel: EPD_NORM_MODE must be classic");
      return EPD_ERR_INVALID_ARG;
    }
    HIP_TRY(c, mx_gemm_init());
    c->mx_o = c->hd_pad == x.hd;
  }

#define NOMEM_IF(cond) do { if (cond) { set_err(c->err, sizeof(c->err), "device allocation failed (weights)"); return EPD_ERR_NOMEM; } } while (0)

  // patch embedding and position embedding
  NOMEM_IF(!make_linear(c, w, wi.pe_w, wi.pe_b, x.D, x.Kp, &c->pe, st, pad_n(x.D), c->Kp_k, id, id, x.D));
  c->pos = make_vec(c, w, wi.pos, (long)x.Nt * x.D, x.Nt * x.D, id, st);
  NOMEM_IF(!c->pos);
  if (x.cls) { c->cls = make_vec(c, w, wi.cls, x.D, x.D, id, st); NOMEM_IF(!c->cls); }

  const float logit_scale = 1.4426950408889634f / sqrtf((float)x.hd);   // log2(e) / sqrt(hd)
  int f_pad = 0;
  for (int l = 0; l < x.L; ++l) {
    const LayerIdx& li = wi.layers[l];
    LayerW lw;
    lw.n1_g = make_vec(c, w, li.n1_g, x.D, x.D, id, st);
    lw.n1_b = make_vec(c, w, li.n1_b, x.D, x.D, id, st);
    lw.n2_g = make_vec(c, w, li.n2_g, x.D, x.D, id, st);
    lw.n2_b = make_vec(c, w, li.n2_b, x.D, x.D, id, st);
    NOMEM_IF(!lw.n1_g || !lw.n2_g);
    if (!bf) {
      NOMEM_IF(!make_linear(c, w, li.qkv_w, li.qkv_b, 3 * x.D, x.D, &lw.qkv, st, 0, 0, id, id, 0));
      NOMEM_IF(!make_linear(c, w, li.o_w, li.o_b, x.D, x.D, &lw.o, st, 0, 0, id, id, 0));
      NOMEM_IF(!make_linear(c, w, li.fc1_w, li.fc1_b, x.F, x.D, &lw.fc1, st, 0, 0, id, id, 0));
      NOMEM_IF(!make_linear(c, w, li.fc2_w, li.fc2_b, x.D, x.F, &lw.fc2, st, 0, 0, id, id, 0));
      if (d.qk_norm) {
        const int n = d.qk_norm == EPD_QKNORM_FULL ? x.D : x.hd;
        lw.qn_g = make_vec(c, w, li.qn_g, n, n, id, st);
        lw.kn_g = make_vec(c, w, li.kn_g, n, n, id, st);
        NOMEM_IF(!lw.qn_g || !lw.kn_g);
      }
    } else {
      // q,k projection (rows [q heads | k heads], heads padded to hd_pad) and the value
      // projection (stored transposed by its epilogue) are two products over the same input
      {
        const int qk_cols = 2 * c->Dq, qk_pad = pad_n(qk_cols), v_pad = pad_n(c->Dq);
        // one block each for the two weight matrices and the two bias vectors, the value projection's behind the
        // q/k projection's: a single slice runs both products as one launch (GemmParams::n2)
        bf16_t* Wqk = (bf16_t*)dalloc(c, (size_t)(qk_pad + v_pad) * c->D_k * sizeof(bf16_t), true, st);
        float* bqk = (float*)dalloc(c, (size_t)(qk_pad + v_pad) * sizeof(float), true, st);
        NOMEM_IF(!Wqk || !bqk);
        bf16_t* Wv = Wqk + (size_t)qk_pad * c->D_k;
        float* bv = bqk + qk_pad;
        pack_matrix_bf16((const bf16_t*)w->tensors[li.qkv_w], 2 * x.D, x.D, Wqk, qk_cols, c->D_k, heads, id, st);
        pack_matrix_bf16((const bf16_t*)w->tensors[li.qkv_w] + 2L * x.D * x.D, x.D, x.D, Wv, c->Dq, c->D_k, heads, id, st);
        pack_vector_f32(w->tensors[li.qkv_b], 1, 2 * x.D, bqk, qk_cols, heads, st);
        pack_vector_f32((const bf16_t*)w->tensors[li.qkv_b] + 2 * x.D, 1, x.D, bv, c->Dq, heads, st);
        // The attention kernel takes its logits in the log2 domain straight from the q . k product: the factor
        // (1 / sqrt(hd)) log2(e) rides on q.  Without a q/k norm it is folded into the q rows of the projection
        // (each weight rounded to bf16 once more: the rounding errors of a row average out over the hidden
        // dimension, unlike a second rounding of q itself); with one, into the norm's gain below.
        lw.qkv.W = Wqk; lw.qkv.b = bqk; lw.qkv.N = qk_cols; lw.qkv.K = c->D_k; lw.qkv.Npad = qk_pad;
        lw.v.W = Wv; lw.v.b = bv; lw.v.N = c->Dq; lw.v.K = c->D_k; lw.v.Npad = v_pad;
        if (c->mx) NOMEM_IF(!mx_make(c, lw.qkv, &lw.mqkv, st) || !mx_make(c, lw.v, &lw.mv, st));   // from the unscaled rows
        if (d.qk_norm == EPD_QKNORM_NONE) scale_rows_by(Wqk, c->Dq, c->D_k, c->D_k, bqk, logit_scale, st);
      }

      NOMEM_IF(!make_linear(c, w, li.o_w, li.o_b, x.D, x.D, &lw.o, st, pad_n(x.D), c->Dq_k, id, heads, x.D));
      if (c->mx_o) NOMEM_IF(!mx_make(c, lw.o, &lw.mo, st));   // before the layer scale below
      f_pad = pad_n(x.F);
      NOMEM_IF(!make_linear(c, w, li.fc1_w, li.fc1_b, x.F, x.D, &lw.fc1, st, f_pad, c->D_k, id, id, x.F));
      NOMEM_IF(!make_linear(c, w, li.fc2_w, li.fc2_b, x.D, x.F, &lw.fc2, st, pad_n(x.D), f_pad, id, id, x.D));
      if (c->mx) NOMEM_IF(!mx_make(c, lw.fc1, &lw.mfc1, st) || !mx_make(c, lw.fc2, &lw.mfc2, st));   // before the layer scale below
      if (d.qk_norm == EPD_QKNORM_FULL) {
        lw.qn_g = make_vec(c, w, li.qn_g, x.D, c->Dq, heads, st);
        lw.kn_g = make_vec(c, w, li.kn_g, x.D, c->Dq, heads, st);
        NOMEM_IF(!lw.qn_g || !lw.kn_g);
        scale_vector(const_cast<float*>(lw.qn_g), c->Dq, logit_scale, st);
      } else if (d.qk_norm == EPD_QKNORM_PER_HEAD) {
        lw.qn_g = make_vec(c, w, li.qn_g, x.hd, c->hd_pad, id, st);
        lw.kn_g = make_vec(c, w, li.kn_g, x.hd, c->hd_pad, id, st);
        NOMEM_IF(!lw.qn_g || !lw.kn_g);
        scale_vector(const_cast<float*>(lw.qn_g), c->hd_pad, logit_scale, st);
      }
    }
    const float* ls1 = nullptr;
    const float* ls2 = nullptr;
    if (d.layer_scale) {
      // layer scale is folded into the branch's last Linear: rows of W and the bias times ls
      ls1 = make_vec(c, w, li.ls1, x.D, x.D, id, st);
      ls2 = make_vec(c, w, li.ls2, x.D, x.D, id, st);
      NOMEM_IF(!ls1 || !ls2);
      scale_rows(const_cast<void*>(lw.o.W), bf ? 1 : 0, x.D, lw.o.K, lw.o.K, const_cast<float*>(lw.o.b), ls1, st);
      scale_rows(const_cast<void*>(lw.fc2.W), bf ? 1 : 0, x.D, lw.fc2.K, lw.fc2.K, const_cast<float*>(lw.fc2.b), ls2, st);
    }
    if (c->mx) {
      // the biases carry the factors by now; the MXFP8 products apply them to the accumulator in the epilogue
      NOMEM_IF(!mx_finish(c, lw.qkv, &lw.mqkv, nullptr, logit_scale, d.qk_norm == EPD_QKNORM_NONE ? c->Dq : 0, st));
      NOMEM_IF(!mx_finish(c, lw.v, &lw.mv, nullptr, 1.f, 0, st));
      NOMEM_IF(!mx_finish(c, lw.fc1, &lw.mfc1, nullptr, 1.f, 0, st));
      NOMEM_IF(!mx_finish(c, lw.fc2, &lw.mfc2, ls2, 1.f, ls2 ? x.D : 0, st));
      if (c->mx_o) NOMEM_IF(!mx_finish(c, lw.o, &lw.mo, ls1, 1.f, ls1 ? x.D : 0, st));
    }
    if (c->fold) {
      float* cs_qk = (float*)dalloc(c, (size_t)lw.qkv.Npad * sizeof(float), true, st);
      float* cs_v = (float*)dalloc(c, (size_t)lw.v.Npad * sizeof(float), true, st);
      float* cs_f = (float*)dalloc(c, (size_t)lw.fc1.Npad * sizeof(float), true, st);
      NOMEM_IF(!cs_qk || !cs_v || !cs_f);
      fold_norm_into_linear((bf16_t*)const_cast<void*>(lw.qkv.W), lw.qkv.Npad, lw.qkv.K, lw.qkv.K, lw.n1_g, lw.n1_b, x.D,
                            const_cast<float*>(lw.qkv.b), cs_qk, st);
      fold_norm_into_linear((bf16_t*)const_cast<void*>(lw.v.W), lw.v.Npad, lw.v.K, lw.v.K, lw.n1_g, lw.n1_b, x.D,
                            const_cast<float*>(lw.v.b), cs_v, st);
      fold_norm_into_linear((bf16_t*)const_cast<void*>(lw.fc1.W), lw.fc1.Npad, lw.fc1.K, lw.fc1.K, lw.n2_g, lw.n2_b, x.D,
                            const_cast<float*>(lw.fc1.b), cs_f, st);
      lw.qkv_cs = cs_qk; lw.v_cs = cs_v; lw.fc1_cs = cs_f;
    }
    c->layers.push_back(lw);
  }
  c->F_k = bf ? (x.L ? f_pad : pad_n(x.F)) : x.F;

  if (d.final_norm) {
    c->fn_g = make_vec(c, w, wi.fn_g, x.D, x.D, id, st);
    c->fn_b = make_vec(c, w, wi.fn_b, x.D, x.D, id, st);
    NOMEM_IF(!c->fn_g);
  }
  if (d.proj_prenorm) {
    c->pn_g = make_vec(c, w, wi.pn_g, x.Pin, x.Pin, id, st);
    c->pn_b = make_vec(c, w, wi.pn_b, x.Pin, x.Pin, id, st);
    NOMEM_IF(!c->pn_g || !c->pn_b);
  }
  if (d.proj_kind == EPD_PROJ_RESAMPLER) {
    Resampler& r = c->rs;
    r.Q = x.Pmid; r.E = x.Pout; r.H = d.proj_heads; r.hd = r.E / r.H;
    const int E = r.E;
    r.hd_pad = bf ? (r.hd <= 64 ? 64 : (r.hd == 72 ? 72 : (r.hd <= 96 ? 96 : 128))) : r.hd;
    r.Eq = r.H * r.hd_pad;
    r.Eq_k = bf ? round_up(r.Eq, 128) : r.Eq;
    r.E_k = bf ? round_up(E, 128) : E;
    const PackMap rh = (bf && r.hd_pad != r.hd) ? PackMap{r.hd, r.hd_pad, r.H} : id;
    const void* in_w = w->tensors[wi.r_in_w];
    const void* in_b = w->tensors[wi.r_in_b];
    Linear lq;
    NOMEM_IF(!make_linear(c, w, wi.r_kv_w, -1, E, x.D, &r.kv, st, pad_n(E), c->D_k, id, id, E));
    NOMEM_IF(!make_linear_p(c, in_w, in_b, E, E, &lq, st, pad_n(r.Eq), r.E_k, rh, id, r.Eq));
    if (bf)   // the projected queries carry the logit scale of the cross attention (see the q rows of the layers)
      scale_rows_by((bf16_t*)const_cast<void*>(lq.W), r.Eq, r.E_k, r.E_k, const_cast<float*>(lq.b),
                    1.4426950408889634f / sqrtf((float)r.hd), st);
    NOMEM_IF(!make_linear_p(c, tensor_at(c, in_w, (long)E * E), tensor_at(c, in_b, E), E, E, &r.k, st, pad_n(r.Eq), r.E_k, rh, id, r.Eq));
    NOMEM_IF(!make_linear_p(c, tensor_at(c, in_w, 2L * E * E), tensor_at(c, in_b, 2L * E), E, E, &r.v, st, pad_n(r.Eq), r.E_k, rh, id, r.Eq));
    NOMEM_IF(!make_linear(c, w, wi.r_out_w, wi.r_out_b, E, E, &r.o, st, pad_n(E), r.Eq_k, id, rh, E));
    NOMEM_IF(!make_linear(c, w, wi.r_proj_w, -1, E, E, &r.proj, st, pad_n(E), r.E_k, id, id, E));
    r.lnkv_g = make_vec(c, w, wi.r_lnkv_g, E, E, id, st); r.lnkv_b = make_vec(c, w, wi.r_lnkv_b, E, E, id, st);
    r.lnp_g = make_vec(c, w, wi.r_lnp_g, E, E, id, st); r.lnp_b = make_vec(c, w, wi.r_lnp_b, E, E, id, st);
    r.pos = make_vec(c, w, wi.r_pos, (long)x.N * E, x.N * E, id, st);
    const float* query = make_vec(c, w, wi.r_query, (long)r.Q * E, r.Q * E, id, st);
    const float* lnq_g = make_vec(c, w, wi.r_lnq_g, E, E, id, st);
    const float* lnq_b = make_vec(c, w, wi.r_lnq_b, E, E, id, st);
    NOMEM_IF(!r.lnkv_g || !r.lnkv_b || !r.lnp_g || !r.lnp_b || !r.pos || !query || !lnq_g || !lnq_b);
    // the queries are the same for every slice: LN_q and their in-projection run once, here
    const long Qp = round_up(r.Q, 256);
    if (bf) {
      bf16_t* qn = (bf16_t*)dalloc(c, (size_t)Qp * r.E_k * 2, true, st);
      r.qp = dalloc(c, (size_t)Qp * r.Eq_k * 2, true, st);
      NOMEM_IF(!qn || !r.qp);
      RowOpParams ro{0, query, E, qn, r.E_k, lnq_g, lnq_b, r.Q, E, 0, x.g, x.D, d.eps, SliceRows{0, 0, 0}};
      bf16_rowop(ro, st);
      GemmParams p = gp(EPI_BIAS, qn, r.E_k, lq, r.Q);
      p.C = (bf16_t*)r.qp; p.ldc = r.Eq_k;
      HIP_TRY(c, bf16_gemm(p, st));
    } else {
      float* qn = (float*)dalloc(c, (size_t)r.Q * E * 4, false, st);
      r.qp = dalloc(c, (size_t)r.Q * E * 4, false, st);
      NOMEM_IF(!qn || !r.qp);
      f32_norm(0, query, E, qn, E, lnq_g, lnq_b, r.Q, E, 1, d.eps, st);
      f32_gemm(EPI_BIAS, qn, E, (const float*)lq.W, lq.b, (float*)r.qp, E, nullptr, 1, r.Q, E, E, st);
    }
  } else if (d.proj_kind == EPD_PROJ_LINEAR) {
    NOMEM_IF(!make_linear(c, w, wi.pa_w, wi.pa_b, x.Pout, x.Pin, &c->pa, st, pad_n(x.Pout), c->Pin_k, id, id, x.Pout));
  } else {
    const int mid_pad = pad_n(x.Pmid);
    c->Pmid_k = bf ? mid_pad : x.Pmid;
    NOMEM_IF(!make_linear(c, w, wi.pa_w, wi.pa_b, x.Pmid, x.Pin, &c->pa, st, mid_pad, c->Pin_k, id, id, x.Pmid));
    NOMEM_IF(!make_linear(c, w, wi.pb_w, wi.pb_b, x.Pout, x.Pmid, &c->pb, st, pad_n(x.Pout), mid_pad, id, id, x.Pout));
  }

  // ---- workspace ----
  c->mb = d.max_tiles_per_call;
  const long M = (long)c->mb * x.Ns, Mo = (long)c->mb * x.N_out;
  c->Mp = (M + 255) / 256 * 256;
  c->Mp_out = (Mo + 255) / 256 * 256;
  if (bf) {
    // the MFMA GEMM addresses its operands through 32-bit buffer offsets
    const long widest = std::max({(long)c->F_k, 2L * c->Dq, (long)c->Dq_k, (long)c->D_k, (long)c->Kp_k, 2L * x.D});
    if (c->Mp * widest * 2 >= (1L << 32) || c->Mp_out * (long)std::max(c->Pin_k, c->Pmid_k) * 2 >= (1L << 32)) {
      set_err(c->err, sizeof(c->err), "max_tiles_per_call %d makes an activation buffer of 4 GiB or more; use a smaller value "
              "(a call is cut into micro-batches of that many slices anyway)", c->mb);
      return EPD_ERR_UNSUPPORTED;
    }
  }
  bool ok = true;
  auto ws = [&](size_t bytes) { void* p = dalloc(c, bytes, true, st); ok = ok && p; return p; };
  // the residual GEMM prefetches whole 256-column tile rows: one padded row of slack behind the last
  c->X = (float*)ws(((size_t)c->Mp * x.D + 256) * sizeof(float));
  c->d_rowmap = (int*)ws((size_t)M * sizeof(int));
  for (int i = 0; i < 2; ++i) {
    if (hipHostMalloc((void**)&c->h_rowmap[i], (size_t)M * sizeof(int), hipHostMallocDefault) != hipSuccess) { c->h_rowmap[i] = nullptr; ok = false; }
    if (hipEventCreateWithFlags(&c->ev_rowmap[i], hipEventDisableTiming) != hipSuccess) { c->ev_rowmap[i] = nullptr; ok = false; }
  }
  if (bf) {
    c->Xn = ws((size_t)c->Mp * c->D_k * 2);
    if (c->fold) {
      c->stats = (float*)ws((size_t)c->Mp * c->n_part * 2 * sizeof(float));
      if (c->n_part > STAT_REGS) c->stats1 = (float*)ws((size_t)c->Mp * 2 * sizeof(float));
    }
    // the attention kernel reads whole 64-key blocks: up to 63 rows / elements past the last slice
    c->QKV = ws((size_t)(c->Mp + 64) * 2 * c->Dq * 2);
    c->VT = ws(((size_t)c->mb * x.H * c->hd_pad * x.Ns + 64) * 2);
    c->O = ws((size_t)c->Mp * c->Dq_k * 2);
    if (c->mx_o) c->OQ = ws((size_t)c->Mp * c->Dq_k + (size_t)(c->Dq_k / 128) * c->Mp * sizeof(unsigned));
    c->Hd = ws((size_t)c->Mp * c->F_k * 2);
    c->Ape = ws((size_t)c->Mp * c->Kp_k * 2);
    c->Pin = ws((size_t)c->Mp_out * c->Pin_k * 2);
    c->Pmid = ws((size_t)c->Mp_out * (c->Pmid_k ? c->Pmid_k : 64) * 2);
  } else {
    c->Xn = ws((size_t)M * x.D * 4);
    c->QKV = ws((size_t)M * 3 * x.D * 4);
    c->O = ws((size_t)M * x.D * 4);
    c->Hd = ws((size_t)M * x.F * 4);
    c->Ape = ws((size_t)M * x.Kp * 4);
    c->Pin = ws((size_t)Mo * x.Pin * 4);
    c->Pmid = ws((size_t)Mo * (x.Pmid > 0 ? x.Pmid : 1) * 4);
  }
  if (d.proj_kind == EPD_PROJ_RESAMPLER) {
    Resampler& r = c->rs;
    const long Mr = round_up(c->mb * x.N, 256), Mq = c->Mp_out;   // patch rows, query rows
    if (bf) {
      if (Mr * (long)std::max(r.E_k, r.Eq_k) * 2 >= (1L << 32)) {
        set_err(c->err, sizeof(c->err), "max_tiles_per_call %d makes a resampler buffer of 4 GiB or more", c->mb);
        return EPD_ERR_UNSUPPORTED;
      }
      r.xin = ws((size_t)Mr * c->D_k * 2); r.kvraw = ws((size_t)Mr * r.E_k * 2);
      r.kin = ws((size_t)Mr * r.E_k * 2); r.vin = ws((size_t)Mr * r.E_k * 2);
      r.K = ws((size_t)Mr * r.Eq_k * 2); r.V = ws((size_t)c->mb * r.H * r.hd_pad * x.N * 2);
      r.O = ws((size_t)Mq * r.Eq_k * 2); r.o2 = ws((size_t)Mq * r.E_k * 2); r.o3 = ws((size_t)Mq * r.E_k * 2);
    } else {
      const size_t e4 = (size_t)c->mb * x.N * r.E * 4, q4 = (size_t)c->mb * r.Q * r.E * 4;
      r.xin = ws((size_t)c->mb * x.N * x.D * 4); r.kvraw = ws(e4); r.kin = ws(e4); r.vin = ws(e4); r.K = ws(e4); r.V = ws(e4);
      r.O = ws(q4); r.o2 = ws(q4); r.o3 = ws(q4);
    }
  }
  if (!ok) { set_err(c->err, sizeof(c->err), "device allocation failed (workspace for %d slices)", c->mb); return EPD_ERR_NOMEM; }
  HIP_TRY(c, hipStreamSynchronize(st));
  HIP_TRY(c, hipGetLastError());
  c->host_keep.clear();
  return EPD_OK;
}

// --------------------------------------------------------------------------
// one micro-batch, fp32 mode
// --------------------------------------------------------------------------
// Which part of the path one call runs.  TRUNK stops after the final norm and writes the
// pre-projection tokens [N, hidden] of every slice into a paged cache; PROJECT starts from such
// tokens (read through a block table) and runs pixel shuffle + projector (Section 3.2.2: shards
// are aligned, projected and merged on the prefill side).
enum Stage { STAGE_FULL = 0, STAGE_TRUNK = 1, STAGE_PROJECT = 2 };

epd_status run_f32(epd_ctx* c, const float* tiles, int T, float* out, hipStream_t st, int stage) {
  const epd_model_desc& d = c->d;
  const Dims& x = c->x;
  const int M = T * x.Ns, Mo = T * x.N_out, Mpatch = T * x.N;
  const SliceRows xr = x.xrows();
  float* X = c->X; float* Xn = (float*)c->Xn; float* QKV = (float*)c->QKV; float* O = (float*)c->O;
  float* Hd = (float*)c->Hd; float* Ape = (float*)c->Ape; float* Pin = (float*)c->Pin; float* Pmid = (float*)c->Pmid;
  const int act_epi = d.act == EPD_ACT_GELU_ERF ? EPI_BIAS_GELU_ERF : EPI_BIAS_GELU_TANH;
  const float scale = 1.0f / sqrtf((float)x.hd);

  if (stage == STAGE_PROJECT) {
    ProfScope ps(c, 5, st);
    blocks_to_stream(c->cur_in_pool, 0, x.D, c->d_rowmap, c->cur_block_tokens, X, x.D, xr, Mpatch, st);
  } else {
    ProfScope ps(c, 0, st);
    f32_im2col(tiles, Ape, T, x.S, x.p, st);
    f32_gemm(EPI_BIAS_POS, Ape, x.Kp, (const float*)c->pe.W, c->pe.b, X, x.D, c->pos + (long)x.cls * x.D, x.N, Mpatch, x.D, x.Kp, st,
             nullptr, 1, xr);
    if (x.Ns != x.N) fill_slice_rows(X, x.D, T, x.Ns, x.Nt, c->cls, c->pos, st); }
  for (int l = 0; l < (stage == STAGE_PROJECT ? 0 : x.L); ++l) {
    const LayerW& w = c->layers[l];
    { ProfScope ps(c, 1, st); f32_norm(d.norm, X, x.D, Xn, x.D, w.n1_g, w.n1_b, M, x.D, 1, d.eps, st); }
    { ProfScope ps(c, 2, st); f32_gemm(EPI_BIAS, Xn, x.D, (const float*)w.qkv.W, w.qkv.b, QKV, 3 * x.D, nullptr, 1, M, 3 * x.D, x.D, st); }
    if (d.qk_norm == EPD_QKNORM_FULL) {
      ProfScope ps(c, 4, st);
      f32_norm(1, QKV, 3 * x.D, QKV, 3 * x.D, w.qn_g, nullptr, M, x.D, 1, d.eps, st);
      f32_norm(1, QKV + x.D, 3 * x.D, QKV + x.D, 3 * x.D, w.kn_g, nullptr, M, x.D, 1, d.eps, st);
    } else if (d.qk_norm == EPD_QKNORM_PER_HEAD) {
      ProfScope ps(c, 4, st);
      f32_norm(1, QKV, 3 * x.D, QKV, 3 * x.D, w.qn_g, nullptr, (long)M * x.H, x.hd, x.H, d.eps, st);
      f32_norm(1, QKV + x.D, 3 * x.D, QKV + x.D, 3 * x.D, w.kn_g, nullptr, (long)M * x.H, x.hd, x.H, d.eps, st);
    }
    { ProfScope ps(c, 3, st); f32_attention(QKV, 3 * x.D, x.Ns, 0, QKV + x.D, QKV + 2 * x.D, 3 * x.D, O, x.D, T, x.Ns, x.H, x.hd, scale, st); }
    { ProfScope ps(c, 6, st); f32_gemm(EPI_BIAS_RESIDUAL, O, x.D, (const float*)w.o.W, w.o.b, X, x.D, nullptr, 1, M, x.D, x.D, st); }
    { ProfScope ps(c, 1, st); f32_norm(d.norm, X, x.D, Xn, x.D, w.n2_g, w.n2_b, M, x.D, 1, d.eps, st); }
    { ProfScope ps(c, 7, st); f32_gemm(act_epi, Xn, x.D, (const float*)w.fc1.W, w.fc1.b, Hd, x.F, nullptr, 1, M, x.F, x.D, st); }
    { ProfScope ps(c, 8, st); f32_gemm(EPI_BIAS_RESIDUAL, Hd, x.F, (const float*)w.fc2.W, w.fc2.b, X, x.D, nullptr, 1, M, x.D, x.F, st); }
  }
  if (d.final_norm && stage != STAGE_PROJECT) { ProfScope ps(c, 1, st); f32_norm(d.norm, X, x.D, X, x.D, c->fn_g, c->fn_b, M, x.D, 1, d.eps, st); }
  if (stage == STAGE_TRUNK) {
    ProfScope ps(c, 5, st);
    stream_to_blocks(X, x.D, xr, out, 0, x.D, c->d_rowmap, c->cur_block_tokens, Mpatch, st);
    HIP_TRY(c, hipGetLastError());
    return EPD_OK;
  }
  if (d.proj_kind == EPD_PROJ_RESAMPLER) {
    const Resampler& r = c->rs;
    const int E = r.E;
    float *kvraw = (float*)r.kvraw, *kin = (float*)r.kin, *vin = (float*)r.vin, *K = (float*)r.K, *V = (float*)r.V;
    float *Oq = (float*)r.O, *o2 = (float*)r.o2, *o3 = (float*)r.o3;
    const float* xin = X;
    { ProfScope ps(c, 5, st);
      if (xr.n) { f32_take_rows(X, xr, (float*)r.xin, Mpatch, x.D, st); xin = (const float*)r.xin; } }
    { ProfScope ps(c, 9, st);
      f32_gemm(EPI_BIAS, xin, x.D, (const float*)r.kv.W, nullptr, kvraw, E, nullptr, 1, Mpatch, E, x.D, st); }
    { ProfScope ps(c, 5, st);
      f32_norm(0, kvraw, E, vin, E, r.lnkv_g, r.lnkv_b, Mpatch, E, 1, d.eps, st);
      f32_add_rows(vin, r.pos, x.N, kin, Mpatch, E, st); }
    { ProfScope ps(c, 9, st);
      f32_gemm(EPI_BIAS, kin, E, (const float*)r.k.W, r.k.b, K, E, nullptr, 1, Mpatch, E, E, st);
      f32_gemm(EPI_BIAS, vin, E, (const float*)r.v.W, r.v.b, V, E, nullptr, 1, Mpatch, E, E, st); }
    { ProfScope ps(c, 3, st);
      f32_attention((const float*)r.qp, E, r.Q, 1, K, V, E, Oq, E, T, x.N, r.H, r.hd, 1.0f / sqrtf((float)r.hd), st); }
    { ProfScope ps(c, 9, st);
      f32_gemm(EPI_BIAS, Oq, E, (const float*)r.o.W, r.o.b, o2, E, nullptr, 1, Mo, E, E, st); }
    { ProfScope ps(c, 5, st); f32_norm(0, o2, E, o3, E, r.lnp_g, r.lnp_b, Mo, E, 1, d.eps, st); }
    { ProfScope ps(c, 9, st);
      f32_gemm(EPI_BIAS, o3, E, (const float*)r.proj.W, nullptr, out, x.Pout, nullptr, 1, Mo, E, E, st,
               c->cur_rowmap, c->cur_block_tokens); }
    HIP_TRY(c, hipGetLastError());
    return EPD_OK;
  }
  const float* pin = X;
  { ProfScope ps(c, 5, st);
    if (d.pixel_shuffle) { f32_shuffle(X, xr, Pin, T, x.g, x.D, st); pin = Pin; }
    else if (xr.n) { f32_take_rows(X, xr, Pin, Mpatch, x.D, st); pin = Pin; }
    if (d.proj_prenorm) { f32_norm(0, pin, x.Pin, Pin, x.Pin, c->pn_g, c->pn_b, Mo, x.Pin, 1, d.eps, st); pin = Pin; } }
  { ProfScope ps(c, 9, st);
    if (d.proj_kind == EPD_PROJ_LINEAR) {
      f32_gemm(EPI_BIAS, pin, x.Pin, (const float*)c->pa.W, c->pa.b, out, x.Pout, nullptr, 1, Mo, x.Pout, x.Pin, st,
               c->cur_rowmap, c->cur_block_tokens);
    } else {
      f32_gemm(EPI_BIAS_GELU_ERF, pin, x.Pin, (const float*)c->pa.W, c->pa.b, Pmid, x.Pmid, nullptr, 1, Mo, x.Pmid, x.Pin, st);
      f32_gemm(EPI_BIAS, Pmid, x.Pmid, (const float*)c->pb.W, c->pb.b, out, x.Pout, nullptr, 1, Mo, x.Pout, x.Pmid, st,
               c->cur_rowmap, c->cur_block_tokens);
    } }
  HIP_TRY(c, hipGetLastError());
  return EPD_OK;
}

// --------------------------------------------------------------------------
// one micro-batch, bf16 mode
// --------------------------------------------------------------------------
GemmParams gp(int epi, const void* A, long lda, const Linear& lin, int M) {
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.epi = epi; p.A = (const bf16_t*)A; p.lda = lda; p.W = (const bf16_t*)lin.W; p.bias = lin.b;
  p.M = M; p.N = lin.N; p.K = lin.K; p.Npad = lin.Npad; p.n_pos = 1;
  return p;
}

epd_status run_bf16(epd_ctx* c, const float* tiles, int T, bf16_t* out, hipStream_t st, int stage) {
  const epd_model_desc& d = c->d;
  const Dims& x = c->x;
  const int M = T * x.Ns, Mo = T * x.N_out, Mpatch = T * x.N;
  const SliceRows xr = x.xrows();
  float* X = c->X;
  bf16_t* Xn = (bf16_t*)c->Xn; bf16_t* QK = (bf16_t*)c->QKV; bf16_t* VT = (bf16_t*)c->VT; bf16_t* O = (bf16_t*)c->O;
  bf16_t* Hd = (bf16_t*)c->Hd; bf16_t* Ape = (bf16_t*)c->Ape; bf16_t* Pin = (bf16_t*)c->Pin; bf16_t* Pmid = (bf16_t*)c->Pmid;
  const int act_epi = d.act == EPD_ACT_GELU_ERF ? EPI_BIAS_GELU_ERF : EPI_BIAS_GELU_TANH;
  const long ld_qk = 2L * c->Dq;

  if (stage == STAGE_PROJECT) {
    ProfScope ps(c, 5, st);
    blocks_to_stream(c->cur_in_pool, 1, x.D, c->d_rowmap, c->cur_block_tokens, X, x.D, xr, Mpatch, st);
  } else {
    ProfScope ps(c, 0, st);
    bf16_im2col(tiles, Ape, c->Kp_k, T, x.S, x.p, st);
    GemmParams p = gp(EPI_BIAS_POS, Ape, c->Kp_k, c->pe, Mpatch);
    p.R = X; p.ldr = x.D; p.pos = c->pos + (long)x.cls * x.D; p.n_pos = x.N; p.xrows = xr;
    HIP_TRY(c, bf16_gemm(p, st));
    if (x.Ns != x.N) fill_slice_rows(X, x.D, T, x.Ns, x.Nt, c->cls, c->pos, st); }
  const int n_layers = stage == STAGE_PROJECT ? 0 : x.L;
  const bool fold = c->fold;
  // folded pre-norm of a product over the bf16 copy of the stream
  const bool wide = fold && c->stats1 != nullptr;
  auto with_norm = [&](GemmParams& p, const float* colsum) {
    if (!fold) return;
    p.stats = wide ? c->stats1 : c->stats; p.colsum = colsum;
    p.n_part = wide ? 1 : c->n_part; p.stat_group = wide ? x.D : STAT_GROUP; p.norm_dim = x.D;
    p.norm_rms = d.norm == EPD_NORM_RMSNORM ? 1 : 0; p.norm_eps = d.eps;
  };
  // wide rows: the emitted pairs become one pair per row in front of the products that read them
  auto combine = [&]() { if (wide) { ProfScope ps(c, 1, st); bf16_combine_stats(c->stats, M, c->n_part, x.D, c->stats1, st); } };
  const bool copy = c->norm_mode == NORM_COPY;
  // residual product that also leaves bf16(x) of the rows it updates (and, folded norms, their statistics)
  auto with_emit = [&](GemmParams& p, bool wanted) {
    if (!(fold || copy) || !wanted) return;
    p.xb = Xn; p.ldxb = c->D_k;
    if (fold) { p.stats_out = c->stats; p.n_part_out = c->n_part; }
  };
  // pre-norm as a kernel of its own: from the fp32 stream, or in place on the bf16 rows a residual epilogue left
  auto norm_kernel = [&](const float* g, const float* b, bool from_stream) {
    if (fold) return;
    ProfScope ps(c, 1, st);
    if (from_stream) {
      RowOpParams r{d.norm, X, x.D, Xn, c->D_k, g, b, M, x.D, 0, x.g, x.D, d.eps};
      bf16_rowop(r, st);
    } else {
      bf16_norm_rows(Xn, c->D_k, g, b, M, x.D, d.norm, d.eps, st);
    }
  };
  // MXFP8 operands (epd_model_desc::mx_fp8): the converted rows live where the bf16 ones would, codes first,
  // their scale words behind them (a bf16 buffer of Mp rows holds both)
  unsigned char* XnQ = (unsigned char*)c->Xn; unsigned* SXn = (unsigned*)(XnQ + (size_t)c->Mp * c->D_k);
  unsigned char* HdQ = (unsigned char*)c->Hd; unsigned* SHd = (unsigned*)(HdQ + (size_t)c->Mp * c->F_k);
  auto mx_norm = [&](const float* g, const float* b) -> hipError_t {
    ProfScope ps(c, 1, st);
    MxRowParams r;
    memset(&r, 0, sizeof(r));
    r.kind = d.norm; r.in = X; r.ld_in = x.D; r.gamma = g; r.beta = b; r.eps = d.eps; r.rows = M; r.dim = x.D;
    r.codes = XnQ; r.ld_codes = c->D_k; r.scales = SXn; r.ld_scales = c->Mp;
    return mx_rows(r, st);
  };
  auto mxp = [&](int epi, const unsigned char* A, long lda, const unsigned* SA, const MxLinear& lin) {
    MxGemmParams p;
    memset(&p, 0, sizeof(p));
    p.epi = epi; p.A = A; p.lda = lda; p.SA = SA; p.sa_ld = c->Mp; p.W = lin.W; p.SW = lin.SW; p.bias = lin.b; p.cscale = lin.cs;
    p.M = M; p.N = lin.N; p.K = lin.K; p.Npad = lin.Npad;
    return p;
  };
  if (fold && n_layers > 0) {   // rows written by the embedding: the only pass of this kind in the call
    ProfScope ps(c, 1, st);
    bf16_row_stats(X, x.D, M, x.D, Xn, c->D_k, c->stats, c->n_part, st);
  }
  if (n_layers > 0) combine();
  for (int l = 0; l < n_layers; ++l) {
    const LayerW& w = c->layers[l];
    if (c->mx) {
      HIP_TRY(c, mx_norm(w.n1_g, w.n1_b));
      { ProfScope ps(c, 2, st);
        MxGemmParams p = mxp(EPI_BIAS, XnQ, c->D_k, SXn, w.mqkv);
        p.C = QK; p.ldc = ld_qk;
        HIP_TRY(c, mx_gemm(p, st)); }
      { ProfScope ps(c, 2, st);
        MxGemmParams pv = mxp(EPI_VT, XnQ, c->D_k, SXn, w.mv);
        pv.VT = VT; pv.hd_pad = c->hd_pad; pv.heads = x.H; pv.n_tok = x.Ns;
        HIP_TRY(c, mx_gemm(pv, st)); }
    } else {
    norm_kernel(w.n1_g, w.n1_b, !copy || l == 0);   // the first layer's rows come from the embedding
    bool paired = false;
    { ProfScope ps(c, 2, st);
      GemmParams p = gp(EPI_BIAS, Xn, c->D_k, w.qkv, M);
      p.C = QK; p.ldc = ld_qk;
      with_norm(p, w.qkv_cs);
      // a slice alone: the value projection rides in the same launch (its weights follow the q/k projection's)
      GemmParams pp = p;
      pp.n2 = w.v.N; pp.n2_pad = w.v.Npad; pp.VT = VT; pp.hd_pad = c->hd_pad; pp.heads = x.H; pp.n_tok = x.Ns;
      paired = (const bf16_t*)w.v.W == (const bf16_t*)w.qkv.W + (size_t)w.qkv.Npad * w.qkv.K && w.v.b == w.qkv.b + w.qkv.Npad &&
               bf16_gemm_pair_fits(pp);
      HIP_TRY(c, bf16_gemm(paired ? pp : p, st)); }
    if (!paired) { ProfScope ps(c, 2, st);
      GemmParams pv = gp(EPI_VT, Xn, c->D_k, w.v, M);
      pv.VT = VT; pv.hd_pad = c->hd_pad; pv.heads = x.H; pv.n_tok = x.Ns;
      with_norm(pv, w.v_cs);
      HIP_TRY(c, bf16_gemm(pv, st)); }
    }
    if (d.qk_norm == EPD_QKNORM_FULL) {
      ProfScope ps(c, 4, st);
      bf16_qknorm(QK, ld_qk, c->Dq, w.qn_g, w.kn_g, M, c->Dq, 1, x.D, d.eps, st);
    } else if (d.qk_norm == EPD_QKNORM_PER_HEAD) {
      ProfScope ps(c, 4, st);
      bf16_qknorm(QK, ld_qk, c->Dq, w.qn_g, w.kn_g, (long)M * x.H, c->hd_pad, x.H, x.hd, d.eps, st);
    }
    if (c->mx_o) {
      // the out-projection's operand as MXFP8: converted inside the attention kernel's output store when a head is
      // whole blocks of 32 (64, 96, 128), by a pass over the bf16 output otherwise (72)
      unsigned char* OQ = (unsigned char*)c->OQ; unsigned* SO = (unsigned*)(OQ + (size_t)c->Mp * c->Dq_k);
      const bool fused = c->hd_pad % 32 == 0;
      { ProfScope ps(c, 3, st);
        HIP_TRY(c, bf16_attention(QK, QK + c->Dq, VT, O, T, x.Ns, x.Nt, x.Ns, 0, x.H, c->hd_pad, ld_qk, c->Dq_k, st,
                                  fused ? OQ : nullptr, fused ? SO : nullptr, c->Mp));
        if (!fused) {
          MxRowParams r;
          memset(&r, 0, sizeof(r));
          r.kind = 2; r.in = O; r.ld_in = c->Dq_k; r.in_bf16 = 1; r.rows = M; r.dim = c->Dq_k;
          r.codes = OQ; r.ld_codes = c->Dq_k; r.scales = SO; r.ld_scales = c->Mp;
          HIP_TRY(c, mx_rows(r, st));
        } }
      { ProfScope ps(c, 6, st);
        MxGemmParams p = mxp(EPI_BIAS_RESIDUAL, OQ, c->Dq_k, SO, w.mo);
        p.R = X; p.ldr = x.D;
        HIP_TRY(c, mx_gemm(p, st)); }
    } else {
    { ProfScope ps(c, 3, st);
      HIP_TRY(c, bf16_attention(QK, QK + c->Dq, VT, O, T, x.Ns, x.Nt, x.Ns, 0, x.H, c->hd_pad, ld_qk, c->Dq_k, st)); }
    { ProfScope ps(c, 6, st);
      GemmParams p = gp(EPI_BIAS_RESIDUAL, O, c->Dq_k, w.o, M);
      p.R = X; p.ldr = x.D;
      with_emit(p, true);
      HIP_TRY(c, bf16_gemm(p, st)); }
    }
    combine();
    if (c->mx) {
      HIP_TRY(c, mx_norm(w.n2_g, w.n2_b));
      { ProfScope ps(c, 7, st);
        MxGemmParams p = mxp(act_epi, XnQ, c->D_k, SXn, w.mfc1);
        p.Cq = HdQ; p.ldcq = c->F_k; p.ncq = c->F_k; p.SC = SHd; p.sc_ld = c->Mp;
        HIP_TRY(c, mx_gemm(p, st)); }
      { ProfScope ps(c, 8, st);
        MxGemmParams p2 = mxp(EPI_BIAS_RESIDUAL, HdQ, c->F_k, SHd, w.mfc2);
        p2.R = X; p2.ldr = x.D;
        HIP_TRY(c, mx_gemm(p2, st)); }
      continue;
    }
    norm_kernel(w.n2_g, w.n2_b, !copy);
    { ProfScope ps(c, 7, st);
      GemmParams p = gp(act_epi, Xn, c->D_k, w.fc1, M);
      p.C = Hd; p.ldc = c->F_k;
      with_norm(p, w.fc1_cs);
      HIP_TRY(c, bf16_gemm(p, st)); }
    { ProfScope ps(c, 8, st);
      GemmParams p2 = gp(EPI_BIAS_RESIDUAL, Hd, c->F_k, w.fc2, M);
      p2.R = X; p2.ldr = x.D;
      with_emit(p2, l + 1 < n_layers);   // the next layer's first norm; nothing reads it after the last layer
      HIP_TRY(c, bf16_gemm(p2, st)); }
    if (l + 1 < n_layers) combine();
  }
  if (d.final_norm && stage != STAGE_PROJECT) { ProfScope ps(c, 1, st); f32_norm(d.norm, X, x.D, X, x.D, c->fn_g, c->fn_b, M, x.D, 1, d.eps, st); }
  if (stage == STAGE_TRUNK) {
    ProfScope ps(c, 5, st);
    stream_to_blocks(X, x.D, xr, out, 1, x.D, c->d_rowmap, c->cur_block_tokens, Mpatch, st);
    HIP_TRY(c, hipGetLastError());
    return EPD_OK;
  }
  if (d.proj_kind == EPD_PROJ_RESAMPLER) {
    const Resampler& r = c->rs;
    bf16_t *xin = (bf16_t*)r.xin, *kvraw = (bf16_t*)r.kvraw, *kin = (bf16_t*)r.kin, *vin = (bf16_t*)r.vin, *K = (bf16_t*)r.K;
    bf16_t *Oq = (bf16_t*)r.O, *o2 = (bf16_t*)r.o2, *o3 = (bf16_t*)r.o3;
    { ProfScope ps(c, 5, st);   // the patch rows of the stream as bf16
      RowOpParams ro{2, X, x.D, xin, c->D_k, nullptr, nullptr, Mpatch, x.D, 0, x.g, x.D, d.eps, xr};
      bf16_rowop(ro, st); }
    { ProfScope ps(c, 9, st);
      GemmParams p = gp(EPI_BIAS, xin, c->D_k, r.kv, Mpatch);
      p.C = kvraw; p.ldc = r.E_k;
      HIP_TRY(c, bf16_gemm(p, st)); }
    { ProfScope ps(c, 5, st);   // values LN_kv(kv), keys LN_kv(kv) + pos
      bf16_ln_rows(kvraw, r.E_k, r.lnkv_g, r.lnkv_b, d.eps, vin, r.E_k, kin, r.pos, x.N, Mpatch, r.E, st); }
    { ProfScope ps(c, 9, st);
      GemmParams pk = gp(EPI_BIAS, kin, r.E_k, r.k, Mpatch);
      pk.C = K; pk.ldc = r.Eq_k;
      HIP_TRY(c, bf16_gemm(pk, st));
      GemmParams pv = gp(EPI_VT, vin, r.E_k, r.v, Mpatch);
      pv.VT = (bf16_t*)r.V; pv.hd_pad = r.hd_pad; pv.heads = r.H; pv.n_tok = x.N;
      HIP_TRY(c, bf16_gemm(pv, st)); }
    { ProfScope ps(c, 3, st);
      HIP_TRY(c, bf16_attention((const bf16_t*)r.qp, K, (const bf16_t*)r.V, Oq, T, x.N, x.N, r.Q, 1, r.H, r.hd_pad, r.Eq_k, r.Eq_k, st)); }
    { ProfScope ps(c, 9, st);
      GemmParams p = gp(EPI_BIAS, Oq, r.Eq_k, r.o, Mo);
      p.C = o2; p.ldc = r.E_k;
      HIP_TRY(c, bf16_gemm(p, st)); }
    { ProfScope ps(c, 5, st);
      bf16_ln_rows(o2, r.E_k, r.lnp_g, r.lnp_b, d.eps, o3, r.E_k, nullptr, nullptr, 1, Mo, r.E, st); }
    { ProfScope ps(c, 9, st);
      GemmParams p = gp(EPI_BIAS, o3, r.E_k, r.proj, Mo);
      p.C = out; p.ldc = x.Pout; p.row_map = c->cur_rowmap; p.block_tokens = c->cur_block_tokens;
      HIP_TRY(c, bf16_gemm(p, st)); }
    HIP_TRY(c, hipGetLastError());
    return EPD_OK;
  }
  { ProfScope ps(c, 5, st);
    RowOpParams r{d.proj_prenorm ? 0 : 2, X, x.D, Pin, c->Pin_k, c->pn_g, c->pn_b, Mo, x.Pin, d.pixel_shuffle, x.g, x.D, d.eps, xr};
    bf16_rowop(r, st); }
  if (d.proj_kind == EPD_PROJ_LINEAR) {
      ProfScope ps(c, 9, st);
      GemmParams p = gp(EPI_BIAS, Pin, c->Pin_k, c->pa, Mo);
      p.C = out; p.ldc = x.Pout; p.row_map = c->cur_rowmap; p.block_tokens = c->cur_block_tokens;
      HIP_TRY(c, bf16_gemm(p, st));
  } else {
    { ProfScope ps(c, 9, st);
      GemmParams p = gp(EPI_BIAS_GELU_ERF, Pin, c->Pin_k, c->pa, Mo);
      p.C = Pmid; p.ldc = c->Pmid_k;
      HIP_TRY(c, bf16_gemm(p, st)); }
    { ProfScope ps(c, 9, st);
      GemmParams p2 = gp(EPI_BIAS, Pmid, c->Pmid_k, c->pb, Mo);
      p2.C = out; p2.ldc = x.Pout; p2.row_map = c->cur_rowmap; p2.block_tokens = c->cur_block_tokens;
      HIP_TRY(c, bf16_gemm(p2, st)); }
  }
  HIP_TRY(c, hipGetLastError());
  return EPD_OK;
}

// One call over slices [b, e) in micro-batches.
//   STAGE_FULL, block_map null: `out` is the contiguous token cache of the packed batch.
//   STAGE_FULL, block_map set:  `out` is a paged pool; block_map[i] is the physical block of logical
//                               block i of the packed batch's output rows (N_out rows per slice).
//   STAGE_TRUNK:   `out` is a paged pool of [hidden]-wide tokens; block_map covers the N rows per slice
//                  of slices [b, e) only, starting at slice b.
//   STAGE_PROJECT: `tiles` unused; `in_pool` + block_map (N rows per slice, slices [b, e)) are the input
//                  and `out` is the contiguous merged token buffer (row 0 = first token of slice b).
epd_status encode_range_impl(epd_ctx* c, const float* tiles, int32_t n_total, int32_t b, int32_t e, void* out,
                             hipStream_t st, const int32_t* block_map = nullptr, int block_tokens = 1,
                             int stage = STAGE_FULL, const void* in_pool = nullptr) {
  if (b < 0 || e < b || e > n_total) {
    set_err(c->err, sizeof(c->err), "tile range [%d, %d) is not inside [0, %d]", b, e, n_total);
    return EPD_ERR_OFFSETS;
  }
  if (e == b) return EPD_OK;
  if ((stage != STAGE_PROJECT && !tiles) || !out) { set_err(c->err, sizeof(c->err), "tiles / out_token_cache is null"); return EPD_ERR_INVALID_ARG; }
  if (((uintptr_t)tiles & 15) || ((uintptr_t)out & 15)) {
    set_err(c->err, sizeof(c->err), "tiles and out_token_cache must be 16-byte aligned");
    return EPD_ERR_INVALID_ARG;
  }
  const Dims& x = c->x;
  const size_t tile_elems = (size_t)3 * x.S * x.S;
  const size_t out_row_bytes = (size_t)x.Pout * (c->bf16 ? 2 : 4);
  // rows per slice the block map speaks about, and the slice its entry 0 belongs to
  const int map_rows = stage == STAGE_FULL ? x.N_out : x.N;
  const int map_origin = stage == STAGE_FULL ? 0 : b;
  const int out_origin = stage == STAGE_PROJECT ? b : 0;
  if (c->prof) { c->ev_used = 0; c->ev_family.clear(); c->ev_kernels.clear(); }
  for (int t0 = b; t0 < e; t0 += c->mb) {
    const int T = (e - t0) < c->mb ? (e - t0) : c->mb;
    const float* tp = tiles ? tiles + (size_t)t0 * tile_elems : nullptr;
    char* op = (char*)out + (size_t)(t0 - out_origin) * x.N_out * out_row_bytes;
    c->cur_rowmap = nullptr;
    c->cur_block_tokens = 1;
    c->cur_in_pool = in_pool;
    if (block_map) {
      // this micro-batch's slice of the map; the copy is stream-ordered behind the previous micro-batch
      const size_t first = (size_t)(t0 - map_origin) * map_rows / block_tokens, count = (size_t)T * map_rows / block_tokens;
      const int turn = c->rowmap_turn;
      c->rowmap_turn ^= 1;
      if (c->rowmap_pending[turn]) HIP_TRY(c, hipEventSynchronize(c->ev_rowmap[turn]));   // its previous upload has left the staging
      memcpy(c->h_rowmap[turn], block_map + first, count * sizeof(int));
      HIP_TRY(c, hipMemcpyAsync(c->d_rowmap, c->h_rowmap[turn], count * sizeof(int), hipMemcpyHostToDevice, st));
      HIP_TRY(c, hipEventRecord(c->ev_rowmap[turn], st));
      c->rowmap_pending[turn] = true;
      c->cur_block_tokens = block_tokens;
      if (stage == STAGE_FULL) c->cur_rowmap = c->d_rowmap;   // final GEMM scatters through the map
      if (stage != STAGE_PROJECT) op = (char*)out;            // paged output: `out` is the pool base
    }
    epd_status s = c->bf16 ? run_bf16(c, tp, T, (bf16_t*)op, st, stage) : run_f32(c, tp, T, (float*)op, st, stage);
    c->cur_rowmap = nullptr;
    c->cur_in_pool = nullptr;
    if (s != EPD_OK) return s;
    c->last_rows = (long)T * x.Nt;
  }
  return EPD_OK;
}

}  // namespace

// ============================================================================
// exported functions
// ============================================================================
extern "C" {

int32_t epd_weight_count(const epd_model_desc* desc) {
  epd_status s = check_desc(desc, g_err, sizeof(g_err));
  if (s != EPD_OK) return (int32_t)s;
  return (int32_t)build_index(*desc).specs.size();
}

epd_status epd_check_desc(const epd_model_desc* desc, char* errbuf, int32_t errbuf_len) {
  epd_status s = check_desc(desc, g_err, sizeof(g_err));
  if (errbuf && errbuf_len > 0) { strncpy(errbuf, s == EPD_OK ? "" : g_err, errbuf_len - 1); errbuf[errbuf_len - 1] = 0; }
  return s;
}

epd_status epd_check_offsets(const int32_t* off, int32_t n_requests, int32_t n_tiles) {
  if (n_requests < 0 || n_tiles < 0) { set_err(g_err, sizeof(g_err), "negative count"); return EPD_ERR_OFFSETS; }
  if (!off) { set_err(g_err, sizeof(g_err), "tile_offsets_per_request is null"); return EPD_ERR_INVALID_ARG; }
  if (off[0] != 0) { set_err(g_err, sizeof(g_err), "tile_offsets[0] must be 0, got %d", off[0]); return EPD_ERR_OFFSETS; }
  for (int r = 0; r < n_requests; ++r)
    if (off[r + 1] < off[r]) { set_err(g_err, sizeof(g_err), "tile_offsets decrease at request %d", r); return EPD_ERR_OFFSETS; }
  if (off[n_requests] != n_tiles) {
    set_err(g_err, sizeof(g_err), "tile_offsets[n_requests] = %d but n_tiles = %d", off[n_requests], n_tiles);
    return EPD_ERR_OFFSETS;
  }
  return EPD_OK;
}

epd_status epd_create(const epd_model_desc* desc, const epd_weights* weights, void* hip_stream, epd_ctx** out) {
  if (!out) { set_err(g_err, sizeof(g_err), "out is null"); return EPD_ERR_INVALID_ARG; }
  *out = nullptr;
  epd_status s = check_desc(desc, g_err, sizeof(g_err));
  if (s != EPD_OK) return s;
  if (!weights || !weights->tensors) { set_err(g_err, sizeof(g_err), "weights is null"); return EPD_ERR_INVALID_ARG; }
  const WeightIndex wi = build_index(*desc);
  if (weights->n_tensors != (int32_t)wi.specs.size()) {
    set_err(g_err, sizeof(g_err), "expected %d weight tensors, got %d", (int)wi.specs.size(), weights->n_tensors);
    return EPD_ERR_INVALID_ARG;
  }
  for (int i = 0; i < weights->n_tensors; ++i)
    if (!weights->tensors[i] || ((uintptr_t)weights->tensors[i] & 3)) {
      set_err(g_err, sizeof(g_err), "weight tensor %d is null or misaligned", i);
      return EPD_ERR_INVALID_ARG;
    }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) {
    set_err(g_err, sizeof(g_err), "no HIP device available");
    return EPD_ERR_HIP;
  }
  epd_ctx* c = new epd_ctx();
  c->d = *desc; c->x = dims_of(*desc); c->bf16 = desc->dtype == EPD_DTYPE_BF16; c->err[0] = 0;
  s = build_ctx(c, weights, (hipStream_t)hip_stream);
  if (s != EPD_OK) {
    strncpy(g_err, c->err, sizeof(g_err) - 1);
    epd_destroy(c);
    return s;
  }
  *out = c;
  return EPD_OK;
}

epd_status epd_encode(epd_ctx* ctx, const float* tiles, int32_t n_tiles, const int32_t* off, int32_t n_requests,
                      void* out, void* hip_stream) {
  if (!ctx) { set_err(g_err, sizeof(g_err), "ctx is null"); return EPD_ERR_INVALID_ARG; }
  epd_status s = epd_check_offsets(off, n_requests, n_tiles);
  if (s != EPD_OK) { strncpy(ctx->err, g_err, sizeof(ctx->err) - 1); return s; }
  return encode_range_impl(ctx, tiles, n_tiles, 0, n_tiles, out, (hipStream_t)hip_stream);
}

epd_status epd_encode_range(epd_ctx* ctx, const float* tiles, int32_t n_tiles_total, int32_t tile_begin,
                            int32_t tile_end, void* out, void* hip_stream) {
  if (!ctx) { set_err(g_err, sizeof(g_err), "ctx is null"); return EPD_ERR_INVALID_ARG; }
  return encode_range_impl(ctx, tiles, n_tiles_total, tile_begin, tile_end, out, (hipStream_t)hip_stream);
}

}  // extern "C"

namespace {
// cache shape against a token width, and `count` table entries against the block manager
// (range, allocated, and for a table the call writes through: no block listed twice)
epd_status check_cache_table(epd_ctx* ctx, epd_mm_cache* cache, int token_dim, int rows_per_slice,
                             const int32_t* table, long count, bool written) {
  if (!cache || !table) { set_err(ctx->err, sizeof(ctx->err), "cache / block_table is null"); return EPD_ERR_INVALID_ARG; }
  if (!cache->pool || cache->token_dim != token_dim || cache->dtype != ctx->d.dtype) {
    set_err(ctx->err, sizeof(ctx->err), "cache token width / dtype (%d, %d) does not match the encoder (%d, %d)",
            cache->token_dim, cache->dtype, token_dim, ctx->d.dtype);
    return EPD_ERR_SHAPE;
  }
  if (rows_per_slice % cache->block_tokens) {
    set_err(ctx->err, sizeof(ctx->err), "tokens per slice %d is not a multiple of the block size %d", rows_per_slice,
            cache->block_tokens);
    return EPD_ERR_UNSUPPORTED;
  }
  for (long i = 0; i < count; ++i)
    if (table[i] < 0 || table[i] >= cache->n_blocks || !cache->used[table[i]]) {
      set_err(ctx->err, sizeof(ctx->err), "block table entry %ld (%d) is out of range or not allocated", i, table[i]);
      return EPD_ERR_OFFSETS;
    }
  if (written) {
    // two logical blocks on one physical block would overwrite each other: `mark` (all zero between calls)
    long dup = -1;
    for (long i = 0; i < count && dup < 0; ++i) {
      if (cache->mark[table[i]]) dup = i;
      else cache->mark[table[i]] = 1;
    }
    for (long i = 0; i < (dup < 0 ? count : dup); ++i) cache->mark[table[i]] = 0;
    if (dup >= 0) {
      set_err(ctx->err, sizeof(ctx->err), "block table entry %ld names block %d a second time", dup, table[dup]);
      return EPD_ERR_OFFSETS;
    }
  }
  return EPD_OK;
}
}  // namespace

extern "C" {

epd_status epd_encode_paged(epd_ctx* ctx, const float* tiles, int32_t n_tiles, const int32_t* off, int32_t n_requests,
                            epd_mm_cache* cache, const int32_t* block_table, const int32_t* block_table_offsets,
                            void* hip_stream) {
  if (!ctx) { set_err(g_err, sizeof(g_err), "ctx is null"); return EPD_ERR_INVALID_ARG; }
  epd_status s = epd_check_offsets(off, n_requests, n_tiles);
  if (s != EPD_OK) { strncpy(ctx->err, g_err, sizeof(ctx->err) - 1); return s; }
  if (n_tiles == 0) return EPD_OK;
  if (!cache || !block_table || !block_table_offsets) {
    set_err(ctx->err, sizeof(ctx->err), "cache / block_table / block_table_offsets is null");
    return EPD_ERR_INVALID_ARG;
  }
  const Dims& x = ctx->x;
  s = check_cache_table(ctx, cache, x.Pout, x.N_out, block_table, 0, false);   // shape only; the entries follow
  if (s != EPD_OK) return s;
  const int bpt = x.N_out / cache->block_tokens;  // blocks per slice
  if (block_table_offsets[0] != 0) { set_err(ctx->err, sizeof(ctx->err), "block_table_offsets[0] must be 0"); return EPD_ERR_OFFSETS; }
  for (int r = 0; r < n_requests; ++r) {
    const long want = (long)(off[r + 1] - off[r]) * bpt;
    if (block_table_offsets[r + 1] - block_table_offsets[r] != want) {
      set_err(ctx->err, sizeof(ctx->err), "request %d needs %ld blocks, its block table holds %d", r, want,
              block_table_offsets[r + 1] - block_table_offsets[r]);
      return EPD_ERR_OFFSETS;
    }
  }
  const long total = (long)n_tiles * bpt;
  s = check_cache_table(ctx, cache, x.Pout, x.N_out, block_table, total, true);
  if (s != EPD_OK) return s;
  // requests are contiguous in slice order and own whole blocks, so the concatenated
  // per-request tables are the logical-block -> physical-block map of the packed batch
  return encode_range_impl(ctx, tiles, n_tiles, 0, n_tiles, cache->pool, (hipStream_t)hip_stream, block_table,
                           cache->block_tokens);
}


epd_status epd_encode_trunk_paged(epd_ctx* ctx, const float* tiles, int32_t n_tiles_total, int32_t tile_begin,
                                  int32_t tile_end, epd_mm_cache* cache, const int32_t* block_table,
                                  void* hip_stream) {
  if (!ctx) { set_err(g_err, sizeof(g_err), "ctx is null"); return EPD_ERR_INVALID_ARG; }
  if (tile_begin < 0 || tile_end < tile_begin || tile_end > n_tiles_total) {
    set_err(ctx->err, sizeof(ctx->err), "tile range [%d, %d) is not inside [0, %d]", tile_begin, tile_end, n_tiles_total);
    return EPD_ERR_OFFSETS;
  }
  if (tile_end == tile_begin) return EPD_OK;
  const Dims& x = ctx->x;
  const long count = cache && cache->block_tokens > 0 ? (long)(tile_end - tile_begin) * (x.N / cache->block_tokens) : 0;
  epd_status s = check_cache_table(ctx, cache, x.D, x.N, block_table, count, true);
  if (s != EPD_OK) return s;
  return encode_range_impl(ctx, tiles, n_tiles_total, tile_begin, tile_end, cache->pool, (hipStream_t)hip_stream,
                           block_table, cache->block_tokens, STAGE_TRUNK);
}

epd_status epd_project_merge(epd_ctx* ctx, const epd_mm_cache* cache, const int32_t* block_table, int32_t n_tiles,
                             void* out_tokens, void* hip_stream) {
  if (!ctx) { set_err(g_err, sizeof(g_err), "ctx is null"); return EPD_ERR_INVALID_ARG; }
  if (n_tiles < 0) { set_err(ctx->err, sizeof(ctx->err), "n_tiles is negative"); return EPD_ERR_OFFSETS; }
  if (n_tiles == 0) return EPD_OK;
  const Dims& x = ctx->x;
  const long count = cache && cache->block_tokens > 0 ? (long)n_tiles * (x.N / cache->block_tokens) : 0;
  epd_status s = check_cache_table(ctx, const_cast<epd_mm_cache*>(cache), x.D, x.N, block_table, count, false);
  if (s != EPD_OK) return s;
  return encode_range_impl(ctx, nullptr, n_tiles, 0, n_tiles, out_tokens, (hipStream_t)hip_stream, block_table,
                           cache->block_tokens, STAGE_PROJECT, cache->pool);
}

int64_t epd_tokens_per_tile(const epd_ctx* ctx) { return ctx ? ctx->x.N_out : -1; }
int64_t epd_out_dim(const epd_ctx* ctx) { return ctx ? ctx->x.Pout : -1; }
const char* epd_last_error(const epd_ctx* ctx) { return ctx ? ctx->err : g_err; }

void epd_destroy(epd_ctx* ctx) {
  if (!ctx) return;
  for (void* p : ctx->allocs) (void)hipFree(p);
  for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
  for (int i = 0; i < 2; ++i) {
    if (ctx->h_rowmap[i]) (void)hipHostFree(ctx->h_rowmap[i]);
    if (ctx->ev_rowmap[i]) (void)hipEventDestroy(ctx->ev_rowmap[i]);
  }
  delete ctx;
}

epd_status epd_debug_read_stream(epd_ctx* ctx, void* dst, int64_t rows, int64_t dst_bytes) {
  if (!ctx || !dst) return EPD_ERR_INVALID_ARG;
  const int64_t bytes = rows * ctx->x.D * 4;
  if (rows < 0 || rows > ctx->Mp || bytes > dst_bytes) return EPD_ERR_INVALID_ARG;
  HIP_TRY(ctx, hipDeviceSynchronize());
  // the stream keeps Ns rows per slice, the caller gets the Nt token rows of each slice back to back
  const Dims& x = ctx->x;
  const size_t tok_bytes = (size_t)x.Nt * x.D * 4, slice_bytes = (size_t)x.Ns * x.D * 4;
  const int64_t whole = rows / x.Nt, rest = rows % x.Nt;
  if (whole * x.Ns + rest > ctx->Mp) return EPD_ERR_INVALID_ARG;
  if (whole > 0) HIP_TRY(ctx, hipMemcpy2D(dst, tok_bytes, ctx->X, slice_bytes, tok_bytes, (size_t)whole, hipMemcpyDeviceToHost));
  if (rest > 0)
    HIP_TRY(ctx, hipMemcpy((char*)dst + whole * tok_bytes, (const char*)ctx->X + whole * slice_bytes, (size_t)rest * x.D * 4,
                           hipMemcpyDeviceToHost));
  return EPD_OK;
}

epd_status epd_op_gemm_bf16(const void* A, const void* W, const float* bias, void* C, int32_t M, int32_t N,
                            int32_t K, int32_t iters, float* ms_per_launch, void* hip_stream) {
  if (!A || !W || !C || M <= 0 || N <= 0 || K <= 0 || M % 256 || N % 128 || K % 128 || iters < 1) {
    set_err(g_err, sizeof(g_err), "epd_op_gemm_bf16: bad argument");
    return EPD_ERR_INVALID_ARG;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  if (bf16_gemm_init() != hipSuccess) return EPD_ERR_HIP;
  float* zb = nullptr;
  if (!bias) {
    if (hipMalloc((void**)&zb, (size_t)N * 4) != hipSuccess) return EPD_ERR_NOMEM;
    (void)hipMemsetAsync(zb, 0, (size_t)N * 4, st);
  }
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.epi = EPI_BIAS; p.A = (const bf16_t*)A; p.lda = K; p.W = (const bf16_t*)W; p.bias = bias ? bias : zb;
  p.M = M; p.N = N; p.K = K; p.Npad = N; p.C = (bf16_t*)C; p.ldc = N; p.n_pos = 1;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  hipError_t err = bf16_gemm(p, st);  // warm-up
  (void)hipEventRecord(e0, st);
  for (int i = 0; i < iters && err == hipSuccess; ++i) err = bf16_gemm(p, st);
  (void)hipEventRecord(e1, st);
  (void)hipEventSynchronize(e1);
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  if (ms_per_launch) *ms_per_launch = ms / iters;
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (zb) (void)hipFree(zb);
  if (err != hipSuccess) { set_err(g_err, sizeof(g_err), "gemm launch failed: %s", hipGetErrorString(err)); return EPD_ERR_HIP; }
  return EPD_OK;
}

epd_status epd_op_gemm_bf16_form(const void* A, const void* W, const float* bias, void* C, float* R, int32_t M,
                                 int32_t N, int32_t K, int32_t epi, int32_t form, void* hip_stream) {
  const bool residual = epi == EPI_BIAS_RESIDUAL;
  if (!A || !W || !bias || (residual ? !R : !C) || M <= 0 || N <= 0 || K <= 0 || N % 128 || K % 128 ||
      !(epi == EPI_BIAS || epi == EPI_BIAS_GELU_ERF || epi == EPI_BIAS_GELU_TANH || residual) ||
      !(form == 0 || form == 1 || form == 2 || form == 3 || (form >= 6 && form <= 12)) ||
      (form == 3 && K % 256) || (form >= 6 && form <= 10 && N % 256) || (form == 9 && residual) || (form == 10 && !residual) ||
      (form == 12 && (!residual || N % 192))) {
    set_err(g_err, sizeof(g_err), "epd_op_gemm_bf16_form: bad argument");
    return EPD_ERR_INVALID_ARG;
  }
  if (bf16_gemm_init() != hipSuccess) return EPD_ERR_HIP;
  hipStream_t st = (hipStream_t)hip_stream;
  // The kernels read whole 256-row tiles of A and of the residual stream (the library's own workspace is
  // padded that way).  The caller's buffers hold exactly M rows, so a ragged M runs on padded copies.
  const long Mp = ((long)M + 255) / 256 * 256;
  void* Ap = nullptr;
  float* Rp = nullptr;
  const bool pad_a = Mp != M, pad_r = residual;   // R also needs 256 floats of slack behind its last row
  auto fail = [&](epd_status code, const char* what) {
    if (Ap) (void)hipFree(Ap);
    if (Rp) (void)hipFree(Rp);
    set_err(g_err, sizeof(g_err), "epd_op_gemm_bf16_form: %s", what);
    return code;
  };
  if (pad_a) {
    if (hipMalloc(&Ap, (size_t)Mp * K * 2) != hipSuccess) return fail(EPD_ERR_NOMEM, "allocation failed");
    if (hipMemsetAsync(Ap, 0, (size_t)Mp * K * 2, st) != hipSuccess ||
        hipMemcpyAsync(Ap, A, (size_t)M * K * 2, hipMemcpyDeviceToDevice, st) != hipSuccess) return fail(EPD_ERR_HIP, "copy failed");
  }
  if (pad_r) {
    const size_t bytes = ((size_t)Mp * N + 256) * 4;
    if (hipMalloc((void**)&Rp, bytes) != hipSuccess) return fail(EPD_ERR_NOMEM, "allocation failed");
    if (hipMemsetAsync(Rp, 0, bytes, st) != hipSuccess ||
        hipMemcpyAsync(Rp, R, (size_t)M * N * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) return fail(EPD_ERR_HIP, "copy failed");
  }
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.epi = epi; p.cfg = form; p.A = (const bf16_t*)(pad_a ? Ap : A); p.lda = K; p.W = (const bf16_t*)W; p.bias = bias;
  p.M = M; p.N = N; p.K = K; p.Npad = N; p.C = (bf16_t*)C; p.ldc = N; p.R = pad_r ? Rp : R; p.ldr = N; p.n_pos = 1;
  const hipError_t err = bf16_gemm(p, st);
  if (err != hipSuccess) { fail(EPD_ERR_HIP, hipGetErrorString(err)); return EPD_ERR_HIP; }
  if (pad_r && hipMemcpyAsync(R, Rp, (size_t)M * N * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) return fail(EPD_ERR_HIP, "copy failed");
  if (pad_a || pad_r) {
    if (hipStreamSynchronize(st) != hipSuccess) return fail(EPD_ERR_HIP, "synchronise failed");
    if (Ap) (void)hipFree(Ap);
    if (Rp) (void)hipFree(Rp);
  }
  return EPD_OK;
}

epd_status epd_op_row_stats(const float* x, int64_t rows, int32_t dim, void* xb, float* stats, void* hip_stream) {
  if (!x || !xb || !stats || rows < 0 || dim <= 0 || dim % 4) return EPD_ERR_INVALID_ARG;
  bf16_row_stats(x, dim, rows, dim, (bf16_t*)xb, dim, stats, (dim + STAT_GROUP - 1) / STAT_GROUP, (hipStream_t)hip_stream);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}

epd_status epd_op_gemm_residual_stats(const void* A, const void* W, const float* bias, float* R, void* xb, float* stats,
                                      int32_t M, int32_t N, int32_t K, int32_t form, void* hip_stream) {
  if (!A || !W || !bias || !R || !xb || !stats || M <= 0 || M % 256 || N <= 0 || N % 128 || K <= 0 || K % 128 ||
      !(form == 0 || form == 1 || form == 2 || form == 3 || form == 6 || form == 7 || form == 8) || (form == 3 && K % 256) || (form >= 6 && N % 256)) {
    set_err(g_err, sizeof(g_err), "epd_op_gemm_residual_stats: bad argument");
    return EPD_ERR_INVALID_ARG;
  }
  if (bf16_gemm_init() != hipSuccess) return EPD_ERR_HIP;
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.epi = EPI_BIAS_RESIDUAL; p.cfg = form; p.A = (const bf16_t*)A; p.lda = K; p.W = (const bf16_t*)W; p.bias = bias;
  p.M = M; p.N = N; p.K = K; p.Npad = N; p.R = R; p.ldr = N; p.n_pos = 1;
  p.xb = (bf16_t*)xb; p.ldxb = N; p.stats_out = stats; p.n_part_out = N / STAT_GROUP;
  const hipError_t err = bf16_gemm(p, (hipStream_t)hip_stream);
  if (err != hipSuccess) { set_err(g_err, sizeof(g_err), "gemm launch failed: %s", hipGetErrorString(err)); return EPD_ERR_HIP; }
  return EPD_OK;
}

epd_status epd_op_norm_gemm_bf16(const float* x, const float* gamma, const float* beta, const void* W, const float* bias,
                                 void* C, int32_t M, int32_t N, int32_t D, float eps, int32_t epi, int32_t form,
                                 void* hip_stream) {
  if (!x || !gamma || !W || !bias || !C || M <= 0 || M % 256 || N <= 0 || N % 128 || D <= 0 || D % 128 ||
      !(epi == EPI_BIAS || epi == EPI_BIAS_GELU_ERF || epi == EPI_BIAS_GELU_TANH) ||
      !(form == 0 || form == 1 || form == 2 || form == 3 || form == 6 || form == 7 || form == 8 || form == 9) || (form == 3 && D % 256) || (form >= 6 && N % 256)) {
    set_err(g_err, sizeof(g_err), "epd_op_norm_gemm_bf16: bad argument");
    return EPD_ERR_INVALID_ARG;
  }
  if (bf16_gemm_init() != hipSuccess) return EPD_ERR_HIP;
  hipStream_t st = (hipStream_t)hip_stream;
  const int n_part = D / STAT_GROUP;
  bf16_t *xb = nullptr, *Wf = nullptr;
  float *stats = nullptr, *bf = nullptr, *cs = nullptr;
  auto done = [&](epd_status code) {
    (void)hipStreamSynchronize(st);
    for (void* q : {(void*)xb, (void*)Wf, (void*)stats, (void*)bf, (void*)cs}) if (q) (void)hipFree(q);
    return code;
  };
  if (hipMalloc((void**)&xb, (size_t)M * D * 2) != hipSuccess || hipMalloc((void**)&Wf, (size_t)N * D * 2) != hipSuccess ||
      hipMalloc((void**)&stats, (size_t)M * n_part * 8) != hipSuccess || hipMalloc((void**)&bf, (size_t)N * 4) != hipSuccess ||
      hipMalloc((void**)&cs, (size_t)N * 4) != hipSuccess) return done(EPD_ERR_NOMEM);
  if (hipMemcpyAsync(Wf, W, (size_t)N * D * 2, hipMemcpyDeviceToDevice, st) != hipSuccess ||
      hipMemcpyAsync(bf, bias, (size_t)N * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) return done(EPD_ERR_HIP);
  bf16_row_stats(x, D, M, D, xb, D, stats, n_part, st);
  float* stats1 = nullptr;
  if (n_part > STAT_REGS) {
    if (hipMalloc((void**)&stats1, (size_t)M * 8) != hipSuccess) return done(EPD_ERR_NOMEM);
    bf16_combine_stats(stats, M, n_part, D, stats1, st);
  }
  fold_norm_into_linear(Wf, N, D, D, gamma, beta, D, bf, cs, st);
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.epi = epi; p.cfg = form; p.A = xb; p.lda = D; p.W = Wf; p.bias = bf; p.M = M; p.N = N; p.K = D; p.Npad = N;
  p.C = (bf16_t*)C; p.ldc = N; p.n_pos = 1;
  p.stats = stats1 ? stats1 : stats; p.colsum = cs; p.n_part = stats1 ? 1 : n_part; p.stat_group = stats1 ? D : STAT_GROUP;
  p.norm_dim = D; p.norm_rms = beta ? 0 : 1; p.norm_eps = eps;
  const hipError_t err = bf16_gemm(p, st);
  const epd_status rc = err != hipSuccess ? EPD_ERR_HIP : (hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP);
  if (err != hipSuccess) set_err(g_err, sizeof(g_err), "gemm launch failed: %s", hipGetErrorString(err));
  (void)hipStreamSynchronize(st);
  if (stats1) (void)hipFree(stats1);
  return done(rc);
}

epd_status epd_op_attention_bf16(const void* q, const void* k, const void* vt, void* o, int32_t n_slices,
                                 int32_t n_tokens, int32_t n_keys, int32_t heads, int32_t hd_pad, int32_t ld_qk,
                                 void* hip_stream) {
  if (!q || !k || !vt || !o) return EPD_ERR_INVALID_ARG;
  if (n_tokens % 64) { set_err(g_err, sizeof(g_err), "epd_op_attention_bf16: n_tokens %% 64 != 0"); return EPD_ERR_UNSUPPORTED; }
  hipError_t e = bf16_attention((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)vt, (bf16_t*)o, n_slices,
                                n_tokens, n_keys, n_tokens, 0, heads, hd_pad, ld_qk, (long)heads * hd_pad, (hipStream_t)hip_stream);
  if (e != hipSuccess) { set_err(g_err, sizeof(g_err), "attention launch failed: %s", hipGetErrorString(e)); return e == hipErrorInvalidValue ? EPD_ERR_UNSUPPORTED : EPD_ERR_HIP; }
  return EPD_OK;
}

epd_status epd_op_attention_mx(const void* q, const void* k, const void* vt, void* codes, void* scales, int32_t n_slices,
                               int32_t n_tokens, int32_t n_keys, int32_t heads, int32_t hd_pad, int32_t ld_qk, void* hip_stream) {
  if (!q || !k || !vt || !codes || !scales) return EPD_ERR_INVALID_ARG;
  if (n_tokens % 64 || hd_pad % 32 || (heads * hd_pad) % 128) {
    set_err(g_err, sizeof(g_err), "epd_op_attention_mx: n_tokens %% 64, hd_pad %% 32 and heads * hd_pad %% 128 must be 0");
    return EPD_ERR_UNSUPPORTED;
  }
  const long rows = (long)n_slices * n_tokens;
  hipError_t e = bf16_attention((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)vt, nullptr, n_slices, n_tokens, n_keys,
                                n_tokens, 0, heads, hd_pad, ld_qk, (long)heads * hd_pad, (hipStream_t)hip_stream,
                                (unsigned char*)codes, (unsigned*)scales, rows);
  if (e != hipSuccess) { set_err(g_err, sizeof(g_err), "attention launch failed: %s", hipGetErrorString(e)); return e == hipErrorInvalidValue ? EPD_ERR_UNSUPPORTED : EPD_ERR_HIP; }
  return EPD_OK;
}

epd_status epd_op_mfma_probe(const void* A, const void* B, float* D, void* hip_stream) {
  if (!A || !B || !D) return EPD_ERR_INVALID_ARG;
  mfma_probe((const bf16_t*)A, (const bf16_t*)B, D, (hipStream_t)hip_stream);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}

epd_status epd_profile_enable(epd_ctx* ctx, int32_t on) {
  if (!ctx) return EPD_ERR_INVALID_ARG;
  if (on && ctx->ev.empty()) {
    ctx->ev.resize(16384);
    for (auto& e : ctx->ev) HIP_TRY(ctx, hipEventCreate(&e));
  }
  ctx->prof = on != 0;
  ctx->ev_used = 0;
  ctx->ev_family.clear();
  ctx->ev_kernels.clear();
  return EPD_OK;
}

epd_status epd_profile_read(epd_ctx* ctx, float* ms, int32_t* launches) {
  if (!ctx || !ms || !launches) return EPD_ERR_INVALID_ARG;
  HIP_TRY(ctx, hipDeviceSynchronize());
  for (int f = 0; f < EPD_PROF_FAMILIES; ++f) { ms[f] = 0.f; launches[f] = 0; }
  for (size_t i = 0; i < ctx->ev_family.size(); ++i) {
    float t = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&t, ctx->ev[2 * i], ctx->ev[2 * i + 1]));
    ms[ctx->ev_family[i]] += t;
    launches[ctx->ev_family[i]] += i < ctx->ev_kernels.size() ? ctx->ev_kernels[i] : 1;
  }
  return EPD_OK;
}

epd_status epd_op_mx_rows(const void* in, int32_t in_bf16, int64_t rows, int32_t dim, int32_t kind, const float* gamma,
                          const float* beta, float eps, void* codes, void* scales, void* hip_stream) {
  if (!in || !codes || !scales || rows <= 0 || dim <= 0 || dim % 128 || kind < 0 || kind > 2) {
    set_err(g_err, sizeof(g_err), "epd_op_mx_rows: bad argument (dim %% 128 == 0, kind 0..2)");
    return EPD_ERR_INVALID_ARG;
  }
  MxRowParams p;
  memset(&p, 0, sizeof(p));
  p.kind = kind; p.in = in; p.ld_in = dim; p.in_bf16 = in_bf16 ? 1 : 0; p.gamma = gamma; p.beta = beta; p.eps = eps;
  p.rows = rows; p.dim = dim; p.codes = (unsigned char*)codes; p.ld_codes = dim; p.scales = (unsigned*)scales; p.ld_scales = rows;
  const hipError_t e = mx_rows(p, (hipStream_t)hip_stream);
  if (e != hipSuccess) { set_err(g_err, sizeof(g_err), "epd_op_mx_rows: %s", hipGetErrorString(e)); return e == hipErrorInvalidValue ? EPD_ERR_INVALID_ARG : EPD_ERR_HIP; }
  return EPD_OK;
}

epd_status epd_op_mx_gemm(int32_t epi, const void* A, const void* SA, const void* W, const void* SW, const float* bias,
                          const float* cscale, int32_t M, int32_t N, int32_t K, void* C, float* R, void* Cq, void* SC,
                          int32_t n_tok, int32_t heads, int32_t hd_pad, void* hip_stream) {
  if (!A || !SA || !W || !SW || !bias || M <= 0 || M % 256 || N <= 0 || N % 256 || K <= 0 || K % 128) {
    set_err(g_err, sizeof(g_err), "epd_op_mx_gemm: bad argument (M %% 256, N %% 256, K %% 128)");
    return EPD_ERR_INVALID_ARG;
  }
  if (epi == EPI_VT && (n_tok <= 0 || heads <= 0 || hd_pad <= 0 || M % n_tok || heads * hd_pad != N)) return EPD_ERR_INVALID_ARG;
  if (mx_gemm_init() != hipSuccess) return EPD_ERR_HIP;
  MxGemmParams p;
  memset(&p, 0, sizeof(p));
  p.epi = epi; p.A = (const unsigned char*)A; p.lda = K; p.SA = (const unsigned*)SA; p.sa_ld = M;
  p.W = (const unsigned char*)W; p.SW = (const unsigned*)SW; p.bias = bias; p.cscale = cscale;
  p.M = M; p.N = N; p.K = K; p.Npad = N;
  p.C = (bf16_t*)C; p.ldc = N; p.R = R; p.ldr = N; p.VT = (bf16_t*)C; p.hd_pad = hd_pad; p.heads = heads; p.n_tok = n_tok;
  p.Cq = (unsigned char*)Cq; p.ldcq = N; p.ncq = N; p.SC = (unsigned*)SC; p.sc_ld = M;
  const hipError_t e = mx_gemm(p, (hipStream_t)hip_stream);
  if (e != hipSuccess) { set_err(g_err, sizeof(g_err), "epd_op_mx_gemm: %s", hipGetErrorString(e)); return e == hipErrorInvalidValue ? EPD_ERR_INVALID_ARG : EPD_ERR_HIP; }
  return EPD_OK;
}

epd_status epd_op_mx_mfma_probe(const void* a, const void* b, const void* sa, const void* sb, float* d, void* hip_stream) {
  if (!a || !b || !sa || !sb || !d) return EPD_ERR_INVALID_ARG;
  mx_mfma_probe((const int*)a, (const int*)b, (const int*)sa, (const int*)sb, d, (hipStream_t)hip_stream);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}

}  // extern "C"
