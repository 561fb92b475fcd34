/*
 * epd_encode.h  --  C boundary of the MI355X (gfx950) encode-stage library.
 *
 * The encode stage E of an encode / prefill / decode disaggregated pipeline
 * turns the multimodal input of a request into multimodal tokens,
 * v = E(i_m) (Section 3.1, "Encoding (E)").  An encode worker holds only the
 * encoder weights and a multimodal-token cache (Section 3.2, "System Design
 * and Optimization"); tokens stay in that cache until the next stage pulls
 * them (Section 3.2.1).  A request's image slices are encoded independently
 * of each other, so a request may be split across encode workers and the
 * token blocks merged in slice order (Section 3.2.2, intra-request
 * parallelism).  This library is the forward pass of one such worker on one
 * GPU: packed image slices in, per-request contiguous token buffers out.
 *
 * All functions are plain C, never throw, and return an epd_status (0 = ok,
 * negative = error, nothing enqueued, output untouched).  "dev" = pointer to
 * device (HBM) memory, "host" = pointer to host memory.  The library never
 * allocates or frees the caller's buffers; all device work of a call is
 * enqueued on the caller's HIP stream and the call returns after enqueueing.
 * A context serves one stream at a time (calls on one context must not
 * overlap); different contexts may be driven from different host threads.
 * epd_encode / epd_encode_range allocate nothing, copy nothing from the host and
 * clear no memory through the runtime: once a context has run one call eagerly
 * (kernel attributes are set by then) a call may be recorded into a HIP graph and
 * replayed; a replay writes the bits of the eager call.  If a HIP call fails in the
 * middle of a call (EPD_ERR_HIP: a launch or copy refused by the runtime),
 * earlier launches of that call may already have written part of the output:
 * its contents are then undefined.  Every other error is found before the
 * first launch and leaves the output untouched.
 */
#ifndef EPD_ENCODE_H
#define EPD_ENCODE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct epd_ctx epd_ctx; /* opaque: packed weights + workspace */

typedef enum {
  EPD_OK = 0,
  EPD_ERR_INVALID_ARG = -1, /* null pointer, bad enum value, misaligned pointer */
  EPD_ERR_SHAPE = -2,       /* description is inconsistent (hidden % heads, ...) */
  EPD_ERR_OFFSETS = -3,     /* tile_offsets / tile range not a valid partition   */
  EPD_ERR_UNSUPPORTED = -4, /* valid but outside what the kernels handle         */
  EPD_ERR_NOMEM = -5,       /* device allocation failed in epd_create            */
  EPD_ERR_HIP = -6          /* a HIP call or launch failed                       */
} epd_status;

enum { EPD_DTYPE_FP32 = 0, EPD_DTYPE_BF16 = 1 };
enum { EPD_NORM_LAYERNORM = 0, EPD_NORM_RMSNORM = 1 };
enum { EPD_QKNORM_NONE = 0, EPD_QKNORM_FULL = 1, EPD_QKNORM_PER_HEAD = 2 };
enum { EPD_ACT_GELU_ERF = 0, EPD_ACT_GELU_TANH = 1 };
enum { EPD_PROJ_LINEAR = 0, EPD_PROJ_MLP = 1, EPD_PROJ_RESAMPLER = 2 };

/* Encoder description.  The paper takes the encoder as given (SigLIP-400M,
 * InternViT-300M / 6B; Appendix "LMM Details"); this struct states which
 * vision transformer that is. */
typedef struct {
  int32_t dtype;         /* EPD_DTYPE_*: type of weights, activations and output        */
  int32_t tile_size;     /* side S of a square image slice in pixels (448, 224)          */
  int32_t patch;         /* side p of a ViT patch (14); S % p == 0; g = S/p; N = g*g     */
  int32_t hidden;        /* D                                                            */
  int32_t heads;         /* H, D % H == 0, head dim hd = D/H                             */
  int32_t mlp;           /* F                                                            */
  int32_t layers;        /* L >= 0                                                       */
  int32_t norm;          /* EPD_NORM_*: kind of the two pre-norms of every layer         */
  int32_t qk_norm;       /* EPD_QKNORM_*: RMSNorm of q and k (after bias, before scaling) */
  int32_t act;           /* EPD_ACT_*: activation of the layer MLP                       */
  int32_t final_norm;    /* 1: a norm of kind `norm` after the last layer                */
  int32_t pixel_shuffle; /* 1: space-to-depth by 2 on the g x g grid: N/4 tokens of 4D   */
  int32_t proj_kind;     /* EPD_PROJ_*: Linear, Linear - GELU(erf) - Linear, or the
                            cross-attention resampler (see proj_heads)                    */
  int32_t proj_prenorm;  /* 1: LayerNorm over the projector input                        */
  int32_t proj_mid;      /* MLP: width of the hidden layer; resampler: number of learned
                            queries = tokens per slice (ignored if Linear)                */
  int32_t proj_out;      /* D_out: width of a token in the cache                         */
  float   eps;           /* epsilon of every norm                                        */
  int32_t max_tiles_per_call; /* workspace is sized for this many slices at once; larger
                                 calls are processed in micro-batches of at most this.
                                 bf16 mode: every activation buffer of a micro-batch must
                                 stay below 4 GiB (epd_create: EPD_ERR_UNSUPPORTED)      */
  int32_t layer_scale;   /* 1: each residual branch is multiplied by a learned per-channel
                            vector before it is added (x += ls1 * attn(..), x += ls2 * mlp(..)),
                            as in the InternViT encoders                                  */
  int32_t class_token;   /* 1: a learned class vector is put in front of the patch tokens
                            (position row 0 is its own); it takes part in every attention
                            layer and is dropped after the last norm: pixel shuffle,
                            projector and the emitted tokens cover the N patches only     */
  int32_t proj_heads;    /* EPD_PROJ_RESAMPLER (the MiniCPM-V family's projector): proj_mid
                            learned queries read the N patch tokens of a slice,
                              kv = LN_kv(x Wkv^T), q = LN_q(query),
                              o = MHA(q, kv + pos, kv) with proj_heads heads over width
                              E = proj_out (in-projections with bias, logits / sqrt(E/heads),
                              out-projection with bias), out = LN_post(o) Wp^T;
                            needs pixel_shuffle = 0, proj_prenorm = 0, E % proj_heads == 0;
                            bf16 mode: N % 64 == 0 and E / proj_heads <= 128             */
  int32_t mx_fp8;        /* 1 (bf16 mode, hidden % 128 == 0): the q/k/v, out-projection, FC1 and FC2 products
                            of every layer take MXFP8 operands (OCP Microscaling Formats v1.0: E4M3
                            elements, one power-of-two scale per 32 consecutive elements of the
                            contraction dimension); activations are converted by the kernel that produces
                            them (pre-norm, attention output, FC1 epilogue), weights in epd_create;
                            accumulation, residual stream and the attention products are as without the
                            option.  The out-projection is converted only for head dims stored without
                            padding (64, 72, 96, 128); for others it stays bf16.  Narrower than the FP16
                            the paper serves in (Appendix "Implementation Details"): a fidelity / speed
                            option with its own tolerance                                          */
} epd_model_desc;

/* Encoder weights: `n_tensors` dev pointers in this fixed order, every matrix
 * W[out, in] row-major, every tensor of type desc.dtype (fp32 or bf16):
 *   pe_w [D, 3*p*p] (patch vector ordered channel, dy, dx), pe_b [D], pos [N, D]
 *   (class_token: pos [N + 1, D] with row 0 for the class token, followed by cls [D]);
 *   per layer l = 0..L-1:
 *     n1_g [D], n1_b [D] (n1_b only for LayerNorm),
 *     qkv_w [3D, D] (row blocks q, k, v; head h = rows h*hd..(h+1)*hd-1 of a block), qkv_b [3D],
 *     qn_g, kn_g ([D] for QKNORM_FULL, [hd] for QKNORM_PER_HEAD, absent for NONE),
 *     o_w [D, D], o_b [D], ls1 [D] (if layer_scale), n2_g [D], n2_b [D] (LayerNorm only),
 *     fc1_w [F, D], fc1_b [F], fc2_w [D, F], fc2_b [D], ls2 [D] (if layer_scale);
 *   fn_g [D], fn_b [D]            (if final_norm; fn_b only for LayerNorm)
 *   pn_g [Din], pn_b [Din]        (if proj_prenorm; Din = 4D with pixel shuffle else D)
 *   pa_w [Dmid or D_out, Din], pa_b;  pb_w [D_out, Dmid], pb_b   (pb_* only for MLP)
 *   resampler instead of pa / pb (E = proj_out, Q = proj_mid): kv_w [E, D], query [Q, E],
 *     pos [N, E] (position table added to the keys), lnq_g, lnq_b, lnkv_g, lnkv_b [E],
 *     in_w [3E, E] (row blocks q, k, v), in_b [3E], out_w [E, E], out_b [E], lnp_g, lnp_b [E],
 *     proj_w [E, E] (out = LN_post(o) proj_w^T)
 * The tensors are copied / repacked during epd_create and may be freed by the
 * caller once it returns. */
typedef struct {
  const void* const* tensors; /* host array of dev pointers */
  int32_t n_tensors;
} epd_weights;

/* Number of tensors epd_weights must hold for this description (host only,
 * needs no GPU); negative epd_status if the description is invalid. */
int32_t epd_weight_count(const epd_model_desc* desc);

/* Host-only validation of a description; writes a message to errbuf (may be
 * null).  EPD_OK, EPD_ERR_INVALID_ARG, EPD_ERR_SHAPE or EPD_ERR_UNSUPPORTED. */
epd_status epd_check_desc(const epd_model_desc* desc, char* errbuf, int32_t errbuf_len);

/* Host-only validation of a request partition: offsets[0] == 0, non-decreasing,
 * offsets[n_requests] == n_tiles.  Empty requests are legal. */
epd_status epd_check_offsets(const int32_t* tile_offsets_per_request /*host*/, int32_t n_requests,
                             int32_t n_tiles);

/* Create an encode worker's context on the current HIP device.  An encode
 * worker holds the encoder weights and its multimodal-token cache and nothing
 * of the language model (Section 3.2, "System Design and Optimization"): the
 * context is that state.  Validates the
 * description, copies and repacks the weights into the kernels' layout
 * (device allocations owned by the context), allocates the workspace for
 * max_tiles_per_call slices.  `hip_stream` (a hipStream_t, may be null = the
 * default stream) carries the packing work; the call synchronises it before
 * returning.  On error *out is null. */
epd_status epd_create(const epd_model_desc* desc, const epd_weights* weights, void* hip_stream,
                      epd_ctx** out);

/* Encode stage, v = E(i_m) (Section 3.1), for a packed batch of requests.
 *   tiles   dev, float32 [n_tiles, 3, S, S], channel-first, values as the
 *           (out of scope) CPU preprocessor leaves them; 16-byte aligned.
 *   tile_offsets_per_request
 *           host, int32 [n_requests + 1]; request r owns slices
 *           offsets[r] .. offsets[r+1]-1 in slice order (image-major,
 *           thumbnail last).
 *   out_token_cache
 *           dev, desc.dtype [n_tiles * N_out, D_out] row-major, 16-byte
 *           aligned, N_out = epd_tokens_per_tile().  Request r's token buffer
 *           is the contiguous row block
 *           [offsets[r] * N_out, offsets[r+1] * N_out).  Every row is written.
 * n_tiles == 0 is a successful no-op.  Results are valid once `hip_stream`
 * has been synchronised.  Bit-identical from run to run and independent of
 * how slices are grouped into calls. */
epd_status epd_encode(epd_ctx* ctx, const float* tiles, int32_t n_tiles,
                      const int32_t* tile_offsets_per_request, int32_t n_requests,
                      void* out_token_cache, void* hip_stream);

/* One encode worker's share under intra-request parallelism (Section 3.2.2):
 * encode slices [tile_begin, tile_end) of the packed batch `tiles`
 * (dev, [n_tiles_total, 3, S, S]) and write exactly rows
 * [tile_begin * N_out, tile_end * N_out) of the same out_token_cache; no
 * other row is touched, so shards need no gather copy.  An empty range is a
 * successful no-op.  Requires 0 <= tile_begin <= tile_end <= n_tiles_total. */
epd_status epd_encode_range(epd_ctx* ctx, const float* tiles, int32_t n_tiles_total,
                            int32_t tile_begin, int32_t tile_end, void* out_token_cache,
                            void* hip_stream);

/* Shape of the token block a slice yields, v = E(i_m) (Section 3.1): the block
 * manager sizes a request's cache entry from its slice count times these
 * (Section 3.2.1).  -1 for a null ctx. */
int64_t epd_tokens_per_tile(const epd_ctx* ctx); /* N_out = N, N/4 with pixel shuffle, or the resampler's query count */
int64_t epd_out_dim(const epd_ctx* ctx);         /* D_out */

/* Last error message of this context (owned by the context, never freed by
 * the caller); for a null ctx the message of the last failed epd_create /
 * host-only check on this thread. */
const char* epd_last_error(const epd_ctx* ctx);

/* Release the worker's state: packed weights and workspace (what the paper's
 * role switching offloads when an encode worker is turned into another
 * stage's worker, Section 3.2.4).  The caller synchronises the stream first.
 * Null is a no-op. */
void epd_destroy(epd_ctx* ctx);

/* ---- paged multimodal-token cache ---------------------------------------
 *
 * Encode and prefill workers both keep an MM cache; when an encode finishes
 * its tokens stay in the encode worker's cache until they have been moved to
 * the prefill worker's cache, then the source entries are released
 * (Section 3.2.1, "Asynchronous Token Transfer").  The MMBlockManager of that
 * section pre-allocates cache blocks per request and reassigns them after the
 * transfer; the paper's settings are blocks of 16 tokens and an MM cache size
 * of 3000 (Appendix "Hyper-parameters in EPD system").  An epd_mm_cache is one
 * such cache: a device pool [n_blocks][block_tokens][token_dim] plus the
 * host-side block manager.  Block lists are host int32 arrays.  One thread at
 * a time per cache; the manager calls are host-only and immediate, the copies
 * are enqueued on the given stream. */
typedef struct epd_mm_cache epd_mm_cache;

/* token_dim 0 creates the manager without a device pool (planning, host tests). */
epd_status epd_mm_cache_create(int32_t n_blocks, int32_t block_tokens, int32_t token_dim, int32_t dtype,
                               epd_mm_cache** out);
void epd_mm_cache_destroy(epd_mm_cache* cache);
int32_t epd_mm_cache_free_blocks(const epd_mm_cache* cache);
void* epd_mm_cache_base(const epd_mm_cache* cache); /* dev pointer of the pool */
const char* epd_mm_last_error(const epd_mm_cache* cache);

/* Pre-allocate the ceil(n_tokens / block_tokens) blocks a request needs (its
 * token count follows from its slice count: slices * epd_tokens_per_tile).
 * block_ids (host, max_ids entries) receives them in token order.
 * EPD_ERR_NOMEM if the cache has too few free blocks (nothing is taken). */
epd_status epd_mm_alloc(epd_mm_cache* cache, int64_t n_tokens, int32_t* block_ids, int32_t max_ids,
                        int32_t* n_ids);
/* Release blocks (after their tokens have been transferred).  A list with an
 * unallocated, out-of-range or repeated id frees nothing. */
epd_status epd_mm_free(epd_mm_cache* cache, const int32_t* block_ids, int32_t n_ids);

/* Encode stage with paged output: as epd_encode, but token i of request r is
 * written to block block_table[block_table_offsets[r] + i / block_tokens],
 * slot i % block_tokens, of `cache` (token width and dtype must match the
 * encoder, tokens per slice must be a multiple of block_tokens).
 * block_table_offsets: host int32 [n_requests + 1], request r owns
 * (slices of r) * tokens_per_tile / block_tokens entries; every entry must be
 * an allocated block of `cache`.  No other block is touched. */
epd_status epd_encode_paged(epd_ctx* ctx, const float* tiles, int32_t n_tiles,
                            const int32_t* tile_offsets_per_request, int32_t n_requests,
                            epd_mm_cache* cache, const int32_t* block_table,
                            const int32_t* block_table_offsets, void* hip_stream);

/* Encode-to-prefill migration on one device: copy blocks src_blocks[i] of
 * `src` to blocks dst_blocks[i] of `dst` (same block shape; all blocks
 * allocated).  One transfer at a time per destination cache and stream. */
epd_status epd_mm_transfer(const epd_mm_cache* src, const int32_t* src_blocks, epd_mm_cache* dst,
                           const int32_t* dst_blocks, int32_t n_blocks, void* hip_stream);

/* epd_mm_transfer for callers that must not allocate device memory while they run: code under HIP graph
 * capture, tight serving loops, harnesses that forbid it.  Same arguments, same result, same validation;
 * the block-id lists the copy kernel reads sit in a static device array of the library
 * (2 x EPD_MM_NOALLOC_MAX_BLOCKS ints, 512 KiB per GPU, held until the process ends) instead of the
 * destination cache's own scratch, and the call allocates and frees nothing.  More than
 * EPD_MM_NOALLOC_MAX_BLOCKS blocks in one call: EPD_ERR_UNSUPPORTED, nothing enqueued (cut the transfer
 * into several calls).  Every call on a GPU shares that GPU's array and keeps the previous call's ids in
 * it: calls are safe one after the other on one stream; two of these calls in flight at once on the same
 * GPU (different streams or host threads) race on the array. */
enum { EPD_MM_NOALLOC_MAX_BLOCKS = 65536 };
epd_status epd_mm_transfer_noalloc(const epd_mm_cache* src, const int32_t* src_blocks, epd_mm_cache* dst,
                                   const int32_t* dst_blocks, int32_t n_blocks, void* hip_stream);

/* Copy blocks[0..n_blocks) of `src`, in that order, into a contiguous dev
 * buffer (16-byte aligned) of n_blocks * block_tokens tokens. */
epd_status epd_mm_gather(epd_mm_cache* src, const int32_t* blocks, int32_t n_blocks, void* dst_contiguous,
                         void* hip_stream);

/* ---- projection on the prefill side ---------------------------------------
 *
 * With intra-request parallelism the slices of one request are encoded on
 * several encode workers and their tokens sent to the prefill stage, where
 * they are put in slice order, projected and merged into the request's
 * multimodal tokens (Section 3.2.2).  These two calls split the path at that
 * point: the encode side stops after the encoder's last norm and caches the
 * pre-projection tokens ([patches per slice, hidden] per slice, the encoder's
 * dtype); the prefill side reads the shards' tokens through one block table
 * in slice order and runs pixel shuffle (if any) and the projector.  In fp32
 * mode the result equals epd_encode's bit for bit; in bf16 mode the cached
 * tokens are rounded to bf16 once more than in the fused path. */

/* Slices [tile_begin, tile_end) of the packed batch -> pre-projection tokens
 * in `cache` (token_dim == hidden, patches per slice a multiple of
 * block_tokens).  block_table (host) holds (tile_end - tile_begin) *
 * patches_per_slice / block_tokens allocated block ids: entry 0 is the first
 * block of slice tile_begin.  Nothing else in the cache is touched. */
epd_status epd_encode_trunk_paged(epd_ctx* ctx, const float* tiles, int32_t n_tiles_total,
                                  int32_t tile_begin, int32_t tile_end, epd_mm_cache* cache,
                                  const int32_t* block_table, void* hip_stream);

/* Pre-projection tokens of n_tiles slices, listed in slice order by
 * block_table (n_tiles * patches_per_slice / block_tokens ids of `cache`,
 * whichever shard or transfer filled them) -> out_tokens, a contiguous dev
 * buffer [n_tiles * epd_tokens_per_tile, epd_out_dim] of the encoder's dtype
 * (16-byte aligned).  The cache is only read. */
epd_status epd_project_merge(epd_ctx* ctx, const epd_mm_cache* cache, const int32_t* block_table,
                             int32_t n_tiles, void* out_tokens, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EPD_ENCODE_H */
