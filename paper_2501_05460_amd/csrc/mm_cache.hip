// Paged multimodal-token cache: device pool + host-side block manager, and
// the block copies that move a request's tokens between two caches (the
// encode worker's and a stand-in for the prefill worker's) or to / from a
// contiguous buffer.  See include/epd_encode.h.
#include "../../include/epd_encode.h"

#include <cstdio>
#include <cstring>

#include "kernels.h"
#include "mm_cache.h"

using namespace epd;

#include <mutex>

// Block-id lists of epd_mm_transfer_noalloc: source ids, then destination ids.  One array per GPU the
// library runs on, held until the process ends; every call on a GPU shares it.
static __device__ __align__(256) int scratch[2 * EPD_MM_NOALLOC_MAX_BLOCKS];

namespace {
// In host code `scratch` is only a handle: the array's address on a device is asked for once per device,
// with that device current, and kept here.
constexpr int MAX_DEVICES = 64;
int* g_scratch_ptr[MAX_DEVICES] = {nullptr};
std::mutex g_scratch_mu;

hipError_t scratch_on_current_device(int** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    int* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

thread_local char g_mm_err[256] = "";
void mm_err(epd_mm_cache* c, const char* msg) {
  snprintf(g_mm_err, sizeof(g_mm_err), "%s", msg);
  if (c) snprintf(c->err, sizeof(c->err), "%s", msg);
}
bool ids_ok(const epd_mm_cache* c, const int32_t* ids, int32_t n, bool must_be_used) {
  for (int i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= c->n_blocks) return false;
    if (must_be_used && !c->used[ids[i]]) return false;
  }
  return true;
}
}  // namespace

extern "C" {

epd_status epd_mm_cache_create(int32_t n_blocks, int32_t block_tokens, int32_t token_dim, int32_t dtype,
                               epd_mm_cache** out) {
  if (!out) return EPD_ERR_INVALID_ARG;
  *out = nullptr;
  if (n_blocks <= 0 || block_tokens <= 0 || token_dim < 0 || (dtype != EPD_DTYPE_FP32 && dtype != EPD_DTYPE_BF16)) {
    mm_err(nullptr, "epd_mm_cache_create: n_blocks, block_tokens must be positive, token_dim >= 0, dtype 0 or 1");
    return EPD_ERR_INVALID_ARG;
  }
  const long elt = dtype == EPD_DTYPE_BF16 ? 2 : 4;
  const long block_bytes = (long)block_tokens * token_dim * elt;
  if (block_bytes % 16 != 0) {
    mm_err(nullptr, "epd_mm_cache_create: a block must be a multiple of 16 bytes");
    return EPD_ERR_UNSUPPORTED;
  }
  epd_mm_cache* c = new epd_mm_cache();
  c->n_blocks = n_blocks; c->block_tokens = block_tokens; c->token_dim = token_dim; c->dtype = dtype;
  c->block_bytes = block_bytes;
  c->used.assign(n_blocks, 0);
  c->mark.assign(n_blocks, 0);
  c->free_list.reserve(n_blocks);
  for (int i = n_blocks - 1; i >= 0; --i) c->free_list.push_back(i);  // block 0 is handed out first
  if (block_bytes > 0) {  // token_dim 0: manager only (planning, host tests), no device memory
    if (hipMalloc(&c->pool, (size_t)n_blocks * block_bytes) != hipSuccess ||
        hipMalloc((void**)&c->d_ids, (size_t)2 * n_blocks * sizeof(int)) != hipSuccess ||
        hipHostMalloc((void**)&c->h_ids, (size_t)2 * n_blocks * sizeof(int), hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_ids, hipEventDisableTiming) != hipSuccess) {
      mm_err(nullptr, "epd_mm_cache_create: device allocation failed");
      epd_mm_cache_destroy(c);
      return EPD_ERR_NOMEM;
    }
  }
  *out = c;
  return EPD_OK;
}

void epd_mm_cache_destroy(epd_mm_cache* c) {
  if (!c) return;
  if (c->pool) (void)hipFree(c->pool);
  if (c->d_ids) (void)hipFree(c->d_ids);
  if (c->h_ids) (void)hipHostFree(c->h_ids);
  if (c->ev_ids) (void)hipEventDestroy(c->ev_ids);
  delete c;
}

int32_t epd_mm_cache_free_blocks(const epd_mm_cache* c) { return c ? (int32_t)c->free_list.size() : -1; }
void* epd_mm_cache_base(const epd_mm_cache* c) { return c ? c->pool : nullptr; }
const char* epd_mm_last_error(const epd_mm_cache* c) { return c ? c->err : g_mm_err; }

epd_status epd_mm_alloc(epd_mm_cache* c, int64_t n_tokens, int32_t* block_ids, int32_t max_ids, int32_t* n_ids) {
  if (!c || !n_ids || n_tokens < 0 || (n_tokens > 0 && !block_ids)) return EPD_ERR_INVALID_ARG;
  const int64_t need = (n_tokens + c->block_tokens - 1) / c->block_tokens;
  *n_ids = 0;
  if (need > max_ids) { mm_err(c, "epd_mm_alloc: block_ids too short for the request"); return EPD_ERR_INVALID_ARG; }
  if (need > (int64_t)c->free_list.size()) { mm_err(c, "epd_mm_alloc: not enough free blocks"); return EPD_ERR_NOMEM; }
  for (int64_t i = 0; i < need; ++i) {
    const int b = c->free_list.back();
    c->free_list.pop_back();
    c->used[b] = 1;
    block_ids[i] = b;
  }
  *n_ids = (int32_t)need;
  return EPD_OK;
}

epd_status epd_mm_free(epd_mm_cache* c, const int32_t* block_ids, int32_t n_ids) {
  if (!c || n_ids < 0 || (n_ids > 0 && !block_ids)) return EPD_ERR_INVALID_ARG;
  // validate everything first: a bad list frees nothing
  if (!ids_ok(c, block_ids, n_ids, true)) { mm_err(c, "epd_mm_free: id out of range or block not allocated"); return EPD_ERR_INVALID_ARG; }
  int dup = -1;   // `mark` is all zero between calls
  for (int i = 0; i < n_ids && dup < 0; ++i) {
    if (c->mark[block_ids[i]]) dup = i;
    else c->mark[block_ids[i]] = 1;
  }
  for (int i = 0; i < (dup < 0 ? n_ids : dup); ++i) c->mark[block_ids[i]] = 0;
  if (dup >= 0) { mm_err(c, "epd_mm_free: duplicate id in the list"); return EPD_ERR_INVALID_ARG; }
  for (int i = 0; i < n_ids; ++i) { c->used[block_ids[i]] = 0; c->free_list.push_back(block_ids[i]); }
  return EPD_OK;
}

}  // extern "C"

namespace {
// `n_lists` id lists of n ints each -> d_dst (c->d_ids, or the static array), back to back, through the
// cache's pinned staging (waits for the previous upload of this cache before the staging is overwritten)
bool upload_ids(epd_mm_cache* c, int* d_dst, const int32_t* const* lists, int n_lists, int n, hipStream_t st) {
  if (c->ev_pending && hipEventSynchronize(c->ev_ids) != hipSuccess) return false;
  for (int l = 0; l < n_lists; ++l) memcpy(c->h_ids + (size_t)l * n, lists[l], (size_t)n * sizeof(int));
  if (hipMemcpyAsync(d_dst, c->h_ids, (size_t)n_lists * n * sizeof(int), hipMemcpyHostToDevice, st) != hipSuccess) return false;
  if (hipEventRecord(c->ev_ids, st) != hipSuccess) return false;
  c->ev_pending = true;
  return true;
}
}  // namespace

namespace {
// body of the two transfer calls; ids_dev: where the id lists go on the device (null: the static array of
// the current device, looked up once every argument has passed its checks)
epd_status transfer_impl(const epd_mm_cache* src, const int32_t* src_blocks, epd_mm_cache* dst,
                         const int32_t* dst_blocks, int32_t n_blocks, int* ids_dev, const char* who, hipStream_t st) {
  char msg[160];
  if (src->block_bytes != dst->block_bytes || src->block_tokens != dst->block_tokens || src->dtype != dst->dtype ||
      !src->pool || !dst->pool) {
    snprintf(msg, sizeof(msg), "%s: the two caches must have the same block shape and a device pool", who);
    mm_err(dst, msg);
    return EPD_ERR_SHAPE;
  }
  if (n_blocks > src->n_blocks || n_blocks > dst->n_blocks || !ids_ok(src, src_blocks, n_blocks, true) ||
      !ids_ok(dst, dst_blocks, n_blocks, true)) {
    snprintf(msg, sizeof(msg), "%s: block id out of range or not allocated", who);
    mm_err(dst, msg);
    return EPD_ERR_OFFSETS;
  }
  if (n_blocks == 0) return EPD_OK;
  if (!ids_dev && scratch_on_current_device(&ids_dev) != hipSuccess) {
    snprintf(msg, sizeof(msg), "%s: the address of the static id array is not available on this device", who);
    mm_err(dst, msg);
    return EPD_ERR_HIP;
  }
  // source ids, then destination ids, one upload
  const int32_t* lists[2] = {src_blocks, dst_blocks};
  if (!upload_ids(dst, ids_dev, lists, 2, n_blocks, st)) {
    snprintf(msg, sizeof(msg), "%s: id upload failed", who);
    mm_err(dst, msg);
    return EPD_ERR_HIP;
  }
  mm_copy_blocks(src->pool, ids_dev, dst->pool, ids_dev + n_blocks, n_blocks, src->block_bytes, st);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}
}  // namespace

extern "C" {

epd_status epd_mm_transfer(const epd_mm_cache* src, const int32_t* src_blocks, epd_mm_cache* dst,
                           const int32_t* dst_blocks, int32_t n_blocks, void* hip_stream) {
  if (!src || !dst || n_blocks < 0 || (n_blocks > 0 && (!src_blocks || !dst_blocks))) return EPD_ERR_INVALID_ARG;
  // id lists travel in the destination cache's own device scratch (one transfer at a time per destination)
  return transfer_impl(src, src_blocks, dst, dst_blocks, n_blocks, dst->d_ids, "epd_mm_transfer", (hipStream_t)hip_stream);
}

epd_status epd_mm_transfer_noalloc(const epd_mm_cache* src, const int32_t* src_blocks, epd_mm_cache* dst,
                                   const int32_t* dst_blocks, int32_t n_blocks, void* hip_stream) {
  if (!src || !dst || n_blocks < 0 || (n_blocks > 0 && (!src_blocks || !dst_blocks))) return EPD_ERR_INVALID_ARG;
  if (n_blocks > EPD_MM_NOALLOC_MAX_BLOCKS) {
    char msg[160];
    snprintf(msg, sizeof(msg), "epd_mm_transfer_noalloc: %d blocks in one call, the static id array holds %d; "
             "cut the transfer into several calls", n_blocks, EPD_MM_NOALLOC_MAX_BLOCKS);
    mm_err(dst, msg);
    return EPD_ERR_UNSUPPORTED;
  }
  // Nothing in the array has to start at zero: entries [0, 2 n_blocks) are rewritten by this call's upload
  // and the kernel reads no others.
  return transfer_impl(src, src_blocks, dst, dst_blocks, n_blocks, nullptr, "epd_mm_transfer_noalloc", (hipStream_t)hip_stream);
}

epd_status epd_mm_gather(epd_mm_cache* src, const int32_t* blocks, int32_t n_blocks, void* dst_contiguous,
                         void* hip_stream) {
  if (!src || n_blocks < 0 || (n_blocks > 0 && (!blocks || !dst_contiguous))) return EPD_ERR_INVALID_ARG;
  if (!src->pool) return EPD_ERR_SHAPE;
  if (((uintptr_t)dst_contiguous & 15) != 0) return EPD_ERR_INVALID_ARG;
  if (n_blocks > src->n_blocks || !ids_ok(src, blocks, n_blocks, true)) {
    mm_err(src, "epd_mm_gather: block id out of range or not allocated");
    return EPD_ERR_OFFSETS;
  }
  if (n_blocks == 0) return EPD_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  const int32_t* lists[1] = {blocks};
  if (!upload_ids(src, src->d_ids, lists, 1, n_blocks, st)) return EPD_ERR_HIP;
  mm_copy_blocks(src->pool, src->d_ids, dst_contiguous, nullptr, n_blocks, src->block_bytes, st);
  return hipGetLastError() == hipSuccess ? EPD_OK : EPD_ERR_HIP;
}

}  // extern "C"
