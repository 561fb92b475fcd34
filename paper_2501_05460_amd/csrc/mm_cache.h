// Paged multimodal-token cache of an encode worker and its block manager
// (internal definition shared by mm_cache.hip and epd_api.hip).
#pragma once
#include <vector>

struct epd_mm_cache {
  int n_blocks = 0, block_tokens = 0, token_dim = 0, dtype = 0;
  long block_bytes = 0;
  void* pool = nullptr;        // device: [n_blocks][block_tokens][token_dim]
  int* d_ids = nullptr;        // device scratch for block id lists (2 * n_blocks ints)
  int* h_ids = nullptr;        // pinned host staging of the same size: one asynchronous upload per call
  hipEvent_t ev_ids = nullptr; // recorded behind the upload; the staging is rewritten only after it
  bool ev_pending = false;
  std::vector<int> free_list;  // LIFO of free block ids
  std::vector<unsigned char> used;
  std::vector<unsigned char> mark;   // scratch of the table checks (duplicate detection), all zero between calls
  char err[256] = "";
};
