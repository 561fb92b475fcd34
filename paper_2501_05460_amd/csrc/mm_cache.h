// Paged multimodal-token cache of an encode worker and its block manager
// (internal definition shared by mm_cache.hip and epd_api.hip).
#pragma once
#include <vector>

struct epd_mm_cache {
  int n_blocks = 0, block_tokens = 0, token_dim = 0, dtype = 0;
  long block_bytes = 0;
  void* pool = nullptr;        // device: [n_blocks][block_tokens][token_dim]
  int* d_ids_a = nullptr;      // device scratch for block id lists (n_blocks each)
  int* d_ids_b = nullptr;
  std::vector<int> free_list;  // LIFO of free block ids
  std::vector<unsigned char> used;
  char err[256] = "";
};
