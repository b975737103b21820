// Internal helpers shared by the host side of the library's entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mc_kv.h"

namespace mc {

constexpr int kPage = 16;        // tokens per page
constexpr int kHeadDim = 128;    // elements per head
constexpr int kRowBytes = kHeadDim * 2;          // one (token, head) row of K or V
constexpr int kHeadPageBytes = kPage * kRowBytes;  // one (page, K|V, head) block: 4 KiB

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape checks common to every call that takes a pool.
inline mc_status check_pool(const mc_pool_desc* pool) {
  if (!pool || !pool->base) return MC_ERR_INVALID;
  if (!aligned16(pool->base)) return MC_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(pool->skipped) & 3u) return MC_ERR_INVALID;
  if (pool->num_layers <= 0 || pool->num_pages <= 0 || pool->num_kv_heads <= 0)
    return MC_ERR_INVALID;
  if (pool->page_size != kPage || pool->head_dim != kHeadDim) return MC_ERR_UNSUPPORTED;
  if (pool->dtype != MC_F16 && pool->dtype != MC_BF16) return MC_ERR_UNSUPPORTED;
  return MC_OK;
}

inline mc_status launch_status() {
  return hipGetLastError() == hipSuccess ? MC_OK : MC_ERR_HIP;
}

// bytes between consecutive pages of one layer, and between layers
inline int64_t page_stride_bytes(const mc_pool_desc* p) {
  return 2ll * p->num_kv_heads * kHeadPageBytes;
}
inline int64_t layer_stride_bytes(const mc_pool_desc* p) {
  return page_stride_bytes(p) * p->num_pages;
}

}  // namespace mc
