// Bandwidth-bound page copies for gfx950: KV append, and the page-range
// gather/scatter behind remote_send / prep_recv (paper Sec. 3.1, Sec. 3.2
// Example 2, Sec. 3.6).  No arithmetic: every lane moves 16 bytes at a time.
//
// Geometry (D = 128, P = 16, 2-byte elements): a (token, head) row is 256 B =
// 16 lanes x 16 B; a (page, K|V, head) block is 16 rows = 4 KiB contiguous in the
// pool; in the packed buffer and in k_new/v_new the Hkv rows of one token are
// contiguous (Hkv x 256 B).  A 256-thread workgroup moves one page of K or V of
// one layer: per head, its 256 lanes cover the 4 KiB block on the pool side
// (fully coalesced) and 16 runs of 256 B on the token-major side.
#include "mc_common.h"

namespace {

using mc::kHeadPageBytes;
using mc::kPage;
using mc::kRowBytes;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxHeadsInFlight = 8;  // 16-byte loads a lane keeps in flight

struct RangeArgs {
  char* pool;             // pool base
  char* buf;              // packed buffer base
  const int32_t* pages;   // one sequence's table
  int64_t layer_stride;   // bytes
  int64_t page_stride;    // bytes
  int32_t num_pages;      // pool pages, for the bounds check
  int32_t n_table_pages;
  int32_t layer_begin;
  int32_t s0, s1;
  int32_t hkv;
  // batched form only (blockIdx.z = sequence): per-sequence ranges, tables and buffer offsets
  const int32_t* cu_pages;
  const int32_t* s0_of;
  const int32_t* s1_of;
  const int64_t* buf_offset;
  int32_t* skipped;       // optional counter of what was left out for being out of bounds
};

// One lane of the workgroup reports a unit (page, sequence, token) left out as out of bounds.
__device__ __forceinline__ void report_skip(int32_t* counter, bool this_lane) {
  if (counter && this_lane) atomicAdd(counter, 1);
}

// grid.x: 2 * (page index within [s0/16, ceil(s1/16))) + (0 = K, 1 = V); grid.y: layer - layer_begin
template <bool kPack, bool kBatched>
__global__ __launch_bounds__(kThreads) void range_copy_kernel(RangeArgs a) {
  if (kBatched) {
    // this sequence's table, range and slice of the buffer; malformed entries are skipped
    const int sq = blockIdx.z;
    const int p0 = a.cu_pages[sq], p1 = a.cu_pages[sq + 1];
    a.s0 = a.s0_of[sq];
    a.s1 = a.s1_of[sq];
    const int64_t off = a.buf_offset[sq];
    if (a.s1 <= a.s0 && a.s0 >= 0) return;   // empty by its own statement
    if (p0 < 0 || p1 < p0 || a.s0 < 0 || off < 0 || (off & 15)) {
      // malformed sequence: counted once (by the workgroup of its first page, K, first layer)
      report_skip(a.skipped, blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0);
      return;
    }
    a.pages += p0;
    a.n_table_pages = p1 - p0;
    a.buf += off;
    if (a.s0 / kPage + (int)(blockIdx.x >> 1) > (a.s1 - 1) / kPage) return;
  }
  // K and V of a page are neighbours in the pool (one 2 x Hkv x 4 KiB run): neighbouring
  // workgroups take them, which measures a few per cent faster than K and V in separate sweeps
  const int tp = a.s0 / kPage + (blockIdx.x >> 1);   // table index
  const int lk = blockIdx.y * 2 + (blockIdx.x & 1);
  const int slot = threadIdx.x >> 4, lane16 = threadIdx.x & 15;
  const int tok = tp * kPage + slot;
  // a page the table does not hold or the pool does not have: counted once (K, first layer)
  const bool reporter = (blockIdx.x & 1) == 0 && blockIdx.y == 0 && threadIdx.x == 0;
  if (tp >= a.n_table_pages) { report_skip(a.skipped, reporter); return; }
  const int32_t page = a.pages[tp];
  if (page < 0 || page >= a.num_pages) { report_skip(a.skipped, reporter); return; }
  const bool live = tok >= a.s0 && tok < a.s1;
  const int layer = a.layer_begin + (lk >> 1), kv = lk & 1;
  const int64_t T = a.s1 - a.s0;
  char* pool_blk = a.pool + layer * a.layer_stride + page * a.page_stride +
                   (int64_t)kv * a.hkv * kHeadPageBytes + slot * kRowBytes + lane16 * 16;
  char* buf_row = a.buf + ((int64_t)lk * T + (tok - a.s0)) * a.hkv * kRowBytes + lane16 * 16;
  if (!live) return;
  for (int h0 = 0; h0 < a.hkv; h0 += kMaxHeadsInFlight) {
    u32x4 r[kMaxHeadsInFlight];
#pragma unroll
    for (int i = 0; i < kMaxHeadsInFlight; ++i) {
      const int h = h0 + i;
      if (h < a.hkv) {
        const char* src = kPack ? pool_blk + (int64_t)h * kHeadPageBytes : buf_row + h * kRowBytes;
        r[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src));
      }
    }
#pragma unroll
    for (int i = 0; i < kMaxHeadsInFlight; ++i) {
      const int h = h0 + i;
      if (h < a.hkv) {
        char* dst = kPack ? buf_row + h * kRowBytes : pool_blk + (int64_t)h * kHeadPageBytes;
        __builtin_nontemporal_store(r[i], reinterpret_cast<u32x4*>(dst));
      }
    }
  }
}

struct AppendArgs {
  char* pool_layer;        // pool base + layer offset
  const char* k_new;
  const char* v_new;
  const int32_t* cu_q;
  const int32_t* begin;
  const int32_t* page_table;
  const int32_t* cu_pages;
  int64_t page_stride;
  int32_t num_pages;
  int32_t batch, total_q, hkv;
  // marked for sending (kSend): tokens [s0_of[s], s1_of[s]) of sequence s also go to its slice of
  // the transfer buffer, laid out as pack writes it
  char* buf;
  const int32_t* s0_of;
  const int32_t* s1_of;
  const int64_t* buf_offset;
  int32_t layer_rel;       // layer - first layer of the transfer buffer
  int32_t* skipped;        // optional counter of tokens left out for being out of bounds
};

// grid.x: 2 * (chunk of 16 consecutive tokens of the ragged new-token stream) + (0 = K, 1 = V)
template <bool kSend>
__global__ __launch_bounds__(kThreads) void append_kernel(AppendArgs a) {
  const int g = (blockIdx.x >> 1) * kPage + (threadIdx.x >> 4);
  const int lane16 = threadIdx.x & 15;
  const int kv = blockIdx.x & 1;
  if (g >= a.total_q) return;
  // sequence of token g: last s with cu_q[s] <= g
  int lo = 0, hi = a.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.cu_q[mid] <= g) lo = mid; else hi = mid;
  }
  const int s = lo;
  const int q0 = a.cu_q[s];
  const bool reporter = kv == 0 && lane16 == 0;      // one lane per token
  if (g < q0 || g >= a.cu_q[s + 1]) { report_skip(a.skipped, reporter); return; }   // malformed offsets
  const int pos = a.begin[s] + (g - q0);
  if (pos < 0) { report_skip(a.skipped, reporter); return; }
  const int p0 = a.cu_pages[s], p1 = a.cu_pages[s + 1];
  const int tp = pos / kPage;
  if (p0 < 0 || tp >= p1 - p0) { report_skip(a.skipped, reporter); return; }       // table too short
  const int32_t page = a.page_table[p0 + tp];
  if (page < 0 || page >= a.num_pages) { report_skip(a.skipped, reporter); return; }
  const char* src = (kv ? a.v_new : a.k_new) + (int64_t)g * a.hkv * kRowBytes + lane16 * 16;
  char* dst = a.pool_layer + page * a.page_stride + (int64_t)kv * a.hkv * kHeadPageBytes +
              (pos % kPage) * kRowBytes + lane16 * 16;
  // the token's row in the transfer buffer, if it is marked: [layer][K|V][token - s0][head][D]
  char* sent = nullptr;
  if (kSend) {
    const int s0 = a.s0_of[s], s1 = a.s1_of[s];
    const int64_t off = a.buf_offset[s];
    if (s0 >= 0 && pos >= s0 && pos < s1 && off >= 0 && (off & 15) == 0)
      sent = a.buf + off +
             ((int64_t)(a.layer_rel * 2 + kv) * (s1 - s0) + (pos - s0)) * a.hkv * kRowBytes + lane16 * 16;
  }
  for (int h0 = 0; h0 < a.hkv; h0 += kMaxHeadsInFlight) {
    u32x4 r[kMaxHeadsInFlight];
#pragma unroll
    for (int i = 0; i < kMaxHeadsInFlight; ++i)
      if (h0 + i < a.hkv)
        r[i] = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4*>(src + (h0 + i) * kRowBytes));
#pragma unroll
    for (int i = 0; i < kMaxHeadsInFlight; ++i)
      if (h0 + i < a.hkv)
        __builtin_nontemporal_store(
            r[i], reinterpret_cast<u32x4*>(dst + (int64_t)(h0 + i) * kHeadPageBytes));
    if (kSend && sent) {
#pragma unroll
      for (int i = 0; i < kMaxHeadsInFlight; ++i)
        if (h0 + i < a.hkv)
          __builtin_nontemporal_store(r[i], reinterpret_cast<u32x4*>(sent + (h0 + i) * kRowBytes));
    }
  }
}

struct PageCopyArgs {
  char* pool;
  int64_t layer_stride, page_stride;
  int32_t layer_begin, src_page, dst_page, slots, hkv;
};

// grid.x: 0 = K, 1 = V; grid.y: layer - layer_begin.  Slots [0, slots) of one page to another.
__global__ __launch_bounds__(kThreads) void page_copy_kernel(PageCopyArgs a) {
  const int slot = threadIdx.x >> 4, lane16 = threadIdx.x & 15;
  if (slot >= a.slots) return;
  const int64_t in_page = (int64_t)blockIdx.x * a.hkv * kHeadPageBytes + slot * kRowBytes + lane16 * 16;
  char* layer = a.pool + (a.layer_begin + (int64_t)blockIdx.y) * a.layer_stride;
  const char* src = layer + a.src_page * a.page_stride + in_page;
  char* dst = layer + a.dst_page * a.page_stride + in_page;
  for (int h = 0; h < a.hkv; ++h)
    *reinterpret_cast<u32x4*>(dst + (int64_t)h * kHeadPageBytes) =
        *reinterpret_cast<const u32x4*>(src + (int64_t)h * kHeadPageBytes);
}

mc_status range_copy(bool pack, const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                     const int32_t* pages, int32_t n_table_pages, int32_t s0, int32_t s1,
                     void* sendbuf, void* stream) {
  mc_status st = mc::check_pool(pool);
  if (st != MC_OK) return st;
  if (layer_begin < 0 || layer_end < layer_begin || layer_end > pool->num_layers)
    return MC_ERR_RANGE;
  if (s0 < 0 || s1 < s0 || n_table_pages < 0) return MC_ERR_RANGE;
  if (s0 == s1 || layer_begin == layer_end) return MC_OK;
  if (!pages || !sendbuf || !mc::aligned16(sendbuf)) return MC_ERR_INVALID;
  const int64_t need = ((int64_t)s1 + kPage - 1) / kPage;
  if (need > n_table_pages) return MC_ERR_RANGE;
  const int64_t gy = layer_end - layer_begin;
  if (gy > 65535) return MC_ERR_UNSUPPORTED;
  RangeArgs a;
  a.pool = static_cast<char*>(pool->base);
  a.buf = static_cast<char*>(sendbuf);
  a.pages = pages;
  a.layer_stride = mc::layer_stride_bytes(pool);
  a.page_stride = mc::page_stride_bytes(pool);
  a.num_pages = pool->num_pages;
  a.n_table_pages = n_table_pages;
  a.layer_begin = layer_begin;
  a.s0 = s0;
  a.s1 = s1;
  a.hkv = pool->num_kv_heads;
  a.cu_pages = nullptr;
  a.s0_of = nullptr;
  a.s1_of = nullptr;
  a.buf_offset = nullptr;
  a.skipped = pool->skipped;
  const int first = s0 / kPage, last = (s1 - 1) / kPage;
  dim3 grid(2u * (last - first + 1), (unsigned)gy);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (pack)
    hipLaunchKernelGGL((range_copy_kernel<true, false>), grid, dim3(kThreads), 0, hs, a);
  else
    hipLaunchKernelGGL((range_copy_kernel<false, false>), grid, dim3(kThreads), 0, hs, a);
  return mc::launch_status();
}

mc_status range_copy_batch(bool pack, const mc_pool_desc* pool, int32_t layer_begin,
                           int32_t layer_end, int32_t batch, const int32_t* page_table,
                           const int32_t* cu_pages, const int32_t* s0, const int32_t* s1,
                           const int64_t* buf_offset, int32_t max_range_pages, void* sendbuf,
                           void* stream) {
  mc_status st = mc::check_pool(pool);
  if (st != MC_OK) return st;
  if (layer_begin < 0 || layer_end < layer_begin || layer_end > pool->num_layers)
    return MC_ERR_RANGE;
  if (batch < 0 || max_range_pages < 0) return MC_ERR_INVALID;
  if (batch == 0 || max_range_pages == 0 || layer_begin == layer_end) return MC_OK;
  if (!page_table || !cu_pages || !s0 || !s1 || !buf_offset || !sendbuf ||
      !mc::aligned16(sendbuf) || (reinterpret_cast<uintptr_t>(buf_offset) & 7u))
    return MC_ERR_INVALID;
  const int64_t gy = layer_end - layer_begin;
  if (gy > 65535 || batch > 65535) return MC_ERR_UNSUPPORTED;
  RangeArgs a;
  a.pool = static_cast<char*>(pool->base);
  a.buf = static_cast<char*>(sendbuf);
  a.pages = page_table;
  a.layer_stride = mc::layer_stride_bytes(pool);
  a.page_stride = mc::page_stride_bytes(pool);
  a.num_pages = pool->num_pages;
  a.n_table_pages = 0;
  a.layer_begin = layer_begin;
  a.s0 = 0;
  a.s1 = 0;
  a.hkv = pool->num_kv_heads;
  a.cu_pages = cu_pages;
  a.s0_of = s0;
  a.s1_of = s1;
  a.buf_offset = buf_offset;
  a.skipped = pool->skipped;
  dim3 grid(2u * (unsigned)max_range_pages, (unsigned)gy, (unsigned)batch);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (pack)
    hipLaunchKernelGGL((range_copy_kernel<true, true>), grid, dim3(kThreads), 0, hs, a);
  else
    hipLaunchKernelGGL((range_copy_kernel<false, true>), grid, dim3(kThreads), 0, hs, a);
  return mc::launch_status();
}

}  // namespace

extern "C" {

mc_status mc_kv_pack_range(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                           const int32_t* pages, int32_t n_table_pages, int32_t s0, int32_t s1,
                           void* sendbuf, void* stream) {
  return range_copy(true, pool, layer_begin, layer_end, pages, n_table_pages, s0, s1, sendbuf,
                    stream);
}

mc_status mc_kv_unpack_range(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                             const int32_t* pages, int32_t n_table_pages, int32_t s0, int32_t s1,
                             const void* sendbuf, void* stream) {
  return range_copy(false, pool, layer_begin, layer_end, pages, n_table_pages, s0, s1,
                    const_cast<void*>(sendbuf), stream);
}

mc_status mc_kv_pack_batch(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                           int32_t batch, const int32_t* page_table, const int32_t* cu_pages,
                           const int32_t* s0, const int32_t* s1, const int64_t* buf_offset,
                           int32_t max_range_pages, void* sendbuf, void* stream) {
  return range_copy_batch(true, pool, layer_begin, layer_end, batch, page_table, cu_pages, s0, s1,
                          buf_offset, max_range_pages, sendbuf, stream);
}

mc_status mc_kv_unpack_batch(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                             int32_t batch, const int32_t* page_table, const int32_t* cu_pages,
                             const int32_t* s0, const int32_t* s1, const int64_t* buf_offset,
                             int32_t max_range_pages, const void* sendbuf, void* stream) {
  return range_copy_batch(false, pool, layer_begin, layer_end, batch, page_table, cu_pages, s0, s1,
                          buf_offset, max_range_pages, const_cast<void*>(sendbuf), stream);
}

static mc_status append_impl(const mc_pool_desc* pool, int32_t layer, const void* k_new,
                             const void* v_new, int32_t batch, int32_t total_q,
                             const int32_t* cu_q, const int32_t* begin, const int32_t* page_table,
                             const int32_t* cu_pages, bool send, int32_t send_layer_begin,
                             const int32_t* s0, const int32_t* s1, const int64_t* buf_offset,
                             void* sendbuf, void* stream) {
  mc_status st = mc::check_pool(pool);
  if (st != MC_OK) return st;
  if (layer < 0 || layer >= pool->num_layers) return MC_ERR_RANGE;
  if (send && (send_layer_begin < 0 || send_layer_begin > layer)) return MC_ERR_RANGE;
  if (batch < 0 || total_q < 0) return MC_ERR_INVALID;
  if (batch == 0 || total_q == 0) return MC_OK;
  if (!k_new || !v_new || !cu_q || !begin || !page_table || !cu_pages) return MC_ERR_INVALID;
  if (!mc::aligned16(k_new) || !mc::aligned16(v_new)) return MC_ERR_INVALID;
  if (send && (!s0 || !s1 || !buf_offset || !sendbuf || !mc::aligned16(sendbuf) ||
               (reinterpret_cast<uintptr_t>(buf_offset) & 7u)))
    return MC_ERR_INVALID;
  AppendArgs a;
  a.pool_layer = static_cast<char*>(pool->base) + layer * mc::layer_stride_bytes(pool);
  a.k_new = static_cast<const char*>(k_new);
  a.v_new = static_cast<const char*>(v_new);
  a.cu_q = cu_q;
  a.begin = begin;
  a.page_table = page_table;
  a.cu_pages = cu_pages;
  a.page_stride = mc::page_stride_bytes(pool);
  a.num_pages = pool->num_pages;
  a.batch = batch;
  a.total_q = total_q;
  a.hkv = pool->num_kv_heads;
  a.buf = static_cast<char*>(sendbuf);
  a.s0_of = s0;
  a.s1_of = s1;
  a.buf_offset = buf_offset;
  a.layer_rel = send ? layer - send_layer_begin : 0;
  a.skipped = pool->skipped;
  dim3 grid(2u * ((total_q + kPage - 1) / kPage));
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (send)
    hipLaunchKernelGGL(append_kernel<true>, grid, dim3(kThreads), 0, hs, a);
  else
    hipLaunchKernelGGL(append_kernel<false>, grid, dim3(kThreads), 0, hs, a);
  return mc::launch_status();
}

mc_status mc_kv_append(const mc_pool_desc* pool, int32_t layer, const void* k_new,
                       const void* v_new, int32_t batch, int32_t total_q, const int32_t* cu_q,
                       const int32_t* begin, const int32_t* page_table, const int32_t* cu_pages,
                       void* stream) {
  return append_impl(pool, layer, k_new, v_new, batch, total_q, cu_q, begin, page_table, cu_pages,
                     false, 0, nullptr, nullptr, nullptr, nullptr, stream);
}

mc_status mc_kv_append_send(const mc_pool_desc* pool, int32_t layer, const void* k_new,
                            const void* v_new, int32_t batch, int32_t total_q,
                            const int32_t* cu_q, const int32_t* begin, const int32_t* page_table,
                            const int32_t* cu_pages, int32_t send_layer_begin, const int32_t* s0,
                            const int32_t* s1, const int64_t* buf_offset, void* sendbuf,
                            void* stream) {
  return append_impl(pool, layer, k_new, v_new, batch, total_q, cu_q, begin, page_table, cu_pages,
                     true, send_layer_begin, s0, s1, buf_offset, sendbuf, stream);
}

mc_status mc_kv_copy_check(const mc_pool_desc* pool, int32_t* skipped_out, void* stream) {
  if (!pool || !pool->skipped || (reinterpret_cast<uintptr_t>(pool->skipped) & 3u))
    return MC_ERR_INVALID;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  int32_t n = 0;
  if (hipMemcpyAsync(&n, pool->skipped, sizeof(n), hipMemcpyDeviceToHost, hs) != hipSuccess ||
      hipMemsetAsync(pool->skipped, 0, sizeof(n), hs) != hipSuccess ||
      hipStreamSynchronize(hs) != hipSuccess)
    return MC_ERR_HIP;
  if (skipped_out) *skipped_out = n;
  return n == 0 ? MC_OK : MC_ERR_RANGE;
}

mc_status mc_kv_copy_page(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                          int32_t src_page, int32_t dst_page, int32_t slots, void* stream) {
  mc_status st = mc::check_pool(pool);
  if (st != MC_OK) return st;
  if (layer_begin < 0 || layer_end < layer_begin || layer_end > pool->num_layers)
    return MC_ERR_RANGE;
  if (src_page < 0 || src_page >= pool->num_pages || dst_page < 0 || dst_page >= pool->num_pages ||
      slots < 0 || slots > kPage)
    return MC_ERR_RANGE;
  if (src_page == dst_page) return MC_ERR_ALIAS;
  if (slots == 0 || layer_begin == layer_end) return MC_OK;
  if (layer_end - layer_begin > 65535) return MC_ERR_UNSUPPORTED;
  PageCopyArgs a;
  a.pool = static_cast<char*>(pool->base);
  a.layer_stride = mc::layer_stride_bytes(pool);
  a.page_stride = mc::page_stride_bytes(pool);
  a.layer_begin = layer_begin;
  a.src_page = src_page;
  a.dst_page = dst_page;
  a.slots = slots;
  a.hkv = pool->num_kv_heads;
  hipLaunchKernelGGL(page_copy_kernel, dim3(2, (unsigned)(layer_end - layer_begin)), dim3(kThreads),
                     0, static_cast<hipStream_t>(stream), a);
  return mc::launch_status();
}

}  // extern "C"
