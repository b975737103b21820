// Paged prefix-prefill attention for gfx950 (CDNA4): attention of the new token
// range [begin, end) of each sequence over the KV already in its pages plus the
// new range itself (paper Sec. 3.1 start_generate, Sec. 3.3 split prefill,
// Sec. 3.4 attention(qkv_data)), and the planning step that precedes it
// (Sec. 3.4 begin_forward: plan the metadata once for all layers).
//
// Kernel shape
//   * one workgroup (4 wavefronts of 64) per (q tile, kv head).  A q tile is
//     128 rows = TOK tokens x G query heads of one kv head's group (TOK = 128/G),
//     so every K/V byte staged in LDS serves the whole GQA group.
//   * the KV loop walks 64-key tiles (4 pages) through the page table; each page
//     contributes one contiguous 4 KiB run of K and one of V for this kv head.
//   * S^T = K Q^T on v_mfma_f32_32x32x16 (A = K rows from LDS, B = Q held in
//     registers): a lane then owns ONE query row (column l%32) and 16 keys per
//     32-key chunk, so the softmax row max / row sum are in-lane plus one
//     exchange with lane l^32, and the rescale factor is a per-lane scalar.
//   * O^T += V^T P^T: P^T is the B operand straight from the S^T accumulators
//     (no LDS round trip); V^T comes from LDS with ds_read_b64_tr_b16, which
//     transposes 4 keys x 16 d per 16-lane group on the way in.
//   * LDS tiles are XOR-swizzled so both the row reads (K) and the transposing
//     reads (V) spread over all banks.
#include <math.h>

#include <type_traits>

#include "mc_common.h"

namespace {

using mc::kHeadPageBytes;
using mc::kPage;
using mc::kRowBytes;

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBM = 128;       // rows (token x head-in-group) per workgroup
constexpr int kBN = 64;        // keys per KV tile
constexpr int kThreads = 256;  // 4 wavefronts, 32 rows each
constexpr int kPlanThreads = 1024;
constexpr int kBuckets = 4096;
constexpr int32_t kPlanMagic = 0x6d63706c;

struct PlanHeader {
  int32_t magic;
  int32_t err;        // mc_status found on the device by the plan kernel
  int32_t num_tiles;  // q tiles in the work list
  int32_t tile_tokens;
  int32_t batch;
  int32_t total_q;
  int32_t pad[10];
};
static_assert(sizeof(PlanHeader) == 64, "header is 64 bytes");

struct WorkspaceLayout {
  size_t cu_tiles, tile_seq, tile_row0, total;
  int32_t max_tiles;
};

inline size_t round16(size_t x) { return (x + 15) & ~size_t(15); }

inline WorkspaceLayout workspace_layout(int32_t batch, int32_t total_q, int32_t tile_tokens) {
  WorkspaceLayout w;
  w.max_tiles = (int32_t)(((int64_t)total_q + tile_tokens - 1) / tile_tokens + batch);
  w.cu_tiles = sizeof(PlanHeader);
  w.tile_seq = w.cu_tiles + round16(sizeof(int32_t) * ((size_t)batch + 1));
  w.tile_row0 = w.tile_seq + round16(sizeof(int32_t) * (size_t)w.max_tiles);
  w.total = w.tile_row0 + round16(sizeof(int32_t) * (size_t)w.max_tiles);
  return w;
}

// ---------------------------------------------------------------- plan ------
struct PlanArgs {
  const int32_t* cu_q;
  const int32_t* begin;
  const int32_t* page_table;
  const int32_t* cu_pages;
  PlanHeader* hdr;
  int32_t* cu_tiles;
  int32_t* tile_seq;
  int32_t* tile_row0;
  int32_t batch, total_q, tile_tokens, num_pages, max_tiles;
};

// Block-wide exclusive scan of one value per thread (kPlanThreads threads).
__device__ int block_exclusive_scan(int v, int* lds, int* total) {
  const int t = threadIdx.x;
  lds[t] = v;
  __syncthreads();
  for (int off = 1; off < kPlanThreads; off <<= 1) {
    int add = t >= off ? lds[t - off] : 0;
    __syncthreads();
    lds[t] += add;
    __syncthreads();
  }
  const int incl = lds[t];
  *total = lds[kPlanThreads - 1];
  __syncthreads();
  return incl - v;
}

// One workgroup.  Validates the ragged-batch arrays, cuts every sequence's new
// range into q tiles of tile_tokens tokens and orders the tiles by decreasing
// number of KV tiles (longest first), so that the tail of the launch is made of
// short work items.
__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs a) {
  __shared__ int scan[kPlanThreads];
  __shared__ int hist[kBuckets];
  __shared__ int s_err, s_maxcost;
  const int t = threadIdx.x;
  if (t == 0) { s_err = 0; s_maxcost = 1; }
  for (int i = t; i < kBuckets; i += kPlanThreads) hist[i] = 0;
  __syncthreads();

  // 1. validate, count tiles per sequence (contiguous chunk of sequences per thread)
  const int per = (a.batch + kPlanThreads - 1) / kPlanThreads;
  const int s_lo = min(t * per, a.batch), s_hi = min(s_lo + per, a.batch);
  int my_tiles = 0, err = 0, maxcost = 1;
  if (t == 0 && (a.cu_q[0] != 0 || a.cu_q[a.batch] != a.total_q || a.cu_pages[0] < 0)) err = 1;
  for (int s = s_lo; s < s_hi; ++s) {
    const int q = a.cu_q[s + 1] - a.cu_q[s], b = a.begin[s];
    const int np = a.cu_pages[s + 1] - a.cu_pages[s];
    if (q < 0 || b < 0 || np < 0 || a.cu_q[s] < 0 || a.cu_q[s + 1] > a.total_q) { err = 1; continue; }
    if (q == 0) continue;
    const int64_t end = (int64_t)b + q;
    if ((end + kPage - 1) / kPage > np) { err = 1; continue; }
    my_tiles += (q + a.tile_tokens - 1) / a.tile_tokens;
    maxcost = max(maxcost, (int)((end + kBN - 1) / kBN));
  }
  if (err) atomicOr(&s_err, 1);
  atomicMax(&s_maxcost, maxcost);
  __syncthreads();
  if (s_err) {
    if (t == 0) { a.hdr->err = MC_ERR_RANGE; a.hdr->num_tiles = 0; a.hdr->magic = kPlanMagic; }
    return;
  }
  // 2. page ids of every needed table entry (one wavefront per sequence at a time)
  for (int s = t >> 6; s < a.batch; s += kPlanThreads >> 6) {
    const int q = a.cu_q[s + 1] - a.cu_q[s];
    if (q == 0) continue;
    const int need = (a.begin[s] + q + kPage - 1) / kPage, p0 = a.cu_pages[s];
    for (int i = t & 63; i < need; i += 64) {
      const int32_t pg = a.page_table[p0 + i];
      if (pg < 0 || pg >= a.num_pages) err = 1;
    }
  }
  if (err) atomicOr(&s_err, 1);
  // 3. exclusive scan of tiles per sequence
  int total_tiles;
  int base = block_exclusive_scan(my_tiles, scan, &total_tiles);
  for (int s = s_lo; s < s_hi; ++s) {
    a.cu_tiles[s] = base;
    const int q = a.cu_q[s + 1] - a.cu_q[s];
    base += (q + a.tile_tokens - 1) / a.tile_tokens;
  }
  if (t == 0) a.cu_tiles[a.batch] = total_tiles;
  __threadfence_block();
  __syncthreads();
  if (s_err || total_tiles > a.max_tiles) {
    if (t == 0) { a.hdr->err = MC_ERR_RANGE; a.hdr->num_tiles = 0; a.hdr->magic = kPlanMagic; }
    return;
  }
  // 4. counting sort of tiles by cost (number of KV tiles), heaviest first
  int shift = 0;
  while ((s_maxcost >> shift) >= kBuckets) ++shift;
  auto locate = [&](int i, int& s, int& row0, int& bucket) {
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.cu_tiles[mid] <= i) lo = mid; else hi = mid;
    }
    s = lo;
    row0 = (i - a.cu_tiles[s]) * a.tile_tokens;
    const int q = a.cu_q[s + 1] - a.cu_q[s];
    const int kv_len = a.begin[s] + min(q, row0 + a.tile_tokens);
    bucket = kBuckets - 1 - (((kv_len + kBN - 1) / kBN) >> shift);
  };
  for (int i = t; i < total_tiles; i += kPlanThreads) {
    int s, row0, bucket;
    locate(i, s, row0, bucket);
    atomicAdd(&hist[bucket], 1);
  }
  __syncthreads();
  {
    constexpr int kPer = kBuckets / kPlanThreads;
    int local[kPer], sum = 0;
    for (int i = 0; i < kPer; ++i) { local[i] = hist[t * kPer + i]; sum += local[i]; }
    int tot, off = block_exclusive_scan(sum, scan, &tot);
    for (int i = 0; i < kPer; ++i) { hist[t * kPer + i] = off; off += local[i]; }
  }
  __syncthreads();
  for (int i = t; i < total_tiles; i += kPlanThreads) {
    int s, row0, bucket;
    locate(i, s, row0, bucket);
    const int pos = atomicAdd(&hist[bucket], 1);
    a.tile_seq[pos] = s;
    a.tile_row0[pos] = row0;
  }
  if (t == 0) {
    a.hdr->err = MC_OK;
    a.hdr->num_tiles = total_tiles;
    a.hdr->tile_tokens = a.tile_tokens;
    a.hdr->batch = a.batch;
    a.hdr->total_q = a.total_q;
    a.hdr->magic = kPlanMagic;
  }
}

// ----------------------------------------------------------- attention ------
template <typename T> struct Mfma;
template <> struct Mfma<_Float16> {
  typedef f16x8 vec8;
  static __device__ __forceinline__ f32x16 run(vec8 a, vec8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float x, float y) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v;
    v[0] = (_Float16)x;
    v[1] = (_Float16)y;
    return __builtin_bit_cast(uint32_t, v);
  }
};
template <> struct Mfma<__bf16> {
  typedef bf16x8 vec8;
  static __device__ __forceinline__ f32x16 run(vec8 a, vec8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float x, float y) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v;
    v[0] = (__bf16)x;
    v[1] = (__bf16)y;
    return __builtin_bit_cast(uint32_t, v);
  }
};

struct AttnArgs {
  const char* pool_layer;  // pool base + layer offset
  const char* q;
  char* out;
  float* lse;
  const int32_t* cu_q;
  const int32_t* begin;
  const int32_t* page_table;
  const int32_t* cu_pages;
  const PlanHeader* hdr;
  const int32_t* tile_seq;
  const int32_t* tile_row0;
  int64_t page_stride;     // bytes
  int32_t num_pages, hkv, hq, batch, total_q;
  float scale, scale_log2;  // softmax scale, and scale * log2(e)
};

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* gbl_void_ptr;
// Read-only metadata is addressed through the constant address space so that wave-uniform
// reads stay scalar loads (no vector-memory counter involved) even after LDS copies and stores.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;

constexpr int kTileBytes = kBN * kRowBytes;   // one K or V tile in LDS: 16 KiB

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(size_t)(lds_void_ptr)(p);
}

// Asynchronous 16-byte-per-lane copy from global memory straight into LDS: lane L's bytes
// land at lds_base + 16 L.  base and lds_base are wave-uniform.  Issued as inline assembly so
// that the compiler does not serialise it against later LDS reads of OTHER buffers; completion
// is awaited explicitly (s_waitcnt vmcnt(0)) before the workgroup barrier that publishes it.
__device__ __forceinline__ void copy16_to_lds(const char* base, uint32_t lane_off,
                                              uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_off), "s"(base), "s"(lds_base) : "memory", "m0");
}

// LDS tile: 64 rows (keys) x 256 B.  16-byte chunk c of row r sits at chunk position
//   K: c ^ (r & 15)        -> 16 lanes reading one chunk of 16 consecutive rows hit 16 positions
//   V: c ^ ((r & 3) << 2)  -> a transposing read of 4 consecutive rows x 64 B hits 16 positions
__device__ __forceinline__ int k_swz(int row, int chunk) { return row * kRowBytes + ((chunk ^ (row & 15)) << 4); }
__device__ __forceinline__ int v_swz(int row, int chunk) { return row * kRowBytes + ((chunk ^ ((row & 3) << 2)) << 4); }

// max of three floats in one instruction (written as assembly: through fmaxf every score would
// first pass a NaN-quieting instruction of its own)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Pipeline of one workgroup (one barrier per KV tile):
//   iteration j   issues the global->LDS copies of K(j+2) and V(j+1)   (asynchronous, no VGPRs)
//                 finds the row max of S(j), rescales O only if the max moved far
//                 computes S(j+1) = K(j+1) Q^T on the MFMA pipe while the VALU does the
//                 exponentials of S(j), then O^T += V(j)^T P(j)^T
//   so K is always one tile ahead of V, and two LDS buffers of each are enough.
template <typename T, int G>
__global__ __launch_bounds__(kThreads, 2) void attn_kernel(AttnArgs a) {
  constexpr int TOK = kBM / G;  // tokens per q tile
  typedef typename Mfma<T>::vec8 vec8;
  __shared__ __attribute__((aligned(1024))) char lds_k[2 * kTileBytes];
  __shared__ __attribute__((aligned(1024))) char lds_v[2 * kTileBytes];

  const int hk = blockIdx.x % a.hkv;
  const int wi = blockIdx.x / a.hkv;
  // the work list must come from a plan made for this very batch
  if (a.hdr->magic != kPlanMagic || wi >= a.hdr->num_tiles || a.hdr->tile_tokens != TOK ||
      a.hdr->batch != a.batch || a.hdr->total_q != a.total_q)
    return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;

  const int seq = a.tile_seq[wi], row0 = a.tile_row0[wi];
  const int q0 = a.cu_q[seq], q_len = a.cu_q[seq + 1] - q0, b = a.begin[seq];
  const int ntok = min(TOK, q_len - row0);          // valid tokens in this tile (>= 1)
  const int first_pos = b + row0;                    // position of the tile's first token
  const int kv_len = first_pos + ntok;               // keys [0, kv_len) are needed
  const int n_kv_tiles = (kv_len + kBN - 1) / kBN;
  const int last_pidx = (kv_len - 1) / kPage;        // last table entry that holds a needed key
  const_i32_ptr table = (const_i32_ptr)(a.page_table + a.cu_pages[seq]);

  // this lane's query row
  const int r = wave * 32 + l32;                     // row in tile, head-major
  const int g = r / TOK, tt = r % TOK;
  const bool row_ok = tt < ntok;
  const int my_pos = first_pos + (row_ok ? tt : ntok - 1);   // causal limit of the row
  const int64_t q_row = ((int64_t)(q0 + row0 + tt) * a.hq + hk * G + g) * kRowBytes;

  // Q as the B operand: lane holds d = 16 kk + 8 half + [0,8) of its row, kk = 0..7
  vec8 qreg[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    u32x4 v = {0, 0, 0, 0};
    if (row_ok) v = *reinterpret_cast<const u32x4*>(a.q + q_row + kk * 32 + half * 16);
    qreg[kk] = __builtin_bit_cast(vec8, v);
  }

  // ---- global -> LDS copies (no VGPR staging) -------------------------------------
  // A wavefront's copy instruction fills 1 KiB of LDS linearly (lane L -> bytes 16 L..),
  // i.e. 4 tile rows.  Copy i of wave w fills rows 16 i + 4 w + L/16 (page i of the tile,
  // slots 4 w..4 w+3); lane L fetches the 16-byte chunk that the swizzle wants at position
  // L%16 of that row.  Rows of keys at or beyond kv_len receive whatever the page holds
  // (K: discarded by the mask; V: zeroed in LDS before the last tile's P.V, since 0 x NaN
  // would poison the accumulators).
  const int ld_slot = 4 * wave + (lane >> 4), ld_pos = lane & 15;
  const char* pool_k = a.pool_layer + (int64_t)hk * kHeadPageBytes;
  const uint32_t k_lane_off = ld_slot * kRowBytes + ((ld_pos ^ ld_slot) << 4);
  const uint32_t v_lane_off = ld_slot * kRowBytes + ((ld_pos ^ ((ld_slot & 3) << 2)) << 4) +
                              (uint32_t)a.hkv * kHeadPageBytes;   // V run sits hkv blocks after K
  const uint32_t page_blocks = 2u * a.hkv;     // 4 KiB blocks per page
  // wave-uniform address of this kv head's K run in each of the 4 pages of tile jt.  Table
  // entries past the last needed one are replaced by the last needed one.
  struct TilePages { const char* base[4]; };
  auto page_base = [&](int32_t pg) {
    pg = min(max(pg, 0), a.num_pages - 1);         // checked by the plan; stay in bounds anyway
    return pool_k + ((uint64_t)((uint32_t)pg * page_blocks) << 12);
  };
  auto tile_pages = [&](int jt) {                  // scalar reads: used before the loop only
    TilePages t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t.base[i] = page_base(table[min(jt * 4 + i, last_pidx)]);
    return t;
  };
  // Inside the loop the 4 page ids of a tile are fetched one iteration early by a vector
  // load (lane i & 3 holds id i) and moved to scalar registers when the addresses are built,
  // so no iteration waits on a page-table read.
  const int32_t* table_g = a.page_table + a.cu_pages[seq];
  auto fetch_ids = [&](int jt) { return table_g[min(jt * 4 + (lane & 3), last_pidx)]; };
  auto pages_from_ids = [&](int32_t ids) {
    TilePages t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t.base[i] = page_base(__builtin_amdgcn_readlane(ids, i));
    return t;
  };
  auto issue_tile = [&](const TilePages& t, bool is_v, char* lds_tile) {
    const uint32_t dst = lds_addr(lds_tile) + wave * 1024;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      copy16_to_lds(t.base[i], is_v ? v_lane_off : k_lane_off, dst + i * 4096);
  };
  auto wait_copies_and_sync = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  // ---- S^T = K Q^T for one tile: two 32-key chunks ----------------------------------
  auto qk_tile = [&](const char* ktile, f32x16 (&s_acc)[2]) {
#pragma unroll
    for (int c = 0; c < 2; ++c) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[c][i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const int row = c * 32 + l32;
        vec8 kfrag = *reinterpret_cast<const vec8*>(ktile + k_swz(row, 2 * kk + half));
        s_acc[c] = Mfma<T>::run(kfrag, qreg[kk], s_acc[c]);
      }
    }
  };

  f32x16 o_acc[4];
#pragma unroll
  for (int dc = 0; dc < 4; ++dc)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[dc][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;   // reference max (raw scores), this lane's partial sum
  const float c2 = a.scale_log2;
  // per-lane constants of the transposing V read: 16-lane group gq, lane j in group
  const int j16 = lane & 15, gq = (lane >> 4) & 1;

  // key held by accumulator register i of chunk c of tile jt: 64 jt + 32 c + 8 (i/4) + 4 half + i%4
  auto mask_tile = [&](int jt, f32x16 (&s)[2]) {
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = jt * kBN + c * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
        if (key > my_pos) s[c][i] = -INFINITY;
      }
  };
  auto row_max = [&](const f32x16 (&s)[2]) {
    float mx = s[0][0];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int i = 0; i < 16; i += 2) mx = max3(mx, s[c][i], s[c][i + 1]);
    // the other 32 keys of the row sit in lane l ^ 32: swap the wave's halves on the VALU
    const uint32_t bits = __builtin_bit_cast(uint32_t, mx);
    const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
    return fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1]));
  };

  // tile j is fully visible to every row of the q tile iff 64 (j+1) <= first_pos + 1
  const int n_full = (first_pos + 1) / kBN;

  f32x16 s_cur[2];
  TilePages pages_next = tile_pages(min(1, n_kv_tiles - 1));   // pages of tile j+1 during tile j
  int32_t ids_next2 = fetch_ids(min(2, n_kv_tiles - 1));       // ids of tile j+2 during tile j
  {
    const TilePages p0 = tile_pages(0);
    issue_tile(p0, false, lds_k);
    issue_tile(p0, true, lds_v);
    issue_tile(pages_next, false, lds_k + kTileBytes);
  }
  wait_copies_and_sync();
  qk_tile(lds_k, s_cur);
  if (n_full == 0) mask_tile(0, s_cur);
  float mx_cur = row_max(s_cur);
  __syncthreads();   // every wave has read K(0) before the first iteration overwrites it

  // One KV tile.  HAS_NEXT: tile j+1 exists; MASK_NEXT: it reaches the causal diagonal.
  auto body = [&](int jt, auto mask_tag, auto next_tag) {
    constexpr bool MASK_NEXT = decltype(mask_tag)::value;
    constexpr bool HAS_NEXT = decltype(next_tag)::value;
    const int par = jt & 1;
    const char* ktile = lds_k + (par ^ 1) * kTileBytes;   // K(j+1)
    const char* vtile = lds_v + par * kTileBytes;         // V(j)
    // Operand fragments are fetched from LDS a fixed number of MFMAs ahead of their use.
    // QK step t (0..15): key chunk c = t & 1, d-step kk = t >> 1 (the two accumulator chains
    // alternate).  PV step u (0..15): key chunk c = u >> 3, 16-key step s = (u >> 2) & 1,
    // d chunk dc = u & 3 (four accumulator chains alternate); the step covers accumulator
    // registers 8s..8s+7 of chunk c, i.e. for this lane-half the keys
    // 32c + 16s + {0..3} + 4 half and 32c + 16s + 8 + {0..3} + 4 half.
    constexpr int kAhead = 4;
    auto k_frag = [&](int t) {
      return *reinterpret_cast<const vec8*>(ktile + k_swz((t & 1) * 32 + l32, 2 * (t >> 1) + half));
    };
    auto v_frag = [&](int u) {
      const int c = u >> 3, st = (u >> 2) & 1, dc = u & 3;
      // 16-lane group reads 4 keys x 16 d; lane j supplies key (j/4), d-quad (j%4)
      const int key_lo = c * 32 + st * 16 + 4 * half + (j16 >> 2);
      const int chunk = dc * 4 + gq * 2 + ((j16 & 3) >> 1);
      const int sub = (j16 & 1) * 8;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_ptr)(vtile + v_swz(key_lo, chunk) + sub));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_ptr)(vtile + v_swz(key_lo + 8, chunk) + sub));
      return __builtin_bit_cast(vec8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    vec8 kf[kAhead], vf[kAhead];
    if (HAS_NEXT) {
#pragma unroll
      for (int t = 0; t < kAhead; ++t) kf[t] = k_frag(t);
      const TilePages pages_next2 = pages_from_ids(ids_next2);
      issue_tile(pages_next2, false, lds_k + par * kTileBytes);
      issue_tile(pages_next, true, lds_v + (par ^ 1) * kTileBytes);
      pages_next = pages_next2;
      ids_next2 = fetch_ids(min(jt + 3, n_kv_tiles - 1));
    } else {
      if (kv_len < (jt + 1) * kBN) {
        // last tile: zero the V rows of keys >= kv_len (their P is 0, their bytes are arbitrary)
        const int valid = kv_len - jt * kBN;
        const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = i * 16 + (tid >> 4);
          if (row >= valid)
            *reinterpret_cast<u32x4*>(lds_v + par * kTileBytes + row * kRowBytes + (tid & 15) * 16) = zero;
        }
        __syncthreads();
      }
#pragma unroll
      for (int u = 0; u < kAhead; ++u) vf[u] = v_frag(u);
    }
    // ---- move the reference max (and rescale O, l) only when some row's max rose by
    //      more than 2^8 in the exp2 domain: p stays below 2^8, sums stay exact
    if (__builtin_amdgcn_ballot_w64((mx_cur - m_run) * c2 > 8.f) != 0) {
      const float m_new = fmaxf(m_run, mx_cur);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[dc][i] *= alpha;
    }
    const float mc2 = m_run * c2;
    __builtin_amdgcn_sched_barrier(0);
    // ---- phase 1: S(j+1) = K(j+1) Q^T on the MFMA pipe, exponentials of S(j) on the VALU.
    //      Each step: one MFMA, one fragment fetch for kAhead steps later, 1/16 of the softmax.
    f32x16 s_next[2];
    const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    float psum = 0.f;
    uint32_t p_pk[2][8];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      {
        const int c = t >> 3, i = 2 * (t & 7);
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[c][i], c2, -mc2));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[c][i + 1], c2, -mc2));
        psum += p0 + p1;   // the unrounded values: LSE must not inherit P's 2-byte rounding
        p_pk[c][t & 7] = Mfma<T>::pack2(p0, p1);
      }
      if (HAS_NEXT) {
        s_next[t & 1] = Mfma<T>::run(kf[t % kAhead], qreg[t >> 1], t < 2 ? zero16 : s_next[t & 1]);
        if (t + kAhead < 16) kf[t % kAhead] = k_frag(t + kAhead);
        else vf[(t + kAhead) % kAhead] = v_frag(t + kAhead - 16);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    l_run += psum;
    if (HAS_NEXT && MASK_NEXT) mask_tile(jt + 1, s_next);
    // ---- phase 2: O^T += V(j)^T P(j)^T on the MFMA pipe, row max of S(j+1) on the VALU ----
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int c = u >> 3, st = (u >> 2) & 1, dc = u & 3;
      u32x4 pw = {p_pk[c][4 * st], p_pk[c][4 * st + 1], p_pk[c][4 * st + 2], p_pk[c][4 * st + 3]};
      o_acc[dc] = Mfma<T>::run(vf[u % kAhead], __builtin_bit_cast(vec8, pw), o_acc[dc]);
      if (u + kAhead < 16) vf[u % kAhead] = v_frag(u + kAhead);
      if (HAS_NEXT) mx = max3(mx, s_next[u >> 3][2 * (u & 7)], s_next[u >> 3][2 * (u & 7) + 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (HAS_NEXT) {
      // the other 32 keys of the row sit in lane l ^ 32: swap the wave's halves on the VALU
      const uint32_t bits = __builtin_bit_cast(uint32_t, mx);
      const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
      mx_cur = fmaxf(__builtin_bit_cast(float, sw[0]), __builtin_bit_cast(float, sw[1]));
      s_cur[0] = s_next[0];
      s_cur[1] = s_next[1];
    }
    wait_copies_and_sync();
  };

  int jt = 0;
  for (; jt < min(n_full, n_kv_tiles) - 1; ++jt) body(jt, std::false_type{}, std::true_type{});
  for (; jt < n_kv_tiles - 1; ++jt) body(jt, std::true_type{}, std::true_type{});
  body(jt, std::true_type{}, std::false_type{});

  // ---- epilogue: normalise, stage O through LDS for full-row stores, write LSE ----
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.f / l_tot;
  char* stage = lds_k + wave * (32 * kRowBytes);   // 8 KiB per wave; all tiles are consumed
#pragma unroll
  for (int dc = 0; dc < 4; ++dc)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // registers 4j..4j+3 hold d = 32 dc + 8 j + 4 half + {0..3}: 8 bytes of chunk 4 dc + j
      u32x2 w;
      w[0] = Mfma<T>::pack2(o_acc[dc][4 * j] * inv, o_acc[dc][4 * j + 1] * inv);
      w[1] = Mfma<T>::pack2(o_acc[dc][4 * j + 2] * inv, o_acc[dc][4 * j + 3] * inv);
      *reinterpret_cast<u32x2*>(stage + k_swz(l32, 4 * dc + j) + half * 8) = w;
    }
  if (row_ok && half == 0)
    a.lse[(int64_t)(q0 + row0 + tt) * a.hq + hk * G + g] = m_run * a.scale + __logf(l_tot);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int lr = 4 * i + (lane >> 4);               // row of this wave's 32
    const int rr = wave * 32 + lr, gg = rr / TOK, t2 = rr % TOK;
    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + k_swz(lr, lane & 15));
    if (t2 < ntok)
      *reinterpret_cast<u32x4*>(a.out + ((int64_t)(q0 + row0 + t2) * a.hq + hk * G + gg) * kRowBytes +
                                (lane & 15) * 16) = v;
  }
}

template <typename T>
mc_status launch_attn(int G, dim3 grid, hipStream_t hs, const AttnArgs& a) {
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_kernel<T, 1>), grid, dim3(kThreads), 0, hs, a); break;
    case 2: hipLaunchKernelGGL((attn_kernel<T, 2>), grid, dim3(kThreads), 0, hs, a); break;
    case 4: hipLaunchKernelGGL((attn_kernel<T, 4>), grid, dim3(kThreads), 0, hs, a); break;
    case 8: hipLaunchKernelGGL((attn_kernel<T, 8>), grid, dim3(kThreads), 0, hs, a); break;
    default: return MC_ERR_UNSUPPORTED;
  }
  return mc::launch_status();
}

mc_status check_attn_shape(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                           int32_t total_q, int* G_out) {
  mc_status st = mc::check_pool(pool);
  if (st != MC_OK) return st;
  if (num_q_heads <= 0 || batch < 0 || total_q < 0) return MC_ERR_INVALID;
  if (num_q_heads % pool->num_kv_heads != 0) return MC_ERR_UNSUPPORTED;
  const int G = num_q_heads / pool->num_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return MC_ERR_UNSUPPORTED;
  *G_out = G;
  return MC_OK;
}

}  // namespace

extern "C" {

size_t mc_attn_workspace_size(int32_t batch, int32_t total_q, int32_t num_q_heads,
                              int32_t num_kv_heads) {
  if (batch < 0 || total_q < 0 || num_q_heads <= 0 || num_kv_heads <= 0) return 0;
  if (num_q_heads % num_kv_heads != 0) return 0;
  const int G = num_q_heads / num_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return 0;
  return workspace_layout(batch, total_q, kBM / G).total;
}

mc_status mc_attn_plan(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                       int32_t total_q, const int32_t* cu_q, const int32_t* begin,
                       const int32_t* page_table, const int32_t* cu_pages, void* workspace,
                       size_t workspace_bytes, void* stream) {
  int G = 0;
  mc_status st = check_attn_shape(pool, num_q_heads, batch, total_q, &G);
  if (st != MC_OK) return st;
  if (!workspace || !mc::aligned16(workspace)) return MC_ERR_INVALID;
  const WorkspaceLayout w = workspace_layout(batch, total_q, kBM / G);
  if (workspace_bytes < w.total) return MC_ERR_INVALID;
  if (batch > 0 && (!cu_q || !begin || !page_table || !cu_pages)) return MC_ERR_INVALID;
  if (batch == 0) {   // nothing to plan: a header with an empty work list
    if (!cu_q || !cu_pages) return MC_ERR_INVALID;
  }
  char* ws = static_cast<char*>(workspace);
  PlanArgs a;
  a.cu_q = cu_q;
  a.begin = begin;
  a.page_table = page_table;
  a.cu_pages = cu_pages;
  a.hdr = reinterpret_cast<PlanHeader*>(ws);
  a.cu_tiles = reinterpret_cast<int32_t*>(ws + w.cu_tiles);
  a.tile_seq = reinterpret_cast<int32_t*>(ws + w.tile_seq);
  a.tile_row0 = reinterpret_cast<int32_t*>(ws + w.tile_row0);
  a.batch = batch;
  a.total_q = total_q;
  a.tile_tokens = kBM / G;
  a.num_pages = pool->num_pages;
  a.max_tiles = w.max_tiles;
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0,
                     static_cast<hipStream_t>(stream), a);
  return mc::launch_status();
}

mc_status mc_attn_plan_check(const void* workspace, void* stream) {
  if (!workspace) return MC_ERR_INVALID;
  PlanHeader h;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (hipMemcpyAsync(&h, workspace, sizeof(h), hipMemcpyDeviceToHost, hs) != hipSuccess)
    return MC_ERR_HIP;
  if (hipStreamSynchronize(hs) != hipSuccess) return MC_ERR_HIP;
  if (h.magic != kPlanMagic) return MC_ERR_INVALID;
  return static_cast<mc_status>(h.err);
}

mc_status mc_prefix_prefill_attn(const mc_pool_desc* pool, int32_t layer, const void* q,
                                 int32_t num_q_heads, int32_t batch, int32_t total_q,
                                 const int32_t* cu_q, const int32_t* begin,
                                 const int32_t* page_table, const int32_t* cu_pages,
                                 float sm_scale, void* out, float* lse, const void* workspace,
                                 size_t workspace_bytes, void* stream) {
  int G = 0;
  mc_status st = check_attn_shape(pool, num_q_heads, batch, total_q, &G);
  if (st != MC_OK) return st;
  if (layer < 0 || layer >= pool->num_layers) return MC_ERR_RANGE;
  if (!(sm_scale >= 0.f) || !isfinite(sm_scale)) return MC_ERR_INVALID;
  if (batch == 0 || total_q == 0) return MC_OK;
  if (!q || !out || !lse || !cu_q || !begin || !page_table || !cu_pages || !workspace)
    return MC_ERR_INVALID;
  if (!mc::aligned16(q) || !mc::aligned16(out) || !mc::aligned16(workspace) ||
      (reinterpret_cast<uintptr_t>(lse) & 3u))
    return MC_ERR_INVALID;
  const WorkspaceLayout w = workspace_layout(batch, total_q, kBM / G);
  if (workspace_bytes < w.total) return MC_ERR_INVALID;
  const int64_t blocks = (int64_t)w.max_tiles * pool->num_kv_heads;
  if (blocks > 0x7fffffffll) return MC_ERR_UNSUPPORTED;
  const char* ws = static_cast<const char*>(workspace);
  AttnArgs a;
  a.pool_layer = static_cast<const char*>(pool->base) + layer * mc::layer_stride_bytes(pool);
  a.q = static_cast<const char*>(q);
  a.out = static_cast<char*>(out);
  a.lse = lse;
  a.cu_q = cu_q;
  a.begin = begin;
  a.page_table = page_table;
  a.cu_pages = cu_pages;
  a.hdr = reinterpret_cast<const PlanHeader*>(ws);
  a.tile_seq = reinterpret_cast<const int32_t*>(ws + w.tile_seq);
  a.tile_row0 = reinterpret_cast<const int32_t*>(ws + w.tile_row0);
  a.page_stride = mc::page_stride_bytes(pool);
  a.num_pages = pool->num_pages;
  a.hkv = pool->num_kv_heads;
  a.hq = num_q_heads;
  a.batch = batch;
  a.total_q = total_q;
  a.scale = sm_scale > 0.f ? sm_scale : 1.0f / sqrtf((float)mc::kHeadDim);
  a.scale_log2 = a.scale * 1.4426950408889634f;
  dim3 grid((unsigned)blocks);
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (pool->dtype == MC_F16) return launch_attn<_Float16>(G, grid, hs, a);
  return launch_attn<__bf16>(G, grid, hs, a);
}

}  // extern "C"
