// Paged prefix-prefill attention for gfx950 (CDNA4): attention of the new token
// range [begin, end) of each sequence over the KV already in its pages plus the
// new range itself (paper Sec. 3.1 start_generate, Sec. 3.3 split prefill,
// Sec. 3.4 attention(qkv_data)), and the planning step that precedes it
// (Sec. 3.4 begin_forward: plan the metadata once for all layers).
//
// Work
//   * plan_kernel cuts the ragged batch into work items: a q tile (128 rows = TOK
//     tokens x G query heads of one kv head's group, TOK = 128/G, token-major; 256
//     rows when the KV ranges are long) over a range of 64-key KV tiles - the whole
//     range, or a chunk of it when the batch alone would not fill the GPU (decode
//     steps, short ranges over long contexts), or the prefix that neighbouring
//     sequences with short new ranges share (Sec. 3.4; fork_sequence, Sec. 3.5).
//     Items are ordered longest first; each record holds what the kernel needs to
//     start its first copies.
//   * attn_kernel: one workgroup (4 wavefronts of 64) per (item, kv head), so every
//     K/V byte staged in LDS serves the whole GQA group.  Items that cover a whole
//     range write out/lse; the others write partial rows that merge_kernel weighs
//     together by their log-sum-exp.
// Kernel shape
//   * the KV loop walks 64-key tiles (4 pages) through the page table; each page
//     contributes one contiguous 4 KiB run of K and one of V for this kv head.
//   * S^T = K Q^T on v_mfma_f32_32x32x16 (A = K rows from LDS, B = Q held in
//     registers): a lane then owns ONE query row (column l%32) and 16 keys per
//     32-key chunk, so the softmax row max / row sum are in-lane plus one
//     exchange with lane l^32, and the rescale factor is a per-lane scalar.  With
//     bf16 the row's reference score is fixed after the first half tile (no row max
//     or rescale per tile; a pass whose sums left the safe range is repeated with
//     the moving reference).
//   * O^T += V^T P^T: P^T is the B operand straight from the S^T accumulators
//     (no LDS round trip); V^T comes from LDS with ds_read_b64_tr_b16, which
//     transposes 4 keys x 16 d per 16-lane group on the way in.
//   * LDS tiles are XOR-swizzled so both the row reads (K) and the transposing
//     reads (V) spread over all banks.
#include <math.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "mc_common.h"

namespace {

using mc::kHeadPageBytes;
using mc::kPage;
using mc::kRowBytes;

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBM = 128;       // rows (token x head-in-group) per workgroup
constexpr int kBN = 64;        // keys per KV tile
constexpr int kThreads = 256;  // 4 wavefronts, 32 rows each
constexpr int kPlanThreads = 1024;      // threads of the planner's one workgroup ...
constexpr int kPlanThreadsSmall = 256;  // ... and for batches of few sequences and q tiles
constexpr int kBuckets = 4096;
constexpr int32_t kPlanMagic = 0x6d63706c;

struct PlanHeader {
  int32_t magic;
  int32_t err;        // mc_status found on the device by the plan kernel
  int32_t num_items;  // work items (q tile x KV chunk) in the work list
  int32_t tile_tokens;
  int32_t batch;
  int32_t total_q;
  int32_t num_merges; // q tiles whose KV range was cut into several chunks
  int32_t chunk_tiles;  // chunk length the planner settled on (KV tiles); 0 = nothing was cut
  int32_t num_groups_rows;  // partial rows written by shared-prefix items (0 = no groups)
  int32_t tail_chunks;  // chunks per q tile of the remainder round (0 = not applied)
  int32_t merge_tokens; // new tokens of all q tiles with partial results (what merge_kernel walks)
  int32_t pad[5];
};
static_assert(sizeof(PlanHeader) == 64, "header is 64 bytes");

// One work item: q tile (seq, row0) over the KV tiles [t0, t1) of its sequence.  t0 is even.
// part < 0: the item covers the tile's whole KV range and writes out/lse itself.  Otherwise it
// writes a partial result (O normalised within the chunk, fp32, and the chunk's LSE) for token
// tt of the tile at row part + tt of the partial arrays, and merge_kernel combines the chunks.
// gsize > 0: a shared-prefix item.  Its rows are the gsize new tokens of consecutive sequences
// starting at seq (neighbours in the q array: tokens cu_q[seq] .. cu_q[seq] + gsize - 1), whose
// page tables begin with the same pages; it covers tiles of that common prefix (all of it
// visible to every row) and always writes partial rows.
// The record also carries what the kernel needs to start its first copies without further
// look-ups (each would be one more dependent memory round trip before the first tile): the
// tile's first token in the q array and its token count, where the sequence's page table starts,
// the last table entry the plan has validated for the sequence, and the page ids of table
// entries 4 t0 .. 4 t0 + 5 (clamped to that last entry).
struct ItemRec {
  int32_t seq, row0, t0, t1, part, gsize;
  int32_t q_first, ntok, table_off, pidx_cap;
  int32_t ids[6];
};
static_assert(sizeof(ItemRec) == 64, "item record is 64 bytes");

// One q tile with partial results: chunk c of its own KV range has its partial rows at
// part + c * ntok; if the tile's sequence belongs to a shared-prefix group, chunk c of the
// prefix has this sequence's rows from g_part + c * g_stride on (g_stride = the group's tokens).
struct MergeRec {
  int32_t q_row;   // index of the tile's first token among all new tokens of the batch
  int32_t ntok, nsplit, part;
  int32_t g_nsplit, g_part, g_stride;
  int32_t tok_off; // tokens of the merge records before this one
};
static_assert(sizeof(MergeRec) == 32, "merge record is 32 bytes");

constexpr int kCuTilesInLds = 1024;
constexpr int kValidateInPlan = 256;  // batches up to this have their page ids checked by plan_kernel
constexpr int kTailTilesMax = 2048;   // q tiles up to which the remainder round is looked at
constexpr int kMinSharedTiles = 8;    // a shared prefix shorter than 512 tokens is not worth a group
constexpr int kMinChunkTiles = 8;     // never cut a KV range into pieces shorter than 512 keys
constexpr int kRoundsWanted = 4;      // cut only while the launch has fewer items than 4 per slot
// ... and then aim for about one item per slot: measured best on decode batches and on 500-token
// ranges over long contexts (more chunks mean more partial rows to write and merge)
constexpr int kItemsPerSlot = 1;

struct WorkspaceLayout {
  size_t cu_tiles, items, merges, part_lse, part_o, total;
  int32_t max_tiles, max_items, part_cap, batch;
};

inline size_t round64(size_t x) { return (x + 63) & ~size_t(63); }

// The attention kernel comes with q tiles of 128 rows (two workgroups per compute unit) and of
// 256 rows (one, with every K/V fragment read from LDS feeding two MFMAs), the wide ones paying
// off on long KV ranges only.  The planner chooses (it sees the lengths, the host does not) and
// says so in the plan's header; the host only rules the wide tiles out where the batch cannot
// want them - fewer than 4096 new tokens per sequence on average, or fewer wide tiles than four
// per compute unit of a 256-unit GPU - and otherwise launches both kernels, of which the one
// the plan was not made for returns at once.  The workspace is laid out for the narrow tiles
// (more of them), which holds either plan.
inline bool wide_tiles_allowed(int32_t batch, int32_t total_q, int G, int num_kv_heads) {
#ifdef MC_WIDE_TILES
  return MC_WIDE_TILES;
#endif
  const int64_t wide_tiles = ((int64_t)total_q * G + 2 * kBM - 1) / (2 * kBM);
  return batch > 0 && total_q / batch >= 4096 && wide_tiles * num_kv_heads >= 1024;
}
constexpr int kWideMinKeys = 8192;   // mean keys per new token from which the planner goes wide

constexpr int kMaxSlots = 1024;   // 512 compute units: beyond any GPU this library is written for
constexpr size_t kPartialBytesCap = size_t(128) << 20;

// Token rows the partial arrays can hold: the planner cuts KV ranges only as far as this
// allows.  None when the batch has so many q tiles that no GPU would need a cut; otherwise two
// chunks for every new token plus room for the many chunks of a few decode rows, within 128 MiB.
inline int32_t partial_capacity(int32_t total_q, int32_t tile_tokens, int32_t num_q_heads,
                                int32_t num_kv_heads) {
  const int64_t tiles = ((int64_t)total_q + tile_tokens - 1) / tile_tokens;
  if (tiles * num_kv_heads >= (int64_t)kRoundsWanted * kMaxSlots) return 0;
  const int64_t want = 2ll * total_q + 4096;
  const int64_t fit = (int64_t)(kPartialBytesCap / (sizeof(float) * num_q_heads * (mc::kHeadDim + 1)));
  return (int32_t)(want < fit ? want : fit);
}

// part_limit >= 0 caps the rows of the partial arrays below what partial_capacity asks for (a
// caller with a fixed amount of memory): the planner then cuts KV ranges less, or not at all.
inline WorkspaceLayout workspace_layout(int32_t batch, int32_t total_q, int32_t tile_tokens,
                                        int32_t num_q_heads, int32_t num_kv_heads,
                                        int32_t part_limit = -1) {
  WorkspaceLayout w;
  w.max_tiles = (int32_t)(((int64_t)total_q + tile_tokens - 1) / tile_tokens + batch);
  w.part_cap = partial_capacity(total_q, tile_tokens, num_q_heads, num_kv_heads);
  if (part_limit >= 0 && part_limit < w.part_cap) w.part_cap = part_limit;
  w.batch = batch;
  // every extra chunk holds at least one partial row; a shared-prefix group adds items too
  w.max_items = w.max_tiles + w.part_cap + batch;
  w.cu_tiles = sizeof(PlanHeader);
  w.items = w.cu_tiles + round64(sizeof(int32_t) * ((size_t)batch + 1));
  w.merges = w.items + sizeof(ItemRec) * (size_t)w.max_items;
  w.part_lse = w.merges + round64(sizeof(MergeRec) * (size_t)w.max_tiles);
  w.part_o = w.part_lse + round64(sizeof(float) * (size_t)w.part_cap * num_q_heads);
  w.total = w.part_o + sizeof(float) * (size_t)w.part_cap * num_q_heads * mc::kHeadDim;
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
  ItemRec* items;
  MergeRec* merges;
  int32_t batch, total_q, tile_tokens, num_pages, max_tiles, max_items, part_cap;
  int32_t hkv, slots;   // kv heads; workgroups the GPU runs at a time
  int32_t allow_groups; // look for decode rows of neighbouring sequences that share a prefix
  int32_t ahead;        // tokens every sequence's begin may still grow by while the plan is in use
  int32_t wide_tile_tokens, slots_wide;   // the wide q tiles, if the host allows them (else 0)
};

// Block-wide exclusive scan of one value per thread (NT threads): a shuffle scan
// inside each wavefront, the 16 wavefront totals through LDS, two barriers in all.
template <int NT>
__device__ int block_exclusive_scan(int v, int* lds, int* total) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  __syncthreads();               // earlier readers of lds are done
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int x = lds[w];
    if (w < wave) before += x;
    all += x;
  }
  *total = all;
  return before + incl - v;
}

// The same for N values per thread at once (two barriers for all of them); lds holds N x 16 ints.
template <int NT, int N>
__device__ void block_exclusive_scan_n(int (&v)[N], int* lds, int (&total)[N]) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int incl[N];
#pragma unroll
  for (int k = 0; k < N; ++k) incl[k] = v[k];
#pragma unroll
  for (int off = 1; off < 64; off <<= 1)
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int up = __shfl_up(incl[k], off);
      if (lane >= off) incl[k] += up;
    }
  __syncthreads();               // earlier readers of lds are done
  if (lane == 63)
#pragma unroll
    for (int k = 0; k < N; ++k) lds[k * (NT / 64) + wave] = incl[k];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < N; ++k) {
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
      const int x = lds[k * (NT / 64) + w];
      if (w < wave) before += x;
      all += x;
    }
    total[k] = all;
    v[k] = before + incl[k] - v[k];
  }
}

// Block-wide sum of one value per thread, to every thread: butterfly inside each wavefront, the
// 16 wavefront sums through LDS (lds holds 2 x 16 ints).
template <int NT>
__device__ long long block_sum(long long v, int* lds) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();               // earlier readers of lds are done
  if (lane == 0) {
    lds[2 * wave] = (int)(v & 0xffffffffll);
    lds[2 * wave + 1] = (int)(v >> 32);
  }
  __syncthreads();
  long long all = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w)
    all += ((long long)lds[2 * w + 1] << 32) | (unsigned int)lds[2 * w];
  return all;
}

// Block-wide inclusive running maximum of one value per thread.
template <int NT>
__device__ int block_inclusive_max_scan(int v, int* lds) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if (lane >= off) incl = max(incl, up);
  }
  __syncthreads();
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  int before = INT32_MIN;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w)
    if (w < wave) before = max(before, lds[w]);
  return max(before, incl);
}

// Page ids of every needed table entry, for batches too large for the planner's one workgroup
// to walk: one wavefront per sequence, many workgroups.  Runs after plan_kernel and, on a bad
// id, turns its verdict into MC_ERR_RANGE with an empty work list.  (Sequences whose offsets
// are malformed were rejected by the planner already; they are skipped here.)
__global__ __launch_bounds__(256) void validate_pages_kernel(PlanArgs a) {
  const int s = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (s >= a.batch || a.hdr->err != MC_OK) return;
  const int q = a.cu_q[s + 1] - a.cu_q[s], b = a.begin[s];
  const int p0 = a.cu_pages[s], np = a.cu_pages[s + 1] - p0;
  if (q <= 0 || b < 0 || p0 < 0) return;
  const int64_t need64 = ((int64_t)b + q + a.ahead + kPage - 1) / kPage;
  if (need64 > np) return;
  const int need = (int)need64;
  int err = 0;
  for (int i = lane; i < need; i += 64 * 8) {   // eight independent loads per lane and trip
    int32_t pg[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) pg[u] = i + 64 * u < need ? a.page_table[p0 + i + 64 * u] : 0;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (pg[u] < 0 || pg[u] >= a.num_pages) err = 1;
  }
  if (__ballot(err) != 0 && lane == 0) {
    a.hdr->num_items = 0;
    a.hdr->num_merges = 0;
    a.hdr->merge_tokens = 0;
    a.hdr->err = MC_ERR_RANGE;
  }
}

// One workgroup.  Validates the ragged-batch arrays, cuts every sequence's new range into q
// tiles of tile_tokens tokens, cuts long KV ranges into chunks when the launch would otherwise
// have too few work items to fill the GPU (decode rows, short batches over long contexts),
// and orders the items by decreasing number of KV tiles (longest first), so that the tail of
// the launch is made of short items.
// NT threads: 1024, or 256 for small batches, whose many block-wide steps then cost a quarter
// of the wavefronts to synchronise.
template <int NT>
__global__ __launch_bounds__(NT) void plan_kernel(PlanArgs a) {
  __shared__ int scan[5 * NT / 64];   // wavefront totals of the block scans and sums
  __shared__ int hist[kBuckets];
  __shared__ int s_err, s_maxcost;
  // per-sequence arrays of batches that fit: the searches and tile look-ups below stay in LDS
  __shared__ int s_cu[kCuTilesInLds + 1], s_cuq[kCuTilesInLds + 1], s_beg[kCuTilesInLds],
      s_cup[kCuTilesInLds + 1];
  // shared-prefix groups, per sequence: pages in common with the next sequence; prefix tiles the
  // group covers (0 = not in a group); the group's first sequence (-1 = none); at that first
  // sequence the group's new tokens, the base of its partial rows and its last sequence
  __shared__ int s_common[kCuTilesInLds], s_gp[kCuTilesInLds], s_glead[kCuTilesInLds],
      s_gsize[kCuTilesInLds], s_gbase[kCuTilesInLds], s_glast[kCuTilesInLds];
  __shared__ int s_groups;
  // remainder round: flags of the q tiles that are cut, the cost bucket at the boundary and how
  // many tiles of it are taken
  __shared__ uint8_t s_tailflag[kTailTilesMax];
  __shared__ int s_tail_bucket, s_tail_take, s_tail_taken;
  const int t = threadIdx.x;
  if (t == 0) { s_err = 0; s_maxcost = 1; }
  for (int i = t; i < kBuckets; i += NT) hist[i] = 0;
  const bool cu_in_lds = a.batch <= kCuTilesInLds;
  if (cu_in_lds) {
    for (int i = t; i <= a.batch; i += NT) {
      s_cuq[i] = a.cu_q[i];
      s_cup[i] = a.cu_pages[i];
      if (i < a.batch) s_beg[i] = a.begin[i];
    }
  }
  __syncthreads();

  // the batch's offset arrays: from LDS when they fit there (one read of global memory in all)
  auto cuq = [&](int i) { return cu_in_lds ? s_cuq[i] : a.cu_q[i]; };
  auto cup = [&](int i) { return cu_in_lds ? s_cup[i] : a.cu_pages[i]; };
  auto beg = [&](int i) { return cu_in_lds ? s_beg[i] : a.begin[i]; };
  const int per = (a.batch + NT - 1) / NT;
  const int s_lo = min(t * per, a.batch), s_hi = min(s_lo + per, a.batch);
  // 0. q tile width: wide tiles when a new token sees kWideMinKeys keys on average
  if (a.wide_tile_tokens > 0) {
    long long keys = 0, rows = 0;
    for (int s = s_lo; s < s_hi; ++s) {
      const long long q = cuq(s + 1) - cuq(s), b = beg(s);
      if (q > 0 && b >= 0) { rows += q; keys += q * b + q * (q + 1) / 2; }
    }
    keys = block_sum<NT>(keys, scan);
    rows = block_sum<NT>(rows, scan);
    if (rows > 0 && keys / rows >= kWideMinKeys) {
      a.tile_tokens = a.wide_tile_tokens;
      a.slots = a.slots_wide;
    }
  }
  // 1. validate, count tiles per sequence (contiguous chunk of sequences per thread)
  int my_tiles = 0, err = 0, maxcost = 1;
  if (t == 0 && (cuq(0) != 0 || cuq(a.batch) != a.total_q || cup(0) < 0)) err = 1;
  for (int s = s_lo; s < s_hi; ++s) {
    const int q = cuq(s + 1) - cuq(s), b = beg(s);
    const int np = cup(s + 1) - cup(s);
    if (q < 0 || b < 0 || np < 0 || cuq(s) < 0 || cuq(s + 1) > a.total_q) { err = 1; continue; }
    if (q == 0) continue;
    const int64_t end = (int64_t)b + q + a.ahead;
    if ((end + kPage - 1) / kPage > np) { err = 1; continue; }
    my_tiles += (q + a.tile_tokens - 1) / a.tile_tokens;
    maxcost = max(maxcost, (int)((end + kBN - 1) / kBN));
  }
  // (one LDS atomic per wavefront, not per thread: 1024 atomics on one address take microseconds)
  if (__ballot(err != 0) != 0 && (t & 63) == 0) atomicOr(&s_err, 1);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) maxcost = max(maxcost, __shfl_xor(maxcost, off));
  if ((t & 63) == 0) atomicMax(&s_maxcost, maxcost);
  __syncthreads();
  if (s_err) {
    if (t == 0) { a.hdr->err = MC_ERR_RANGE; a.hdr->num_items = 0; a.hdr->num_merges = 0; a.hdr->merge_tokens = 0; a.hdr->magic = kPlanMagic; }
    return;
  }
  // 2. page ids of every needed table entry.  Small batches (their offsets sit in LDS): a
  //    wavefront takes four sequences per trip and has up to 32 loads per lane in flight (the loop is
  //    bound by memory latency); entries beyond the first 512 of a sequence follow one
  //    sequence at a time.
  if (a.batch <= kValidateInPlan) {
    for (int s4 = (t >> 6) * 4; s4 < a.batch; s4 += (NT >> 6) * 4) {
      int32_t pg[4][8];
      int need[4], p0[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int s = s4 + k;
        const int q = s < a.batch ? s_cuq[s + 1] - s_cuq[s] : 0;
        need[k] = q > 0 ? (s_beg[s] + q + a.ahead + kPage - 1) / kPage : 0;
        p0[k] = s < a.batch ? s_cup[s] : 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = (t & 63) + 64 * u;
          pg[k][u] = i < need[k] ? a.page_table[p0[k] + i] : 0;
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (pg[k][u] < 0 || pg[k][u] >= a.num_pages) err = 1;
        for (int i = 512 + (t & 63); i < need[k]; i += 64) {
          const int32_t x = a.page_table[p0[k] + i];
          if (x < 0 || x >= a.num_pages) err = 1;
        }
      }
    }
  }
  // (batches beyond that: validate_pages_kernel, launched after this kernel, on many workgroups)
  if (__ballot(err != 0) != 0 && (t & 63) == 0) atomicOr(&s_err, 1);
  // 3. exclusive scan of tiles per sequence
  int total_tiles;
  int base = block_exclusive_scan<NT>(my_tiles, scan, &total_tiles);
  for (int s = s_lo; s < s_hi; ++s) {
    a.cu_tiles[s] = base;
    if (cu_in_lds) s_cu[s] = base;
    const int q = cuq(s + 1) - cuq(s);
    base += (q + a.tile_tokens - 1) / a.tile_tokens;
  }
  if (t == 0) {
    a.cu_tiles[a.batch] = total_tiles;
    if (cu_in_lds) s_cu[a.batch] = total_tiles;
  }
  __threadfence_block();
  __syncthreads();
  if (s_err || total_tiles > a.max_tiles) {
    if (t == 0) { a.hdr->err = MC_ERR_RANGE; a.hdr->num_items = 0; a.hdr->num_merges = 0; a.hdr->merge_tokens = 0; a.hdr->magic = kPlanMagic; }
    return;
  }

  // 3b. shared-prefix groups (Sec. 3.4, fork_sequence in Sec. 3.5: sequences may share the pages of a common
  //     prefix).  The new tokens of neighbouring sequences with short new ranges (decode rows,
  //     or a few tokens each) whose tables start with the same pages attend that prefix together
  //     as one q tile - their tokens are neighbours in the q array, and every key of the prefix
  //     lies before every one of them, so no mask is involved - one K/V read for all of them,
  //     and their own remainders one by one; the parts are merged by LSE like any other chunks.
  const bool try_groups = a.allow_groups && cu_in_lds && a.batch >= 2 && a.batch <= NT;
  if (t == 0) s_groups = 0;
  if (try_groups) {
    for (int i = t; i < a.batch; i += NT) { s_common[i] = 0; s_gp[i] = 0; s_glead[i] = -1; s_gsize[i] = 0; }
    __syncthreads();
    // pages in common between s and s+1, among the whole pages cached by both.  First every
    // pair at once, one thread each: unrelated sequences differ in their first page and are
    // done (s_common = 1 marks a pair that is not).  Then one wavefront a remaining pair.
    constexpr int kMinPages = kMinSharedTiles * kBN / kPage;
    // a sequence can be a member if its new range leaves room for another token in a q tile
    auto is_short = [&](int sq) {
      const int q = s_cuq[sq + 1] - s_cuq[sq];
      return q >= 1 && q < a.tile_tokens;
    };
    if (t + 1 < a.batch && is_short(t) && is_short(t + 1) &&
        min(s_beg[t], s_beg[t + 1]) / kPage >= kMinPages &&
        a.page_table[s_cup[t]] == a.page_table[s_cup[t + 1]])
      s_common[t] = 1;
    __syncthreads();
    for (int sq = t >> 6; sq + 1 < a.batch; sq += NT >> 6) {
      if (s_common[sq] == 0) continue;
      const int lim = min(s_beg[sq], s_beg[sq + 1]) / kPage;
      const int pa = s_cup[sq], pb = s_cup[sq + 1];
      int common = 0;
      for (int i0 = 0; i0 < lim; i0 += 64) {
        const int i = i0 + (t & 63);
        const bool differ = i < lim && a.page_table[pa + i] != a.page_table[pb + i];
        const unsigned long long m = __ballot(differ);
        if (m) { common = i0 + __ffsll((long long)m) - 1; break; }
        common = min(lim, i0 + 64);
      }
      if ((t & 63) == 0) s_common[sq] = common;
    }
    __syncthreads();
    // Runs of such sequences linked by enough common pages, cut greedily into groups of at most
    // tile_tokens new tokens.  The thread of a run's first sequence walks the run group by
    // group (cu_q is the prefix sum of the new tokens: the end of a group is a binary search);
    // everything per member is done by the member's own thread.
    const bool mine = t < a.batch;
    auto linked = [&](int sq) {   // sq and sq+1 sit in one run
      return sq >= 0 && sq + 1 < a.batch && is_short(sq) && is_short(sq + 1) &&
             s_common[sq] >= kMinPages;
    };
    const bool in_run = mine && is_short(t) && (linked(t) || linked(t - 1));
    // (unrelated sequences, the usual case: nothing is linked and the rest is skipped)
    if (__ballot(in_run) != 0 && (t & 63) == 0) s_groups = -1;
    __syncthreads();
    const bool any_run = s_groups != 0;
    __syncthreads();
    if (t == 0) s_groups = 0;
    if (any_run) {
      // last sequence of the run a sequence sits in: the nearest j >= t that is not linked to j + 1
      // (a running maximum over the reversed index)
      {
        const int j = a.batch - 1 - t;     // this thread's element of the reversed scan
        const bool ends = j >= 0 && !linked(j);
        const int v = block_inclusive_max_scan<NT>(ends ? -j : INT32_MIN, scan);
        if (j >= 0) s_gbase[j] = -v;       // scratch until step 5: run end of sequence j
      }
      __syncthreads();
      if (in_run && !linked(t - 1)) {      // first sequence of a run
        const int run_end = s_gbase[t];
        for (int lead = t; lead <= run_end;) {
          // the last member: the largest e <= run_end with cu_q[e + 1] - cu_q[lead] <= tile_tokens
          int lo = lead, hi = run_end;
          const int limit = s_cuq[lead] + a.tile_tokens;
          while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_cuq[mid + 1] <= limit) lo = mid; else hi = mid - 1;
          }
          if (lo > lead) {                 // two members or more: a group
            s_gsize[lead] = s_cuq[lo + 1] - s_cuq[lead];   // rows of the group's q tile
            s_glast[lead] = lo;
            s_gbase[lead] = INT32_MAX;     // becomes the fewest pages two neighbouring members share
            s_groups = 1;
          }
          lead = lo + 1;
        }
      }
      __syncthreads();
      // every sequence finds the nearest group lead at or before it and checks that it is a member
      const int near = block_inclusive_max_scan<NT>(mine && s_gsize[t] > 0 ? t : -1, scan);
      const bool member = in_run && near >= 0 && t <= s_glast[near];
      if (member && t < s_glast[near]) atomicMin(&s_gbase[near], s_common[t]);
      __syncthreads();
      if (member && t == near)
        s_gbase[t] = (s_gbase[t] / (2 * kBN / kPage)) * 2;   // prefix tiles, even (scratch until step 5)
      __syncthreads();
      if (mine) {
        s_glead[t] = member ? near : -1;
        s_gp[t] = member ? s_gbase[near] : 0;
      }
    }
    __syncthreads();
  }
  bool groups = try_groups && s_groups != 0;

  // q tile i: its sequence, first row, token count, KV tiles, the last even tile index at which
  // a chunk may start (every row must see at least the first key of every chunk), the prefix
  // tiles its shared-prefix group covers, and the group's new tokens if this tile leads one
  struct Tile { int s, row0, ntok, T, dmax, pt, gm; };
  auto locate = [&](int i) {
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if ((cu_in_lds ? s_cu[mid] : a.cu_tiles[mid]) <= i) lo = mid; else hi = mid;
    }
    Tile x;
    x.s = lo;
    x.row0 = (i - (cu_in_lds ? s_cu[lo] : a.cu_tiles[lo])) * a.tile_tokens;
    const int q = cu_in_lds ? s_cuq[lo + 1] - s_cuq[lo] : a.cu_q[lo + 1] - a.cu_q[lo];
    const int b = cu_in_lds ? s_beg[lo] : a.begin[lo];
    x.ntok = min(a.tile_tokens, q - x.row0);
    x.T = (b + x.row0 + x.ntok + a.ahead + kBN - 1) / kBN;   // room for the range to move up
    x.dmax = ((b + x.row0) / kBN) & ~1;
    x.pt = groups ? s_gp[lo] : 0;
    x.gm = groups && s_glead[lo] == lo ? s_gsize[lo] : 0;
    return x;
  };
  // own chunks of L tiles (L even) from the end of the group's prefix: [pt, pt+L), ...,
  // [pt+kL, T) with pt + kL <= dmax; the group's prefix itself in chunks of L
  auto own_splits = [&](const Tile& x, int L) { return L > 0 ? (x.dmax - x.pt) / L + 1 : 1; };
  auto grp_splits = [&](const Tile& x, int L) { return x.pt > 0 ? (L > 0 ? (x.pt + L - 1) / L : 1) : 0; };
  auto part_rows = [&](const Tile& x, int L) {
    const int ns = own_splits(x, L);
    return (ns > 1 || x.pt > 0 ? ns * x.ntok : 0) + (x.gm ? grp_splits(x, L) * x.gm : 0);
  };
  auto total_part_rows = [&](int L) {   // block-wide
    long long rows = 0;
    for (int i = t; i < total_tiles; i += NT) rows += part_rows(locate(i), L);
    return block_sum<NT>(rows, scan);
  };

  // 4. chunk length.  No cutting when the q tiles alone give the GPU kRoundsWanted rounds of
  //    work; otherwise a length that would make about kItemsPerSlot items per slot, never
  //    below kMinChunkTiles, doubled until the partial rows fit the workspace.
  int L = 0;
  if ((int64_t)total_tiles * a.hkv < (int64_t)kRoundsWanted * a.slots) {
    long long cost = 0;
    for (int i = t; i < total_tiles; i += NT) {
      const Tile x = locate(i);
      cost += x.T - x.pt + (x.gm ? x.pt : 0);
    }
    cost = block_sum<NT>(cost, scan);
    const long long want =
        (cost * a.hkv + (long long)kItemsPerSlot * a.slots - 1) / ((long long)kItemsPerSlot * a.slots);
    L = want < kMinChunkTiles ? kMinChunkTiles : want > (1 << 28) ? (1 << 28) : (int)want;
    L = (L + 1) & ~1;
    for (;;) {
      if (L >= s_maxcost) { L = 0; break; }   // nothing is long enough to be cut
      if (total_part_rows(L) <= a.part_cap) break;
      L *= 2;
    }
  }
  // without cuts the groups still need partial rows: no room, no groups
  if (L == 0 && groups && total_part_rows(0) > a.part_cap) groups = false;

  int shift = 0;
  while ((s_maxcost >> shift) >= kBuckets) ++shift;
  auto bucket = [&](int len) { return kBuckets - 1 - (len >> shift); };

  // 4b. remainder round.  Between one and kRoundsWanted rounds of uncut, similar items the last
  //     round is the problem: n items on S slots take ceil(n / S) rounds although the last one
  //     may hold few items.  The n mod S shortest items (they run last) are then cut into
  //     c = ceil(S / (n mod S)) chunks each, which fill that round with items 1/c as long.
  int tail_c = 0;
  {
    const int64_t n = (int64_t)total_tiles * a.hkv;
    const int rem = (int)(n % a.slots);
    const int rem_tiles = rem / a.hkv;
    const int c = rem > 0 ? min(8, (a.slots + rem - 1) / rem) : 0;
    if (L == 0 && !groups && total_tiles <= kTailTilesMax && n >= a.slots &&
        n < (int64_t)kRoundsWanted * a.slots && rem_tiles >= 1 && 10 * rem <= 7 * a.slots && c >= 2 &&
        (int64_t)rem_tiles * a.tile_tokens * c <= a.part_cap) {
      if (t == 0) { s_tail_bucket = kBuckets; s_tail_take = 0; s_tail_taken = 0; }
      for (int i = t; i < total_tiles; i += NT) atomicAdd(&hist[bucket(locate(i).T)], 1);
      __syncthreads();
      // shortest first: walk the buckets from the last to the first until rem_tiles tiles are in
      constexpr int kPer = kBuckets / NT;
      int local[kPer], sum = 0;
      for (int i = 0; i < kPer; ++i) { local[i] = hist[kBuckets - 1 - (t * kPer + i)]; sum += local[i]; }
      int tot, before = block_exclusive_scan<NT>(sum, scan, &tot);
      for (int i = 0; i < kPer; ++i) {
        if (before < rem_tiles && before + local[i] >= rem_tiles) {
          s_tail_bucket = kBuckets - 1 - (t * kPer + i);
          s_tail_take = rem_tiles - before;
        }
        before += local[i];
      }
      __syncthreads();
      for (int i = t; i < total_tiles; i += NT) {
        const int bk = bucket(locate(i).T);
        s_tailflag[i] = bk > s_tail_bucket ||
                        (bk == s_tail_bucket && atomicAdd(&s_tail_taken, 1) < s_tail_take);
      }
      for (int i = t; i < kBuckets; i += NT) hist[i] = 0;
      __syncthreads();
      tail_c = c;
    }
  }
  // chunk length of q tile i: the batch's, or its own if it is cut for the remainder round
  auto chunk_len = [&](int i, const Tile& x) {
    if (tail_c == 0 || !s_tailflag[i]) return L;
    const int len = ((x.T + tail_c - 1) / tail_c + 1) & ~1;
    return max(len, kMinChunkTiles);
  };

  // 5. items and merge records: count per contiguous range of tiles, scan, histogram of costs
  const int tper = (total_tiles + NT - 1) / NT;
  const int i_lo = min(t * tper, total_tiles), i_hi = min(i_lo + tper, total_tiles);
  int n_items = 0, n_own = 0, n_grp = 0, n_merge = 0, n_mtok = 0;
  for (int i = i_lo; i < i_hi; ++i) {
    const Tile x = locate(i);
    const int Li = chunk_len(i, x);
    const int ns = own_splits(x, Li), ng = x.gm ? grp_splits(x, Li) : 0;
    n_items += ns + ng;
    if (ns > 1 || x.pt > 0) { n_own += ns * x.ntok; ++n_merge; n_mtok += x.ntok; }
    n_grp += ng * x.gm;
    for (int c = 0; c < ns; ++c)
      atomicAdd(&hist[bucket(c + 1 < ns ? Li : x.T - x.pt - c * Li)], 1);
    for (int c = 0; c < ng; ++c)
      atomicAdd(&hist[bucket(Li > 0 ? min(Li, x.pt - c * Li) : x.pt)], 1);
  }
  int offs[5] = {n_items, n_own, n_grp, n_merge, n_mtok}, tots[5];
  block_exclusive_scan_n<NT>(offs, scan, tots);
  const int tot_items = tots[0], tot_own = tots[1], tot_grp = tots[2], tot_merge = tots[3],
            tot_mtok = tots[4];
  int own_off = offs[1], grp_off = offs[2], merge_off = offs[3], mtok_off = offs[4];
  {
    constexpr int kPer = kBuckets / NT;
    int local[kPer], sum = 0;
    for (int i = 0; i < kPer; ++i) { local[i] = hist[t * kPer + i]; sum += local[i]; }
    int tot, off = block_exclusive_scan<NT>(sum, scan, &tot);
    for (int i = 0; i < kPer; ++i) { hist[t * kPer + i] = off; off += local[i]; }
  }
  __syncthreads();
  if (tot_items > a.max_items || tot_own + tot_grp > a.part_cap || tot_merge > a.max_tiles) {   // cannot happen
    if (t == 0) { a.hdr->err = MC_ERR_RANGE; a.hdr->num_items = 0; a.hdr->num_merges = 0; a.hdr->merge_tokens = 0; a.hdr->magic = kPlanMagic; }
    return;
  }
  // where each group's partial rows start (after all the tiles' own): its members need it
  if (groups) {
    int off = tot_own + grp_off;
    for (int i = i_lo; i < i_hi; ++i) {
      const Tile x = locate(i);
      if (x.gm) { s_gbase[x.s] = off; off += grp_splits(x, chunk_len(i, x)) * x.gm; }
    }
    __syncthreads();
  }
  // 6. emit: counting sort of the items by cost (number of KV tiles), heaviest first
  for (int i = i_lo; i < i_hi; ++i) {
    const Tile x = locate(i);
    const int Li = chunk_len(i, x);
    const int ns = own_splits(x, Li), ng = grp_splits(x, Li);
    const bool merged = ns > 1 || x.pt > 0;
    if (merged) {
      MergeRec m;
      m.q_row = (cu_in_lds ? s_cuq[x.s] : a.cu_q[x.s]) + x.row0;
      m.ntok = x.ntok;
      m.nsplit = ns;
      m.part = own_off;
      m.g_nsplit = ng;
      m.g_part = x.pt > 0 ? s_gbase[s_glead[x.s]] + (s_cuq[x.s] - s_cuq[s_glead[x.s]]) : 0;
      m.g_stride = x.pt > 0 ? s_gsize[s_glead[x.s]] : 0;
      m.tok_off = mtok_off;
      mtok_off += x.ntok;
      a.merges[merge_off++] = m;
    }
    // what every item of this tile's sequence shares
    const int sq0 = cu_in_lds ? s_cuq[x.s] : a.cu_q[x.s];
    const int sq_len = (cu_in_lds ? s_cuq[x.s + 1] : a.cu_q[x.s + 1]) - sq0;
    const int sb = cu_in_lds ? s_beg[x.s] : a.begin[x.s];
    const int tab = cu_in_lds ? s_cup[x.s] : a.cu_pages[x.s];
    const int cap = (int)(((int64_t)sb + sq_len + a.ahead + kPage - 1) / kPage) - 1;   // validated above
    auto finish = [&](ItemRec& it, int q_first, int ntok) {
      it.q_first = q_first;
      it.ntok = ntok;
      it.table_off = tab;
      it.pidx_cap = cap;
#pragma unroll
      for (int k = 0; k < 6; ++k) it.ids[k] = a.page_table[tab + min(4 * it.t0 + k, cap)];
      a.items[atomicAdd(&hist[bucket(it.t1 - it.t0)], 1)] = it;
    };
    for (int c = 0; c < ns; ++c) {
      ItemRec it;
      it.seq = x.s;
      it.row0 = x.row0;
      it.t0 = x.pt + c * Li;
      it.t1 = (c + 1 < ns ? x.pt + (c + 1) * Li : x.T);
      it.part = merged ? own_off + c * x.ntok : -1;
      it.gsize = 0;
      finish(it, sq0 + x.row0, x.ntok);
    }
    for (int c = 0; x.gm && c < ng; ++c) {
      ItemRec it;
      it.seq = x.s;
      it.row0 = 0;
      it.t0 = c * Li;
      it.t1 = Li > 0 ? min((c + 1) * Li, x.pt) : x.pt;
      it.part = s_gbase[x.s] + c * x.gm;
      it.gsize = x.gm;
      finish(it, sq0, x.gm);
    }
    if (merged) own_off += ns * x.ntok;
  }
  if (t == 0) {
    a.hdr->err = MC_OK;
    a.hdr->num_items = tot_items;
    a.hdr->num_merges = tot_merge;
    a.hdr->merge_tokens = tot_mtok;
    a.hdr->chunk_tiles = L;
    a.hdr->tile_tokens = a.tile_tokens;
    a.hdr->batch = a.batch;
    a.hdr->total_q = a.total_q;
    a.hdr->num_groups_rows = tot_grp;
    a.hdr->tail_chunks = tail_c;
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
  // the same instruction with its result pinned to vector registers (see attn_kernel: with
  // two row blocks the allocator would otherwise park the scores in accumulation registers,
  // which the softmax's vector instructions cannot read)
  static __device__ __forceinline__ void run_v0(vec8 a, vec8 b, f32x16& c) {
    asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, 0" : "=v"(c) : "v"(a), "v"(b));
  }
  static __device__ __forceinline__ void run_v(vec8 a, vec8 b, f32x16& c) {
    asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
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
  static __device__ __forceinline__ void run_v0(vec8 a, vec8 b, f32x16& c) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(c) : "v"(a), "v"(b));
  }
  static __device__ __forceinline__ void run_v(vec8 a, vec8 b, f32x16& c) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
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
  const ItemRec* items;
  float* part_lse;         // [partial row][hq]
  float* part_o;           // [partial row][hq][128]
  int64_t page_stride;     // bytes
  int32_t num_pages, hkv, hq, batch, total_q;
  float scale, scale_log2;  // softmax scale, and scale * log2(e)
};

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
// Read-only metadata is addressed through the constant address space so that wave-uniform
// reads stay scalar loads (no vector-memory counter involved) even after LDS copies and stores.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;

constexpr int kTileBytes = kBN * kRowBytes;   // one K or V tile in LDS: 16 KiB

// The fixed-reference pass (see attn_kernel's run_pass) is tried first where P keeps fp32's
// exponent range.  fp16 holds p only up to 2^16: there the reference must follow the row max.
template <typename T> constexpr bool kTryFixedRef = false;
#ifndef MC_NO_FIXED_REF
template <> constexpr bool kTryFixedRef<__bf16> = true;
#endif
// A row sum below this proves that no exponential of the pass overflowed (every p is at most
// the sum) and that P fitted its 2-byte type; the O accumulators are checked for finiteness
// separately.  Reached only when a score exceeds the first half tile's maximum by more than
// 60 in the exp2 domain (about 41 in natural units).
constexpr float kFixedRefSumLimit = 0x1p+60f;
// register pairs of S(h) whose exponentials run in phase 2 of a fixed-reference half step
#ifndef MC_PAIRS_LATE
#define MC_PAIRS_LATE 4
#endif
constexpr int kPairsLate = MC_PAIRS_LATE;
// MFMA slot (0..15 of a half step) after which the first of a tile's eight copies is issued in
// the main loop; one more follows after each later slot
#ifndef MC_COPY_SLOT0
#define MC_COPY_SLOT0 4
#endif
constexpr int kCopySlot0 = MC_COPY_SLOT0;
static_assert(kCopySlot0 >= 1 && kCopySlot0 <= 8, "eight copy slots and one for the addresses before them");
static_assert(kPairsLate >= 0 && kPairsLate <= 4, "operand words 4..7 are read from phase 2's step 4 on");

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
// first pass a NaN-quieting instruction of its own).  The compiler does not see what an assembly
// statement reads, so it inserts none of the wait states a vector instruction needs before it
// may read the registers an MFMA is still writing: the first read of a fresh MFMA result goes
// through fmaxf, which the compiler does protect, and only the later ones through this.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Pipeline of one workgroup.  A KV tile (64 keys, 4 pages) is the unit of the V staging
// and of the workgroup barrier; a half tile (32 keys, 2 pages) is the unit of the K staging and
// of the softmax pipeline.  Half tile h lives in slot h % 4 of a ring of four K buffers, V
// tile j in V buffer j % 2.
//   tile j        issues the global->LDS copies of V(j+1) and of K halves 2j+3, 2j+4
//                 (asynchronous, no VGPRs), runs half steps 2j and 2j+1, waits for the copies
//   half step h   phase 1: S(h+1) = K(h+1) Q^T on the MFMA pipe, exponentials of S(h) on the VALU
//                 phase 2: O^T += V(h)^T P(h)^T on the MFMA pipe, row max of S(h+1) on the VALU
//                 O is rescaled only if a row max moved far
// The two score register sets swap roles every half step, so a tile starts and ends with the
// same set and nothing is copied.  Each step of a phase is one MFMA, at most one LDS fragment
// fetch (4 MFMAs ahead of its use) and a slice of the VALU work; the order is pinned.
// kGate: wavefronts none of whose rows exists skip the arithmetic.  Worth it for batches with
// many short q tiles (decode steps); the plain variant is ~2 % faster when all tiles are full.
// kCB: blocks of 32 rows per wavefront.  1: q tiles of 128 rows, two workgroups per compute
// unit.  2: q tiles of 256 rows, one workgroup per compute unit with twice the registers: every
// K and V fragment read from LDS feeds two MFMAs, every tile copied to LDS serves twice the rows.
template <typename T, int G, bool kGate, int kCB>
__global__ __launch_bounds__(kThreads, kCB == 1 ? 2 : 1) void attn_kernel(AttnArgs a) {
  constexpr int kWaveRows = 32 * kCB;       // rows per wavefront
  constexpr int TOK = kBM * kCB / G;        // tokens per q tile
  constexpr int kHalf = kBN / 2;
  constexpr int kHalfBytes = kTileBytes / 2;
  typedef typename Mfma<T>::vec8 vec8;
  // 4 K half tiles then 2 V tiles; reused as the output staging area at the end
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];
  __shared__ int s_redo;   // a row of the fixed-reference pass overflowed: run the pass again

  const int hk = blockIdx.x % a.hkv;
  const int wi = blockIdx.x / a.hkv;
  // The item record is requested together with the plan's header (the grid never exceeds the
  // room for records, whatever the header says): one memory round trip instead of two.
  typedef int32_t i32x8 __attribute__((ext_vector_type(8)));
  const auto* rec = (const __attribute__((address_space(4))) i32x8*)(a.items + wi);
  const i32x8 item = rec[0], item_b = rec[1];
  // the work list must come from a plan made for this very batch
  if (a.hdr->magic != kPlanMagic || wi >= a.hdr->num_items || a.hdr->tile_tokens != TOK ||
      a.hdr->batch != a.batch || a.hdr->total_q != a.total_q)
    return;

  const int tid = threadIdx.x, lane = tid & 63;
  if (tid == 0) s_redo = 0;   // published by the prologue's barrier
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;

  const int seq = item[0], row0 = item[1];
  const int t0 = item[2];                            // first KV tile of the item (even)
  const int part = item[4];                          // >= 0: partial result, merged afterwards
  const int gsize = item[5];                         // > 0: shared-prefix item over gsize tokens
  const int q_first = item[6];                       // the tile's first token in the q array
  const int ntok = item[7];                          // valid tokens in this tile (>= 1)
  const int table_off = item_b[0], pidx_cap = item_b[1];
  // a record that cannot come from the planner (a workspace written over by something else)
  if ((unsigned)seq >= (unsigned)a.batch || row0 < 0 || t0 < 0 || item[3] <= t0 || gsize < 0 ||
      gsize > TOK || ntok < 1 || ntok > TOK || (gsize > 0 && ntok != gsize) || q_first < 0 ||
      (int64_t)q_first + ntok > a.total_q || table_off < 0 || pidx_cap < 0)
    return;
  // begin is read here, not taken from the plan (one plan may serve many decode steps); it is
  // the only look-up between the record and the first copies
  const int b = a.begin[seq];
  // The position of the tile's first token.  The rows of a shared-prefix item are new tokens of
  // consecutive sequences; all of them lie beyond the prefix, so any position at or past the
  // item's last key serves.
  const int first_pos = gsize > 0 ? item[3] * kBN : b + row0;
  // keys [64 t0, kv_len) are this item's: up to the end of its chunk, or of the tile's range
  const int kv_len = min(first_pos + ntok, item[3] * kBN);
  const int n_kv_tiles = (kv_len + kBN - 1) / kBN;   // (absolute) index after the last KV tile
  const int n_halves = (kv_len + kHalf - 1) / kHalf;
  // half h is fully visible to every row of the q tile iff 32 (h+1) <= first_pos + 1
  const int n_full = (first_pos + 1) / kHalf;
  // A begin that no longer fits the item - negative, or so small that the item's first tile
  // lies past the range - ends the workgroup before any page is read; table indices never
  // pass the last entry the plan validated for the sequence.
  if (b < 0 || kv_len <= kBN * t0) {
    // a chunk that is not computed says so in its partial rows (no key seen: LSE = -inf), so
    // that the merge gives it no weight, and writes nothing if no chunk of the row was computed
    if (part >= 0)
      for (int i = tid; i < ntok * G; i += kThreads)
        a.part_lse[(int64_t)(part + i / G) * a.hq + hk * G + i % G] = -INFINITY;
    return;
  }
  const int last_pidx = min((kv_len - 1) / kPage, pidx_cap);   // last entry that holds a needed key

  // this lane's query rows, one per row block
  int g[kCB], tt[kCB], my_pos[kCB];
  bool row_ok[kCB];
  // Q as the B operand: lane holds d = 16 kk + 8 half + [0,8) of its row, kk = 0..7
  vec8 qreg[kCB][8];
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    const int r = wave * kWaveRows + cb * 32 + l32;    // row in tile
    g[cb] = r % G;                                     // token-major: the rows of a short tile
    tt[cb] = r / G;                                    // (a decode step's G rows) fill whole waves
    row_ok[cb] = tt[cb] < ntok;
    my_pos[cb] = first_pos + (row_ok[cb] ? tt[cb] : ntok - 1);   // causal limit of the row
    const int64_t q_row = ((int64_t)(q_first + tt[cb]) * a.hq + hk * G + g[cb]) * kRowBytes;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 v = {0, 0, 0, 0};
      if (row_ok[cb]) v = *reinterpret_cast<const u32x4*>(a.q + q_row + kk * 32 + half * 16);
      qreg[cb][kk] = __builtin_bit_cast(vec8, v);
    }
  }
  // a wavefront none of whose rows exists only helps with the copies and the barriers
  const bool wave_active = !kGate || wave * kWaveRows < ntok * G;

  // ---- global -> LDS copies (no VGPR staging) -------------------------------------
  // A wavefront's copy instruction fills 1 KiB of LDS linearly (lane L -> bytes 16 L..),
  // i.e. 4 rows.  A page is 16 rows: wave w fills rows 4 w + L/16 of the page (slots
  // 4 w..4 w+3); lane L fetches the 16-byte chunk that the swizzle wants at position L%16 of
  // that row.  Rows of keys at or beyond kv_len receive whatever the page holds (K: discarded
  // by the mask; V: zeroed in LDS before the last tile's P.V, since 0 x NaN would poison the
  // accumulators).
  const int ld_slot = 4 * wave + (lane >> 4), ld_pos = lane & 15;
  const char* pool_k = a.pool_layer + (int64_t)hk * kHeadPageBytes;
  const uint32_t k_lane_off = ld_slot * kRowBytes + ((ld_pos ^ ld_slot) << 4);
  const uint32_t v_lane_off = ld_slot * kRowBytes + ((ld_pos ^ ((ld_slot & 3) << 2)) << 4) +
                              (uint32_t)a.hkv * kHeadPageBytes;   // V run sits hkv blocks after K
  const uint32_t page_blocks = 2u * a.hkv;     // 4 KiB blocks per page
  const uint32_t lds_k = lds_addr(lds), lds_v = lds_k + 2 * kTileBytes;
  // wave-uniform address of this kv head's K run in the page of table entry pidx; entries
  // past the last needed one are replaced by the last needed one
  auto page_base = [&](int32_t pg) __attribute__((always_inline)) {
    pg = min(max(pg, 0), a.num_pages - 1);         // checked by the plan; stay in bounds anyway
    return pool_k + ((uint64_t)((uint32_t)pg * page_blocks) << 12);
  };
  auto copy_page = [&](const char* base, bool is_v, uint32_t lds_page) __attribute__((always_inline)) {   // 16 rows = 4 KiB
    copy16_to_lds(base, is_v ? v_lane_off : k_lane_off, lds_page + wave * 1024);
  };
  // ---- the page ids of the next copies -----------------------------------------------
  // The page ids of a tile's copies are fetched one tile early by a vector load (lane i & 7
  // holds table entry first + i).  It is an ordinary load, which the compiler tracks: wherever
  // the value is next needed (or moved, or spilled) the compiler waits for it, and since memory
  // operations complete in the order of their issue that wait also covers the copies issued
  // before it, which the compiler does not know of.  (As an untracked assembly load the register
  // could be spilled, under register pressure, before its data had arrived.)  arrive() is the
  // explicit wait for the copies - assembly statements, uncounted by the compiler - ahead of
  // the workgroup barrier.
  const int32_t* table_g = a.page_table + table_off;
  struct PageIds {
    int32_t reg;
    const int32_t* table;
    int lane7, last;
    __device__ __forceinline__ void issue(int first) {
      reg = __builtin_nontemporal_load(table + min(first + lane7, last));
    }
    __device__ __forceinline__ void arrive() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
    __device__ __forceinline__ int32_t value() const { return reg; }
  } ids;                                  // table entries of the next tile's copies
  ids.table = table_g;
  ids.lane7 = lane & 7;
  ids.last = last_pidx;
  auto wait_copies_and_sync = [&]() __attribute__((always_inline)) {
    ids.arrive();
    __syncthreads();
  };

  // ---- LDS fragment fetches ----------------------------------------------------------
  // K fragment f (0..7) of a half tile = d-step kk: rows l32, 16-byte chunk 2 kk + half.
  // V fragment g (0..7) of a half tile (rows crow..crow+31 of its tile): 16-key step st = g >> 2,
  // d chunk dc = g & 3; a 16-lane group reads 4 keys x 16 d, lane j supplies key (j/4) and d-quad
  // (j%4); the two reads cover accumulator registers 8 st..8 st+7, i.e. for this lane-half the
  // keys 16 st + {0..3} + 4 half and 16 st + 8 + {0..3} + 4 half.
  const int j16 = lane & 15, gq = (lane >> 4) & 1;
  auto k_frag = [&](uint32_t khalf, int f) __attribute__((always_inline)) {
    return *reinterpret_cast<const vec8 __attribute__((address_space(3)))*>(
        (size_t)(khalf + k_swz(l32, 2 * f + half)));
  };
  auto v_frag = [&](uint32_t vtile, int crow, int gi) __attribute__((always_inline)) {
    const int st = gi >> 2, dc = gi & 3;
    const int key_lo = crow + st * 16 + 4 * half + (j16 >> 2);
    const int chunk = dc * 4 + gq * 2 + ((j16 & 3) >> 1);
    const int sub = (j16 & 1) * 8;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(size_t)(vtile + v_swz(key_lo, chunk) + sub));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(size_t)(vtile + v_swz(key_lo + 8, chunk) + sub));
    return __builtin_bit_cast(vec8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // key held by accumulator register i of half h: 32 h + 8 (i/4) + 4 half + i%4
  auto mask_half = [&](int h, f32x16& sc, int cb) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = h * kHalf + 8 * (i >> 2) + 4 * half + (i & 3);
      if (key > my_pos[cb]) sc[i] = -INFINITY;
    }
  };
  // the other 16 keys of the row's half tile sit in lane l ^ 32: swap the wave's halves on the VALU
  // with one v_permlane32_swap: given the value in both operands, the first comes back holding
  // the lower half's value in both halves and the second the upper half's.  Written as assembly
  // (with the two wait states the instruction needs after a vector write of its operands):
  // through __builtin_amdgcn_permlane32_swap this compiler hands out the first result twice.
  auto max_across_halves = [&](float mx) __attribute__((always_inline)) {
    uint32_t lo = __builtin_bit_cast(uint32_t, mx), hi = lo;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
    return fmaxf(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
  };

  f32x16 o_acc[kCB][4];
  float m_run[kCB], l_run[kCB];           // reference score of the row (raw), this lane's partial sum
  float mx_cur[kCB];                      // row max of the half tile about to be exponentiated
  const float c2 = a.scale_log2;
  const f32x16 zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  constexpr int kAhead = 4;               // fragments in flight
  vec8 kf[kAhead];                        // first K fragments of the next phase 1
  f32x16 s_a[kCB], s_b[kCB];

  // ---- one half step.  s_cur = S(h) in, s_next = S(h+1) out (computed even when half h+1
  //      does not exist: its LDS rows are then stale, the result is never used).
  //      k_next: LDS address of K half h+1; k_after: of K half h+2, whose first fragments are
  //      fetched at the end of this step if fetch_after; v_cur/crow: V tile and row offset of
  //      half h.  mask_next: half h+1 reaches the causal diagonal.
  //      fixed_ref: the row's reference score stays where the prologue put it (see run_pass):
  //      no row max, no rescale, and the exponentials of the last kPairsLate register pairs move
  //      into phase 2, whose VALU slots the row max no longer needs.
  auto half_step = [&](auto fixed_ref, int h, uint32_t k_next, bool fetch_after, uint32_t k_after,
                       uint32_t v_cur, int crow, f32x16 (&s_cur)[kCB], f32x16 (&s_next)[kCB],
                       bool mask_next, auto&& slot_extra) __attribute__((always_inline)) {
    constexpr bool kFixed = decltype(fixed_ref)::value;
    constexpr int kPairs = 8 * kCB;                       // register pairs of S(h), all row blocks
    constexpr int kLate = kFixed ? kPairsLate * kCB : 0;  // ... of which phase 2 takes this many
    vec8 vf[kAhead];
    if constexpr (!kFixed) {
      // ---- move the reference max (and rescale O, l) only when some row's max rose by more
      //      than 2^8 in the exp2 domain: p stays below 2^8, sums stay exact
      bool moved = false;
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) moved |= (mx_cur[cb] - m_run[cb]) * c2 > 8.f;
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
        for (int cb = 0; cb < kCB; ++cb) {
          const float m_new = fmaxf(m_run[cb], mx_cur[cb]);
          const float alpha = __builtin_amdgcn_exp2f((m_run[cb] - m_new) * c2);
          m_run[cb] = m_new;
          l_run[cb] *= alpha;
#pragma unroll
          for (int dc = 0; dc < 4; ++dc)
#pragma unroll
            for (int i = 0; i < 16; ++i) o_acc[cb][dc][i] *= alpha;
        }
      }
    }
    float mc2[kCB];
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) mc2[cb] = m_run[cb] * c2;
    uint32_t p_pk[kCB][8];
    // softmax of register pair t of S(h) of row block cb (registers 2t, 2t+1 -> packed operand
    // word t).  The row sum takes the unrounded values: LSE must not inherit P's 2-byte rounding.
    // (The empty assembly statement keeps the additions here, beside their exponentials: left
    // alone the compiler gathers them at the end of the half step and keeps all values live.)
    auto soft_pair = [&](int cb, int t) __attribute__((always_inline)) {
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[cb][2 * t], c2, -mc2[cb]));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[cb][2 * t + 1], c2, -mc2[cb]));
      l_run[cb] += p0 + p1;
      asm volatile("" : "+v"(l_run[cb]));
      p_pk[cb][t] = Mfma<T>::pack2(p0, p1);
    };
    // pairs in the order phase 2 needs them: words 0..3 of every row block, then words 4..7
    auto soft_nth = [&](int i) __attribute__((always_inline)) {
      soft_pair((i / 4) % kCB, (i / (4 * kCB)) * 4 + i % 4);
    };
    __builtin_amdgcn_sched_barrier(0);
    // ---- phase 1: 8 steps.  Step t: d-step t of S(h+1) for every row block (one K fragment
    //      feeds kCB MFMAs); beside each MFMA the softmax of a register pair of S(h).
#pragma unroll
    for (int t = 0; t < 8; ++t) {
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        if (t * kCB + cb < kPairs - kLate) soft_nth(t * kCB + cb);
        if constexpr (kFixed && kCB == 2) {
          // (nothing reads these registers before the next half step's softmax, a whole phase
          // of MFMAs later, except the mask below, which waits for the matrix pipe first)
          if (t == 0) Mfma<T>::run_v0(kf[t % kAhead], qreg[cb][t], s_next[cb]);
          else Mfma<T>::run_v(kf[t % kAhead], qreg[cb][t], s_next[cb]);
        } else {
          s_next[cb] = Mfma<T>::run(kf[t % kAhead], qreg[cb][t], t == 0 ? zero16 : s_next[cb]);
        }
        if (cb + 1 < kCB) __builtin_amdgcn_sched_barrier(0);
      }
      if (t + kAhead < 8) kf[t % kAhead] = k_frag(k_next, t + kAhead);
      else vf[t % kAhead] = v_frag(v_cur, crow, t + kAhead - 8);
      slot_extra(t);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (mask_next) {
      // the scores may come from MFMAs the compiler does not see as such: let the last of them
      // (8 passes of 4 cycles) leave the pipe before vector instructions rewrite its registers
      if constexpr (kFixed && kCB == 2) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) mask_half(h + 1, s_next[cb], cb);
    }
    // ---- phase 2: 8 steps.  Step u: V fragment u (16-key step st = u >> 2 -> operand words
    //      4 st..4 st+3, d chunk dc = u & 3) for every row block; beside the MFMAs the row max
    //      over register pair u of S(h+1), or the softmax pairs phase 1 left over.
    float mx[kCB];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int st = u >> 2, dc = u & 3;
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        u32x4 pw = {p_pk[cb][4 * st], p_pk[cb][4 * st + 1], p_pk[cb][4 * st + 2], p_pk[cb][4 * st + 3]};
        o_acc[cb][dc] = Mfma<T>::run(vf[u % kAhead], __builtin_bit_cast(vec8, pw), o_acc[cb][dc]);
        if constexpr (kFixed) {
          if (u * kCB + cb < kLate) soft_nth(kPairs - kLate + u * kCB + cb);   // words 4..7: first read at step 4
        } else {
          mx[cb] = u == 0 ? fmaxf(s_next[cb][0], s_next[cb][1])
                          : max3(mx[cb], s_next[cb][2 * u], s_next[cb][2 * u + 1]);
        }
        if (cb + 1 < kCB) __builtin_amdgcn_sched_barrier(0);
      }
      if (u + kAhead < 8) vf[u % kAhead] = v_frag(v_cur, crow, u + kAhead);
      else if (fetch_after) kf[u % kAhead] = k_frag(k_after, u + kAhead - 8);
      slot_extra(8 + u);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (!kFixed) {
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) mx_cur[cb] = max_across_halves(mx[cb]);
    }
  };

  // ---- the copies of one tile.  par = j & 1 fixes every LDS address of the tile: K halves 2j+1,
  //      2j+2 are read from ring slots 1, 2 (even j) or 3, 0 (odd j) while halves 2j+3, 2j+4 are
  //      copied into the other two; V(j) is read from V buffer par while V(j+1) is copied into
  //      the other.  Table entries 4j+4 .. 4j+9 are involved: V(j+1) is entries +4..+7, K halves
  //      2j+3, 2j+4 are +6..+9.  Every lane turns the id it holds into its page's address (two
  //      vector instructions); the six addresses then move to scalar registers.
  const uint64_t pool_k_u = (uint64_t)(size_t)pool_k;
  const uint32_t page_stride_b = page_blocks << 12;
  struct TilePages { const char* pb[6]; };
  auto tile_pages = [&](int jt) __attribute__((always_inline)) {
    const int32_t pg = min(max(ids.value(), 0), a.num_pages - 1);   // checked by the plan; stay in bounds anyway
    const uint64_t addr = pool_k_u + (uint64_t)(uint32_t)pg * page_stride_b;
    const uint32_t lo = (uint32_t)addr, hi = (uint32_t)(addr >> 32);
    TilePages tp;
#pragma unroll
    for (int i = 0; i < 6; ++i)
      tp.pb[i] = (const char*)(size_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane(hi, i) << 32) |
                                       (uint32_t)__builtin_amdgcn_readlane(lo, i));
    ids.issue(4 * jt + 8);
    return tp;
  };
  // copy c of the tile's eight: the pages of K half 2j+3, the first two of V(j+1), K half 2j+4,
  // the last two of V(j+1) - the order in which the next tile needs them
  auto tile_copy = [&](const TilePages& tp, const int par, int c) __attribute__((always_inline)) {
    const uint32_t k_h3 = lds_k + (par ? 1 : 3) * kHalfBytes;     // K half 2j+3 (copy target)
    const uint32_t k_h4 = lds_k + (par ? 2 : 0) * kHalfBytes;     // K half 2j+4 (copy target)
    const uint32_t v_nxt = lds_v + (par ^ 1) * kTileBytes;
    switch (c) {
      case 0: copy_page(tp.pb[2], false, k_h3); break;
      case 1: copy_page(tp.pb[3], false, k_h3 + 4096); break;
      case 2: copy_page(tp.pb[0], true, v_nxt); break;
      case 3: copy_page(tp.pb[1], true, v_nxt + 4096); break;
      case 4: copy_page(tp.pb[4], false, k_h4); break;
      case 5: copy_page(tp.pb[5], false, k_h4 + 4096); break;
      case 6: copy_page(tp.pb[2], true, v_nxt + 2 * 4096); break;
      default: copy_page(tp.pb[3], true, v_nxt + 3 * 4096); break;
    }
  };
  // last tile: zero the V rows of keys >= kv_len (their P is 0, their bytes are arbitrary)
  auto zero_v_tail = [&](int jt, const int par) __attribute__((always_inline)) {
    const uint32_t v_cur = lds_v + par * kTileBytes;
    const int valid = kv_len - jt * kBN;
    const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = i * 16 + (tid >> 4);
      if (row >= valid)
        *reinterpret_cast<u32x4 __attribute__((address_space(3)))*>(
            (size_t)(v_cur + row * kRowBytes + (tid & 15) * 16)) = zero;
    }
    __syncthreads();
  };
  auto tile_copies = [&](int jt, const int par, bool in_main_loop) __attribute__((always_inline)) {
    if (in_main_loop || jt + 1 < n_kv_tiles) {
      const TilePages tp = tile_pages(jt);
#pragma unroll
      for (int c = 0; c < 8; ++c) tile_copy(tp, par, c);
    } else if (kv_len < (jt + 1) * kBN) {
      zero_v_tail(jt, par);
    }
  };

  // ---- one pass over the item's KV range, from its first tile: leaves o_acc, m_run, l_run.
  //      fixed_ref = false: the row's reference score follows the running row max (moved, with
  //      a rescale of O and l, when a half tile's max exceeds it by more than 2^8 in the exp2
  //      domain), so p <= 2^8 whatever the scores are.
  //      fixed_ref = true: the reference stays at the row max of the first half tile.  Any
  //      reference gives the same O and LSE as long as nothing overflows; this one costs no row
  //      max, no exchange between the wavefront's halves and no branch per half step.  Its p is
  //      unbounded, so it is only used where P keeps fp32's exponent range (bf16), and the
  //      caller checks the row sums afterwards.
  auto run_pass = [&](auto fixed_ref) __attribute__((always_inline)) {
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
#pragma unroll
      for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[cb][dc][i] = 0.f;
      m_run[cb] = -INFINITY;
      l_run[cb] = 0.f;
    }
    // ---- prologue: K halves 0, 1, 2 and V(0) in flight together; S(half 0) -------------
    {
      // table entries 0..5 of the item (K halves 0..2), 0..3 (V tile 0): their ids are in the record
      const char* pb[6];
#pragma unroll
      for (int i = 0; i < 6; ++i) pb[i] = page_base(item_b[2 + i]);
#pragma unroll
      for (int i = 0; i < 6; ++i) copy_page(pb[i], false, lds_k + i * 4096);
#pragma unroll
      for (int i = 0; i < 4; ++i) copy_page(pb[i], true, lds_v + i * 4096);
    }
    ids.issue(4 * t0 + 4);
    wait_copies_and_sync();
    if (wave_active) {
#pragma unroll
      for (int f = 0; f < 8; ++f) {
        const vec8 kfr = k_frag(lds_k, f);
#pragma unroll
        for (int cb = 0; cb < kCB; ++cb) {
          if constexpr (decltype(fixed_ref)::value && kCB == 2) {
            if (f == 0) Mfma<T>::run_v0(kfr, qreg[cb][f], s_a[cb]);
            else Mfma<T>::run_v(kfr, qreg[cb][f], s_a[cb]);
          } else {
            s_a[cb] = Mfma<T>::run(kfr, qreg[cb][f], f == 0 ? zero16 : s_a[cb]);
          }
        }
      }
      // (MFMAs written as assembly: the matrix pipe must have drained before their results are read)
      if constexpr (decltype(fixed_ref)::value && kCB == 2)
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
#pragma unroll
      for (int cb = 0; cb < kCB; ++cb) {
        if (n_full <= 2 * t0) mask_half(2 * t0, s_a[cb], cb);
        float mx = fmaxf(s_a[cb][0], s_a[cb][1]);
#pragma unroll
        for (int i = 2; i < 16; i += 2) mx = max3(mx, s_a[cb][i], s_a[cb][i + 1]);
        mx_cur[cb] = max_across_halves(mx);
        if constexpr (decltype(fixed_ref)::value) m_run[cb] = mx_cur[cb];
      }
    }
    __syncthreads();   // every wave has read K half 0 before tile 0 overwrites its slot

    // A wavefront none of whose rows exists (short tiles: a decode step has G rows) takes its
    // share of the copies and of the barriers, tile by tile, and nothing else.
    if (kGate && !wave_active) {
      for (int jt = t0; jt < n_kv_tiles; ++jt) {
        tile_copies(jt, jt & 1, false);
        wait_copies_and_sync();
      }
      return;
    }

    // ---- one tile
    auto tile = [&](int jt, const int par, bool mask0, bool mask1,
                    bool in_main_loop) __attribute__((always_inline)) {
      const uint32_t k_h1 = lds_k + (par ? 3 : 1) * kHalfBytes;     // K half 2j+1
      const uint32_t k_h2 = lds_k + (par ? 0 : 2) * kHalfBytes;     // K half 2j+2
      const uint32_t v_cur = lds_v + par * kTileBytes;
#pragma unroll
      for (int f = 0; f < kAhead; ++f) kf[f] = k_frag(k_h1, f);
      auto nothing = [](int) __attribute__((always_inline)) {};
      if (in_main_loop) {
        // the tile's copies go out one per MFMA slot of the first half step's second phase
        // (addresses in the slot before), under the matrix pipe's work instead of ahead of it
        TilePages tp;
        half_step(fixed_ref, 2 * jt, k_h1, true, k_h2, v_cur, 0, s_a, s_b, mask0,
                  [&](int slot) __attribute__((always_inline)) {
                    if (slot == kCopySlot0 - 1) tp = tile_pages(jt);
                    if (slot >= kCopySlot0 && slot < kCopySlot0 + 8) tile_copy(tp, par, slot - kCopySlot0);
                  });
      } else {
        tile_copies(jt, par, false);
        half_step(fixed_ref, 2 * jt, k_h1, true, k_h2, v_cur, 0, s_a, s_b, mask0, nothing);
      }
      if (in_main_loop || 2 * jt + 1 < n_halves)
        half_step(fixed_ref, 2 * jt + 1, k_h2, false, 0, v_cur, kHalf, s_b, s_a, mask1, nothing);
      wait_copies_and_sync();
    };

    // Tiles whose two half steps need no mask on their successor halves (2j+1, 2j+2 below the
    // diagonal) run two per iteration with constant LDS addresses; the rest follow one by one.
    const int n_main = max(t0, min(n_full - 2, 2 * n_kv_tiles - 2) / 2);   // tiles j with 2j+2 < n_full
    int jt = t0;
    for (; jt + 1 < n_main; jt += 2) {
      tile(jt, 0, false, false, true);
      tile(jt + 1, 1, false, false, true);
    }
    for (; jt < n_kv_tiles; ++jt)
      tile(jt, jt & 1, 2 * jt + 1 >= n_full, 2 * jt + 2 >= n_full, false);
  };

  if constexpr (kTryFixedRef<T>) {
    // First with the fixed reference.  A row whose sum left the range in which nothing can have
    // overflowed (or is not a number) sends the whole workgroup through the pass again with the
    // moving reference; on scores like the workloads' (a few units wide) that never happens.
    run_pass(std::true_type{});
    bool sums_ok = true;
    float o_chk = 0.f;                     // NaN if any accumulator is infinite or not a number
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
      sums_ok = sums_ok && l_run[cb] + __shfl_xor(l_run[cb], 32) < kFixedRefSumLimit;
#pragma unroll
      for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_chk = __builtin_fmaf(o_acc[cb][dc][i], 0.f, o_chk);
    }
    const bool bad = wave_active && !(sums_ok && o_chk == 0.f);
    if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) s_redo = 1;
    __syncthreads();
    if (s_redo != 0) run_pass(std::false_type{});
  } else {
    run_pass(std::false_type{});
  }
  if (kGate && !wave_active) return;

  // ---- epilogue: normalise, stage O through LDS for full-row stores, write LSE ----
  float l_tot[kCB], inv[kCB];
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    l_tot[cb] = l_run[cb] + __shfl_xor(l_run[cb], 32);
    inv[cb] = 1.f / l_tot[cb];
  }
  if (part >= 0) {
    // One chunk of a cut KV range: O normalised within the chunk (fp32) and the chunk's LSE go
    // to the partial arrays; merge_kernel weighs the chunks together.  A lane holds, for its
    // row, d = 32 dc + 8 j + 4 half + {0..3}: 16 bytes per (dc, j).
#pragma unroll
    for (int cb = 0; cb < kCB; ++cb) {
      if (!row_ok[cb]) continue;
      const int64_t prow = (int64_t)(part + tt[cb]) * a.hq + hk * G + g[cb];
      float* po = a.part_o + prow * mc::kHeadDim;
#pragma unroll
      for (int dc = 0; dc < 4; ++dc)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          typedef float f32x4 __attribute__((ext_vector_type(4)));
          f32x4 v = {o_acc[cb][dc][4 * j] * inv[cb], o_acc[cb][dc][4 * j + 1] * inv[cb],
                     o_acc[cb][dc][4 * j + 2] * inv[cb], o_acc[cb][dc][4 * j + 3] * inv[cb]};
          *reinterpret_cast<f32x4*>(po + 32 * dc + 8 * j + 4 * half) = v;
        }
      if (half == 0) a.part_lse[prow] = m_run[cb] * a.scale + __logf(l_tot[cb]);
    }
    return;
  }
  // 8 KiB per wave and row block; all tiles are consumed
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    char* stage = lds + (wave * kCB + cb) * (32 * kRowBytes);
#pragma unroll
    for (int dc = 0; dc < 4; ++dc)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // registers 4j..4j+3 hold d = 32 dc + 8 j + 4 half + {0..3}: 8 bytes of chunk 4 dc + j
        u32x2 w;
        w[0] = Mfma<T>::pack2(o_acc[cb][dc][4 * j] * inv[cb], o_acc[cb][dc][4 * j + 1] * inv[cb]);
        w[1] = Mfma<T>::pack2(o_acc[cb][dc][4 * j + 2] * inv[cb], o_acc[cb][dc][4 * j + 3] * inv[cb]);
        *reinterpret_cast<u32x2*>(stage + k_swz(l32, 4 * dc + j) + half * 8) = w;
      }
    if (row_ok[cb] && half == 0)
      a.lse[(int64_t)(q_first + tt[cb]) * a.hq + hk * G + g[cb]] =
          m_run[cb] * a.scale + __logf(l_tot[cb]);
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int cb = 0; cb < kCB; ++cb) {
    const char* stage = lds + (wave * kCB + cb) * (32 * kRowBytes);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int lr = 4 * i + (lane >> 4);               // row of this block's 32
      const int rr = wave * kWaveRows + cb * 32 + lr, gg = rr % G, t2 = rr / G;
      const u32x4 v = *reinterpret_cast<const u32x4*>(stage + k_swz(lr, lane & 15));
      if (t2 < ntok)
        *reinterpret_cast<u32x4*>(a.out + ((int64_t)(q_first + t2) * a.hq + hk * G + gg) * kRowBytes +
                                  (lane & 15) * 16) = v;
    }
  }
}

// Combines the chunks of every q tile whose KV range was cut: with L_c the chunk LSEs,
// LSE = log sum_c exp(L_c) and O = sum_c exp(L_c - LSE) O_c.  The grid walks the (token, four q
// heads) pairs of those tiles - the host does not know how many tiles were cut, usually none, so
// it sizes the grid for the batch's new tokens - one wavefront per q head, two d per lane; a
// chunk's loads do not depend on another chunk's, so they are all in flight together.
struct MergeArgs {
  const PlanHeader* hdr;
  const MergeRec* merges;
  const float* part_lse;
  const float* part_o;
  char* out;
  float* lse;
  int32_t hq, tile_tokens;
};

template <typename T>
__global__ __launch_bounds__(256) void merge_kernel(MergeArgs a) {
  if (a.hdr->magic != kPlanMagic) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int head_groups = (a.hq + 3) / 4;
  const int n_rec = a.hdr->num_merges;
  const int64_t total = (int64_t)a.hdr->merge_tokens * head_groups;   // usually 0: nothing was cut
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  for (int64_t wk = blockIdx.x; wk < total; wk += gridDim.x) {
    const int tok = (int)(wk / head_groups), h = (int)(wk % head_groups) * 4 + wave;
    // the record whose token range [tok_off, tok_off + ntok) holds tok: a search that looks at
    // 64 records per round, one per lane (one memory latency for up to 64 records, two for 4096)
    int lo = 0, cnt = n_rec;
    while (cnt > 1) {
      const int step = (cnt + 63) / 64, end = lo + cnt;
      const int i = lo + lane * step;
      const bool le = i < end && a.merges[i].tok_off <= tok;
      const int k = max(__popcll(__ballot(le)) - 1, 0);   // tok_off rises with the record index
      lo += k * step;
      cnt = min(step, end - lo);
    }
    const MergeRec m = a.merges[lo];
    const int tt = tok - m.tok_off;
    if (tt < 0 || tt >= m.ntok || h >= a.hq) continue;
    // partial row of chunk c: the shared prefix's chunks first, then the tile's own
    auto row_of = [&](int c) {
      return (int64_t)(c < m.g_nsplit ? m.g_part + c * m.g_stride + tt
                                      : m.part + (c - m.g_nsplit) * m.ntok + tt) * a.hq + h;
    };
    const int nchunks = m.g_nsplit + m.nsplit;
    // the chunks' LSEs: one per lane (in rounds of 64), so that their loads are in flight
    // together instead of one after the other; the maximum by a butterfly over the wavefront
    float mx = -INFINITY;
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
      const int c = c0 + lane;
      mx = fmaxf(mx, c < nchunks ? a.part_lse[row_of(c)] : -INFINITY);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (!(mx > -INFINITY)) continue;   // no chunk of this row was computed: nothing to write
    float den = 0.f;
    f32x2 acc = {0.f, 0.f};
    for (int c0 = 0; c0 < nchunks; c0 += 64) {
      const int c = c0 + lane;
      // exp(-inf) = 0 for a chunk with no key, and for the lanes beyond the last chunk
      const float w_lane = c < nchunks ? __expf(a.part_lse[row_of(c)] - mx) : 0.f;
      float sum = w_lane;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
      den += sum;
      const int n = min(64, nchunks - c0);
      for (int k = 0; k < n; ++k) {
        const float w = __shfl(w_lane, k);
        const f32x2 v =
            *reinterpret_cast<const f32x2*>(a.part_o + row_of(c0 + k) * mc::kHeadDim + 2 * lane);
        acc += v * w;
      }
    }
    const float inv = 1.f / den;
    const int64_t orow = (int64_t)(m.q_row + tt) * a.hq + h;
    *reinterpret_cast<uint32_t*>(a.out + orow * kRowBytes + 4 * lane) =
        Mfma<T>::pack2(acc[0] * inv, acc[1] * inv);
    if (lane == 0) a.lse[orow] = mx + __logf(den);
  }
}

template <typename T, bool kGate, int kCB>
mc_status launch_attn_g(int G, dim3 grid, hipStream_t hs, const AttnArgs& a) {
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_kernel<T, 1, kGate, kCB>), grid, dim3(kThreads), 0, hs, a); break;
    case 2: hipLaunchKernelGGL((attn_kernel<T, 2, kGate, kCB>), grid, dim3(kThreads), 0, hs, a); break;
    case 4: hipLaunchKernelGGL((attn_kernel<T, 4, kGate, kCB>), grid, dim3(kThreads), 0, hs, a); break;
    case 8: hipLaunchKernelGGL((attn_kernel<T, 8, kGate, kCB>), grid, dim3(kThreads), 0, hs, a); break;
    default: return MC_ERR_UNSUPPORTED;
  }
  return mc::launch_status();
}

template <typename T>
mc_status launch_attn(int G, bool gate, int row_blocks, dim3 grid, hipStream_t hs, const AttnArgs& a) {
  if (row_blocks == 2) return launch_attn_g<T, false, 2>(G, grid, hs, a);
  return gate ? launch_attn_g<T, true, 1>(G, grid, hs, a) : launch_attn_g<T, false, 1>(G, grid, hs, a);
}

// Workgroups of the attention kernel the current GPU runs at a time: two per compute unit
// (one with the wide q tiles).
// The compute-unit count is asked for once per device (the query costs microseconds, which a
// decode step notices); the current device is a thread-local read.
int device_slots(int row_blocks = 1) {
  constexpr int kDevs = 64;
  static std::atomic<int> cached[kDevs];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) return -1;
  if (dev < kDevs) {
    const int c = cached[dev].load(std::memory_order_relaxed);
    if (c > 0) return row_blocks == 2 ? c / 2 : c;
  }
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      cus <= 0)
    return -1;
  if (dev < kDevs) cached[dev].store(2 * cus, std::memory_order_relaxed);
  return row_blocks == 2 ? cus : 2 * cus;
}

// The planner cuts KV ranges only if the q tiles times kv heads are fewer than kRoundsWanted per
// slot; the number of q tiles is at least total_q / tile_tokens, which the host knows.
bool may_cut(const WorkspaceLayout& w, int hkv, int slots) {
  return w.part_cap > 0 && (int64_t)(w.max_tiles - w.batch) * hkv < (int64_t)kRoundsWanted * slots;
}

// Shared-prefix groups are made of sequences with one new token each: worth looking for only
// when the batch could hold a fair share of those (fewer than two q tiles' worth of new tokens
// per sequence on average), and possible only with room for partial rows.
bool may_group(const WorkspaceLayout& w, int32_t total_q, int tile_tokens) {
  return w.part_cap > 0 && w.batch >= 2 && w.batch <= kCuTilesInLds &&
         (int64_t)total_q < 2ll * w.batch * tile_tokens;
}

// Upper bound of the planner's item count: a q tile with T KV tiles becomes at most T / L + 1
// items, and the planner's chunk length L is at least (sum of T) x hkv / (kRoundsWanted x slots).
// A shared-prefix group adds at most one item per sequence beyond that.
int32_t item_bound(const WorkspaceLayout& w, int hkv, int slots, bool groups) {
  int64_t b = w.max_tiles;
  if (may_cut(w, hkv, slots)) b += (int64_t)kRoundsWanted * slots / hkv + 1;
  if (groups) b += w.batch;
  return (int32_t)(b < w.max_items ? b : w.max_items);
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

mc_status plan_impl(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                    int32_t total_q, const int32_t* cu_q, const int32_t* begin,
                    const int32_t* page_table, const int32_t* cu_pages, int32_t ahead_tokens,
                    void* workspace, size_t workspace_bytes, int32_t part_limit, void* stream) {
  if (ahead_tokens < 0 || ahead_tokens > (1 << 20)) return MC_ERR_RANGE;
  int G = 0;
  mc_status st = check_attn_shape(pool, num_q_heads, batch, total_q, &G);
  if (st != MC_OK) return st;
  if (!workspace || !mc::aligned16(workspace)) return MC_ERR_INVALID;
  const int tile_tokens = kBM / G;
  const WorkspaceLayout w =
      workspace_layout(batch, total_q, tile_tokens, num_q_heads, pool->num_kv_heads, part_limit);
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
  a.items = reinterpret_cast<ItemRec*>(ws + w.items);
  a.merges = reinterpret_cast<MergeRec*>(ws + w.merges);
  a.batch = batch;
  a.total_q = total_q;
  a.tile_tokens = tile_tokens;
  a.num_pages = pool->num_pages;
  a.max_tiles = w.max_tiles;
  a.hkv = pool->num_kv_heads;
  a.slots = device_slots(1);
  if (a.slots <= 0) return MC_ERR_HIP;
  const bool wide = wide_tiles_allowed(batch, total_q, G, pool->num_kv_heads);
  a.wide_tile_tokens = wide ? 2 * tile_tokens : 0;
  a.slots_wide = device_slots(2);
  a.allow_groups = may_group(w, total_q, tile_tokens);
  a.max_items = item_bound(w, a.hkv, a.slots, a.allow_groups);
  a.part_cap = w.part_cap;
  a.ahead = ahead_tokens;
  // (few sequences only: the page-id checks and the table comparisons of shared prefixes go
  // a wavefront per sequence or pair and want the wavefronts of the large workgroup)
  if (batch <= 16 && w.max_tiles <= 8 * kPlanThreadsSmall)
    hipLaunchKernelGGL(plan_kernel<kPlanThreadsSmall>, dim3(1), dim3(kPlanThreadsSmall), 0,
                       static_cast<hipStream_t>(stream), a);
  else
    hipLaunchKernelGGL(plan_kernel<kPlanThreads>, dim3(1), dim3(kPlanThreads), 0,
                       static_cast<hipStream_t>(stream), a);
  if (batch > kValidateInPlan)
    hipLaunchKernelGGL(validate_pages_kernel, dim3((batch + 3) / 4), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
  return mc::launch_status();
}


mc_status attn_impl(const mc_pool_desc* pool, int32_t layer, const void* q, int32_t num_q_heads,
                    int32_t batch, int32_t total_q, const int32_t* cu_q, const int32_t* begin,
                    const int32_t* page_table, const int32_t* cu_pages, float sm_scale, void* out,
                    float* lse, void* workspace, size_t workspace_bytes, int32_t part_limit,
                    void* stream) {
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
  const int tile_tokens = kBM / G;
  const WorkspaceLayout w =
      workspace_layout(batch, total_q, tile_tokens, num_q_heads, pool->num_kv_heads, part_limit);
  if (workspace_bytes < w.total) return MC_ERR_INVALID;
  const int slots = device_slots(1);
  if (slots <= 0) return MC_ERR_HIP;
  const bool groups = may_group(w, total_q, tile_tokens);
  const int64_t blocks =
      (int64_t)item_bound(w, pool->num_kv_heads, slots, groups) * pool->num_kv_heads;
  if (blocks > 0x7fffffffll) return MC_ERR_UNSUPPORTED;
  char* ws = static_cast<char*>(workspace);
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
  a.items = reinterpret_cast<const ItemRec*>(ws + w.items);
  a.part_lse = reinterpret_cast<float*>(ws + w.part_lse);
  a.part_o = reinterpret_cast<float*>(ws + w.part_o);
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
  // many sequences for the number of q tiles: a good share of the tiles is short
  const bool gate = 4ll * batch >= w.max_tiles - batch;
  st = pool->dtype == MC_F16 ? launch_attn<_Float16>(G, gate, 1, grid, hs, a)
                             : launch_attn<__bf16>(G, gate, 1, grid, hs, a);
  if (st == MC_OK && wide_tiles_allowed(batch, total_q, G, pool->num_kv_heads)) {
    // the plan may be one of wide q tiles (fewer items than the grid's bound, which holds for
    // either width): that kernel, too; the one the plan was not made for finds the other tile
    // size in the header and returns
    st = pool->dtype == MC_F16 ? launch_attn<_Float16>(G, false, 2, grid, hs, a)
                               : launch_attn<__bf16>(G, false, 2, grid, hs, a);
  }
  if (st != MC_OK || !(may_cut(w, pool->num_kv_heads, slots) || groups)) return st;
  // the planner may have cut KV ranges: weigh the chunks together (does nothing if it did not)
  MergeArgs m;
  m.hdr = a.hdr;
  m.merges = reinterpret_cast<const MergeRec*>(ws + w.merges);
  m.part_lse = a.part_lse;
  m.part_o = a.part_o;
  m.out = a.out;
  m.lse = a.lse;
  m.hq = num_q_heads;
  m.tile_tokens = tile_tokens;
  // one workgroup per (token, four q heads) pair if they all run at once, else a grid-stride walk
  const int64_t pairs = (int64_t)total_q * ((num_q_heads + 3) / 4);
  const dim3 mgrid((unsigned)(pairs < 4ll * slots ? pairs : 4ll * slots));
  if (pool->dtype == MC_F16)
    hipLaunchKernelGGL(merge_kernel<_Float16>, mgrid, dim3(256), 0, hs, m);
  else
    hipLaunchKernelGGL(merge_kernel<__bf16>, mgrid, dim3(256), 0, hs, m);
  return mc::launch_status();
}


// ---- scratch of the entry point that allocates nothing ---------------------------------
// The attention workspace (work list, partial rows) of mc_prefix_prefill_attn_noalloc lives in
// this array; every GPU the library runs on holds its own copy until the process ends.
constexpr size_t kScratchBytes = size_t(8) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of the current device's copy of `scratch` (in host code the array's name is
// only a handle for this look-up, never an address a kernel may use).  Looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

mc_status scratch_of_current_device(void** ptr_out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MC_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *ptr_out = g_scratch_ptr[dev];
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
  return workspace_layout(batch, total_q, kBM / G, num_q_heads, num_kv_heads).total;
}

mc_status mc_attn_plan(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                       int32_t total_q, const int32_t* cu_q, const int32_t* begin,
                       const int32_t* page_table, const int32_t* cu_pages, void* workspace,
                       size_t workspace_bytes, void* stream) {
  return mc_attn_plan_ahead(pool, num_q_heads, batch, total_q, cu_q, begin, page_table, cu_pages,
                            0, workspace, workspace_bytes, stream);
}

mc_status mc_attn_plan_ahead(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                             int32_t total_q, const int32_t* cu_q, const int32_t* begin,
                             const int32_t* page_table, const int32_t* cu_pages,
                             int32_t ahead_tokens, void* workspace, size_t workspace_bytes,
                             void* stream) {
  return plan_impl(pool, num_q_heads, batch, total_q, cu_q, begin, page_table, cu_pages,
                   ahead_tokens, workspace, workspace_bytes, -1, stream);
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
                                 float sm_scale, void* out, float* lse, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  return attn_impl(pool, layer, q, num_q_heads, batch, total_q, cu_q, begin, page_table, cu_pages,
                   sm_scale, out, lse, workspace, workspace_bytes, -1, stream);
}

mc_status mc_prefix_prefill_attn_noalloc(const mc_pool_desc* pool, int32_t layer, const void* q,
                                         int32_t num_q_heads, int32_t batch, int32_t total_q,
                                         const int32_t* cu_q, const int32_t* begin,
                                         const int32_t* page_table, const int32_t* cu_pages,
                                         float sm_scale, void* out, float* lse, void* stream) {
  int G = 0;
  mc_status st = check_attn_shape(pool, num_q_heads, batch, total_q, &G);
  if (st != MC_OK) return st;
  // the work list alone must fit; what is left holds partial rows (32-byte item record, LSE
  // and O per row and q head), fewer than the caller-workspace variant may ask for
  const int tile_tokens = kBM / G;
  const WorkspaceLayout fixed =
      workspace_layout(batch, total_q, tile_tokens, num_q_heads, pool->num_kv_heads, 0);
  if (fixed.total + 4096 > kScratchBytes) return MC_ERR_RANGE;
  const size_t per_row = sizeof(ItemRec) + sizeof(float) * (size_t)num_q_heads * (mc::kHeadDim + 1);
  int32_t part_limit = (int32_t)((kScratchBytes - fixed.total - 4096) / per_row);
  while (part_limit > 0 &&
         workspace_layout(batch, total_q, tile_tokens, num_q_heads, pool->num_kv_heads, part_limit)
                 .total > kScratchBytes)
    --part_limit;
  void* ws = nullptr;
  st = scratch_of_current_device(&ws);
  if (st != MC_OK) return st;
  st = plan_impl(pool, num_q_heads, batch, total_q, cu_q, begin, page_table, cu_pages, 0, ws,
                 kScratchBytes, part_limit, stream);
  if (st != MC_OK) return st;
  return attn_impl(pool, layer, q, num_q_heads, batch, total_q, cu_q, begin, page_table, cu_pages,
                   sm_scale, out, lse, ws, kScratchBytes, part_limit, stream);
}

}  // extern "C"
