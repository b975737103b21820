/*
 * mc_kv.h -- C ABI of the MI355X (gfx950) paged KV-cache hot path.
 *
 * The calls are the data-plane half of the unified KV cache interface of
 * "A System for Microserving of LLMs" (arXiv 2412.12488), Sec. 3.4:
 *   - prep_recv matches the prompt against the engine's context cache and
 *     allocates KV entries (page index + slot index, Sec. 3.2 Examples 2, 3)
 *     for the part the engine does not hold; the addresses travel in a
 *     compressed form
 *            -> mc_prefix_index_*, mc_prep_recv, mc_kv_alloc_pages, mc_addr_*
 *   - begin_forward plans the metadata once for all attention layers
 *                                                   -> mc_attn_plan
 *   - attention(qkv_data) writes the new K/V into the cache and attends the
 *     new tokens over the cached prefix and themselves (start_generate
 *     prefills prompt[begin:] over the cached prompt[:begin], Sec. 3.1; the
 *     balanced split continues with prompt[s:], fused with the decode steps
 *     of other sequences, Sec. 3.3; sequences forked from one prompt share its
 *     pages, Sec. 3.4 and fork_sequence in Sec. 3.5)
 *                                   -> mc_kv_append, mc_prefix_prefill_attn
 *   - remote_send moves the KV of prompt[begin:end] into the entries the
 *     receiver reserved (Sec. 3.1), layer by layer beside the computation
 *     (Sec. 3.6); on one GPU the wire is replaced by a contiguous buffer in HBM;
 *     which ranges the sender copies, computes and sends follows from what the
 *     two engines have cached (Sec. 3.5, Cases 1 and 2)
 *            -> mc_plan_remote_send, mc_kv_pack_range, mc_kv_unpack_range
 *
 * The paper fixes no dtype, page size, page layout, softmax scale or LSE base;
 * the choices below are this library's.
 *
 * Conventions for every call
 *   - Plain pointers and sizes only.  "device" = HIP device memory of the
 *     current device, "host" = ordinary host memory.
 *   - All device memory is owned by the caller and must stay valid until the
 *     work queued on `stream` has finished.  The library owns only the host
 *     objects made by mc_kv_allocator_create and mc_prefix_index_create.
 *   - Calls that take a `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) only enqueue kernels: they never synchronise, never
 *     allocate, never copy from host.  Arguments are validated on the host
 *     before anything is launched; on any error nothing is launched.
 *   - Values that live in device arrays (page ids, offsets) cannot be seen by
 *     the host.  Kernels bounds-check every page id against the pool and every
 *     page-table index against the sequence's table; an entry that fails is
 *     skipped (no read, no write) and reported: for attention through
 *     mc_attn_plan_check, for the copies through mc_kv_copy_check.
 *   - Return value: mc_status (MC_OK = 0).
 *
 * Layouts (2-byte elements, fp16 or bf16, head_dim D = 128, page size P = 16)
 *   pool     [layer][page][2: 0=K 1=V][kv_head][slot][D]
 *            one (layer,page,K|V,kv_head) block is a contiguous 4 KiB run
 *   q, out   [token][q_head][D]        tokens of all sequences back to back
 *   k_new    [token][kv_head][D]       (v_new likewise)
 *   lse      [token][q_head]  float32, natural log of sum_j exp(scale * q.k_j)
 *   sendbuf  [layer - layer_begin][2][token - s0][kv_head][D]
 *   page_table  int32 page ids of all sequences back to back; sequence s owns
 *            entries [cu_pages[s], cu_pages[s+1]); entry i holds tokens
 *            [16 i, 16 i + 16) of the sequence
 *   cu_q     int32 [batch+1], cu_q[s+1]-cu_q[s] = new tokens of sequence s
 *   begin    int32 [batch], cached prefix length of sequence s; its new tokens
 *            are positions [begin[s], begin[s] + q_s)
 * Ranges are token-granular: begin, end, s0, s1 need not be multiples of 16.
 */
#ifndef MC_KV_H_
#define MC_KV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MC_OK = 0,
  MC_ERR_INVALID = 1,     /* null pointer, negative size, misaligned pointer, bad handle */
  MC_ERR_NO_PAGES = 2,    /* allocator cannot satisfy the request; nothing was taken */
  MC_ERR_RANGE = 3,       /* layer / token range / table length outside the pool or table */
  MC_ERR_ALIAS = 4,       /* a destination page is listed twice */
  MC_ERR_UNSUPPORTED = 5, /* head_dim != 128, page_size != 16, unknown dtype, GQA ratio */
  MC_ERR_HIP = 6          /* a HIP launch failed */
} mc_status;

typedef enum { MC_F16 = 0, MC_BF16 = 1 } mc_dtype;

/* One page pool.  `base` is device memory, 16-byte aligned, of
 * num_layers*num_pages*2*num_kv_heads*page_size*head_dim 2-byte elements. */
typedef struct {
  void* base;
  int32_t num_layers;
  int32_t num_pages;
  int32_t page_size;    /* must be 16 */
  int32_t num_kv_heads;
  int32_t head_dim;     /* must be 128 */
  int32_t dtype;        /* mc_dtype */
  int32_t* skipped;     /* device int32 counter, 4-byte aligned, or NULL: see mc_kv_copy_check */
} mc_pool_desc;

/* Human-readable name of a status code (static storage). */
const char* mc_status_string(int32_t status);
/* Bumped on any incompatible change of this header. */
int32_t mc_abi_version(void);

/* ---- page allocator (prep_recv reserves the entries that will receive KV, Sec. 3.1) ----
 * Host-only LIFO free list over page ids [0, num_pages).  A fresh allocator
 * hands out 0, 1, 2, ...; freed pages are pushed in argument order, so the last
 * page of the last free call is handed out next.  Not thread-safe. */
mc_status mc_kv_allocator_create(int32_t num_pages, void** alloc_out /* host */);
mc_status mc_kv_allocator_destroy(void* alloc);
/* All-or-nothing: MC_ERR_NO_PAGES leaves the allocator unchanged. */
mc_status mc_kv_alloc_pages(void* alloc, int32_t n, int32_t* pages_out /* host, n entries */);
/* MC_ERR_INVALID (nothing freed) if a page is out of range, not allocated, or listed twice. */
mc_status mc_kv_free_pages(void* alloc, int32_t n, const int32_t* pages /* host */);
mc_status mc_kv_allocator_num_free(void* alloc, int32_t* num_free_out /* host */);
/* Host check of a destination page table before append / unpack: MC_ERR_RANGE if an
 * id is outside [0,num_pages), MC_ERR_ALIAS if one appears twice, else MC_OK. */
mc_status mc_kv_check_page_table(const int32_t* pages /* host */, int64_t n, int32_t num_pages);

/* ---- what the copy kernels skipped -------------------------------------------
 * append, append_send, pack and unpack (single and batched) never read or write
 * out of bounds: a token whose table index lies beyond its sequence's table or
 * whose page id lies outside the pool, and a sequence of a batched call whose
 * offsets are malformed (negative or reversed table offsets, negative or
 * misaligned buffer offset), is left out.  With pool->skipped set, every kernel
 * adds the number of units it left out for such a reason (tokens for append,
 * pages or sequences for pack / unpack) to that counter; ranges that are empty
 * by their own statement (s0 >= s1) are not counted.  The caller zeroes the
 * counter before first use (it is only ever added to).
 * mc_kv_copy_check synchronises `stream`, reads the counter into *skipped_out
 * (host, may be NULL), sets it back to zero and returns MC_OK if it was zero,
 * MC_ERR_RANGE otherwise; MC_ERR_INVALID without a counter.  Like
 * mc_attn_plan_check it blocks; the copy calls themselves never do. */
mc_status mc_kv_copy_check(const mc_pool_desc* pool, int32_t* skipped_out /* host */,
                           void* stream);

/* ---- append: write new K/V into their (page, slot) entries -----------------
 * (the KV-write half of attention(qkv_data), Sec. 3.4; remote_send computes the KV
 * it does not hold before it sends them, Sec. 3.1).
 * Token g of sequence s (cu_q[s] <= g < cu_q[s+1]) has position
 * pos = begin[s] + g - cu_q[s] and goes to page page_table[cu_pages[s] + pos/16],
 * slot pos%16, of `layer`.  No other byte of the pool is written.  Two tokens
 * mapping to one (page, slot) is a caller error (undefined which one lands).
 * total_q = cu_q[batch] (host copy, sizes the launch); 0 is legal. */
mc_status mc_kv_append(const mc_pool_desc* pool, int32_t layer,
                       const void* k_new /* device [total_q][Hkv][D] */,
                       const void* v_new /* device [total_q][Hkv][D] */,
                       int32_t batch, int32_t total_q,
                       const int32_t* cu_q /* device [batch+1] */,
                       const int32_t* begin /* device [batch] */,
                       const int32_t* page_table /* device */,
                       const int32_t* cu_pages /* device [batch+1] */,
                       void* stream);

/* mark_send (Sec. 3.4; with it set, attention also sends the sequence's KV, Sec. 3.5,
 * layer by layer while the computation goes on, Sec. 3.6): mc_kv_append, and in the same pass the tokens of
 * the new range that lie in the marked range [s0[s], s1[s]) of their sequence
 * are written to the sequence's slice of a transfer buffer as well - the bytes
 * mc_kv_pack_batch(pool, send_layer_begin, ..., s0, s1, buf_offset, ...) would
 * write for this layer and these tokens, without reading them back from the
 * pages.  The part of a marked range that was cached before ([s0, begin)) is
 * mc_kv_pack_batch's.  s0[s] < 0 or s0[s] >= s1[s] marks nothing for sequence s.
 * send_layer_begin: first layer of the buffer's layout (<= layer, else
 * MC_ERR_RANGE); the other errors are those of mc_kv_append and mc_kv_pack_batch. */
mc_status mc_kv_append_send(const mc_pool_desc* pool, int32_t layer,
                            const void* k_new /* device [total_q][Hkv][D] */,
                            const void* v_new /* device [total_q][Hkv][D] */,
                            int32_t batch, int32_t total_q,
                            const int32_t* cu_q /* device [batch+1] */,
                            const int32_t* begin /* device [batch] */,
                            const int32_t* page_table /* device */,
                            const int32_t* cu_pages /* device [batch+1] */,
                            int32_t send_layer_begin,
                            const int32_t* s0 /* device [batch] */,
                            const int32_t* s1 /* device [batch] */,
                            const int64_t* buf_offset /* device [batch], bytes */,
                            void* sendbuf /* device */, void* stream);

/* ---- attention of the new range over the paged cache -----------------------
 * For sequence s, new token at position i in [begin[s], begin[s]+q_s), head h:
 *   out[i,h,:] = sum_j softmax_j(scale * q[i,h].k[j,h/G]) * v[j,h/G,:],  j in [0, i]
 *   lse[i,h]   = ln sum_j exp(scale * q[i,h].k[j,h/G])
 * with G = num_q_heads / num_kv_heads in {1,2,4,8}; K and V of every j,
 * including the new range, are read from the pages (mc_kv_append of this layer
 * comes first on the same stream).  Accumulation and softmax are fp32, out is
 * rounded to the pool dtype.  Page tables of different sequences may share
 * pages (shared prefixes, Sec. 3.4; fork_sequence, Sec. 3.5); when neighbouring sequences
 * of the batch each bring one new token and their tables start with the same
 * pages (at least 512 tokens' worth, cached by all of them), the plan lets
 * them attend that prefix together, reading its K/V once, and merges the result
 * with each sequence's own remainder.  The results are those of the formula
 * above either way.
 *
 * mc_attn_plan is the declaration stage (begin_forward, Sec. 3.4): it turns the
 * ragged batch into a work list in `workspace`, validates the device arrays and
 * is valid for every layer as long as the arrays it was given are unchanged.
 * mc_prefix_prefill_attn requires a workspace planned with the same arguments.
 * When a batch has too few (new token, kv head) tiles to fill the GPU - decode
 * steps (one new token per sequence, Sec. 3.3: the prefill of the remaining
 * prompt is fused with decode), short ranges over long contexts - the plan
 * cuts long KV ranges into chunks that run side by side; the attention call
 * then keeps the chunks' partial results in the workspace and merges them
 * (by their log-sum-exp) before it returns control of the stream.  Calls that
 * use one workspace must therefore run one after the other, never concurrently.
 * mc_attn_workspace_size gives the bytes needed (0 on bad arguments; room
 * for those partial results, at most 128 MiB, is part of it unless the batch is
 * large enough never to need them); workspace must be 16-byte aligned. */
size_t mc_attn_workspace_size(int32_t batch, int32_t total_q, int32_t num_q_heads,
                              int32_t num_kv_heads);
mc_status mc_attn_plan(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                       int32_t total_q,
                       const int32_t* cu_q /* device [batch+1] */,
                       const int32_t* begin /* device [batch] */,
                       const int32_t* page_table /* device */,
                       const int32_t* cu_pages /* device [batch+1] */,
                       void* workspace /* device */, size_t workspace_bytes, void* stream);
/* The same plan, made to last for several decode steps: it stays valid while cu_q
 * is unchanged and every sequence's begin has grown by at most ahead_tokens since
 * the plan (begin is read again by every attention call; the page-table entries
 * of the tokens to come must already be in place: they are validated here, and
 * a table too short for begin + q + ahead_tokens is MC_ERR_RANGE at the check).
 * Work is still cut and ordered for the lengths at planning time.
 * ahead_tokens < 0 or > 2^20: MC_ERR_RANGE. */
mc_status mc_attn_plan_ahead(const mc_pool_desc* pool, int32_t num_q_heads, int32_t batch,
                             int32_t total_q, const int32_t* cu_q, const int32_t* begin,
                             const int32_t* page_table, const int32_t* cu_pages,
                             int32_t ahead_tokens, void* workspace /* device */,
                             size_t workspace_bytes, void* stream);
/* Synchronises `stream` and reports what the plan kernel found: MC_OK, or
 * MC_ERR_RANGE if an offset array is not monotone, a sequence's table is too
 * short for begin+q tokens, or a page id is outside the pool (then the work
 * list is empty and attention writes nothing).  The only call here that blocks. */
mc_status mc_attn_plan_check(const void* workspace /* device */, void* stream);
mc_status mc_prefix_prefill_attn(const mc_pool_desc* pool, int32_t layer,
                                 const void* q /* device [total_q][Hq][D] */,
                                 int32_t num_q_heads, int32_t batch, int32_t total_q,
                                 const int32_t* cu_q, const int32_t* begin,
                                 const int32_t* page_table, const int32_t* cu_pages,
                                 float sm_scale /* 0 -> 1/sqrt(D) */,
                                 void* out /* device [total_q][Hq][D], pool dtype */,
                                 float* lse /* device [total_q][Hq] */,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory and so cannot bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  mc_attn_plan followed by mc_prefix_prefill_attn with the same
 * arguments and results, the workspace being an 8 MiB array inside the library
 * (one copy per GPU the library has run on, held until the process ends).  The
 * call allocates nothing and does not synchronise.
 *   - Limit: the work list of the batch must fit the array - MC_ERR_RANGE, nothing
 *     launched, for batches beyond about 80000 q tiles; the room left over holds
 *     partial results, so KV ranges are cut into fewer chunks than with a full
 *     workspace (the results agree within the rounding of the merge).
 *   - There is no blocking check: malformed offsets, short tables or page ids
 *     outside the pool leave out and lse unwritten, as after a failed plan.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time
 *     on one GPU (different streams, different host threads) race.  Calls on one
 *     stream, one after the other, are fine; nothing needs clearing in between. */
mc_status mc_prefix_prefill_attn_noalloc(const mc_pool_desc* pool, int32_t layer,
                                         const void* q /* device [total_q][Hq][D] */,
                                         int32_t num_q_heads, int32_t batch, int32_t total_q,
                                         const int32_t* cu_q, const int32_t* begin,
                                         const int32_t* page_table, const int32_t* cu_pages,
                                         float sm_scale /* 0 -> 1/sqrt(D) */,
                                         void* out /* device [total_q][Hq][D], pool dtype */,
                                         float* lse /* device [total_q][Hq] */, void* stream);

/* ---- transfer payload: pages <-> contiguous buffer -------------------------
 * (sender and receiver side of remote_send: KV of prompt[begin:end] goes to the
 * page/slot entries reserved by prep_recv, Sec. 3.1, Sec. 3.2 Example 2; a
 * layer's KV can go as soon as the layer is done, Sec. 3.6, hence layer-major.)
 * pages: device int32 table of ONE sequence, n_table_pages entries, must cover
 * token s1-1 (MC_ERR_RANGE otherwise).  Tokens [s0,s1), layers
 * [layer_begin, layer_end).  pack reads only those slots and writes only
 * sendbuf; unpack reads only sendbuf and writes only those slots.
 * s0 == s1 or layer_begin == layer_end: MC_OK, nothing is launched. */
mc_status mc_kv_pack_range(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                           const int32_t* pages /* device */, int32_t n_table_pages, int32_t s0,
                           int32_t s1, void* sendbuf /* device, 16-byte aligned */, void* stream);
mc_status mc_kv_unpack_range(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                             const int32_t* pages /* device */, int32_t n_table_pages, int32_t s0,
                             int32_t s1, const void* sendbuf /* device */, void* stream);

/* Batched form of the two calls above: one launch moves the ranges of `batch` sequences.
 * Sequence s owns table
 * entries [cu_pages[s], cu_pages[s+1]) of page_table, tokens [s0[s], s1[s]) and the buffer
 * slice starting buf_offset[s] bytes into sendbuf (a multiple of 16; layout
 * [layer - layer_begin][2][token - s0[s]][kv_head][D] as above; slices must not overlap).
 * All five arrays are device memory; buf_offset is int64.  max_range_pages (host) is the
 * largest number of table entries any range touches, (s1-1)/16 - s0/16 + 1; it sizes the
 * launch, pages beyond it are not moved.  A sequence whose entries are malformed (empty or
 * reversed range, negative or misaligned offset, table too short, page id outside the pool)
 * is skipped in whole or in part, never read or written out of bounds.  The result for each
 * sequence equals that of the single-sequence call. */
mc_status mc_kv_pack_batch(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                           int32_t batch, const int32_t* page_table /* device */,
                           const int32_t* cu_pages /* device [batch+1] */,
                           const int32_t* s0 /* device [batch] */,
                           const int32_t* s1 /* device [batch] */,
                           const int64_t* buf_offset /* device [batch] */,
                           int32_t max_range_pages, void* sendbuf /* device */, void* stream);
mc_status mc_kv_unpack_batch(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                             int32_t batch, const int32_t* page_table /* device */,
                             const int32_t* cu_pages /* device [batch+1] */,
                             const int32_t* s0 /* device [batch] */,
                             const int32_t* s1 /* device [batch] */,
                             const int64_t* buf_offset /* device [batch] */,
                             int32_t max_range_pages, const void* sendbuf /* device */,
                             void* stream);

/* ---- fork_sequence (Sec. 3.5) -------------------------------------------------
 * A new sequence that continues the first n_tokens tokens of a parent.  Its page
 * table lists the parent's whole pages (shared, read-only for both from now on:
 * attention and pack may read shared pages, Sec. 3.4) and, if n_tokens is not a
 * multiple of 16, a fresh page for the partly filled last one, because each of
 * the two sequences goes on appending at slot n_tokens % 16.
 * mc_kv_fork_sequence (host): child_pages_out[0, ceil(n_tokens/16)) and the copy
 * that is still to be made: slots [0, *copy_slots_out) of page *copy_src_out to
 * page *copy_dst_out in every layer (-1, -1, 0 when no copy is needed).
 * MC_ERR_NO_PAGES changes nothing.  The allocator does not count references:
 * freeing a shared page while another sequence lists it is the caller's error.
 * mc_kv_copy_page (device, asynchronous on stream): that copy, for layers
 * [layer_begin, layer_end); no other byte of the pool is written.  Page ids
 * outside the pool, slots outside [0, 16]: MC_ERR_RANGE; src == dst: MC_ERR_ALIAS. */
mc_status mc_kv_fork_sequence(void* alloc, const int32_t* parent_pages /* host */,
                              int32_t n_tokens, int32_t* child_pages_out /* host */,
                              int32_t* copy_src_out, int32_t* copy_dst_out,
                              int32_t* copy_slots_out);
mc_status mc_kv_copy_page(const mc_pool_desc* pool, int32_t layer_begin, int32_t layer_end,
                          int32_t src_page, int32_t dst_page, int32_t slots, void* stream);

/* ---- host arithmetic of remote_send ------------------------------------------
 * Which token ranges a sender copies, computes and sends (Sec. 3.5, the two
 * prefix-matching cases of the attention/transfer interface).  The sender's
 * cache holds prompt[0, sender_match), the receiver's prompt[0, receiver_match)
 * (what its prep_recv matched, Sec. 3.2); remote_send(begin, end) has to leave
 * prompt[begin, end) on the receiver.  With need = [max(begin, receiver_match), end):
 *   copy    = the part of need the sender has cached: sent as it is
 *             (Case 1, sender matched more than the receiver);
 *   prefill = [sender_match, end) if need reaches past the sender's cache: the
 *             sender computes every token it has not cached (attention needs the
 *             whole context), also below need (Case 2, receiver matched more);
 *   send    = the part of need inside the prefilled range: sent once computed.
 * Empty ranges have begin == end.  All arguments are token counts, >= 0, and
 * begin <= end, else MC_ERR_RANGE; plan NULL is MC_ERR_INVALID.  Host only. */
typedef struct {
  int32_t copy_begin, copy_end;
  int32_t prefill_begin, prefill_end;
  int32_t send_begin, send_end;
} mc_send_plan;
mc_status mc_plan_remote_send(int32_t sender_match, int32_t receiver_match, int32_t begin,
                              int32_t end, mc_send_plan* plan /* host */);

/* The "compressed form" in which prep_recv returns the addresses of the entries
 * it reserved (Sec. 3.1): a page list as runs of consecutive page ids,
 * runs[2 i] = first page, runs[2 i + 1] = count.  mc_addr_compress writes at
 * most n runs (runs_out holds 2 n int32) and their number; mc_addr_expand
 * writes the page list back (capacity = room in pages_out; MC_ERR_RANGE if the
 * runs hold more pages, a count is <= 0 or a page id is negative).  Host only;
 * n == 0 is legal; null pointers with n > 0 are MC_ERR_INVALID. */
mc_status mc_addr_compress(const int32_t* pages /* host */, int32_t n,
                           int32_t* runs_out /* host [2 n] */, int32_t* n_runs_out);
mc_status mc_addr_expand(const int32_t* runs /* host [2 n_runs] */, int32_t n_runs,
                         int32_t* pages_out /* host */, int32_t capacity, int32_t* n_out);

/* ---- context cache index behind prep_recv ------------------------------------
 * prep_recv looks the prompt up in the engine's context cache and reports how long
 * a prefix of it is already there (match_len; Sec. 3.1, Sec. 3.2 Example 3).
 * The index records which page holds the KV of which 16-token block of which
 * token prefix: a trie over whole pages (a block is shared only if every token
 * before it is the same, and a partly filled last page is never shared, since
 * the sequence that owns it still appends to it).  Host only, not thread-safe.
 * The index does not own pages: freeing, eviction and reference counts of
 * shared pages are the caller's.
 *   insert: the KV of tokens[0, n_tokens) lives in pages[0, n_tokens / 16)
 *           (whole pages only; a block that is already recorded keeps its page).
 *   match:  the longest recorded prefix of whole pages of tokens[0, n_tokens):
 *           *match_len_out tokens (a multiple of 16), their pages in
 *           pages_out[0, match_len / 16) (room for n_tokens / 16 entries).
 *   mc_prep_recv(prompt, end): match prompt[0, end), then take pages for the rest
 *           from the allocator: pages_out[0, ceil(end / 16)) = the matched pages
 *           followed by fresh ones; MC_ERR_NO_PAGES changes nothing.
 * Null handles or pointers (with n > 0) are MC_ERR_INVALID, negative counts
 * MC_ERR_RANGE, a negative page id in insert MC_ERR_RANGE. */
mc_status mc_prefix_index_create(void** index_out /* host */);
mc_status mc_prefix_index_destroy(void* index);
mc_status mc_prefix_index_insert(void* index, const int32_t* tokens /* host */, int32_t n_tokens,
                                 const int32_t* pages /* host */);
mc_status mc_prefix_index_match(void* index, const int32_t* tokens /* host */, int32_t n_tokens,
                                int32_t* pages_out /* host */, int32_t* match_len_out);
mc_status mc_prep_recv(void* index, void* alloc, const int32_t* prompt /* host */, int32_t end,
                       int32_t* pages_out /* host */, int32_t* match_len_out);

#ifdef __cplusplus
}
#endif
#endif /* MC_KV_H_ */
