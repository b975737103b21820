/*
 * mc_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, fp64 CPU statement of what the paged KV-cache hot path computes:
 * attention of a token range [begin,end) over the KV already held in pages
 * (paper Sec. 3.1: start_generate prefills prompt[begin:] over the cached
 * prompt[:begin]; Sec. 3.3: the decode engine continues with prompt[s:];
 * Sec. 3.4: attention(qkv_data) runs over the KV cache), the write of new KV
 * into (page, slot) entries (Sec. 3.1 remote_send: new KVs are materialised by
 * prefill), the gather/scatter of a token range between pages and a contiguous
 * transfer buffer (Sec. 3.2 Example 2: KV is written to page-index/slot-index
 * entries reserved by prep_recv), and the page allocator behind prep_recv.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use this
 * file.  It shares no code, header or table with the GPU library.
 *
 * Everything the paper leaves open (dtype, page layout, scale, LSE base) is a
 * reading of this build; the layouts are
 *   pool    [layer][page][2 (0=K,1=V)][kv_head][slot][head_dim]   2-byte elements
 *   q, out  [token][q_head][head_dim]
 *   k_new   [token][kv_head][head_dim]        (v_new likewise)
 *   sendbuf [layer - layer_begin][2][token - s0][kv_head][head_dim]
 * and softmax uses scale * q.k with natural-log LSE.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t num_layers, num_pages, page_size, num_kv_heads, head_dim;
  int32_t dtype; /* 0 = IEEE binary16, 1 = bfloat16 */
} orc_shape;

/* ---- exact 2-byte -> fp64 decode ---------------------------------------- */

static double orc_decode_f16(uint16_t b) {
  int sign = (b >> 15) & 1, ex = (b >> 10) & 0x1f, man = b & 0x3ff;
  double v;
  if (ex == 0) v = ldexp((double)man, -24);              /* subnormal / zero */
  else if (ex == 31) v = man ? NAN : INFINITY;
  else v = ldexp((double)(man | 0x400), ex - 25);
  return sign ? -v : v;
}

static double orc_decode_bf16(uint16_t b) {
  int sign = (b >> 15) & 1, ex = (b >> 7) & 0xff, man = b & 0x7f;
  double v;
  if (ex == 0) v = ldexp((double)man, -133);
  else if (ex == 255) v = man ? NAN : INFINITY;
  else v = ldexp((double)(man | 0x80), ex - 134);
  return sign ? -v : v;
}

double orc_decode(uint16_t bits, int32_t dtype) {
  return dtype == 0 ? orc_decode_f16(bits) : orc_decode_bf16(bits);
}

void orc_decode_array(const uint16_t* bits, int64_t n, int32_t dtype, double* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = orc_decode(bits[i], dtype);
}

/* element offset of pool[layer][page][kv][head][slot][0] */
static int64_t orc_off(const orc_shape* s, int64_t layer, int64_t page, int64_t kv,
                       int64_t head, int64_t slot) {
  return ((((layer * s->num_pages + page) * 2 + kv) * s->num_kv_heads + head) *
              s->page_size + slot) * (int64_t)s->head_dim;
}

/* ---- step 1: gather one sequence's K and V for tokens [0,n) as fp64 ------ */
/* k_full, v_full: [n][kv_head][head_dim] */
int orc_gather_kv(const uint16_t* pool, const orc_shape* s, int32_t layer,
                  const int32_t* pages, int32_t n, double* k_full, double* v_full) {
  const int P = s->page_size, H = s->num_kv_heads, D = s->head_dim;
  for (int j = 0; j < n; ++j) {
    int32_t page = pages[j / P];
    if (page < 0 || page >= s->num_pages) return 1;
    for (int h = 0; h < H; ++h)
      for (int d = 0; d < D; ++d) {
        k_full[((int64_t)j * H + h) * D + d] =
            orc_decode(pool[orc_off(s, layer, page, 0, h, j % P) + d], s->dtype);
        v_full[((int64_t)j * H + h) * D + d] =
            orc_decode(pool[orc_off(s, layer, page, 1, h, j % P) + d], s->dtype);
      }
  }
  return 0;
}

/* ---- steps 2-4: naive masked-softmax attention for chosen (row, head) ----
 * q:       [end-begin][num_q_heads][head_dim] 2-byte, row r is token begin+r
 * sel_row/sel_head: n_sel pairs to compute (row relative to begin).
 * out:     [n_sel][head_dim] fp64,  lse: [n_sel] fp64 (natural log).
 * Token i sees keys j in [0, i]: every cached token and the new tokens up to
 * and including itself. */
int orc_attention_rows(const uint16_t* pool, const orc_shape* s, int32_t layer,
                       const int32_t* pages, const uint16_t* q, int32_t num_q_heads,
                       int32_t begin, int32_t end, double scale, int64_t n_sel,
                       const int32_t* sel_row, const int32_t* sel_head, double* out,
                       double* lse) {
  const int H = s->num_kv_heads, D = s->head_dim;
  if (num_q_heads % H != 0 || begin < 0 || end < begin) return 1;
  const int G = num_q_heads / H;
  if (end == 0 || n_sel == 0) return 0;
  double* k_full = (double*)malloc(sizeof(double) * (size_t)end * H * D);
  double* v_full = (double*)malloc(sizeof(double) * (size_t)end * H * D);
  if (!k_full || !v_full) { free(k_full); free(v_full); return 2; }
  int rc = orc_gather_kv(pool, s, layer, pages, end, k_full, v_full);
  if (rc) { free(k_full); free(v_full); return rc; }

#pragma omp parallel
  {
    double* sc = (double*)malloc(sizeof(double) * (size_t)end);
    double* qd = (double*)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 4)
    for (int64_t t = 0; t < n_sel; ++t) {
      const int r = sel_row[t], h = sel_head[t], hk = h / G;
      const int i = begin + r; /* absolute position of this query token */
      for (int d = 0; d < D; ++d)
        qd[d] = orc_decode(q[((int64_t)r * num_q_heads + h) * D + d], s->dtype);
      double m = -INFINITY;
      for (int j = 0; j <= i; ++j) {
        const double* kj = k_full + ((int64_t)j * H + hk) * D;
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += qd[d] * kj[d];
        sc[j] = scale * acc;
        if (sc[j] > m) m = sc[j];
      }
      double z = 0.0;
      for (int j = 0; j <= i; ++j) { sc[j] = exp(sc[j] - m); z += sc[j]; }
      double* o = out + t * D;
      for (int d = 0; d < D; ++d) o[d] = 0.0;
      for (int j = 0; j <= i; ++j) {
        const double p = sc[j] / z;
        const double* vj = v_full + ((int64_t)j * H + hk) * D;
        for (int d = 0; d < D; ++d) o[d] += p * vj[d];
      }
      lse[t] = m + log(z);
    }
    free(sc);
    free(qd);
  }
  free(k_full);
  free(v_full);
  return 0;
}

/* ---- step 7: merge of two partial softmax results over disjoint key sets -- */
void orc_lse_merge(const double* o1, const double* l1, const double* o2, const double* l2,
                   int64_t n, int32_t D, double* o, double* l) {
  for (int64_t t = 0; t < n; ++t) {
    double mx = l1[t] > l2[t] ? l1[t] : l2[t];
    double L = mx + log(exp(l1[t] - mx) + exp(l2[t] - mx));
    double w1 = exp(l1[t] - L), w2 = exp(l2[t] - L);
    for (int d = 0; d < D; ++d) o[t * D + d] = w1 * o1[t * D + d] + w2 * o2[t * D + d];
    l[t] = L;
  }
}

/* ---- step 5: page copies (bytes only) ------------------------------------ */

/* write K/V of tokens [begin, begin+q_len) of one sequence into their slots */
int orc_append(uint16_t* pool, const orc_shape* s, int32_t layer, const uint16_t* k_new,
               const uint16_t* v_new, int32_t q_len, int32_t begin, const int32_t* pages) {
  const int P = s->page_size, H = s->num_kv_heads, D = s->head_dim;
  for (int t = 0; t < q_len; ++t) {
    const int pos = begin + t;
    const int32_t page = pages[pos / P];
    if (page < 0 || page >= s->num_pages) return 1;
    for (int h = 0; h < H; ++h) {
      memcpy(pool + orc_off(s, layer, page, 0, h, pos % P), k_new + ((int64_t)t * H + h) * D,
             sizeof(uint16_t) * D);
      memcpy(pool + orc_off(s, layer, page, 1, h, pos % P), v_new + ((int64_t)t * H + h) * D,
             sizeof(uint16_t) * D);
    }
  }
  return 0;
}

/* gather tokens [s0,s1), layers [layer_begin,layer_end) into the transfer buffer */
int orc_pack(const uint16_t* pool, const orc_shape* s, int32_t layer_begin, int32_t layer_end,
             const int32_t* pages, int32_t s0, int32_t s1, uint16_t* buf) {
  const int P = s->page_size, H = s->num_kv_heads, D = s->head_dim;
  const int64_t T = s1 - s0;
  for (int l = layer_begin; l < layer_end; ++l)
    for (int kv = 0; kv < 2; ++kv)
      for (int pos = s0; pos < s1; ++pos) {
        const int32_t page = pages[pos / P];
        if (page < 0 || page >= s->num_pages) return 1;
        for (int h = 0; h < H; ++h)
          memcpy(buf + ((((int64_t)(l - layer_begin) * 2 + kv) * T + (pos - s0)) * H + h) * D,
                 pool + orc_off(s, l, page, kv, h, pos % P), sizeof(uint16_t) * D);
      }
  return 0;
}

/* scatter the transfer buffer into the (page, slot) entries of tokens [s0,s1) */
int orc_unpack(uint16_t* pool, const orc_shape* s, int32_t layer_begin, int32_t layer_end,
               const int32_t* pages, int32_t s0, int32_t s1, const uint16_t* buf) {
  const int P = s->page_size, H = s->num_kv_heads, D = s->head_dim;
  const int64_t T = s1 - s0;
  for (int l = layer_begin; l < layer_end; ++l)
    for (int kv = 0; kv < 2; ++kv)
      for (int pos = s0; pos < s1; ++pos) {
        const int32_t page = pages[pos / P];
        if (page < 0 || page >= s->num_pages) return 1;
        for (int h = 0; h < H; ++h)
          memcpy(pool + orc_off(s, l, page, kv, h, pos % P),
                 buf + ((((int64_t)(l - layer_begin) * 2 + kv) * T + (pos - s0)) * H + h) * D,
                 sizeof(uint16_t) * D);
      }
  return 0;
}

/* ---- step 6: page allocator (last-in first-out free list) ---------------- */

typedef struct {
  int32_t num_pages, n_free;
  int32_t* stack;   /* stack[n_free-1] is handed out next */
  uint8_t* in_use;
} orc_alloc;

orc_alloc* orc_alloc_create(int32_t num_pages) {
  if (num_pages < 0) return NULL;
  orc_alloc* a = (orc_alloc*)malloc(sizeof(orc_alloc));
  a->num_pages = num_pages;
  a->n_free = num_pages;
  a->stack = (int32_t*)malloc(sizeof(int32_t) * (size_t)(num_pages ? num_pages : 1));
  a->in_use = (uint8_t*)calloc((size_t)(num_pages ? num_pages : 1), 1);
  for (int32_t i = 0; i < num_pages; ++i) a->stack[i] = num_pages - 1 - i; /* page 0 on top */
  return a;
}

void orc_alloc_destroy(orc_alloc* a) {
  if (!a) return;
  free(a->stack);
  free(a->in_use);
  free(a);
}

int32_t orc_alloc_num_free(const orc_alloc* a) { return a->n_free; }

/* all-or-nothing: 0 ok, 2 not enough pages (nothing taken), 1 bad argument */
int orc_alloc_take(orc_alloc* a, int32_t n, int32_t* pages_out) {
  if (n < 0) return 1;
  if (n > a->n_free) return 2;
  for (int32_t i = 0; i < n; ++i) {
    int32_t p = a->stack[--a->n_free];
    a->in_use[p] = 1;
    pages_out[i] = p;
  }
  return 0;
}

/* pages return to the free list in argument order; a page not handed out, out of
 * range, or listed twice is an error and then nothing is returned */
int orc_alloc_give(orc_alloc* a, int32_t n, const int32_t* pages) {
  if (n < 0) return 1;
  int32_t bad = 0, seen = 0;
  for (; seen < n; ++seen) {
    int32_t p = pages[seen];
    if (p < 0 || p >= a->num_pages || a->in_use[p] != 1) { bad = 1; break; }
    a->in_use[p] = 2; /* 2 = listed earlier in this very call */
  }
  if (bad) {
    for (int32_t i = 0; i < seen; ++i) a->in_use[pages[i]] = 1;
    return 1;
  }
  for (int32_t i = 0; i < n; ++i) {
    a->in_use[pages[i]] = 0;
    a->stack[a->n_free++] = pages[i];
  }
  return 0;
}
