// Exercises the CPU oracle (oracle/mc_oracle.c) and the host half of the library
// (csrc/mc_host.hip: allocator, table check, send-range planner, address runs, prefix index,
// prep_recv, fork_sequence) in one executable built with -fsanitize=address,undefined.
// Random traffic with results cross-checked between the two allocators and against simple
// models; any sanitizer report or failed check ends the run with a non-zero status.
// Built and run by tests/test_sanitize_host.py; touches no GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "mc_kv.h"

extern "C" {
typedef struct {
  int32_t num_layers, num_pages, page_size, num_kv_heads, head_dim;
  int32_t dtype;
} orc_shape;
typedef struct orc_alloc orc_alloc;
double orc_decode(uint16_t bits, int32_t dtype);
int orc_gather_kv(const uint16_t* pool, const orc_shape* s, int32_t layer, const int32_t* pages,
                  int32_t n, double* k_full, double* v_full);
int orc_attention_rows(const uint16_t* pool, const orc_shape* s, int32_t layer,
                       const int32_t* pages, const uint16_t* q, int32_t num_q_heads, int32_t begin,
                       int32_t end, double scale, int64_t n_sel, const int32_t* sel_row,
                       const int32_t* sel_head, double* out, double* lse);
void orc_lse_merge(const double* o1, const double* l1, const double* o2, const double* l2, int64_t n,
                   int32_t D, double* o, double* l);
int orc_append(uint16_t* pool, const orc_shape* s, int32_t layer, const uint16_t* k_new,
               const uint16_t* v_new, int32_t q_len, int32_t begin, const int32_t* pages);
int orc_pack(const uint16_t* pool, const orc_shape* s, int32_t layer_begin, int32_t layer_end,
             const int32_t* pages, int32_t s0, int32_t s1, uint16_t* buf);
int orc_unpack(uint16_t* pool, const orc_shape* s, int32_t layer_begin, int32_t layer_end,
               const int32_t* pages, int32_t s0, int32_t s1, const uint16_t* buf);
orc_alloc* orc_alloc_create(int32_t num_pages);
void orc_alloc_destroy(orc_alloc* a);
int32_t orc_alloc_num_free(const orc_alloc* a);
int orc_alloc_take(orc_alloc* a, int32_t n, int32_t* pages_out);
int orc_alloc_give(orc_alloc* a, int32_t n, const int32_t* pages);
}

#define CHECK(c)                                                              \
  do {                                                                        \
    if (!(c)) {                                                               \
      std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c);    \
      std::exit(1);                                                           \
    }                                                                         \
  } while (0)

static std::mt19937 rng(12345);
static int rnd(int lo, int hi) { return lo + (int)(rng() % (uint32_t)(hi - lo + 1)); }

static void allocators() {
  for (int num_pages : {0, 1, 5, 64, 777}) {
    void* a = nullptr;
    CHECK(mc_kv_allocator_create(num_pages, &a) == MC_OK);
    orc_alloc* o = orc_alloc_create(num_pages);
    std::vector<int32_t> held;
    for (int it = 0; it < 400; ++it) {
      if (held.empty() || rnd(0, 99) < 55) {
        const int n = rnd(0, num_pages / 3 + 2);
        std::vector<int32_t> got(n + 1), ref(n + 1);
        const int rc = orc_alloc_take(o, n, ref.data());
        const mc_status st = mc_kv_alloc_pages(a, n, got.data());
        CHECK((rc == 0) == (st == MC_OK));
        if (st != MC_OK) CHECK(st == MC_ERR_NO_PAGES);
        else {
          CHECK(std::memcmp(got.data(), ref.data(), sizeof(int32_t) * n) == 0);
          held.insert(held.end(), got.begin(), got.begin() + n);
        }
      } else {
        const int k = rnd(1, (int)held.size());
        std::vector<int32_t> give;
        for (int i = 0; i < k; ++i) {
          const int j = rnd(0, (int)held.size() - 1);
          give.push_back(held[j]);
          held.erase(held.begin() + j);
        }
        CHECK(orc_alloc_give(o, k, give.data()) == 0);
        CHECK(mc_kv_free_pages(a, k, give.data()) == MC_OK);
        // a second free of the same pages is refused and changes nothing
        CHECK(mc_kv_free_pages(a, k, give.data()) == MC_ERR_INVALID);
      }
      int32_t nf = -1;
      CHECK(mc_kv_allocator_num_free(a, &nf) == MC_OK && nf == orc_alloc_num_free(o));
    }
    const int32_t bad[2] = {-1, num_pages};
    CHECK(mc_kv_free_pages(a, 2, bad) == MC_ERR_INVALID);
    CHECK(mc_kv_allocator_destroy(a) == MC_OK);
    orc_alloc_destroy(o);
  }
  const int32_t dup[3] = {1, 2, 1}, out[2] = {0, 9};
  CHECK(mc_kv_check_page_table(dup, 3, 4) == MC_ERR_ALIAS);
  CHECK(mc_kv_check_page_table(out, 2, 4) == MC_ERR_RANGE);
  CHECK(mc_kv_check_page_table(out, 1, 4) == MC_OK);
  CHECK(mc_kv_check_page_table(nullptr, 0, 4) == MC_OK);
}

static void send_ranges_and_runs() {
  for (int sm = 0; sm <= 12; ++sm)
    for (int rm = 0; rm <= 12; ++rm)
      for (int b = 0; b <= 12; ++b)
        for (int e = b; e <= 12; ++e) {
          mc_send_plan p;
          CHECK(mc_plan_remote_send(sm, rm, b, e, &p) == MC_OK);
          // token by token: what the receiver lacks is sent, from the cache or once computed
          for (int t = 0; t < 13; ++t) {
            const bool need = t >= b && t < e && t >= rm;
            const bool copied = t >= p.copy_begin && t < p.copy_end;
            const bool sent = t >= p.send_begin && t < p.send_end;
            CHECK(need == (copied || sent) && !(copied && sent));
            if (copied) CHECK(t < sm);
            if (sent) CHECK(t >= sm && t >= p.prefill_begin && t < p.prefill_end);
          }
        }
  CHECK(mc_plan_remote_send(0, 0, 3, 2, nullptr) != MC_OK);
  for (int it = 0; it < 300; ++it) {
    const int n = rnd(0, 40);
    std::vector<int32_t> pages(n + 1), runs(2 * n + 2), back(n + 1);
    int next = rnd(0, 50);
    for (int i = 0; i < n; ++i) {
      pages[i] = next;
      next = rnd(0, 3) ? next + 1 : rnd(0, 1000);
    }
    int32_t nr = -1, nb = -1;
    CHECK(mc_addr_compress(pages.data(), n, runs.data(), &nr) == MC_OK && nr <= n);
    CHECK(mc_addr_expand(runs.data(), nr, back.data(), n, &nb) == MC_OK && nb == n);
    CHECK(std::memcmp(pages.data(), back.data(), sizeof(int32_t) * n) == 0);
    if (n > 0) CHECK(mc_addr_expand(runs.data(), nr, back.data(), n - 1, &nb) == MC_ERR_RANGE);
  }
}

static void prefix_index_and_forks() {
  void *ix = nullptr, *al = nullptr;
  CHECK(mc_prefix_index_create(&ix) == MC_OK && mc_kv_allocator_create(256, &al) == MC_OK);
  std::vector<std::vector<int32_t>> prompts;
  for (int it = 0; it < 120; ++it) {
    // a new prompt: a prefix of an old one (if any) plus fresh tokens
    std::vector<int32_t> p;
    if (!prompts.empty() && rnd(0, 2)) {
      const auto& src = prompts[rnd(0, (int)prompts.size() - 1)];
      p.assign(src.begin(), src.begin() + rnd(0, (int)src.size()));
    }
    const int extra = rnd(0, 70);
    for (int i = 0; i < extra; ++i) p.push_back(rnd(0, 3));
    const int end = (int)p.size();
    std::vector<int32_t> pages(end / 16 + 2), again(end / 16 + 2);
    int32_t match = -1, match2 = -1, nf0 = 0, nf1 = 0;
    CHECK(mc_kv_allocator_num_free(al, &nf0) == MC_OK);
    const mc_status st = mc_prep_recv(ix, al, p.data(), end, pages.data(), &match);
    CHECK(mc_kv_allocator_num_free(al, &nf1) == MC_OK);
    if (st == MC_ERR_NO_PAGES) { CHECK(nf0 == nf1); continue; }
    CHECK(st == MC_OK && match % 16 == 0 && match <= end);
    CHECK(nf0 - nf1 == (end + 15) / 16 - match / 16);
    CHECK(mc_prefix_index_insert(ix, p.data(), end, pages.data()) == MC_OK);
    CHECK(mc_prefix_index_match(ix, p.data(), end, again.data(), &match2) == MC_OK);
    CHECK(match2 == end / 16 * 16);
    CHECK(std::memcmp(again.data(), pages.data(), sizeof(int32_t) * (match / 16)) == 0);
    prompts.push_back(p);
    // fork at a random length: whole pages shared, a fresh page for a partly filled one
    const int nt = rnd(0, end);
    std::vector<int32_t> child(nt / 16 + 2);
    int32_t src = -2, dst = -2, slots = -2;
    const mc_status fs = mc_kv_fork_sequence(al, pages.data(), nt, child.data(), &src, &dst, &slots);
    if (fs == MC_OK) {
      CHECK(std::memcmp(child.data(), pages.data(), sizeof(int32_t) * (nt / 16)) == 0);
      if (nt % 16) CHECK(src == pages[nt / 16] && dst == child[nt / 16] && slots == nt % 16 && dst != src);
      else CHECK(src == -1 && dst == -1 && slots == 0);
    } else {
      CHECK(fs == MC_ERR_NO_PAGES);
    }
  }
  CHECK(mc_prefix_index_destroy(ix) == MC_OK && mc_kv_allocator_destroy(al) == MC_OK);
}

static void oracle_paths() {
  for (int dtype = 0; dtype < 2; ++dtype) {
    const orc_shape s = {2, 9, 16, 2, 128, dtype};
    const int64_t page_elems = 2ll * s.num_kv_heads * 16 * 128;
    std::vector<uint16_t> pool(s.num_layers * s.num_pages * page_elems), pool_b(pool.size());
    for (auto& x : pool) x = (uint16_t)(0x3c00 + rnd(-40, 40));   // finite values near 1
    const int n = 70, b = 21, Hq = 4;
    const int32_t pages[5] = {7, 0, 3, 8, 5}, pages_b[5] = {1, 2, 6, 4, 0};
    std::vector<uint16_t> k(n * s.num_kv_heads * 128), v(k.size()), q((n - b) * Hq * 128);
    for (auto* t : {&k, &v, &q})
      for (auto& x : *t) x = (uint16_t)((dtype ? 0x3f80 : 0x3c00) + rnd(-60, 60) + (rnd(0, 1) << 15));
    CHECK(orc_append(pool.data(), &s, 1, k.data(), v.data(), b, 0, pages) == 0);
    CHECK(orc_append(pool.data(), &s, 1, k.data() + (size_t)b * s.num_kv_heads * 128,
                     v.data() + (size_t)b * s.num_kv_heads * 128, n - b, b, pages) == 0);
    std::vector<double> kf((size_t)n * s.num_kv_heads * 128), vf(kf.size());
    CHECK(orc_gather_kv(pool.data(), &s, 1, pages, n, kf.data(), vf.data()) == 0);
    for (size_t i = 0; i < kf.size(); ++i) CHECK(kf[i] == orc_decode(k[i], dtype));
    // all rows and heads, then the same through a selection; LSE merge of two halves of a row
    std::vector<int32_t> rows, heads;
    for (int r = 0; r < n - b; ++r)
      for (int h = 0; h < Hq; ++h) { rows.push_back(r); heads.push_back(h); }
    std::vector<double> o(rows.size() * 128), l(rows.size());
    CHECK(orc_attention_rows(pool.data(), &s, 1, pages, q.data(), Hq, b, n, 0.0883883, (int64_t)rows.size(),
                             rows.data(), heads.data(), o.data(), l.data()) == 0);
    for (double x : l) CHECK(x == x);
    std::vector<double> om(128), lm(1);
    orc_lse_merge(o.data(), l.data(), o.data() + 128, l.data() + 1, 1, 128, om.data(), lm.data());
    CHECK(lm[0] >= l[0] && lm[0] >= l[1]);
    // token-granular pack / unpack round trip into other pages of a second pool
    const int s0 = 13, s1 = 66;
    std::vector<uint16_t> buf((size_t)2 * 2 * (s1 - s0) * s.num_kv_heads * 128);
    CHECK(orc_pack(pool.data(), &s, 0, 2, pages, s0, s1, buf.data()) == 0);
    CHECK(orc_unpack(pool_b.data(), &s, 0, 2, pages_b, s0, s1, buf.data()) == 0);
    std::vector<uint16_t> buf2(buf.size());
    CHECK(orc_pack(pool_b.data(), &s, 0, 2, pages_b, s0, s1, buf2.data()) == 0);
    CHECK(buf == buf2);
  }
}

int main() {
  allocators();
  send_ranges_and_runs();
  prefix_index_and_forks();
  oracle_paths();
  CHECK(std::strcmp(mc_status_string(0), "MC_OK") == 0 && mc_abi_version() == 2);
  std::puts("host sanitize run ok");
  return 0;
}
