// Host-only parts of the library: status names, the page allocator behind
// prep_recv (paper Sec. 3.1: the receiver reserves entries for the part of the prompt it
// does not hold), and a host check of destination page tables.
#include <algorithm>
#include <array>
#include <map>
#include <new>
#include <utility>
#include <vector>

#include "mc_common.h"

namespace {

struct Allocator {
  int32_t num_pages;
  std::vector<int32_t> free_stack;  // back() is handed out next
  std::vector<uint8_t> state;       // 0 free, 1 handed out, 2 = seen earlier in this free call
};

// Trie over 16-token blocks: (parent node, the block's tokens) -> node; a node knows its page.
struct PrefixIndex {
  typedef std::pair<int32_t, std::array<int32_t, mc::kPage>> Key;
  std::map<Key, int32_t> child;
  std::vector<int32_t> page_of;   // by node id

  static Key key(int32_t parent, const int32_t* block) {
    Key k;
    k.first = parent;
    std::copy(block, block + mc::kPage, k.second.begin());
    return k;
  }
  // whole pages of tokens[0, n) found: their pages go to pages_out (if given)
  int32_t match(const int32_t* tokens, int32_t n, int32_t* pages_out) const {
    int32_t node = -1, blocks = 0;
    for (; (blocks + 1) * mc::kPage <= n; ++blocks) {
      auto it = child.find(key(node, tokens + blocks * mc::kPage));
      if (it == child.end()) break;
      node = it->second;
      if (pages_out) pages_out[blocks] = page_of[node];
    }
    return blocks;
  }
};

}  // namespace

extern "C" {

const char* mc_status_string(int32_t status) {
  switch (status) {
    case MC_OK: return "MC_OK";
    case MC_ERR_INVALID: return "MC_ERR_INVALID";
    case MC_ERR_NO_PAGES: return "MC_ERR_NO_PAGES";
    case MC_ERR_RANGE: return "MC_ERR_RANGE";
    case MC_ERR_ALIAS: return "MC_ERR_ALIAS";
    case MC_ERR_UNSUPPORTED: return "MC_ERR_UNSUPPORTED";
    case MC_ERR_HIP: return "MC_ERR_HIP";
    default: return "MC_ERR_UNKNOWN";
  }
}

int32_t mc_abi_version(void) { return 2; }

mc_status mc_kv_allocator_create(int32_t num_pages, void** alloc_out) {
  if (!alloc_out || num_pages < 0) return MC_ERR_INVALID;
  Allocator* a = new (std::nothrow) Allocator();
  if (!a) return MC_ERR_INVALID;
  a->num_pages = num_pages;
  a->free_stack.resize(num_pages);
  for (int32_t i = 0; i < num_pages; ++i) a->free_stack[i] = num_pages - 1 - i;
  a->state.assign(num_pages, 0);
  *alloc_out = a;
  return MC_OK;
}

mc_status mc_kv_allocator_destroy(void* alloc) {
  if (!alloc) return MC_ERR_INVALID;
  delete static_cast<Allocator*>(alloc);
  return MC_OK;
}

mc_status mc_kv_alloc_pages(void* alloc, int32_t n, int32_t* pages_out) {
  Allocator* a = static_cast<Allocator*>(alloc);
  if (!a || n < 0 || (n > 0 && !pages_out)) return MC_ERR_INVALID;
  if (static_cast<size_t>(n) > a->free_stack.size()) return MC_ERR_NO_PAGES;
  for (int32_t i = 0; i < n; ++i) {
    int32_t p = a->free_stack.back();
    a->free_stack.pop_back();
    a->state[p] = 1;
    pages_out[i] = p;
  }
  return MC_OK;
}

mc_status mc_kv_free_pages(void* alloc, int32_t n, const int32_t* pages) {
  Allocator* a = static_cast<Allocator*>(alloc);
  if (!a || n < 0 || (n > 0 && !pages)) return MC_ERR_INVALID;
  int32_t seen = 0;
  bool bad = false;
  for (; seen < n; ++seen) {
    int32_t p = pages[seen];
    if (p < 0 || p >= a->num_pages || a->state[p] != 1) { bad = true; break; }
    a->state[p] = 2;
  }
  if (bad) {
    for (int32_t i = 0; i < seen; ++i) a->state[pages[i]] = 1;
    return MC_ERR_INVALID;
  }
  for (int32_t i = 0; i < n; ++i) {
    a->state[pages[i]] = 0;
    a->free_stack.push_back(pages[i]);
  }
  return MC_OK;
}

mc_status mc_kv_allocator_num_free(void* alloc, int32_t* num_free_out) {
  Allocator* a = static_cast<Allocator*>(alloc);
  if (!a || !num_free_out) return MC_ERR_INVALID;
  *num_free_out = static_cast<int32_t>(a->free_stack.size());
  return MC_OK;
}

mc_status mc_kv_check_page_table(const int32_t* pages, int64_t n, int32_t num_pages) {
  if (n < 0 || num_pages < 0 || (n > 0 && !pages)) return MC_ERR_INVALID;
  std::vector<uint8_t> seen(static_cast<size_t>(num_pages), 0);
  for (int64_t i = 0; i < n; ++i) {
    if (pages[i] < 0 || pages[i] >= num_pages) return MC_ERR_RANGE;
    if (seen[pages[i]]) return MC_ERR_ALIAS;
    seen[pages[i]] = 1;
  }
  return MC_OK;
}

mc_status mc_plan_remote_send(int32_t sender_match, int32_t receiver_match, int32_t begin,
                              int32_t end, mc_send_plan* plan) {
  if (!plan) return MC_ERR_INVALID;
  if (sender_match < 0 || receiver_match < 0 || begin < 0 || end < begin) return MC_ERR_RANGE;
  const int32_t need_begin = std::min(std::max(begin, receiver_match), end);   // need = [., end)
  const int32_t cached_end = std::min(sender_match, end);
  plan->copy_begin = std::min(need_begin, cached_end);
  plan->copy_end = cached_end;
  if (plan->copy_begin == plan->copy_end) plan->copy_begin = plan->copy_end = need_begin;
  const bool past_cache = need_begin < end && sender_match < end;   // need reaches uncached tokens
  plan->prefill_begin = past_cache ? sender_match : end;
  plan->prefill_end = end;
  plan->send_begin = past_cache ? std::max(need_begin, sender_match) : end;
  plan->send_end = end;
  return MC_OK;
}

mc_status mc_addr_compress(const int32_t* pages, int32_t n, int32_t* runs_out,
                           int32_t* n_runs_out) {
  if (n < 0 || !n_runs_out || (n > 0 && (!pages || !runs_out))) return MC_ERR_INVALID;
  int32_t r = 0;
  for (int32_t i = 0; i < n; ++i) {
    if (pages[i] < 0) return MC_ERR_RANGE;
    if (r > 0 && runs_out[2 * r - 2] + runs_out[2 * r - 1] == pages[i]) {
      ++runs_out[2 * r - 1];
    } else {
      runs_out[2 * r] = pages[i];
      runs_out[2 * r + 1] = 1;
      ++r;
    }
  }
  *n_runs_out = r;
  return MC_OK;
}

mc_status mc_addr_expand(const int32_t* runs, int32_t n_runs, int32_t* pages_out, int32_t capacity,
                         int32_t* n_out) {
  if (n_runs < 0 || capacity < 0 || !n_out || (n_runs > 0 && !runs) ||
      (capacity > 0 && !pages_out))
    return MC_ERR_INVALID;
  int64_t n = 0;
  for (int32_t i = 0; i < n_runs; ++i) {
    const int32_t first = runs[2 * i], count = runs[2 * i + 1];
    if (first < 0 || count <= 0 || (int64_t)first + count - 1 > 0x7fffffffll) return MC_ERR_RANGE;
    if (n + count > capacity) return MC_ERR_RANGE;
    for (int32_t k = 0; k < count; ++k) pages_out[n + k] = first + k;
    n += count;
  }
  *n_out = (int32_t)n;
  return MC_OK;
}

mc_status mc_prefix_index_create(void** index_out) {
  if (!index_out) return MC_ERR_INVALID;
  PrefixIndex* x = new (std::nothrow) PrefixIndex();
  if (!x) return MC_ERR_INVALID;
  *index_out = x;
  return MC_OK;
}

mc_status mc_prefix_index_destroy(void* index) {
  if (!index) return MC_ERR_INVALID;
  delete static_cast<PrefixIndex*>(index);
  return MC_OK;
}

mc_status mc_prefix_index_insert(void* index, const int32_t* tokens, int32_t n_tokens,
                                 const int32_t* pages) {
  PrefixIndex* x = static_cast<PrefixIndex*>(index);
  if (!x) return MC_ERR_INVALID;
  if (n_tokens < 0) return MC_ERR_RANGE;
  const int32_t blocks = n_tokens / mc::kPage;
  if (blocks > 0 && (!tokens || !pages)) return MC_ERR_INVALID;
  for (int32_t b = 0; b < blocks; ++b)
    if (pages[b] < 0) return MC_ERR_RANGE;
  int32_t node = -1;
  for (int32_t b = 0; b < blocks; ++b) {
    const PrefixIndex::Key k = PrefixIndex::key(node, tokens + b * mc::kPage);
    auto it = x->child.find(k);
    if (it == x->child.end()) {
      x->page_of.push_back(pages[b]);
      it = x->child.emplace(k, (int32_t)x->page_of.size() - 1).first;
    }
    node = it->second;
  }
  return MC_OK;
}

mc_status mc_prefix_index_match(void* index, const int32_t* tokens, int32_t n_tokens,
                                int32_t* pages_out, int32_t* match_len_out) {
  const PrefixIndex* x = static_cast<const PrefixIndex*>(index);
  if (!x || !match_len_out) return MC_ERR_INVALID;
  if (n_tokens < 0) return MC_ERR_RANGE;
  if (n_tokens >= mc::kPage && (!tokens || !pages_out)) return MC_ERR_INVALID;
  *match_len_out = x->match(tokens, n_tokens, pages_out) * mc::kPage;
  return MC_OK;
}

mc_status mc_prep_recv(void* index, void* alloc, const int32_t* prompt, int32_t end,
                       int32_t* pages_out, int32_t* match_len_out) {
  const PrefixIndex* x = static_cast<const PrefixIndex*>(index);
  if (!x || !alloc || !match_len_out) return MC_ERR_INVALID;
  if (end < 0) return MC_ERR_RANGE;
  if (end > 0 && (!prompt || !pages_out)) return MC_ERR_INVALID;
  const int32_t total = (end + mc::kPage - 1) / mc::kPage;
  std::vector<int32_t> matched(static_cast<size_t>(end / mc::kPage));
  const int32_t m = x->match(prompt, end, matched.data());
  mc_status st = mc_kv_alloc_pages(alloc, total - m, pages_out + m);   // all or nothing
  if (st != MC_OK) return st;
  std::copy(matched.begin(), matched.begin() + m, pages_out);
  *match_len_out = m * mc::kPage;
  return MC_OK;
}

mc_status mc_kv_fork_sequence(void* alloc, const int32_t* parent_pages, int32_t n_tokens,
                              int32_t* child_pages_out, int32_t* copy_src_out,
                              int32_t* copy_dst_out, int32_t* copy_slots_out) {
  if (!alloc || !copy_src_out || !copy_dst_out || !copy_slots_out) return MC_ERR_INVALID;
  if (n_tokens < 0) return MC_ERR_RANGE;
  const int32_t whole = n_tokens / mc::kPage, rest = n_tokens % mc::kPage;
  if (n_tokens > 0 && (!parent_pages || !child_pages_out)) return MC_ERR_INVALID;
  *copy_src_out = *copy_dst_out = -1;
  *copy_slots_out = 0;
  if (rest) {   // the fork appends to a copy of the partly filled page, never to the parent's
    int32_t fresh;
    mc_status st = mc_kv_alloc_pages(alloc, 1, &fresh);
    if (st != MC_OK) return st;
    child_pages_out[whole] = fresh;
    *copy_src_out = parent_pages[whole];
    *copy_dst_out = fresh;
    *copy_slots_out = rest;
  }
  std::copy(parent_pages, parent_pages + whole, child_pages_out);
  return MC_OK;
}

}  // extern "C"
