// Host-side bookkeeping of the paged KV cache: free pages, reference counts, fork and
// copy-on-write (rules at marl_page_pool_* in marl_decode.h).  The samples of a prompt share its
// pages (Parallel Sampling, Section 5.1 of the paper) and diverge afterwards; the paper leaves
// the mechanism to its inference backend.  No GPU code in this file: the device work that a
// copy-on-write needs is marl_kv_copy_pages.
#include <new>
#include <vector>

#include "marl_decode.h"

struct marl_page_pool {
  std::vector<int32_t> count;      // per page: 0 = free
  std::vector<int32_t> free_stack; // top = back()
  std::vector<int32_t> scratch;    // per page, all zero between calls: occurrences inside one call

  bool valid(int32_t page) const { return page >= 0 && (size_t)page < count.size(); }
  int32_t take() {
    const int32_t page = free_stack.back();
    free_stack.pop_back();
    count[page] = 1;
    return page;
  }
  void unref(int32_t page) {
    if (--count[page] == 0) free_stack.push_back(page);
  }
  // every id valid and in use; for a release, no page listed more often than it is referenced
  bool check_list(const int32_t* pages, int32_t n, bool releasing) {
    bool ok = true;
    int32_t marked = 0;
    for (int32_t i = 0; i < n; ++i) {
      const int32_t page = pages[i];
      if (!valid(page) || count[page] == 0) { ok = false; break; }
      ++scratch[page];
      ++marked;
      if (releasing && scratch[page] > count[page]) { ok = false; break; }
    }
    for (int32_t i = 0; i < marked; ++i) scratch[pages[i]] = 0;
    return ok;
  }
};

extern "C" {

int marl_page_pool_create(int32_t num_pages, marl_page_pool** out) {
  if (num_pages < 1 || !out) return MARL_INVALID_ARG;
  marl_page_pool* p = new (std::nothrow) marl_page_pool;
  if (!p) return MARL_OUT_OF_MEMORY;
  // the only host allocations of a pool's life (the free stack never outgrows num_pages entries);
  // a failure here must not cross the C boundary as an exception
  try {
    p->count.assign(num_pages, 0);
    p->scratch.assign(num_pages, 0);
    p->free_stack.resize(num_pages);
  } catch (...) {
    delete p;
    return MARL_OUT_OF_MEMORY;
  }
  for (int32_t i = 0; i < num_pages; ++i) p->free_stack[i] = num_pages - 1 - i;   // pops 0, 1, 2, ...
  *out = p;
  return MARL_OK;
}

void marl_page_pool_destroy(marl_page_pool* p) { delete p; }

int marl_page_pool_alloc(marl_page_pool* p, int32_t n, int32_t* pages_out) {
  if (!p || n < 0 || (n > 0 && !pages_out)) return MARL_INVALID_ARG;
  if ((size_t)n > p->free_stack.size()) return MARL_WORKSPACE_TOO_SMALL;
  for (int32_t i = 0; i < n; ++i) pages_out[i] = p->take();
  return MARL_OK;
}

int marl_page_pool_retain(marl_page_pool* p, const int32_t* pages, int32_t n) {
  if (!p || n < 0 || (n > 0 && !pages)) return MARL_INVALID_ARG;
  if (!p->check_list(pages, n, false)) return MARL_INVALID_ARG;
  for (int32_t i = 0; i < n; ++i) ++p->count[pages[i]];
  return MARL_OK;
}

int marl_page_pool_release(marl_page_pool* p, const int32_t* pages, int32_t n) {
  if (!p || n < 0 || (n > 0 && !pages)) return MARL_INVALID_ARG;
  if (!p->check_list(pages, n, true)) return MARL_INVALID_ARG;
  for (int32_t i = 0; i < n; ++i) p->unref(pages[i]);
  return MARL_OK;
}

int marl_page_pool_fork(marl_page_pool* p, const int32_t* parent_row, int32_t len, int32_t* child_row) {
  if (!p || len < 0 || (len > 0 && (!parent_row || !child_row))) return MARL_INVALID_ARG;
  const int32_t n = (len + 15) / 16;
  const int rc = marl_page_pool_retain(p, parent_row, n);
  if (rc != MARL_OK) return rc;
  for (int32_t i = 0; i < n; ++i) child_row[i] = parent_row[i];
  return MARL_OK;
}

int marl_page_pool_prepare_append(marl_page_pool* p, int32_t* row, int32_t max_pages, int32_t len,
                                  int32_t* copy_src, int32_t* copy_dst) {
  if (!p || !row || !copy_src || !copy_dst || max_pages < 1 || len < 0) return MARL_INVALID_ARG;
  if (len >= (int64_t)max_pages * 16) return MARL_INVALID_ARG;
  *copy_src = *copy_dst = -1;
  const int32_t slot = len / 16;
  if (len % 16 == 0) {
    if (p->free_stack.empty()) return MARL_WORKSPACE_TOO_SMALL;
    row[slot] = p->take();
    return MARL_OK;
  }
  const int32_t old = row[slot];
  if (!p->valid(old) || p->count[old] == 0) return MARL_INVALID_ARG;
  if (p->count[old] == 1) return MARL_OK;           // sole holder: write in place
  if (p->free_stack.empty()) return MARL_WORKSPACE_TOO_SMALL;
  const int32_t fresh = p->take();
  p->unref(old);                                     // count > 1 before: stays in use
  row[slot] = fresh;
  *copy_src = old;
  *copy_dst = fresh;
  return MARL_OK;
}

int marl_page_pool_drop(marl_page_pool* p, const int32_t* row, int32_t len) {
  if (!p || len < 0 || (len > 0 && !row)) return MARL_INVALID_ARG;
  return marl_page_pool_release(p, row, (len + 15) / 16);
}

int marl_page_pool_query(const marl_page_pool* p, int32_t page, int32_t* refcount, int32_t* free_pages) {
  if (!p) return MARL_INVALID_ARG;
  if (refcount) {
    if (!p->valid(page)) return MARL_INVALID_ARG;
    *refcount = p->count[page];
  }
  if (free_pages) *free_pages = (int32_t)p->free_stack.size();
  return MARL_OK;
}

}  // extern "C"
