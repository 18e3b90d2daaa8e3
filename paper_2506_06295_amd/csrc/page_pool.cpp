// Host-side page allocator for the paged cache layout: a pool of equally sized pages, handed out
// and taken back by id.  Plain C++ (no HIP): the library only needs the ids a caller puts into a
// context's page table; this allocator is the bookkeeping for callers that share one pool between
// contexts (pages of a finished generation go back to the pool and serve the next context).
#include <cstdint>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/dllmc.h"
#include "paging_host.hpp"

namespace dllmc {

std::vector<int> build_row_map(int B, int n, int page_rows, int pool_pages, const int32_t* table) {
  if (B < 1 || n < 1 || page_rows < 1 || pool_pages < 1 || !table) return {};
  const int pps = pages_per_seq(n, page_rows);
  std::vector<char> seen(static_cast<size_t>(pool_pages), 0);
  for (long long i = 0; i < static_cast<long long>(B) * pps; ++i) {
    const int32_t p = table[i];
    if (p < 0 || p >= pool_pages || seen[static_cast<size_t>(p)]) return {};
    seen[static_cast<size_t>(p)] = 1;
  }
  std::vector<int> map(static_cast<size_t>(B) * n);
  for (int b = 0; b < B; ++b)
    for (int pos = 0; pos < n; ++pos)
      map[static_cast<size_t>(b) * n + pos] =
          table[static_cast<size_t>(b) * pps + pos / page_rows] * page_rows + pos % page_rows;
  return map;
}

}  // namespace dllmc

struct dllmc_page_pool {
  std::mutex mu;
  std::vector<int32_t> free_ids;   // stack of free page ids; lowest ids are handed out first
  std::vector<uint8_t> in_use;     // per page
};

extern "C" {

int dllmc_pool_create(dllmc_page_pool** out, int32_t pool_pages) {
  if (!out) return DLLMC_EINVAL;
  *out = nullptr;
  if (pool_pages < 1) return DLLMC_EINVAL;
  dllmc_page_pool* p = new (std::nothrow) dllmc_page_pool();
  if (!p) return DLLMC_ENOMEM;
  try {
    p->in_use.assign(static_cast<size_t>(pool_pages), 0);
    p->free_ids.reserve(static_cast<size_t>(pool_pages));
    for (int32_t i = pool_pages - 1; i >= 0; --i) p->free_ids.push_back(i);
  } catch (const std::bad_alloc&) {
    delete p;
    return DLLMC_ENOMEM;
  }
  *out = p;
  return DLLMC_OK;
}

int32_t dllmc_pool_available(dllmc_page_pool* pool) {
  if (!pool) return DLLMC_EINVAL;
  std::lock_guard<std::mutex> lock(pool->mu);
  return static_cast<int32_t>(pool->free_ids.size());
}

int dllmc_pool_alloc(dllmc_page_pool* pool, int32_t count, int32_t* ids_out) {
  if (!pool || count < 0 || (count > 0 && !ids_out)) return DLLMC_EINVAL;
  std::lock_guard<std::mutex> lock(pool->mu);
  if (static_cast<size_t>(count) > pool->free_ids.size()) return DLLMC_ENOMEM;  // all or nothing
  for (int32_t i = 0; i < count; ++i) {
    const int32_t id = pool->free_ids.back();
    pool->free_ids.pop_back();
    pool->in_use[static_cast<size_t>(id)] = 1;
    ids_out[i] = id;
  }
  return DLLMC_OK;
}

int dllmc_pool_free(dllmc_page_pool* pool, const int32_t* ids, int32_t count) {
  if (!pool || count < 0 || (count > 0 && !ids)) return DLLMC_EINVAL;
  std::lock_guard<std::mutex> lock(pool->mu);
  const int32_t n = static_cast<int32_t>(pool->in_use.size());
  // validate everything first: a bad id (out of range, not allocated, listed twice) frees nothing
  for (int32_t i = 0; i < count; ++i) {
    if (ids[i] < 0 || ids[i] >= n || pool->in_use[static_cast<size_t>(ids[i])] != 1) {
      for (int32_t j = 0; j < i; ++j) pool->in_use[static_cast<size_t>(ids[j])] = 1;
      return DLLMC_EINVAL;
    }
    pool->in_use[static_cast<size_t>(ids[i])] = 2;  // marked: catches a second listing
  }
  for (int32_t i = 0; i < count; ++i) {
    pool->in_use[static_cast<size_t>(ids[i])] = 0;
    pool->free_ids.push_back(ids[i]);
  }
  return DLLMC_OK;
}

int dllmc_pool_destroy(dllmc_page_pool* pool) {
  if (!pool) return DLLMC_EINVAL;
  delete pool;
  return DLLMC_OK;
}

}  // extern "C"
