// Exercises the host-only paging code (page-id allocator, row-map construction) as a plain C++
// program, so that it can be built with -fsanitize=address,undefined and run without a GPU.
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "../../include/dllmc.h"
#include "../../paper_2506_06295_amd/csrc/paging_host.hpp"

#define REQUIRE(c) do { if (!(c)) { std::printf("FAILED line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main() {
  dllmc_page_pool* pool = nullptr;
  REQUIRE(dllmc_pool_create(&pool, 0) == DLLMC_EINVAL && pool == nullptr);
  REQUIRE(dllmc_pool_create(&pool, 10) == DLLMC_OK);
  REQUIRE(dllmc_pool_available(pool) == 10);
  int32_t a[4], b[7];
  REQUIRE(dllmc_pool_alloc(pool, 4, a) == DLLMC_OK);
  REQUIRE(a[0] == 0 && a[1] == 1 && a[2] == 2 && a[3] == 3);
  REQUIRE(dllmc_pool_alloc(pool, 7, b) == DLLMC_ENOMEM);       // all or nothing
  REQUIRE(dllmc_pool_available(pool) == 6);
  const int32_t dup[2] = {1, 1}, range[1] = {10}, unalloc[1] = {7};
  REQUIRE(dllmc_pool_free(pool, dup, 2) == DLLMC_EINVAL);
  REQUIRE(dllmc_pool_free(pool, range, 1) == DLLMC_EINVAL);
  REQUIRE(dllmc_pool_free(pool, unalloc, 1) == DLLMC_EINVAL);
  REQUIRE(dllmc_pool_available(pool) == 6);                    // nothing was freed
  const int32_t back[2] = {2, 0};
  REQUIRE(dllmc_pool_free(pool, back, 2) == DLLMC_OK);
  REQUIRE(dllmc_pool_free(pool, back, 2) == DLLMC_EINVAL);     // double free
  int32_t c[2];
  REQUIRE(dllmc_pool_alloc(pool, 2, c) == DLLMC_OK && c[0] == 0 && c[1] == 2);
  // concurrent callers: every id handed out exactly once
  std::vector<std::vector<int32_t>> got(4);
  std::vector<std::thread> th;
  for (int t = 0; t < 4; ++t)
    th.emplace_back([&, t] {
      for (int i = 0; i < 50; ++i) {
        int32_t id;
        if (dllmc_pool_alloc(pool, 1, &id) == DLLMC_OK) { got[t].push_back(id); if (i % 3 == 0) { dllmc_pool_free(pool, &id, 1); got[t].pop_back(); } }
      }
    });
  for (auto& t : th) t.join();
  std::vector<int> count(10, 0);
  for (auto& g : got) for (int32_t id : g) ++count[id];
  for (int32_t id : a) if (id != 0 && id != 2) ++count[id];
  for (int32_t id : c) ++count[id];
  for (int i = 0; i < 10; ++i) REQUIRE(count[i] <= 1);
  REQUIRE(dllmc_pool_destroy(pool) == DLLMC_OK);

  // row map: B = 2 sequences of n = 10 rows, pages of 4 rows (3 pages each), pool of 8 pages
  const int32_t table[6] = {5, 0, 7, 2, 6, 1};
  std::vector<int> map = dllmc::build_row_map(2, 10, 4, 8, table);
  REQUIRE(map.size() == 20);
  for (int bq = 0; bq < 2; ++bq)
    for (int pos = 0; pos < 10; ++pos) REQUIRE(map[bq * 10 + pos] == table[bq * 3 + pos / 4] * 4 + pos % 4);
  const int32_t twice[6] = {5, 0, 7, 2, 5, 1}, outside[6] = {5, 0, 8, 2, 6, 1}, negative[6] = {5, 0, -1, 2, 6, 1};
  REQUIRE(dllmc::build_row_map(2, 10, 4, 8, twice).empty());
  REQUIRE(dllmc::build_row_map(2, 10, 4, 8, outside).empty());
  REQUIRE(dllmc::build_row_map(2, 10, 4, 8, negative).empty());
  REQUIRE(dllmc::build_row_map(2, 10, 0, 8, table).empty());
  REQUIRE(dllmc::build_row_map(2, 10, 4, 8, nullptr).empty());
  std::printf("paging host logic ok\n");
  return 0;
}
