// Host-only helpers of the paged cache layout (plain C++, no HIP): shared by the C ABI layer and
// the page-id allocator's source file so that they can be built and run under host sanitizers.
#pragma once

#include <cstdint>
#include <vector>

namespace dllmc {

inline int pages_per_seq(int n, int page_rows) { return (n + page_rows - 1) / page_rows; }

// Cache row of every logical row b * n + pos under a page table [B][pages_per_seq(n, page_rows)]:
// table[b][pos / page_rows] * page_rows + pos % page_rows.  Empty when the table is malformed
// (an entry outside [0, pool_pages), or a page listed twice) or an argument is out of range.
std::vector<int> build_row_map(int B, int n, int page_rows, int pool_pages, const int32_t* table);

}  // namespace dllmc
