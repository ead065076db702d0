// Internal helpers of libtreetrain (not part of the C ABI).
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>
#include "treetrain.h"

namespace tt {

// Records the message returned by tt_last_error() for this thread and returns `code`.
tt_status fail(tt_status code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Validates an attention descriptor (dtype, sizes, head counts, strides, scale, flags).
tt_status check_attn_desc(const tt_attn_desc* d);

// A validated forest: child lists in ascending input id and the DFS pre-order (paper Eq. 8).
struct Forest {
  std::vector<int32_t> first_child, next_sibling, roots;   // input numbering
  std::vector<int32_t> order;                              // order[rank] = input id
  std::vector<int32_t> rank;                               // rank[input id]
  int64_t n_tokens = 0;
  int32_t n_leaves = 0;
};

// Validates the parent array (range, cycles, sizes) and fills `f`.  Children keep ascending input id.
tt_status build_forest(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len, int32_t n_prefix, Forest& f);

}  // namespace tt
