// Host-side tree partitioning (Section "Redundancy-Free Tree Partitioning") and the bookkeeping of
// partition boundaries (Appendix "Zero-Overhead Partition Boundaries": cached slice, ancestor-aware
// bias, depth-based position offset), flattened into the arrays the device driver consumes.
// The packer is a deterministic greedy rule (stated at tt_tree_partition_plan); the paper's solver
// is not part of this library.  O(nodes + tokens + total slice length), no recursion.
#include <climits>
#include <vector>
#include "tt_internal.h"

namespace {

struct Plan {
  int32_t n_parts = 0;
  int32_t n_tokens = 0;
  std::vector<int32_t> part_of_node, part_node_off, part_nodes, part_parent, part_cut_node, part_pos_offset;
  std::vector<int32_t> part_tok_off, own_tok;
  std::vector<int64_t> part_prefix_off;
  std::vector<int32_t> prefix_tok;
  std::vector<uint8_t> prefix_visible;
  std::vector<int32_t> loc_start;      // per node (input id): offset inside its partition's own sequence
  std::vector<int32_t> loc_sub_end;    // per node: end of its subtree inside the partition's own sequence
};

// Greedy assignment + boundary bookkeeping.  `want_slices` = false stops after the sizes are known
// (slice contents are not materialised; their lengths still are).
tt_status make_plan(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len, int32_t capacity,
                    bool want_slices, Plan& pl, std::vector<int64_t>& prefix_len) {
  if (capacity < 1) return tt::fail(TT_ERR_SHAPE, "capacity=%d must be >= 1", capacity);
  tt::Forest f;
  if (tt_status s = tt::build_forest(n_nodes, parent, seg_len, 0, f)) return s;
  pl.n_tokens = (int32_t)f.n_tokens;

  // whole-tree DFS token start of every node (input numbering)
  std::vector<int32_t> node_start(n_nodes, 0);
  {
    int64_t t = 0;
    for (int32_t rk = 0; rk < n_nodes; rk++) { node_start[f.order[rk]] = (int32_t)t; t += seg_len[f.order[rk]]; }
  }

  // ---- greedy packing ----
  pl.part_of_node.assign(n_nodes, -1);
  pl.part_nodes.reserve(n_nodes);
  pl.part_node_off.push_back(0);
  std::vector<int32_t> pending(f.roots);            // first-in-first-out: consumed through `head`
  pending.reserve(n_nodes);
  struct Frame { int32_t node, cursor; };
  std::vector<Frame> stack;
  for (size_t head = 0; head < pending.size(); head++) {
    const int32_t p = pl.n_parts++;
    int64_t size = 0;
    auto take = [&](int32_t node) {
      pl.part_nodes.push_back(node);
      pl.part_of_node[node] = p;
      size += seg_len[node];
      stack.push_back({node, f.first_child[node]});
    };
    take(pending[head]);
    while (!stack.empty()) {
      Frame& top = stack.back();
      const int32_t c = top.cursor;
      if (c < 0) { stack.pop_back(); continue; }
      top.cursor = f.next_sibling[c];
      if (size + seg_len[c] <= capacity) take(c);       // `top` is not used after this push
      else pending.push_back(c);
    }
    pl.part_node_off.push_back((int32_t)pl.part_nodes.size());
  }

  // ---- own sequences: local offsets, local subtree ends, whole-tree token ids ----
  const int32_t np = pl.n_parts;
  pl.loc_start.assign(n_nodes, 0);
  pl.loc_sub_end.assign(n_nodes, 0);
  pl.part_tok_off.assign(np + 1, 0);
  if (want_slices) pl.own_tok.resize(pl.n_tokens);
  std::vector<int64_t> sub(n_nodes, 0);
  for (int32_t p = 0; p < np; p++) {
    const int32_t b = pl.part_node_off[p], e = pl.part_node_off[p + 1];
    int32_t run = 0;
    const int32_t base = pl.part_tok_off[p];
    for (int32_t k = b; k < e; k++) {
      const int32_t node = pl.part_nodes[k];
      pl.loc_start[node] = run;
      if (want_slices)
        for (int32_t j = 0; j < seg_len[node]; j++) pl.own_tok[base + run + j] = node_start[node] + j;
      run += seg_len[node];
    }
    pl.part_tok_off[p + 1] = base + run;
    for (int32_t k = e - 1; k >= b; k--) {              // reverse pre-order: children before parents
      const int32_t node = pl.part_nodes[k];
      sub[node] += seg_len[node];
      pl.loc_sub_end[node] = (int32_t)(pl.loc_start[node] + sub[node]);
      if (k > b) sub[parent[node]] += sub[node];        // every non-root node's parent is in the partition
    }
  }

  // ---- boundaries, parents first ----
  pl.part_parent.assign(np, -1);
  pl.part_cut_node.assign(np, -1);
  pl.part_pos_offset.assign(np, 0);
  pl.part_prefix_off.assign(np + 1, 0);
  prefix_len.assign(np, 0);
  for (int32_t p = 0; p < np; p++) {
    const int32_t root = pl.part_nodes[pl.part_node_off[p]];
    const int32_t nc = parent[root];
    if (nc >= 0) {
      const int32_t P = pl.part_of_node[nc];
      const int32_t e_nc = pl.loc_start[nc] + seg_len[nc];
      pl.part_parent[p] = P;
      pl.part_cut_node[p] = nc;
      prefix_len[p] = prefix_len[P] + e_nc;
      if (prefix_len[p] + (pl.part_tok_off[p + 1] - pl.part_tok_off[p]) >= INT32_MAX)
        return tt::fail(TT_ERR_SHAPE, "partition %d: slice + own tokens do not fit int32", p);
    }
    pl.part_prefix_off[p + 1] = pl.part_prefix_off[p] + prefix_len[p];
  }
  if (!want_slices) {
    // position offsets are cheap and part of no size; skipped here
    return TT_OK;
  }
  pl.prefix_tok.resize((size_t)pl.part_prefix_off[np]);
  pl.prefix_visible.resize((size_t)pl.part_prefix_off[np]);
  for (int32_t p = 0; p < np; p++) {
    const int32_t nc = pl.part_cut_node[p];
    if (nc < 0) continue;
    const int32_t P = pl.part_parent[p];
    const int32_t e_nc = pl.loc_start[nc] + seg_len[nc];
    int32_t* tok = pl.prefix_tok.data() + pl.part_prefix_off[p];
    uint8_t* vis = pl.prefix_visible.data() + pl.part_prefix_off[p];
    const int64_t past = prefix_len[P];
    // P's own slice, flags carried over
    for (int64_t j = 0; j < past; j++) {
      tok[j] = pl.prefix_tok[pl.part_prefix_off[P] + j];
      vis[j] = pl.prefix_visible[pl.part_prefix_off[P] + j];
    }
    // P's own tokens up to the end of the cut node, all masked at first
    for (int32_t j = 0; j < e_nc; j++) {
      tok[past + j] = pl.own_tok[pl.part_tok_off[P] + j];
      vis[past + j] = 0;
    }
    // nodes on the path P.root .. n_c become visible; their lengths above n_c give n_c's depth in P
    const int32_t p_root = pl.part_nodes[pl.part_node_off[P]];
    int64_t depth_nc = 0;
    for (int32_t a = nc;; a = parent[a]) {
      for (int32_t j = 0; j < seg_len[a]; j++) vis[past + pl.loc_start[a] + j] = 1;
      if (a != nc) depth_nc += seg_len[a];
      if (a == p_root) break;
    }
    pl.part_pos_offset[p] = (int32_t)(pl.part_pos_offset[P] + depth_nc + seg_len[nc]);
  }
  return TT_OK;
}

int64_t n_ktiles_of(int64_t n_prefix, int64_t n_own) {
  return tt::ceil_div(n_prefix, TT_KTILE) + tt::ceil_div(n_own, TT_KTILE);
}

template <typename T>
void copy_out(T* dst, const std::vector<T>& src) {
  if (dst) for (size_t i = 0; i < src.size(); i++) dst[i] = src[i];
}

}  // namespace

extern "C" tt_status tt_tree_partition_sizes(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                             int32_t capacity, tt_partition_sizes* out) {
  tt::clear_error();
  if (!out) return tt::fail(TT_ERR_NULL, "out is NULL");
  Plan pl;
  std::vector<int64_t> prefix_len;
  if (tt_status s = make_plan(n_nodes, parent, seg_len, capacity, false, pl, prefix_len)) return s;
  out->n_parts = pl.n_parts;
  out->n_tokens = pl.n_tokens;
  out->max_part_tokens = 0;
  out->max_prefix = 0;
  out->sum_prefix = pl.part_prefix_off[pl.n_parts];
  out->sum_ktiles = 0;
  for (int32_t p = 0; p < pl.n_parts; p++) {
    const int32_t n_own = pl.part_tok_off[p + 1] - pl.part_tok_off[p];
    if (n_own > out->max_part_tokens) out->max_part_tokens = n_own;
    if (prefix_len[p] > out->max_prefix) out->max_prefix = (int32_t)prefix_len[p];
    out->sum_ktiles += n_ktiles_of(prefix_len[p], n_own);
  }
  return TT_OK;
}

extern "C" tt_status tt_tree_partition_plan(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                            int32_t capacity,
                                            int32_t* part_of_node, int32_t* part_node_off, int32_t* part_nodes,
                                            int32_t* part_parent, int32_t* part_cut_node, int32_t* part_pos_offset,
                                            int32_t* part_tok_off, int32_t* own_tok,
                                            int64_t* part_prefix_off, int32_t* prefix_tok, uint8_t* prefix_visible,
                                            int32_t* kend, int64_t* part_ktile_off, int32_t* kt_min, int32_t* kt_max,
                                            int32_t* part_own_start, int32_t* part_prefix_start) {
  tt::clear_error();
  if ((kt_min || kt_max) && !(kt_min && kt_max))
    return tt::fail(TT_ERR_NULL, "kt_min and kt_max are written together; one of them is NULL");
  Plan pl;
  std::vector<int64_t> prefix_len;
  if (tt_status s = make_plan(n_nodes, parent, seg_len, capacity, true, pl, prefix_len)) return s;
  copy_out(part_of_node, pl.part_of_node);
  copy_out(part_node_off, pl.part_node_off);
  copy_out(part_nodes, pl.part_nodes);
  copy_out(part_parent, pl.part_parent);
  copy_out(part_cut_node, pl.part_cut_node);
  copy_out(part_pos_offset, pl.part_pos_offset);
  copy_out(part_tok_off, pl.part_tok_off);
  copy_out(own_tok, pl.own_tok);
  copy_out(part_prefix_off, pl.part_prefix_off);
  copy_out(prefix_tok, pl.prefix_tok);
  copy_out(prefix_visible, pl.prefix_visible);

  // partitions whose rows are one ascending run of whole-tree indices need no gather
  auto run_start = [](const int32_t* tok, int64_t n) -> int32_t {
    if (n == 0) return -1;
    for (int64_t j = 1; j < n; j++) if (tok[j] != tok[0] + j) return -1;
    return tok[0];
  };
  for (int32_t p = 0; p < pl.n_parts; p++) {
    if (part_own_start)
      part_own_start[p] = run_start(pl.own_tok.data() + pl.part_tok_off[p], pl.part_tok_off[p + 1] - pl.part_tok_off[p]);
    if (part_prefix_start)
      part_prefix_start[p] = run_start(pl.prefix_tok.data() + pl.part_prefix_off[p], prefix_len[p]);
  }

  // visibility bounds and their tile summaries, partition by partition
  std::vector<int32_t> ke;
  int64_t tile_off = 0;
  for (int32_t p = 0; p < pl.n_parts; p++) {
    const int64_t P = prefix_len[p];
    const int32_t n_own = pl.part_tok_off[p + 1] - pl.part_tok_off[p];
    ke.resize((size_t)(P + n_own));
    const uint8_t* vis = pl.prefix_visible.data() + pl.part_prefix_off[p];
    for (int64_t j = 0; j < P; j++) ke[j] = vis[j] ? INT32_MAX : 0;
    for (int32_t k = pl.part_node_off[p]; k < pl.part_node_off[p + 1]; k++) {
      const int32_t node = pl.part_nodes[k];
      const int32_t bound = (int32_t)(P + pl.loc_sub_end[node]);
      for (int32_t j = 0; j < seg_len[node]; j++) ke[P + pl.loc_start[node] + j] = bound;
    }
    if (kend) {
      int32_t* dst = kend + pl.part_prefix_off[p] + pl.part_tok_off[p];
      for (size_t j = 0; j < ke.size(); j++) dst[j] = ke[j];
    }
    if (part_ktile_off) part_ktile_off[p] = tile_off;
    // the slice and the own keys are tiled separately, each from its first key
    const int64_t region_begin[2] = {0, P}, region_end[2] = {P, P + n_own};
    for (int r = 0; r < 2; r++)
      for (int64_t j0 = region_begin[r]; j0 < region_end[r]; j0 += TT_KTILE) {
        int32_t mn = INT32_MAX, mx = INT32_MIN;
        const int64_t j1 = j0 + TT_KTILE < region_end[r] ? j0 + TT_KTILE : region_end[r];
        for (int64_t j = j0; j < j1; j++) { mn = ke[j] < mn ? ke[j] : mn; mx = ke[j] > mx ? ke[j] : mx; }
        if (kt_min) { kt_min[tile_off] = mn; kt_max[tile_off] = mx; }
        tile_off++;
      }
  }
  if (part_ktile_off) part_ktile_off[pl.n_parts] = tile_off;
  return TT_OK;
}
