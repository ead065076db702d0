// Host-side tree metadata: DFS serialisation (paper Eq. 8), path counts g_n / K ("Derivation"),
// tree position ids (Eq. 9, Appendix "Depth-Based Position Offset"), loss weights (Eq. 4) and the
// per-key visibility bound with its tile summaries (Section "Attention Mask", Appendix
// "Ancestor-Aware Attention Bias").  O(nodes + tokens), no recursion (trees can be deep chains).
#include <climits>
#include <algorithm>
#include <vector>
#include "tt_internal.h"

namespace tt {

tt_status build_forest(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len, int32_t n_prefix,
                       Forest& f) {
  if (n_nodes < 0 || n_prefix < 0) return tt::fail(TT_ERR_SHAPE, "n_nodes=%d, n_prefix=%d must be >= 0", n_nodes, n_prefix);
  if (n_nodes > 0 && (!parent || !seg_len)) return tt::fail(TT_ERR_NULL, "parent / seg_len is NULL");
  f.first_child.assign(n_nodes, -1);
  f.next_sibling.assign(n_nodes, -1);
  std::vector<int32_t> last_child(n_nodes, -1);
  int64_t total = 0;
  for (int32_t i = 0; i < n_nodes; i++) {
    const int32_t p = parent[i];
    if (seg_len[i] < 0) return tt::fail(TT_ERR_SHAPE, "seg_len[%d]=%d is negative", i, seg_len[i]);
    total += seg_len[i];
    if (p < -1 || p >= n_nodes || p == i) return tt::fail(TT_ERR_TREE, "parent[%d]=%d is out of range", i, p);
    if (p < 0) {
      f.roots.push_back(i);
    } else {
      if (last_child[p] < 0) f.first_child[p] = i; else f.next_sibling[last_child[p]] = i;
      last_child[p] = i;
    }
  }
  if (total + n_prefix >= INT32_MAX) return tt::fail(TT_ERR_SHAPE, "tokens + prefix = %lld does not fit int32", (long long)(total + n_prefix));
  f.n_tokens = total;
  f.order.reserve(n_nodes);
  std::vector<int32_t> stack;
  for (int32_t r : f.roots) {
    stack.push_back(r);
    while (!stack.empty()) {
      const int32_t i = stack.back();
      stack.pop_back();
      f.order.push_back(i);
      if (f.next_sibling[i] >= 0) stack.push_back(f.next_sibling[i]);   // visited after i's subtree
      if (f.first_child[i] >= 0) stack.push_back(f.first_child[i]);
      else f.n_leaves++;
    }
  }
  if ((int32_t)f.order.size() != n_nodes)
    return tt::fail(TT_ERR_TREE, "parent array has a cycle: %d of %d nodes reachable from a root", (int)f.order.size(), n_nodes);
  f.rank.assign(n_nodes, 0);
  for (int32_t rk = 0; rk < n_nodes; rk++) f.rank[f.order[rk]] = rk;
  return TT_OK;
}

}  // namespace tt

namespace {

using tt::Forest;
using tt::build_forest;

int32_t n_ktiles_of(int64_t n_prefix, int64_t n_tokens) {
  return (int32_t)(tt::ceil_div(n_prefix, TT_KTILE) + tt::ceil_div(n_tokens, TT_KTILE));
}

}  // namespace

extern "C" tt_status tt_tree_meta_sizes(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                        int32_t n_prefix, tt_meta_sizes* out) {
  tt::clear_error();
  if (!out) return tt::fail(TT_ERR_NULL, "out is NULL");
  Forest f;
  if (tt_status s = build_forest(n_nodes, parent, seg_len, n_prefix, f)) return s;
  out->n_nodes = n_nodes;
  out->n_tokens = (int32_t)f.n_tokens;
  out->n_leaves = f.n_leaves;
  out->n_roots = (int32_t)f.roots.size();
  out->n_ktiles = n_ktiles_of(n_prefix, f.n_tokens);
  return TT_OK;
}

extern "C" tt_status tt_tree_build_meta(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                        const uint8_t* trained, const int32_t* root_pos_offset,
                                        const int32_t* g_override, int32_t K_override,
                                        int32_t n_prefix, const uint8_t* prefix_visible,
                                        int32_t* dfs_order, int32_t* node_start, int32_t* node_end,
                                        int32_t* subtree_end, int32_t* node_parent, int32_t* node_g,
                                        int32_t* tok_node, int32_t* tok_pos, int32_t* tok_pred,
                                        float* tok_weight,
                                        int32_t* kend, int32_t* ktile_kend_min, int32_t* ktile_kend_max) {
  tt::clear_error();
  Forest f;
  if (tt_status s = build_forest(n_nodes, parent, seg_len, n_prefix, f)) return s;
  if ((g_override != nullptr) != (K_override > 0))
    return tt::fail(TT_ERR_SHAPE, "g_override and K_override must be given together (K_override=%d)", K_override);
  if (K_override < 0) return tt::fail(TT_ERR_SHAPE, "K_override=%d is negative", K_override);
  const int32_t N = (int32_t)f.n_tokens;

  // Per-node quantities in DFS rank.  Pre-order puts a parent before its children, so one
  // forward sweep gives starts and positions and one backward sweep gives subtree ends and g.
  std::vector<int32_t> start(n_nodes), end(n_nodes), sub_end(n_nodes), par(n_nodes), g(n_nodes), pos0(n_nodes), pred0(n_nodes);
  int32_t tok = 0;
  int32_t root_no = 0;
  // roots in f.roots are ascending id and are visited in that order
  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk];
    start[rk] = tok;
    tok += seg_len[i];
    end[rk] = tok;
    if (parent[i] < 0) {
      par[rk] = -1;
      pos0[rk] = root_pos_offset ? root_pos_offset[root_no] : 0;
      pred0[rk] = -1;
      root_no++;
    } else {
      const int32_t p = f.rank[parent[i]];
      par[rk] = p;
      const int64_t ps = (int64_t)pos0[p] + seg_len[parent[i]];
      if (ps + seg_len[i] >= INT32_MAX) return tt::fail(TT_ERR_SHAPE, "position id overflows int32 at node %d", i);
      pos0[rk] = (int32_t)ps;
      // last token of the nearest ancestor that has any token
      pred0[rk] = seg_len[parent[i]] > 0 ? end[p] - 1 : pred0[p];
    }
  }
  for (int32_t rk = n_nodes - 1; rk >= 0; rk--) {
    const int32_t i = f.order[rk];
    if (f.first_child[i] < 0) { sub_end[rk] = end[rk]; g[rk] = 1; }
  }
  // children come after parents: accumulate leaves upwards, subtree end = max over descendants
  {
    std::vector<int32_t> acc_g(n_nodes, 0), acc_end(n_nodes, 0);
    for (int32_t rk = n_nodes - 1; rk >= 0; rk--) {
      const int32_t i = f.order[rk];
      if (f.first_child[i] >= 0) { g[rk] = acc_g[rk]; sub_end[rk] = acc_end[rk] > end[rk] ? acc_end[rk] : end[rk]; }
      if (par[rk] >= 0) {
        acc_g[par[rk]] += g[rk];
        if (sub_end[rk] > acc_end[par[rk]]) acc_end[par[rk]] = sub_end[rk];
      }
    }
  }
  const int32_t K = K_override > 0 ? K_override : f.n_leaves;

  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk];
    if (dfs_order) dfs_order[rk] = i;
    if (node_start) node_start[rk] = start[rk];
    if (node_end) node_end[rk] = end[rk];
    if (subtree_end) subtree_end[rk] = sub_end[rk];
    if (node_parent) node_parent[rk] = par[rk];
    const int32_t gn = g_override ? g_override[i] : g[rk];
    if (node_g) node_g[rk] = gn;
    const float tr = (!trained || trained[i]) ? 1.0f : 0.0f;
    const float w = K > 0 ? tr * ((float)gn / (float)K) : 0.0f;
    for (int32_t t = start[rk]; t < end[rk]; t++) {
      if (tok_node) tok_node[t] = rk;
      if (tok_pos) tok_pos[t] = pos0[rk] + (t - start[rk]);
      if (tok_pred) tok_pred[t] = t == start[rk] ? pred0[rk] : t - 1;
      if (tok_weight) tok_weight[t] = w;
      if (kend) kend[n_prefix + t] = n_prefix + sub_end[rk];
    }
  }
  if (kend)
    for (int32_t j = 0; j < n_prefix; j++) kend[j] = (!prefix_visible || prefix_visible[j]) ? INT32_MAX : 0;

  if (ktile_kend_min || ktile_kend_max) {
    // computed from the same rule as kend so that they can be requested without it
    auto kend_at = [&](int32_t j, const std::vector<int32_t>& tok_sub_end) -> int32_t {
      if (j < n_prefix) return (!prefix_visible || prefix_visible[j]) ? INT32_MAX : 0;
      return n_prefix + tok_sub_end[j - n_prefix];
    };
    std::vector<int32_t> tok_sub_end(N);
    for (int32_t rk = 0; rk < n_nodes; rk++)
      for (int32_t t = start[rk]; t < end[rk]; t++) tok_sub_end[t] = sub_end[rk];
    int32_t tile = 0;
    const int32_t lo[2] = {0, n_prefix}, hi[2] = {n_prefix, n_prefix + N};
    for (int region = 0; region < 2; region++) {
      for (int32_t s = lo[region]; s < hi[region]; s += TT_KTILE, tile++) {
        int32_t mn = INT32_MAX, mx = INT32_MIN;
        const int32_t e = s + TT_KTILE < hi[region] ? s + TT_KTILE : hi[region];
        for (int32_t j = s; j < e; j++) {
          const int32_t v = kend_at(j, tok_sub_end);
          mn = v < mn ? v : mn;
          mx = v > mx ? v : mx;
        }
        if (ktile_kend_min) ktile_kend_min[tile] = mn;
        if (ktile_kend_max) ktile_kend_max[tile] = mx;
      }
    }
  }
  return TT_OK;
}

extern "C" tt_status tt_tree_path_weights(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len,
                                          const uint8_t* trained, int32_t scheme, const float* path_weight,
                                          const float* advantage, float* tok_weight, int32_t* leaf_node) {
  tt::clear_error();
  Forest f;
  if (tt_status s = build_forest(n_nodes, parent, seg_len, 0, f)) return s;
  if (scheme != TT_WEIGHT_PATH_SUM && scheme != TT_WEIGHT_UNIFORM && scheme != TT_WEIGHT_PATH_TOKEN_MEAN)
    return tt::fail(TT_ERR_UNSUPPORTED, "unknown weight scheme %d", scheme);
  if (scheme == TT_WEIGHT_PATH_SUM && f.n_leaves > 0 && !path_weight)
    return tt::fail(TT_ERR_NULL, "path_weight is NULL for TT_WEIGHT_PATH_SUM");
  if (f.n_tokens > 0 && !tok_weight) return tt::fail(TT_ERR_NULL, "tok_weight is NULL");
  auto is_trained = [&](int32_t i) { return !trained || trained[i]; };

  // w_k per leaf (fp64), leaves numbered in DFS order; then lambda of a node = sum over the leaves of
  // its subtree, accumulated children-to-parent in reverse pre-order.
  std::vector<double> lam(n_nodes, 0.0);
  std::vector<int64_t> trained_above(n_nodes, 0);      // trained tokens on the path root .. node (pre-order rank)
  const int32_t K = f.n_leaves;
  int32_t leaf = 0;
  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk];
    const int64_t up = parent[i] < 0 ? 0 : trained_above[f.rank[parent[i]]];
    trained_above[rk] = up + (is_trained(i) ? seg_len[i] : 0);
    if (f.first_child[i] >= 0) continue;
    if (leaf_node) leaf_node[leaf] = i;
    if (scheme == TT_WEIGHT_PATH_SUM) lam[rk] = (double)path_weight[leaf];
    else if (scheme == TT_WEIGHT_PATH_TOKEN_MEAN) lam[rk] = trained_above[rk] > 0 ? 1.0 / ((double)K * (double)trained_above[rk]) : 0.0;
    leaf++;
  }
  for (int32_t rk = n_nodes - 1; rk >= 0; rk--) {
    const int32_t i = f.order[rk];
    if (parent[i] >= 0) lam[f.rank[parent[i]]] += lam[rk];
  }
  int64_t t = 0;
  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk];
    float w = scheme == TT_WEIGHT_UNIFORM ? 1.0f : (float)lam[rk];
    if (!is_trained(i)) w = 0.0f;
    for (int32_t j = 0; j < seg_len[i]; j++, t++) tok_weight[t] = advantage ? w * advantage[t] : w;
  }
  return TT_OK;
}

namespace {

// Tokens whose successors on some branch do not directly follow them in DFS order, for the backward of
// the tree convolution.  A "jump" token t (tok_pred[t] >= 0 and != t-1) is such a successor of each
// of its first K-1 predecessors; pairs come out grouped by predecessor, ascending.
tt_status conv_pairs(int64_t n_tokens, const int32_t* tok_pred, int32_t K, std::vector<int32_t>& s_of, std::vector<int32_t>& t_of,
                     std::vector<int32_t>& r_of) {
  if (n_tokens < 0 || n_tokens >= INT32_MAX) return tt::fail(TT_ERR_SHAPE, "n_tokens=%lld out of range", (long long)n_tokens);
  if (K < 2 || K > 4) return tt::fail(TT_ERR_UNSUPPORTED, "kernel_size=%d: only 2, 3, 4 are built", K);
  if (n_tokens > 0 && !tok_pred) return tt::fail(TT_ERR_NULL, "tok_pred is NULL");
  for (int64_t t = 0; t < n_tokens; t++)
    if (tok_pred[t] < -1 || tok_pred[t] >= t) return tt::fail(TT_ERR_TREE, "tok_pred[%lld]=%d is not an earlier token", (long long)t, tok_pred[t]);
  // count per predecessor, then fill (stable: pairs of one predecessor stay in ascending t)
  std::vector<int32_t> cnt(n_tokens + 1, 0);
  auto for_each_pair = [&](auto&& fn) {
    for (int64_t t = 0; t < n_tokens; t++) {
      if (tok_pred[t] < 0 || tok_pred[t] == t - 1) continue;
      int32_t a = tok_pred[t];
      for (int32_t r = 1; r < K && a >= 0; r++, a = tok_pred[a]) fn(a, (int32_t)t, r);
    }
  };
  for_each_pair([&](int32_t a, int32_t, int32_t) { cnt[a + 1]++; });
  for (int64_t i = 0; i < n_tokens; i++) cnt[i + 1] += cnt[i];
  const int32_t total = n_tokens ? cnt[n_tokens] : 0;
  s_of.assign(total, 0); t_of.assign(total, 0); r_of.assign(total, 0);
  std::vector<int32_t> cur(cnt.begin(), cnt.end() - 1);
  for_each_pair([&](int32_t a, int32_t t, int32_t r) {
    const int32_t k = cur[a]++;
    s_of[k] = a; t_of[k] = t; r_of[k] = r;
  });
  return TT_OK;
}

}  // namespace

extern "C" tt_status tt_tree_conv_plan_sizes(int64_t n_tokens, const int32_t* tok_pred, int32_t kernel_size, int32_t* n_fix,
                                             int32_t* n_pairs) {
  tt::clear_error();
  if (!n_fix || !n_pairs) return tt::fail(TT_ERR_NULL, "n_fix / n_pairs is NULL");
  std::vector<int32_t> s_of, t_of, r_of;
  if (tt_status s = conv_pairs(n_tokens, tok_pred, kernel_size, s_of, t_of, r_of)) return s;
  int32_t nf = 0;
  for (size_t k = 0; k < s_of.size(); k++) nf += k == 0 || s_of[k] != s_of[k - 1];
  *n_fix = nf;
  *n_pairs = (int32_t)s_of.size();
  return TT_OK;
}

extern "C" tt_status tt_tree_conv_plan(int64_t n_tokens, const int32_t* tok_pred, int32_t kernel_size, int32_t* fix_tok,
                                       int32_t* fix_off, int32_t* fix_t, int32_t* fix_r) {
  tt::clear_error();
  if (!fix_off) return tt::fail(TT_ERR_NULL, "fix_off is NULL");
  std::vector<int32_t> s_of, t_of, r_of;
  if (tt_status s = conv_pairs(n_tokens, tok_pred, kernel_size, s_of, t_of, r_of)) return s;
  if (!s_of.empty() && (!fix_tok || !fix_t || !fix_r)) return tt::fail(TT_ERR_NULL, "fix_tok / fix_t / fix_r is NULL");
  int32_t nf = 0;
  for (size_t k = 0; k < s_of.size(); k++) {
    if (k == 0 || s_of[k] != s_of[k - 1]) { fix_tok[nf] = s_of[k]; fix_off[nf] = (int32_t)k; nf++; }
    fix_t[k] = t_of[k];
    fix_r[k] = r_of[k];
  }
  fix_off[nf] = (int32_t)s_of.size();
  return TT_OK;
}

namespace {

struct GdnPlan {
  std::vector<int32_t> tok0, len, src, dst, cap;
  int32_t n_slots = 0;
};

// Chunk program of the gated-delta-rule scan: nodes in DFS order, TT_GDN_CHUNK tokens per chunk.
tt_status gdn_plan(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len, int32_t n_capture,
                   const int32_t* capture_node, GdnPlan& pl) {
  if (n_capture < 0 || (n_capture > 0 && !capture_node)) return tt::fail(TT_ERR_NULL, "n_capture=%d with capture_node NULL", n_capture);
  Forest f;
  if (tt_status s = build_forest(n_nodes, parent, seg_len, 0, f)) return s;
  // nearest token-bearing ancestor (input numbering), -1 if none
  std::vector<int32_t> eff(n_nodes, -1), branches(n_nodes, 0), slot(n_nodes, -1), last_chunk(n_nodes, -1);
  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk], p = parent[i];
    eff[i] = p < 0 ? -1 : (seg_len[p] > 0 ? p : eff[p]);
    if (seg_len[i] > 0 && eff[i] >= 0) branches[eff[i]]++;
  }
  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk];
    if (branches[i] >= 2) slot[i] = pl.n_slots++;     // a single continuation stays on chip
  }
  int64_t tok = 0;
  for (int32_t rk = 0; rk < n_nodes; rk++) {
    const int32_t i = f.order[rk];
    for (int32_t off = 0; off < seg_len[i]; off += TT_GDN_CHUNK) {
      const int32_t n = seg_len[i] - off < TT_GDN_CHUNK ? seg_len[i] - off : TT_GDN_CHUNK;
      int32_t src = -2;
      if (off == 0) {
        const int32_t e = eff[i];
        if (e < 0) src = -1;
        else if (slot[e] < 0) src = -2;      // the only continuation: directly after its parent's last chunk
        else src = slot[e];                  // every branch of a branch point starts from the saved state, the first one
                                             // too: the branches are then independent of each other (tt_tree_gdn_schedule)
      }
      pl.tok0.push_back((int32_t)(tok + off));
      pl.len.push_back(n);
      pl.src.push_back(src);
      pl.dst.push_back(-1);
    }
    if (seg_len[i] > 0) {
      last_chunk[i] = (int32_t)pl.tok0.size() - 1;
      pl.dst.back() = slot[i];
    }
    tok += seg_len[i];
  }
  pl.cap.assign(pl.tok0.size(), -1);
  for (int32_t k = 0; k < n_capture; k++) {
    int32_t node = capture_node[k];
    if (node < 0 || node >= n_nodes) return tt::fail(TT_ERR_SHAPE, "capture_node[%d]=%d is not a node", k, node);
    if (seg_len[node] == 0) node = eff[node];
    if (node < 0) return tt::fail(TT_ERR_SHAPE, "capture_node[%d] has no token on or above it: its state is the initial state", k);
    int32_t& slot_of_chunk = pl.cap[last_chunk[node]];
    if (slot_of_chunk >= 0) return tt::fail(TT_ERR_SHAPE, "capture nodes %d and %d end in the same chunk", slot_of_chunk, k);
    slot_of_chunk = k;
  }
  return TT_OK;
}

}  // namespace

namespace {

// Segments of a chunk program: maximal runs of chunks whose state stays on chip (every chunk but the first has
// src == -2).  A segment depends only on the segment that saved the slot its first chunk loads, so segments form a
// forest; level 0 = segments that start from the initial state, level l + 1 = segments whose slot is saved by a
// segment of level l.  Segments of one level are independent of each other.
struct GdnSchedule {
  std::vector<int32_t> c0, c1, level_off;        // segments in level order (stable: chunk order inside a level)
  std::vector<int32_t> cons_off, cons;           // per slot: the segments (positions in c0 / c1) that start from it
};

tt_status gdn_schedule(int32_t n_chunks, const int32_t* src, const int32_t* dst, int32_t n_slots, GdnSchedule& sc) {
  if (n_chunks < 0 || n_slots < 0) return tt::fail(TT_ERR_SHAPE, "n_chunks=%d, n_slots=%d", n_chunks, n_slots);
  if (n_chunks > 0 && (!src || !dst)) return tt::fail(TT_ERR_NULL, "chunk_src / chunk_dst is NULL");
  std::vector<int32_t> first, last, level, slot_seg(n_slots, -1), seg_slot;
  for (int32_t c = 0; c < n_chunks; c++) {
    if (src[c] < -2 || src[c] >= n_slots || dst[c] < -1 || dst[c] >= n_slots)
      return tt::fail(TT_ERR_TREE, "chunk %d: src=%d / dst=%d out of range", c, src[c], dst[c]);
    if (c == 0 && src[c] == -2) return tt::fail(TT_ERR_TREE, "the first chunk cannot continue a previous one");
    if (src[c] != -2) {
      int32_t lv = 0;
      if (src[c] >= 0) {
        if (slot_seg[src[c]] < 0) return tt::fail(TT_ERR_TREE, "chunk %d starts from slot %d before any chunk saved it", c, src[c]);
        lv = level[slot_seg[src[c]]] + 1;
      }
      first.push_back(c); last.push_back(c + 1); level.push_back(lv); seg_slot.push_back(src[c]);
    } else {
      last.back() = c + 1;
    }
    if (dst[c] >= 0) {
      if (slot_seg[dst[c]] >= 0) return tt::fail(TT_ERR_TREE, "slot %d is saved twice", dst[c]);
      slot_seg[dst[c]] = (int32_t)first.size() - 1;
    }
  }
  const int32_t n_seg = (int32_t)first.size();
  int32_t n_levels = 0;
  for (int32_t l : level) n_levels = l + 1 > n_levels ? l + 1 : n_levels;
  sc.level_off.assign(n_levels + 1, 0);
  for (int32_t l : level) sc.level_off[l + 1]++;
  for (int32_t l = 0; l < n_levels; l++) sc.level_off[l + 1] += sc.level_off[l];
  // position of every segment: by level, inside a level the longest first (a level's segments are dealt to the
  // compute units in this order, so the long ones start first and the short ones fill in), ties in chunk order
  std::vector<int32_t> by_pos(n_seg), pos(n_seg);
  for (int32_t s = 0; s < n_seg; s++) by_pos[s] = s;
  std::stable_sort(by_pos.begin(), by_pos.end(), [&](int32_t x, int32_t y) {
    if (level[x] != level[y]) return level[x] < level[y];
    return last[x] - first[x] > last[y] - first[y];
  });
  sc.c0.resize(n_seg); sc.c1.resize(n_seg);
  for (int32_t i = 0; i < n_seg; i++) {
    pos[by_pos[i]] = i;
    sc.c0[i] = first[by_pos[i]]; sc.c1[i] = last[by_pos[i]];
  }
  sc.cons_off.assign(n_slots + 1, 0);
  for (int32_t s = 0; s < n_seg; s++)
    if (seg_slot[s] >= 0) sc.cons_off[seg_slot[s] + 1]++;
  for (int32_t k = 0; k < n_slots; k++) sc.cons_off[k + 1] += sc.cons_off[k];
  sc.cons.resize(sc.cons_off[n_slots]);
  std::vector<int32_t> cc(sc.cons_off.begin(), sc.cons_off.end() - 1);
  for (int32_t s = 0; s < n_seg; s++)
    if (seg_slot[s] >= 0) sc.cons[cc[seg_slot[s]]++] = pos[s];
  return TT_OK;
}

}  // namespace

extern "C" tt_status tt_tree_gdn_schedule_sizes(int32_t n_chunks, const int32_t* chunk_src, const int32_t* chunk_dst, int32_t n_slots,
                                                int32_t* n_segments, int32_t* n_levels, int32_t* n_consumers) {
  tt::clear_error();
  if (!n_segments || !n_levels || !n_consumers) return tt::fail(TT_ERR_NULL, "an output is NULL");
  GdnSchedule sc;
  if (tt_status s = gdn_schedule(n_chunks, chunk_src, chunk_dst, n_slots, sc)) return s;
  *n_segments = (int32_t)sc.c0.size();
  *n_levels = (int32_t)sc.level_off.size() - 1;
  *n_consumers = (int32_t)sc.cons.size();
  return TT_OK;
}

extern "C" tt_status tt_tree_gdn_schedule(int32_t n_chunks, const int32_t* chunk_src, const int32_t* chunk_dst, int32_t n_slots,
                                          int32_t* seg_chunk0, int32_t* seg_chunk1, int32_t* level_off, int32_t* slot_cons_off,
                                          int32_t* slot_cons) {
  tt::clear_error();
  GdnSchedule sc;
  if (tt_status s = gdn_schedule(n_chunks, chunk_src, chunk_dst, n_slots, sc)) return s;
  if (!level_off || !slot_cons_off || (!sc.c0.empty() && (!seg_chunk0 || !seg_chunk1)) || (!sc.cons.empty() && !slot_cons))
    return tt::fail(TT_ERR_NULL, "an output array is NULL");
  for (size_t i = 0; i < sc.c0.size(); i++) { seg_chunk0[i] = sc.c0[i]; seg_chunk1[i] = sc.c1[i]; }
  for (size_t i = 0; i < sc.level_off.size(); i++) level_off[i] = sc.level_off[i];
  for (size_t i = 0; i < sc.cons_off.size(); i++) slot_cons_off[i] = sc.cons_off[i];
  for (size_t i = 0; i < sc.cons.size(); i++) slot_cons[i] = sc.cons[i];
  return TT_OK;
}

extern "C" tt_status tt_tree_gdn_plan_sizes(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len, int32_t* n_chunks,
                                            int32_t* n_slots) {
  tt::clear_error();
  if (!n_chunks || !n_slots) return tt::fail(TT_ERR_NULL, "n_chunks / n_slots is NULL");
  GdnPlan pl;
  if (tt_status s = gdn_plan(n_nodes, parent, seg_len, 0, nullptr, pl)) return s;
  *n_chunks = (int32_t)pl.tok0.size();
  *n_slots = pl.n_slots;
  return TT_OK;
}

extern "C" tt_status tt_tree_gdn_plan(int32_t n_nodes, const int32_t* parent, const int32_t* seg_len, int32_t n_capture,
                                      const int32_t* capture_node, int32_t* chunk_tok0, int32_t* chunk_len, int32_t* chunk_src,
                                      int32_t* chunk_dst, int32_t* chunk_cap) {
  tt::clear_error();
  GdnPlan pl;
  if (tt_status s = gdn_plan(n_nodes, parent, seg_len, n_capture, capture_node, pl)) return s;
  if (n_capture > 0 && !chunk_cap) return tt::fail(TT_ERR_NULL, "chunk_cap is NULL");
  if (!pl.tok0.empty() && (!chunk_tok0 || !chunk_len || !chunk_src || !chunk_dst)) return tt::fail(TT_ERR_NULL, "an output array is NULL");
  for (size_t c = 0; c < pl.tok0.size(); c++) {
    chunk_tok0[c] = pl.tok0[c]; chunk_len[c] = pl.len[c]; chunk_src[c] = pl.src[c]; chunk_dst[c] = pl.dst[c];
    if (chunk_cap) chunk_cap[c] = pl.cap[c];
  }
  return TT_OK;
}
