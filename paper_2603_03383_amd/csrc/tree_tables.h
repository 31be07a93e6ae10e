// Compile-time tables of the static candidate trees (Section 3.2, "Tensorization of Tree
// Topology": the tree is fixed offline and shipped as constant tensors).
//
// A node is a tuple of per-head candidate ranks (r_1..r_m), r_i < caps[i-1]; it is kept iff
// prod(r_i + 1) <= budgets[m-1].  The tables are produced level by level at compile time: the
// children of the nodes of depth m-1, taken in order, give depth m in lexicographic order.
#pragma once
#include <stdint.h>

namespace mdz {

constexpr int kMaxT = 64;      // nodes
constexpr int kMaxK = 5;       // Medusa heads (tree depth)
constexpr int kMaxPaths = 64;  // leaves

struct TreeTables {
  int T, K, n_paths, n_cand;
  int caps[8];
  int parent[kMaxT];
  int depth[kMaxT];
  int cand_slot[kMaxT];
  uint64_t anc_mask[kMaxT];            // bit j of anc_mask[i]: node j is i or an ancestor of i
  int retrieve[kMaxPaths][kMaxK + 1];  // root->leaf node indices per leaf, -1 padded
};

struct TreeRule {
  int K;
  int caps[kMaxK];
  int budgets[kMaxK];
};

constexpr TreeTables make_tree(TreeRule rule) {
  TreeTables t{};
  int prod[kMaxT] = {};
  int rank[kMaxT] = {};
  t.K = rule.K;
  t.T = 1;
  t.parent[0] = -1;
  t.depth[0] = 0;
  prod[0] = 1;
  int level_begin = 0, level_end = 1;
  for (int m = 1; m <= rule.K; ++m) {
    for (int p = level_begin; p < level_end; ++p)
      for (int r = 0; r < rule.caps[m - 1]; ++r)
        if (prod[p] * (r + 1) <= rule.budgets[m - 1]) {
          int n = t.T++;
          t.parent[n] = p;
          t.depth[n] = m;
          prod[n] = prod[p] * (r + 1);
          rank[n] = r;
        }
    level_begin = level_end;
    level_end = t.T;
  }
  int seg = 1;  // start of head m's segment in the flat candidate buffer
  int seg_of_depth[kMaxK + 1] = {};
  for (int m = 1; m <= rule.K; ++m) {
    seg_of_depth[m] = seg;
    seg += rule.caps[m - 1];
    t.caps[m - 1] = rule.caps[m - 1];
  }
  t.n_cand = seg;
  bool has_child[kMaxT] = {};
  for (int n = 0; n < t.T; ++n) {
    t.cand_slot[n] = n == 0 ? 0 : seg_of_depth[t.depth[n]] + rank[n];
    t.anc_mask[n] = (uint64_t(1) << n) | (n == 0 ? 0 : t.anc_mask[t.parent[n]]);
    if (n) has_child[t.parent[n]] = true;
  }
  t.n_paths = 0;
  for (int n = 0; n < t.T; ++n) {
    if (has_child[n]) continue;
    int row = t.n_paths++;
    for (int c = 0; c <= kMaxK; ++c) t.retrieve[row][c] = -1;
    for (int v = n; v >= 0; v = t.parent[v]) t.retrieve[row][t.depth[v]] = v;
  }
  return t;
}

constexpr TreeTables kTree15 = make_tree(TreeRule{3, {2, 2, 2, 0, 0}, {2, 4, 8, 0, 0}});
constexpr TreeTables kTree64 = make_tree(TreeRule{4, {10, 10, 4, 4, 0}, {10, 12, 4, 3, 0}});
// Five heads (the paper's final configuration trains five: Table 2), still 64 nodes: widths 1/9/26/13/9/6, 34 leaves.
constexpr TreeTables kTree64K5 = make_tree(TreeRule{5, {9, 10, 4, 3, 2}, {9, 10, 4, 3, 2}});
// The degenerate tree: the root alone (no Medusa head).  A verify step over it is one ordinary autoregressive
// decode step, the baseline the paper's Overhead and Speedup metrics are defined against (Section 4.1).
constexpr TreeTables kTree1 = make_tree(TreeRule{0, {0, 0, 0, 0, 0}, {0, 0, 0, 0, 0}});

static_assert(kTree15.T == 15 && kTree15.n_paths == 8 && kTree15.n_cand == 7, "15-node tree");
static_assert(kTree64.T == 64 && kTree64.n_paths == 38 && kTree64.n_cand == 29, "64-node tree");
static_assert(kTree64K5.T == 64 && kTree64K5.n_paths == 34 && kTree64K5.n_cand == 29, "64-node tree of depth 5");
static_assert(kTree1.T == 1 && kTree1.n_paths == 1 && kTree1.n_cand == 1 && kTree1.retrieve[0][0] == 0, "single node");

constexpr int kNumTrees = 4;

inline const TreeTables* host_tree(int id) {
  return id == 0 ? &kTree15 : id == 1 ? &kTree64 : id == 2 ? &kTree1 : id == 3 ? &kTree64K5 : nullptr;
}

}  // namespace mdz
