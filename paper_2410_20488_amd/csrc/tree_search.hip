// Choice of the draft-tree topology for a node budget (host code, no device work).
//
// The paper fixes k and searches, for every budget of tree nodes, for the best tree structure
// (Experiment / Setup; the comparison of average acceptance lengths under node budgets).  With
// greedy verification a draft node is accepted exactly when all its ancestors are and its own
// candidate is the target's token, so for acceptance rates a[level][rank] that depend on the
// prediction step and on the candidate's rank only, the node with rank path (r_1 .. r_l) is
// accepted with probability a[1][r_1] * ... * a[l][r_l] and the expected number of tokens per
// step is 1 + the sum of these products over the draft nodes.  A product never grows along a
// path, so the n - 1 largest products always form an ancestor-closed set: a best-first
// expansion from the root finds an optimal tree.  Ties go to the shallower node, then to the
// smaller rank path, which makes the result unique.
#include <queue>
#include <vector>

#include "../../include/firp.h"

namespace {
struct Cand {
  double p;
  int level;               // 1-based level of this node
  int parent;              // node id of the parent (already in the tree)
  int rank;
  std::vector<int> path;   // ranks from the root's child down to this node
};
struct Worse {
  bool operator()(const Cand& x, const Cand& y) const {
    if (x.p != y.p) return x.p < y.p;
    if (x.level != y.level) return x.level > y.level;
    return x.path > y.path;
  }
};
}  // namespace

extern "C" firp_status firp_build_tree(const float* accept, int32_t k, int32_t b, int32_t n_nodes,
                                       int32_t* parent, int32_t* rank, int32_t* n_out,
                                       double* expected_tokens) {
  if (!accept || !parent || !rank || !n_out) return FIRP_EINVAL;
  if (k < 0 || k > FIRP_MAX_K || b < 1 || b > FIRP_MAX_B || n_nodes < 1) return FIRP_EINVAL;
  for (int i = 0; i < k * b; ++i)
    if (!(accept[i] >= 0.f && accept[i] <= 1.f)) return FIRP_EINVAL;
  std::priority_queue<Cand, std::vector<Cand>, Worse> heap;
  std::vector<std::vector<int>> paths;   // rank path of every chosen node
  std::vector<double> prob;
  parent[0] = -1;
  rank[0] = 0;
  paths.push_back({});
  prob.push_back(1.0);
  int n = 1;
  double expect = 1.0;
  auto push_children = [&](int v) {
    int level = (int)paths[v].size() + 1;
    if (level > k) return;
    for (int r = 0; r < b; ++r) {
      Cand c{prob[v] * (double)accept[(level - 1) * b + r], level, v, r, paths[v]};
      c.path.push_back(r);
      heap.push(c);
    }
  };
  push_children(0);
  while (n < n_nodes && !heap.empty()) {
    Cand c = heap.top();
    heap.pop();
    if (c.p <= 0.0) break;   // a node that is never accepted adds nothing
    parent[n] = c.parent;
    rank[n] = c.rank;
    paths.push_back(c.path);
    prob.push_back(c.p);
    expect += c.p;
    push_children(n);
    ++n;
  }
  *n_out = n;
  if (expected_tokens) *expected_tokens = expect;
  return FIRP_OK;
}
