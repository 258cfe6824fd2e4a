// Exact average consensus on the context's graph as a short sequence of sparse
// matrices (Lemma 1 of the paper): the spanning-tree construction its
// supplementary material describes under the name GATHER-PROPAGATE.
//
// A breadth-first spanning tree is grown from the chosen root.  Gather: level by
// level from the deepest, every node adds what it holds to its parent and keeps
// nothing, so after depth steps the root holds the sum.  Propagate: level by
// level from the root, a node that holds d_u averages' worth (d_u = size of its
// subtree) keeps one and hands d_v to each child v.  Each step only moves values
// along tree edges, so every matrix has the graph's sparsity; there are
// R = 2*depth of them, between D and 2D for a graph of diameter D.
#include <algorithm>
#include <deque>

#include "detag_internal.h"

namespace detag {

bool build_consensus_factors(const HostW &W, int root, std::vector<HostFactor> &out, std::string &err) {
  const int n = W.n;
  out.clear();
  if (root < 0 || root >= n) return err = "root is not a worker index", false;
  // undirected support of W's off-diagonal entries
  std::vector<std::vector<int>> adj(n);
  for (int i = 0; i < n; ++i)
    for (int k = W.rowptr[i]; k < W.rowptr[i + 1]; ++k) {
      const int j = W.colidx[k];
      if (j != i && W.vals[k] != 0.0) adj[i].push_back(j), adj[j].push_back(i);
    }
  for (auto &a : adj) {
    std::sort(a.begin(), a.end());
    a.erase(std::unique(a.begin(), a.end()), a.end());
  }
  std::vector<int> parent(n, -1), level(n, -1);
  std::deque<int> q{root};
  level[root] = 0;
  int depth = 0;
  while (!q.empty()) {
    const int u = q.front();
    q.pop_front();
    for (int v : adj[u])
      if (level[v] < 0) {
        level[v] = level[u] + 1, parent[v] = u;
        depth = std::max(depth, level[v]);
        q.push_back(v);
      }
  }
  for (int v = 0; v < n; ++v)
    if (level[v] < 0) return err = "the graph is not connected", false;
  std::vector<int64_t> size(n, 1);
  for (int lv = depth; lv >= 1; --lv)
    for (int v = 0; v < n; ++v)
      if (level[v] == lv) size[parent[v]] += size[v];

  // rows[i] = list of (j, A_ij), j ascending
  auto emit = [&](const std::vector<std::vector<std::pair<int, double>>> &rows) {
    HostFactor f;
    f.rowptr.assign(n + 1, 0);
    for (int i = 0; i < n; ++i) {
      auto r = rows[i];
      std::sort(r.begin(), r.end());
      for (auto &e : r) f.colidx.push_back(e.first), f.vals.push_back(e.second);
      f.rowptr[i + 1] = int32_t(f.colidx.size());
    }
    out.push_back(std::move(f));
  };
  for (int lv = depth; lv >= 1; --lv) {  // gather
    std::vector<std::vector<std::pair<int, double>>> rows(n);
    for (int v = 0; v < n; ++v) {
      if (level[v] == lv) rows[parent[v]].push_back({v, 1.0});  // and v itself keeps nothing: empty row
      else rows[v].push_back({v, 1.0});
    }
    emit(rows);
  }
  for (int lv = 0; lv < depth; ++lv) {  // propagate
    std::vector<std::vector<std::pair<int, double>>> rows(n);
    std::vector<char> has_child(n, 0);
    for (int v = 0; v < n; ++v)
      if (level[v] == lv + 1) has_child[parent[v]] = 1;
    for (int v = 0; v < n; ++v) {
      if (level[v] == lv + 1) rows[v].push_back({parent[v], double(size[v]) / double(size[parent[v]])});
      else if (level[v] == lv && has_child[v]) rows[v].push_back({v, 1.0 / double(size[v])});
      else rows[v].push_back({v, 1.0});
    }
    emit(rows);
  }
  return true;
}

}  // namespace detag
