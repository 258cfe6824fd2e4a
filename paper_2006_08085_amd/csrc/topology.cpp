// Host-side construction and validation of the gossip matrix W, its spectrum
// and the acceleration parameter eta.  No device code here.
//
// Paper: the gossip matrix class W_n and lambda = max(|lambda_2|, |lambda_n|)
// are defined in the "Protocol Layer" subsection; eta is the second line of
// Algorithm 3; the slack matrix W_kappa is in the "Experiments" section.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <limits>
#include <map>
#include <queue>
#include <set>
#include <utility>

#include "detag_internal.h"

namespace detag {
namespace {

using Edge = std::pair<int, int>;

struct SplitMix64 {
  uint64_t s;
  explicit SplitMix64(uint64_t seed) : s(seed) {}
  uint64_t next() {
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  // unbiased integer in [0, m)
  uint64_t below(uint64_t m) {
    const uint64_t lim = std::numeric_limits<uint64_t>::max() - std::numeric_limits<uint64_t>::max() % m;
    uint64_t r;
    do r = next(); while (r >= lim);
    return r % m;
  }
};

Edge norm_edge(int a, int b) { return a < b ? Edge(a, b) : Edge(b, a); }

bool edges_ring(int n, std::set<Edge> &e) {
  for (int i = 0; n >= 2 && i < n; ++i)
    if ((i + 1) % n != i) e.insert(norm_edge(i, (i + 1) % n));
  return true;
}

bool edges_torus(int rows, int cols, std::set<Edge> &e) {
  for (int r = 0; r < rows; ++r)
    for (int c = 0; c < cols; ++c) {
      const int v = r * cols + c;
      const int down = ((r + 1) % rows) * cols + c, right = r * cols + (c + 1) % cols;
      if (down != v) e.insert(norm_edge(v, down));
      if (right != v) e.insert(norm_edge(v, right));
    }
  return true;
}

// Union of degree/2 random Hamiltonian cycles, redrawn until no edge repeats:
// simple, `degree`-regular and connected by construction.
bool edges_random_regular(int n, int degree, uint64_t seed, std::set<Edge> &e, std::string &err) {
  if (degree < 2 || degree % 2 || n <= degree) {
    err = "random regular graph needs an even degree >= 2 and n > degree";
    return false;
  }
  SplitMix64 rng(seed ^ 0xD1B54A32D192ED03ull);
  std::vector<int> p(n);
  for (int attempt = 0; attempt < 100000; ++attempt) {
    e.clear();
    bool ok = true;
    for (int cyc = 0; cyc < degree / 2 && ok; ++cyc) {
      for (int i = 0; i < n; ++i) p[i] = i;
      for (int i = n - 1; i > 0; --i) std::swap(p[i], p[rng.below(uint64_t(i) + 1)]);
      for (int i = 0; i < n && ok; ++i) ok = e.insert(norm_edge(p[i], p[(i + 1) % n])).second;
    }
    if (ok) return true;
  }
  err = "could not draw a simple random regular graph";
  return false;
}

bool fail(std::string &err, const char *msg) {
  err = msg;
  return false;
}

// Dense symmetric W from an undirected edge set.
bool weights_from_edges(int n, const std::set<Edge> &edges, int kind, std::vector<double> &W, std::string &err) {
  W.assign(size_t(n) * n, 0.0);
  if (n == 1) {
    W[0] = 1.0;
    return true;
  }
  std::vector<int> deg(n, 0);
  for (const Edge &ed : edges) {
    ++deg[ed.first];
    ++deg[ed.second];
  }
  if (kind == DETAG_W_UNIFORM) {
    for (int i = 1; i < n; ++i)
      if (deg[i] != deg[0]) return fail(err, "uniform weights need a regular graph; use DETAG_W_METROPOLIS");
    const double w = 1.0 / (deg[0] + 1.0);
    for (const Edge &ed : edges) W[size_t(ed.first) * n + ed.second] = W[size_t(ed.second) * n + ed.first] = w;
    for (int i = 0; i < n; ++i) W[size_t(i) * n + i] = w;
  } else if (kind == DETAG_W_METROPOLIS) {
    for (const Edge &ed : edges) {
      const double w = 1.0 / (1.0 + std::max(deg[ed.first], deg[ed.second]));
      W[size_t(ed.first) * n + ed.second] = W[size_t(ed.second) * n + ed.first] = w;
    }
    for (int i = 0; i < n; ++i) {
      double off = 0;
      for (int j = 0; j < n; ++j)
        if (j != i) off += W[size_t(i) * n + j];
      W[size_t(i) * n + i] = 1.0 - off;
    }
  } else {
    return fail(err, "unknown weight kind");
  }
  return true;
}

}  // namespace

// Cyclic Jacobi: rotate away every off-diagonal pair until the off-diagonal
// mass is at rounding level.  O(n^3) per sweep, n is at most a few hundred.
void symmetric_eigenvalues(std::vector<double> &a, int n, std::vector<double> &ev) {
  auto A = [&](int i, int j) -> double & { return a[size_t(i) * n + j]; };
  for (int sweep = 0; sweep < 60; ++sweep) {
    double off = 0, diag = 0;
    for (int i = 0; i < n; ++i) {
      diag += A(i, i) * A(i, i);
      for (int j = i + 1; j < n; ++j) off += A(i, j) * A(i, j);
    }
    if (off <= 1e-32 * (diag + 1e-300)) break;
    for (int p = 0; p < n - 1; ++p)
      for (int q = p + 1; q < n; ++q) {
        const double apq = A(p, q);
        if (std::fabs(apq) < 1e-300) continue;
        const double theta = (A(q, q) - A(p, p)) / (2.0 * apq);
        const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
        const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
        for (int k = 0; k < n; ++k) {  // columns p, q
          const double akp = A(k, p), akq = A(k, q);
          A(k, p) = c * akp - s * akq;
          A(k, q) = s * akp + c * akq;
        }
        for (int k = 0; k < n; ++k) {  // rows p, q
          const double apk = A(p, k), aqk = A(q, k);
          A(p, k) = c * apk - s * aqk;
          A(q, k) = s * apk + c * aqk;
        }
      }
  }
  ev.resize(n);
  for (int i = 0; i < n; ++i) ev[i] = A(i, i);
  std::sort(ev.begin(), ev.end());
}

detag_status build_gossip_matrix(const detag_topology *topo, int n, HostW &out, std::string &err) {
  if (!topo) return err = "topology is NULL", DETAG_EINVAL;
  if (n < 1) return err = "n must be >= 1", DETAG_EINVAL;
  if (!(topo->kappa > 0.0 && topo->kappa <= 1.0)) return err = "kappa must be in (0, 1]", DETAG_EINVAL;
  const double kappa = topo->kappa;

  // ---- W as a list of (i, j, W_ji) triplets: row i of the CSR ----------------
  std::vector<std::map<int, double>> rows(n);
  std::set<Edge> edges;
  bool from_graph = true;
  switch (topo->kind) {
    case DETAG_TOPO_RING:
      edges_ring(n, edges);
      break;
    case DETAG_TOPO_TORUS2D:
      if (topo->rows < 1 || topo->cols < 1 || int64_t(topo->rows) * topo->cols != n)
        return err = "torus needs rows*cols == n", DETAG_EINVAL;
      edges_torus(topo->rows, topo->cols, edges);
      break;
    case DETAG_TOPO_RANDOM_REGULAR:
      if (!edges_random_regular(n, topo->degree, topo->seed, edges, err)) return DETAG_EINVAL;
      break;
    case DETAG_TOPO_EDGES: {
      if (topo->n_edges < 0 || (topo->n_edges > 0 && !topo->edges))
        return err = "edge list is NULL", DETAG_EINVAL;
      for (int64_t k = 0; k < topo->n_edges; ++k) {
        const int a = topo->edges[2 * k], b = topo->edges[2 * k + 1];
        if (a < 0 || b < 0 || a >= n || b >= n || a == b)
          return err = "edge endpoint out of range or a self-loop", DETAG_EINVAL;
        if (!edges.insert(norm_edge(a, b)).second) return err = "repeated edge", DETAG_EINVAL;
      }
      break;
    }
    case DETAG_TOPO_CSR: {
      from_graph = false;
      if (!topo->rowptr || !topo->colidx || !topo->vals) return err = "CSR arrays are NULL", DETAG_EINVAL;
      if (topo->rowptr[0] != 0) return err = "rowptr[0] must be 0", DETAG_EINVAL;
      for (int i = 0; i < n; ++i) {
        if (topo->rowptr[i + 1] < topo->rowptr[i]) return err = "rowptr must not decrease", DETAG_EINVAL;
        for (int k = topo->rowptr[i]; k < topo->rowptr[i + 1]; ++k) {
          const int j = topo->colidx[k];
          if (j < 0 || j >= n) return err = "CSR column index out of range", DETAG_EINVAL;
          if (!rows[i].emplace(j, topo->vals[k]).second) return err = "repeated CSR entry", DETAG_EINVAL;
        }
      }
      break;
    }
    default:
      return err = "unknown topology kind", DETAG_EINVAL;
  }
  if (from_graph) {
    std::vector<double> Wd;
    if (!weights_from_edges(n, edges, topo->weights, Wd, err)) return DETAG_EINVAL;
    for (int i = 0; i < n; ++i)
      for (int j = 0; j < n; ++j)
        if (Wd[size_t(j) * n + i] != 0.0) rows[i][j] = Wd[size_t(j) * n + i];
  }
  if (kappa != 1.0)
    for (int i = 0; i < n; ++i) {
      for (auto &kv : rows[i]) kv.second *= kappa;
      rows[i][i] += 1.0 - kappa;
    }

  // ---- checks: membership in the gossip matrix class -----------------------
  std::vector<double> colsum(n, 0.0), rowsum(n, 0.0);
  for (int i = 0; i < n; ++i)
    for (const auto &kv : rows[i]) {
      if (!(kv.second >= 0.0) || !std::isfinite(kv.second))
        return err = "W has a negative or non-finite weight", DETAG_ENOT_DOUBLY_STOCHASTIC;
      colsum[i] += kv.second;         // sum_j W_ji : column i of W
      rowsum[kv.first] += kv.second;  // sum_i W_ji : row j of W
    }
  for (int i = 0; i < n; ++i)
    if (std::fabs(colsum[i] - 1.0) > 1e-9 || std::fabs(rowsum[i] - 1.0) > 1e-9) {
      char buf[160];
      std::snprintf(buf, sizeof buf, "W is not doubly stochastic: worker %d has column sum %.12g, row sum %.12g", i,
                    colsum[i], rowsum[i]);
      return err = buf, DETAG_ENOT_DOUBLY_STOCHASTIC;
    }
  {  // connectivity of the undirected support
    std::vector<std::vector<int>> adj(n);
    for (int i = 0; i < n; ++i)
      for (const auto &kv : rows[i])
        if (kv.first != i && kv.second != 0.0) {
          adj[i].push_back(kv.first);
          adj[kv.first].push_back(i);
        }
    std::vector<char> seen(n, 0);
    std::queue<int> q;
    q.push(0);
    seen[0] = 1;
    int cnt = 1;
    while (!q.empty()) {
      const int v = q.front();
      q.pop();
      for (int w : adj[v])
        if (!seen[w]) seen[w] = 1, ++cnt, q.push(w);
    }
    if (cnt != n) return err = "the graph of W is not connected (lambda = 1)", DETAG_EDISCONNECTED;
  }

  // ---- CSR ------------------------------------------------------------------
  out = HostW();
  out.n = n;
  out.rowptr.assign(1, 0);
  for (int i = 0; i < n; ++i) {
    for (const auto &kv : rows[i])
      if (kv.second != 0.0 || kv.first == i) {
        out.colidx.push_back(kv.first);
        out.vals.push_back(kv.second);
      }
    out.rowptr.push_back(int32_t(out.colidx.size()));
    out.max_row_nnz = std::max(out.max_row_nnz, out.rowptr[i + 1] - out.rowptr[i]);
  }

  // ---- spectrum and eta --------------------------------------------------------
  std::vector<double> dense(size_t(n) * n, 0.0);
  for (int i = 0; i < n; ++i)
    for (const auto &kv : rows[i]) dense[size_t(kv.first) * n + i] = kv.second;  // W[j][i]
  out.symmetric = true;
  for (int i = 0; i < n && out.symmetric; ++i)
    for (int j = i + 1; j < n; ++j)
      if (std::fabs(dense[size_t(i) * n + j] - dense[size_t(j) * n + i]) > 1e-12) {
        out.symmetric = false;
        break;
      }
  const double nan = std::numeric_limits<double>::quiet_NaN();
  if (n == 1) {
    out.lambda2 = out.lambdan = out.lambda = out.eta = 0.0;
  } else if (out.symmetric) {
    std::vector<double> ev;
    symmetric_eigenvalues(dense, n, ev);
    out.lambda2 = ev[n - 2];
    out.lambdan = ev[0];
    out.lambda = std::max(std::fabs(out.lambda2), std::fabs(out.lambdan));
    if (out.lambda >= 1.0 - 1e-12)
      return err = "lambda = max(|lambda_2|,|lambda_n|) is 1: W does not contract (periodic or disconnected)",
             DETAG_EDISCONNECTED;
    const double s = std::sqrt(1.0 - out.lambda * out.lambda);
    out.eta = (1.0 - s) / (1.0 + s);
  } else {
    out.lambda2 = out.lambdan = out.lambda = out.eta = nan;
  }

  // ---- structured patterns for the register-resident kernels ----------------
  // (on these regular graphs both weight rules give 1/(deg+1))
  if (from_graph) {
    if (topo->kind == DETAG_TOPO_RING && n >= 3) {
      out.structure = kRing;
      out.w_nb = kappa / 3.0;
      out.w_self = kappa / 3.0 + (1.0 - kappa);
    } else if (topo->kind == DETAG_TOPO_TORUS2D && topo->rows >= 3 && topo->cols >= 3) {
      out.structure = kTorus;
      out.trows = topo->rows;
      out.tcols = topo->cols;
      out.w_nb = kappa / 5.0;
      out.w_self = kappa / 5.0 + (1.0 - kappa);
    }
  }
  return DETAG_OK;
}

}  // namespace detag
