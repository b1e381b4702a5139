// Extraction step of operator fusion (paper Section 4.1, "Extraction").
//
// The dataflow DAG is acyclic, so its post-dominator tree is built in one sweep against the
// direction of the data: the immediate post-dominator of an operator is the lowest common
// ancestor, in the tree built so far, of the operators that read it (an operator nobody
// reads hangs under a virtual exit).  Groups are then formed in dataflow order: an operator
// joins its immediate post-dominator, and takes every operator on the paths between them
// along, when
//   - all those operators (the post-dominator included) are elementwise/broadcast, so that
//     neither an opaque operator nor a second contraction is swallowed, and
//   - the united group keeps at most one contraction.
// Opaque operators stay alone.  Because the post-dominator is where all paths out of the
// operator meet, a group built this way has exactly one operator that is read from outside
// (its last one): the body of one primitive function with one result.  This is also what
// fuses diamonds: a fork whose branches are elementwise joins the group at the merge point.
#include "fusion.hpp"

#include <algorithm>

namespace relay {
namespace {

struct UnionFind {
  std::vector<int32_t> parent, smallest, contractions;
  explicit UnionFind(int32_t n) : parent(n), smallest(n), contractions(n, 0) {
    for (int32_t i = 0; i < n; ++i) parent[i] = smallest[i] = i;
  }
  int32_t find(int32_t x) {
    while (parent[x] != x) {
      parent[x] = parent[parent[x]];
      x = parent[x];
    }
    return x;
  }
  void unite(int32_t a, int32_t b) {
    a = find(a);
    b = find(b);
    if (a == b) return;
    parent[b] = a;
    smallest[a] = std::min(smallest[a], smallest[b]);
    contractions[a] += contractions[b];
  }
};

}  // namespace

void fuse_extract(int32_t n, const int32_t* pattern, const int32_t* in_offsets, const int32_t* in_nodes,
                  std::vector<int32_t>& ipdom, std::vector<int32_t>& group) {
  // consumers in CSR form
  std::vector<int32_t> c_off(n + 1, 0);
  for (int32_t e = 0; e < in_offsets[n]; ++e) ++c_off[in_nodes[e] + 1];
  for (int32_t i = 0; i < n; ++i) c_off[i + 1] += c_off[i];
  std::vector<int32_t> c_nodes(in_offsets[n]), fill(c_off.begin(), c_off.end() - 1);
  for (int32_t i = 0; i < n; ++i)
    for (int32_t e = in_offsets[i]; e < in_offsets[i + 1]; ++e) c_nodes[fill[in_nodes[e]]++] = i;

  // post-dominator tree: node n stands for the exit while the tree is built
  ipdom.assign(n, kExit);
  std::vector<int32_t> up(n + 1, n), depth(n + 1, 0);
  auto lca = [&](int32_t a, int32_t b) {
    while (a != b) {
      if (depth[a] < depth[b]) std::swap(a, b);
      a = up[a];
    }
    return a;
  };
  for (int32_t i = n - 1; i >= 0; --i) {
    int32_t d = n;
    if (c_off[i] < c_off[i + 1]) {
      d = c_nodes[c_off[i]];
      for (int32_t e = c_off[i] + 1; e < c_off[i + 1] && d != n; ++e) d = lca(d, c_nodes[e]);
    }
    up[i] = d;
    depth[i] = depth[d] + 1;
    ipdom[i] = d == n ? kExit : d;
  }

  // groups
  UnionFind uf(n);
  for (int32_t i = 0; i < n; ++i) uf.contractions[i] = pattern[i] == PAT_CONTRACTION ? 1 : 0;
  std::vector<int32_t> mark(n, -1), stack, on_paths, roots;
  for (int32_t i = 0; i < n; ++i) {
    const int32_t d = ipdom[i];
    if (pattern[i] == PAT_OPAQUE || d == kExit) continue;
    // operators on the paths i -> d: everything reachable from i, stopping at d (every path
    // out of i runs through d, so the walk cannot leave the region between them)
    bool ok = true;
    on_paths.clear();
    stack.assign(1, i);
    mark[i] = i;
    while (!stack.empty() && ok) {
      const int32_t u = stack.back();
      stack.pop_back();
      for (int32_t e = c_off[u]; e < c_off[u + 1]; ++e) {
        const int32_t v = c_nodes[e];
        if (mark[v] == i) continue;
        mark[v] = i;
        if (pattern[v] != PAT_ELEMWISE) {
          ok = false;
          break;
        }
        on_paths.push_back(v);
        if (v != d) stack.push_back(v);
      }
    }
    if (!ok) continue;
    // contractions of the united group: count every distinct group once
    roots.assign(1, uf.find(i));
    int32_t total = uf.contractions[roots[0]];
    bool fits = true;
    for (int32_t v : on_paths) {
      const int32_t r = uf.find(v);
      if (std::find(roots.begin(), roots.end(), r) != roots.end()) continue;
      roots.push_back(r);
      total += uf.contractions[r];
      if (total > 1) {
        fits = false;
        break;
      }
    }
    if (!fits) continue;
    for (int32_t v : on_paths) uf.unite(i, v);
  }
  group.resize(n);
  for (int32_t i = 0; i < n; ++i) group[i] = uf.smallest[uf.find(i)];
}

}  // namespace relay
