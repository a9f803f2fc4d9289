#include "model.hpp"

#include <algorithm>
#include <map>
#include <numeric>
#include <set>

namespace fc {

int map_arity(int fn) {
  switch (fn) {
    case FC_FN_IDENT: case FC_FN_AFFINE: case FC_FN_SIN_X_MUL_X: case FC_FN_SQ_PLUS_ONE:
    case FC_FN_EXP_NEG: case FC_FN_MOD_EQ: return 1;
    case FC_FN_MUL2: case FC_FN_ADD2: return 2;
    case FC_FN_ADD3: return 3;
    case FC_FN_ADD5: return 5;
    default: return -1;
  }
}

static bool is_reducer(int fn) { return fn == FC_OP_ADD || fn == FC_OP_MAX || fn == FC_OP_MUL; }

InOrder Model::in_order(int b, int slot) const {
  switch (nodes[b].kind) {
    case FC_MAP: case FC_FOLD: return InOrder::SameAsOut;
    case FC_GATHER: return slot == 0 ? InOrder::SameAsOut : InOrder::Label;
    case FC_FOLDSEG: return slot == 0 ? InOrder::SameAsOut : InOrder::None;
    case FC_SCANL: return InOrder::Zero;
    case FC_SCANR: return InOrder::One;
    case FC_SCATTER: return slot == 0 ? InOrder::None : InOrder::SameAsOut;  // src order, in {0,1}
    default: return InOrder::None;  // force: unordered
  }
}

int build_model(const fc_graph *g, Model &m, std::string &err) {
  if (!g || g->n < 0 || (g->n > 0 && !g->nodes)) { err = "null graph"; return FC_E_ARG; }
  m = Model();
  m.n = g->n;
  m.nodes.assign(g->nodes, g->nodes + g->n);
  m.out_edges.assign(m.n, {});
  m.in_edges.assign(m.n, {});
  m.label.assign(m.n, -1);
  auto bad = [&](int i, const std::string &what) {
    err = "node " + std::to_string(i) + ": " + what;
    return FC_E_BADGRAPH;
  };
  for (int i = 0; i < m.n; ++i) {
    fc_node &nd = m.nodes[i];
    if (nd.kind < FC_INPUT || nd.kind > FC_FORCE) return bad(i, "unknown kind");
    if (nd.dtype != FC_F32 && nd.dtype != FC_I32) return bad(i, "unknown dtype");
    if (nd.rank < 1 || nd.rank > 2) return bad(i, "rank must be 1 or 2");
    if (nd.rank == 1) nd.shape[1] = 1;
    if (nd.shape[0] < 0 || nd.shape[1] < 0) return bad(i, "negative extent");
    if (nd.shape[0] * nd.shape[1] > INT32_MAX) { err = "array above 2^31-1 elements"; return FC_E_LIMIT; }
    if (nd.nargs < 0 || nd.nargs > FC_MAX_ARGS) return bad(i, "bad argument count");
    for (int k = 0; k < nd.nargs; ++k)
      if (nd.arg[k] < 0 || nd.arg[k] >= i) return bad(i, "argument is not an earlier node (graph must be topologically ordered)");
    auto A = [&](int k) -> const fc_node & { return m.nodes[nd.arg[k]]; };
    auto same_shape = [&](const fc_node &o) { return o.shape[0] * o.shape[1] == nd.shape[0] * nd.shape[1]; };
    switch (nd.kind) {
      case FC_INPUT:
        if (nd.nargs != 0) return bad(i, "input takes no arguments");
        break;
      case FC_MAP: {
        int ar = map_arity(nd.fn);
        if (ar < 0) return bad(i, "unknown map function");
        if (nd.nargs != ar) return bad(i, "map arity mismatch");
        for (int k = 0; k < ar; ++k) {
          // zipWith over arrays of different sizes is rejected: the paper would first
          // gather them to a common size (section 2, last paragraph)
          if (!same_shape(A(k))) return bad(i, "map arguments must have the size of the result");
        }
        if (nd.fn == FC_FN_MOD_EQ) {
          if (nd.dtype != FC_I32 || A(0).dtype != FC_I32) return bad(i, "mod_eq is i32 -> i32");
          if (nd.iparam[0] <= 0) return bad(i, "mod_eq needs a positive modulus");
        } else if (nd.fn == FC_FN_IDENT) {
          if (A(0).dtype != nd.dtype) return bad(i, "dtype mismatch");
        } else {
          if (nd.dtype != FC_F32) return bad(i, "this map function is f32 only");
          for (int k = 0; k < ar; ++k) if (A(k).dtype != FC_F32) return bad(i, "dtype mismatch");
        }
        break;
      }
      case FC_GENERATE:
        if (nd.nargs != 0) return bad(i, "generate takes no array arguments");
        if (nd.dtype != FC_I32) return bad(i, "generate produces i32 indices");
        if (nd.fn < FC_FN_IOTA || nd.fn > FC_FN_CONST_I32) return bad(i, "unknown generate function");
        if ((nd.fn == FC_FN_CLAMP_SHIFT_2D || nd.fn == FC_FN_ROW_OF_2D) && nd.rank != 2)
          return bad(i, "2-D index function on a 1-D shape");
        break;
      case FC_GATHER:
        if (nd.nargs != 2) return bad(i, "gather takes (indices, source)");
        if (A(0).dtype != FC_I32) return bad(i, "gather indices must be i32");
        if (!same_shape(A(0))) return bad(i, "gather result has the size of its index array");
        if (A(1).dtype != nd.dtype) return bad(i, "dtype mismatch");
        m.label[i] = 2 + m.n_gathers++;
        break;
      case FC_FOLD:
        if (nd.nargs != 1) return bad(i, "fold takes one array");
        if (!is_reducer(nd.fn)) return bad(i, "unknown reducer");
        if (A(0).dtype != nd.dtype) return bad(i, "dtype mismatch");
        if (!(nd.rank == 1 && nd.shape[0] == 1) &&
            !(A(0).rank == 2 && nd.rank == 1 && nd.shape[0] == A(0).shape[0]))
          return bad(i, "fold result must have shape (1) or the outer extent of a 2-D argument");
        break;
      case FC_FOLDSEG:
        if (nd.nargs != 2) return bad(i, "foldSeg takes (values, offsets)");
        if (!is_reducer(nd.fn)) return bad(i, "unknown reducer");
        if (A(0).dtype != nd.dtype || A(1).dtype != FC_I32) return bad(i, "dtype mismatch");
        if (nd.rank != 1 || A(1).shape[0] * A(1).shape[1] != nd.shape[0] + 1)
          return bad(i, "offsets must have rows+1 entries");
        break;
      case FC_SCANL: case FC_SCANR:
        if (nd.nargs != 1) return bad(i, "scan takes one array");
        if (nd.fn != FC_OP_ADD) return bad(i, "scan supports (+) only");
        if (A(0).dtype != nd.dtype || !same_shape(A(0))) return bad(i, "scan keeps dtype and shape");
        break;
      case FC_SCATTER:
        if (nd.nargs != 3 && nd.nargs != 4) return bad(i, "scatter takes (dest, index, value[, flag])");
        if (nd.fn != FC_OP_OVERWRITE && nd.fn != FC_OP_ADD) return bad(i, "unknown scatter function");
        if (A(0).dtype != nd.dtype || !same_shape(A(0))) return bad(i, "scatter result has dtype and shape of dest");
        if (A(1).dtype != FC_I32 || A(2).dtype != nd.dtype) return bad(i, "dtype mismatch");
        if (A(1).shape[0] * A(1).shape[1] != A(2).shape[0] * A(2).shape[1]) return bad(i, "index and value sizes differ");
        if (nd.nargs == 4 && (A(3).dtype != FC_I32 || A(3).shape[0] * A(3).shape[1] != A(1).shape[0] * A(1).shape[1]))
          return bad(i, "flag must be i32 of the source size");
        // the destination is updated in place while the other arguments are being read
        for (int k = 1; k < nd.nargs; ++k)
          if (nd.arg[k] == nd.arg[0]) return bad(i, "scatter reads its destination as index, value or flag");
        break;
      case FC_FORCE:
        if (nd.nargs != 1) return bad(i, "force takes one array");
        if (A(0).dtype != nd.dtype || !same_shape(A(0))) return bad(i, "force keeps dtype and shape");
        break;
    }
    for (int k = 0; k < nd.nargs; ++k) {
      int a = nd.arg[k];
      int ka = m.nodes[a].kind;
      bool fusible = !(ka == FC_INPUT || ka == FC_FORCE || ka == FC_SCATTER) && nd.kind != FC_FORCE &&
                     !(nd.kind == FC_SCATTER && k == 0) && !(nd.kind == FC_FOLDSEG && k == 1) &&
                     !((nd.infusible_args >> k) & 1u);
      int e = (int)m.edges.size();
      m.edges.push_back({a, i, k, fusible});
      m.out_edges[a].push_back(e);
      m.in_edges[i].push_back(e);
    }
  }
  return FC_OK;
}

namespace {
struct UnionFind {
  std::vector<int> p, konst;  // konst: -1 = none
  explicit UnionFind(int n) : p(n), konst(n, -1) { std::iota(p.begin(), p.end(), 0); }
  int find(int a) { while (p[a] != a) a = p[a] = p[p[a]]; return a; }
  bool set_const(int a, int c) {
    a = find(a);
    if (konst[a] >= 0 && konst[a] != c) return false;
    konst[a] = c;
    return true;
  }
  bool unite(int a, int b) {
    a = find(a); b = find(b);
    if (a == b) return true;
    if (konst[a] >= 0 && konst[b] >= 0 && konst[a] != konst[b]) return false;
    if (konst[a] < 0) konst[a] = konst[b];
    p[b] = a;
    return true;
  }
};
}  // namespace

int derive_and_check(const Model &m, const std::vector<int> &pi, Clustering &c, std::string &err) {
  const int n = m.n;
  if ((int)pi.size() != n) { err = "pi has the wrong length"; return FC_E_ARG; }
  auto illegal = [&](const std::string &s) { err = s; return FC_E_ILLEGAL_PARTITION; };
  c.pi = pi;
  c.x.assign(m.edges.size(), 1);
  c.fused_away.assign(n, 0);
  c.order_out.assign(n, 0);
  c.order_in.assign(m.edges.size(), 0);
  for (int a = 0; a < n; ++a)
    if (pi[a] < 0 || pi[a] > n) return illegal("pi out of [0, n] at node " + std::to_string(a));
  // pi_a <= pi_b, x_ab <= pi_b - pi_a <= n x_ab, x = 1 on infusible edges
  for (size_t e = 0; e < m.edges.size(); ++e) {
    const Edge &ed = m.edges[e];
    if (pi[ed.a] > pi[ed.b])
      return illegal("edge " + std::to_string(ed.a) + "->" + std::to_string(ed.b) + " runs backwards in cluster order");
    c.x[e] = pi[ed.a] != pi[ed.b];
    if (!ed.fusible && !c.x[e])
      return illegal("infusible edge " + std::to_string(ed.a) + "->" + std::to_string(ed.b) + " inside a cluster");
  }
  // temporal uniqueness of scatter: every other use of dest comes strictly earlier
  for (int j = 0; j < n; ++j) {
    if (m.nodes[j].kind != FC_SCATTER) continue;
    int d = m.nodes[j].arg[0];
    for (int e : m.out_edges[d]) {
      int i = m.edges[e].b;
      if (i == j) continue;
      if (!(pi[i] < pi[j]))
        return illegal("node " + std::to_string(i) + " uses the destination of scatter " + std::to_string(j) + " but is not in an earlier cluster");
    }
  }
  // m_a: fused away iff it has consumers, all fused over, and is not a program result
  for (int a = 0; a < n; ++a) {
    bool all_fused = !m.out_edges[a].empty() && !(m.nodes[a].flags & FC_NODE_OUTPUT) && !m.is_input(a);
    for (int e : m.out_edges[a]) all_fused = all_fused && !c.x[e];
    c.fused_away[a] = all_fused;
  }
  // traversal orders: equalities d^o_a = d^i_(b,slot) over fused edges
  UnionFind uf(n);
  for (int a = 0; a < n; ++a) {
    if (m.nodes[a].kind == FC_SCANL && !uf.set_const(a, 0)) return illegal("scanl order");
    if (m.nodes[a].kind == FC_SCANR && !uf.set_const(a, 1)) return illegal("scanr order");
  }
  for (size_t e = 0; e < m.edges.size(); ++e) {
    if (c.x[e]) continue;
    const Edge &ed = m.edges[e];
    bool ok = true;
    switch (m.in_order(ed.b, ed.slot)) {
      case InOrder::SameAsOut: ok = uf.unite(ed.a, ed.b); break;
      case InOrder::Label: ok = uf.set_const(ed.a, m.label[ed.b]); break;
      case InOrder::Zero: ok = uf.set_const(ed.a, 0); break;
      case InOrder::One: ok = uf.set_const(ed.a, 1); break;
      case InOrder::None: ok = false; break;
    }
    if (!ok)
      return illegal("traversal orders conflict on fused edge " + std::to_string(ed.a) + "->" + std::to_string(ed.b));
  }
  // d^o_a <= 1 + g m_a: a manifest array (and the source tuple of a scatter) is produced in order 0 or 1
  for (int a = 0; a < n; ++a) {
    int k = uf.konst[uf.find(a)];
    bool needs01 = !c.fused_away[a] || m.nodes[a].kind == FC_SCATTER;
    if (needs01 && k > 1)
      return illegal("array " + std::to_string(a) + " would be produced in the order of a gather but is not fused away");
  }
  for (int a = 0; a < n; ++a) {
    int k = uf.konst[uf.find(a)];
    c.order_out[a] = k < 0 ? 0 : k;
  }
  for (size_t e = 0; e < m.edges.size(); ++e) {
    const Edge &ed = m.edges[e];
    switch (m.in_order(ed.b, ed.slot)) {
      case InOrder::SameAsOut: c.order_in[e] = c.order_out[ed.b]; break;
      case InOrder::Label: c.order_in[e] = m.label[ed.b]; break;
      case InOrder::Zero: c.order_in[e] = 0; break;
      case InOrder::One: c.order_in[e] = 1; break;
      case InOrder::None: c.order_in[e] = -1 - ed.b; break;  // unordered access: never shared
    }
  }
  return FC_OK;
}

bool orders_completable(const Model &m, const std::vector<int> &block, std::vector<int> *resolved) {
  const int n = m.n;
  UnionFind uf(n);
  for (int a = 0; a < n; ++a) {
    if (block[a] < 0) continue;
    if (m.nodes[a].kind == FC_SCANL && !uf.set_const(a, 0)) return false;
    if (m.nodes[a].kind == FC_SCANR && !uf.set_const(a, 1)) return false;
  }
  for (const Edge &ed : m.edges) {
    if (block[ed.a] < 0 || block[ed.b] < 0 || block[ed.a] != block[ed.b]) continue;
    bool ok = true;
    switch (m.in_order(ed.b, ed.slot)) {
      case InOrder::SameAsOut: ok = uf.unite(ed.a, ed.b); break;
      case InOrder::Label: ok = uf.set_const(ed.a, m.label[ed.b]); break;
      case InOrder::Zero: ok = uf.set_const(ed.a, 0); break;
      case InOrder::One: ok = uf.set_const(ed.a, 1); break;
      case InOrder::None: ok = false; break;
    }
    if (!ok) return false;
  }
  for (int a = 0; a < n; ++a) {
    if (block[a] < 0) continue;
    if (uf.konst[uf.find(a)] <= 1) continue;
    bool manifest = m.nodes[a].kind == FC_SCATTER || m.out_edges[a].empty() || (m.nodes[a].flags & FC_NODE_OUTPUT);
    for (int e : m.out_edges[a]) {
      const int b = m.edges[e].b;
      manifest = manifest || (block[b] >= 0 && block[b] != block[a]);
    }
    if (manifest) return false;
  }
  if (resolved) {
    resolved->assign(n, -1);
    for (int a = 0; a < n; ++a) if (block[a] >= 0) (*resolved)[a] = uf.konst[uf.find(a)];
  }
  return true;
}

double evaluate_cost(const Model &m, const Clustering &c, int cost_fn) {
  const int n = m.n;
  auto reads = [&](bool weighted) {
    double total = 0;
    for (int a = 0; a < n; ++a) {
      std::set<std::pair<int, int>> keys;  // (consuming cluster, order)
      for (int e : m.out_edges[a])
        if (c.x[e]) keys.insert({c.pi[m.edges[e].b], c.order_in[e]});
      total += (double)keys.size() * (weighted ? (double)m.bytes(a) : 1.0);
    }
    return total;
  };
  auto writes = [&](bool weighted) {
    double total = 0;
    for (int a = 0; a < n; ++a)
      if (!m.is_input(a) && !c.fused_away[a]) total += weighted ? (double)m.bytes(a) : 1.0;
    return total;
  };
  switch (cost_fn) {
    case FC_COST_CLUSTERS: {
      std::set<int> levels;
      for (int a = 0; a < n; ++a) if (!m.is_input(a)) levels.insert(c.pi[a]);
      return (double)levels.size();
    }
    case FC_COST_FUSED_EDGES: {
      double s = 0;
      for (size_t e = 0; e < m.edges.size(); ++e) if (m.edges[e].fusible) s += c.x[e];
      return s;
    }
    case FC_COST_ARRAYS: return writes(false);
    case FC_COST_READS: return reads(false);
    case FC_COST_READS_WRITES: return reads(false) + writes(false);
    case FC_COST_BYTES: return reads(true) + writes(true);
    default: return -1.0;
  }
}

int renumber_levels(const Model &m, Clustering &c) {
  std::map<int, int> remap;
  for (int a = 0; a < m.n; ++a) if (!m.is_input(a)) remap[c.pi[a]] = 0;
  int k = 0;
  for (auto &kv : remap) kv.second = ++k;
  for (int a = 0; a < m.n; ++a) c.pi[a] = m.is_input(a) ? 0 : remap[c.pi[a]];
  return k;
}

int split_components(const Model &m, Clustering &c) {
  const int n = m.n;
  // union nodes of one level that are joined by a fused edge or read the same
  // parent array in the same traversal order
  std::vector<int> comp(n);
  std::iota(comp.begin(), comp.end(), 0);
  auto find = [&](int a) { while (comp[a] != a) a = comp[a] = comp[comp[a]]; return a; };
  auto unite = [&](int a, int b) { a = find(a); b = find(b); if (a != b) comp[std::max(a, b)] = std::min(a, b); };
  for (size_t e = 0; e < m.edges.size(); ++e)
    if (!c.x[e]) unite(m.edges[e].a, m.edges[e].b);
  for (int a = 0; a < n; ++a) {
    std::map<std::pair<int, int>, int> first;  // (level, order) -> a consumer
    for (int e : m.out_edges[a]) {
      if (!c.x[e] || c.order_in[e] < 0) continue;
      int b = m.edges[e].b;
      auto key = std::make_pair(c.pi[b], c.order_in[e]);
      auto it = first.find(key);
      if (it == first.end()) first[key] = b; else unite(it->second, b);
    }
  }
  // order the components: by level, then by smallest member
  std::map<std::pair<int, int>, int> ids;
  for (int a = 0; a < n; ++a) if (!m.is_input(a)) ids[{c.pi[a], find(a)}] = 0;
  int k = 0;
  for (auto &kv : ids) kv.second = ++k;
  for (int a = 0; a < n; ++a) c.pi[a] = m.is_input(a) ? 0 : ids[{c.pi[a], find(a)}];
  for (size_t e = 0; e < m.edges.size(); ++e) c.x[e] = c.pi[m.edges[e].a] != c.pi[m.edges[e].b];
  return k;
}

}  // namespace fc
