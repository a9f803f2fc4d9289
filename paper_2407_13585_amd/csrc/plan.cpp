// The chooser: exact solution of the clustering ILP (Fig. "Total ILP
// formulation") by branch and bound, and the work-duplication rewrite.
//
// A feasible point of the ILP is fixed by pi alone: x_ab = [pi_a != pi_b],
// m_a = 1 exactly when every edge out of a is fused over (any other choice is
// never better for the cost functions of section 4.1), and the traversal orders
// follow from the equalities over fused edges.  The search therefore enumerates
// the level sets of pi -- set partitions of the non-input nodes, built in
// program order -- and prunes with a lower bound of the cost that holds for every
// completion.  The numerical values of pi are irrelevant beyond their order
// (section 5.2), so blocks are numbered by a topological order of the quotient
// graph at the leaves.
#include "plan.hpp"

#include <algorithm>
#include <chrono>
#include <map>
#include <set>

namespace fc {

namespace {

constexpr int kCosts = FC_COST_BYTES + 1;

struct Search {
  const Model &m;
  double weight[kCosts];           // the objective is sum_k weight[k] * cost_k; one cost function = a unit vector
  std::vector<int> order;          // non-input nodes in program order
  std::vector<int> block;          // per node, -1 = unassigned (inputs: -2)
  int n_blocks = 0;
  double best = 1e300;
  std::vector<int> best_pi;
  long long visited = 0;
  long long limit;
  bool aborted = false;
  std::vector<int> forced;         // per node: representative of the set it must share a cluster with
  bool stop_at_first = false;      // feasibility question only
  double seconds = 0;                       // wall-clock limit of the search, 0 = none
  double share = 1.0;                       // the part of it the running phase may use up to
  bool timed_out = false;                   // the search ended on the clock (not on the node limit)
  std::vector<int> moved_block;             // the clustering the local improvement has reached, to go on from
  int moved_n_blocks = 0;
  std::chrono::steady_clock::time_point started = std::chrono::steady_clock::now();
  const Admissible *admissible = nullptr;   // extra condition on complete clusterings
  bool split = true;                        // it is judged after the connected-component split
  // block graph: adj[b] = bitmask of blocks that must run strictly after b
  std::vector<uint64_t> adj;

  Search(const Model &m_, const double *w, long long lim) : m(m_), block(m_.n, -1), limit(lim), adj(64, 0) {
    for (int k = 0; k < kCosts; ++k) weight[k] = w[k];
    for (int a = 0; a < m.n; ++a) {
      if (m.is_input(a)) block[a] = -2; else order.push_back(a);
    }
    forced.resize(m.n);
    for (int a = 0; a < m.n; ++a) forced[a] = a;
    // What an array costs whatever the clustering: a write if it cannot be fused away, and then at least
    // one read unless it is manifest only for being a result; an input is read once per traversal order
    // asked of it.  An array cannot be fused away if it is a result or has no consumer, if an edge out
    // of it is infusible, or if its consumers cannot all read it in the one order it would be produced
    // in: two different fixed orders (a scan from the left and one from the right, the sources of two
    // gathers), a fixed order other than the scan's own for a scan result, or the source of a gather
    // next to a consumer that reads in its own order and is itself manifest for sure (a manifest array is
    // in order 0 or 1, a gather's source is read in the gather's label).  Consumers come later in
    // program order, so one pass from the back knows each consumer's status.
    sure_write.assign(m.n, 0);
    sure_reads.assign(m.n, 0);
    for (int a = m.n - 1; a >= 0; --a) {
      std::vector<int> fixed;                        // distinct constant orders among the consumers
      bool infusible = false, low = false;           // low: some consumer reads it in order 0 or 1, whichever
      for (int e : m.out_edges[a]) {
        const Edge &ed = m.edges[e];
        infusible = infusible || !ed.fusible;
        int k = -1;
        switch (m.in_order(ed.b, ed.slot)) {
          case InOrder::Label: k = m.label[ed.b]; break;
          case InOrder::Zero: k = 0; break;
          case InOrder::One: k = 1; break;
          case InOrder::SameAsOut: low = low || sure_write[ed.b]; break;
          default: break;
        }
        if (k >= 0 && std::find(fixed.begin(), fixed.end(), k) == fixed.end()) fixed.push_back(k);
      }
      int labels = 0, zero_one = 0;
      for (int k : fixed) if (k >= 2) ++labels; else ++zero_one;
      if (m.is_input(a)) {
        sure_reads[a] = m.out_edges[a].empty() ? 0 : std::max(1, labels + std::max(zero_one, low ? 1 : 0));
      } else {
        const int made = m.nodes[a].kind == FC_SCANL ? 0 : m.nodes[a].kind == FC_SCANR ? 1 : -1;
        bool clash = fixed.size() > 1 || (low && labels > 0);
        if (made >= 0) for (int k : fixed) clash = clash || k != made;
        const bool result = m.out_edges[a].empty() || (m.nodes[a].flags & FC_NODE_OUTPUT);
        const bool split = infusible || clash;
        sure_write[a] = result || split;
        sure_reads[a] = split ? 1 : 0;
      }
    }
  }
  std::vector<char> sure_write;
  std::vector<int> resolved;       // per placed node: the constant its order is tied to, -1 if none (empty: not computed)
  std::vector<int> sure_reads;

  int forced_root(int a) const { while (forced[a] != a) a = forced[a]; return a; }
  void force_together(int a, int b) {
    a = forced_root(a); b = forced_root(b);
    if (a != b) forced[std::max(a, b)] = std::min(a, b);
  }

  bool reaches(int from, int to) const {
    uint64_t seen = 0, frontier = 1ull << from;
    while (frontier) {
      int b = __builtin_ctzll(frontier);
      frontier &= frontier - 1;
      if (seen >> b & 1) continue;
      seen |= 1ull << b;
      if (adj[b] >> to & 1) return true;
      frontier |= adj[b] & ~seen;
    }
    return false;
  }

  // cost of the decisions taken so far; never above the cost of any completion (every
  // cost function only grows as nodes are placed, and the weights are not negative)
  static constexpr int kMaxTracked = 48;      // reader blocks and known orders tracked per array; more only loosen the bound
  double lower_bound() const {
    double reads = 0, writes = 0, unfused = 0, bytes = 0;
    for (int a = 0; a < m.n; ++a) {
      if (block[a] == -1) {
        // not placed yet: what it costs whatever happens
        writes += sure_write[a];
        reads += sure_reads[a];
        bytes += (double)m.bytes(a) * (sure_write[a] + sure_reads[a]);
        continue;
      }
      // A block reads the array once per traversal order it asks for.  Orders known by now: the fixed ones
      // (a gather's source, a scan's argument) and those of consumers whose own order is tied to a constant;
      // a consumer whose order nothing ties yet may still come to share a read with any of them.
      int n_readers = 0, reader[kMaxTracked], n_known = 0, known_block[kMaxTracked], known_order[kMaxTracked];
      bool manifest = !m.is_input(a) && (m.out_edges[a].empty() || (m.nodes[a].flags & FC_NODE_OUTPUT));
      int untracked = 0;
      for (int e : m.out_edges[a]) {
        const Edge &ed = m.edges[e];
        const int rb = block[ed.b];
        if (rb < 0 || rb == block[a]) continue;
        if (!m.is_input(a)) manifest = true;
        if (ed.fusible) unfused += 1;
        bool seen = false;
        for (int i = 0; i < n_readers; ++i) seen = seen || reader[i] == rb;
        if (!seen) { if (n_readers < kMaxTracked) reader[n_readers++] = rb; else ++untracked; }
        int k = -1;
        switch (m.in_order(ed.b, ed.slot)) {
          case InOrder::Label: k = m.label[ed.b]; break;
          case InOrder::Zero: k = 0; break;
          case InOrder::One: k = 1; break;
          case InOrder::SameAsOut: k = resolved.empty() ? -1 : resolved[ed.b]; break;
          default: break;
        }
        if (k < 0 || n_known == kMaxTracked) continue;
        bool have = false;
        for (int i = 0; i < n_known; ++i) have = have || (known_block[i] == rb && known_order[i] == k);
        if (!have) { known_block[n_known] = rb; known_order[n_known] = k; ++n_known; }
      }
      int r = untracked;
      for (int i = 0; i < n_readers; ++i) {
        int distinct = 0;
        for (int j = 0; j < n_known; ++j) distinct += known_block[j] == reader[i];
        r += std::max(1, distinct);
      }
      r = std::max(r, sure_reads[a]);
      manifest = manifest || sure_write[a];
      reads += r;
      if (manifest) writes += 1;
      bytes += (double)m.bytes(a) * (r + (manifest ? 1 : 0));
    }
    return weight[FC_COST_CLUSTERS] * n_blocks + weight[FC_COST_FUSED_EDGES] * unfused + weight[FC_COST_ARRAYS] * writes +
           weight[FC_COST_READS] * reads + weight[FC_COST_READS_WRITES] * (reads + writes) + weight[FC_COST_BYTES] * bytes;
  }

  double objective(const Clustering &c) const {
    double v = 0;
    for (int k = 0; k < kCosts; ++k) if (weight[k] != 0) v += weight[k] * evaluate_cost(m, c, k);
    return v;
  }

  void leaf() {
    // number the blocks in a topological order of the block graph
    std::vector<int> indeg(n_blocks, 0), topo;
    for (int b = 0; b < n_blocks; ++b)
      for (int d = 0; d < n_blocks; ++d) if (adj[b] >> d & 1) ++indeg[d];
    std::vector<int> ready;
    for (int b = n_blocks - 1; b >= 0; --b) if (!indeg[b]) ready.push_back(b);
    while (!ready.empty()) {
      int b = ready.back();
      ready.pop_back();
      topo.push_back(b);
      for (int d = n_blocks - 1; d >= 0; --d) if ((adj[b] >> d & 1) && --indeg[d] == 0) ready.push_back(d);
    }
    if ((int)topo.size() != n_blocks) return;   // cyclic: not a valid cluster order
    std::vector<int> level(n_blocks);
    for (int k = 0; k < n_blocks; ++k) level[topo[k]] = k + 1;
    std::vector<int> pi(m.n, 0);
    for (int a : order) pi[a] = level[block[a]];
    Clustering c;
    std::string err;
    if (derive_and_check(m, pi, c, err) != FC_OK) return;
    double cost = objective(c);
    if (!(cost < best)) return;
    if (admissible && *admissible) {
      Clustering shaped = c, again;
      if (split) split_components(m, shaped); else renumber_levels(m, shaped);
      if (derive_and_check(m, shaped.pi, again, err) != FC_OK || !(*admissible)(again)) return;
    }
    best = cost;
    best_pi = pi;
    if (stop_at_first) aborted = true;
  }

  // Is the clustering "placed nodes in their blocks, every other combinator alone" a legal one?
  // If so `pi` receives its cluster numbers.  Used by the greedy construction below: a step that
  // keeps this true can always be completed.
  bool legal_with_the_rest_alone(std::vector<int> &pi) const {
    std::vector<int> blk(m.n, -1);
    int nb = n_blocks;
    for (int a : order) blk[a] = block[a] >= 0 ? block[a] : nb++;
    std::vector<std::vector<int>> after(nb);          // block -> blocks that must run later
    std::vector<int> indeg(nb, 0);
    auto before = [&](int x, int y) { after[x].push_back(y); ++indeg[y]; };
    for (const Edge &ed : m.edges) {
      if (m.is_input(ed.a)) continue;
      if (blk[ed.a] != blk[ed.b]) before(blk[ed.a], blk[ed.b]);
    }
    for (int j : order) {
      if (m.nodes[j].kind != FC_SCATTER) continue;
      const int d = m.nodes[j].arg[0];
      for (int e : m.out_edges[d]) {
        const int i = m.edges[e].b;
        if (i == j) continue;
        if (blk[i] == blk[j]) return false;
        before(blk[i], blk[j]);
      }
    }
    std::vector<int> ready, level(nb, 0);
    for (int b = nb - 1; b >= 0; --b) if (!indeg[b]) ready.push_back(b);
    int done = 0;
    while (!ready.empty()) {
      const int b = ready.back();
      ready.pop_back();
      level[b] = ++done;
      for (int d : after[b]) if (--indeg[d] == 0) ready.push_back(d);
    }
    if (done != nb) return false;
    pi.assign(m.n, 0);
    for (int a : order) pi[a] = level[blk[a]];
    Clustering c;
    std::string why;
    return derive_and_check(m, pi, c, why) == FC_OK;
  }

  // the extra condition, judged on the clustering as it would be returned
  bool passes(const std::vector<int> &pi) const {
    if (!admissible || !*admissible) return true;
    Clustering c, again;
    std::string why;
    if (derive_and_check(m, pi, c, why) != FC_OK) return false;
    if (split) split_components(m, c); else renumber_levels(m, c);
    return derive_and_check(m, c.pi, again, why) == FC_OK && (*admissible)(again);
  }

  // A clustering built without backtracking: the combinators in program order, each into the block
  // (one that holds a producer of it or reads one of its arguments, or a new one) that keeps the partial
  // cost lowest among those that leave a legal clustering when the remaining combinators stay alone.
  // It gives the exact search something to improve on; on large programs the search's first descents
  // tend to end in clusterings that turn out illegal only once complete.
  void greedy_incumbent() {
    std::vector<int> pi;
    for (int a : order) {
      std::vector<int> cand;
      auto add = [&](int b) { if (b >= 0 && std::find(cand.begin(), cand.end(), b) == cand.end()) cand.push_back(b); };
      for (int e : m.in_edges[a]) {
        add(block[m.edges[e].a]);
        for (int e2 : m.out_edges[m.edges[e].a]) add(block[m.edges[e2].b]);      // readers of the same array
      }
      cand.push_back(n_blocks);
      int best_b = -1;
      double best_lb = 1e300;
      for (int b : cand) {
        block[a] = b;
        const bool fresh = b == n_blocks;
        if (fresh) ++n_blocks;
        if (legal_with_the_rest_alone(pi) && passes(pi)) {
          const double lb = lower_bound();
          if (lb < best_lb) { best_lb = lb; best_b = b; }
        }
        if (fresh) --n_blocks;
        block[a] = -1;
      }
      if (best_b < 0) { best_b = n_blocks; }           // cannot happen for a legal program
      block[a] = best_b;
      if (best_b == n_blocks) ++n_blocks;
    }
    improve_by_moves(false);
    for (int a : order) block[a] = -1;
    n_blocks = 0;
  }

  // goes on from where the local improvement stopped, with random moves, until the phase's time is up
  void keep_improving() {
    if (moved_block.empty() || !(seconds > 0)) return;
    block = moved_block;
    n_blocks = moved_n_blocks;
    improve_by_moves(true);
    for (int a : order) block[a] = -1;
    n_blocks = 0;
  }

  // Cost of the complete clustering held in `block` (1e300 if it is not legal or fails the extra condition).
  double cost_of_blocks(std::vector<int> &pi) const {
    Clustering c;
    std::string why;
    if (!legal_with_the_rest_alone(pi) || derive_and_check(m, pi, c, why) != FC_OK || !passes(pi)) return 1e300;
    return objective(c);
  }

  // Local improvement of the greedy clustering.  A move: a combinator goes to a neighbouring block (one
  // that holds a producer or a consumer of it, or another reader of one of its arguments) or to a block
  // of its own, or its whole block joins such a block.  `descend` takes the best improving move of each
  // combinator in turn until none helps: the construction above never revisits a decision, this repairs
  // the early ones that later combinators made wrong.  With a time limit (an anytime search) it goes on
  // from there for `share` of the limit: a few random legal moves, a descent, kept unless it ends higher.
  // The result is the incumbent of the exact search and what an anytime search returns for a program it
  // cannot finish.  The random numbers come from a fixed seed.
  std::vector<int> neighbouring_blocks(int a) const {
    std::vector<int> cand;
    auto add = [&](int b) { if (b >= 0 && b != block[a] && std::find(cand.begin(), cand.end(), b) == cand.end()) cand.push_back(b); };
    for (int e : m.in_edges[a]) {
      add(block[m.edges[e].a]);
      for (int e2 : m.out_edges[m.edges[e].a]) add(block[m.edges[e2].b]);
    }
    for (int e : m.out_edges[a]) add(block[m.edges[e].b]);
    cand.push_back(n_blocks);                                   // a block of its own
    return cand;
  }

  bool past(double part) const {
    return seconds > 0 && std::chrono::duration<double>(std::chrono::steady_clock::now() - started).count() > seconds * part;
  }

  double descend(double cur, std::vector<int> &pi_of_cur) {
    std::vector<int> pi;
    for (int round = 0, moved = 1; moved && round < 16 && !past(share); ++round) {
      moved = 0;
      for (int a : order) {
        if (past(share)) break;
        const int home = block[a];
        int best_b = home, best_kind = 0;
        double best_cost = cur;
        std::vector<int> best_pi_here;
        for (int b : neighbouring_blocks(a)) {
          const bool fresh = b == n_blocks;
          block[a] = b;                                     // (1) the combinator alone moves
          if (fresh) ++n_blocks;
          const double c1 = cost_of_blocks(pi);
          if (c1 < best_cost * (1.0 - 1e-12)) { best_cost = c1; best_b = b; best_kind = 1; best_pi_here = pi; }
          if (fresh) --n_blocks;
          block[a] = home;
          if (fresh) continue;
          std::vector<int> members;                         // (2) its whole block joins block b
          for (int x : order) if (block[x] == home) members.push_back(x);
          if (members.size() > 1) {
            for (int x : members) block[x] = b;
            const double c2 = cost_of_blocks(pi);
            if (c2 < best_cost * (1.0 - 1e-12)) { best_cost = c2; best_b = b; best_kind = 2; best_pi_here = pi; }
            for (int x : members) block[x] = home;
          }
        }
        if (best_kind == 1) {
          block[a] = best_b;
          if (best_b == n_blocks) ++n_blocks;
        } else if (best_kind == 2) {
          for (int x : order) if (block[x] == home) block[x] = best_b;
        }
        if (best_kind) { cur = best_cost; pi_of_cur = best_pi_here; moved = 1; }
      }
    }
    return cur;
  }

  void renumber_blocks() {
    std::vector<int> id(n_blocks, -1);
    int next = 0;
    for (int a : order) {
      if (id[block[a]] < 0) id[block[a]] = next++;
      block[a] = id[block[a]];
    }
    n_blocks = next;
  }

  void improve_by_moves(bool with_random_moves) {
    std::vector<int> pi, pi_of_cur;
    double cur = cost_of_blocks(pi);
    if (cur >= 1e300 || order.empty()) return;
    pi_of_cur = pi;
    cur = descend(cur, pi_of_cur);
    auto record = [&]() {
      if (cur < best) { best = cur * (1.0 + 1e-12) + 1e-9; best_pi = pi_of_cur; }
      moved_block = block;
      moved_n_blocks = n_blocks;
    };
    record();
    if (!with_random_moves) return;
    unsigned long long state = 0x9E3779B97F4A7C15ull;
    auto draw = [&](size_t below) {
      state = state * 6364136223846793005ull + 1442695040888963407ull;
      return (size_t)((state >> 33) % below);
    };
    while (!past(share)) {
      renumber_blocks();
      const std::vector<int> kept_block = block, kept_pi = pi_of_cur;
      const int kept_n = n_blocks;
      const double kept = cur;
      for (int k = 0; k < 3; ++k) {
        const int a = order[draw(order.size())];
        const std::vector<int> cand = neighbouring_blocks(a);
        const int b = cand[draw(cand.size())], home = block[a];
        block[a] = b;
        if (b == n_blocks) ++n_blocks;
        const double c = cost_of_blocks(pi);
        if (c >= 1e300) block[a] = home;          // not a legal clustering: taken back (a fresh block number stays unused)
        else { cur = c; pi_of_cur = pi; }
      }
      cur = descend(cur, pi_of_cur);
      if (cur <= kept * (1.0 + 1e-12)) record();
      else { block = kept_block; n_blocks = kept_n; cur = kept; pi_of_cur = kept_pi; }
    }
  }

  // the blocks that hold a combinator linked to `a` by a chain of edges and common arguments whose inner
  // members are all still unplaced
  uint64_t blocks_in_reach(int a) const {
    std::vector<char> seen(m.n, 0);
    std::vector<int> stack(1, a);
    uint64_t blocks = 0;
    seen[a] = 1;
    auto touch = [&](int v) {
      if (seen[v]) return;
      seen[v] = 1;
      if (m.is_input(v)) return;
      if (block[v] >= 0) blocks |= 1ull << block[v]; else stack.push_back(v);
    };
    // the order an edge reads its array in, if it is fixed (-1: the consumer's own order, open)
    auto fixed_order = [&](const Edge &ed) {
      switch (m.in_order(ed.b, ed.slot)) {
        case InOrder::Label: return m.label[ed.b];
        case InOrder::Zero: return 0;
        case InOrder::One: return 1;
        default: return -1;
      }
    };
    while (!stack.empty()) {
      const int u = stack.back();
      stack.pop_back();
      for (int e : m.out_edges[u]) if (m.edges[e].fusible) touch(m.edges[e].b);     // an edge that can be fused
      for (int e : m.in_edges[u]) {
        const Edge &mine = m.edges[e];
        if (mine.fusible) touch(mine.a);
        // the other readers of this argument, unless both orders are fixed and differ (no read to share)
        const int k = fixed_order(mine);
        for (int e2 : m.out_edges[mine.a]) {
          const int k2 = fixed_order(m.edges[e2]);
          if (k < 0 || k2 < 0 || k == k2) touch(m.edges[e2].b);
        }
      }
    }
    return blocks;
  }

  void go(size_t k) {
    if (aborted) return;
    if (++visited > limit) { aborted = true; return; }
    if (seconds > 0 && (visited & 1023) == 0 && past(share)) {
      aborted = timed_out = true;
      return;
    }
    if (k == order.size()) { leaf(); return; }
    const int a = order[k];
    // candidate blocks: those holding a producer of `a` first, then the others, then a new one
    std::vector<int> cand;
    for (int e : m.in_edges[a]) {
      int b = block[m.edges[e].a];
      if (b >= 0 && std::find(cand.begin(), cand.end(), b) == cand.end()) cand.push_back(b);
    }
    // A cluster whose members fall into groups that share nothing (no edge between them, no array
    // read by both) costs what the groups cost as clusters of their own, and those are legal when it is
    // (section 4.1, the split into connected components).  So `a` need only try the blocks it can still
    // come to share something with: those reached from it over edges and common arguments through
    // combinators that are not placed yet.  (The number of clusters is the one cost a block of strangers lowers.)
    if (weight[FC_COST_CLUSTERS] == 0) {
      const uint64_t useful = blocks_in_reach(a);
      for (int b = 0; b < n_blocks; ++b)
        if ((useful >> b & 1) && std::find(cand.begin(), cand.end(), b) == cand.end()) cand.push_back(b);
    } else {
      for (int b = 0; b < n_blocks; ++b) if (std::find(cand.begin(), cand.end(), b) == cand.end()) cand.push_back(b);
    }
    if (n_blocks < 64) cand.push_back(n_blocks);
    // a node tied to already placed nodes has no choice
    int must = -1;
    for (size_t j = 0; j < k; ++j)
      if (forced_root(order[j]) == forced_root(a)) { must = block[order[j]]; break; }
    if (must >= 0) cand.assign(1, must);
    for (int b : cand) {
      const bool fresh = b == n_blocks;
      // edges into `a`: infusible ones need another block; all of them order the blocks
      bool ok = true;
      std::vector<std::pair<int, int>> added;   // (from block, to block) bits set here
      auto order_blocks = [&](int from, int to) {
        if (from == to) { ok = false; return; }
        if (!(adj[from] >> to & 1)) {
          if (reaches(to, from)) { ok = false; return; }
          adj[from] |= 1ull << to;
          added.push_back({from, to});
        }
      };
      for (int e : m.in_edges[a]) {
        if (!ok) break;
        const Edge &ed = m.edges[e];
        int pb = block[ed.a];
        if (pb < 0) continue;   // producer is a program input
        if (pb == b) { if (!ed.fusible) ok = false; continue; }
        order_blocks(pb, b);
      }
      // temporal uniqueness of scatter, in both roles `a` can play
      if (ok && m.nodes[a].kind == FC_SCATTER) {
        int d = m.nodes[a].arg[0];
        for (int e : m.out_edges[d]) {
          int i = m.edges[e].b;
          if (i != a && block[i] >= 0 && ok) order_blocks(block[i], b);
        }
      }
      if (ok) {
        for (int e : m.in_edges[a]) {
          int d = m.edges[e].a;
          for (int e2 : m.out_edges[d]) {
            int j = m.edges[e2].b;
            if (j != a && m.nodes[j].kind == FC_SCATTER && m.nodes[j].arg[0] == d && block[j] >= 0 && ok)
              order_blocks(b, block[j]);
          }
        }
      }
      if (ok) {
        block[a] = b;
        if (fresh) ++n_blocks;
        if (orders_completable(m, block, &resolved) && lower_bound() < best) go(k + 1);
        resolved.clear();
        if (fresh) --n_blocks;
        block[a] = -1;
      }
      for (auto &p : added) adj[p.first] &= ~(1ull << p.second);
    }
  }
};

}  // namespace

namespace {
void unit_weights(int cost_fn, double *w) {
  for (int k = 0; k < kCosts; ++k) w[k] = k == cost_fn ? 1.0 : 0.0;
}
}  // namespace

int choose_clustering(const Model &m, int cost_fn, bool split, Clustering &out, int &n_clusters, double &cost,
                      std::string &err, const Admissible &admissible, SearchBudget *budget) {
  if (cost_fn < FC_COST_CLUSTERS || cost_fn > FC_COST_BYTES) { err = "unknown cost function"; return FC_E_ARG; }
  double w[kCosts];
  unit_weights(cost_fn, w);
  return choose_clustering_weighted(m, w, split, out, n_clusters, cost, err, admissible, budget);
}

int choose_clustering_weighted(const Model &m, const double *weights, bool split, Clustering &out, int &n_clusters,
                               double &cost, std::string &err, const Admissible &admissible, SearchBudget *budget) {
  SearchBudget standard;
  if (!budget) budget = &standard;
  budget->proven = true;
  bool any = false;
  for (int k = 0; k < kCosts; ++k) {
    if (!(weights[k] >= 0) || weights[k] > 1e300) { err = "cost weights must be finite and not negative"; return FC_E_ARG; }
    any = any || weights[k] > 0;
  }
  if (!any) { err = "all cost weights are zero"; return FC_E_ARG; }
  int non_input = 0;
  for (int a = 0; a < m.n; ++a) non_input += !m.is_input(a);
  if (non_input > 64 && !budget->anytime) { err = "the exact chooser handles at most 64 combinators"; return FC_E_LIMIT; }
  Search s(m, weights, budget->nodes);
  s.seconds = budget->seconds;
  s.admissible = &admissible;
  s.split = split;
  {
    // a first incumbent: every combinator a cluster of its own, in program order (legal whenever the
    // program is); the search only has to improve on it, and a search that is cut short has it to return
    std::vector<int> alone(m.n, 0);
    int next = 0;
    for (int a = 0; a < m.n; ++a) if (!m.is_input(a)) alone[a] = ++next;
    Clustering c;
    std::string why;
    if (derive_and_check(m, alone, c, why) == FC_OK && (!admissible || admissible(c))) {
      s.best = s.objective(c) * (1.0 + 1e-12) + 1e-9;   // kept if nothing cheaper exists
      s.best_pi = alone;
    }
  }
  s.greedy_incumbent();
  if (non_input > 64) {
    // the search keeps its blocks in 64-bit sets: the greedy clustering, improved by moves for the time allowed, stands
    s.keep_improving();
    s.aborted = true;
  } else if (budget->seconds > 0) {
    // the search first, for 0.6 of the time (programs it can finish end here, proven); if that was not enough,
    // random moves and descents from the greedy clustering for the rest
    s.share = 0.6;
    s.go(0);
    if (s.timed_out) {
      s.share = 1.0;
      s.keep_improving();
    }
  } else {
    s.go(0);
  }
  if (s.aborted) {
    if (!budget->anytime || s.best_pi.empty()) { err = "search limit reached before optimality was proven"; return FC_E_LIMIT; }
    budget->proven = false;          // the best clustering found so far: legal, maybe not the cheapest
  }
  if (s.best_pi.empty() && non_input > 0) {
    if (admissible) { err = "no clustering passes the extra condition"; return FC_E_UNSUPPORTED; }
    err = "no feasible clustering";
    return FC_E_ILLEGAL_PARTITION;
  }
  std::vector<int> pi = s.best_pi.empty() ? std::vector<int>(m.n, 0) : s.best_pi;
  int rc = derive_and_check(m, pi, out, err);
  if (rc != FC_OK) return rc;
  cost = s.objective(out);
  n_clusters = split ? split_components(m, out) : renumber_levels(m, out);
  // the split changes cluster numbers only; re-derive the per-edge and per-node variables
  Clustering again;
  rc = derive_and_check(m, out.pi, again, err);
  if (rc != FC_OK) return rc;
  out = again;
  return FC_OK;
}

// --------------------------------------------------------------------------- greedy
int choose_greedy(const Model &m, int direction, int cost_fn, bool split, Clustering &out, int &n_clusters, double &cost,
                  std::string &err, const Admissible &admissible) {
  if (cost_fn < FC_COST_CLUSTERS || cost_fn > FC_COST_BYTES) { err = "unknown cost function"; return FC_E_ARG; }
  int non_input = 0;
  for (int a = 0; a < m.n; ++a) non_input += !m.is_input(a);
  if (non_input > 64) { err = "the greedy chooser handles at most 64 combinators"; return FC_E_LIMIT; }
  std::vector<int> edges;
  for (size_t e = 0; e < m.edges.size(); ++e) if (m.edges[e].fusible) edges.push_back((int)e);
  // top-down: edges nearest the inputs first; bottom-up: edges nearest the results first
  std::stable_sort(edges.begin(), edges.end(), [&](int x, int y) {
    const Edge &a = m.edges[x], &b = m.edges[y];
    if (direction == 0) return a.a != b.a ? a.a < b.a : a.b < b.b;
    return a.b != b.b ? a.b > b.b : a.a > b.a;
  });
  std::vector<std::pair<int, int>> accepted;
  double w[kCosts];
  unit_weights(cost_fn, w);
  auto make_search = [&](bool first_only) {
    Search s(m, w, 200000000LL);
    for (auto &p : accepted) s.force_together(p.first, p.second);
    s.stop_at_first = first_only;
    s.admissible = &admissible;
    s.split = split;
    return s;
  };
  for (int e : edges) {
    accepted.push_back({m.edges[e].a, m.edges[e].b});
    Search s = make_search(true);
    s.go(0);
    if (s.best_pi.empty()) {
      if (s.aborted && s.visited > s.limit) { err = "search limit reached"; return FC_E_LIMIT; }
      accepted.pop_back();          // no clustering fuses this edge together with the ones taken so far
    }
  }
  Search s = make_search(false);
  s.go(0);
  if (s.best_pi.empty() && !s.aborted && admissible) { err = "no clustering passes the extra condition"; return FC_E_UNSUPPORTED; }
  if (s.aborted || s.best_pi.empty()) { err = "greedy search failed"; return FC_E_LIMIT; }
  int rc = derive_and_check(m, s.best_pi, out, err);
  if (rc != FC_OK) return rc;
  cost = evaluate_cost(m, out, cost_fn);
  n_clusters = split ? split_components(m, out) : renumber_levels(m, out);
  Clustering again;
  rc = derive_and_check(m, out.pi, again, err);
  if (rc != FC_OK) return rc;
  out = again;
  return FC_OK;
}

// --------------------------------------------------------------------------- duplication
int duplicate_producers(const Model &m, std::vector<fc_node> &out_nodes, std::vector<int> &origin) {
  const int n = m.n;
  // versions[a]: order classes in which a copy of node a is needed.  Class 0 is the
  // natural order; class g+1 is "read as the source of gather g".
  std::vector<std::vector<int>> versions(n);
  auto cloneable = [&](int a) { return m.nodes[a].kind == FC_MAP || m.nodes[a].kind == FC_GENERATE; };
  for (int a = n - 1; a >= 0; --a) {
    std::set<int> classes;
    if (m.out_edges[a].empty() || (m.nodes[a].flags & FC_NODE_OUTPUT)) classes.insert(0);
    for (int e : m.out_edges[a]) {
      const Edge &ed = m.edges[e];
      switch (m.in_order(ed.b, ed.slot)) {
        case InOrder::Label: classes.insert(ed.b + 1); break;
        case InOrder::SameAsOut: for (int t : versions[ed.b]) classes.insert(t); break;
        default: classes.insert(0);
      }
    }
    if (!cloneable(a) && classes.size() > 1) classes = {0};
    versions[a].assign(classes.begin(), classes.end());
  }
  // emit in program order; version (a, t) takes the version of each argument that matches its class
  std::map<std::pair<int, int>, int> id;
  out_nodes.clear();
  origin.clear();
  auto version_of = [&](int p, int cls) {
    auto it = id.find({p, cls});
    if (it != id.end()) return it->second;
    it = id.find({p, 0});
    if (it != id.end()) return it->second;
    return id.lower_bound({p, -1})->second;   // the only version there is
  };
  for (int a = 0; a < n; ++a) {
    for (size_t v = 0; v < versions[a].size(); ++v) {
      int t = versions[a][v];
      fc_node nd = m.nodes[a];
      if (t != 0 && versions[a].size() > 1 && std::find(versions[a].begin(), versions[a].end(), 0) != versions[a].end())
        nd.flags &= ~FC_NODE_OUTPUT;
      for (int k = 0; k < nd.nargs; ++k) {
        int cls = 0;
        switch (m.in_order(a, k)) {
          case InOrder::Label: cls = a + 1; break;
          case InOrder::SameAsOut: cls = t; break;
          default: cls = 0;
        }
        nd.arg[k] = version_of(m.nodes[a].arg[k], cls);
      }
      id[{a, t}] = (int)out_nodes.size();
      out_nodes.push_back(nd);
      origin.push_back(a);
    }
  }
  return FC_OK;
}

}  // namespace fc
