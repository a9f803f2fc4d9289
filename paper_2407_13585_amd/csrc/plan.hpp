// Chooser (exact ILP solution) and work-duplication rewrite, host only.
#pragma once

#include <functional>
#include <string>
#include <vector>

#include "model.hpp"

namespace fc {

// An extra condition on complete clusterings (after the connected-component split, if one is
// asked for): the choosers below only return clusterings for which it holds.  Empty = none.
// The library uses it to restrict the choice to clusterings it has kernels for.
using Admissible = std::function<bool(const Clustering &)>;

// How long the exact chooser may search, and what it does when that is not enough.  The search
// is a branch and bound whose time grows exponentially with the number of combinators; the best
// clustering found so far is a legal one at any moment (section 5.2 of the paper makes the same
// point about stopping an ILP solver early).
struct SearchBudget {
  long long nodes = 200000000LL;   // branch-and-bound nodes visited before the search gives up
  double seconds = 0;              // wall-clock limit, 0 = none
  bool anytime = false;            // true: return the best clustering found instead of FC_E_LIMIT
  bool proven = true;              // (out) the returned clustering was proven optimal
};

// Minimises cost_fn over the feasible clusterings of the ILP.  `split` applies
// the connected-component post-pass.  `cost` is the objective value of the ILP
// solution (before the split).
int choose_clustering(const Model &m, int cost_fn, bool split, Clustering &out, int &n_clusters, double &cost,
                      std::string &err, const Admissible &admissible = Admissible(), SearchBudget *budget = nullptr);

// The same for a linear combination of the cost functions (section 5.1 names it as the
// way to cost functions fitted to a machine): weights[k] multiplies cost function k of
// fc_cost; none negative, not all zero.  `cost` is the weighted sum for the ILP solution.
int choose_clustering_weighted(const Model &m, const double *weights, bool split, Clustering &out, int &n_clusters,
                               double &cost, std::string &err, const Admissible &admissible = Admissible(),
                               SearchBudget *budget = nullptr);

// The greedy comparison arms of section 5 ("Greedy"): walk the fusible edges from the top
// (direction 0) or from the bottom (direction 1) of the graph, fuse an edge whenever some
// legal clustering still fuses it together with the edges taken so far; the result is
// locally maximal.  Among the clusterings that fuse exactly those edges the cheapest
// under cost_fn is returned.
int choose_greedy(const Model &m, int direction, int cost_fn, bool split, Clustering &out, int &n_clusters, double &cost,
                  std::string &err, const Admissible &admissible = Admissible());

// Clones map / generate nodes so that every copy is read in one traversal order.
int duplicate_producers(const Model &m, std::vector<fc_node> &out_nodes, std::vector<int> &origin);

}  // namespace fc
