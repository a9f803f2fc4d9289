// Chooser (exact ILP solution) and work-duplication rewrite, host only.
#pragma once

#include <string>
#include <vector>

#include "model.hpp"

namespace fc {

// Minimises cost_fn over the feasible clusterings of the ILP.  `split` applies
// the connected-component post-pass.  `cost` is the objective value of the ILP
// solution (before the split).
int choose_clustering(const Model &m, int cost_fn, bool split, Clustering &out, int &n_clusters, double &cost,
                      std::string &err);

// Clones map / generate nodes so that every copy is read in one traversal order.
int duplicate_producers(const Model &m, std::vector<fc_node> &out_nodes, std::vector<int> &origin);

}  // namespace fc
