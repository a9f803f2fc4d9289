// Host-side model of a combinator program and of a clustering.
//
// Follows the data dependence graph (n, N, F, I) of section 4.1 and the
// variables pi, x, m, d^o, d^i of Fig. "Total ILP formulation".
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/fc.h"

namespace fc {

struct Edge {
  int a;         // producer
  int b;         // consumer
  int slot;      // argument position in b
  bool fusible;  // member of F (else of I)
};

// Order a consumer reads one of its arguments in, relative to its own output
// order (Table 1, section 4.2).
enum class InOrder { SameAsOut, Label, Zero, One, None };

struct Model {
  int n = 0;
  std::vector<fc_node> nodes;
  std::vector<Edge> edges;                  // consumer ascending, slot ascending
  std::vector<std::vector<int>> out_edges;  // per node: edge ids leaving it
  std::vector<std::vector<int>> in_edges;   // per node: edge ids entering it (slot order)
  std::vector<int> label;                   // gather nodes: 2 + ordinal; others -1
  int n_gathers = 0;

  int64_t size(int a) const { return nodes[a].shape[0] * nodes[a].shape[1]; }
  int64_t bytes(int a) const { return size(a) * 4; }
  bool is_input(int a) const { return nodes[a].kind == FC_INPUT; }
  InOrder in_order(int b, int slot) const;
};

// Validates the graph (arity, dtypes, shapes, topological order, known
// functions) and builds the edge lists.  Returns FC_OK or FC_E_*.
int build_model(const fc_graph *g, Model &m, std::string &err);

int map_arity(int fn);  // -1: not a map function

// A clustering with everything derived from pi.
struct Clustering {
  std::vector<int> pi;
  std::vector<uint8_t> x;           // per edge
  std::vector<uint8_t> fused_away;  // m_a
  std::vector<int> order_out;       // d^o_a
  std::vector<int> order_in;        // per edge: order the consumer reads the array in
};

// Derives x, m and the traversal orders from pi and checks every constraint.
// Returns FC_OK or FC_E_ILLEGAL_PARTITION (err says which rule).
int derive_and_check(const Model &m, const std::vector<int> &pi, Clustering &c, std::string &err);

// Can a partial clustering still be completed as far as traversal orders go?  block[a] >= 0:
// the cluster node a has been put into; -1: not placed yet; -2: a program input.  The order
// equalities over edges inside one cluster only grow as nodes are added, so a conflict among
// the placed nodes stays one; likewise an array that is certainly manifest (a result, or read
// from another cluster already) cannot take the order of a gather.
// `resolved`, if given, receives per placed node the constant its traversal order is tied to so far
// (0, 1 or a gather's label), -1 where nothing ties it yet.
bool orders_completable(const Model &m, const std::vector<int> &block, std::vector<int> *resolved = nullptr);

double evaluate_cost(const Model &m, const Clustering &c, int cost_fn);

// Connected-component split (section 4.1, "Performance and correctness"):
// renumbers pi so that every cluster is connected through fusible edges or a
// parent read in the same order, keeping an executable (topological) order.
// Input nodes receive pi = -1... they are given the number 0 and all executable
// clusters the numbers 1..n_clusters.  Returns the number of executable clusters.
int split_components(const Model &m, Clustering &c);

// Renumber pi densely without splitting (inputs 0, clusters 1..k in a valid order).
int renumber_levels(const Model &m, Clustering &c);

}  // namespace fc
