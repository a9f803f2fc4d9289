// Cluster matcher and runner (host side).
#pragma once

#include <hip/hip_runtime_api.h>

#include <string>
#include <vector>

#include "expr.hpp"
#include "model.hpp"
#include "registry.hpp"

namespace fc {

// How one cluster is executed: a kernel instance with its arguments, or (for
// force) an alias of another array's buffer.
struct ClusterLaunch {
  enum Kind { Kernel, Alias } kind = Kernel;
  std::string sig;
  const Instance *instance = nullptr;
  KArgs args;
  std::vector<int> externals;          // node ids bound to args.in[k]
  int out_nodes[kMaxOut] = {-1, -1, -1, -1};
  int offsets_node = -1;               // foldSeg: node bound to args.in[kMaxIn-1]
  int aux = 0, h = 1, w = 1;
  int alias_of = -1, alias_node = -1;
};

// clusters in execution order (ascending pi), input nodes left out
std::vector<std::vector<int>> clusters_of(const Model &m, const Clustering &c);

int plan_cluster(const Model &m, const Clustering &c, const std::vector<int> &members, ClusterLaunch &out,
                 std::string &err);

size_t scratch_bytes_for(const Model &m, const Clustering &c);

// A validated program with every cluster matched to its kernel instance; what
// remains per call is binding buffers and launching.
struct PreparedRun {
  Model model;
  Clustering clustering;
  std::vector<ClusterLaunch> launches;
  size_t scratch_need = 0;             // scratch_bytes_for(model, clustering)
};

int prepare_run(PreparedRun &r, std::string &err);

int run_prepared(const PreparedRun &r, const fc_buffer *bufs, void *scratch, size_t scratch_bytes, hipStream_t stream,
                 std::string &err);

}  // namespace fc
