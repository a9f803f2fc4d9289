// extern "C" entry points (include/fc.h).  Argument checking and marshalling
// only; no exception leaves this file.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <exception>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "model.hpp"
#include "plan.hpp"
#include "run.hpp"

// Scratch of fc_run_fused_static: one copy per device, zero when the code object is
// loaded (which is what the control block at its start needs the first time), held until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// memory is reached through the address that call returns (static_scratch_of below).
static __device__ __align__(256) unsigned char static_scratch[FC_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_error;

// Address of the current device's copy of static_scratch, looked up once per device.
constexpr int kMaxDevices = 64;
int static_scratch_of(void **out, std::string &err) {
  static std::mutex mu;
  static void *known[kMaxDevices];                 // zero-initialised: not looked up yet
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { err = std::string("hipGetDevice: ") + hipGetErrorString(e); return FC_E_HIP; }
  if (dev < 0 || dev >= kMaxDevices) { err = "device ordinal " + std::to_string(dev) + " is out of range"; return FC_E_LIMIT; }
  std::lock_guard<std::mutex> lock(mu);
  if (!known[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch));
    if (e != hipSuccess || !ptr) {
      err = std::string("hipGetSymbolAddress(static_scratch): ") + hipGetErrorString(e);
      return FC_E_HIP;
    }
    known[dev] = ptr;
  }
  *out = known[dev];
  return FC_OK;
}

int fail(int code, const std::string &msg) {
  g_error = msg;
  return code;
}

template <class F> int guarded(F &&f) {
  try {
    g_error.clear();
    return f();
  } catch (const std::exception &e) {
    return fail(FC_E_ARG, std::string("internal error: ") + e.what());
  } catch (...) {
    return fail(FC_E_ARG, "internal error");
  }
}

int fill_partition(const fc::Model &m, const fc::Clustering &c, int n_clusters, double cost, fc_partition *out, bool proven = true) {
  if (!out || out->n_nodes < m.n || out->n_edges < (int)m.edges.size())
    return fail(FC_E_ARG, "partition arrays are too small");
  if (m.n && (!out->pi || !out->fused_away || !out->order_out)) return fail(FC_E_ARG, "null partition array");
  if (!m.edges.empty() && !out->edge_unfused) return fail(FC_E_ARG, "null partition array");
  for (int a = 0; a < m.n; ++a) {
    out->pi[a] = c.pi[a];
    out->fused_away[a] = c.fused_away[a];
    out->order_out[a] = c.order_out[a];
  }
  for (size_t e = 0; e < m.edges.size(); ++e) out->edge_unfused[e] = c.x[e];
  out->n_clusters = n_clusters;
  out->cost = cost;
  out->proven = proven ? 1 : 0;
  return FC_OK;
}

// FC_PLAN_ANYTIME: a search of a few seconds, the best clustering found if it does not finish
fc::SearchBudget budget_of(uint32_t flags) {
  fc::SearchBudget b;
  if (flags & FC_PLAN_ANYTIME) { b.seconds = 2.0; b.anytime = true; }
  return b;
}

// Every combinator in a cluster of its own.  The clusters are numbered in a topological
// order of the program that also puts every other reader of a scatter's destination before
// the scatter (the destination is updated in place, so the scatter is its last use: section
// 4.1, the constraints on scatter); among the orders that do, the one closest to program
// order.  A program in which a reader of the destination depends on the scatter itself has
// no such order: it keeps program order and the check reports the reader.
void trivial_numbering(const fc::Model &m, std::vector<int> &pi) {
  const int n = m.n;
  std::vector<std::vector<int>> after(n);
  std::vector<int> waiting(n, 0);
  auto before = [&](int a, int b) { after[a].push_back(b); ++waiting[b]; };
  for (const fc::Edge &e : m.edges) before(e.a, e.b);
  for (int j = 0; j < n; ++j) {
    if (m.nodes[j].kind != FC_SCATTER) continue;
    for (int e : m.out_edges[m.nodes[j].arg[0]])
      if (m.edges[e].b != j) before(m.edges[e].b, j);
  }
  std::vector<char> placed(n, 0);
  int next = 0;
  for (int k = 0; k < n; ++k) {
    int a = 0;
    while (a < n && (placed[a] || waiting[a] != 0)) ++a;   // the first combinator in program order that is free
    if (a == n) {                                          // a cycle through a scatter's destination
      for (int b = 0; b < n; ++b) pi[b] = b;
      return;
    }
    placed[a] = 1;
    pi[a] = next++;
    for (int b : after[a]) --waiting[b];
  }
}

int load_clustering(const fc::Model &m, const fc_partition *p, fc::Clustering &c, std::string &err) {
  std::vector<int> pi(m.n);
  if (p) {
    if (p->n_nodes < m.n || (m.n && !p->pi)) { err = "partition does not cover the graph"; return FC_E_ARG; }
    for (int a = 0; a < m.n; ++a) pi[a] = p->pi[a];
  } else {
    trivial_numbering(m, pi);
  }
  return fc::derive_and_check(m, pi, c, err);
}

}  // namespace

extern "C" {

const char *fc_last_error(void) { return g_error.c_str(); }

int fc_num_edges(const fc_graph *g, int32_t *n_edges) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    if (!n_edges) return fail(FC_E_ARG, "null result pointer");
    *n_edges = (int32_t)m.edges.size();
    return FC_OK;
  });
}

// FC_PLAN_EXECUTABLE: only clusterings every cluster of which has a kernel instance
static fc::Admissible executable_only(const fc::Model &m, uint32_t flags) {
  if (!(flags & FC_PLAN_EXECUTABLE)) return fc::Admissible();
  return [&m](const fc::Clustering &c) {
    for (const auto &members : fc::clusters_of(m, c)) {
      fc::ClusterLaunch cl;
      std::string why;
      if (fc::plan_cluster(m, c, members, cl, why) != FC_OK) return false;
    }
    return true;
  };
}

int fc_plan(const fc_graph *g, int cost_fn, uint32_t flags, fc_partition *out) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    fc::Clustering c;
    int n_clusters = 0;
    double cost = 0;
    fc::SearchBudget budget = budget_of(flags);
    rc = fc::choose_clustering(m, cost_fn, !(flags & FC_PLAN_NO_SPLIT), c, n_clusters, cost, err, executable_only(m, flags),
                               &budget);
    if (rc != FC_OK) return fail(rc, err);
    return fill_partition(m, c, n_clusters, cost, out, budget.proven);
  });
}

int fc_plan_weighted(const fc_graph *g, const double *weights, uint32_t flags, fc_partition *out) {
  return guarded([&]() {
    if (!weights) return fail(FC_E_ARG, "weights is NULL");
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    fc::Clustering c;
    int n_clusters = 0;
    double cost = 0;
    fc::SearchBudget budget = budget_of(flags);
    rc = fc::choose_clustering_weighted(m, weights, !(flags & FC_PLAN_NO_SPLIT), c, n_clusters, cost, err,
                                        executable_only(m, flags), &budget);
    if (rc != FC_OK) return fail(rc, err);
    return fill_partition(m, c, n_clusters, cost, out, budget.proven);
  });
}

int fc_plan_greedy(const fc_graph *g, int direction, int cost_fn, uint32_t flags, fc_partition *out) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    if (direction != 0 && direction != 1) return fail(FC_E_ARG, "direction must be 0 (top-down) or 1 (bottom-up)");
    fc::Clustering c;
    int n_clusters = 0;
    double cost = 0;
    rc = fc::choose_greedy(m, direction, cost_fn, !(flags & FC_PLAN_NO_SPLIT), c, n_clusters, cost, err,
                           executable_only(m, flags));
    if (rc != FC_OK) return fail(rc, err);
    return fill_partition(m, c, n_clusters, cost, out);
  });
}

int fc_partition_trivial(const fc_graph *g, fc_partition *out) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    fc::Clustering c;
    rc = load_clustering(m, nullptr, c, err);
    if (rc != FC_OK) return fail(rc, err);
    int k = fc::renumber_levels(m, c);
    return fill_partition(m, c, k, fc::evaluate_cost(m, c, FC_COST_READS_WRITES), out);
  });
}

int fc_partition_check(const fc_graph *g, fc_partition *p, int cost_fn, double *cost) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    if (!p) return fail(FC_E_ARG, "null partition");
    fc::Clustering c;
    rc = load_clustering(m, p, c, err);
    if (rc != FC_OK) return fail(rc, err);
    double v = fc::evaluate_cost(m, c, cost_fn);
    if (v < 0) return fail(FC_E_ARG, "unknown cost function");
    if (cost) *cost = v;
    int k = (int)fc::clusters_of(m, c).size();
    return fill_partition(m, c, k, v, p);
  });
}

int fc_duplicate(const fc_graph *g, fc_node *out_nodes, int32_t capacity, int32_t *out_n, int32_t *origin) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    std::vector<fc_node> nodes;
    std::vector<int> org;
    rc = fc::duplicate_producers(m, nodes, org);
    if (rc != FC_OK) return fail(rc, "duplication failed");
    if (!out_n) return fail(FC_E_ARG, "null result pointer");
    *out_n = (int32_t)nodes.size();
    if ((int)nodes.size() > capacity || !out_nodes) return fail(FC_E_ARG, "node capacity too small");
    for (size_t i = 0; i < nodes.size(); ++i) {
      out_nodes[i] = nodes[i];
      if (origin) origin[i] = org[i];
    }
    return FC_OK;
  });
}

int fc_scratch_bytes(const fc_graph *g, const fc_partition *p, size_t *bytes) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    fc::Clustering c;
    rc = load_clustering(m, p, c, err);
    if (rc != FC_OK) return fail(rc, err);
    if (!bytes) return fail(FC_E_ARG, "null result pointer");
    *bytes = fc::scratch_bytes_for(m, c);
    return FC_OK;
  });
}

// Validating a program and matching its clusters to kernel instances depends only
// on the nodes and on pi, so the result is memoised: repeated runs of one program
// (the common case) go straight to buffer resolution and launch.
struct Prepared {
  std::vector<unsigned char> key;
  std::shared_ptr<const fc::PreparedRun> run;
};

// use_static: run in the device's static scratch array instead of a buffer of the caller
static int run_common(const fc_graph *g, const fc_partition *p, const fc_buffer *bufs, void *scratch,
                      size_t scratch_bytes, void *hip_stream, bool use_static = false) {
  static std::mutex mu;
  static std::vector<Prepared> cache;        // most recently used first
  if (!g || g->n < 0 || (g->n > 0 && !g->nodes)) return fail(FC_E_ARG, "null graph");
  if (p && (p->n_nodes < g->n || (g->n && !p->pi))) return fail(FC_E_ARG, "partition does not cover the graph");
  std::vector<unsigned char> key(sizeof(int) + (size_t)g->n * (sizeof(fc_node) + sizeof(int32_t)));
  std::memcpy(key.data(), &g->n, sizeof(int));
  for (int i = 0; i < g->n; ++i) {
    // field by field: padding bytes of the caller's structs are not part of the program
    fc_node nd;
    std::memset(&nd, 0, sizeof(nd));
    const fc_node &s = g->nodes[i];
    nd.kind = s.kind; nd.dtype = s.dtype; nd.fn = s.fn; nd.nargs = s.nargs; nd.rank = s.rank;
    nd.flags = s.flags; nd.infusible_args = s.infusible_args;
    std::memcpy(nd.fparam, s.fparam, sizeof(nd.fparam));
    std::memcpy(nd.iparam, s.iparam, sizeof(nd.iparam));
    std::memcpy(nd.arg, s.arg, sizeof(nd.arg));
    std::memcpy(nd.shape, s.shape, sizeof(nd.shape));
    std::memcpy(key.data() + sizeof(int) + (size_t)i * sizeof(fc_node), &nd, sizeof(nd));
    int32_t pi = p ? p->pi[i] : -1;
    std::memcpy(key.data() + sizeof(int) + (size_t)g->n * sizeof(fc_node) + (size_t)i * sizeof(int32_t), &pi, sizeof(pi));
  }
  std::shared_ptr<const fc::PreparedRun> run;
  {
    std::lock_guard<std::mutex> lock(mu);
    for (size_t k = 0; k < cache.size(); ++k)
      if (cache[k].key == key) {
        run = cache[k].run;
        if (k) std::rotate(cache.begin(), cache.begin() + k, cache.begin() + k + 1);
        break;
      }
  }
  std::string err;
  if (!run) {
    auto fresh = std::make_shared<fc::PreparedRun>();
    int rc = fc::build_model(g, fresh->model, err);
    if (rc != FC_OK) return fail(rc, err);
    rc = load_clustering(fresh->model, p, fresh->clustering, err);
    if (rc != FC_OK) return fail(rc, err);
    rc = fc::prepare_run(*fresh, err);
    if (rc != FC_OK) return fail(rc, err);
    fresh->scratch_need = fc::scratch_bytes_for(fresh->model, fresh->clustering);
    run = fresh;
    std::lock_guard<std::mutex> lock(mu);
    cache.insert(cache.begin(), Prepared{key, run});
    if (cache.size() > 32) cache.pop_back();
  }
  if (use_static) {
    if (run->scratch_need > (size_t)FC_STATIC_SCRATCH_BYTES)
      return fail(FC_E_LIMIT, "the program needs " + std::to_string(run->scratch_need) + " bytes of scratch, the static buffer holds " +
                                  std::to_string((size_t)FC_STATIC_SCRATCH_BYTES) + ": use fc_run_fused with a buffer of the caller");
    int rc = static_scratch_of(&scratch, err);
    if (rc != FC_OK) return fail(rc, err);
    scratch_bytes = FC_STATIC_SCRATCH_BYTES;
  }
  int rc = fc::run_prepared(*run, bufs, scratch, scratch_bytes, static_cast<hipStream_t>(hip_stream), err);
  if (rc != FC_OK) return fail(rc, err);
  return FC_OK;
}

int fc_run_fused(const fc_graph *g, const fc_partition *p, const fc_buffer *bufs, void *scratch, size_t scratch_bytes,
                 void *hip_stream) {
  return guarded([&]() {
    if (!p) return fail(FC_E_ARG, "null partition");
    return run_common(g, p, bufs, scratch, scratch_bytes, hip_stream);
  });
}

int fc_run_fused_static(const fc_graph *g, const fc_partition *p, const fc_buffer *bufs, void *hip_stream) {
  return guarded([&]() {
    if (!p) return fail(FC_E_ARG, "null partition");
    return run_common(g, p, bufs, nullptr, 0, hip_stream, true);
  });
}

int fc_run_unfused(const fc_graph *g, const fc_buffer *bufs, void *scratch, size_t scratch_bytes, void *hip_stream) {
  return guarded([&]() { return run_common(g, nullptr, bufs, scratch, scratch_bytes, hip_stream); });
}

int fc_check(void *scratch, void *hip_stream) {
  return guarded([&]() {
    if (!scratch) {                       // the buffer fc_run_fused_static uses on the current device
      std::string err;
      int rc = static_scratch_of(&scratch, err);
      if (rc != FC_OK) return fail(rc, err);
    }
    if ((uintptr_t)scratch & 255u) return fail(FC_E_SCRATCH, "scratch must be a 256-byte aligned device buffer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // the control block starts with { epoch, error }: see prim.hpp, Control
    unsigned words[2] = {0u, 0u};
    hipError_t e = hipMemcpyAsync(words, scratch, sizeof(words), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(FC_E_HIP, hipGetErrorString(e));
    if (words[1] == 0u) return FC_OK;
    const unsigned zero = 0u;
    e = hipMemcpyAsync(static_cast<char *>(scratch) + sizeof(unsigned), &zero, sizeof(zero), hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(FC_E_HIP, hipGetErrorString(e));
    return fail(FC_E_DEVICE_WAIT,
                "a workgroup gave up waiting for a partial result of another workgroup of its launch; the results "
                "of the calls on this scratch buffer since the last check are invalid (launch counter " +
                    std::to_string(words[0]) + ")");
  });
}

int fc_cluster_kernel(const fc_graph *g, const fc_partition *p, int32_t cluster, char *name, size_t capacity) {
  return guarded([&]() {
    fc::Model m;
    std::string err;
    int rc = fc::build_model(g, m, err);
    if (rc != FC_OK) return fail(rc, err);
    fc::Clustering c;
    rc = load_clustering(m, p, c, err);
    if (rc != FC_OK) return fail(rc, err);
    auto cl = fc::clusters_of(m, c);
    if (cluster < 0 || cluster >= (int)cl.size()) return fail(FC_E_ARG, "cluster index out of range");
    fc::ClusterLaunch launch;
    rc = fc::plan_cluster(m, c, cl[cluster], launch, err);
    if (rc != FC_OK) return fail(rc, err);
    std::string s = launch.sig;
    if (launch.instance && launch.instance->variant[0]) s += std::string(" {") + launch.instance->variant + "}";
    if (!name || capacity < s.size() + 1) return fail(FC_E_ARG, "name buffer too small");
    std::memcpy(name, s.c_str(), s.size() + 1);
    return FC_OK;
  });
}

}  // extern "C"
