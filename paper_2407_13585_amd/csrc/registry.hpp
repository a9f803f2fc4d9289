// Table of the kernel instances compiled into the library.  A cluster is
// executed by the instance whose signature equals the signature the matcher
// derives from the cluster's combinators.
#pragma once

#include <hip/hip_runtime_api.h>

#include <string>
#include <vector>

namespace fc {

struct KArgs;
struct Control;

struct LaunchCtx {
  hipStream_t stream;
  Control *ctl;                   // DEVICE: control block at the start of scratch
  unsigned long long *partials;             // DEVICE: per-workgroup partial results of a fold
  unsigned long long *status;     // DEVICE: tile status words of the single-pass scan
  size_t max_tiles;
};

using Launcher = hipError_t (*)(const KArgs &, const LaunchCtx &);

struct Instance {
  std::string sig;
  Launcher launch;
  bool (*accept)(const KArgs &) = nullptr;   // extra conditions on parameters / extents
  const char *variant = "";                  // distinguishes instances that share a signature
};

const std::vector<Instance> &registry();
// first instance with this signature whose accept() (if any) passes
const Instance *find_instance(const std::string &sig, const KArgs &a);

}  // namespace fc
