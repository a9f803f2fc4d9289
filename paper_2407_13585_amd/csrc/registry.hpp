// Table of the kernel instances compiled into the library.  A cluster is
// executed by the instance whose signature equals the signature the matcher
// derives from the cluster's combinators.
#pragma once

#include <hip/hip_runtime_api.h>

#include <map>
#include <mutex>
#include <string>
#include <utility>
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
  void *workspace;                // DEVICE: what Instance::workspace asked for (256-byte aligned), or NULL
};

using Launcher = hipError_t (*)(const KArgs &, const LaunchCtx &);

struct Instance {
  std::string sig;
  Launcher launch;
  bool (*accept)(const KArgs &) = nullptr;   // extra conditions on parameters / extents
  const char *variant = "";                  // distinguishes instances that share a signature
  size_t (*workspace)(const KArgs &) = nullptr;   // bytes of scratch beyond the control block a launch needs
};

// Workgroups of `threads` threads of a kernel that are resident on the current
// device at once (0 if the runtime cannot tell).  Launches are sized by it: one
// workgroup more than the device holds starts a second round that lasts as long
// as the first (the reversed dot product at 2^26 elements: 51 us with 64
// registers per lane and 8 workgroups per CU; 69 us with 66 registers, hence 7
// per CU, under a grid of 8 per CU).
template <class... P>
unsigned resident_workgroups(void (*kernel)(P...), int threads) {
  static std::mutex mu;
  static std::map<std::pair<int, const void *>, unsigned> known;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  std::lock_guard<std::mutex> lock(mu);
  const auto key = std::make_pair(dev, reinterpret_cast<const void *>(kernel));
  auto it = known.find(key);
  if (it != known.end()) return it->second;
  int cus = 0, per_cu = 0;
  unsigned r = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kernel), threads, 0) ==
          hipSuccess &&
      cus > 0 && per_cu > 0)
    r = (unsigned)cus * (unsigned)per_cu;
  known[key] = r;
  return r;
}

// compute units of the current device (0 if the runtime cannot tell)
inline int device_compute_units() {
  static std::mutex mu;
  static std::map<int, int> known;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  std::lock_guard<std::mutex> lock(mu);
  auto it = known.find(dev);
  if (it != known.end()) return it->second;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
  known[dev] = cus;
  return cus;
}

const std::vector<Instance> &registry();
// the kernel that interprets KArgs::code: takes elementwise clusters that no entry of the registry matches
const Instance *interpreter_instance();
// first instance with this signature whose accept() (if any) passes
const Instance *find_instance(const std::string &sig, const KArgs &a);

}  // namespace fc
