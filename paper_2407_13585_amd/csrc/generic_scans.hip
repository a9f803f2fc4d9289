// Instances that take any element program (Interp<K, T> runs it from the launch's code):
// the single-pass scans, alone and with the scatter and the total of a compaction.
#include "launchers.hpp"

namespace fc {

void append_generic_scan_instances(std::vector<Instance> &r) {
  const size_t first = r.size();
  // the scan kernels run kScanBlock threads; the second element program is the scattered value
  using SI0 = Interp<0, int, kScanBlock>;
  using SF0 = Interp<0, float, kScanBlock>;
  using SI1 = Interp<1, int, kScanBlock>;
  using SF1 = Interp<1, float, kScanBlock>;
  r.push_back(scan_<SI0, SI0, kOffs>());
  r.push_back(scan_<SI0, SI0, kOffs, true>());
  r.push_back(scan_<SI0, SI0, kOffs | kCount>());
  r.push_back(scan_<SI0, SI1, kScatter>());
  r.push_back(scan_<SI0, SF1, kScatter>());
  r.push_back(scan_<SI0, SI1, kScatter | kCount>());
  r.push_back(scan_<SI0, SF1, kScatter | kCount>());
  r.push_back(scan_<SI0, SI1, kOffs | kScatter | kCount>());
  r.push_back(scan_<SI0, SF1, kOffs | kScatter | kCount>());
  // the scanned stream stored as well
  r.push_back(scan_<SI0, SI0, kOffs | kStoreX>());
  r.push_back(scan_<SI0, SI0, kOffs | kStoreX, true>());
  r.push_back(scan_<SI0, SI0, kOffs | kCount | kStoreX>());
  r.push_back(scan_<SI0, SI1, kScatter | kCount | kStoreX>());
  r.push_back(scan_<SI0, SF1, kScatter | kCount | kStoreX>());
  r.push_back(scan_<SI0, SI1, kOffs | kScatter | kCount | kStoreX>());
  r.push_back(scan_<SI0, SF1, kOffs | kScatter | kCount | kStoreX>());
  r.push_back(scan_f32_<SF0>());
  r.push_back(scan_f32_<SF0, true>());
  r.push_back(scan_f32_<SF0, false, true>());
  r.push_back(scan_f32_<SF0, true, true>());
  for (size_t k = first; k < r.size(); ++k) r[k].variant = "element programs interpreted";
}

}  // namespace fc
