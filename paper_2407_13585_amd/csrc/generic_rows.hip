// Instances that take any element program (Interp<K, T> runs it from the launch's code):
// folds and scans over the rows of a two-dimensional array.
#include "launchers.hpp"

namespace fc {

void append_generic_row_instances(std::vector<Instance> &r) {
  const size_t first = r.size();
  using XF0 = Interp<0, float>;
  using XI0 = Interp<0, int>;
  using XI1 = Interp<1, int>;
  r.push_back(rowscan_<XI0>());
  r.push_back(rowscan_<XI0, true>());
  r.push_back(rowscan_<XF0>());
  r.push_back(rowscan_<XF0, true>());
  // the scanned array stored as well
  r.push_back(rowscan_<XI0, false, true>());
  r.push_back(rowscan_<XI0, true, true>());
  r.push_back(rowscan_<XF0, false, true>());
  r.push_back(rowscan_<XF0, true, true>());
  r.push_back(rowfold_<AddF32, NoSecondOp, XF0>());
  r.push_back(rowfold_<MulF32, NoSecondOp, XF0>());
  r.push_back(rowfold_<MaxF32, NoSecondOp, XF0>());
  r.push_back(rowfold_<AddI32, NoSecondOp, XI0>());
  r.push_back(rowfold_<AddF32, NoSecondOp, XF0, XI1>());     // consumed by a gather that picks the row
  r.push_back(rowfold_<AddF32, MulF32, XF0>());              // two reducers over one element program
  for (size_t k = first; k < r.size(); ++k) r[k].variant = "element programs interpreted";
}

}  // namespace fc
