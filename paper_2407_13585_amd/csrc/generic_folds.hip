// Instances that take any element program (Interp<K, T> runs it from the launch's code):
// segmented folds and scatters.  The matcher turns to them when no instance was compiled
// for a cluster's own element programs.
#include "launchers.hpp"

namespace fc {

void append_generic_fold_instances(std::vector<Instance> &r) {
  const size_t first = r.size();
  using XF0 = Interp<0, float>;
  using XI0 = Interp<0, int>;
  using XF1 = Interp<1, float>;
  using XI1 = Interp<1, int>;
  using XI2 = Interp<2, int>;
  r.push_back(foldseg_<AddF32, XF0>());
  r.push_back(foldseg_<MaxF32, XF0>());
  r.push_back(foldseg_<AddI32, XI0>());
  // index, value, flag (or none); overwrite or combine
  r.push_back(scatter_<XI0, XF1, XI2>());
  r.push_back(scatter_<XI0, XI1, XI2>());
  r.push_back(scatter_<XI0, XF1, AlwaysOne>());
  r.push_back(scatter_<XI0, XI1, AlwaysOne>());
  r.push_back(scatter_<XI0, XF1, XI2, true>());
  r.push_back(scatter_<XI0, XI1, XI2, true>());
  r.push_back(scatter_<XI0, XF1, AlwaysOne, true>());
  r.push_back(scatter_<XI0, XI1, AlwaysOne, true>());
  for (size_t k = first; k < r.size(); ++k) r[k].variant = "element programs interpreted";
}

}  // namespace fc
