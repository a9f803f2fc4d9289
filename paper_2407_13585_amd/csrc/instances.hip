// Kernel instances: the cluster shapes the library can execute, each a skeleton
// (kernels.hpp) specialised with an element program (expr.hpp).  The unfused arm
// runs one singleton cluster per combinator through the same skeletons, so fused
// and unfused execution share every primitive.
#include "launchers.hpp"
#include "stencil.hpp"

#include <algorithm>

namespace fc {

namespace {

using F0 = In<0, float>;
using F1 = In<1, float>;
using F2 = In<2, float>;
using F3 = In<3, float>;
using F4 = In<4, float>;
using I0 = In<0, int>;
using I1 = In<1, int>;
using I2 = In<2, int>;

// element programs of the fused pipelines
// r = fold(+)(zipWith(*) (map(ax+b) xs) (gather(reverse, map(ax+b) xs)))      [map duplicated per order]
using ReverseDot = Map<FnMul2, Map<FnAffine, F0>, Gather<Gen<GenIotaRev>, Map<FnAffine, F0>>>;
// r = fold(+)(map(z*z+1)(gather(idx, map(sin x * x) xs)))                      [`simple1` shape]
using PermGather = Map<FnSqPlusOne, Gather<I0, Map<FnSinXMulX, F1>>>;
// y = foldSeg(+)(zipWith(*) vals (gather(col, x)))
using SpmvTerm = Map<FnMul2, F0, Gather<I1, F2>>;
// compaction: flags = map(v mod k == r) v, value = v
using ModFlag = Map<FnModEq, I0>;
// stencil with the producer recomputed at every gathered position
using ExpNeg0 = Map<FnExpNeg, F0>;
using ShiftedExp = Gather<Gen<GenClampShift2D>, ExpNeg0>;
using Stencil5 = Map<FnAdd5, ExpNeg0, ShiftedExp, ShiftedExp, ShiftedExp, ShiftedExp>;
// the same stencil reading a materialised p
using ShiftedIn = Gather<Gen<GenClampShift2D>, F0>;
using Stencil5Mat = Map<FnAdd5, F0, ShiftedIn, ShiftedIn, ShiftedIn, ShiftedIn>;

// specialised instances come first: they share the signature of a generic one
// and take over when their accept() passes
void append_stencil_instances(std::vector<Instance> &r) {
  // pre-order slots of Stencil5: 0 add5, 1 exp, 2 in, then (gather, gen, exp, in) x 4
  static_assert(Stencil5::kNodes == 19 && Stencil5Mat::kNodes == 14, "slot numbering");
  Instance a = store_fold_<Stencil5, MaxF32, ExpNeg0>();
  a.launch = &launch_stencil5<FnExpNeg, 1, true>;
  a.accept = &stencil5_accept<FnExpNeg, 1, true, 4, 4>;
  a.variant = "rows-in-registers";
  r.push_back(a);
  Instance b = store_<Stencil5>();
  b.launch = &launch_stencil5<FnExpNeg, 1, false>;
  b.accept = &stencil5_accept<FnExpNeg, 1, false, 4, 4>;
  b.variant = "rows-in-registers";
  r.push_back(b);
  // pre-order slots of Stencil5Mat: 0 add5, 1 in, then (gather, gen, in) x 4
  Instance c = store_<Stencil5Mat>();
  c.launch = &launch_stencil5<FnIdentF, 0, false>;
  c.accept = &stencil5_accept<FnIdentF, 0, false, 3, 3>;
  c.variant = "rows-in-registers";
  r.push_back(c);
}

std::vector<Instance> build_registry() {
  std::vector<Instance> r;
  append_stencil_instances(r);
  // ---- singleton clusters (the unfused arm) ----
  r.push_back(store_<Map<FnIdentF, F0>>());
  r.push_back(store_<Map<FnIdentI, I0>>());
  r.push_back(store_<Map<FnAffine, F0>>());
  r.push_back(store_<Map<FnSinXMulX, F0>>());
  r.push_back(store_<Map<FnSqPlusOne, F0>>());
  r.push_back(store_<Map<FnExpNeg, F0>>());
  r.push_back(store_<Map<FnMul2, F0, F1>>());
  r.push_back(store_<Map<FnAdd2, F0, F1>>());
  r.push_back(store_<Map<FnAdd3, F0, F1, F2>>());
  r.push_back(store_<Map<FnAdd5, F0, F1, F2, F3, F4>>());
  r.push_back(store_<Map<FnModEq, I0>>());
  r.push_back(store_<Gen<GenIota>>());
  r.push_back(store_<Gen<GenIotaRev>>());
  r.push_back(store_<Gen<GenClampShift2D>>());
  r.push_back(store_<Gen<GenRowOf2D>>());
  r.push_back(store_<Gen<GenConst>>());
  r.push_back(store_<Gather<I0, F1>>());
  r.push_back(store_<Gather<I0, I1>>());
  r.push_back(fold_<AddF32, F0>());
  r.push_back(fold_<MaxF32, F0>());
  r.push_back(fold_<MulF32, F0>());
  r.push_back(fold_<AddI32, I0>());
  r.push_back(fold_<MaxI32, I0>());
  r.push_back(foldseg_<AddF32, F0>());
  r.push_back(foldseg_<MaxF32, F0>());
  r.push_back(foldseg_<AddI32, I0>());
  r.push_back(scan_<I0, I0, kOffs>());
  r.push_back(scan_<I0, I0, kOffs, true>());                  // scanr: the same pass over the mirrored index space
  // scans of two-dimensional arrays: every row on its own; the second with its producer fused in
  r.push_back(rowscan_<I0>());
  r.push_back(rowscan_<I0, true>());
  r.push_back(rowscan_<ModFlag>());
  r.push_back(rowscan_<ModFlag, true>());
  r.push_back(rowscan_<ModFlag, false, true>());                 // the flags stored as well
  // prefix sums of fp32 arrays, alone and with a producer fused in
  r.push_back(scan_f32_<F0>());
  r.push_back(scan_f32_<F0, true>());
  r.push_back(scan_f32_<Map<FnAffine, F0>>());
  r.push_back(scan_f32_<Map<FnAffine, F0>, false, true>());       // the scanned array stored as well
  r.push_back(scan_f32_<Map<FnMul2, F0, F1>>());
  r.push_back(rowscan_<F0>());
  r.push_back(rowscan_<F0, true>());
  r.push_back(scatter_<I0, I1, I2>());
  r.push_back(scatter_<I0, F1, I2>());
  // the instances that take any element program (the matcher turns to them when none of
  // this file matches a cluster's own element programs)
  append_generic_fold_instances(r);
  append_generic_row_instances(r);
  append_generic_scan_instances(r);
  // ---- fused clusters ----
  r.push_back(fold_<AddF32, ReverseDot>());
  {
    // the gathered table does not fit one L2 but its ranges fit LDS: indices binned by range, gathers from LDS (first match wins)
    Instance fine = fold_<AddF32, PermGather>();
    fine.launch = &launch_fold_fine<AddF32, PermGather>;
    fine.accept = &fold_fine_accept<PermGather>;
    fine.workspace = &fold_fine_workspace<PermGather>;
    fine.variant = "binned, table ranges in LDS";
    r.push_back(fine);
  }
  {
    // the gathered table does not fit one L2: indices binned by table range first (first match wins)
    Instance binned = fold_<AddF32, PermGather>();
    binned.launch = &launch_fold_binned<AddF32, PermGather>;
    binned.accept = &fold_binned_accept<PermGather>;
    binned.workspace = &fold_binned_workspace;
    binned.variant = "binned";
    r.push_back(binned);
  }
  r.push_back(fold_<AddF32, PermGather>());
  {
    // SpMV-shaped cluster over a table that no L2 holds, up to 2^24 elements: sorted through LDS (first match wins)
    Instance sorted = foldseg_<AddF32, SpmvTerm>();
    sorted.launch = &launch_foldseg_sorted<AddF32, FnMul2, 0, 1, 2>;
    sorted.accept = &foldseg_sorted_accept<2>;
    sorted.workspace = &foldseg_sorted_workspace<2>;
    sorted.variant = "sorted through LDS";
    r.push_back(sorted);
  }
  {
    // SpMV-shaped cluster over a table of one to four L2s: column blocked (first match wins)
    Instance blocked = foldseg_<AddF32, SpmvTerm>();
    blocked.launch = &launch_foldseg_blocked<AddF32, FnMul2, 0, 1, 2>;
    blocked.accept = &foldseg_blocked_accept<2>;
    blocked.workspace = &foldseg_blocked_workspace;
    blocked.variant = "column-blocked";
    r.push_back(blocked);
  }
  r.push_back(foldseg_<AddF32, SpmvTerm>());
  r.push_back(scan_<ModFlag, I0, kScatter | kCount>());
  r.push_back(scan_<ModFlag, I0, kScatter>());
  r.push_back(scan_<ModFlag, I0, kOffs | kCount>());
  // the predicate is a result as well (stored from the registers it was computed into)
  r.push_back(scan_<ModFlag, I0, kOffs | kStoreX>());
  r.push_back(scan_<ModFlag, I0, kScatter | kCount | kStoreX>());
  r.push_back(store_fold_<Stencil5, MaxF32, ExpNeg0>());
  r.push_back(store_fold_<ExpNeg0, MaxF32, ExpNeg0>());       // diagonal: p stored and folded
  r.push_back(store_<Stencil5Mat>());
  r.push_back(store_<Stencil5>());
  // clusters of the strict (no duplication) optimum of the reverse-dot pipeline
  r.push_back(fold_<AddF32, Map<FnMul2, F0, Gather<Gen<GenIotaRev>, F0>>>());
  // partial fusions used by tests of the fusion rules
  r.push_back(store_<Gather<I0, Map<FnAffine, F1>>>());       // `simple1`
  r.push_back(store_<Gather<I0, Gather<I1, F2>>>());          // `simple2`
  r.push_back(store_<Gather<Gen<GenIotaRev>, F0>>());         // reverse / backpermute
  r.push_back(store_<Map<FnSqPlusOne, Gather<I0, Map<FnSinXMulX, F1>>>>());
  r.push_back(fold_<AddF32, Map<FnSqPlusOne, F0>>());
  r.push_back(fold_<AddF32, Gather<I0, F1>>());               // bare gather + fold: the gather-rate ceiling
  // ---- example programs of the paper ----
  // `singleLoop`: one loop, no intermediates, the input read in two orders
  r.push_back(store_<Map<FnAdd3, Gather<Gen<GenIotaRev>, F0>, Map<FnAffine, F0>, Map<FnSqPlusOne, Map<FnAffine, F0>>>>());
  // `greedyTopDownBad`: cs fused vertically into es and the fold; bs read twice from memory
  r.push_back(fold_<AddF32, Map<FnAdd2, Map<FnAffine, F0>, Map<FnIdentF, F0>>>());
  // `simple5`: one array read in order 0 and in a gather's order inside one loop
  r.push_back(store_<Map<FnMul2, Map<FnSqPlusOne, F0>, Gather<I1, F0>>>());
  // diagonal fusion: a map stored and forwarded to the next map, which is stored too
  r.push_back(store2_<Map<FnAffine, F0>, Map<FnAffine, Map<FnAffine, F0>>>());
  r.push_back(store2_<Map<FnIdentI, I0>, Map<FnIdentI, I0>>());
  // `scatterExample`: combining scatter with its source tuple fused in
  r.push_back(scatter_<Map<FnIdentI, I0>, Map<FnIdentI, I0>, AlwaysOne, true>());
  r.push_back(scatter_<I0, I1, AlwaysOne, true>());
  r.push_back(scatter_<I0, I0, AlwaysOne, true>());
  r.push_back(scatter_<I0, I1, I2, true>());
  r.push_back(scatter_<I0, F1, AlwaysOne, true>());          // fp32 sums: the order of the updates is not fixed
  r.push_back(scatter_<I0, F1, I2, true>());
  r.push_back(scatter_<I0, I1, AlwaysOne>());
  r.push_back(scatter_<I0, F1, AlwaysOne>());
  // row folds: alone (the unfused arm), under a gather (`simple4`), and two folds that
  // contract a gathered 2-D array (`greedyBottomUpBad`)
  r.push_back(rowfold_<AddF32, NoSecondOp, F0>());
  r.push_back(rowfold_<MulF32, NoSecondOp, F0>());
  r.push_back(rowfold_<MaxF32, NoSecondOp, F0>());
  r.push_back(rowfold_<AddI32, NoSecondOp, I0>());
  r.push_back(rowfold_<AddF32, NoSecondOp, F0, I1>());
  r.push_back(rowfold_<AddF32, MulF32, Gather<Gen<GenRowOf2D>, F0>>());
  r.push_back(rowfold_<AddF32, NoSecondOp, Gather<Gen<GenRowOf2D>, F0>>());
  r.push_back(rowfold_<MulF32, NoSecondOp, Gather<Gen<GenRowOf2D>, F0>>());
  r.push_back(store_<Gather<Gen<GenRowOf2D>, F0>>());
  r.push_back(store_<Map<FnMul2, F0, Gather<I1, F2>>>());
  return r;
}

}  // namespace

const std::vector<Instance> &registry() {
  static const std::vector<Instance> r = build_registry();
  return r;
}

static hipError_t launch_interp(const KArgs &a, const LaunchCtx &c) {
  // a fold of the cluster keeps a partial per workgroup; there may be kInterpFolds of them
  const unsigned cap = std::min<unsigned>(resident_grid(&interp_kernel<>), kMaxPartials / kInterpFolds);
  return launch_k(&interp_kernel<>, grid_for(a.n, kBlock * kVec, cap), c.stream, a, c.ctl, c.partials);
}
const Instance *interpreter_instance() {
  static const Instance inst = [] {
    Instance i{"", &launch_interp};
    i.variant = "interpreted";
    return i;
  }();
  return &inst;
}

const Instance *find_instance(const std::string &sig, const KArgs &a) {
  for (const Instance &i : registry())
    if (i.sig == sig && (!i.accept || i.accept(a))) return &i;
  return nullptr;
}

}  // namespace fc
