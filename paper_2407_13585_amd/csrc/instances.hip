// Kernel instances: the cluster shapes the library can execute, each a skeleton
// (kernels.hpp) specialised with an element program (expr.hpp).  The unfused arm
// runs one singleton cluster per combinator through the same skeletons, so fused
// and unfused execution share every primitive.
#include "kernels.hpp"
#include "registry.hpp"
#include "stencil.hpp"

#include <algorithm>

namespace fc {

namespace {

constexpr unsigned kMaxGrid = 2048;   // 256 CUs x 8 workgroups

unsigned grid_for(int n, int tile, unsigned cap) {
  long long g = ((long long)n + tile - 1) / tile;
  return (unsigned)std::max<long long>(1, std::min<long long>(g, cap));
}

// ---- launchers ------------------------------------------------------------
// Launch through hipLaunchKernel so that the status returned is that of this
// launch (hipGetLastError would also report an error an earlier, unrelated call
// left behind on the thread).
template <class... P, size_t... I>
hipError_t launch_impl(void (*k)(P...), dim3 grid, dim3 block, hipStream_t s, std::tuple<P...> &vals,
                       std::index_sequence<I...>) {
  void *ptrs[] = {static_cast<void *>(&std::get<I>(vals))...};
  return hipLaunchKernel(reinterpret_cast<const void *>(k), grid, block, ptrs, 0, s);
}
template <class... P>
hipError_t launch_k(void (*k)(P...), unsigned grid, hipStream_t s, int block, P... a) {
  std::tuple<P...> vals(a...);
  return launch_impl(k, dim3(grid), dim3(block), s, vals, std::index_sequence_for<P...>());
}
template <class... P>
hipError_t launch_k(void (*k)(P...), unsigned grid, hipStream_t s, P... a) {
  return launch_k(k, grid, s, (int)kBlock, a...);
}
// the kernels that stride over tiles are launched with as many workgroups as are resident at once
template <class... P>
unsigned resident_grid(void (*k)(P...)) {
  const unsigned r = resident_workgroups(k, kBlock);
  return r ? std::min<unsigned>(r, kMaxPartials) : kMaxGrid;
}

template <class E> hipError_t launch_store(const KArgs &a, const LaunchCtx &c) {
  if (a.n == 0) return hipSuccess;
  return launch_k(&store_kernel<E>, grid_for(a.n, kTile, resident_grid(&store_kernel<E>)), c.stream, a);
}
template <class Op, class E> hipError_t launch_fold(const KArgs &a, const LaunchCtx &c) {
  return launch_k(&fold_kernel<Op, E>, grid_for(a.n, kTile, resident_grid(&fold_kernel<Op, E>)), c.stream, a, c.ctl,
                  c.partials);
}
template <class ES, class Op, class EF> hipError_t launch_store_fold(const KArgs &a, const LaunchCtx &c) {
  return launch_k(&store_fold_kernel<ES, Op, EF>, grid_for(a.n, kTile, resident_grid(&store_fold_kernel<ES, Op, EF>)),
                  c.stream, a, c.ctl, c.partials);
}
template <class Op, class E> hipError_t launch_foldseg(const KArgs &a, const LaunchCtx &c) {
  if (a.aux == 0) return hipSuccess;
  return launch_k(&foldseg_kernel<Op, E>, grid_for(a.aux, kBlock / 16, kMaxGrid * 8), c.stream, a);
}
// ---- column-blocked segmented fold: for tables of more than one and at most four L2s ----
constexpr size_t kL2Bytes = 4u << 20;                 // L2 of one XCD
template <int KT> size_t blocked_table_bytes(const KArgs &a) {
  // the table is the last leaf of Map<F, EV, Gather<EI, In<KT>>>; its slot holds its extents
  for (int k = kMaxSlots - 1; k >= 0; --k)
    if (a.p[k].ext[0] != 0) return (size_t)a.p[k].ext[0] * (size_t)a.p[k].ext[1] * 4;
  return 0;
}
template <int KT> bool foldseg_blocked_accept(const KArgs &a) {
  const size_t table = blocked_table_bytes<KT>(a);
  const size_t units = ((size_t)a.aux + kBlockedRows - 1) / kBlockedRows;
  return a.n > 0 && (unsigned long long)a.n * 4 < (1ull << 31) && table > kL2Bytes && table <= kQuarters * kL2Bytes && units >= 64 &&
         units * kQuarters <= kMaxTiles;
}
size_t foldseg_blocked_workspace(const KArgs &a) { return (size_t)kQuarters * (size_t)a.aux * sizeof(unsigned long long); }
template <class Op, class F, int KV, int KI, int KT>
hipError_t launch_foldseg_blocked(const KArgs &a, const LaunchCtx &c) {
  if (!c.workspace) return hipErrorInvalidValue;
  const unsigned units = ((unsigned)a.aux + kBlockedRows - 1) / kBlockedRows;
  unsigned grid = resident_grid(&foldseg_blocked_kernel<Op, F, KV, KI, KT>) / 8 * 8;   // whole rounds of the eight XCDs
  grid = std::max(8u, std::min(grid, units * kQuarters / 8 * 8));
  const size_t elems = blocked_table_bytes<KT>(a) / 4;
  const int range_len = (int)(((elems + kQuarters - 1) / kQuarters + 31) / 32 * 32);    // whole 128-byte lines
  return launch_k(&foldseg_blocked_kernel<Op, F, KV, KI, KT>, grid, c.stream, a, c.ctl, c.partials, c.status,
                  static_cast<unsigned long long *>(c.workspace), range_len);
}

// ---- fold over a gathered table of one to sixty-four L2s: indices sorted by table range first ----
template <class E> size_t binned_table_elems(const KArgs &a) {
  constexpr int slot = GatherChain<E>::template source_slot<0>();
  return (size_t)a.p[slot].ext[0] * (size_t)a.p[slot].ext[1];
}
inline size_t binned_tiles(const KArgs &a) { return ((size_t)(a.n & ~3) + kBinTile - 1) / kBinTile; }
inline size_t binned_counts_bytes(const KArgs &a) { return (binned_tiles(a) * kBins * sizeof(int) + 255) / 256 * 256; }
template <class E> bool fold_binned_accept(const KArgs &a) {
  const size_t bytes = binned_table_elems<E>(a) * 4;
  // Below two million positions the direct kernel is over before two launches would be.  Up to
  // 64 MiB the ranges are half an L2 or less; measured at 2^24 positions: 64 MiB 124 us (direct
  // 307), 128 MiB 132 us (319), 256 MiB, where half of a range fits, 201 us (326).
  return a.n >= (1 << 21) && bytes > kL2Bytes && bytes <= kBins * (kL2Bytes * 2) &&
         binned_tiles(a) * kBins * kBinCap * sizeof(int) < (1ull << 31);
}
size_t fold_binned_workspace(const KArgs &a) { return binned_counts_bytes(a) + binned_tiles(a) * kBins * kBinCap * sizeof(int); }
template <class Op, class E> hipError_t launch_fold_binned(const KArgs &a, const LaunchCtx &c) {
  if (!c.workspace) return hipErrorInvalidValue;
  const unsigned tiles = (unsigned)binned_tiles(a);
  int *counts = static_cast<int *>(c.workspace);
  int *entries = reinterpret_cast<int *>(static_cast<char *>(c.workspace) + binned_counts_bytes(a));
  const size_t range_len = (binned_table_elems<E>(a) + kBins - 1) / kBins;
  const unsigned inv_range = (unsigned)(((1ull << 32) + range_len - 1) / range_len);
  const unsigned first = std::min(tiles, std::min<unsigned>(resident_grid(&bin_indices_kernel<Op, E>), kMaxPartials / 2));
  hipError_t e = launch_k(&bin_indices_kernel<Op, E>, first, c.stream, a, c.ctl, c.partials, counts, entries, tiles, inv_range);
  if (e != hipSuccess) return e;
  // One workgroup per compute unit for the second kernel.  A compute unit's vector cache returns
  // data in request order, so its gathers (L2 hits) queue behind the entry reads (from memory) of
  // whichever wave issued some: with eight workgroups per unit the kernel took 130 us where the
  // gathers alone take 66 and the entry reads alone 27; with one or two it takes their sum.
  const int cus = device_compute_units();
  const unsigned second = std::max(8u, (unsigned)(cus > 0 ? cus : 256) / 8 * 8);
  return launch_k(&fold_binned_kernel<Op, E>, second, c.stream, a, c.ctl, c.partials, static_cast<const int *>(counts),
                  static_cast<const int *>(entries), tiles, first);
}

template <class EX, class EV, int Mode, bool Reverse = false> hipError_t launch_scan(const KArgs &a, const LaunchCtx &c) {
  long long tiles = std::max<long long>(1, ((long long)a.n + kScanTile - 1) / kScanTile);
  if (scan_status_words((size_t)tiles) > c.max_tiles) return hipErrorInvalidValue;
  return launch_k(&scan_kernel<EX, EV, Mode, Reverse>, (unsigned)tiles, c.stream, kScanBlock, a, c.ctl, c.status, (unsigned)tiles);
}
// lanes per row by row length, as for the row folds
template <class EX, bool Reverse = false> hipError_t launch_scan_f32(const KArgs &a, const LaunchCtx &c) {
  long long tiles = std::max<long long>(1, ((long long)a.n + kScanFTile - 1) / kScanFTile);
  if (scan_status_words((size_t)tiles) > c.max_tiles) return hipErrorInvalidValue;
  return launch_k(&scan_f32_kernel<EX, Reverse>, (unsigned)tiles, c.stream, kScanBlock, a, c.ctl, c.status, (unsigned)tiles);
}
template <class E, bool Reverse> hipError_t launch_rowscan(const KArgs &a, const LaunchCtx &c) {
  if (a.aux == 0 || a.w == 0) return hipSuccess;
  if (a.w <= 64)
    return launch_k(&rowscan_kernel<E, Reverse, 16>, grid_for(a.aux, kBlock / 16, resident_grid(&rowscan_kernel<E, Reverse, 16>)), c.stream, a);
  if (a.w <= 1024)
    return launch_k(&rowscan_kernel<E, Reverse, kWave>, grid_for(a.aux, kBlock / kWave, resident_grid(&rowscan_kernel<E, Reverse, kWave>)), c.stream, a);
  return launch_k(&rowscan_kernel<E, Reverse, kBlock>, grid_for(a.aux, 1, resident_grid(&rowscan_kernel<E, Reverse, kBlock>)), c.stream, a);
}
template <class EI, class EV, class EF, bool Add> hipError_t launch_scatter(const KArgs &a, const LaunchCtx &c) {
  if (a.n == 0) return hipSuccess;
  return launch_k(&scatter_kernel<EI, EV, EF, Add>, grid_for(a.n, kTile, resident_grid(&scatter_kernel<EI, EV, EF, Add>)), c.stream, a);
}
template <class E1, class E2> hipError_t launch_store2(const KArgs &a, const LaunchCtx &c) {
  if (a.n == 0) return hipSuccess;
  return launch_k(&store2_kernel<E1, E2>, grid_for(a.n, kTile, resident_grid(&store2_kernel<E1, E2>)), c.stream, a);
}
// lanes per row by row length: a 16-lane DPP row, a wave, or the whole workgroup
template <class Op1, class Op2, class E, class RI> hipError_t launch_rowfold(const KArgs &a, const LaunchCtx &c) {
  if (a.aux == 0) return hipSuccess;
  if (a.w <= 64) return launch_k(&rowfold_kernel<Op1, Op2, E, RI, 16>, grid_for(a.aux, kBlock / 16, kMaxGrid * 4), c.stream, a);
  if (a.w <= 2048) return launch_k(&rowfold_kernel<Op1, Op2, E, RI, kWave>, grid_for(a.aux, kBlock / kWave, kMaxGrid * 4), c.stream, a);
  if (a.aux < 1024 && a.w >= 4 * kTile) {
    // few long rows: cut every row into chunks (a multiple of the 128-bit stride) so that ~2048 workgroups run
    unsigned splits = std::min<unsigned>((unsigned)(a.w / kTile), std::max(1u, 2048u / (unsigned)a.aux));
    splits = std::min<unsigned>(splits, (unsigned)(kMaxPartials / 2) / (unsigned)a.aux);
    if (splits > 1) {
      unsigned chunk = (((unsigned)a.w + splits - 1) / splits + kBlock * kVec - 1) / (kBlock * kVec) * (kBlock * kVec);
      splits = ((unsigned)a.w + chunk - 1) / chunk;
      return launch_k(&rowfold_split_kernel<Op1, Op2, E, RI>, (unsigned)a.aux * splits, c.stream, a, c.ctl, c.partials,
                      splits, chunk);
    }
  }
  return launch_k(&rowfold_kernel<Op1, Op2, E, RI, kBlock>, grid_for(a.aux, 1, kMaxGrid * 4), c.stream, a);
}

// ---- signatures -----------------------------------------------------------
template <class E> std::string sig_of() { std::string s; E::sig(s); return s; }
template <class E> Instance store_() { return {"store[" + sig_of<E>() + "]", &launch_store<E>}; }
template <class Op, class E> Instance fold_() {
  return {std::string("fold.") + Op::name() + "[" + sig_of<E>() + "]", &launch_fold<Op, E>};
}
template <class ES, class Op, class EF> Instance store_fold_() {
  return {"store[" + sig_of<ES>() + "]+fold." + Op::name() + "[" + sig_of<EF>() + "]", &launch_store_fold<ES, Op, EF>};
}
template <class Op, class E> Instance foldseg_() {
  return {std::string("foldseg.") + Op::name() + "[" + sig_of<E>() + "]", &launch_foldseg<Op, E>};
}
template <class EX, class EV, int Mode, bool Reverse = false> Instance scan_() {
  std::string s = std::string(Reverse ? "scanr[" : "scan[") + sig_of<EX>() + "]";
  if (Mode & kOffs) s += "+offs";
  if (Mode & kScatter) s += "+scatter[" + sig_of<EV>() + "]";
  if (Mode & kCount) s += "+count";
  return {s, &launch_scan<EX, EV, Mode, Reverse>};
}
template <class EX, bool Reverse = false> Instance scan_f32_() {
  return {std::string(Reverse ? "scanr[" : "scan[") + sig_of<EX>() + "]+offs", &launch_scan_f32<EX, Reverse>};
}
template <class E, bool Reverse = false> Instance rowscan_() {
  return {std::string(Reverse ? "rowscanr[" : "rowscan[") + sig_of<E>() + "]+offs", &launch_rowscan<E, Reverse>};
}
template <class EI, class EV, class EF, bool Add = false> Instance scatter_() {
  return {std::string(Add ? "scatter.add[" : "scatter[") + sig_of<EI>() + "," + sig_of<EV>() + "," + sig_of<EF>() + "]",
          &launch_scatter<EI, EV, EF, Add>};
}
template <class E1, class E2> Instance store2_() {
  return {"store[" + sig_of<E1>() + "]+store[" + sig_of<E2>() + "]", &launch_store2<E1, E2>};
}
template <class Op1, class Op2, class E, class RI = NoRowIndex> Instance rowfold_() {
  std::string s = std::string("rowfold.") + Op1::name();
  if (!std::is_same<Op2, NoSecondOp>::value) s += std::string("+") + Op2::name();
  s += "[" + sig_of<E>() + "]";
  if (!std::is_same<RI, NoRowIndex>::value) s += "@gather(" + sig_of<RI>() + ")";
  return {s, &launch_rowfold<Op1, Op2, E, RI>};
}

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
  // prefix sums of fp32 arrays, alone and with a producer fused in
  r.push_back(scan_f32_<F0>());
  r.push_back(scan_f32_<F0, true>());
  r.push_back(scan_f32_<Map<FnAffine, F0>>());
  r.push_back(scan_f32_<Map<FnMul2, F0, F1>>());
  r.push_back(rowscan_<F0>());
  r.push_back(rowscan_<F0, true>());
  r.push_back(scatter_<I0, I1, I2>());
  r.push_back(scatter_<I0, F1, I2>());
  // ---- fused clusters ----
  r.push_back(fold_<AddF32, ReverseDot>());
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
  return launch_k(&interp_kernel, grid_for(a.n, kBlock * kVec, resident_grid(&interp_kernel)), c.stream, a, c.ctl, c.partials);
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
