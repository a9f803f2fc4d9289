// Launchers and instance builders shared by the translation units that fill the registry
// (instances.hip: the instances compiled for particular element programs; generic_*.hip:
// the instances that take any element program).  Everything here has internal linkage.
#pragma once

#include "kernels.hpp"
#include "registry.hpp"

#include <algorithm>
#include <cmath>
#include <string>
#include <tuple>
#include <utility>
#include <vector>

namespace fc {

// defined in generic_folds.hip, generic_rows.hip, generic_scans.hip
void append_generic_fold_instances(std::vector<Instance> &r);
void append_generic_row_instances(std::vector<Instance> &r);
void append_generic_scan_instances(std::vector<Instance> &r);

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
  return !(a.flags & kSinglePass) && a.n > 0 && (unsigned long long)a.n * 4 < (1ull << 31) && table > kL2Bytes && table <= kQuarters * kL2Bytes && units >= 64 &&
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
  return !(a.flags & kSinglePass) && a.n >= (1 << 21) && bytes > kL2Bytes && bytes <= kBins * (kL2Bytes * 2) &&
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

// ---- the same fold with the table ranges in LDS: tables of more than one L2 and at most 2^24 elements ----
// The table in kFineBins ranges of equal length (a multiple of four elements, so that every range
// starts on a 128-bit boundary) and the multiplication that stands for the division by that length.
// With 2^k >= limit * range and magic = floor(2^k / range) + 1, umulhi(j, magic) >> (k - 32) is
// j / range for every j < limit; the check below walks the range boundaries inside the table, where a
// wrong quotient would show first, and an empty FineCut (bins == 0) says that this table is not to be
// cut this way.
inline FineCut fine_cut(size_t elems, unsigned max_bins = kFineBins, unsigned max_range = kFineSlice) {
  const FineCut none = {0, 0, 0, 0};
  if (elems == 0 || elems > (size_t)kFineIndexLimit || max_bins == 0) return none;
  const unsigned range = (unsigned)(((elems + max_bins - 1) / max_bins + 3) / 4 * 4);
  if (range > max_range) return none;
  unsigned log2_up = 0;
  while ((1u << log2_up) < range) ++log2_up;
  const unsigned k = 24 + log2_up;
  if (k < 32) return none;
  const unsigned long long magic = (1ull << k) / range + 1;
  if (magic >> 32) return none;
  const FineCut cut = {range, (unsigned)((elems + range - 1) / range), (unsigned)magic, k - 32};
  auto quotient = [&](unsigned j) { return (unsigned)(((unsigned long long)j * cut.magic) >> 32) >> cut.shift; };
  for (unsigned q = 1; q <= cut.bins; ++q) {                  // indices past the table are undefined and clamped by the kernels
    const unsigned at = q * range;
    if (quotient(at - 1) != q - 1 || (at < kFineIndexLimit && quotient(at) != q)) return none;
  }
  return cut;
}
inline unsigned fine_tiles(const KArgs &a) { return (unsigned)(((size_t)(a.n & ~3) + kFineTile - 1) / kFineTile); }
template <class E> bool fold_fine_accept(const KArgs &a) {
  const size_t elems = binned_table_elems<E>(a);
  // Worth it from two million positions on, for tables that no L2 holds, and while there are at
  // least half as many positions as table elements: the second kernel evaluates the whole table.
  // The index array and a range's slots are addressed with 32-bit byte offsets.
  if ((a.flags & kSinglePass) || a.n < (1 << 21) || a.n > (1 << 29) || elems * 4 <= kL2Bytes || (size_t)a.n * 2 < elems) return false;
  return fine_cut(elems).bins != 0;
}
template <class E> size_t fold_fine_workspace(const KArgs &a) {
  // a slot per (range, tile) for all kFineBins ranges: the first kernel writes the empty ones past the table's end too
  return fine_cut(binned_table_elems<E>(a)).bins != 0 ? (size_t)kFineBins * fine_tiles(a) * kFineSlotWords * sizeof(unsigned) : 0;
}
template <class Op, class E> hipError_t launch_fold_fine(const KArgs &a, const LaunchCtx &c) {
  const unsigned elems = (unsigned)binned_table_elems<E>(a);
  const FineCut cut = fine_cut(elems);
  if (!c.workspace || cut.bins == 0) return hipErrorInvalidValue;
  const unsigned tiles = fine_tiles(a);
  unsigned *slots = static_cast<unsigned *>(c.workspace);
  // both kernels fill the LDS of a compute unit: one workgroup of kFineBlock threads per unit
  const int cus = device_compute_units();
  const unsigned units = (unsigned)(cus > 0 ? cus : 256);
  const unsigned first = std::min(tiles, units);
  hipError_t e = launch_k(&bin_fine_kernel<Op, E>, first, c.stream, (int)kFineBlock, a, c.ctl, c.partials, slots, tiles, cut);
  if (e != hipSuccess) return e;
  return launch_k(&fold_fine_kernel<Op, E>, std::min(cut.bins, units), c.stream, (int)kFineBlock, a, c.ctl, c.partials,
                  static_cast<const unsigned *>(slots), tiles, cut, elems, first);
}

// ---- segmented fold over a gathered table, sorted through LDS: tables of more than one L2 and at most 2^24 elements ----
// Ranges as long as LDS takes (so that a slot per range and tile is long and its slack small); a slot holds
// the mean of a uniform spread plus one and a quarter standard deviations (rounded up to whole lines), as far
// as the tile's slots fit their LDS image: every entry of a slot is written and read whether in use or not,
// while the few elements in a thousand that find their slot full cost a gather from memory and six bytes on
// the tile's list each.
inline SegPlan seg_plan(size_t elems, long long n) {
  SegPlan p = {{0, 0, 0, 0}, 0, 0};
  if (elems == 0 || n <= 0) return p;
  const unsigned want = (unsigned)std::min<size_t>((elems + kSegSlice - 1) / kSegSlice, kSegMaxBins);
  p.cut = fine_cut(elems, want, kSegSlice);
  if (p.cut.bins == 0 || p.cut.bins > (unsigned)kSegMaxBins) { p.cut.bins = 0; return p; }
  const double mean = (double)kSegTile / p.cut.bins;
  // whole 128-byte lines of values per slot where that costs little (long slots), whole 128-bit groups anyway
  const unsigned grain = mean >= 96.0 ? 32u : 8u;
  unsigned cap = ((unsigned)(mean + 1.25 * std::sqrt(mean)) + grain - 1) / grain * grain;
  cap = std::min(cap, (unsigned)kSegImageWords / p.cut.bins / 8 * 8);
  p.cap = std::max(cap, 8u);
  p.tiles = (unsigned)(((size_t)n + kSegTile - 1) / kSegTile);
  return p;
}
// the pieces of the workspace, each on a 256-byte boundary
struct SegSpace { size_t offsets, places, gathered, list_place, list_index, list_count, first_row, head, tail, total; };
inline SegSpace seg_space(const SegPlan &p) {
  auto up = [](size_t b) { return (b + 255) / 256 * 256; };
  const size_t entries = (size_t)p.cut.bins * p.tiles * p.cap, positions = (size_t)p.tiles * kSegTile;
  SegSpace s;
  size_t at = 0;
  s.offsets = at;    at += up(entries * 2);
  s.places = at;     at += up(entries * 2);
  s.gathered = at;   at += up(entries * 4);
  s.list_place = at; at += up(positions * 2);
  s.list_index = at; at += up(positions * 4);
  s.list_count = at; at += up((size_t)p.tiles * 4);
  s.first_row = at;  at += up((size_t)p.tiles * 4);
  s.head = at;       at += up((size_t)p.tiles * 4);
  s.tail = at;       at += up((size_t)p.tiles * 4);
  s.total = at;
  return s;
}
template <int KT> bool foldseg_sorted_accept(const KArgs &a) {
  const size_t table = blocked_table_bytes<KT>(a);
  // From four million elements on, for tables that no L2 holds: measured at sixteen elements a row over
  // tables of 8, 16 and 64 MiB, 2^21 elements take 50-56 us this way and 37-47 us with the kernels above,
  // 2^22 elements 61-70 against 58-87, 2^23 elements 81-91 against 100-167.  Positions and byte offsets
  // into a range's slots are 32-bit numbers.
  if ((a.flags & kSinglePass) || a.n < (1 << 22) || a.n > (1 << 28) || a.aux <= 0 || table <= kL2Bytes) return false;
  return seg_plan(table / 4, a.n).cut.bins != 0;
}
template <int KT> size_t foldseg_sorted_workspace(const KArgs &a) {
  const SegPlan p = seg_plan(blocked_table_bytes<KT>(a) / 4, a.n);
  return p.cut.bins != 0 ? seg_space(p).total : 0;
}
template <class Op, class F, int KV, int KI, int KT>
hipError_t launch_foldseg_sorted(const KArgs &a, const LaunchCtx &c) {
  using T = typename Op::T;
  const unsigned elems = (unsigned)(blocked_table_bytes<KT>(a) / 4);
  const SegPlan p = seg_plan(elems, a.n);
  if (!c.workspace || p.cut.bins == 0) return hipErrorInvalidValue;
  const SegSpace s = seg_space(p);
  char *w = static_cast<char *>(c.workspace);
  unsigned short *offsets = reinterpret_cast<unsigned short *>(w + s.offsets), *places = reinterpret_cast<unsigned short *>(w + s.places);
  T *gathered = reinterpret_cast<T *>(w + s.gathered);
  unsigned short *list_place = reinterpret_cast<unsigned short *>(w + s.list_place);
  unsigned *list_index = reinterpret_cast<unsigned *>(w + s.list_index);
  unsigned *list_count = reinterpret_cast<unsigned *>(w + s.list_count), *first_row = reinterpret_cast<unsigned *>(w + s.first_row);
  T *head = reinterpret_cast<T *>(w + s.head), *tail = reinterpret_cast<T *>(w + s.tail);
  const int cus = device_compute_units();
  const unsigned units = (unsigned)(cus > 0 ? cus : 256);
  hipError_t e = launch_k(&seg_bin_kernel<KI>, std::min(p.tiles, units), c.stream, (int)kSegBlock, a, offsets, places,
                          list_place, list_index, list_count, p, elems);
  if (e != hipSuccess) return e;
  // A table range is read into LDS by every workgroup that works on it, and a workgroup fills the LDS of a compute
  // unit: as few parts per range as give whole rounds of workgroups, or nearly (128 ranges in two parts each on 256
  // units: 102 us; in four parts, two rounds: 106 us; 114 ranges in three parts, a round and a third: 110 us)
  unsigned parts = 1;
  {
    // rounds of workgroups times the share of the work a workgroup takes, for one to eight parts per range
    auto cost = [&](unsigned q) { return (double)((p.cut.bins * q + units - 1) / units) / (p.cut.bins * q); };
    for (unsigned q = 2; q <= 8; ++q)
      if (cost(q) < cost(parts) * 0.999) parts = q;
  }
  e = launch_k(&seg_gather_kernel<T, KT>, p.cut.bins * parts, c.stream, (int)kSegBlock, a, static_cast<const unsigned short *>(offsets),
               gathered, first_row, p, elems, parts);
  if (e != hipSuccess) return e;
  e = launch_k(&seg_rows_kernel<Op, F, KV, KT>, p.tiles, c.stream, (int)kSegRowsBlock, a, static_cast<const unsigned short *>(places),
               static_cast<const T *>(gathered), static_cast<const unsigned short *>(list_place), static_cast<const unsigned *>(list_index),
               static_cast<const unsigned *>(list_count), static_cast<const unsigned *>(first_row), head, tail, p);
  if (e != hipSuccess) return e;
  return launch_k(&seg_join_kernel<Op>, (p.tiles + kBlock - 1) / kBlock, c.stream, a, static_cast<const unsigned *>(first_row),
                  static_cast<const T *>(head), static_cast<const T *>(tail), p.tiles);
}

template <class EX, class EV, int Mode, bool Reverse = false> hipError_t launch_scan(const KArgs &a, const LaunchCtx &c) {
  long long tiles = std::max<long long>(1, ((long long)a.n + kScanTile - 1) / kScanTile);
  if (scan_status_words((size_t)tiles) > c.max_tiles) return hipErrorInvalidValue;
  return launch_k(&scan_kernel<EX, EV, Mode, Reverse>, (unsigned)tiles, c.stream, kScanBlock, a, c.ctl, c.status, (unsigned)tiles);
}
// lanes per row by row length, as for the row folds
template <class EX, bool Reverse = false, bool StoreX = false> hipError_t launch_scan_f32(const KArgs &a, const LaunchCtx &c) {
  long long tiles = std::max<long long>(1, ((long long)a.n + kScanFTile - 1) / kScanFTile);
  if (scan_status_words((size_t)tiles) > c.max_tiles) return hipErrorInvalidValue;
  return launch_k(&scan_f32_kernel<EX, Reverse, StoreX>, (unsigned)tiles, c.stream, kScanBlock, a, c.ctl, c.status, (unsigned)tiles);
}
template <class E, bool Reverse, bool StoreX = false> hipError_t launch_rowscan(const KArgs &a, const LaunchCtx &c) {
  if (a.aux == 0 || a.w == 0) return hipSuccess;
  if (a.w <= 64)
    return launch_k(&rowscan_kernel<E, Reverse, 16, StoreX>, grid_for(a.aux, kBlock / 16, resident_grid(&rowscan_kernel<E, Reverse, 16, StoreX>)), c.stream, a);
  if (a.w <= 1024)
    return launch_k(&rowscan_kernel<E, Reverse, kWave, StoreX>, grid_for(a.aux, kBlock / kWave, resident_grid(&rowscan_kernel<E, Reverse, kWave, StoreX>)), c.stream, a);
  return launch_k(&rowscan_kernel<E, Reverse, kBlock, StoreX>, grid_for(a.aux, 1, resident_grid(&rowscan_kernel<E, Reverse, kBlock, StoreX>)), c.stream, a);
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
  if (Mode & kStoreX) s += "+input";
  return {s, &launch_scan<EX, EV, Mode, Reverse>};
}
template <class EX, bool Reverse = false, bool StoreX = false> Instance scan_f32_() {
  return {std::string(Reverse ? "scanr[" : "scan[") + sig_of<EX>() + "]+offs" + (StoreX ? "+input" : ""),
          &launch_scan_f32<EX, Reverse, StoreX>};
}
template <class E, bool Reverse = false, bool StoreX = false> Instance rowscan_() {
  return {std::string(Reverse ? "rowscanr[" : "rowscan[") + sig_of<E>() + "]+offs" + (StoreX ? "+input" : ""),
          &launch_rowscan<E, Reverse, StoreX>};
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

}  // namespace

}  // namespace fc
