// Cluster skeletons: one kernel template per consumer shape.  The element
// program of the cluster (expr.hpp) is a template argument, so a cluster is one
// kernel and its intermediates live in registers (sections 1 and 3: vertical
// fusion forwards a value, horizontal fusion shares a load, diagonal fusion
// forwards and stores).
#pragma once

#include <tuple>
#include <utility>

#include "expr.hpp"

namespace fc {

constexpr int kVec = 4;                            // elements per 128-bit access
constexpr int kUnroll = 4;                         // independent accesses in flight per lane
constexpr int kTile = kBlock * kVec * kUnroll;     // 4096 elements per workgroup step

template <class T>
__device__ __forceinline__ void store4(T *p, const Vec4<T> &v) {
  using V = T __attribute__((ext_vector_type(4)));
  V x = {v.v[0], v.v[1], v.v[2], v.v[3]};
  *reinterpret_cast<V *>(p) = x;
}

// ------------------------------------------------------------------ elementwise: out[i] = E(i)
template <class E>
__global__ __launch_bounds__(kBlock) void store_kernel(const KArgs a) {
  using T = typename E::R;
  T *out = static_cast<T *>(a.out[0]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  for (unsigned base = blockIdx.x * kTile; base < n4; base += gridDim.x * kTile) {
    Vec4<T> v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < n4) v[u] = E::template eval4<0>(a, (int)i);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < n4) store4(out + i, v[u]);
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) out[n4 + threadIdx.x] = E::template eval<0>(a, (int)(n4 + threadIdx.x));
}

// ------------------------------------------------------------------ fold (and store + fold)
// Per-lane accumulation in a fixed order, DPP wave reduction, LDS workgroup
// reduction, one partial per workgroup; the workgroup that finishes last
// combines the partials in index order, so the result does not depend on
// scheduling.  fold is one stage of a multi-stage parallel reduction (section 2, fold).
template <class Op>
__device__ __forceinline__ void fold_finish(typename Op::T acc, const KArgs &a, int out_slot, Control *ctl,
                                            unsigned long long *partials) {
  using T = typename Op::T;
  __shared__ T lds[kWavesPerBlock + 1];
  const unsigned epoch = load_agent(&ctl->epoch);
  const unsigned tag = tag_of_epoch(epoch);
  T r = block_reduce<Op>(acc, lds);
  if (threadIdx.x == 0) store_agent64(&partials[blockIdx.x], pack_word((unsigned)as_bits(r), tag, 1u));
  // the workgroup with the highest index is dispatched last; it waits for the
  // partials of all others and combines them in index order
  if (blockIdx.x == gridDim.x - 1) {
    T s = Op::identity();
    for (unsigned k = threadIdx.x; k < gridDim.x; k += kBlock) {
      unsigned long long w = wait_word(&partials[k], tag, ctl);
      s = Op::apply(s, w ? from_bits<T>((int)(unsigned)(w >> 32)) : Op::identity());
    }
    s = block_reduce<Op>(s, lds);
    if (threadIdx.x == 0) {
      *static_cast<T *>(a.out[out_slot]) = s;
      store_agent(&ctl->epoch, epoch + 1u);
    }
  }
}

template <class Op, class E>
__global__ __launch_bounds__(kBlock) void fold_kernel(const KArgs a, Control *ctl, unsigned long long *partials) {
  using T = typename Op::T;
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  T acc = Op::identity();
  for (unsigned base = blockIdx.x * kTile; base < n4; base += gridDim.x * kTile) {
    Vec4<T> v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < n4) {
        v[u] = E::template eval4<0>(a, (int)i);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[u].v[c] = Op::identity();
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc = Op::apply(acc, v[u].v[c]);
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) acc = Op::apply(acc, E::template eval<0>(a, (int)(n4 + threadIdx.x)));
  fold_finish<Op>(acc, a, 0, ctl, partials);
}

// out[0][i] = ES(i) and out[1] = fold(Op, EF(i)) in one pass
template <class ES, class Op, class EF>
__global__ __launch_bounds__(kBlock) void store_fold_kernel(const KArgs a, Control *ctl, unsigned long long *partials) {
  using T = typename Op::T;
  using S = typename ES::R;
  S *out = static_cast<S *>(a.out[0]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  T acc = Op::identity();
  for (unsigned base = blockIdx.x * kTile; base < n4; base += gridDim.x * kTile) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < n4) {
        Vec4<S> s = ES::template eval4<0>(a, (int)i);
        Vec4<T> f = EF::template eval4<ES::kNodes>(a, (int)i);
        store4(out + i, s);
#pragma unroll
        for (int c = 0; c < 4; ++c) acc = Op::apply(acc, f.v[c]);
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) {
    int i = (int)(n4 + threadIdx.x);
    out[i] = ES::template eval<0>(a, i);
    acc = Op::apply(acc, EF::template eval<ES::kNodes>(a, i));
  }
  fold_finish<Op>(acc, a, 1, ctl, partials);
}

// ------------------------------------------------------------------ segmented fold
// y[r] = fold(Op, E(k) for k in [off[r], off[r+1])).  One 16-lane DPP row per
// segment: lanes stride through the segment, the row is reduced with row_shr
// steps, lane 15 stores.  Offsets are external array kMaxIn-1.  An empty segment
// yields the identity.
template <class Op, class E>
__global__ __launch_bounds__(kBlock) void foldseg_kernel(const KArgs a) {
  using T = typename Op::T;
  const int *off = static_cast<const int *>(a.in[kMaxIn - 1]);
  T *y = static_cast<T *>(a.out[0]);
  const unsigned rows = (unsigned)a.aux;
  const unsigned sub = threadIdx.x & 15u;
  const unsigned rows_per_step = gridDim.x * (kBlock / 16);
  // every lane of a wave runs the same number of steps so the DPP moves stay converged
  const unsigned steps = (rows + rows_per_step - 1) / rows_per_step;
  for (unsigned s = 0; s < steps; ++s) {
    unsigned r = s * rows_per_step + blockIdx.x * (kBlock / 16) + threadIdx.x / 16;
    int lo = 0, hi = 0;
    if (r < rows) { lo = off[r]; hi = off[r + 1]; }
    T acc = Op::identity();
    for (int k = lo + (int)sub; k < hi; k += 16) acc = Op::apply(acc, E::template eval<0>(a, k));
    acc = row_scan_inclusive<Op>(acc);
    if (sub == 15 && r < rows) y[r] = acc;
  }
}

// ------------------------------------------------------------------ single-pass scan / compaction
// Exclusive (+) scan of the int32 stream EX in one pass over the data (section
// 2: a scan inside a cluster must be a single pass; the chained scan is one of
// the implementations named there).  Tile t is processed by workgroup t; each
// tile publishes its aggregate, then looks back over the status words of its
// predecessors until it meets an inclusive prefix (decoupled look-back).
// Workgroups are dispatched in index order, so the lowest unfinished tile is
// always running and can always finish; every wait is bounded all the same.
// The scan result never reaches memory unless asked for: kOffs stores it,
// kScatter writes EV(i) to dest[offs[i]] where EX(i) != 0 (scatter with
// collision-free indices: plain stores, no atomics), kCount stores the total.
constexpr int kScanBlock = 512;                       // threads per workgroup of the scan kernels
constexpr int kScanWaves = kScanBlock / kWave;
constexpr int kScanItems = 16;                        // per lane
constexpr int kScanTile = kScanBlock * kScanItems;    // 8192 elements
constexpr int kOffs = 1, kScatter = 2, kCount = 4;

template <class EX, class EV, int Mode>
__global__ __launch_bounds__(kScanBlock) void scan_kernel(const KArgs a, Control *ctl, unsigned long long *status) {
  __shared__ int lds_wave[kScanWaves];
  __shared__ int lds_part[kScanWaves];
  __shared__ int lds_found[kScanWaves];
  using V = typename EV::R;
  const unsigned n = (unsigned)a.n;
  const unsigned n_tiles = gridDim.x;
  const unsigned tile = blockIdx.x;
  const int lane = lane_id(), wave = wave_id();
  const unsigned epoch = load_agent(&ctl->epoch);
  const unsigned tag = tag_of_epoch(epoch);

  // wave-striped layout: wave w owns 1024 consecutive elements; access j of a
  // lane covers elements base + j*256 + lane*4 .. +3 (fully coalesced)
  const unsigned wbase = tile * kScanTile + wave * (kWave * kScanItems);
  int x[4][4];
  V val[4][4];
  int s[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    unsigned i = wbase + j * (kWave * kVec) + lane * kVec;
    if (i + 3 < n) {
      Vec4<int> v = EX::template eval4<0>(a, (int)i);
#pragma unroll
      for (int c = 0; c < 4; ++c) x[j][c] = v.v[c];
      if (Mode & kScatter) {
        Vec4<V> u = EV::template eval4<EX::kNodes>(a, (int)i);
#pragma unroll
        for (int c = 0; c < 4; ++c) val[j][c] = u.v[c];
      }
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        x[j][c] = (i + c < n) ? EX::template eval<0>(a, (int)(i + c)) : 0;
        if (Mode & kScatter) val[j][c] = (i + c < n) ? EV::template eval<EX::kNodes>(a, (int)(i + c)) : V(0);
      }
    }
    s[j] = (x[j][0] + x[j][1]) + (x[j][2] + x[j][3]);
  }
  // exclusive prefix of each access inside the wave
  int excl[4];
  int carry = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int inc = wave_scan_inclusive<AddI32>(s[j]);
    excl[j] = carry + inc - s[j];
    carry += __builtin_amdgcn_readlane(inc, 63);
  }
  if (lane == 0) lds_wave[wave] = carry;
  __syncthreads();
  int wave_excl = 0, aggregate = 0;
#pragma unroll
  for (int k = 0; k < kScanWaves; ++k) {
    int t = lds_wave[k];
    if (k < wave) wave_excl += t;
    aggregate += t;
  }

  // publish the aggregate, then look back: thread t inspects tile - 1 - t, so one
  // round covers the kScanBlock nearest predecessors.  The window has to be wide:
  // the front of known prefixes advances by at most one window per memory round
  // trip, and it must outrun the rate at which tiles stream through the chip.
  if (threadIdx.x == 0) store_agent64(&status[tile], pack_word((unsigned)aggregate, tag, tile == 0 ? 2u : 1u));
  int prefix = 0;
  if (tile > 0) {
    int pred = (int)tile - 1 - (int)threadIdx.x;
    while (true) {
      int value = 0;
      unsigned state = 2u;                 // before the first tile: prefix 0
      if (pred >= 0) {
        unsigned long long w = wait_word(&status[pred], tag, ctl);
        value = (int)(unsigned)(w >> 32);
        state = w ? ((unsigned)w & 3u) : 2u;   // a wait that gave up ends the look-back
      }
      unsigned long long has_prefix = __ballot(state == 2u);
      int first = has_prefix ? (int)__builtin_ctzll(has_prefix) : kWave;
      int part = wave_reduce<AddI32>(lane <= first ? value : 0);
      if (lane == 0) { lds_part[wave] = part; lds_found[wave] = has_prefix != 0; }
      __syncthreads();
      bool found = false;
#pragma unroll
      for (int k = 0; k < kScanWaves; ++k) {
        if (!found) { prefix += lds_part[k]; found = lds_found[k] != 0; }
      }
      __syncthreads();
      if (found) break;
      pred -= kScanBlock;
    }
    if (threadIdx.x == 0) store_agent64(&status[tile], pack_word((unsigned)(prefix + aggregate), tag, 2u));
  }
  const int tile_excl = prefix;

  if (tile == n_tiles - 1 && threadIdx.x == 0) {
    if (Mode & kCount) *static_cast<int *>(a.out[2]) = tile_excl + aggregate;
    // the last tile has seen a prefix that covers every other tile, so all of them
    // have taken their tag: the next launch may use the next one
    store_agent(&ctl->epoch, epoch + 1u);
  }

#pragma unroll
  for (int j = 0; j < 4; ++j) {
    unsigned i = wbase + j * (kWave * kVec) + lane * kVec;
    int o[4];
    o[0] = tile_excl + wave_excl + excl[j];
    o[1] = o[0] + x[j][0];
    o[2] = o[1] + x[j][1];
    o[3] = o[2] + x[j][2];
    if (Mode & kOffs) {
      int *offs = static_cast<int *>(a.out[1]);
      if (i + 3 < n) {
        store4(offs + i, Vec4<int>{{o[0], o[1], o[2], o[3]}});
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) if (i + c < n) offs[i + c] = o[c];
      }
    }
    if (Mode & kScatter) {
      V *dest = static_cast<V *>(a.out[0]);
#pragma unroll
      for (int c = 0; c < 4; ++c) if (i + c < n && x[j][c] != 0) dest[o[c]] = val[j][c];
    }
  }
}

// ------------------------------------------------------------------ scatter (elementwise)
// for every i with EF(i) != 0: dest[EI(i)] = EV(i).  Indices are taken to be
// distinct (overwrite scatter), so plain stores suffice.
template <class EI, class EV, class EF>
__global__ __launch_bounds__(kBlock) void scatter_kernel(const KArgs a) {
  using V = typename EV::R;
  V *dest = static_cast<V *>(a.out[0]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  for (unsigned base = blockIdx.x * kTile; base < n4; base += gridDim.x * kTile) {
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < n4) {
        Vec4<int> f = EF::template eval4<EI::kNodes + EV::kNodes>(a, (int)i);
        Vec4<int> j = EI::template eval4<0>(a, (int)i);
        Vec4<V> v = EV::template eval4<EI::kNodes>(a, (int)i);
#pragma unroll
        for (int c = 0; c < 4; ++c) if (f.v[c] != 0) dest[j.v[c]] = v.v[c];
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) {
    int i = (int)(n4 + threadIdx.x);
    if (EF::template eval<EI::kNodes + EV::kNodes>(a, i) != 0) dest[EI::template eval<0>(a, i)] = EV::template eval<EI::kNodes>(a, i);
  }
}

}  // namespace fc
