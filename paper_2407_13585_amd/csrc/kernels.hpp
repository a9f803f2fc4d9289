// Cluster skeletons: one kernel template per consumer shape.  The element
// program of the cluster (expr.hpp) is a template argument, so a cluster is one
// kernel and its intermediates live in registers (sections 1 and 3: vertical
// fusion forwards a value, horizontal fusion shares a load, diagonal fusion
// forwards and stores).
#pragma once

#include <tuple>
#include <type_traits>
#include <utility>

#include "expr.hpp"

namespace fc {

constexpr int kVec = 4;                            // elements per 128-bit access
constexpr int kUnroll = 4;                         // independent accesses in flight per lane
constexpr int kTile = kBlock * kVec * kUnroll;     // 4096 elements per workgroup step

// 128-bit store to an array in memory.  A result of the program is written once and not read
// again, so its stores are non-temporal (measured with a plain copy of 256 MiB: 6.3 TB/s with
// non-temporal loads and stores, 5.8 TB/s with ordinary stores).  An array that a later cluster
// of the program reads back (Keep; KArgs::keeps) is written with ordinary stores, so that what
// fits the caches is still there (one kernel per combinator, compaction of 2^26 elements: 355 us
// this way, 391 us with every store non-temporal).  Keep is a compile-time choice: a store
// under a run-time condition is merged with its twin and loses the non-temporal mark.
template <bool Keep, class T>
__device__ __forceinline__ void store4(T *p, const Vec4<T> &v) {
  using V = T __attribute__((ext_vector_type(4)));
  V x = {v.v[0], v.v[1], v.v[2], v.v[3]};
  if (Keep) *reinterpret_cast<V *>(p) = x; else __builtin_nontemporal_store(x, reinterpret_cast<V *>(p));
}
// runs body(std::true_type) or body(std::false_type): the two forms of a kernel's loop
template <class B> __device__ __forceinline__ void with_keep(bool keep, B &&body) {
  if (keep) body(std::true_type()); else body(std::false_type());
}
// the same to LDS
template <class T>
__device__ __forceinline__ void store4_lds(T *p, const Vec4<T> &v) {
  using V = T __attribute__((ext_vector_type(4)));
  V x = {v.v[0], v.v[1], v.v[2], v.v[3]};
  *reinterpret_cast<V *>(p) = x;
}

// Iteration of the elementwise and fold kernels: a workgroup takes tiles of
// kTile elements, a lane kUnroll 128-bit groups per tile.  load(i) evaluates the
// group at element index i, use(i, value) consumes it; all loads of a tile are
// issued before the first use.  A tile that lies wholly inside [0, n4) takes a
// path without per-lane conditions: behind a bounds check the compiler waits for
// every read before it issues the next, which leaves a wave with one read in
// flight.  Only the last tile is guarded.
template <class A, class B> struct Two { A first; B second; };

template <class L, class U>
__device__ __forceinline__ void for_each_group(unsigned n4, L &&load, U &&use) {
  for (unsigned base = blockIdx.x * kTile; base < n4; base += gridDim.x * kTile) {
    const unsigned i0 = base + threadIdx.x * kVec;
    decltype(load(0u)) v[kUnroll];
    if (base + kTile <= n4) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) v[u] = load(i0 + u * (kBlock * kVec));
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) use(i0 + u * (kBlock * kVec), v[u]);
    } else {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) if (i0 + u * (kBlock * kVec) < n4) v[u] = load(i0 + u * (kBlock * kVec));
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) if (i0 + u * (kBlock * kVec) < n4) use(i0 + u * (kBlock * kVec), v[u]);
    }
  }
}

// The same for element programs that read an array forwards and through
// `reverse` (two traversal orders of one array in one loop, section 3.3
// `simple5`).  Position i reads a[i] and a[n-1-i]; position n-1-i reads the same
// two.  A lane therefore takes the 128-bit group at i together with its mirror
// image at n4-4-i: the two groups issue the same two 128-bit reads, the second
// pair hits in the vector cache, and the array comes from HBM once instead of
// twice.  Every group of [0, n4) is used once.  Short arrays stay in the caches
// whatever the order and are better spread over twice as many workgroups
// (measured at 2^16 elements: 8.3 us plain, 9.8 us mirrored), so the kernels take
// this path from kMirrorMin elements on.
constexpr unsigned kMirrorMin = 1u << 20;
template <class L, class U>
__device__ __forceinline__ void for_each_mirrored_group(unsigned n4, L &&load, U &&use) {
  const unsigned half = ((n4 / 4 + 1) / 2) * 4;     // the first half, the middle group included
  // Every tile takes the guarded form here, on purpose: the second read of a line has
  // to reach the vector cache while the first is still on its way, and that works best
  // with few reads in flight per lane.  Measured on the reversed dot product at 2^26
  // elements: 51 us in this form (the compiler waits after each group and its mirror
  // image), 55 us with the sixteen reads of a tile issued back to back, 61 us with the
  // mirror images read after the groups have been used.
  for (unsigned base = blockIdx.x * kTile; base < half; base += gridDim.x * kTile) {
    decltype(load(0u)) v[kUnroll][2];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < half) {
        v[u][0] = load(i);
        v[u][1] = load(n4 - 4 - i);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const unsigned i = base + u * (kBlock * kVec) + threadIdx.x * kVec;
      if (i < half) {
        use(i, v[u][0]);
        if (n4 - 4 - i != i) use(n4 - 4 - i, v[u][1]);
      }
    }
  }
}

// The same pairing when every `reverse` of the element program runs over exactly the n4 elements
// of the iteration space (E::mirrors_whole): the groups at i and at n4-4-i are evaluated together
// (eval4_pair), every array read of the pair is issued once, so the streams can be read
// non-temporally like any other and a full tile has all its reads in flight.  Measured on the
// reversed dot product at 2^26 elements: 52 us with for_each_mirrored_group, 43 us this way; a
// read-only pass over as many bytes takes 39 us.
template <class L, class U>
__device__ __forceinline__ void for_each_mirrored_pair(unsigned n4, L &&load_pair, U &&use) {
  const unsigned half = ((n4 / 4 + 1) / 2) * 4;     // the first half, the middle group included
  for (unsigned base = blockIdx.x * kTile; base < half; base += gridDim.x * kTile) {
    decltype(load_pair(0u, 0u)) v[kUnroll];
    const unsigned i0 = base + threadIdx.x * kVec;
    if (base + kTile <= half) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) v[u] = load_pair(i0 + u * (kBlock * kVec), n4 - 4 - (i0 + u * (kBlock * kVec)));
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const unsigned i = i0 + u * (kBlock * kVec), ip = n4 - 4 - i;
        use(i, v[u].first);
        if (ip != i) use(ip, v[u].second);
      }
    } else {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const unsigned i = i0 + u * (kBlock * kVec);
        if (i < half) v[u] = load_pair(i, n4 - 4 - i);
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const unsigned i = i0 + u * (kBlock * kVec), ip = n4 - 4 - i;
        if (i < half) {
          use(i, v[u].first);
          if (ip != i) use(ip, v[u].second);
        }
      }
    }
  }
}
// the two groups of a pair, evaluated together
template <class E>
__device__ __forceinline__ Two<Vec4<typename E::R>, Vec4<typename E::R>> eval_pair(const KArgs &a, unsigned i, unsigned ip) {
  Two<Vec4<typename E::R>, Vec4<typename E::R>> r;
  E::template eval4_pair<0>(a, (int)i, (int)ip, r.first, r.second);
  return r;
}

// ------------------------------------------------------------------ elementwise: out[i] = E(i)
template <class E>
__global__ __launch_bounds__(kBlock) void store_kernel(const KArgs a) {
  using T = typename E::R;
  T *out = static_cast<T *>(a.out[0]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  with_keep(a.keeps(0), [&](auto keep) {
    auto use = [&](unsigned i, const Vec4<T> &v) { store4<decltype(keep)::value>(out + i, v); };
    if constexpr (E::kMirror) {
      if (n4 >= kMirrorMin && n == n4 && E::template mirrors_whole<0>(a, (int)n))
        for_each_mirrored_pair(n4, [&](unsigned i, unsigned ip) { return eval_pair<E>(a, i, ip); }, use);
      else if (n4 >= kMirrorMin)
        for_each_mirrored_group(n4, [&](unsigned i) { return KeepLoads<E>::type::template eval4<0>(a, (int)i); }, use);
      else
        for_each_group(n4, [&](unsigned i) { return E::template eval4<0>(a, (int)i); }, use);
    } else {
      for_each_group(n4, [&](unsigned i) { return E::template eval4<0>(a, (int)i); }, use);
    }
  });
  if (blockIdx.x == 0 && threadIdx.x < n - n4) out[n4 + threadIdx.x] = E::template eval<0>(a, (int)(n4 + threadIdx.x));
}

// two arrays written in one pass (diagonal fusion: a value is forwarded to the next
// combinator in registers and stored as well; section 1, Fig. "Three types of fusion")
template <class E1, class E2>
__global__ __launch_bounds__(kBlock) void store2_kernel(const KArgs a) {
  using T1 = typename E1::R;
  using T2 = typename E2::R;
  using K1 = typename KeepLoads<E1>::type;
  using K2 = typename KeepLoads<E2>::type;
  using Both = Two<Vec4<T1>, Vec4<T2>>;
  T1 *out1 = static_cast<T1 *>(a.out[0]);
  T2 *out2 = static_cast<T2 *>(a.out[1]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  // one choice for both arrays: ordinary stores as soon as one of them is read back
  with_keep(a.keeps(0) || a.keeps(1), [&](auto keep) {
    auto use = [&](unsigned i, const Both &v) {
      store4<decltype(keep)::value>(out1 + i, v.first);
      store4<decltype(keep)::value>(out2 + i, v.second);
    };
    if ((E1::kMirror || E2::kMirror) && n4 >= kMirrorMin)
      for_each_mirrored_group(
          n4, [&](unsigned i) { return Both{K1::template eval4<0>(a, (int)i), K2::template eval4<E1::kNodes>(a, (int)i)}; }, use);
    else
      for_each_group(
          n4, [&](unsigned i) { return Both{E1::template eval4<0>(a, (int)i), E2::template eval4<E1::kNodes>(a, (int)i)}; }, use);
  });
  if (blockIdx.x == 0 && threadIdx.x < n - n4) {
    int i = (int)(n4 + threadIdx.x);
    out1[i] = E1::template eval<0>(a, i);
    out2[i] = E2::template eval<E1::kNodes>(a, i);
  }
}

// ------------------------------------------------------------------ fold (and store + fold)
// Per-lane accumulation in a fixed order, DPP wave reduction, LDS workgroup
// reduction, one partial per workgroup; the workgroup that finishes last
// combines the partials in index order, so the result does not depend on
// scheduling.  fold is one stage of a multi-stage parallel reduction (section 2, fold).
// `earlier` partials, at the front of `partials`, were left there under the same tag
// by a kernel that ran before this one on the stream; they are combined first.
template <class Op, int Waves = kWavesPerBlock>
__device__ __forceinline__ void fold_finish(typename Op::T acc, const KArgs &a, int out_slot, Control *ctl,
                                            unsigned long long *partials, unsigned earlier = 0) {
  using T = typename Op::T;
  __shared__ T lds[Waves + 1];
  const unsigned epoch = load_agent(&ctl->epoch);
  const unsigned tag = tag_of_epoch(epoch);
  T r = block_reduce<Op, Waves>(acc, lds);
  if (threadIdx.x == 0) store_agent64(&partials[earlier + blockIdx.x], pack_word((unsigned)as_bits(r), tag, 1u));
  // the workgroup with the highest index is dispatched last; it waits for the
  // partials of all others and combines them in index order
  if (blockIdx.x == gridDim.x - 1) {
    T s = Op::identity();
    for (unsigned k = threadIdx.x; k < earlier + gridDim.x; k += Waves * kWave) {
      unsigned long long w = wait_word(&partials[k], tag, ctl);
      s = Op::apply(s, w ? from_bits<T>((int)(unsigned)(w >> 32)) : Op::identity());
    }
    s = block_reduce<Op, Waves>(s, lds);
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
  auto use = [&](unsigned, const Vec4<T> &v) {
#pragma unroll
    for (int c = 0; c < 4; ++c) acc = Op::apply(acc, v.v[c]);
  };
  if constexpr (E::kMirror) {
    if (n4 >= kMirrorMin && n == n4 && E::template mirrors_whole<0>(a, (int)n))
      for_each_mirrored_pair(n4, [&](unsigned i, unsigned ip) { return eval_pair<E>(a, i, ip); }, use);
    else if (n4 >= kMirrorMin)
      for_each_mirrored_group(n4, [&](unsigned i) { return KeepLoads<E>::type::template eval4<0>(a, (int)i); }, use);
    else
      for_each_group(n4, [&](unsigned i) { return E::template eval4<0>(a, (int)i); }, use);
  } else {
    for_each_group(n4, [&](unsigned i) { return E::template eval4<0>(a, (int)i); }, use);
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) acc = Op::apply(acc, E::template eval<0>(a, (int)(n4 + threadIdx.x)));
  fold_finish<Op>(acc, a, 0, ctl, partials);
}

// out[0][i] = ES(i) and out[1] = fold(Op, EF(i)) in one pass
template <class ES, class Op, class EF>
__global__ __launch_bounds__(kBlock) void store_fold_kernel(const KArgs a, Control *ctl, unsigned long long *partials) {
  using T = typename Op::T;
  using S = typename ES::R;
  using KS = typename KeepLoads<ES>::type;
  using KF = typename KeepLoads<EF>::type;
  using Both = Two<Vec4<S>, Vec4<T>>;
  S *out = static_cast<S *>(a.out[0]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  T acc = Op::identity();
  with_keep(a.keeps(0), [&](auto keep) {
    auto use = [&](unsigned i, const Both &v) {
      store4<decltype(keep)::value>(out + i, v.first);
#pragma unroll
      for (int c = 0; c < 4; ++c) acc = Op::apply(acc, v.second.v[c]);
    };
    if ((ES::kMirror || EF::kMirror) && n4 >= kMirrorMin)
      for_each_mirrored_group(
          n4, [&](unsigned i) { return Both{KS::template eval4<0>(a, (int)i), KF::template eval4<ES::kNodes>(a, (int)i)}; }, use);
    else
      for_each_group(
          n4, [&](unsigned i) { return Both{ES::template eval4<0>(a, (int)i), EF::template eval4<ES::kNodes>(a, (int)i)}; }, use);
  });
  if (blockIdx.x == 0 && threadIdx.x < n - n4) {
    int i = (int)(n4 + threadIdx.x);
    out[i] = ES::template eval<0>(a, i);
    acc = Op::apply(acc, EF::template eval<ES::kNodes>(a, i));
  }
  fold_finish<Op>(acc, a, 1, ctl, partials);
}

// ------------------------------------------------------------------ interpreted elementwise clusters
// Any cluster of maps, generates and gathers that ends in up to kMaxOut stored arrays
// or in stored arrays and up to two folds, for which no kernel was compiled: the element
// programs are run from KArgs::code, four elements per lane at a time.  The top of the
// value stack stays in registers, what lies below in LDS (a column per lane: registers
// cannot be indexed by a run-time number); the positions that gathers suspend are at most
// kInterpGathers deep and stay in registers.  Every branch depends on the code only, which
// is the same for all lanes.  Results are the same as a compiled instance's: the same
// element functions, applied in the same order.  A fallback: several times the
// instructions of a compiled instance per element, 4-byte accesses.
// x[k][e]: argument k of element e; the function is picked once for the V elements
template <int V>
__device__ __forceinline__ void interp_map(int fn, const Slot &s, const unsigned (&x)[5][V], unsigned (&r)[V]) {
  auto f = [&](int k, int e) { return from_bits<float>((int)x[k][e]); };
  auto bits = [](float v) { return (unsigned)as_bits(v); };
#define FC_EACH(expr) _Pragma("unroll") for (int e = 0; e < V; ++e) r[e] = (expr); break
  switch (fn) {
    case FC_FN_IDENT: FC_EACH(x[0][e]);
    case FC_FN_AFFINE: FC_EACH(bits(FnAffine::apply(s, f(0, e))));
    case FC_FN_SIN_X_MUL_X: FC_EACH(bits(FnSinXMulX::apply(s, f(0, e))));
    case FC_FN_SQ_PLUS_ONE: FC_EACH(bits(FnSqPlusOne::apply(s, f(0, e))));
    case FC_FN_MUL2: FC_EACH(bits(FnMul2::apply(s, f(0, e), f(1, e))));
    case FC_FN_ADD2: FC_EACH(bits(FnAdd2::apply(s, f(0, e), f(1, e))));
    case FC_FN_ADD3: FC_EACH(bits(FnAdd3::apply(s, f(0, e), f(1, e), f(2, e))));
    case FC_FN_ADD5: FC_EACH(bits(FnAdd5::apply(s, f(0, e), f(1, e), f(2, e), f(3, e), f(4, e))));
    case FC_FN_EXP_NEG: FC_EACH(bits(FnExpNeg::apply(s, f(0, e))));
    case FC_FN_MOD_EQ: FC_EACH((unsigned)FnModEq::apply(s, (int)x[0][e]));
    default: FC_EACH(0u);
  }
}
template <int V>
__device__ __forceinline__ void interp_gen(int fn, const Slot &s, const KArgs &a, const int (&at)[V], unsigned (&r)[V]) {
  switch (fn) {
    case FC_FN_IOTA: FC_EACH((unsigned)GenIota::apply(s, a, at[e]));
    case FC_FN_IOTA_REV: FC_EACH((unsigned)GenIotaRev::apply(s, a, at[e]));
    case FC_FN_CLAMP_SHIFT_2D: FC_EACH((unsigned)GenClampShift2D::apply(s, a, at[e]));
    case FC_FN_ROW_OF_2D: FC_EACH((unsigned)GenRowOf2D::apply(s, a, at[e]));
    case FC_FN_CONST_I32: FC_EACH((unsigned)GenConst::apply(s, a, at[e]));
    default: FC_EACH(0u);
  }
}
#undef FC_EACH
__device__ __forceinline__ unsigned interp_fold(int op, unsigned acc, unsigned v) {
  switch (op) {
    case kFoldAddF32: return (unsigned)as_bits(AddF32::apply(from_bits<float>((int)acc), from_bits<float>((int)v)));
    case kFoldMaxF32: return (unsigned)as_bits(MaxF32::apply(from_bits<float>((int)acc), from_bits<float>((int)v)));
    case kFoldMulF32: return (unsigned)as_bits(MulF32::apply(from_bits<float>((int)acc), from_bits<float>((int)v)));
    case kFoldAddI32: return (unsigned)AddI32::apply((int)acc, (int)v);
    default: return (unsigned)MaxI32::apply((int)acc, (int)v);
  }
}
__device__ __forceinline__ unsigned interp_identity(int op) {
  switch (op) {
    case kFoldAddF32: return (unsigned)as_bits(AddF32::identity());
    case kFoldMaxF32: return (unsigned)as_bits(MaxF32::identity());
    case kFoldMulF32: return (unsigned)as_bits(MulF32::identity());
    case kFoldAddI32: return (unsigned)AddI32::identity();
    default: return (unsigned)MaxI32::identity();
  }
}

// Runs the cluster's code for the V consecutive elements that start at `first` (V = 4: a
// 128-bit group, `first` a multiple of four; V = 1: one element), so that the cost of
// reading and decoding an instruction is shared by four elements.  `below` is this
// lane's column of the value stack.
// Starts at instruction `pc`; a kCodeYield ends the run with the program's values in `result`.
template <int V, int Threads>
__device__ __forceinline__ void interp_run(const KArgs &a, int pc, unsigned first, unsigned (*below)[kVec][Threads],
                                           unsigned (&acc)[kInterpFolds], unsigned (&result)[V]) {
  using Raw = unsigned __attribute__((ext_vector_type(4)));
  int at[V];                                           // the positions element programs read at
  int suspended[kInterpGathers][V];
  unsigned top[V];
#pragma unroll
  for (int e = 0; e < V; ++e) { at[e] = (int)first + e; top[e] = 0u; }
  int gathers = 0, count = 0;                          // the same in every lane
  auto push_room = [&]() {
    if (count > 0) {
#pragma unroll
      for (int e = 0; e < V; ++e) below[count - 1][e][threadIdx.x] = top[e];
    }
    ++count;
  };
  auto pop = [&]() {
    --count;
    if (count > 0) {
#pragma unroll
      for (int e = 0; e < V; ++e) top[e] = below[count - 1][e][threadIdx.x];
    }
  };
  for (; pc < kMaxCode; ++pc) {
    const Code c = a.code[pc];
    if (c.op == kCodeEnd) break;
    if (c.op == kCodeYield) {
#pragma unroll
      for (int e = 0; e < V; ++e) result[e] = top[e];
      break;
    }
    switch (c.op) {
      case kCodeIn: {
        push_room();
        const unsigned *p = static_cast<const unsigned *>(a.in[c.a]);
        if (V == 4 && gathers == 0) {                  // the elements' own positions: one 128-bit read
          const Raw v = *reinterpret_cast<const Raw *>(p + first);
          top[0] = v.x; if (V > 1) { top[1 % V] = v.y; top[2 % V] = v.z; top[3 % V] = v.w; }
        } else {
#pragma unroll
          for (int e = 0; e < V; ++e) top[e] = p[at[e]];
        }
        break;
      }
      case kCodeGen:
        push_room();
        interp_gen<V>(c.a, a.p[c.b], a, at, top);
        break;
      case kCodeMap: {
        const int nargs = c.c;
        // the last argument is the top of the stack, the others lie below it in order
        unsigned x[5][V];
#pragma unroll
        for (int k = 0; k < 5; ++k)
#pragma unroll
          for (int e = 0; e < V; ++e)
            x[k][e] = k >= nargs ? 0u : k == nargs - 1 ? top[e] : below[count - nargs + k][e][threadIdx.x];
        count -= nargs - 1;
        interp_map<V>(c.a, a.p[c.b], x, top);
        break;
      }
      case kCodeEnter: {
#pragma unroll
        for (int e = 0; e < V; ++e) {
          if (gathers == 0) suspended[0][e] = at[e]; else if (gathers == 1) suspended[1][e] = at[e]; else suspended[2][e] = at[e];
          at[e] = (int)top[e];
        }
        ++gathers;
        pop();
        break;
      }
      case kCodeLeave:
        --gathers;
#pragma unroll
        for (int e = 0; e < V; ++e) at[e] = gathers == 0 ? suspended[0][e] : gathers == 1 ? suspended[1][e] : suspended[2][e];
        break;
      case kCodeStore: {
        unsigned *p = static_cast<unsigned *>(a.out[c.a]) + first;
        if (V == 4) {
          *reinterpret_cast<Raw *>(p) = Raw{top[0], top[1 % V], top[2 % V], top[3 % V]};
        } else {
          p[0] = top[0];
        }
        pop();
        break;
      }
      case kCodeDup: push_room(); break;               // the top goes below and stays the top
      default: {                                        // kCodeFold
        unsigned v = c.c == 0 ? acc[0] : acc[1];
#pragma unroll
        for (int e = 0; e < V; ++e) v = interp_fold(c.b, v, top[e]);
        if (c.c == 0) acc[0] = v; else acc[1] = v;
        pop();
        break;
      }
    }
  }
}

// Workgroup reduction with the reducer picked at run time (the same for the whole grid).
__device__ __forceinline__ unsigned interp_block_reduce(int op, unsigned v, unsigned *lds) {
  switch (op) {
    case kFoldAddF32: return (unsigned)as_bits(block_reduce<AddF32>(from_bits<float>((int)v), reinterpret_cast<float *>(lds)));
    case kFoldMaxF32: return (unsigned)as_bits(block_reduce<MaxF32>(from_bits<float>((int)v), reinterpret_cast<float *>(lds)));
    case kFoldMulF32: return (unsigned)as_bits(block_reduce<MulF32>(from_bits<float>((int)v), reinterpret_cast<float *>(lds)));
    case kFoldAddI32: return (unsigned)block_reduce<AddI32>((int)v, reinterpret_cast<int *>(lds));
    default: return (unsigned)block_reduce<MaxI32>((int)v, reinterpret_cast<int *>(lds));
  }
}

template <class Tag = void>            // a template only so that every translation unit may see the definition
__global__ __launch_bounds__(kBlock) void interp_kernel(const KArgs a, Control *ctl, unsigned long long *partials) {
  __shared__ unsigned below[kInterpDepth][kVec][kBlock];
  __shared__ unsigned lds[kWavesPerBlock + 1];
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  // the folds of the cluster (at most kInterpFolds), each with an accumulator of its own
  int n_folds = 0, fold_op[kInterpFolds] = {0, 0}, fold_out[kInterpFolds] = {0, 0};
  for (int pc = 0; pc < kMaxCode && a.code[pc].op != kCodeEnd; ++pc)
    if (a.code[pc].op == kCodeFold) {
      const int k = a.code[pc].c == 0 ? 0 : 1;
      if (k == 0) { fold_op[0] = a.code[pc].b; fold_out[0] = a.code[pc].a; } else { fold_op[1] = a.code[pc].b; fold_out[1] = a.code[pc].a; }
      n_folds = n_folds > k + 1 ? n_folds : k + 1;
    }
  unsigned acc[kInterpFolds] = {interp_identity(fold_op[0]), interp_identity(fold_op[1])};
  unsigned none4[kVec], none1[1];
  for (unsigned i = (blockIdx.x * kBlock + threadIdx.x) * kVec; i < n4; i += gridDim.x * kBlock * kVec)
    interp_run<kVec, kBlock>(a, 0, i, below, acc, none4);
  if (blockIdx.x == 0 && threadIdx.x < n - n4) interp_run<1, kBlock>(a, 0, n4 + threadIdx.x, below, acc, none1);
  if (n_folds == 0) return;                              // the same for the whole grid
  // as fold_finish, for up to two accumulators under one tag: fold k keeps its partials at
  // [k * gridDim.x, (k + 1) * gridDim.x); the last workgroup combines them and takes the next tag
  const unsigned epoch = load_agent(&ctl->epoch);
  const unsigned tag = tag_of_epoch(epoch);
  for (int k = 0; k < n_folds; ++k) {
    const unsigned r = interp_block_reduce(k == 0 ? fold_op[0] : fold_op[1], k == 0 ? acc[0] : acc[1], lds);
    if (threadIdx.x == 0) store_agent64(&partials[(size_t)k * gridDim.x + blockIdx.x], pack_word(r, tag, 1u));
  }
  if (blockIdx.x != gridDim.x - 1) return;
  for (int k = 0; k < n_folds; ++k) {
    const int op = k == 0 ? fold_op[0] : fold_op[1];
    unsigned s = interp_identity(op);
    for (unsigned j = threadIdx.x; j < gridDim.x; j += kBlock) {
      const unsigned long long w = wait_word(&partials[(size_t)k * gridDim.x + j], tag, ctl);
      s = interp_fold(op, s, w ? (unsigned)(w >> 32) : interp_identity(op));
    }
    s = interp_block_reduce(op, s, lds);
    if (threadIdx.x == 0) static_cast<unsigned *>(a.out[k == 0 ? fold_out[0] : fold_out[1]])[0] = s;
  }
  if (threadIdx.x == 0) store_agent(&ctl->epoch, epoch + 1u);
}

// Element program K of a cluster as an expression node: evaluated by running its code
// (KArgs::code from KArgs::root[K] to the kCodeYield).  With it every skeleton of this
// file has an instance that takes any element program: what the matcher cannot pair with a
// compiled element program runs through these.  Threads = threads of the workgroup (the
// lanes' stack columns live in LDS).
template <int Threads>
__device__ __forceinline__ unsigned (*interp_stack())[kVec][Threads] {
  __shared__ unsigned below[kInterpDepth][kVec][Threads];
  return below;
}
template <int K, class T, int Threads = kBlock>
struct Interp {
  using R = T;
  static constexpr int kNodes = 0;                     // the code names its parameter slots itself
  static constexpr bool kMirror = false;
  template <int Base, bool Stream = false> static __device__ __forceinline__ T eval(const KArgs &a, int i) {
    unsigned r[1] = {0u}, none[kInterpFolds] = {0u, 0u};
    interp_run<1, Threads>(a, a.root[K], (unsigned)i, interp_stack<Threads>(), none, r);
    return from_bits<T>((int)r[0]);
  }
  // i is a multiple of four (the callers read 128-bit groups)
  template <int Base> static __device__ __forceinline__ Vec4<T> eval4(const KArgs &a, int i) {
    unsigned r[kVec] = {0u, 0u, 0u, 0u}, none[kInterpFolds] = {0u, 0u};
    interp_run<kVec, Threads>(a, a.root[K], (unsigned)i, interp_stack<Threads>(), none, r);
    return Vec4<T>{{from_bits<T>((int)r[0]), from_bits<T>((int)r[1]), from_bits<T>((int)r[2]), from_bits<T>((int)r[3])}};
  }
  static void sig(std::string &s) { s += std::string("*") + DtypeName<T>::s(); }
};

// ------------------------------------------------------------------ fold over a gathered table, indices binned first
// r = fold(Op, f(table[index[i]])) for a table of more than one L2 (4 MiB per XCD) and
// indices in no particular order.  Read directly, nearly every gather misses L2 and costs
// a 128-byte line from the memory side, whose rate (about 52 G lines/s on this chip) then
// bounds the kernel; gathers that hit L2 run four times faster.  A fold with a commutative
// operator may visit the positions in any order (the order of evaluation inside a fold is
// not part of its meaning: section 2, fold), and this element program depends on a
// position only through the index found there.  So the launch takes two kernels:
//
//  1. bin_indices_kernel cuts the table into kBins ranges and sorts every tile of
//     kBinTile indices by range.  The entries of (range, tile) go to a slot of kBinCap
//     words at a fixed place, their number to counts[range][tile]: no workgroup waits
//     for another.  Uniformly spread indices put kBinTile / kBins = 256 entries into a
//     slot, give or take 16; the few that a slot cannot take are evaluated on the spot.
//  2. fold_binned_kernel: every XCD takes the ranges r with r % 8 equal to its number,
//     one after the other, and reads all slots of the range.  Its gathers go to one
//     range, half an L2 or less for tables up to 64 MiB (the ranges of two rounds fit
//     side by side while the workgroups of an XCD are not all in the same round), and
//     hit; the slots are read past L2 (agent scope, read once), so that they do not
//     displace the table.
//
// The indices are read once and written and read once more as entries: three times their
// bytes instead of a line of 128 bytes for each.
constexpr int kBins = 32;
constexpr int kBinItems = 16;                          // indices per thread and pass
constexpr int kBinPasses = 2;                          // passes of kBlock * kBinItems indices that fill one tile's slots
constexpr int kBinPass = kBlock * kBinItems;
constexpr int kBinTile = kBinPass * kBinPasses;
constexpr int kBinGroups = 5;                          // a slot holds this many entries per lane of the wave that reads it
constexpr int kBinCap = kBinGroups * kWave;            // 320 = 256 + 4 standard deviations of a uniform spread
constexpr unsigned kBinAtOnce = 2;                     // slots a wave of the second kernel works on at a time
static_assert(kBins <= kWave, "one thread of the first wave per range");

// range of table position `j`: j / range_len, as a multiplication (the host passes
// ceil(2^32 / range_len)); a quotient that comes out one too high at a boundary only
// moves the boundary, the same for every position.  Positions outside the table land
// in the last range.
__device__ __forceinline__ unsigned bin_of(int j, unsigned inv_range) {
  const unsigned b = __umulhi((unsigned)j, inv_range);
  return b < kBins ? b : kBins - 1;
}

template <class Op, class E>
__global__ __launch_bounds__(kBlock) void bin_indices_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                             int *counts, int *entries, unsigned tiles, unsigned inv_range) {
  using T = typename Op::T;
  using C = GatherChain<E>;
  using Index = In<C::kIndex, int>;
  __shared__ unsigned wave_count[kWavesPerBlock][kBins];
  __shared__ unsigned wave_first[kWavesPerBlock][kBins];   // start of a wave's elements of a range in `staged`
  __shared__ unsigned range_first[kBins];                   // start of a range in `staged`
  __shared__ unsigned range_count[kBins];                   // elements of a range in this pass
  __shared__ unsigned slot_filled[kBins];                   // entries of the tile's slot before this pass
  __shared__ unsigned any_crowded;
  __shared__ int staged[kBinPass];                          // the indices of a pass, sorted by range
  __shared__ T lds[kWavesPerBlock + 1];
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  const unsigned wave = (unsigned)wave_id(), lane = (unsigned)lane_id();
  constexpr unsigned kNone = 0xffu;                    // range of a position past the end
  T acc = Op::identity();
  for (unsigned tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    unsigned filled = 0;                               // thread b < kBins: entries in slot (b, tile) so far
    for (unsigned pass = 0; pass < (unsigned)kBinPasses; ++pass) {
      const unsigned first = tile * kBinTile + pass * kBinPass;
      const unsigned base = first + threadIdx.x * kVec;
      int index[kBinItems];
      unsigned place[kBinItems];                       // range << 16 | rank among the wave's elements of that range
      if (first + kBinPass <= n4) {
#pragma unroll
        for (int u = 0; u < kBinItems / kVec; ++u) {
          Vec4<int> v = Index::template eval4<0>(a, (int)(base + u * (kBlock * kVec)));
#pragma unroll
          for (int c = 0; c < kVec; ++c) { index[u * kVec + c] = v.v[c]; place[u * kVec + c] = bin_of(v.v[c], inv_range) << 16; }
        }
      } else {
#pragma unroll
        for (int u = 0; u < kBinItems / kVec; ++u) {
          const unsigned i = base + u * (kBlock * kVec);
          Vec4<int> v = {{0, 0, 0, 0}};
          if (i < n4) v = Index::template eval4<0>(a, (int)i);
#pragma unroll
          for (int c = 0; c < kVec; ++c) {
            index[u * kVec + c] = v.v[c];
            place[u * kVec + c] = (i < n4 ? bin_of(v.v[c], inv_range) : kNone) << 16;
          }
        }
      }
      // rank of every element among the wave's elements of its range in this pass: a
      // counter per wave and range in LDS, one add per element (the waves do not share
      // counters, and LDS operations of one wave take effect in program order)
      if (lane < (unsigned)kBins) wave_count[wave][lane] = 0;
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int s = 0; s < kBinItems; ++s) {
        if ((place[s] >> 16) != kNone)
          place[s] |= __hip_atomic_fetch_add(&wave_count[wave][place[s] >> 16], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
      }
      __syncthreads();
      // the first wave lays the pass out: ranges one after the other, inside a range the waves in order
      if (wave == 0) {
        unsigned total = 0;
        if (lane < (unsigned)kBins) {
#pragma unroll
          for (int w = 0; w < kWavesPerBlock; ++w) total += wave_count[w][lane];
        }
        const unsigned start = (unsigned)wave_scan_inclusive<AddI32>((int)total) - total;
        if (lane < (unsigned)kBins) {
          unsigned run = start;
#pragma unroll
          for (int w = 0; w < kWavesPerBlock; ++w) { wave_first[w][lane] = run; run += wave_count[w][lane]; }
          range_first[lane] = start;
          range_count[lane] = total;
          slot_filled[lane] = filled;
          filled += total;
        }
        const unsigned long long over = __builtin_amdgcn_ballot_w64(lane < (unsigned)kBins && filled > (unsigned)kBinCap);
        if (lane == 0) any_crowded = over != 0 ? 1u : 0u;
      }
      __syncthreads();
      const bool crowded = any_crowded != 0;           // some slot of this tile is full: the same for the whole workgroup
#pragma unroll
      for (int s = 0; s < kBinItems; ++s)
        if ((place[s] >> 16) != kNone) staged[wave_first[wave][place[s] >> 16] + (place[s] & 0xffffu)] = index[s];
      __syncthreads();
      // every wave copies a quarter of the ranges to their slots, consecutive lanes to consecutive words
      for (unsigned b = wave; b < (unsigned)kBins; b += kWavesPerBlock) {
        const unsigned from = range_first[b], to = slot_filled[b];
        const unsigned room = to < (unsigned)kBinCap ? (unsigned)kBinCap - to : 0u;
        const unsigned count = range_count[b] < room ? range_count[b] : room;
        int *slot = entries + ((size_t)b * tiles + tile) * kBinCap + to;
        for (unsigned j = lane; j < count; j += kWave) slot[j] = staged[from + j];
      }
      // what the slots cannot take (indices that crowd into few ranges) is evaluated here, by the
      // whole workgroup and two gathers per lane at a time
      constexpr int kOver = 2;
      for (unsigned b = 0; crowded && b < (unsigned)kBins; ++b) {
        const unsigned from = range_first[b], to = slot_filled[b], count = range_count[b];
        const unsigned room = to < (unsigned)kBinCap ? (unsigned)kBinCap - to : 0u;
        for (unsigned j0 = room; j0 < count; j0 += kBlock * kOver) {     // the same for the whole workgroup
          typename C::Leaf x[kOver];
#pragma unroll
          for (int c = 0; c < kOver; ++c) {
            const unsigned j = j0 + c * kBlock + threadIdx.x;
            x[c] = typename C::Leaf();
            if (j < count) x[c] = C::leaf(a, staged[from + j]);
          }
#pragma unroll
          for (int c = 0; c < kOver; ++c) {
            const T v = C::template from_leaf<0>(a, x[c]);
            if (j0 + c * kBlock + threadIdx.x < count) acc = Op::apply(acc, v);
          }
        }
      }
    }
    if (threadIdx.x < kBins) counts[(size_t)threadIdx.x * tiles + tile] = (int)(filled < (unsigned)kBinCap ? filled : (unsigned)kBinCap);
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) acc = Op::apply(acc, E::template eval<0>(a, (int)(n4 + threadIdx.x)));
  // one partial per workgroup; the second kernel combines them with its own
  const unsigned tag = tag_of_epoch(load_agent(&ctl->epoch));
  T r = block_reduce<Op>(acc, lds);
  if (threadIdx.x == 0) store_agent64(&partials[blockIdx.x], pack_word((unsigned)as_bits(r), tag, 1u));
}

template <class Op, class E>
__global__ __launch_bounds__(kBlock) void fold_binned_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                             const int *counts, const int *entries, unsigned tiles,
                                                             unsigned earlier) {
  using T = typename Op::T;
  using C = GatherChain<E>;
  using Leaf = typename C::Leaf;
  constexpr unsigned kXcds = 8;                        // workgroup b runs on XCD b % 8
  constexpr int kPastL2 = 0x12;                        // cache policy of the buffer loads: sc1 | nt
  const unsigned xcd = blockIdx.x % kXcds, team = blockIdx.x / kXcds, teams = gridDim.x / kXcds;
  const unsigned wave = (unsigned)wave_id(), lane = (unsigned)lane_id();
  // raw buffer views: byte offsets, and an offset past the end reads as zero without a memory access
  const unsigned slots = kBins * tiles;
  const __amdgpu_buffer_rsrc_t count_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<int *>(counts), 0, (int)(slots * 4u), 0x00020000);
  const __amdgpu_buffer_rsrc_t entry_buf =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int *>(entries), 0, (int)(slots * (unsigned)kBinCap * 4u), 0x00020000);
  // A wave takes kBinAtOnce slots per step.  Step q of a workgroup: range xcd + 8 * (q / per), tiles
  // 4 * kBinAtOnce * item and following with item = team + teams * (q % per); the ranges follow each
  // other without a gap in the reads.
  constexpr unsigned kPerItem = kWavesPerBlock * kBinAtOnce;
  const unsigned items = (tiles + kPerItem - 1) / kPerItem;
  const unsigned per = (items + teams - 1) / teams;
  const unsigned steps = per * (kBins / kXcds);
  constexpr unsigned kNoSlot = 0xffffffffu;
  auto slot_of = [&](unsigned q, unsigned sub) {
    const unsigned item = team + teams * (q % per), t = (item * kBinAtOnce + sub) * kWavesPerBlock + wave;
    return q < steps && item < items && t < tiles ? (xcd + kXcds * (q / per)) * tiles + t : kNoSlot;
  };
  // Lane l takes entries 4l .. 4l+3 of a slot in one 128-bit read, and entry 256 + l if the slot
  // has that many (the cache asks L2 for 128 bytes at a time on behalf of 128-bit reads, for 64 on
  // behalf of 32-bit ones).
  static_assert(kBinGroups == kVec + 1, "a 128-bit read per lane and a last group");
  using Raw = int __attribute__((ext_vector_type(4)));
  struct Slot5 { int count; Raw e; int last; };
  struct Batch { Slot5 s[kBinAtOnce]; };
  // a slot that does not exist reads as empty: an offset past the end of the buffer yields zero
  auto fetch_counts = [&](unsigned q, Batch &b) {
#pragma unroll
    for (unsigned sub = 0; sub < kBinAtOnce; ++sub) {
      const unsigned slot = slot_of(q, sub);
      b.s[sub].count = __builtin_amdgcn_raw_buffer_load_b32(count_buf, slot != kNoSlot ? slot * 4u : kNoSlot, 0, 0);
    }
  };
  auto fetch_entries = [&](unsigned q, Batch &b) {
#pragma unroll
    for (unsigned sub = 0; sub < kBinAtOnce; ++sub) {
      Slot5 &s = b.s[sub];
      const unsigned count = (unsigned)__builtin_amdgcn_readfirstlane(s.count);
      const unsigned at = slot_of(q, sub) * (unsigned)kBinCap * 4u;
      // both reads are always issued, the second with an offset past the end (no memory access) when
      // the slot ends before it: reads that are issued only sometimes cannot be waited for one by one
      s.e = __builtin_amdgcn_raw_buffer_load_b128(entry_buf, count ? at + lane * 16u : kNoSlot, 0, kPastL2);
      s.last = __builtin_amdgcn_raw_buffer_load_b32(entry_buf, count > (unsigned)(kVec * kWave) ? at + (kVec * kWave + lane) * 4u : kNoSlot,
                                                    0, kPastL2);
    }
  };
  T acc = Op::identity();
  // Works on the slots in `use` (step q).  Once their gathers are on their way it starts the reads
  // of the entries of step q + 1 into `fill`, whose counts the step before asked for, and asks for
  // the counts of step q + 2.  The memory counter retires in order: a read issued before the
  // gathers would have to land before the first gathered value can be used.
  auto step = [&](Batch &use, Batch &fill, unsigned q) {
    // All reads so far were issued a step ago; with every one of them landed no gather below has
    // to wait for an entry, which (in-order counter again) would mean waiting for the gathers
    // issued before it.
    __builtin_amdgcn_s_waitcnt(0x0f70);                  // vmcnt(0), the other counters left alone
    Leaf x[kBinAtOnce][kBinGroups];
    bool mine[kBinAtOnce][kBinGroups];
#pragma unroll
    for (unsigned sub = 0; sub < kBinAtOnce; ++sub) {
      const unsigned count = (unsigned)__builtin_amdgcn_readfirstlane(use.s[sub].count);
#pragma unroll
      for (int k = 0; k < kVec; ++k) mine[sub][k] = lane * kVec + k < count;
      mine[sub][kVec] = kVec * kWave + lane < count;
#pragma unroll
      for (int k = 0; k < kBinGroups; ++k) {
        x[sub][k] = Leaf();
        if (mine[sub][k]) x[sub][k] = C::leaf(a, k < kVec ? use.s[sub].e[k] : use.s[sub].last);
      }
    }
    fetch_counts(q + 2, use);
    fetch_entries(q + 1, fill);
#pragma unroll
    for (unsigned sub = 0; sub < kBinAtOnce; ++sub)
#pragma unroll
      for (int k = 0; k < kBinGroups; ++k)
        if (__builtin_amdgcn_ballot_w64(mine[sub][k]) != 0) {   // the same for the whole wave
          const T v = C::template from_leaf<0>(a, x[sub][k]);
          if (mine[sub][k]) acc = Op::apply(acc, v);
        }
  };
  // two batches in turn, so that no register has to be copied while its read is in flight
  Batch even, odd;
  fetch_counts(0, even);
  fetch_counts(1, odd);
  fetch_entries(0, even);
  for (unsigned q = 0; q < steps; q += 2) {
    step(even, odd, q);
    step(odd, even, q + 1);
  }
  fold_finish<Op>(acc, a, 0, ctl, partials, earlier);
}

// The same fold for tables of up to 2^24 elements (64 MiB), with the ranges made so small that
// a range of the table fits the LDS of a compute unit: gathers from LDS cost a few cycles per
// wave, gathers that hit L2 are bound by the rate at which an L2 takes requests (12 per clock and
// XCD: 71 us for 2^24 gathers whatever else the kernel does).  Two kernels again, both with
// workgroups of kFineBlock = 1024 threads (one per compute unit: they fill its LDS):
//
//  1. bin_fine_kernel cuts the table into kFineBins ranges of equal length (FineCut: the range of
//     an index is a multiplication and a shift that the host has checked against the division,
//     because the offsets inside a range are kept as 16-bit numbers and have to be exact) and
//     sorts every tile of kFineTile indices by range.  A thread keeps its 32 indices in
//     registers; every element takes a rank from an LDS counter per (wave, range) -- one LDS
//     operation per element -- a scan over the ranges lays the tile out, every offset goes to its
//     place in LDS, and the waves copy the ranges to their slots, consecutive lanes to
//     consecutive words.  A slot is kFineCap 16-bit entries at a fixed place per (range, tile);
//     uniformly spread indices fill it with 64 +- 8, the places left over hold kFineNone, and
//     what does not fit is evaluated on the spot.
//  2. fold_fine_kernel: a workgroup takes a range at a time, applies the maps of the chain to the
//     range's table elements once and keeps the values in LDS (128 KiB), with the identity of the
//     fold behind them at kFineNone.  Then it streams the range's slots, which lie one behind the
//     other, and gathers from LDS without looking at counts.  The table of the next range and
//     the first entries are under way while a range is evaluated.
//
// Every order in here is fixed (lanes within a wave, waves, ranges, tiles), so a launch gives
// the same bits every time.
constexpr int kFineBlock = 1024;                       // threads per workgroup of both kernels
constexpr int kFineWaves = kFineBlock / kWave;
constexpr int kFineBins = 512;
constexpr int kFineTile = 32768;                       // indices per tile
constexpr int kFineVecs = kFineTile / (kFineBlock * kVec);   // 128-bit reads per thread and tile
constexpr int kFineCap = 96;                           // entries per slot: mean 64 + 4 standard deviations of a uniform spread
constexpr int kFineSlotWords = kFineCap / 2;           // two entries per 32-bit word
constexpr int kFineSlice = 32768;                      // elements of a range at most (offsets are below 2^15)
constexpr unsigned kFineNone = kFineSlice;             // the entry of a place that holds no index
constexpr unsigned kFineIndexLimit = 1u << 24;         // table elements at most: FineCut is exact below it
static_assert(kFineCap % 8 == 0 && kFineSlotWords <= kWave, "a slot is whole 128-bit groups and at most a word per lane");
static_assert(kFineBins <= kFineBlock && kFineVecs * kFineBlock * kVec == kFineTile, "a thread per range in the scan; whole reads");
static_assert(kFineBins % 32 == 0 && kFineNone < 65536u, "a bit per range in whole words; entries are 16-bit numbers");

// How the table is cut: `range` elements per range (a multiple of four), `bins` ranges, and
// j / range == __umulhi(j, magic) >> shift for every j below kFineIndexLimit.
struct FineCut { unsigned range, bins, magic, shift; };

template <class Op, class E>
__global__ __launch_bounds__(kFineBlock) void bin_fine_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                              unsigned *slots, unsigned tiles, const FineCut cut) {
  using T = typename Op::T;
  using C = GatherChain<E>;
  using Raw = int __attribute__((ext_vector_type(4)));
  using Chunk = unsigned __attribute__((ext_vector_type(4)));
  constexpr unsigned kChunks = kFineBins * kFineCap / 8;    // 128-bit groups of eight entries in the tile's slots
  __shared__ unsigned cursor[kFineWaves][kFineBins];        // per (wave, range): the count, then the wave's first place in the slot
  __shared__ Chunk image[kChunks];                          // the tile's slots as they go to memory: kFineCap entries per range
  __shared__ T lds[kFineWaves + 1];
  unsigned short *entries = reinterpret_cast<unsigned short *>(image);
  const int *index = static_cast<const int *>(a.in[C::kIndex]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  const unsigned wave = (unsigned)wave_id();
  // raw buffer view of the index array (at most 2^31 bytes): an offset past the end reads zero without a memory access
  const __amdgpu_buffer_rsrc_t index_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<int *>(index), 0, (int)(n4 * 4u), 0x00020000);
  constexpr unsigned kPastEnd = 0xfffffff0u;
  // and of all slots (the tile limit keeps them below 2^31 bytes), addressed as range part + tile part
  const __amdgpu_buffer_rsrc_t slot_buf =
      __builtin_amdgcn_make_buffer_rsrc(slots, 0, (int)((unsigned)kFineBins * tiles * (kFineSlotWords * 4u)), 0x00020000);
  // group u of the thread's indices of a tile; a tile past the last one reads as zeros
  auto fetch_group = [&](unsigned tile, int u) {
    const unsigned i = tile * kFineTile + threadIdx.x * kVec + u * (kFineBlock * kVec);
    return __builtin_amdgcn_raw_buffer_load_b128(index_buf, tile < tiles && i < n4 ? (int)(i * 4u) : (int)kPastEnd, 0, 0x2);
  };
  const Chunk nothing = {kFineNone | (kFineNone << 16), kFineNone | (kFineNone << 16), kFineNone | (kFineNone << 16),
                         kFineNone | (kFineNone << 16)};
  T acc = Op::identity();
  Raw v[kFineVecs];
#pragma unroll
  for (int u = 0; u < kFineVecs; ++u) v[u] = fetch_group(blockIdx.x, u);
  // between tiles the counters are zero and every place of the image holds kFineNone
  auto clear_counters = [&]() {                             // a wave its own
    for (unsigned b = (unsigned)lane_id(); b < (unsigned)kFineBins; b += kWave) cursor[wave][b] = 0u;
  };
  clear_counters();
  for (unsigned q = threadIdx.x; q < kChunks; q += kFineBlock) image[q] = nothing;
  __syncthreads();
  for (unsigned tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const unsigned base = tile * kFineTile + threadIdx.x * kVec;
    // rank of every element among the wave's elements of its range (range << 16 | rank is kept).  An index
    // outside the table (undefined anyway) gets the last range, so that everything stays inside LDS.
    unsigned where[kFineVecs][kVec];
#pragma unroll
    for (int u = 0; u < kFineVecs; ++u) {
      const bool in = base + u * (kFineBlock * kVec) < n4;
#pragma unroll
      for (int c = 0; c < kVec; ++c) {
        const unsigned b = min(__umulhi((unsigned)v[u][c], cut.magic) >> cut.shift, cut.bins - 1u);
        where[u][c] = b << 16;
        if (in) where[u][c] |= __hip_atomic_fetch_add(&cursor[wave][b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
      }
    }
    __syncthreads();
    // inside a range's slot the waves in order: thread t < kFineBins turns the counts of range t into first places
    if (threadIdx.x < (unsigned)kFineBins) {
      unsigned count[kFineWaves];                             // all read before any is written: one round trip to LDS, not sixteen
#pragma unroll
      for (int w = 0; w < kFineWaves; ++w) count[w] = cursor[w][threadIdx.x];
      unsigned run = 0;
#pragma unroll
      for (int w = 0; w < kFineWaves; ++w) {
        cursor[w][threadIdx.x] = run;
        run += count[w];
      }
    }
    __syncthreads();
    // every offset to its place in the image.  What a slot cannot take (indices that crowd into few
    // ranges) is evaluated on the spot; a wave skips that for a 128-bit group in which none of its lanes
    // has such an element.  As a group is done with, the same group of the workgroup's next tile is asked
    // for: asked for all at once, the reads would hold the waves up until most of them had come back.
#pragma unroll
    for (int u = 0; u < kFineVecs; ++u) {
      unsigned left = 0u;                                     // bit c: element c of the group found its slot full
      if (base + u * (kFineBlock * kVec) < n4) {
#pragma unroll
        for (int c = 0; c < kVec; ++c) {
          const unsigned b = where[u][c] >> 16;
          const unsigned offset = min((unsigned)v[u][c] - b * cut.range, cut.range - 1u);
          const unsigned place = cursor[wave][b] + (where[u][c] & 0xffffu);
          if (place < (unsigned)kFineCap) entries[b * kFineCap + place] = (unsigned short)offset;
          else left |= 1u << c;
        }
      }
      if (left != 0u) {
        typename C::Leaf x[kVec];
#pragma unroll
        for (int c = 0; c < kVec; ++c) {
          x[c] = typename C::Leaf();
          if (left >> c & 1u) x[c] = C::leaf(a, v[u][c]);
        }
#pragma unroll
        for (int c = 0; c < kVec; ++c) {
          const T val = C::template from_leaf<0>(a, x[c]);
          if (left >> c & 1u) acc = Op::apply(acc, val);
        }
      }
      v[u] = fetch_group(tile + gridDim.x, u);
    }
    __syncthreads();
    // the image goes to the tile's slots as it is, 128 bits a thread and step, and is emptied on the way;
    // ranges past the table's last one are empty and have slots of their own
    {
      constexpr unsigned kPerSlot = kFineCap / 8;
      constexpr int kSteps = kChunks / kFineBlock;
      static_assert(kSteps * kFineBlock == kChunks, "whole steps");
      Chunk out[kSteps];
#pragma unroll
      for (int k = 0; k < kSteps; ++k) out[k] = image[threadIdx.x + k * kFineBlock];
#pragma unroll
      for (int k = 0; k < kSteps; ++k) {
        unsigned q = threadIdx.x + k * kFineBlock;
        asm volatile("" : "+v"(q));                           // the offsets are worked out here, not kept in registers from tile to tile
        const unsigned b = q / kPerSlot, part = q - b * kPerSlot;
        image[q] = nothing;
        __builtin_amdgcn_raw_buffer_store_b128(out[k], slot_buf, (int)((b * tiles * kFineSlotWords + part * 4u) * 4u),
                                               (int)(tile * (kFineSlotWords * 4u)), 0);
      }
    }
    // No barrier here.  A wave goes on to rank the next tile in its own counters, which it clears itself;
    // the counts are not looked at by others, and the image not written to again, before the barriers that
    // follow the ranking, which no wave passes before all are done with this tile.
    clear_counters();
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4) acc = Op::apply(acc, E::template eval<0>(a, (int)(n4 + threadIdx.x)));
  // one partial per workgroup; the second kernel combines them with its own
  const unsigned tag = tag_of_epoch(load_agent(&ctl->epoch));
  T r = block_reduce<Op, kFineWaves>(acc, lds);
  if (threadIdx.x == 0) store_agent64(&partials[blockIdx.x], pack_word((unsigned)as_bits(r), tag, 1u));
}

template <class Op, class E>
__global__ __launch_bounds__(kFineBlock) void fold_fine_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                               const unsigned *slots, unsigned tiles, const FineCut cut,
                                                               unsigned elems, unsigned earlier) {
  using T = typename Op::T;
  using C = GatherChain<E>;
  using Leaf = typename C::Leaf;
  using Raw = unsigned __attribute__((ext_vector_type(4)));
  using RawI = int __attribute__((ext_vector_type(4)));
  constexpr int kStream = 0x2;                                // cache policy of the buffer loads: nt
  static_assert(sizeof(Leaf) == 4 && sizeof(T) == 4, "table elements and values are 32-bit words");
  __shared__ T slice[kFineSlice + kVec];                      // the values of the range's table elements, then the identity
  const Leaf *table = static_cast<const Leaf *>(a.in[C::kTable]);
  constexpr int kAhead = kFineSlice / (kFineBlock * kVec);    // 128-bit reads of table elements per thread and range
  constexpr int kInFlight = 6;                                // 128-bit reads of entries a lane has in flight
  constexpr unsigned kVecsPerSlot = kFineCap / 8;             // a 128-bit group holds eight entries
  // the whole 128-bit groups of range b, one read per thread and group: a group past the end of the
  // range, and every group of a range past the last, reads as zero without a memory access
  auto fetch_group = [&](unsigned b, int u) {
    const unsigned lo = b < cut.bins ? b * cut.range : 0u;
    const unsigned len = b < cut.bins ? min(cut.range, elems - lo) : 0u;
    const __amdgpu_buffer_rsrc_t range_buf =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<Leaf *>(table + lo), 0, (int)((len & ~3u) * 4u), 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(range_buf, (int)((threadIdx.x + u * kFineBlock) * (kVec * 4u)), 0, kStream);
  };
  if (threadIdx.x == 0) slice[kFineNone] = Op::identity();    // nothing else writes there
  T acc = Op::identity();
  RawI v[kAhead];
#pragma unroll
  for (int u = 0; u < kAhead; ++u) v[u] = fetch_group(blockIdx.x, u);
  for (unsigned b = blockIdx.x; b < cut.bins; b += gridDim.x) {
    const unsigned lo = b * cut.range;
    const unsigned len = min(cut.range, elems - lo), len4 = len & ~3u;
    // the range's slots lie one behind the other: one stream of 128-bit groups
    const unsigned groups = tiles * kVecsPerSlot;
    const __amdgpu_buffer_rsrc_t slot_buf = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned *>(slots + (size_t)b * tiles * kFineSlotWords), 0, (int)(groups * 16u), 0x00020000);
    Raw w[kInFlight];
    auto fetch_entries = [&](unsigned g0) {
#pragma unroll
      for (int u = 0; u < kInFlight; ++u)
        w[u] = __builtin_bit_cast(Raw, __builtin_amdgcn_raw_buffer_load_b128(slot_buf, (int)((g0 + u * kFineBlock) * 16u), 0, kStream));
    };
    __syncthreads();                                          // the range before is done with LDS
    // Values of the range's table elements.  As a group is used up, a group of the range's first entries
    // and the same group of the workgroup's next range are asked for: a compute unit has about a hundred
    // requests under way at a time, a wave that asks for more is held up until there is room, and it should
    // be held up here, where the other waves have values to work out, rather than with nothing to do.
    static_assert(kInFlight <= kAhead, "a group of entries per group of table elements");
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const unsigned i = (threadIdx.x + u * kFineBlock) * kVec;
      RawI val;
#pragma unroll
      for (int c = 0; c < kVec; ++c) val[c] = as_bits(C::template from_leaf<0>(a, from_bits<Leaf>(v[u][c])));
      if (i < len4) *reinterpret_cast<RawI *>(&slice[i]) = val;
      if (u < kInFlight)
        w[u] = __builtin_bit_cast(Raw, __builtin_amdgcn_raw_buffer_load_b128(slot_buf, (int)((threadIdx.x + u * kFineBlock) * 16u), 0, kStream));
      v[u] = fetch_group(b + gridDim.x, u);
    }
    if (threadIdx.x < len - len4) slice[len4 + threadIdx.x] = C::template from_leaf<0>(a, table[lo + len4 + threadIdx.x]);
    __syncthreads();
    for (unsigned g0 = threadIdx.x; g0 < groups; g0 += kFineBlock * kInFlight) {
#pragma unroll
      for (int u = 0; u < kInFlight; ++u) {
        if (g0 + u * kFineBlock < groups) {
          T x[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) x[k] = slice[(w[u][k / 2] >> (16 * (k & 1))) & 0xffffu];
#pragma unroll
          for (int k = 0; k < 8; ++k) acc = Op::apply(acc, x[k]);
        }
      }
      if (g0 - threadIdx.x + kFineBlock * kInFlight < groups) fetch_entries(g0 + kFineBlock * kInFlight);   // the same for the whole workgroup
    }
  }
  fold_finish<Op, kFineWaves>(acc, a, 0, ctl, partials, earlier);
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
    // unsigned: the step past a segment that ends at 2^31 - 1 must not wrap
    for (unsigned k = (unsigned)lo + sub; k < (unsigned)hi; k += 16) acc = Op::apply(acc, E::template eval<0>(a, (int)k));
    acc = row_scan_inclusive<Op>(acc);
    if (sub == 15 && r < rows) y[r] = acc;
  }
}

// ------------------------------------------------------------------ segmented fold over a gathered table, column blocked
// y[r] = fold(+, F(values[k], table[index[k]]) for k in segment r) where the table
// is too large for the L2 of one XCD (4 MiB) but not for four of them.  Random
// 4-byte gathers that miss L2 cost a 128-byte line each from the memory side, and
// the rate of those (about 52 G lines/s on this chip: its bandwidth in lines) bounds
// the plain kernel; gathers that hit L2 run four times faster.
// So the table is cut into kQuarters column ranges and every XCD works for one
// range only: workgroup b takes range b % 4 (workgroups go to the eight XCDs in
// turn, so XCDs q and q + 4 serve range q and keep it in their L2), reads the whole
// index and value streams of its rows and accumulates the terms whose index falls
// into its range.
//  * The streams must not push the table out of L2 and should cost as few requests
//    as possible: a unit's stretch of both arrays is read with 128-bit buffer loads
//    marked agent scope and non-temporal (sc1 nt: whole lines per request, not kept
//    in L2; reads past the end of the array return zero).  Measured: 4-byte
//    non-temporal reads 958 us, 27 % of the gathers missing L2; 128-bit reads with
//    sc1 alone 35 % missing, with sc1 nt 16 %.
//  * A thread keeps the elements it has read in registers, gathers for those whose
//    index falls into its range -- one gather instruction per element position,
//    issued for the lanes that have such an element only (the address unit takes a
//    cycle per lane of a gather, hit or not), all in flight together -- and puts the
//    terms (the identity for the other ranges) into LDS.  Then four lanes per row add
//    up the row's terms from LDS.  Every element is looked at by four workgroups, so
//    the arithmetic per element counts: the range test is done once per element and
//    kept as a bit, and the row sums take two DPP steps per 64 rows (sixteen lanes per
//    row and a row scan took 880 us, this form 745 us).
//  * The four workgroups 4i .. 4i+3 walk the same units of kBlockedRows rows.  For
//    unit u the one of range u % 4 combines: the other three pass their partial row
//    sums through memory (tagged words, then a tagged flag per unit), the combiner
//    adds the four partials in range order, so the result does not depend on timing.
//    Combining lags one unit behind, so nobody sits waiting for a partner.
// The streams are read four times over: 2.1 GB in whole lines, and 1.3 GB of gathered
// lines that still miss (the quarter is as large as the L2 it should stay in), instead
// of 7.5 GB.
constexpr int kQuarters = 4;
constexpr int kBlockedRows = kBlock;                  // rows of a unit: one per thread at the exchange
constexpr int kUnitCap = 4608;                        // elements of a unit staged in LDS (a unit of 16-element rows has 4096)
constexpr int kUnitVecs = (kUnitCap / kVec + kBlock - 1) / kBlock;   // 128-bit reads per thread and array

template <class Op, class F, int KV, int KI, int KT>
__global__ __launch_bounds__(kBlock) void foldseg_blocked_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                                 unsigned long long *flags, unsigned long long *work, int range_len) {
  using T = typename Op::T;
  using Raw = int __attribute__((ext_vector_type(4)));
  static_assert(sizeof(T) == 4, "partials travel as 32-bit words");
  __shared__ T sums_of[2][kBlockedRows];            // double buffered: a unit is combined one unit later
  __shared__ int row_start[kBlockedRows + 1];
  __shared__ T term_of[kUnitCap];                   // the unit's terms of this range, the identity elsewhere
  const int *off = static_cast<const int *>(a.in[kMaxIn - 1]);
  const int *index = static_cast<const int *>(a.in[KI]);
  const T *values = static_cast<const T *>(a.in[KV]);
  const T *table = static_cast<const T *>(a.in[KT]);
  T *y = static_cast<T *>(a.out[0]);
  const unsigned rows = (unsigned)a.aux;
  const unsigned n_units = (rows + kBlockedRows - 1) / kBlockedRows;
  const unsigned q = blockIdx.x % kQuarters, team = blockIdx.x / kQuarters, teams = gridDim.x / kQuarters;
  const unsigned lo_col = q * (unsigned)range_len;
  const unsigned epoch = load_agent(&ctl->epoch);
  const unsigned tag = tag_of_epoch(epoch);
  // raw buffer views of the two streams: byte offsets, range checked against the array's size
  const __amdgpu_buffer_rsrc_t index_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<int *>(index), 0, a.n * 4, 0x00020000);
  const __amdgpu_buffer_rsrc_t value_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(values), 0, a.n * 4, 0x00020000);
  constexpr int kAgentScope = 0x12;                 // cache policy of the buffer loads: sc1 | nt

  // Adds the partials of the four ranges of unit `unit` in range order and stores its rows;
  // `own` holds this workgroup's partials of that unit.
  auto combine = [&](unsigned unit, const T *own) {
    if (threadIdx.x < kQuarters && threadIdx.x != q)
      (void)wait_word(&flags[(size_t)unit * kQuarters + threadIdx.x], tag, ctl);
    __syncthreads();
    const unsigned r = unit * kBlockedRows + threadIdx.x;
    if (r < rows) {
      // the flags live in the control block, which starts out as zeros, so a flag of this
      // launch means that the partials have been stored; the tag of each word covers the
      // case that a word becomes visible after its flag.  The three words are read together
      // (one round trip to memory instead of three); one that does not carry the tag yet is waited for.
      unsigned long long w[kQuarters];
#pragma unroll
      for (unsigned p = 0; p < (unsigned)kQuarters; ++p) w[p] = p != q ? load_agent64(work + (size_t)p * rows + r) : 0ull;
      T v = Op::identity();
#pragma unroll
      for (unsigned p = 0; p < (unsigned)kQuarters; ++p) {
        T part = own[threadIdx.x];
        if (p != q) {
          const unsigned lo = (unsigned)w[p];
          if ((lo >> 2) != tag || (lo & 3u) == 0u) w[p] = wait_word(work + (size_t)p * rows + r, tag, ctl);
          part = w[p] ? from_bits<T>((int)(unsigned)(w[p] >> 32)) : Op::identity();
        }
        v = Op::apply(v, part);
      }
      __builtin_nontemporal_store(v, y + r);     // a result: written once, and nothing but the table should settle in L2
    }
  };

  // A unit is a chain of round trips to memory (row offsets, streams, gathers, the partners' partials), and a
  // workgroup walks its units one after the other: the row offsets of the next unit are asked for while this
  // one is worked on, which takes one link out of every chain.  (Asking for the next unit's streams that early
  // as well costs thirty registers, a third of the resident workgroups, and gains nothing: 739 us against 730.)
  // (agent scope, like the streams: nothing but the table should settle in L2)
  const unsigned *offu = reinterpret_cast<const unsigned *>(off);
  auto offset_of_row = [&](unsigned unit, unsigned local) {
    const unsigned r = unit * kBlockedRows + local;
    return unit < n_units ? (int)load_agent(offu + (r < rows ? r : rows)) : 0;
  };
  int next_start = offset_of_row(team, threadIdx.x), next_end = threadIdx.x == 0 ? offset_of_row(team, kBlockedRows) : 0;
  unsigned iter = 0, prev = ~0u;
  for (unsigned u = team; u < n_units; u += teams, ++iter) {
    T *sums = sums_of[iter & 1];
    // the unit's row offsets, read once and coalesced (rows past the end are empty)
    row_start[threadIdx.x] = next_start;
    if (threadIdx.x == 0) row_start[kBlockedRows] = next_end;
    next_start = offset_of_row(u + teams, threadIdx.x);
    if (threadIdx.x == 0) next_end = offset_of_row(u + teams, kBlockedRows);
    __syncthreads();
    // the unit's stretch of both streams, from the 16-byte boundary below its first element:
    // read, gather, multiply, and leave the terms in LDS
    const int base = row_start[0] & ~(kVec - 1);
    const int staged = min(row_start[kBlockedRows] - base, kUnitCap);
    {
      Raw ci[kUnitVecs], cv[kUnitVecs];
#pragma unroll
      for (int i = 0; i < kUnitVecs; ++i) {
        const int e = ((int)threadIdx.x + i * kBlock) * kVec;
        ci[i] = Raw{-1, -1, -1, -1};                 // -1 is in no range
        cv[i] = Raw{0, 0, 0, 0};
        if (e < staged) {
          ci[i] = __builtin_amdgcn_raw_buffer_load_b128(index_buf, (base + e) * 4, 0, kAgentScope);
          cv[i] = __builtin_amdgcn_raw_buffer_load_b128(value_buf, (base + e) * 4, 0, kAgentScope);
        }
      }
      // the values wait in LDS (where the terms will stand) while the gathers are in flight:
      // fewer registers per thread, more workgroups per compute unit
#pragma unroll
      for (int i = 0; i < kUnitVecs; ++i) {
        const int e = ((int)threadIdx.x + i * kBlock) * kVec;
        if (e < staged) *reinterpret_cast<Raw *>(&term_of[e]) = cv[i];
      }
      // which of this thread's elements fall into the range: one bit each, tested once
      unsigned mine = 0;
#pragma unroll
      for (int i = 0; i < kUnitVecs; ++i)
#pragma unroll
        for (int c = 0; c < kVec; ++c) mine |= (unsigned)((unsigned)ci[i][c] - lo_col < (unsigned)range_len) << (i * kVec + c);
      T x[kUnitVecs][kVec];
#pragma unroll
      for (int i = 0; i < kUnitVecs; ++i)
#pragma unroll
        for (int c = 0; c < kVec; ++c) {
          x[i][c] = Op::identity();
          if (mine >> (i * kVec + c) & 1u) x[i][c] = table[ci[i][c]];
        }
#pragma unroll
      for (int i = 0; i < kUnitVecs; ++i) {
        const int e = ((int)threadIdx.x + i * kBlock) * kVec;
        if (e < staged) {
          using TV = T __attribute__((ext_vector_type(4)));
          const TV v = *reinterpret_cast<const TV *>(&term_of[e]);        // this thread's own store above
          Vec4<T> t;
#pragma unroll
          for (int c = 0; c < kVec; ++c)
            t.v[c] = (mine >> (i * kVec + c) & 1u) ? F::apply(a.p[0], v[c], x[i][c]) : Op::identity();
          store4_lds(&term_of[e], t);
        }
      }
    }
    __syncthreads();
    // four lanes per row add up its terms (64 rows at a time), then the quad combines; a
    // unit with more than kUnitCap elements takes the rest from memory
    constexpr int kRowsPerStep4 = kBlock / 4;
    const unsigned ql = threadIdx.x & 3u;
    for (unsigned step = 0; step < kBlockedRows / kRowsPerStep4; ++step) {
      const unsigned local = step * kRowsPerStep4 + threadIdx.x / 4;
      const int lo = row_start[local], hi = row_start[local + 1];
      T acc = Op::identity();
      for (int k = lo + (int)ql; k < hi; k += 4) {
        const int e = k - base;
        if (e < kUnitCap) {
          acc = Op::apply(acc, term_of[e]);
        } else {
          const int c = In<KI, int>::template eval<0, true>(a, k);
          if ((unsigned)c - lo_col < (unsigned)range_len)
            acc = Op::apply(acc, F::apply(a.p[0], In<KV, T>::template eval<0, true>(a, k), table[c]));
        }
      }
      acc = Op::apply(acc, dpp_move<0xB1>(Op::identity(), acc));    // quad_perm [1,0,3,2]
      acc = Op::apply(acc, dpp_move<0x4E>(Op::identity(), acc));    // quad_perm [2,3,0,1]
      if (ql == 0) sums[local] = acc;
    }
    __syncthreads();
    // The workgroup of range u % 4 combines unit u; the other three publish their partials:
    // every partial as a tagged word (value and tag travel in one 64-bit store, so a reader
    // can tell a word of this launch from whatever lay there before), then, once the stores
    // of all threads are out, the unit's flag.
    if (q != u % kQuarters) {
      const unsigned r = u * kBlockedRows + threadIdx.x;
      if (r < rows) store_agent64(work + (size_t)q * rows + r, pack_word((unsigned)as_bits(sums[threadIdx.x]), tag, 1u));
      __syncthreads();
      if (threadIdx.x == 0) store_agent64(&flags[(size_t)u * kQuarters + q], pack_word(1u, tag, 1u));
    }
    // Combining lags one unit behind: by now the partials of the previous unit have long
    // been published, so the combiner does not sit waiting for its three partners.
    if (prev != ~0u && q == prev % kQuarters) combine(prev, sums_of[(iter & 1) ^ 1]);
    prev = u;
  }
  if (prev != ~0u && q == prev % kQuarters) combine(prev, sums_of[(iter & 1) ^ 1]);
  // every workgroup has taken its tag once its word is out; the last one then moves the epoch on
  if (threadIdx.x == 0) store_agent64(&partials[blockIdx.x], pack_word(0u, tag, 1u));
  if (blockIdx.x == gridDim.x - 1) {
    for (unsigned k = threadIdx.x; k < gridDim.x; k += kBlock) (void)wait_word(&partials[k], tag, ctl);
    __syncthreads();
    if (threadIdx.x == 0) store_agent(&ctl->epoch, epoch + 1u);
  }
}

// ------------------------------------------------------------------ segmented fold over a gathered table, sorted through LDS
// The same computation, y[r] = fold(+, F(values[k], table[index[k]]) for k in segment r), for tables
// of up to 2^24 elements, without a gather that leaves the compute unit.  Gathers from L2 are bound
// by the rate at which an L2 takes requests and cost the streams a reading per column range (the
// kernel above); gathers from LDS cost a few cycles a wave, but a compute unit holds 1/128 of such
// a table, and a row has an element or none in a range that small: the gathered values have to go
// back to their positions before rows can be added up.  Four kernels, all streaming:
//
//  1. seg_bin_kernel sorts every tile of kSegTile positions by table range, as bin_fine_kernel
//     does (an LDS counter per wave and range, the tile's slots built in LDS as they go to memory),
//     and keeps two 16-bit numbers per element, in two arrays: the offset inside the range and the
//     position inside the tile (offsets slot after slot for every range, positions tile after tile).
//     An element that finds its slot full (a few in a thousand of evenly spread indices; most
//     of indices that crowd into few ranges) goes onto the tile's list of (position, index) pairs.
//  2. seg_gather_kernel: a workgroup reads a table range into LDS and turns a stretch of the
//     range's offsets into values, slot for slot (the slots of a range lie one behind the other).
//  3. seg_rows_kernel: a workgroup per tile puts the tile's values (one slot per range, then those
//     of the list, gathered from memory) back at their positions in LDS, multiplies by the tile's
//     stretch of `values`, and adds up the rows, four lanes a row.  A row belongs to the tile it
//     starts in; the part of a row that lies in another tile than its own, and the part of a
//     tile's last row when the row goes on, are kept per tile,
//  4. and seg_join_kernel adds those up, tile after tile, for the rows that cross a tile boundary.
//
// Every element has one place at every stage and every sum a fixed order: the same bits on every
// launch.  Bytes per element: 4 + 4 (first kernel), 2 + 4 (second), 4 + 2 + 4 (third), times the
// slots' slack (a slot holds little more than the mean of a uniform spread: what overflows is listed).
constexpr int kSegBlock = 1024;                        // threads per workgroup of the first two kernels
constexpr int kSegWaves = kSegBlock / kWave;
constexpr int kSegTile = 16384;                        // positions per tile: 14-bit positions, a tile of values is 64 KiB of LDS
constexpr int kSegVecs = kSegTile / (kSegBlock * kVec);      // 128-bit reads per thread and tile
constexpr int kSegImageWords = 24576;                  // words of a tile's slots in LDS at most (96 KiB)
constexpr int kSegMaxBins = 512;
constexpr int kSegRowsBlock = 512;                     // threads per workgroup of the third kernel: two workgroups per compute unit
constexpr int kSegRowsStaged = 2048;                   // row starts of a tile kept in LDS (a tile of 16-element rows has 1024)
constexpr unsigned kSegNoPlace = 0xffffu;              // the position of a slot's place that holds no element
constexpr int kSegSlice = 36864;                       // elements of a table range at most: 144 KiB of LDS in the second kernel
constexpr unsigned kSegNone = kSegSlice;               // the offset of a slot's place that holds no element
constexpr unsigned kSegNothing = kSegNone | (kSegNoPlace << 16);
static_assert(kSegNone < 65536u, "offsets are 16-bit numbers");
static_assert(kSegVecs * kSegBlock * kVec == kSegTile && kSegTile <= (int)kSegNoPlace, "whole reads; positions are 16-bit numbers");

// How a launch is cut: the table into ranges, the elements into tiles, a slot per (range, tile).
struct SegPlan {
  FineCut cut;
  unsigned cap;        // entries per slot, a multiple of eight
  unsigned tiles;
};

template <int KI>
__global__ __launch_bounds__(kSegBlock) void seg_bin_kernel(const KArgs a, unsigned short *offsets, unsigned short *places,
                                                            unsigned short *list_place, unsigned *list_index, unsigned *list_count,
                                                            const SegPlan plan, unsigned elems) {
  using Raw = int __attribute__((ext_vector_type(4)));
  using Chunk = unsigned __attribute__((ext_vector_type(4)));
  __shared__ unsigned cursor[kSegWaves][kSegMaxBins];       // per (wave, range): the count, then the wave's first place in the slot
  __shared__ Chunk image[kSegImageWords / 4];               // the tile's slots: offset | position << 16 per element
  __shared__ unsigned listed;                               // elements on the tile's list so far
  __shared__ unsigned list_wait[kSegWaves][kWave][2];       // per wave: (position, index) of elements that wait to go onto the list together
  unsigned *entry = reinterpret_cast<unsigned *>(image);
  const int *index = static_cast<const int *>(a.in[KI]);
  const FineCut cut = plan.cut;
  const unsigned cap = plan.cap, tiles = plan.tiles, bins = cut.bins;
  const unsigned n = (unsigned)a.n;
  const unsigned wave = (unsigned)wave_id();
  const unsigned words = bins * cap;                        // of the image that are in use
  // raw buffer view of the index array: a 32-bit word past the end reads as zero without a memory access
  const __amdgpu_buffer_rsrc_t index_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<int *>(index), 0, (int)(n * 4u), 0x00020000);
  constexpr unsigned kPastEnd = 0xfffffff0u;
  auto fetch_group = [&](unsigned tile, int u) {
    const unsigned i = tile * kSegTile + threadIdx.x * kVec + u * (kSegBlock * kVec);
    return __builtin_amdgcn_raw_buffer_load_b128(index_buf, tile < tiles && i < n ? (int)(i * 4u) : (int)kPastEnd, 0, 0x2);
  };
  const Chunk nothing = {kSegNothing, kSegNothing, kSegNothing, kSegNothing};
  Raw v[kSegVecs];
#pragma unroll
  for (int u = 0; u < kSegVecs; ++u) v[u] = fetch_group(blockIdx.x, u);
  auto clear_counters = [&]() {                             // a wave its own, of the ranges there are
    for (unsigned b = (unsigned)lane_id(); b < bins; b += kWave) cursor[wave][b] = 0u;
  };
  // where the groups of eight entries that this thread copies out lie in a range's run of slots: worked out once
  constexpr int kCopies = kSegImageWords / 8 / kSegBlock;
  static_assert(kCopies * kSegBlock * 8 == kSegImageWords, "whole steps");
  unsigned copy_to[kCopies];                                // b * tiles * cap + part, without the tile's share
#pragma unroll
  for (int k = 0; k < kCopies; ++k) {
    const unsigned q = threadIdx.x + k * kSegBlock, b = q * 8u / cap, part = q * 8u - b * cap;
    copy_to[k] = b * tiles * cap + part;
  }
  // between tiles the counters are zero, every place of the image holds nothing and the list is empty
  clear_counters();
  for (unsigned q = threadIdx.x; q < words / 4u; q += kSegBlock) image[q] = nothing;
  if (threadIdx.x == 0) listed = 0u;
  __syncthreads();
  for (unsigned tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    if (threadIdx.x == 0) listed = 0u;                      // read last before the barrier that ended the tile before; added to after the next two
    const unsigned first = threadIdx.x * kVec;              // this thread's first position in the tile, group 0
    const unsigned base = tile * kSegTile;
    // rank of every element among the wave's elements of its range (range << 16 | rank is kept).  An index
    // outside the table (undefined anyway) gets the last range, so that everything stays inside LDS.
    unsigned where[kSegVecs][kVec];
    const unsigned here = n - base;                         // positions of this tile that exist (or more)
#pragma unroll
    for (int u = 0; u < kSegVecs; ++u) {
#pragma unroll
      for (int c = 0; c < kVec; ++c) {
        const unsigned b = min(__umulhi((unsigned)v[u][c], cut.magic) >> cut.shift, bins - 1u);
        where[u][c] = b << 16;
        if (first + u * (kSegBlock * kVec) + c < here)
          where[u][c] |= __hip_atomic_fetch_add(&cursor[wave][b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
      }
    }
    __syncthreads();
    // inside a range's slot the waves in order: thread t < bins turns the counts of range t into first places
    if (threadIdx.x < bins) {
      unsigned count[kSegWaves];                              // all read before any is written: one round trip to LDS, not sixteen
#pragma unroll
      for (int w = 0; w < kSegWaves; ++w) count[w] = cursor[w][threadIdx.x];
      unsigned run = 0;
#pragma unroll
      for (int w = 0; w < kSegWaves; ++w) {
        cursor[w][threadIdx.x] = run;
        run += count[w];
      }
    }
    __syncthreads();
    // Every element to its place in the image, or with its index onto the list: a wave collects such
    // elements in LDS (places from a ballot, no atomic in the way) and appends them to the tile's list sixty-
    // four at a time at most, reserving the places with one atomic.  As a group is done with, the same
    // group of the workgroup's next tile is asked for.
    unsigned waiting = 0;                                     // elements in this wave's part of list_wait: the same in all lanes
    auto append = [&]() {                                     // the whole wave, converged
      unsigned at_list = 0;
      if (lane_id() == 0) at_list = atomicAdd(&listed, waiting);
      at_list = (unsigned)__builtin_amdgcn_readfirstlane((int)at_list);
      if ((unsigned)lane_id() < waiting) {
        list_place[(size_t)base + at_list + (unsigned)lane_id()] = (unsigned short)list_wait[wave][lane_id()][0];
        list_index[(size_t)base + at_list + (unsigned)lane_id()] = list_wait[wave][lane_id()][1];
      }
      waiting = 0;
    };
#pragma unroll
    for (int u = 0; u < kSegVecs; ++u) {
#pragma unroll
      for (int c = 0; c < kVec; ++c) {
        const unsigned at = first + u * (kSegBlock * kVec) + c;
        const unsigned b = where[u][c] >> 16;
        const unsigned offset = min((unsigned)v[u][c] - b * cut.range, cut.range - 1u);
        const unsigned place = cursor[wave][b] + (where[u][c] & 0xffffu);
        const bool real = at < here;
        if (real && place < cap) entry[b * cap + place] = offset | (at << 16);
        const bool over = real && place >= cap;
        const unsigned long long overs = __builtin_amdgcn_ballot_w64(over);
        if (overs != 0ull) {                                  // the same for the whole wave
          const unsigned more = (unsigned)__builtin_popcountll(overs);
          if (waiting + more > (unsigned)kWave) append();
          if (over) {
            const unsigned k = waiting + __builtin_amdgcn_mbcnt_hi((unsigned)(overs >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)overs, 0u));
            list_wait[wave][k][0] = at;
            list_wait[wave][k][1] = min((unsigned)v[u][c], elems - 1u);
          }
          waiting += more;
        }
      }
      v[u] = fetch_group(tile + gridDim.x, u);
    }
    if (waiting != 0u) append();
    __syncthreads();
    // the image goes to the tile's slots, eight entries a thread and step (128 bits of offsets, 128 bits
    // of positions), and is emptied on the way
#pragma unroll
    for (int k = 0; k < kCopies; ++k) {
      const unsigned q = threadIdx.x + k * kSegBlock;
      if (q < words / 8u) {
        const Chunk lo = image[2u * q], hi = image[2u * q + 1u];
        image[2u * q] = nothing;
        image[2u * q + 1u] = nothing;
        const size_t at = (size_t)copy_to[k] + (size_t)tile * cap;
        Chunk o, p;
        o[0] = (lo[0] & 0xffffu) | (lo[1] << 16);
        o[1] = (lo[2] & 0xffffu) | (lo[3] << 16);
        o[2] = (hi[0] & 0xffffu) | (hi[1] << 16);
        o[3] = (hi[2] & 0xffffu) | (hi[3] << 16);
        p[0] = (lo[0] >> 16) | (lo[1] & 0xffff0000u);
        p[1] = (lo[2] >> 16) | (lo[3] & 0xffff0000u);
        p[2] = (hi[0] >> 16) | (hi[1] & 0xffff0000u);
        p[3] = (hi[2] >> 16) | (hi[3] & 0xffff0000u);
        *reinterpret_cast<Chunk *>(offsets + at) = o;
        *reinterpret_cast<Chunk *>(places + (size_t)tile * words + q * 8u) = p;
      }
    }
    // No barrier here.  A wave goes on to rank the next tile in its own counters, which it clears itself;
    // the counts are not looked at by others, and the image and the list not written to again, before the
    // barriers that follow the ranking, which no wave passes before all are done with this tile.
    clear_counters();
    if (threadIdx.x == 0) list_count[tile] = listed;          // settled before the barrier above
  }
}

// The number of rows r in [0, rows) with start[r] < target, start ascending: all lanes of a wave take
// part, sixty-four probes a step.
__device__ __forceinline__ unsigned wave_rows_below(const unsigned *start, unsigned rows, unsigned target) {
  unsigned lo = 0, len = rows;
  const unsigned lane = (unsigned)lane_id();
  while (len != 0u) {                                         // the same for the whole wave
    const unsigned stride = (len + kWave - 1u) / kWave;
    const unsigned probe = lo + (lane + 1u) * stride - 1u;    // the last row of this lane's stretch
    const bool inside = probe < lo + len;
    const bool below = inside && start[probe] < target;
    const unsigned k = (unsigned)__builtin_popcountll(__builtin_amdgcn_ballot_w64(below));
    // stretches 0 .. k-1 lie below the target; the first row at or above it is in stretch k, whose last
    // row is known not to be below if that row exists
    const unsigned next = lo + k * stride;
    const unsigned left = lo + len > next ? lo + len - next : 0u;
    const bool last_known = k < (unsigned)kWave && next + stride - 1u < lo + len;
    len = last_known ? stride - 1u : min(left, stride);
    lo = next;
  }
  return lo;
}

template <class T, int KT>
__global__ __launch_bounds__(kSegBlock) void seg_gather_kernel(const KArgs a, const unsigned short *offsets, T *gathered,
                                                               unsigned *first_row, const SegPlan plan, unsigned elems, unsigned parts) {
  using Raw = unsigned __attribute__((ext_vector_type(4)));
  using RawI = int __attribute__((ext_vector_type(4)));
  using TV = T __attribute__((ext_vector_type(4)));
  constexpr int kStream = 0x2;                                // cache policy of the buffer loads: nt
  static_assert(sizeof(T) == 4, "table elements are 32-bit words");
  __shared__ T slice[kSegSlice + kVec];                       // the range of the table, then an element for the places that hold nothing
  const T *table = static_cast<const T *>(a.in[KT]);
  const FineCut cut = plan.cut;
  const unsigned b = blockIdx.x / parts, part = blockIdx.x - b * parts;      // the grid is bins * parts workgroups
  const unsigned lo = b * cut.range, len = min(cut.range, elems - lo), len4 = len & ~3u;
  {
    const __amdgpu_buffer_rsrc_t range_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(table + lo), 0, (int)(len4 * 4u), 0x00020000);
    constexpr int kAhead = kSegSlice / (kSegBlock * kVec);
    static_assert(kAhead * kSegBlock * kVec == kSegSlice, "whole reads");
    RawI v[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u)
      v[u] = __builtin_amdgcn_raw_buffer_load_b128(range_buf, (int)((threadIdx.x + u * kSegBlock) * (kVec * 4u)), 0, 0);
    // On the side, for the third kernel: the first row that starts in a tile, for every tile, a wave a tile
    // (the waves of this launch share the tiles out); the lookups run while the table range is on its way.
    {
      const unsigned *row_start = reinterpret_cast<const unsigned *>(a.in[kMaxIn - 1]);
      const unsigned rows = (unsigned)a.aux;
      for (unsigned t = blockIdx.x * kSegWaves + (unsigned)wave_id(); t < plan.tiles; t += gridDim.x * kSegWaves) {
        const unsigned r = wave_rows_below(row_start, rows, t * kSegTile);
        if (lane_id() == 0) first_row[t] = r;
      }
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const unsigned i = (threadIdx.x + u * kSegBlock) * kVec;
      if (i < len4) *reinterpret_cast<RawI *>(&slice[i]) = v[u];
    }
    if (threadIdx.x < len - len4) slice[len4 + threadIdx.x] = table[lo + len4 + threadIdx.x];
    if (threadIdx.x == 0) slice[kSegNone] = T();
  }
  __syncthreads();
  // The range's slots lie one behind the other: a stream of groups of four offsets (64 bits in, 128 bits
  // of values out, both without gaps from lane to lane), of which this workgroup takes the stretch
  // `part`.  The reads of the next batch are under way while a batch is worked on.
  const unsigned groups = plan.tiles * (plan.cap / 4u);
  const unsigned per = (groups + parts - 1u) / parts;
  const unsigned g_lo = part * per, g_hi = min(g_lo + per, groups);
  const size_t start = (size_t)b * plan.tiles * plan.cap;
  const __amdgpu_buffer_rsrc_t offset_buf =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short *>(offsets + start), 0, (int)(groups * 8u), 0x00020000);
  T *out = gathered + start;
  constexpr int kInFlight = 8;
  using Pair = unsigned __attribute__((ext_vector_type(2)));
  auto fetch = [&](unsigned g0, Pair (&w)[kInFlight]) {       // a group past the stretch reads as zeros without a memory access
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const unsigned g = g0 + u * kSegBlock;
      w[u] = __builtin_bit_cast(Pair, __builtin_amdgcn_raw_buffer_load_b64(offset_buf, g < g_hi ? (int)(g * 8u) : (int)0xfffffff0u, 0, kStream));
    }
  };
  auto work = [&](unsigned g0, const Pair (&w)[kInFlight]) {
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const unsigned g = g0 + u * kSegBlock;
      if (g < g_hi) {
        TV x;
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = slice[(w[u][k / 2] >> (16 * (k & 1))) & 0xffffu];
        *reinterpret_cast<TV *>(out + (size_t)g * 4u) = x;
      }
    }
  };
  constexpr unsigned kStep = kSegBlock * kInFlight;
  Pair w0[kInFlight], w1[kInFlight];
  unsigned g0 = g_lo + threadIdx.x;
  fetch(g0, w0);
  while (g0 - threadIdx.x < g_hi) {                           // the same for the whole workgroup
    fetch(g0 + kStep, w1);
    work(g0, w0);
    g0 += kStep;
    if (!(g0 - threadIdx.x < g_hi)) break;
    fetch(g0 + kStep, w0);
    work(g0, w1);
    g0 += kStep;
  }
}

template <class Op, class F, int KV, int KT>
__global__ __launch_bounds__(kSegRowsBlock) void seg_rows_kernel(const KArgs a, const unsigned short *places, const typename Op::T *gathered,
                                                                 const unsigned short *list_place, const unsigned *list_index,
                                                                 const unsigned *list_count, const unsigned *first_row,
                                                                 typename Op::T *head, typename Op::T *tail, const SegPlan plan) {
  using T = typename Op::T;
  using TV = T __attribute__((ext_vector_type(4)));
  using Pair = unsigned __attribute__((ext_vector_type(2)));
  using RawI = int __attribute__((ext_vector_type(4)));
  __shared__ T term[kSegTile];                                // the tile's gathered values, then its terms, by position
  __shared__ unsigned row_at[kSegRowsStaged + 1];             // where the tile's first kSegRowsStaged rows start, and the row after them
  const unsigned *start = reinterpret_cast<const unsigned *>(a.in[kMaxIn - 1]);
  const T *values = static_cast<const T *>(a.in[KV]);
  const T *table = static_cast<const T *>(a.in[KT]);
  T *y = static_cast<T *>(a.out[0]);
  const unsigned rows = (unsigned)a.aux, n = (unsigned)a.n;
  const unsigned tile = blockIdx.x, tiles = plan.tiles, cap = plan.cap, bins = plan.cut.bins;
  const unsigned t_lo = tile * kSegTile, t_hi = min(t_lo + (unsigned)kSegTile, n);
  // the tile's stretch of `values` is asked for first and used last (a 32-bit word past the end of the array reads as zero)
  constexpr int kSteps = kSegTile / (kSegRowsBlock * kVec);
  RawI factor[kSteps];
  {
    const __amdgpu_buffer_rsrc_t value_buf = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(values), 0, (int)(n * 4u), 0x00020000);
#pragma unroll
    for (int k = 0; k < kSteps; ++k) {
      const unsigned e = (threadIdx.x + k * kSegRowsBlock) * kVec;
      factor[k] = __builtin_amdgcn_raw_buffer_load_b128(value_buf, t_lo + e < n ? (int)((t_lo + e) * 4u) : (int)0xfffffff0u, 0, 0x2);
    }
  }
  // The elements on the tile's list (those that found their slot full) are asked for now as well, a thread
  // an element: count, then position and index, then the table element -- three round trips in a row that
  // are over by the time the slots have been put in place.
  const unsigned listed = list_count[tile];
  unsigned listed_place = 0;
  T listed_value = T();
  if (threadIdx.x < listed) {
    listed_place = list_place[(size_t)t_lo + threadIdx.x];
    listed_value = table[list_index[(size_t)t_lo + threadIdx.x]];
  }
  // the first row that starts in this tile and in the next (the last tile takes the empty rows at the end);
  // the row before reaches into the tile if it ends behind the tile's first position (start[rows] is the
  // number of elements)
  const unsigned row_lo = first_row[tile], row_hi = tile + 1u < tiles ? first_row[tile + 1u] : rows;
  const unsigned r_first = row_lo - (row_lo > 0u && start[row_lo] > t_lo ? 1u : 0u);
  // The values back to their positions: four entries a thread and step, the reads of the next steps under
  // way while those of the last ones are put in place.  Range and place of a step are carried along from
  // step to step, not divided out.
  {
    const unsigned per_slot = cap / 4u, quads = bins * per_slot;
    constexpr int kAtOnce = 4;
    const unsigned step_slot = (unsigned)kSegRowsBlock / per_slot, step_part = (unsigned)kSegRowsBlock - step_slot * per_slot;
    unsigned q = threadIdx.x;                                 // the step that is asked for next
    unsigned b = q / per_slot, part = q - b * per_slot;
    // raw buffer views (a launch's slots stay below 2^31 bytes): a step past the last one reads zeros and is not used
    const __amdgpu_buffer_rsrc_t value_view = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T *>(gathered), 0, (int)(bins * tiles * cap * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t place_view = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned short *>(places + (size_t)tile * (bins * cap)), 0, (int)(bins * cap * 2u), 0x00020000);
    auto fetch = [&](TV (&x)[kAtOnce], Pair (&p)[kAtOnce]) {
#pragma unroll
      for (int u = 0; u < kAtOnce; ++u) {
        const bool real = q < quads;
        x[u] = __builtin_bit_cast(TV, __builtin_amdgcn_raw_buffer_load_b128(
            value_view, real ? (int)((b * tiles * cap + part * 4u) * 4u) : (int)0xfffffff0u, (int)(tile * cap * 4u), 0x2));
        p[u] = __builtin_bit_cast(Pair, __builtin_amdgcn_raw_buffer_load_b64(place_view, real ? (int)(q * 8u) : (int)0xfffffff0u, 0, 0x2));
        q += kSegRowsBlock;
        b += step_slot;
        part += step_part;
        if (part >= per_slot) { part -= per_slot; ++b; }
      }
    };
    auto put = [&](unsigned q0, const TV (&x)[kAtOnce], const Pair (&p)[kAtOnce]) {
#pragma unroll
      for (int u = 0; u < kAtOnce; ++u) {
        if (q0 + u * kSegRowsBlock < quads) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const unsigned place = (p[u][c / 2] >> (16 * (c & 1))) & 0xffffu;
            if (place != kSegNoPlace) term[place] = x[u][c];
          }
        }
      }
    };
    constexpr unsigned kStep = kSegRowsBlock * kAtOnce;
    TV x0[kAtOnce], x1[kAtOnce];
    Pair p0[kAtOnce], p1[kAtOnce];
    unsigned q0 = threadIdx.x;                                // the first step of the batch that is put in place next
    fetch(x0, p0);
    while (q0 - threadIdx.x < quads) {                        // the same for the whole workgroup
      fetch(x1, p1);
      put(q0, x0, p0);
      q0 += kStep;
      if (!(q0 - threadIdx.x < quads)) break;
      fetch(x0, p0);
      put(q0, x1, p1);
      q0 += kStep;
    }
    if (threadIdx.x < listed) term[listed_place] = listed_value;
    for (unsigned k = threadIdx.x + kSegRowsBlock; k < listed; k += kSegRowsBlock)
      term[list_place[(size_t)t_lo + k]] = table[list_index[(size_t)t_lo + k]];
  }
  __syncthreads();
  // Rows: the tile's own are those that start in it; the row that reaches into it from before (if there
  // is one) comes first.  Where the first kSegRowsStaged of them start goes to LDS while the values are
  // multiplied in.
  const unsigned staged = min(row_hi - r_first, (unsigned)kSegRowsStaged);
  {
    constexpr int kLoads = kSegRowsStaged / kSegRowsBlock + 1;
    unsigned at[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const unsigned i = threadIdx.x + k * kSegRowsBlock;
      at[k] = i <= staged ? start[r_first + i] : 0u;          // r_first + staged <= rows: start has that entry
    }
#pragma unroll
    for (int k = 0; k < kSteps; ++k) {
      const unsigned e = (threadIdx.x + k * kSegRowsBlock) * kVec;
      TV g = *reinterpret_cast<const TV *>(&term[e]);
#pragma unroll
      for (int c = 0; c < kVec; ++c) g[c] = F::apply(a.p[0], from_bits<T>(factor[k][c]), g[c]);
      *reinterpret_cast<TV *>(&term[e]) = g;
    }
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      const unsigned i = threadIdx.x + k * kSegRowsBlock;
      if (i <= staged) row_at[i] = at[k];
    }
  }
  __syncthreads();
  // Four lanes a row, kRowsAtOnce rows a lane and step: their starts are read from LDS together, then the
  // first kRowAhead terms a lane takes of each (every fourth of the row), so that a step is two round trips
  // to LDS and not two per row.  A row that lies in the tile whole is stored; of a row that began before,
  // the part in this tile is the tile's head; of the tile's last row, when it goes on, the part in this
  // tile is the tile's tail.
  const unsigned ql = threadIdx.x & 3u;
  constexpr int kRowsAtOnce = 4, kRowAhead = 6;
  constexpr unsigned kRowsPerStep = kSegRowsBlock / 4;
  for (unsigned r0 = r_first; r0 < row_hi; r0 += kRowsPerStep * kRowsAtOnce) {  // the same for the whole workgroup
    unsigned lo[kRowsAtOnce], hi[kRowsAtOnce];
#pragma unroll
    for (int m = 0; m < kRowsAtOnce; ++m) {
      const unsigned r = r0 + m * kRowsPerStep + threadIdx.x / 4u, i = r - r_first;
      lo[m] = hi[m] = 0u;
      if (r < row_hi) {
        lo[m] = i < staged ? row_at[i] : start[r];
        hi[m] = i < staged ? row_at[i + 1u] : start[r + 1u];
      }
    }
    T first_terms[kRowsAtOnce][kRowAhead];
#pragma unroll
    for (int m = 0; m < kRowsAtOnce; ++m) {
      const unsigned from = max(lo[m], t_lo), to = min(hi[m], t_hi);
#pragma unroll
      for (int j = 0; j < kRowAhead; ++j) {
        const unsigned k = from + ql + 4u * j;
        first_terms[m][j] = k < to ? term[k - t_lo] : Op::identity();
      }
    }
#pragma unroll
    for (int m = 0; m < kRowsAtOnce; ++m) {
      const unsigned r = r0 + m * kRowsPerStep + threadIdx.x / 4u;
      const unsigned from = max(lo[m], t_lo), to = min(hi[m], t_hi);
      T acc = Op::identity();
#pragma unroll
      for (int j = 0; j < kRowAhead; ++j) acc = Op::apply(acc, first_terms[m][j]);
      for (unsigned k = from + ql + 4u * kRowAhead; k < to; k += 4u) acc = Op::apply(acc, term[k - t_lo]);
      acc = Op::apply(acc, dpp_move<0xB1>(Op::identity(), acc));    // quad_perm [1,0,3,2]
      acc = Op::apply(acc, dpp_move<0x4E>(Op::identity(), acc));    // quad_perm [2,3,0,1]
      if (r < row_hi && ql == 0u) {
        if (lo[m] < t_lo) head[tile] = acc;
        else if (hi[m] > t_hi) tail[tile] = acc;
        else y[r] = acc;
      }
    }
  }
}

template <class Op>
__global__ __launch_bounds__(kBlock) void seg_join_kernel(const KArgs a, const unsigned *first_row, const typename Op::T *head,
                                                          const typename Op::T *tail, unsigned tiles) {
  using T = typename Op::T;
  const unsigned *start = reinterpret_cast<const unsigned *>(a.in[kMaxIn - 1]);
  T *y = static_cast<T *>(a.out[0]);
  const unsigned n = (unsigned)a.n;
  const unsigned t = blockIdx.x * kBlock + threadIdx.x;
  if (t + 1u >= tiles) return;                                // the last tile's rows end with the array
  const unsigned row_lo = first_row[t], row_hi = first_row[t + 1u];
  if (row_hi == row_lo) return;                               // no row starts in this tile
  const unsigned r = row_hi - 1u, end = start[r + 1u];
  if (end <= (t + 1u) * kSegTile) return;                     // its last row ends in it
  T s = tail[t];
  for (unsigned t2 = t + 1u; t2 < tiles; ++t2) {
    s = Op::apply(s, head[t2]);
    if (end <= min((t2 + 1u) * (unsigned)kSegTile, n)) break;
  }
  y[r] = s;
}

// ------------------------------------------------------------------ single-pass scan / compaction
// Exclusive (+) scan of the int32 stream EX in one pass over the data (section
// 2: a scan inside a cluster must be a single pass; the chained scan is one of
// the implementations named there).  Tile t is processed by workgroup t.
//
// Cross-tile step.  A classic decoupled look-back chains tiles through their
// inclusive prefixes: the front of known prefixes advances one look-back window
// per memory round trip, and on this chip that chain, not bandwidth, set the
// pace.  Here no tile ever waits for a prefix.  Every tile publishes its
// aggregate as soon as its data is reduced; tiles form groups of kScanGroup; the
// last tile of a group sums the group's aggregates and publishes the group total;
// a tile's exclusive prefix is the sum of the totals of all earlier groups plus
// the aggregates of the earlier tiles of its own group -- all of which depend on
// aggregates only, so the wait is a constant number of round trips wherever the
// tile sits.  Workgroups are dispatched in index order, so every word a tile
// waits for belongs to a tile that is already running; every wait is bounded all
// the same.  The scan result never reaches memory unless asked for: kOffs stores
// it, kScatter writes EV(i) to dest[offs[i]] where EX(i) != 0 (scatter with
// collision-free indices: plain stores, no atomics), kCount stores the total.
constexpr int kScanBlock = 512;                       // threads per workgroup of the scan kernels
constexpr int kScanWaves = kScanBlock / kWave;
constexpr int kScanItems = 24;                        // per lane: six 128-bit accesses (measured best of 16..32)
constexpr int kScanAcc = kScanItems / kVec;
constexpr int kScanTile = kScanBlock * kScanItems;    // 12288 elements
constexpr int kScanGroup = 256;                       // tiles per group
constexpr int kOffs = 1, kScatter = 2, kCount = 4;
constexpr int kStoreX = 8;                            // the scanned stream is a result too: stored to out[3] (diagonal fusion)
// A compaction (the scanned stream is a 0/1 predicate, the kept elements are
// scattered, the offsets are not stored) parks the kept elements of a tile in
// LDS (see scan_kernel); the other forms hold the tile in registers across the
// wait.  The LDS buffer takes half a tile; a tile that keeps more uses registers.
template <class EX, int Mode> struct ScanParks {
  static constexpr bool value = (Mode & kScatter) != 0 && (Mode & kOffs) == 0 && YieldsZeroOne<EX>::value;
  static constexpr int cap = value ? kScanTile / 2 : 1;
};

// number of status words a launch over n_tiles tiles uses (tile words, then group words)
__host__ __device__ inline size_t scan_status_words(size_t n_tiles) {
  return ((n_tiles + 15) / 16) * 16 + (n_tiles + kScanGroup - 1) / kScanGroup;
}

// sum over the workgroup of an int held by every thread; all threads receive it
__device__ __forceinline__ int scan_block_sum(int v, int *lds) {
  int w = wave_reduce<AddI32>(v);
  __syncthreads();
  if (lane_id() == 0) lds[wave_id()] = w;
  __syncthreads();
  int r = 0;
#pragma unroll
  for (int k = 0; k < kScanWaves; ++k) r += lds[k];
  return r;
}

// Is the scanned stream a unary map of the scattered value stream (compaction by a
// predicate on the element itself)?  Then the flags are computed from the values
// already loaded instead of reading the array a second time.
template <class EX, class EV> struct FlagOfValue {
  static constexpr bool value = false;
  static __device__ __forceinline__ int apply(const KArgs &, typename EV::R) { return 0; }
};
template <class F, class EV> struct FlagOfValue<Map<F, EV>, EV> {
  static constexpr bool value = true;
  static __device__ __forceinline__ int apply(const KArgs &a, typename EV::R v) { return F::apply(a.p[0], v); }
};

// Two tagged words (16-byte aligned) in one 128-bit read at agent scope: a read marked sc1
// does not take a line from this XCD's L2, which may hold the words of an earlier launch, but
// goes where the agent-scope stores of the other workgroups went.  Each 64-bit word was written
// by one store and is validated by its own tag, so the two need not be read atomically together.
using TaggedPair = unsigned long long __attribute__((ext_vector_type(2)));
// `base` is the same for the whole wave (it becomes a buffer descriptor), `k` is the lane's word.
__device__ __forceinline__ TaggedPair load_tagged_pair(const unsigned long long *base, unsigned k) {
  using Raw = int __attribute__((ext_vector_type(4)));
  constexpr int kAgentScope = 0x10;                 // cache policy of the buffer load: sc1
  const __amdgpu_buffer_rsrc_t words =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned long long *>(base), 0, 0x7fffffff, 0x00020000);
  const Raw r = __builtin_amdgcn_raw_buffer_load_b128(words, (int)(k * 8u), 0, kAgentScope);
  return __builtin_bit_cast(TaggedPair, r);
}

// Sum of the values of `count` tagged words starting at p (16-byte aligned), this
// thread's share.  Words are written once per launch, so a word that carries the
// launch's tag is final: the fast path reads pairs of words with wide agent-scope
// loads, coalesced over the lanes; a word that does not validate (not yet
// published) is polled until it does.
template <int Threads = kScanBlock, class T = int>
__device__ __forceinline__ T sum_tagged_words(const unsigned long long *p, unsigned count, unsigned tag,
                                              Control *ctl) {
  using Pair = TaggedPair;
  T sum = T();
  for (unsigned k = 2 * (threadIdx.x % Threads); k < count; k += 2 * Threads) {
    Pair w = load_tagged_pair(p, k);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (k + j >= count) break;
      unsigned long long v = j ? w.y : w.x;
      unsigned lo = (unsigned)v;
      if ((lo >> 2) != tag || (lo & 3u) == 0u) v = wait_word(p + k + j, tag, ctl);
      sum += from_bits<T>((int)(unsigned)(v >> 32));
    }
  }
  return sum;
}

// The same sum with the reads split from their use: the constructor issues this
// thread's first Pairs reads of the range, sum() validates
// them and goes on with sum_tagged_words for whatever lies beyond.  Two ranges
// constructed back to back have their reads in flight together.
template <int Threads, int Pairs>
struct TaggedPairs {
  using Pair = TaggedPair;
  const unsigned long long *p;
  unsigned count;
  Pair w[Pairs];
  __device__ __forceinline__ TaggedPairs(const unsigned long long *p_, unsigned count_) : p(p_), count(count_) {
#pragma unroll
    for (int u = 0; u < Pairs; ++u) {
      const unsigned k = 2 * (threadIdx.x % Threads) + u * 2 * Threads;
      w[u] = Pair{0ull, 0ull};
      if (k < count) w[u] = load_tagged_pair(p, k);
    }
  }
  __device__ __forceinline__ int sum(unsigned tag, Control *ctl) const {
    int s = 0;
#pragma unroll
    for (int u = 0; u < Pairs; ++u) {
      const unsigned k = 2 * (threadIdx.x % Threads) + u * 2 * Threads;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (k + j >= count) break;
        unsigned long long v = j ? w[u].y : w[u].x;
        const unsigned lo = (unsigned)v;
        if ((lo >> 2) != tag || (lo & 3u) == 0u) v = wait_word(p + k + j, tag, ctl);
        s += (int)(unsigned)(v >> 32);
      }
    }
    const unsigned done = Pairs * 2 * Threads;
    if (count > done) s += sum_tagged_words<Threads>(p + done, count - done, tag, ctl);
    return s;
  }
};

// What a lane holds of one tile between loading it and writing its results.
// Registers bound how many tiles are in flight, and tiles in flight bound
// bandwidth, so a scanned stream of zeros and ones (a predicate) is kept as one
// bit per element -- a single register for the 24 elements of a lane.
template <class EX, class EV, int Mode, bool Reverse>
struct ScanPayload {
  using V = typename EV::R;
  static constexpr bool kScat = (Mode & kScatter) != 0;
  static constexpr bool kBits = YieldsZeroOne<EX>::value;
  static_assert(kScanItems <= 32, "one bit per element in a 32-bit register");
  int x[kBits ? 1 : kScanAcc][4];
  unsigned bits;
  V val[kScat ? kScanAcc : 1][4];

  // element c of access j of the scanned stream; positions past the end of the array read 0
  __device__ __forceinline__ int flag(int j, int c) const {
    return kBits ? (int)((bits >> (j * 4 + c)) & 1u) : x[kBits ? 0 : j][c];
  }
  __device__ __forceinline__ void set(int j, int c, int v) {
    if (kBits) bits |= (unsigned)(v != 0) << (j * 4 + c); else x[kBits ? 0 : j][c] = v;
  }
  // wave-striped layout: a wave owns kWave * kScanItems consecutive elements; access j
  // of a lane covers elements base + j*256 + lane*4 .. +3 (fully coalesced).
  // A tile that lies wholly inside the array takes a path without any
  // per-lane condition, so that its 128-bit reads are issued back to back and
  // are all in flight together; the last tile (and scanr of a length that is not a
  // multiple of four) takes the guarded path.
  __device__ __forceinline__ void load(const KArgs &a, unsigned tile, unsigned n) {
    const unsigned wbase = tile * kScanTile + wave_id() * (kWave * kScanItems);
    bits = 0u;
    if (!Reverse && (unsigned long long)(tile + 1) * kScanTile <= n) {
      if (kScat) {
#pragma unroll
        for (int j = 0; j < kScanAcc; ++j) {
          Vec4<V> u = EV::template eval4<EX::kNodes>(a, (int)(wbase + j * (kWave * kVec) + lane_id() * kVec));
#pragma unroll
          for (int c = 0; c < 4; ++c) val[kScat ? j : 0][c] = u.v[c];
        }
      }
      if (kScat && FlagOfValue<EX, EV>::value) {
#pragma unroll
        for (int j = 0; j < kScanAcc; ++j)
#pragma unroll
          for (int c = 0; c < 4; ++c) set(j, c, FlagOfValue<EX, EV>::apply(a, val[kScat ? j : 0][c]));
      } else {
        Vec4<int> v[kScanAcc];
#pragma unroll
        for (int j = 0; j < kScanAcc; ++j)
          v[j] = EX::template eval4<0>(a, (int)(wbase + j * (kWave * kVec) + lane_id() * kVec));
#pragma unroll
        for (int j = 0; j < kScanAcc; ++j)
#pragma unroll
          for (int c = 0; c < 4; ++c) set(j, c, v[j].v[c]);
      }
      return;
    }
    if (Reverse && !kScat && (n & 3u) == 0u && (unsigned long long)(tile + 1) * kScanTile <= n) {
      // scanr of a whole tile: the group at position i of the pass is elements n-4-i .. n-1-i
      // taken backwards, one 128-bit read when the length is a multiple of four
      Vec4<int> v[kScanAcc];
#pragma unroll
      for (int j = 0; j < kScanAcc; ++j)
        v[j] = EX::template eval4<0>(a, (int)(n - 4 - (wbase + j * (kWave * kVec) + lane_id() * kVec)));
#pragma unroll
      for (int j = 0; j < kScanAcc; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) set(j, c, v[j].v[3 - c]);
      return;
    }
#pragma unroll
    for (int j = 0; j < kScanAcc; ++j) {
      const unsigned i = wbase + j * (kWave * kVec) + lane_id() * kVec;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        // scanr walks the array from its end: position i + c of the pass is element n - 1 - (i + c)
        const int e = Reverse ? (int)(n - 1 - (i + c)) : (int)(i + c);
        const bool in = i + c < n;
        if (kScat) val[kScat ? j : 0][c] = in ? EV::template eval<EX::kNodes>(a, e) : V(0);
        if (kScat && FlagOfValue<EX, EV>::value)
          set(j, c, in ? FlagOfValue<EX, EV>::apply(a, val[kScat ? j : 0][c]) : 0);
        else
          set(j, c, in ? EX::template eval<0>(a, e) : 0);
      }
    }
  }
};

template <class EX, class EV, int Mode, bool Reverse>
__global__ __launch_bounds__(kScanBlock, 8) void scan_kernel(const KArgs a, Control *ctl, unsigned long long *status,
                                                             unsigned n_tiles) {
  __shared__ int lds_wave[kScanWaves];
  __shared__ int lds_sum[kScanWaves];
  using P = ScanPayload<EX, EV, Mode, Reverse>;
  using V = typename EV::R;
  constexpr bool kPark = ScanParks<EX, Mode>::value;
  constexpr int kParkCap = ScanParks<EX, Mode>::cap;
  __shared__ V parked[kParkCap];
  const unsigned n = (unsigned)a.n;
  const int lane = lane_id(), wave = wave_id();
  const unsigned epoch = epoch_at_start(ctl);
  const unsigned tag = tag_of_epoch(epoch);
  unsigned long long *group_word = status + ((n_tiles + 15) / 16) * 16;

  P cur;
  const unsigned tile = blockIdx.x;
  cur.load(a, tile, n);
  if (Mode & kStoreX) {
    // the scanned stream is stored as well as scanned: straight from the registers it was loaded into
    int *xs = static_cast<int *>(a.out[3]);
    const unsigned base = tile * kScanTile + wave * (kWave * kScanItems);
    const bool whole = (unsigned long long)(tile + 1) * kScanTile <= n && (!Reverse || (n & 3u) == 0u);
#pragma unroll
    for (int j = 0; j < kScanAcc; ++j) {
      const unsigned i = base + j * (kWave * kVec) + lane * kVec;
      const Vec4<int> v = {{cur.flag(j, 0), cur.flag(j, 1), cur.flag(j, 2), cur.flag(j, 3)}};
      if (whole) {
        if (Reverse) store4<true>(xs + (n - 4 - i), Vec4<int>{{v.v[3], v.v[2], v.v[1], v.v[0]}}); else store4<true>(xs + i, v);
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) if (i + c < n) xs[Reverse ? n - 1 - (i + c) : i + c] = v.v[c];
      }
    }
  }
  {
    const unsigned wbase = tile * kScanTile + wave * (kWave * kScanItems);
    int s[kScanAcc];
#pragma unroll
    for (int j = 0; j < kScanAcc; ++j) {
      int f[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) f[c] = cur.flag(j, c);
      s[j] = (f[0] + f[1]) + (f[2] + f[3]);
    }
    // exclusive prefix of each access inside the wave
    int excl[kScanAcc];
    int carry = 0;
#pragma unroll
    for (int j = 0; j < kScanAcc; ++j) {
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

    if (threadIdx.x == 0) store_agent64(&status[tile], pack_word((unsigned)aggregate, tag, 1u));
    const unsigned group = tile / kScanGroup, first = group * kScanGroup;
    const unsigned n_mine = tile - first;          // earlier tiles of my group

    if (kPark && aggregate <= kParkCap) {
      // Compaction.  Registers bound how many tiles are being loaded, and a tile
      // that sat in registers until its prefix arrived held them for about twice
      // the time its loads took.  So the kept elements are put into LDS in their
      // final order, seven of the eight waves end here and give their registers
      // and wave slots to the next tile, and one wave alone waits for the prefix
      // and copies the run to its place.  Every word it waits for is published by
      // a tile's loading phase, which waits for nothing.  Which wave stays rotates
      // with the tile, so that the waiting waves spread over the four SIMDs.
#pragma unroll
      for (int j = 0; j < kScanAcc; ++j) {
        int o = wave_excl + excl[j];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (cur.flag(j, c) != 0) parked[o++] = cur.val[P::kScat ? j : 0][c];
        }
      }
      __syncthreads();
      if (wave != (int)(tile % kScanWaves)) return;
      if (lane == 0 && tile > 0)
        (void)wait_word(n_mine > 0 ? &status[tile - 1] : &group_word[group - 1], tag, ctl);
      // the aggregates of the group's earlier tiles and the totals of the earlier groups
      // are independent reads: both are issued before either is looked at
      TaggedPairs<kWave, kScanGroup / (2 * kWave)> mine(status + first, n_mine);
      TaggedPairs<kWave, 1> before(group_word, group);
      int sum_group = wave_reduce<AddI32>(mine.sum(tag, ctl));
      if (n_mine == kScanGroup - 1 && lane == 0)
        store_agent64(&group_word[group], pack_word((unsigned)(sum_group + aggregate), tag, 1u));
      const int tile_excl = sum_group + wave_reduce<AddI32>(before.sum(tag, ctl));
      if (tile == n_tiles - 1 && lane == 0) {
        if (Mode & kCount) *static_cast<int *>(a.out[2]) = tile_excl + aggregate;
        store_agent(&ctl->epoch, epoch + 1u);
      }
      // copy the run to its place with 128-bit stores: single elements up to the first
      // 16-byte boundary of the destination, whole groups of four, single elements again
      V *dest = static_cast<V *>(a.out[0]) + tile_excl;
      const int head = min((int)((16u - (unsigned)(reinterpret_cast<size_t>(dest) & 15u)) & 15u) / (int)sizeof(V), aggregate);
      const int groups = (aggregate - head) / kVec;
      if (lane < head) dest[lane] = parked[lane];
      constexpr int kCopy = 4;
      for (int g0 = 0; g0 < groups; g0 += kCopy * kWave) {
        Vec4<V> v[kCopy];
#pragma unroll
        for (int u = 0; u < kCopy; ++u) {
          const int k = head + min(g0 + u * kWave + lane, groups - 1) * kVec;
#pragma unroll
          for (int c = 0; c < 4; ++c) v[u].v[c] = parked[k + c];
        }
#pragma unroll
        for (int u = 0; u < kCopy; ++u) {
          const int g = g0 + u * kWave + lane;
          if (g < groups) store4<false>(dest + head + g * kVec, v[u]);
        }
      }
      const int tail = head + groups * kVec;
      if (tail + lane < aggregate) dest[tail + lane] = parked[tail + lane];
      return;
    }
    // Gate: one lane waits for the word that is published last among those this tile
    // needs (its immediate predecessor's, or the previous group's total).  Words
    // become valid nearly in tile order, so after the gate the wide reads below
    // succeed at once; hundreds of lanes spinning on fresh words would flood the
    // few memory channels that hold them and slow every stream of the kernel.
    if (threadIdx.x == 0 && tile > 0)
      (void)wait_word(n_mine > 0 ? &status[tile - 1] : &group_word[group - 1], tag, ctl);
    __syncthreads();
    // aggregates of the earlier tiles of my group
    int sum_group = sum_tagged_words(status + first, n_mine, tag, ctl);
    if (n_mine == kScanGroup - 1) {
      // last tile of a full group: publish the group total before waiting for anything else
      sum_group = scan_block_sum(sum_group, lds_sum);
      if (threadIdx.x == 0) store_agent64(&group_word[group], pack_word((unsigned)(sum_group + aggregate), tag, 1u));
      if (threadIdx.x != 0) sum_group = 0;         // counted once in the sum below
    }
    // totals of all earlier groups
    int sum_before = sum_group + sum_tagged_words(group_word, group, tag, ctl);
    const int tile_excl = scan_block_sum(sum_before, lds_sum);

    if (tile == n_tiles - 1 && threadIdx.x == 0) {
      if (Mode & kCount) *static_cast<int *>(a.out[2]) = tile_excl + aggregate;
      // the last tile has read a word of every other tile or of its group, so all of
      // them have taken their tag: the next launch may use the next one
      store_agent(&ctl->epoch, epoch + 1u);
    }

#pragma unroll
    for (int j = 0; j < kScanAcc; ++j) {
      unsigned i = wbase + j * (kWave * kVec) + lane * kVec;
      int f[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) f[c] = cur.flag(j, c);
      int o[4];
      o[0] = tile_excl + wave_excl + excl[j];
      o[1] = o[0] + f[0];
      o[2] = o[1] + f[1];
      o[3] = o[2] + f[2];
      if (Mode & kOffs) {
        int *offs = static_cast<int *>(a.out[1]);
        if (!Reverse && i + 3 < n) {
          store4<true>(offs + i, Vec4<int>{{o[0], o[1], o[2], o[3]}});
        } else if (Reverse && (n & 3u) == 0u && i + 3 < n) {
          store4<true>(offs + (n - 4 - i), Vec4<int>{{o[3], o[2], o[1], o[0]}});
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) if (i + c < n) offs[Reverse ? n - 1 - (i + c) : i + c] = o[c];
        }
      }
      if (Mode & kScatter) {
        V *dest = static_cast<V *>(a.out[0]);
#pragma unroll
        for (int c = 0; c < 4; ++c) if (f[c] != 0) dest[o[c]] = cur.val[P::kScat ? j : 0][c];
      }
    }
  }
}

// ------------------------------------------------------------------ single-pass scan of an fp32 stream
// Exclusive (+) scan of the fp32 stream EX, stored; the same cross-tile scheme as
// scan_kernel (aggregates and group totals as tagged words, no tile waits for a
// prefix), the values travelling as their bit patterns.  The sums are taken in a
// fixed order (four elements of a 128-bit group, the lanes of a wave, the waves of
// a tile, the tiles of a group, the groups), so a launch gives the same bits every
// time; the order is not the sequential one, so a prefix differs from the
// sequential fp32 sum by rounding, within the bound of any summation order.
constexpr int kScanFItems = 16;                       // per lane: four 128-bit accesses
constexpr int kScanFAcc = kScanFItems / kVec;
constexpr int kScanFTile = kScanBlock * kScanFItems;  // 8192 elements

__device__ __forceinline__ float scan_block_sum_f32(float v, float *lds) {
  float w = wave_reduce<AddF32>(v);
  __syncthreads();
  if (lane_id() == 0) lds[wave_id()] = w;
  __syncthreads();
  float r = 0.0f;
#pragma unroll
  for (int k = 0; k < kScanWaves; ++k) r += lds[k];
  return r;
}

template <class EX, bool Reverse, bool StoreX = false>
__global__ __launch_bounds__(kScanBlock) void scan_f32_kernel(const KArgs a, Control *ctl, unsigned long long *status,
                                                              unsigned n_tiles) {
  static_assert(std::is_same<typename EX::R, float>::value, "fp32 stream");
  __shared__ float lds_wave[kScanWaves];
  __shared__ float lds_sum[kScanWaves];
  const unsigned n = (unsigned)a.n;
  const int lane = lane_id(), wave = wave_id();
  const unsigned epoch = epoch_at_start(ctl);
  const unsigned tag = tag_of_epoch(epoch);
  unsigned long long *group_word = status + ((n_tiles + 15) / 16) * 16;
  float *offs = static_cast<float *>(a.out[1]);
  const unsigned tile = blockIdx.x;
  const unsigned wbase = tile * kScanFTile + wave * (kWave * kScanFItems);
  // position i of the pass is element i, for scanr element n - 1 - i; positions past the end read 0
  // a whole tile is read and written in 128-bit groups; for scanr the group at position i is
  // elements n-4-i .. n-1-i taken backwards, which is a group only if n is a multiple of four
  const bool whole = (size_t)(tile + 1) * kScanFTile <= n && (!Reverse || (n & 3u) == 0u);
  float x[kScanFAcc][kVec];
  if (whole) {
#pragma unroll
    for (int j = 0; j < kScanFAcc; ++j) {
      const unsigned i = wbase + j * (kWave * kVec) + lane * kVec;
      const Vec4<float> v = EX::template eval4<0>(a, (int)(Reverse ? n - 4 - i : i));
#pragma unroll
      for (int c = 0; c < kVec; ++c) x[j][c] = v.v[Reverse ? 3 - c : c];
    }
  } else {
#pragma unroll
    for (int j = 0; j < kScanFAcc; ++j)
#pragma unroll
      for (int c = 0; c < kVec; ++c) {
        const unsigned i = wbase + j * (kWave * kVec) + lane * kVec + c;
        x[j][c] = i < n ? EX::template eval<0>(a, (int)(Reverse ? n - 1 - i : i)) : 0.0f;
      }
  }
  if (StoreX) {
    // the scanned array is a result as well: stored from the registers it was loaded into
    float *xs = static_cast<float *>(a.out[3]);
#pragma unroll
    for (int j = 0; j < kScanFAcc; ++j) {
      const unsigned i = wbase + j * (kWave * kVec) + lane * kVec;
      if (whole) {
        if (Reverse)
          store4<true>(xs + (n - 4 - i), Vec4<float>{{x[j][3], x[j][2], x[j][1], x[j][0]}});
        else
          store4<true>(xs + i, Vec4<float>{{x[j][0], x[j][1], x[j][2], x[j][3]}});
      } else {
#pragma unroll
        for (int c = 0; c < kVec; ++c)
          if (i + c < n) xs[Reverse ? n - 1 - (i + c) : i + c] = x[j][c];
      }
    }
  }
  // exclusive prefix of each access inside the wave
  float excl[kScanFAcc];
  float carry = 0.0f;
#pragma unroll
  for (int j = 0; j < kScanFAcc; ++j) {
    const float s = (x[j][0] + x[j][1]) + (x[j][2] + x[j][3]);
    const float inc = wave_scan_inclusive<AddF32>(s);
    excl[j] = carry + lane_prev(0.0f, inc);
    carry += from_bits<float>(__builtin_amdgcn_readlane(as_bits(inc), kWave - 1));
  }
  if (lane == 0) lds_wave[wave] = carry;
  __syncthreads();
  float wave_excl = 0.0f, aggregate = 0.0f;
#pragma unroll
  for (int k = 0; k < kScanWaves; ++k) {
    const float t = lds_wave[k];
    if (k < wave) wave_excl += t;
    aggregate += t;
  }
  if (threadIdx.x == 0) store_agent64(&status[tile], pack_word((unsigned)as_bits(aggregate), tag, 1u));
  const unsigned group = tile / kScanGroup, first = group * kScanGroup;
  const unsigned n_mine = tile - first;            // earlier tiles of my group
  // gate: one lane waits for the word that is published last among those this tile needs
  if (threadIdx.x == 0 && tile > 0)
    (void)wait_word(n_mine > 0 ? &status[tile - 1] : &group_word[group - 1], tag, ctl);
  __syncthreads();
  float sum_group = sum_tagged_words<kScanBlock, float>(status + first, n_mine, tag, ctl);
  if (n_mine == kScanGroup - 1) {
    // last tile of a full group: publish the group total before waiting for anything else
    sum_group = scan_block_sum_f32(sum_group, lds_sum);
    if (threadIdx.x == 0) store_agent64(&group_word[group], pack_word((unsigned)as_bits(sum_group + aggregate), tag, 1u));
    if (threadIdx.x != 0) sum_group = 0.0f;        // counted once in the sum below
  }
  const float sum_before = sum_group + sum_tagged_words<kScanBlock, float>(group_word, group, tag, ctl);
  const float tile_excl = scan_block_sum_f32(sum_before, lds_sum);
  if (tile == n_tiles - 1 && threadIdx.x == 0) store_agent(&ctl->epoch, epoch + 1u);
#pragma unroll
  for (int j = 0; j < kScanFAcc; ++j) {
    const unsigned i = wbase + j * (kWave * kVec) + lane * kVec;
    Vec4<float> o;
    o.v[0] = tile_excl + (wave_excl + excl[j]);
    o.v[1] = o.v[0] + x[j][0];
    o.v[2] = o.v[1] + x[j][1];
    o.v[3] = o.v[2] + x[j][2];
    if (whole) {
      if (Reverse)
        store4<true>(offs + (n - 4 - i), Vec4<float>{{o.v[3], o.v[2], o.v[1], o.v[0]}});
      else
        store4<true>(offs + i, o);
    } else {
#pragma unroll
      for (int c = 0; c < kVec; ++c)
        if (i + c < n) offs[Reverse ? n - 1 - (i + c) : i + c] = o.v[c];
    }
  }
}

// ------------------------------------------------------------------ row scans
// scanl / scanr of a two-dimensional array scan every row on its own (section 2:
// in a multidimensional array the scan is performed over each row).  A row is one
// pass: L lanes walk it in steps of L elements, a carry links the steps, rows are
// independent.  L is a 16-lane DPP row, a wave, or the workgroup, by row length.
// out[1] receives the exclusive prefix sums; scanr is the same pass from the right.
template <class E, bool Reverse, int L, bool StoreX = false>
__global__ __launch_bounds__(kBlock) void rowscan_kernel(const KArgs a) {
  static_assert(L == 16 || L == kWave || L == kBlock, "lanes per row");
  using T = typename E::R;
  using Op = typename std::conditional<std::is_same<T, float>::value, AddF32, AddI32>::type;
  constexpr int kRows = kBlock / L;                     // rows a workgroup handles at a time
  __shared__ T lds[kWavesPerBlock];
  T *out = static_cast<T *>(a.out[1]);
  // unsigned throughout: the steps past the last row and past a row's end must not wrap
  const unsigned rows = (unsigned)a.aux, w = (unsigned)a.w;
  const unsigned sub = threadIdx.x % L, which = threadIdx.x / L;
  for (unsigned r0 = blockIdx.x * kRows; r0 < rows; r0 += gridDim.x * kRows) {
    const unsigned r = r0 + which;
    T carry = T();
    // every lane runs the same number of steps, so DPP and the barriers stay converged
    for (unsigned c0 = 0; c0 < w; c0 += L) {
      const unsigned c = c0 + sub;
      const bool live = r < rows && c < w;
      const int e = live ? (int)(r * w + (Reverse ? w - 1 - c : c)) : 0;
      const T x = live ? E::template eval<0>(a, e) : T();
      if (StoreX && live) static_cast<T *>(a.out[3])[e] = x;      // the scanned array is a result as well
      // inclusive prefix over the L lanes, the exclusive one by moving it one lane on (a
      // floating-point sum cannot give its last term back), and the step's total
      T inc, exc, total;
      if (L == 16) {
        inc = row_scan_inclusive<Op>(x);
        exc = dpp_move<kRowShr1>(T(), inc);
        total = __shfl(inc, 15, 16);
      } else if (L == kWave) {
        inc = wave_scan_inclusive<Op>(x);
        exc = lane_prev(T(), inc);
        total = from_bits<T>(__builtin_amdgcn_readlane(as_bits(inc), kWave - 1));
      } else {
        inc = wave_scan_inclusive<Op>(x);
        exc = lane_prev(T(), inc);
        __syncthreads();                                  // lds of the previous step has been read
        if (lane_id() == kWave - 1) lds[wave_id()] = inc;
        __syncthreads();
        T before = T();
        total = T();
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) {
          const T t = lds[k];
          if (k < wave_id()) before += t;
          total += t;
        }
        exc = before + exc;
      }
      if (live) out[e] = carry + exc;
      carry += total;
    }
  }
}

// ------------------------------------------------------------------ scatter (elementwise)
// for every i with EF(i) != 0: dest[EI(i)] = f(dest[EI(i)], EV(i)).  Overwrite: the
// indices are taken to be distinct, so plain stores suffice (no atomics).  Add:
// colliding indices combine with hardware atomics.  Integer sums are exact in any
// order.  fp32 sums depend on the order of the updates, which nothing fixes
// (section 2, scatter: no guarantee on the order when the operator is not
// associative and commutative); every single addition is correctly rounded.
template <bool Add, class T> __device__ __forceinline__ void scatter_one(T *dest, int j, T v) {
  if (Add) atomicAdd(dest + j, v); else dest[j] = v;
}
template <> __device__ __forceinline__ void scatter_one<true, float>(float *dest, int j, float v) {
  unsafeAtomicAdd(dest + j, v);      // the hardware's fp32 add, not a compare-and-swap loop
}

template <class EI, class EV, class EF, bool Add>
__global__ __launch_bounds__(kBlock) void scatter_kernel(const KArgs a) {
  using V = typename EV::R;
  struct Item { Vec4<int> f, j; Vec4<V> v; };
  V *dest = static_cast<V *>(a.out[0]);
  const unsigned n = (unsigned)a.n, n4 = n & ~3u;
  for_each_group(
      n4,
      [&](unsigned i) {
        return Item{EF::template eval4<EI::kNodes + EV::kNodes>(a, (int)i), EI::template eval4<0>(a, (int)i),
                    EV::template eval4<EI::kNodes>(a, (int)i)};
      },
      [&](unsigned, const Item &t) {
#pragma unroll
        for (int c = 0; c < 4; ++c) if (t.f.v[c] != 0) scatter_one<Add>(dest, t.j.v[c], t.v.v[c]);
      });
  if (blockIdx.x == 0 && threadIdx.x < n - n4) {
    int i = (int)(n4 + threadIdx.x);
    if (EF::template eval<EI::kNodes + EV::kNodes>(a, i) != 0)
      scatter_one<Add>(dest, EI::template eval<0>(a, i), EV::template eval<EI::kNodes>(a, i));
  }
}

// ------------------------------------------------------------------ row folds
// y[i] = fold(Op, E(row(i) * m + j) for j < m): fold over the innermost dimension
// of a 2-D iteration space (section 2, fold).  row(i) = i, or RI(i) when a gather
// consumes the fold inside the cluster: the gather picks the row and the fold
// loops over it (section 3.3, `simple4`).  A second reducer folds the same
// element program in the same pass (two folds sharing a contracted producer,
// section 5, `greedyBottomUpBad`).  L lanes cooperate on a row.
struct NoRowIndex {
  static constexpr int kNodes = 0;
  template <int Base> static __device__ __forceinline__ int eval(const KArgs &, int i) { return i; }
  static void sig(std::string &) {}
};
struct NoSecondOp {
  using T = float;
  static __device__ __forceinline__ T identity() { return 0.0f; }
  static __device__ __forceinline__ T apply(T a, T) { return a; }
  static const char *name() { return ""; }
};

template <class Op1, class Op2, class E, class RI, int L>
__global__ __launch_bounds__(kBlock) void rowfold_kernel(const KArgs a) {
  using T = typename Op1::T;
  constexpr bool kTwo = !std::is_same<Op2, NoSecondOp>::value;
  __shared__ T lds1[kWavesPerBlock + 1];
  __shared__ typename Op2::T lds2[kWavesPerBlock + 1];
  const unsigned rows = (unsigned)a.aux, m = (unsigned)a.w;
  constexpr unsigned kRowsPerBlock = kBlock / L;
  const unsigned sub = threadIdx.x % L;
  const unsigned steps = (rows + gridDim.x * kRowsPerBlock - 1) / (gridDim.x * kRowsPerBlock);
  for (unsigned s = 0; s < steps; ++s) {          // same trip count for every thread: barriers and DPP stay converged
    const unsigned r = (s * gridDim.x + blockIdx.x) * kRowsPerBlock + threadIdx.x / L;
    T acc1 = Op1::identity();
    typename Op2::T acc2 = Op2::identity();
    if (r < rows) {
      const unsigned base = (unsigned)RI::template eval<E::kNodes>(a, (int)r) * m;
      if ((m & 3u) == 0) {
        for (unsigned j = sub * 4; j < m; j += L * 4) {
          Vec4<T> v = E::template eval4<0>(a, (int)(base + j));
#pragma unroll
          for (int c = 0; c < 4; ++c) { acc1 = Op1::apply(acc1, v.v[c]); if (kTwo) acc2 = Op2::apply(acc2, v.v[c]); }
        }
      } else {
        for (unsigned j = sub; j < m; j += L) {
          T v = E::template eval<0>(a, (int)(base + j));
          acc1 = Op1::apply(acc1, v);
          if (kTwo) acc2 = Op2::apply(acc2, v);
        }
      }
    }
    if (L == 16) {
      acc1 = row_scan_inclusive<Op1>(acc1);
      if (kTwo) acc2 = row_scan_inclusive<Op2>(acc2);
    } else if (L == kWave) {
      acc1 = wave_scan_inclusive<Op1>(acc1);
      if (kTwo) acc2 = wave_scan_inclusive<Op2>(acc2);
    } else {
      acc1 = block_reduce<Op1>(acc1, lds1);
      if (kTwo) acc2 = block_reduce<Op2>(acc2, lds2);
    }
    if (sub == L - 1 && r < rows) {
      static_cast<T *>(a.out[0])[r] = acc1;
      if (kTwo) static_cast<typename Op2::T *>(a.out[1])[r] = acc2;
    }
  }
}

// Few long rows: a row is cut into `splits` chunks, one workgroup each, so that the
// whole chip works on it.  Chunk results are published as tagged words; the
// workgroup of a row's last chunk waits for the row's other chunks and combines
// them in chunk order.  The very last workgroup waits for every chunk of the
// launch before it advances the epoch.
template <class Op1, class Op2, class E, class RI>
__global__ __launch_bounds__(kBlock) void rowfold_split_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                               unsigned splits, unsigned chunk_len) {
  using T = typename Op1::T;
  using U = typename Op2::T;
  constexpr bool kTwo = !std::is_same<Op2, NoSecondOp>::value;
  __shared__ T lds1[kWavesPerBlock + 1];
  __shared__ U lds2[kWavesPerBlock + 1];
  const unsigned m = (unsigned)a.w;
  const unsigned r = blockIdx.x / splits, chunk = blockIdx.x % splits;
  const unsigned epoch = load_agent(&ctl->epoch);
  const unsigned tag = tag_of_epoch(epoch);
  unsigned long long *second = partials + kMaxPartials / 2;
  const unsigned base = (unsigned)RI::template eval<E::kNodes>(a, (int)r) * m;
  const unsigned lo = chunk * chunk_len, hi = min(m, lo + chunk_len);
  T acc1 = Op1::identity();
  U acc2 = Op2::identity();
  if ((m & 3u) == 0) {
    for (unsigned j = lo + threadIdx.x * 4; j < hi; j += kBlock * 4) {
      Vec4<T> v = E::template eval4<0>(a, (int)(base + j));
#pragma unroll
      for (int c = 0; c < 4; ++c) { acc1 = Op1::apply(acc1, v.v[c]); if (kTwo) acc2 = Op2::apply(acc2, v.v[c]); }
    }
  } else {
    for (unsigned j = lo + threadIdx.x; j < hi; j += kBlock) {
      T v = E::template eval<0>(a, (int)(base + j));
      acc1 = Op1::apply(acc1, v);
      if (kTwo) acc2 = Op2::apply(acc2, v);
    }
  }
  acc1 = block_reduce<Op1>(acc1, lds1);
  if (kTwo) acc2 = block_reduce<Op2>(acc2, lds2);
  if (threadIdx.x == 0) {
    store_agent64(&partials[blockIdx.x], pack_word((unsigned)as_bits(acc1), tag, 1u));
    if (kTwo) store_agent64(&second[blockIdx.x], pack_word((unsigned)as_bits(acc2), tag, 1u));
  }
  if (chunk == splits - 1 && threadIdx.x == 0) {
    T s1 = Op1::identity();
    U s2 = Op2::identity();
    for (unsigned k = 0; k < splits; ++k) {
      unsigned long long w = wait_word(&partials[r * splits + k], tag, ctl);
      s1 = Op1::apply(s1, w ? from_bits<T>((int)(unsigned)(w >> 32)) : Op1::identity());
      if (kTwo) {
        unsigned long long w2 = wait_word(&second[r * splits + k], tag, ctl);
        s2 = Op2::apply(s2, w2 ? from_bits<U>((int)(unsigned)(w2 >> 32)) : Op2::identity());
      }
    }
    static_cast<T *>(a.out[0])[r] = s1;
    if (kTwo) static_cast<U *>(a.out[1])[r] = s2;
  }
  if (blockIdx.x == gridDim.x - 1) {
    // every workgroup has taken its tag once its word is visible
    for (unsigned k = threadIdx.x; k < gridDim.x; k += kBlock) (void)wait_word(&partials[k], tag, ctl);
    __syncthreads();
    if (threadIdx.x == 0) store_agent(&ctl->epoch, epoch + 1u);
  }
}

}  // namespace fc
