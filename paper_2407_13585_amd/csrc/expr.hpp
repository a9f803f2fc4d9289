// Element-level programs of a fused cluster as expression types.
//
// A cluster's producers (map / zipWith, generate, gather; Table 1) form a tree
// that is evaluated in registers for one iteration index.  A gather pushes its
// index through the producers of its source (section 3.3, `simple1`,
// `simple2`): Gather<EI, ES> evaluates ES at the index EI yields, so a producer
// below a gather is recomputed at the gathered position and never stored.
//
// Every expression type offers
//   eval(args, i)     value at iteration index i
//   eval4(args, i)    values at i .. i+3 (i a multiple of 4), 128-bit loads on leaves
//   sig(std::string&) the textual signature the host matcher compares against
//   kNodes            number of combinator nodes in the tree (parameter slots)
//   kMirror           the tree reads an array through `reverse` as well (tile order, kernels.hpp)
//   eval4_pair(args, i, ip, at_i, at_ip)   values at the 128-bit groups i and ip, where ip is
//                     the mirror image of i (ip = n - 4 - i); see for_each_mirrored_pair
//   mirrors_whole(args, n)   every `reverse` of the tree runs over exactly n elements
// Parameter slots are numbered in pre-order, leaves included.
#pragma once

#include <hip/hip_runtime.h>

#include <string>
#include <tuple>
#include <utility>

#include "prim.hpp"

namespace fc {

constexpr int kMaxIn = 8;
constexpr int kMaxOut = 4;
constexpr int kMaxSlots = 24;

struct Slot {     // parameters of one combinator node
  float f[2];
  int i[2];       // the node's own integer parameters
  int ext[2];     // the node's own extents (outer, inner); inner is 1 for 1-D arrays
  unsigned m[3];  // constants the host derives from the parameters (mod_eq_constants, div_constants)
};

// x mod k == r for x >= 0 without a division.  With k = 2^s * d, d odd, and
// inv = d^-1 mod 2^32: t is a multiple of k exactly if rotr(t * inv, s) <= (2^32-1) / k
// (test for a zero remainder by multiplying with the inverse of the odd part);
// apply it to t = x - r, which needs x >= r.  A residue outside [0, k) matches no x.
inline void mod_eq_constants(Slot &s) {
  const unsigned k = (unsigned)s.i[0];
  if (s.i[0] <= 0 || s.i[1] < 0 || s.i[1] >= s.i[0]) {
    s.i[1] = (int)0x80000000u;                // no non-negative int32 reaches it
    s.m[0] = s.m[1] = s.m[2] = 0;
    return;
  }
  unsigned shift = 0, d = k;
  while ((d & 1u) == 0) { d >>= 1; ++shift; }
  unsigned inv = d;                            // Newton steps double the number of correct low bits (3 to start with)
  for (int it = 0; it < 5; ++it) inv *= 2u - d * inv;
  s.m[0] = inv;
  s.m[1] = shift;
  s.m[2] = 0xffffffffu / k;
}

// The element programs of a cluster once more, as code for the interpreting kernel
// (interp_kernel), which runs clusters that no compiled instance matches.  A stack
// machine in post-order: a value per array read, generated or computed, consumed by the
// map, store or fold above it; a gather evaluates its index, then its source with the
// index as the position (kCodeEnter / kCodeLeave).
constexpr int kMaxCode = 64;
constexpr int kMaxRoots = 4;          // element programs of one cluster that yield a value each
constexpr int kInterpDepth = 6;       // values below the top of the interpreter's stack
constexpr int kInterpGathers = 3;     // nesting of gathers it follows
enum : unsigned char {
  kCodeEnd = 0,
  kCodeIn,      // a = external array: push its element at the position
  kCodeGen,     // a = index function, b = slot: push its value at the position
  kCodeMap,     // a = element function, b = slot, c = number of arguments: replace them by the result
  kCodeEnter,   // pop an index and make it the position
  kCodeLeave,   // back to the position before the matching kCodeEnter
  kCodeStore,   // a = output array: pop a value into it at the element's own position
  kCodeFold,    // a = output array, b = reducer (kFold...), c = accumulator: pop a value into it
  kCodeYield,   // the value on the stack is the result of this element program (Interp<K, T>)
  kCodeDup      // push a copy of the top of the stack (an array with several consumers is computed once)
};
constexpr int kInterpFolds = 2;       // folds of one interpreted cluster
enum : unsigned char { kFoldAddF32 = 0, kFoldMaxF32, kFoldMulF32, kFoldAddI32, kFoldMaxI32 };
struct Code { unsigned char op, a, b, c; };

struct KArgs {    // arguments of one cluster launch
  const void *in[kMaxIn];   // external arrays read by the cluster
  void *out[kMaxOut];       // arrays the cluster writes
  int n;                    // iteration size
  int w;                    // inner extent of 2-D index functions (1 for 1-D)
  int h;                    // outer extent
  int aux;                  // skeleton specific (rows of a segmented fold, ...)
  Slot p[kMaxSlots];
  Code code[kMaxCode];      // kCodeEnd after the last instruction
  unsigned char root[kMaxRoots];   // where element program K of a cluster with another consumer starts in `code`
  unsigned flags;           // kSinglePass: a fold of the cluster carries FC_NODE_SINGLE_PASS;
                            // kKeepOut << k: out[k] is read back by a later cluster of the program
  __host__ __device__ bool keeps(int k) const { return (flags >> (8 + k)) & 1u; }
};
constexpr unsigned kSinglePass = 1u;
constexpr unsigned kKeepOut = 1u << 8;

template <class T> struct Vec4 { T v[4]; };

template <class T> struct DtypeName;
template <> struct DtypeName<float> { static const char *s() { return "f32"; } };
template <> struct DtypeName<int> { static const char *s() { return "i32"; } };

// ------------------------------------------------------------------ element functions
struct FnIdentF { using R = float; static constexpr int kFn = FC_FN_IDENT;
  static __device__ __forceinline__ R apply(const Slot &, float x) { return x; } };
struct FnIdentI { using R = int; static constexpr int kFn = FC_FN_IDENT;
  static __device__ __forceinline__ R apply(const Slot &, int x) { return x; } };
struct FnAffine { using R = float; static constexpr int kFn = FC_FN_AFFINE;
  static __device__ __forceinline__ R apply(const Slot &s, float x) { float t = s.f[0] * x; return t + s.f[1]; } };
struct FnSinXMulX { using R = float; static constexpr int kFn = FC_FN_SIN_X_MUL_X;
  static __device__ __forceinline__ R apply(const Slot &, float x) { return sinf(x) * x; } };
struct FnSqPlusOne { using R = float; static constexpr int kFn = FC_FN_SQ_PLUS_ONE;
  static __device__ __forceinline__ R apply(const Slot &, float x) { float t = x * x; return t + 1.0f; } };
struct FnMul2 { using R = float; static constexpr int kFn = FC_FN_MUL2;
  static __device__ __forceinline__ R apply(const Slot &, float a, float b) { return a * b; } };
struct FnAdd2 { using R = float; static constexpr int kFn = FC_FN_ADD2;
  static __device__ __forceinline__ R apply(const Slot &, float a, float b) { return a + b; } };
struct FnAdd3 { using R = float; static constexpr int kFn = FC_FN_ADD3;
  static __device__ __forceinline__ R apply(const Slot &, float a, float b, float c) { return (a + b) + c; } };
struct FnAdd5 { using R = float; static constexpr int kFn = FC_FN_ADD5;
  static __device__ __forceinline__ R apply(const Slot &, float a, float b, float c, float d, float e) {
    return (((a + b) + c) + d) + e; } };
struct FnExpNeg { using R = float; static constexpr int kFn = FC_FN_EXP_NEG;
  static __device__ __forceinline__ R apply(const Slot &, float x) { return expf(-x); } };
struct FnModEq { using R = int; static constexpr int kFn = FC_FN_MOD_EQ;
  static __device__ __forceinline__ R apply(const Slot &s, int x) {
    const unsigned t = (unsigned)x - (unsigned)s.i[1];
    const unsigned p = t * s.m[0];
    const unsigned q = __builtin_amdgcn_alignbit(p, p, s.m[1]);     // rotate right
    return (int)((unsigned)((unsigned)x >= (unsigned)s.i[1]) & (unsigned)(q <= s.m[2])); } };   // no branch: both tests always

// i / d for 0 <= i < 2^31 and a divisor that is fixed for the launch, without a
// division: with L = ceil(log2 d) and M = ceil(2^(31+L) / d) < 2^32 the quotient is
// (i * M) >> (31 + L) (division by an invariant integer through multiplication).
// The index functions divide every element index by a row length; the compiler
// turns a division by a run-time value into some forty instructions.
inline void div_constants(Slot &s, int d) {
  unsigned L = 0;
  while ((1ull << L) < (unsigned long long)(d > 0 ? d : 1)) ++L;
  const unsigned long long two = 1ull << (31 + L), dd = (unsigned long long)(d > 0 ? d : 1);
  s.m[0] = (unsigned)((two + dd - 1) / dd);
  s.m[1] = 31 + L;
}
__device__ __forceinline__ int fast_div(const Slot &s, int i) {
  return (int)(((unsigned long long)(unsigned)i * s.m[0]) >> s.m[1]);
}

// element functions whose result is 0 or 1
template <class E> struct YieldsZeroOne { static constexpr bool value = false; };

// index functions of generate
struct GenIota { static constexpr int kFn = FC_FN_IOTA;
  static __device__ __forceinline__ int apply(const Slot &, const KArgs &, int i) { return i; } };
struct GenIotaRev { static constexpr int kFn = FC_FN_IOTA_REV;
  static __device__ __forceinline__ int apply(const Slot &s, const KArgs &, int i) { return s.ext[0] * s.ext[1] - 1 - i; } };
struct GenClampShift2D { static constexpr int kFn = FC_FN_CLAMP_SHIFT_2D;
  static __device__ __forceinline__ int apply(const Slot &s, const KArgs &, int i) {
    const int h = s.ext[0], w = s.ext[1];
    int r = fast_div(s, i), c = i - r * w;
    r = min(max(r + s.i[0], 0), h - 1);
    c = min(max(c + s.i[1], 0), w - 1);
    return r * w + c; } };
struct GenRowOf2D { static constexpr int kFn = FC_FN_ROW_OF_2D;
  static __device__ __forceinline__ int apply(const Slot &s, const KArgs &, int i) { return fast_div(s, i); } };
struct GenConst { static constexpr int kFn = FC_FN_CONST_I32;
  static __device__ __forceinline__ int apply(const Slot &s, const KArgs &, int) { return s.i[0]; } };

// ------------------------------------------------------------------ expression nodes
// external array number K of the cluster, element type T
template <int K, class T>
struct In {
  using R = T;
  static constexpr int kNodes = 1;
  static constexpr bool kMirror = false;
  // Stream: the element is read once, in order (non-temporal: it does not displace
  // gathered arrays from the caches); a gather turns it off for its source
  template <int Base, bool Stream = false> static __device__ __forceinline__ T eval(const KArgs &a, int i) {
    const T *p = static_cast<const T *>(a.in[K]) + i;
    return Stream ? __builtin_nontemporal_load(p) : *p;
  }
  template <int Base> static __device__ __forceinline__ Vec4<T> eval4(const KArgs &a, int i) {
    using V = T __attribute__((ext_vector_type(4)));
    V v = __builtin_nontemporal_load(reinterpret_cast<const V *>(static_cast<const T *>(a.in[K]) + i));
    return Vec4<T>{{v.x, v.y, v.z, v.w}};
  }
  template <int Base>
  static __device__ __forceinline__ void eval4_pair(const KArgs &a, int i, int ip, Vec4<T> &at_i, Vec4<T> &at_ip) {
    at_i = eval4<Base>(a, i);
    at_ip = eval4<Base>(a, ip);
  }
  template <int Base> static __device__ __forceinline__ bool mirrors_whole(const KArgs &, int) { return true; }
  static void sig(std::string &s) { s += "in" + std::to_string(K) + ":" + DtypeName<T>::s(); }
};

template <int Base, int K, class... E> struct ChildBase;
template <int Base, class E0, class... E> struct ChildBase<Base, 0, E0, E...> { static constexpr int value = Base; };
template <int Base, int K, class E0, class... E> struct ChildBase<Base, K, E0, E...> {
  static constexpr int value = ChildBase<Base + E0::kNodes, K - 1, E...>::value;
};

template <class F, class... E>
struct Map {
  using R = typename F::R;
  static constexpr int kNodes = 1 + (E::kNodes + ... + 0);
  static constexpr bool kMirror = (E::kMirror || ... || false);
  template <int Base, bool Stream, int... K>
  static __device__ __forceinline__ R eval_(const KArgs &a, int i, std::integer_sequence<int, K...>) {
    return F::apply(a.p[Base], E::template eval<ChildBase<Base + 1, K, E...>::value, Stream>(a, i)...);
  }
  template <int Base, bool Stream = false> static __device__ __forceinline__ R eval(const KArgs &a, int i) {
    return eval_<Base, Stream>(a, i, std::make_integer_sequence<int, sizeof...(E)>());
  }
  template <int Base, int... K>
  static __device__ __forceinline__ Vec4<R> eval4_(const KArgs &a, int i, std::integer_sequence<int, K...>) {
    auto t = std::make_tuple(E::template eval4<ChildBase<Base + 1, K, E...>::value>(a, i)...);
    Vec4<R> r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r.v[c] = F::apply(a.p[Base], std::get<K>(t).v[c]...);
    return r;
  }
  template <int Base> static __device__ __forceinline__ Vec4<R> eval4(const KArgs &a, int i) {
    return eval4_<Base>(a, i, std::make_integer_sequence<int, sizeof...(E)>());
  }
  template <int Base, int... K>
  static __device__ __forceinline__ void eval4_pair_(const KArgs &a, int i, int ip, Vec4<R> &at_i, Vec4<R> &at_ip,
                                                     std::integer_sequence<int, K...>) {
    std::tuple<Vec4<typename E::R>...> x, xp;
    (E::template eval4_pair<ChildBase<Base + 1, K, E...>::value>(a, i, ip, std::get<K>(x), std::get<K>(xp)), ...);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      at_i.v[c] = F::apply(a.p[Base], std::get<K>(x).v[c]...);
      at_ip.v[c] = F::apply(a.p[Base], std::get<K>(xp).v[c]...);
    }
  }
  template <int Base>
  static __device__ __forceinline__ void eval4_pair(const KArgs &a, int i, int ip, Vec4<R> &at_i, Vec4<R> &at_ip) {
    eval4_pair_<Base>(a, i, ip, at_i, at_ip, std::make_integer_sequence<int, sizeof...(E)>());
  }
  template <int Base, int... K>
  static __device__ __forceinline__ bool mirrors_whole_(const KArgs &a, int n, std::integer_sequence<int, K...>) {
    return (E::template mirrors_whole<ChildBase<Base + 1, K, E...>::value>(a, n) && ... && true);
  }
  template <int Base> static __device__ __forceinline__ bool mirrors_whole(const KArgs &a, int n) {
    return mirrors_whole_<Base>(a, n, std::make_integer_sequence<int, sizeof...(E)>());
  }
  static void sig(std::string &s) {
    s += "map" + std::to_string(F::kFn) + "(";
    bool first = true;
    ((s += (first ? "" : ","), first = false, E::sig(s)), ...);
    s += ")";
  }
};

template <class... E> struct YieldsZeroOne<Map<FnModEq, E...>> { static constexpr bool value = true; };

template <class G>
struct Gen {
  using R = int;
  static constexpr int kNodes = 1;
  static constexpr bool kMirror = false;
  template <int Base, bool Stream = false> static __device__ __forceinline__ int eval(const KArgs &a, int i) {
    return G::apply(a.p[Base], a, i);
  }
  template <int Base> static __device__ __forceinline__ Vec4<int> eval4(const KArgs &a, int i) {
    Vec4<int> r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r.v[c] = G::apply(a.p[Base], a, i + c);
    return r;
  }
  template <int Base>
  static __device__ __forceinline__ void eval4_pair(const KArgs &a, int i, int ip, Vec4<int> &at_i, Vec4<int> &at_ip) {
    at_i = eval4<Base>(a, i);
    at_ip = eval4<Base>(a, ip);
  }
  template <int Base> static __device__ __forceinline__ bool mirrors_whole(const KArgs &, int) { return true; }
  static void sig(std::string &s) { s += "gen" + std::to_string(G::kFn); }
};

// the constant 1: stands for the flag of a scatter that has none (takes no parameter slot)
struct AlwaysOne {
  using R = int;
  static constexpr int kNodes = 0;
  static constexpr bool kMirror = false;
  template <int Base, bool Stream = false> static __device__ __forceinline__ int eval(const KArgs &, int) { return 1; }
  template <int Base> static __device__ __forceinline__ Vec4<int> eval4(const KArgs &, int) { return Vec4<int>{{1, 1, 1, 1}}; }
  template <int Base>
  static __device__ __forceinline__ void eval4_pair(const KArgs &, int, int, Vec4<int> &at_i, Vec4<int> &at_ip) {
    at_i = at_ip = Vec4<int>{{1, 1, 1, 1}};
  }
  template <int Base> static __device__ __forceinline__ bool mirrors_whole(const KArgs &, int) { return true; }
  static void sig(std::string &s) { s += "1"; }
};

// EI yields the index, ES is evaluated there
template <class EI, class ES>
struct Gather {
  using R = typename ES::R;
  static constexpr int kNodes = 1 + EI::kNodes + ES::kNodes;
  static constexpr bool kMirror = EI::kMirror || ES::kMirror;
  template <int Base, bool Stream = false> static __device__ __forceinline__ R eval(const KArgs &a, int i) {
    int j = EI::template eval<Base + 1, Stream>(a, i);
    return ES::template eval<Base + 1 + EI::kNodes>(a, j);
  }
  template <int Base> static __device__ __forceinline__ Vec4<R> eval4(const KArgs &a, int i) {
    Vec4<int> j = EI::template eval4<Base + 1>(a, i);
    Vec4<R> r;
#pragma unroll
    for (int c = 0; c < 4; ++c) r.v[c] = ES::template eval<Base + 1 + EI::kNodes>(a, j.v[c]);
    return r;
  }
  template <int Base>
  static __device__ __forceinline__ void eval4_pair(const KArgs &a, int i, int ip, Vec4<R> &at_i, Vec4<R> &at_ip) {
    at_i = eval4<Base>(a, i);
    at_ip = eval4<Base>(a, ip);
  }
  // a `reverse` below an arbitrary gather is evaluated at gathered positions: it pairs with nothing
  template <int Base> static __device__ __forceinline__ bool mirrors_whole(const KArgs &a, int n) {
    return EI::template mirrors_whole<Base + 1>(a, n) && !ES::kMirror;
  }
  static void sig(std::string &s) {
    s += "gather(";
    EI::sig(s);
    s += ",";
    ES::sig(s);
    s += ")";
  }
};

// `reverse` (section 2, gather: the index is generate(n-1-i)): the source is read
// backwards, so four consecutive results are one 128-bit read of the source,
// taken in the opposite order, whenever the extent is a multiple of four.
template <class ES>
struct Gather<Gen<GenIotaRev>, ES> {
  using R = typename ES::R;
  using EI = Gen<GenIotaRev>;
  static constexpr int kNodes = 1 + EI::kNodes + ES::kNodes;
  static constexpr bool kMirror = true;
  template <int Base, bool Stream = false> static __device__ __forceinline__ R eval(const KArgs &a, int i) {
    int j = EI::template eval<Base + 1, Stream>(a, i);
    return ES::template eval<Base + 1 + EI::kNodes>(a, j);
  }
  template <int Base> static __device__ __forceinline__ Vec4<R> eval4(const KArgs &a, int i) {
    const int total = a.p[Base + 1].ext[0] * a.p[Base + 1].ext[1];
    Vec4<R> r;
    if ((total & 3) == 0) {
      Vec4<R> v = ES::template eval4<Base + 1 + EI::kNodes>(a, total - 4 - i);
#pragma unroll
      for (int c = 0; c < 4; ++c) r.v[c] = v.v[3 - c];
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) r.v[c] = ES::template eval<Base + 1 + EI::kNodes>(a, total - 1 - (i + c));
    }
    return r;
  }
  // Over exactly n elements (mirrors_whole, n a multiple of four) the group that `reverse` reads
  // for position i is the one at ip taken backwards, and the other way round: the source is
  // evaluated at the same two groups as a direct read of it, with the roles swapped, so that the
  // reads of an array which the program takes forwards and backwards coincide (same addresses in
  // the same registers: each is issued once).
  template <int Base>
  static __device__ __forceinline__ void eval4_pair(const KArgs &a, int i, int ip, Vec4<R> &at_i, Vec4<R> &at_ip) {
    Vec4<R> v, vp;
    ES::template eval4_pair<Base + 1 + EI::kNodes>(a, ip, i, v, vp);     // v: source at ip, vp: source at i
#pragma unroll
    for (int c = 0; c < 4; ++c) { at_i.v[c] = v.v[3 - c]; at_ip.v[c] = vp.v[3 - c]; }
  }
  template <int Base> static __device__ __forceinline__ bool mirrors_whole(const KArgs &a, int n) {
    return a.p[Base + 1].ext[0] * a.p[Base + 1].ext[1] == n && ES::template mirrors_whole<Base + 1 + EI::kNodes>(a, n);
  }
  static void sig(std::string &s) {
    s += "gather(";
    EI::sig(s);
    s += ",";
    ES::sig(s);
    s += ")";
  }
};

// KeepLoads<E>::type is E with every external array read by ordinary loads
// instead of non-temporal ones.  Streams are read non-temporally so that they do
// not displace gathered arrays from the caches; a program that reads one array
// forwards and mirrored wants the opposite: the second read of a line should find
// it (measured on the reversed dot product at 2^26 elements: 1.37x the array's
// bytes fetched with non-temporal loads, 1.00x with ordinary ones).
template <int K, class T>
struct InKeep : In<K, T> {
  template <int Base> static __device__ __forceinline__ Vec4<T> eval4(const KArgs &a, int i) {
    using V = T __attribute__((ext_vector_type(4)));
    V v = *reinterpret_cast<const V *>(static_cast<const T *>(a.in[K]) + i);
    return Vec4<T>{{v.x, v.y, v.z, v.w}};
  }
};
template <class E> struct KeepLoads { using type = E; };
template <int K, class T> struct KeepLoads<In<K, T>> { using type = InKeep<K, T>; };
template <class F, class... E> struct KeepLoads<Map<F, E...>> { using type = Map<F, typename KeepLoads<E>::type...>; };
template <class EI, class ES> struct KeepLoads<Gather<EI, ES>> {
  using type = Gather<typename KeepLoads<EI>::type, typename KeepLoads<ES>::type>;
};

// GatherChain<E> describes an element program that is a chain of one-argument maps over one
// gather whose index is an external array read in order and whose source is again a chain of
// one-argument maps over one external array (the table).  Its value at a position depends on
// the index found there and on nothing else, which lets a commutative consumer visit the
// positions in any order.  leaf() reads the table, from_leaf<Base>() applies the maps to what
// was read, so a kernel can issue many table reads before it uses the first.
template <class E> struct GatherChain;            // only the shapes below
template <int K, class T> struct GatherChain<In<K, T>> {
  using Leaf = T;
  static constexpr int kTable = K;
  static constexpr int kIndex = -1;               // no gather at or below this node
  template <int Base> static constexpr int source_slot() { return -1; }
  static __device__ __forceinline__ T leaf(const KArgs &a, int j) { return static_cast<const T *>(a.in[K])[j]; }
  template <int Base> static __device__ __forceinline__ T from_leaf(const KArgs &, T x) { return x; }
};
template <class F, class E0> struct GatherChain<Map<F, E0>> {
  using Inner = GatherChain<E0>;
  using Leaf = typename Inner::Leaf;
  static constexpr int kTable = Inner::kTable;
  static constexpr int kIndex = Inner::kIndex;
  template <int Base> static constexpr int source_slot() { return Inner::template source_slot<Base + 1>(); }
  static __device__ __forceinline__ Leaf leaf(const KArgs &a, int j) { return Inner::leaf(a, j); }
  template <int Base> static __device__ __forceinline__ typename F::R from_leaf(const KArgs &a, Leaf x) {
    return F::apply(a.p[Base], Inner::template from_leaf<Base + 1>(a, x));
  }
};
template <int KI, class ES> struct GatherChain<Gather<In<KI, int>, ES>> {
  using Inner = GatherChain<ES>;
  using Leaf = typename Inner::Leaf;
  static constexpr int kTable = Inner::kTable;
  static constexpr int kIndex = KI;
  template <int Base> static constexpr int source_slot() { return Base + 2; }     // gather, its index, then its source
  static __device__ __forceinline__ Leaf leaf(const KArgs &a, int j) { return Inner::leaf(a, j); }
  template <int Base> static __device__ __forceinline__ typename ES::R from_leaf(const KArgs &a, Leaf x) {
    return Inner::template from_leaf<Base + 2>(a, x);
  }
};

}  // namespace fc
