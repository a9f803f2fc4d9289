// Wavefront and workgroup primitives for gfx950 (wave64).
//
// Cross-lane steps use DPP modifiers: row_shr inside the four 16-lane rows of a
// wave, row_bcast:15 / row_bcast:31 to carry row totals across rows.  Workgroup
// steps go through LDS.  Cross-workgroup steps use agent-scope atomics, because
// the eight XCDs of the chip have separate L2 caches.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/fc.h"

namespace fc {

constexpr int kWave = 64;
constexpr int kBlock = 256;            // threads per workgroup in every kernel
constexpr int kWavesPerBlock = kBlock / kWave;

// ------------------------------------------------------------------ reducers
struct AddF32 {
  using T = float;
  static __device__ __forceinline__ T identity() { return 0.0f; }
  static __device__ __forceinline__ T apply(T a, T b) { return a + b; }
  static const char *name() { return "add.f32"; }
};
struct MaxF32 {
  using T = float;
  static __device__ __forceinline__ T identity() { return -__builtin_inff(); }
  static __device__ __forceinline__ T apply(T a, T b) { return fmaxf(a, b); }
  static const char *name() { return "max.f32"; }
};
struct MulF32 {
  using T = float;
  static __device__ __forceinline__ T identity() { return 1.0f; }
  static __device__ __forceinline__ T apply(T a, T b) { return a * b; }
  static const char *name() { return "mul.f32"; }
};
struct AddI32 {
  using T = int;
  static __device__ __forceinline__ T identity() { return 0; }
  static __device__ __forceinline__ T apply(T a, T b) { return a + b; }
  static const char *name() { return "add.i32"; }
};
struct MaxI32 {
  using T = int;
  static __device__ __forceinline__ T identity() { return INT32_MIN; }
  static __device__ __forceinline__ T apply(T a, T b) { return a > b ? a : b; }
  static const char *name() { return "max.i32"; }
};

// ------------------------------------------------------------------ bit casts
template <class T> __device__ __forceinline__ int as_bits(T v) { return __builtin_bit_cast(int, v); }
template <class T> __device__ __forceinline__ T from_bits(int v) { return __builtin_bit_cast(T, v); }

// DPP controls
constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;
constexpr int kWaveShl1 = 0x130, kWaveShr1 = 0x138;

// value of `v` moved by a DPP control; lanes without a source keep `fill`
template <int Ctrl, int RowMask = 0xf, class T>
__device__ __forceinline__ T dpp_move(T fill, T v) {
  return from_bits<T>(__builtin_amdgcn_update_dpp(as_bits(fill), as_bits(v), Ctrl, RowMask, 0xf, false));
}

// Inclusive scan across the 64 lanes of a wave (lane order).  Lane 63 ends up
// with the reduction of the whole wave.
template <class Op>
__device__ __forceinline__ typename Op::T wave_scan_inclusive(typename Op::T v) {
  using T = typename Op::T;
  const T id = Op::identity();
  v = Op::apply(dpp_move<kRowShr1>(id, v), v);
  v = Op::apply(dpp_move<kRowShr2>(id, v), v);
  v = Op::apply(dpp_move<kRowShr4>(id, v), v);
  v = Op::apply(dpp_move<kRowShr8>(id, v), v);
  // lane 15 of rows 0 and 2 into every lane of rows 1 and 3
  v = Op::apply(dpp_move<kRowBcast15, 0xa>(id, v), v);
  // lane 31 into every lane of rows 2 and 3
  v = Op::apply(dpp_move<kRowBcast31, 0xc>(id, v), v);
  return v;
}

template <class Op>
__device__ __forceinline__ typename Op::T wave_reduce(typename Op::T v) {
  using T = typename Op::T;
  v = wave_scan_inclusive<Op>(v);
  return from_bits<T>(__builtin_amdgcn_readlane(as_bits(v), 63));
}

// Inclusive scan inside each 16-lane row only; lane 15 of a row holds the row total.
template <class Op>
__device__ __forceinline__ typename Op::T row_scan_inclusive(typename Op::T v) {
  using T = typename Op::T;
  const T id = Op::identity();
  v = Op::apply(dpp_move<kRowShr1>(id, v), v);
  v = Op::apply(dpp_move<kRowShr2>(id, v), v);
  v = Op::apply(dpp_move<kRowShr4>(id, v), v);
  v = Op::apply(dpp_move<kRowShr8>(id, v), v);
  return v;
}

// value of the previous / next lane of the wave (lane 0 / lane 63 receive `fill`)
template <class T> __device__ __forceinline__ T lane_prev(T fill, T v) { return dpp_move<kWaveShr1>(fill, v); }
template <class T> __device__ __forceinline__ T lane_next(T fill, T v) { return dpp_move<kWaveShl1>(fill, v); }

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x / kWave); }

// Reduction over the workgroup in a fixed order (lane order inside waves, wave
// order across them).  Every thread receives the result.  `lds` holds
// Waves + 1 words (Waves: waves of the workgroup) and may be reused after the call returns.
template <class Op, int Waves = kWavesPerBlock>
__device__ __forceinline__ typename Op::T block_reduce(typename Op::T v, typename Op::T *lds) {
  using T = typename Op::T;
  T w = wave_reduce<Op>(v);
  __syncthreads();
  if (lane_id() == 0) lds[wave_id()] = w;
  __syncthreads();
  T r = lds[0];
#pragma unroll
  for (int k = 1; k < Waves; ++k) r = Op::apply(r, lds[k]);
  return r;
}

// ------------------------------------------------------------------ agent-scope memory
__device__ __forceinline__ void store_agent(unsigned *p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned load_agent(const unsigned *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent64(unsigned long long *p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_agent64(const unsigned long long *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------ scratch control block
// Layout of the first bytes of the caller's scratch buffer.  Cross-workgroup
// steps use no read-modify-write atomics: device-scope atomics on one address
// serialise (tens of nanoseconds each), which would dominate a kernel of a few
// thousand workgroups.  Instead every launch takes a tag from `epoch`, results
// that other workgroups wait for are published as 64-bit words carrying that tag
// (one agent-scope store), and readers poll until the tag matches.  Words left by
// earlier launches carry older tags and a zero-filled buffer carries tag 0, which
// is never used, so nothing has to be cleared between launches.  The workgroup
// that finishes the launch's protocol last by construction (it has seen the
// words of all others) advances `epoch`.
struct Control {
  unsigned epoch;       // launches of tagged kernels so far
  unsigned error;       // set to 1 when a bounded wait gave up (results of that launch are invalid)
  unsigned pad[62];
};
constexpr int kMaxPartials = 8192;                 // workgroups of a fold launch
constexpr size_t kPartialsOffset = sizeof(Control);
constexpr size_t kStatusOffset = kPartialsOffset + kMaxPartials * sizeof(unsigned long long);
constexpr size_t kMaxTiles = (FC_SCRATCH_CONTROL_BYTES - kStatusOffset) / sizeof(unsigned long long);
constexpr unsigned kSpinLimit = 1u << 22;          // polls before a wait gives up: never hang the device

// `epoch` read at the very start of a kernel, with an ordinary load.  The word changes only once
// every workgroup of the launch has taken its tag from it (the workgroup that advances it has
// seen a tagged word of all others), and the kernel boundary before the launch makes the store
// of the launch before visible, so the value is the same as an agent-scope load's.  The
// difference is where it travels: a uniform ordinary load goes through the scalar unit and
// returns on its own counter, whereas an agent-scope load is a vector memory operation, and
// the wait for it (a round trip to memory) would stand in front of the kernel's first reads
// (single-pass compaction of 2^26 elements: every tile issued its reads a round trip late).
__device__ __forceinline__ unsigned epoch_at_start(const Control *ctl) { return ctl->epoch; }

__device__ __forceinline__ unsigned tag_of_epoch(unsigned epoch) { return epoch % 0x3ffffffeu + 1u; }  // 30 bits, never 0

// word = value (high 32 bits) | tag << 2 | state (low 2 bits, 0 = not ready)
__device__ __forceinline__ unsigned long long pack_word(unsigned value, unsigned tag, unsigned state) {
  return ((unsigned long long)value << 32) | (unsigned long long)((tag << 2) | state);
}

// Polls `p` until it carries `tag` with a non-zero state; returns the word, or 0
// after kSpinLimit polls (and raises the error word).
__device__ __forceinline__ unsigned long long wait_word(const unsigned long long *p, unsigned tag, Control *ctl) {
  for (unsigned spins = 0; spins < kSpinLimit; ++spins) {
    unsigned long long w = load_agent64(p);
    unsigned lo = (unsigned)w;
    if ((lo >> 2) == tag && (lo & 3u) != 0u) return w;
    __builtin_amdgcn_s_sleep(1);
  }
  store_agent(&ctl->error, 1u);
  return 0ull;
}

}  // namespace fc
