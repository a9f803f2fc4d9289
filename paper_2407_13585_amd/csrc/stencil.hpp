// Specialised instance for the cluster
//     out = add5(p, gather(N, p), gather(S, p), gather(W, p), gather(E, p))  [+ m = fold(max) p]
// where p = F(in) is a producer shared by consumers that read it in five
// different traversal orders (section 3.3, `simple5`: one array read in several
// orders inside one loop) and N, S, W, E are clamped unit shifts of a 2-D index.
//
// The generic element program would evaluate F five times per point and do
// integer division for every index.  Here each wave walks down a strip of the
// grid: a lane owns four adjacent columns, keeps rows r-1, r, r+1 of p in
// registers, takes its west / east neighbours from the adjacent lanes with DPP
// wave shifts, and evaluates F once per loaded element.  Lanes 0 and 63 of a
// wave only supply halo columns, so a wave produces 62 * 4 = 248 columns.
#pragma once

#include "kernels.hpp"
#include "registry.hpp"

namespace fc {

constexpr int kStripCols = (kWave - 2) * kVec;   // 248 output columns per wave
constexpr int kBandRows = 32;                    // rows per wave (a multiple of kRowsPerStep)
constexpr int kRowsPerStep = 4;                  // row loads in flight per lane

struct Quad { float x, y, z, w; };

template <class F>
__device__ __forceinline__ Quad load_row(const float *g, const Slot &s, int r, int c, int H, int W) {
  r = min(max(r, 0), H - 1);
  const float *row = g + (size_t)r * (size_t)W;
  Quad v;
  if (c >= 0 && c + 3 < W) {
    using V = float __attribute__((ext_vector_type(4)));
    // non-temporal: the streamed grid must not displace the halo rows in L2 (measured: 18 % faster)
    V t = __builtin_nontemporal_load(reinterpret_cast<const V *>(row + c));
    v = {t.x, t.y, t.z, t.w};
  } else {
    v.x = row[min(max(c, 0), W - 1)];
    v.y = row[min(max(c + 1, 0), W - 1)];
    v.z = row[min(max(c + 2, 0), W - 1)];
    v.w = row[min(max(c + 3, 0), W - 1)];
  }
  return {F::apply(s, v.x), F::apply(s, v.y), F::apply(s, v.z), F::apply(s, v.w)};
}

// F: element function of the shared producer (FnExpNeg, or FnIdentF when p is
// read from memory).  WithMax: also fold(max) over p into out[1].
template <class F, int FSlot, bool WithMax>
__global__ __launch_bounds__(kBlock) void stencil5_kernel(const KArgs a, Control *ctl, unsigned long long *partials,
                                                          int n_groups, int n_bands, int band_rows) {
  const int H = a.h, W = a.w;
  const float *g = static_cast<const float *>(a.in[0]);
  float *out = static_cast<float *>(a.out[0]);
  const Slot &fs = a.p[FSlot];

  // workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
  // range of (band, strip group) tiles so that halo rows are re-read from its own L2
  const int n_blocks = n_groups * n_bands;
  const int per_xcd = (n_blocks + 7) / 8;
  const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
  float m = -__builtin_inff();
  if (logical < n_blocks) {
    const int band = logical / n_groups, group = logical - band * n_groups;
    const int strip = group * kWavesPerBlock + wave_id();
    const int lane = lane_id();
    const int c = strip * kStripCols - kVec + lane * kVec;
    const bool writes = lane >= 1 && lane <= kWave - 2 && c < W;
    const int r0 = band * band_rows, r1 = min(r0 + band_rows, H);
    if (strip * kStripCols < W) {
      Quad prev = load_row<F>(g, fs, r0 - 1, c, H, W);
      Quad cur = load_row<F>(g, fs, r0, c, H, W);
      for (int r = r0; r < r1; r += kRowsPerStep) {
        Quad nxt[kRowsPerStep];
#pragma unroll
        for (int k = 0; k < kRowsPerStep; ++k) nxt[k] = load_row<F>(g, fs, r + 1 + k, c, H, W);
#pragma unroll
        for (int k = 0; k < kRowsPerStep; ++k) {
          const float left = lane_prev(0.0f, cur.w);
          const float right = lane_next(0.0f, cur.x);
          // (((p + N) + S) + W) + E, the order of add5
          Quad o;
          o.x = (((cur.x + prev.x) + nxt[k].x) + left) + cur.y;
          o.y = (((cur.y + prev.y) + nxt[k].y) + cur.x) + cur.z;
          o.z = (((cur.z + prev.z) + nxt[k].z) + cur.y) + cur.w;
          o.w = (((cur.w + prev.w) + nxt[k].w) + cur.z) + right;
          if (writes && r + k < r1) {
            using V = float __attribute__((ext_vector_type(4)));
            V t = {o.x, o.y, o.z, o.w};
            *reinterpret_cast<V *>(out + (size_t)(r + k) * (size_t)W + c) = t;
            if (WithMax) m = fmaxf(fmaxf(fmaxf(m, cur.x), fmaxf(cur.y, cur.z)), cur.w);
          }
          prev = cur;
          cur = nxt[k];
        }
      }
    }
  }
  if (WithMax) fold_finish<MaxF32>(m, a, 1, ctl, partials);
}

template <class F, int FSlot, bool WithMax, int G0, int GStride>
bool stencil5_accept(const KArgs &a) {
  static const int want[4][2] = {{-1, 0}, {1, 0}, {0, -1}, {0, 1}};
  if (a.h < 1 || a.w < 4 || (a.w % 4) != 0) return false;
  for (int k = 0; k < 4; ++k) {
    const Slot &s = a.p[G0 + k * GStride];
    if (s.i[0] != want[k][0] || s.i[1] != want[k][1] || s.ext[0] != a.h || s.ext[1] != a.w) return false;
  }
  return true;
}

template <class F, int FSlot, bool WithMax>
hipError_t launch_stencil5(const KArgs &a, const LaunchCtx &c) {
  if (a.n == 0 && !WithMax) return hipSuccess;
  const int strips = (a.w + kStripCols - 1) / kStripCols;
  const int groups = (strips + kWavesPerBlock - 1) / kWavesPerBlock;
  // Bands of kBandRows rows whatever the device holds at once: bands sized so that the
  // launch is a single round of resident workgroups were measured slower (8192 x 8192:
  // 107 us with 40-row bands in one round, 102 us with 32-row bands in 1.125 rounds).
  int band_rows = kBandRows;
  while ((long long)groups * ((a.h + band_rows - 1) / band_rows) > kMaxPartials - 8) band_rows *= 2;
  const int bands = std::max(1, (a.h + band_rows - 1) / band_rows);
  const int blocks = ((groups * bands + 7) / 8) * 8;
  KArgs args = a;
  Control *ctl = c.ctl;
  unsigned long long *partials = c.partials;
  int g = groups, b = bands, br = band_rows;
  void *ptrs[] = {&args, &ctl, &partials, &g, &b, &br};
  return hipLaunchKernel(reinterpret_cast<const void *>(&stencil5_kernel<F, FSlot, WithMax>), dim3(blocks),
                         dim3(kBlock), ptrs, 0, c.stream);
}

}  // namespace fc
