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
// wave shifts, and evaluates F once per loaded element.  A wave's strip is 256
// columns = eight whole 128-byte lines per row; the column left of the strip and
// the one right of it are read by lanes 0 and 63 with one extra 4-byte load per
// row.  Those two lines are being read by the neighbouring waves at the same
// time, so they come from the cache.  (Strips of 248 columns with the halo
// inside the 128-bit loads straddled nine lines per row and fetched 17 % more
// than the grid from HBM.)
#pragma once

#include "kernels.hpp"
#include "registry.hpp"

namespace fc {

constexpr int kStripCols = kWave * kVec;         // 256 output columns per wave
constexpr int kBandRows = 32;                    // least rows per wave (a multiple of kRowsPerStep)
constexpr int kMaxBandRows = 128;
constexpr int kRowsPerStep = 4;                  // row loads in flight per lane

struct Quad { float x, y, z, w; };

// Row r (clamped to the grid) of the input at columns c .. c+3, before F.  W is a
// multiple of four and c >= 0, so the 128-bit read is taken at min(c, W-4) and is
// always inside the row.  Nothing here depends on the loaded value, so the row
// reads of a step are issued back to back and are in flight together.
using RawRow = float __attribute__((ext_vector_type(4)));
__device__ __forceinline__ RawRow load_row(const float *g, int r, int c, int H, int W) {
  r = min(max(r, 0), H - 1);
  // non-temporal: the streamed grid must not displace the halo rows in L2 (measured: 18 % faster)
  return __builtin_nontemporal_load(reinterpret_cast<const RawRow *>(g + (size_t)r * (size_t)W + min(c, W - kVec)));
}

// p = F(row); a lane right of the grid stands for the clamped column W-1
template <class F>
__device__ __forceinline__ Quad apply_row(const Slot &s, const RawRow &t, bool outside) {
  const float w = F::apply(s, t.w);
  if (outside) return {w, w, w, w};
  return {F::apply(s, t.x), F::apply(s, t.y), F::apply(s, t.z), w};
}

// p at the column left of the strip (lane 0) or right of it (lane 63), clamped to the grid
// Only the load sits under the lane condition; F is applied by the caller on
// all lanes, so that no wait for the load is needed inside the branch and the
// loads of a step stay in flight together.
__device__ __forceinline__ float load_halo(const float *g, int r, int c0, int lane, int H, int W) {
  float v = 0.0f;
  if (lane == 0 || lane == kWave - 1) {
    r = min(max(r, 0), H - 1);
    const int c = lane == 0 ? max(c0 - 1, 0) : min(c0 + kStripCols, W - 1);
    v = g[(size_t)r * (size_t)W + c];
  }
  return v;
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
    const int c0 = strip * kStripCols, c = c0 + lane * kVec;
    const bool writes = c < W, outside = !writes;
    const int r0 = band * band_rows, r1 = min(r0 + band_rows, H);
    if (strip * kStripCols < W) {
      Quad prev = apply_row<F>(fs, load_row(g, r0 - 1, c, H, W), outside);
      Quad cur = apply_row<F>(fs, load_row(g, r0, c, H, W), outside);
      float hcur = F::apply(fs, load_halo(g, r0, c0, lane, H, W));
      for (int r = r0; r < r1; r += kRowsPerStep) {
        RawRow raw[kRowsPerStep];
        Quad nxt[kRowsPerStep];
        float hnxt[kRowsPerStep];
#pragma unroll
        for (int k = 0; k < kRowsPerStep; ++k) hnxt[k] = load_halo(g, r + 1 + k, c0, lane, H, W);
#pragma unroll
        for (int k = 0; k < kRowsPerStep; ++k) raw[k] = load_row(g, r + 1 + k, c, H, W);
#pragma unroll
        for (int k = 0; k < kRowsPerStep; ++k) {
          nxt[k] = apply_row<F>(fs, raw[k], outside);
          hnxt[k] = F::apply(fs, hnxt[k]);
        }
#pragma unroll
        for (int k = 0; k < kRowsPerStep; ++k) {
          const float left = lane_prev(hcur, cur.w);     // lane 0 keeps its halo value
          const float right = lane_next(hcur, cur.x);    // lane 63 keeps its halo value
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
          hcur = hnxt[k];
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
  // Higher bands re-read fewer halo rows (two per band), lower bands give more
  // workgroups: the bands are as high as they can be, up to kMaxBandRows, while the
  // launch still has four workgroups per compute unit.  Measured at 8192 x 8192 inside
  // the five-pipeline step: 96 us with 32-row bands (8 workgroups per CU), 94 us with
  // 64 (4 per CU), 99 us with 48 (5.3 per CU, uneven), 102 us with 128 (2 per CU).
  int band_rows = kBandRows;
  const long long enough = 4LL * device_compute_units();
  while (band_rows + kRowsPerStep <= kMaxBandRows &&
         (long long)groups * ((a.h + band_rows + kRowsPerStep - 1) / (band_rows + kRowsPerStep)) >= enough)
    band_rows += kRowsPerStep;
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
