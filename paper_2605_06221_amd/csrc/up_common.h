// Shared host/device helpers of the UniPrefill operator library (gfx950).
//
// Everything here is integer geometry of the packed batch: block partition,
// retained-token counts and closed-form offsets.  None of it is used by, or
// shared with, the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define UP_HD __host__ __device__ __forceinline__

namespace up {

#if defined(__HIPCC__)      // (device vector types; the host-only build of the argument checks never names them)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
#endif

constexpr int kMaxNObs = 1024;

// Selection geometry of one sequence (block partition of "Token Importance
// Estimation"; sinks and query window of "Top-p Token Selection").
struct SeqGeom {
  int N;        // sequence length
  int G;        // block size
  int n_obs;    // last n tokens always kept
  int n_sink;   // first A tokens always kept
  double rho;   // keep ratio (float widened to double: rho * L is exact)
};

UP_HD int imin(int a, int b) { return a < b ? a : b; }
UP_HD int imax(int a, int b) { return a > b ? a : b; }
UP_HD int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Tokens of [lo, hi) that are always retained: index < A or index >= N - n.
UP_HD int forced_in(const SeqGeom& s, int lo, int hi) {
  const int sink_hi = imin(hi, s.n_sink);
  const int win_lo = imax(lo, s.N - s.n_obs);
  const int sink = imax(0, sink_hi - lo);
  const int win = imax(0, hi - win_lo);
  const int both = imax(0, sink_hi - win_lo);
  return sink + win - both;
}

// ceil(rho * L) clamped to [1, L].
UP_HD int quota(double rho, int L) {
  const double v = rho * (double)L;   // exact: 24-bit significand times a small integer
  int q = (int)v;
  if ((double)q < v) ++q;
  return imin(L, imax(1, q));
}

// Tokens kept in block g: the quota, but never fewer than the forced tokens.
UP_HD int block_kept(const SeqGeom& s, int g) {
  const int lo = g * s.G;
  const int hi = imin(s.N, lo + s.G);
  return imax(quota(s.rho, hi - lo), forced_in(s, lo, hi));
}

// Sum of block_kept over blocks [0, g).  Blocks wholly inside the sinks keep
// all G tokens, blocks between the sinks and the query window keep the plain
// quota; only the few blocks touching a boundary are evaluated one by one.
UP_HD int kept_before(const SeqGeom& s, int g) {
  const int nb = ceil_div(s.N, s.G);
  if (g > nb) g = nb;
  if (g <= 0) return 0;
  const int full_sink = imin(s.n_sink / s.G, nb - 1);          // blocks wholly forced by sinks
  const int g_a = imin(nb, imax(full_sink, ceil_div(imin(s.n_sink, s.N), s.G)));
  int g_t = imax(0, s.N - s.n_obs) / s.G;                      // first block touching the window
  g_t = imin(g_t, nb - 1);                                     // the ragged last block is special too
  if (g_t < g_a) g_t = g_a;
  int sum = imin(g, full_sink) * s.G;
  for (int b = full_sink; b < imin(g, g_a); ++b) sum += block_kept(s, b);
  if (g > g_a) sum += (imin(g, g_t) - g_a) * quota(s.rho, s.G);
  for (int b = g_t; b < g; ++b) sum += block_kept(s, b);
  return sum;
}

UP_HD int seq_kept(const SeqGeom& s) { return kept_before(s, ceil_div(s.N, s.G)); }

// Packed units (key chunks, selection blocks) are numbered without a prefix
// scan: sequence r owns slots [cu[r]/unit + r, ...), which never overlap
// because floor((c+N)/u) - floor(c/u) + 1 >= ceil(N/u).
// (spare = 2: one more slot per sequence, for units that are not aligned with the sequence start)
UP_HD int slot_base(int cu_r, int r, int unit, int spare = 1) { return cu_r / unit + spare * r; }

// Rows of per-sequence statistics: sequence r owns row slots starting at
// min(cu[r], r * n_obs); consecutive starts differ by at least min(N_r, n_obs).
UP_HD int rowslot_base(int cu_r, int r, int n_obs) {
  const long long b = (long long)r * n_obs;
  return b < (long long)cu_r ? (int)b : cu_r;
}

#if defined(__HIPCC__)
// Largest r in [0, R) with slot_base(cu[r], r, unit) <= slot.
__device__ __forceinline__ int locate_slot(const int* __restrict__ cu, int R, int unit, int slot,
                                           int spare = 1) {
  int lo = 0, hi = R - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (slot_base(cu[mid], mid, unit, spare) <= slot) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Largest r in [0, R) with rowslot_base(cu[r], r, n_obs) <= u.
__device__ __forceinline__ int locate_rowslot(const int* __restrict__ cu, int R, int n_obs, int u) {
  int lo = 0, hi = R - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (rowslot_base(cu[mid], mid, n_obs) <= u) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Sequence that owns packed row `tok`: largest r with cu[r] <= tok and cu[r+1] > tok.
__device__ __forceinline__ int locate_token(const int* __restrict__ cu, int R, int tok) {
  int lo = 0, hi = R - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= tok) lo = mid; else hi = mid - 1;
  }
  return lo;
}
#endif

}  // namespace up
