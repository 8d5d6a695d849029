// Integer index code of the early-stage window mask (paper sections 4.1 and
// 4.2), shared by the host-side inspection helpers and every kernel.
// Query p may attend key j  iff  j < row_limit(p).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define BEAGLE_HD __host__ __device__ __forceinline__
#else
#define BEAGLE_HD inline
#endif

namespace beagle {

// Value ranges (enforced by the descriptor check): positions and lengths below 2^30, 1 <= k <= 2^30,
// 0 <= eps < k.  Inside them no expression below leaves the int32 range.
struct MaskParams {
  int32_t k;        // window size >= 1
  int32_t eps;      // window offset in [0, k)
  int32_t seq_kv;   // L
  int32_t all_visible;  // decode: every query sees all L keys
};

// Start of the window that holds query p: windows start at eps + w*k for every
// integer w; queries before eps sit in a partial leading window that starts
// below zero and therefore see nothing.
BEAGLE_HD int32_t window_start(int32_t p, int32_t k, int32_t eps) {
  int32_t t = p - eps;
  if (t < 0) return 0;
  return eps + (t / k) * k;
}

// Start of the window that holds position p, NOT clamped: below zero for the
// partial leading window (floor division toward minus infinity).
BEAGLE_HD int32_t window_start_raw(int32_t p, int32_t k, int32_t eps) {
  int32_t t = p - eps;
  int32_t w = t >= 0 ? t / k : -((-t + k - 1) / k);
  return eps + w * k;
}

// Late-stage simulation, step t (section 4.2, second half): the predicted keys
// that query p may attend are [lo, hi): the first t positions of p's own
// window that lie before p.  hi <= lo: none.  Any t >= k shows the whole window
// (t is clamped first: w0 + t must not overflow for a caller's large step count).
BEAGLE_HD void sim_band(int32_t p, int32_t k, int32_t eps, int32_t t, int32_t seq_kv, int32_t& lo, int32_t& hi) {
  int32_t w0 = window_start_raw(p, k, eps);
  lo = w0 > 0 ? w0 : 0;
  hi = w0 + (t < k ? t : k);
  if (hi > p) hi = p;
  if (hi > seq_kv) hi = seq_kv;
}

// Number of keys visible to query p (they are keys 0 .. limit-1).
BEAGLE_HD int32_t row_limit(int32_t p, const MaskParams& mp) {
  if (mp.all_visible) return mp.seq_kv;
  int32_t w = window_start(p, mp.k, mp.eps);
  return w < mp.seq_kv ? w : mp.seq_kv;
}

// First query that can see key j (the start of the window after j's window);
// may be >= S, meaning no query sees j.
BEAGLE_HD int32_t first_query_seeing(int32_t j, const MaskParams& mp) {
  if (mp.all_visible) return 0;
  int32_t t = j - mp.eps;
  if (t < 0) return mp.eps;               // j is in the partial leading window
  return mp.eps + (t / mp.k + 1) * mp.k;
}

enum TileClass : uint8_t { TILE_SKIP = 0, TILE_PARTIAL = 1, TILE_FULL = 2 };

// Class of the tile of queries [q0, q1) x keys [j0, j1), q1 <= S, j1 <= L.
// Row limits never decrease with p, so the first and last row decide.
BEAGLE_HD TileClass tile_class(int32_t q0, int32_t q1, int32_t j0, int32_t j1, const MaskParams& mp) {
  int32_t hi = row_limit(q1 - 1, mp);
  if (hi <= j0) return TILE_SKIP;
  int32_t lo = row_limit(q0, mp);
  return lo >= j1 ? TILE_FULL : TILE_PARTIAL;
}

}  // namespace beagle
