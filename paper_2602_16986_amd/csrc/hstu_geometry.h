// Integer geometry of the HSTU attention mask: visibility predicate, enumeration of the tiles
// that hold a visible pair, and tile classification.  Plain C++ with no device intrinsics, so
// the same header serves the HIP kernels and a host-side check of the tiling logic.
#pragma once

#if defined(__HIPCC__)
#define HSTU_HD __host__ __device__ __forceinline__
#else
#define HSTU_HD inline
#endif

namespace hstu {

HSTU_HD int imin(int a, int b) { return a < b ? a : b; }
HSTU_HD int imax(int a, int b) { return a > b ? a : b; }

// Geometry of one sequence under the mask of paper Section 4.2.1 (ordinary 0-based
// orientation: query row i sees key j <= i) extended with trailing candidate rows.
struct SeqGeom {
  int L;    // tokens
  int n;    // history tokens, L - num_targets
  int K1;   // local window (< 0: dense causal)
  int K2;   // global prefix
};

// visible(i, j) and the relative-position distance fed to the bias table.
HSTU_HD bool visible(const SeqGeom& g, int i, int j, int& delta) {
  const bool self = (i >= g.n) && (j == i);
  const int p = i < g.n ? i : g.n;
  const bool hist = (j < g.n) && (j <= p) && (g.K1 < 0 || p - j < g.K1 || j < g.K2);
  delta = self ? 0 : p - j;
  return (i < g.L) && (self || hist);
}

// Column tiles (width BN) that hold at least one visible key for the query rows
// [r0, r1] (inclusive, r1 < L) of one sequence: up to three disjoint ascending
// half-open ranges: the global prefix, the local band, the candidates' own diagonal.
struct TileRanges {
  int a0, a1, b0, b1, c0, c1;
  HSTU_HD int count() const { return (a1 - a0) + (b1 - b0) + (c1 - c0); }
  HSTU_HD int at(int idx) const {
    if (idx < a1 - a0) return a0 + idx;
    idx -= a1 - a0;
    if (idx < b1 - b0) return b0 + idx;
    return c0 + idx - (b1 - b0);
  }
};

HSTU_HD TileRanges tile_ranges(const SeqGeom& g, int r0, int r1, int BN) {
  TileRanges t = {0, 0, 0, 0, 0, 0};
  const bool has_hist = r0 < g.n;
  const bool has_cand = r1 >= g.n;
  const int p_lo = has_hist ? r0 : g.n;                      // smallest effective position
  const int p_hi = has_cand ? g.n : r1;                      // largest effective position
  const int maxkey = imin(p_hi, g.n - 1);                     // last history key any row may see
  int end = 0;
  if (maxkey >= 0) {
    if (g.K1 < 0) {
      t.a1 = maxkey / BN + 1;
      end = t.a1;
    } else {
      const int pre = imin(g.K2, maxkey + 1);                 // prefix keys [0, pre)
      t.a1 = (pre + BN - 1) / BN;
      end = t.a1;
      const int lo = imax(0, p_lo - g.K1 + 1);                // band keys [lo, maxkey]
      if (g.K1 > 0 && lo <= maxkey) {
        t.b0 = imax(lo / BN, end);
        t.b1 = imax(maxkey / BN + 1, t.b0);
        end = t.b1;
      }
    }
  }
  if (t.b1 == 0) { t.b0 = t.b1 = end; }
  if (has_cand) {                                            // self pairs of candidate rows
    const int c_lo = imax(r0, g.n);
    t.c0 = imax(c_lo / BN, end);
    t.c1 = imax(r1 / BN + 1, t.c0);
  } else {
    t.c0 = t.c1 = end;
  }
  return t;
}

// Query-row tiles (height BN) that see at least one key of [k0, k1] (k1 < L): the mirror image of
// tile_ranges(), used by the key-stationary backward pass.
HSTU_HD TileRanges row_tile_ranges(const SeqGeom& g, int k0, int k1, int BN) {
  TileRanges t = {0, 0, 0, 0, 0, 0};
  int end = 0;
  bool cands_see_block = false;
  if (k0 < g.n) {
    const int kh1 = imin(k1, g.n - 1);
    int hi = -1;
    if (g.K1 < 0 || k0 < g.K2) hi = g.n - 1;
    else if (g.K1 > 0) hi = imin(kh1 + g.K1 - 1, g.n - 1);
    if (hi >= k0) {
      t.a0 = k0 / BN;
      t.a1 = hi / BN + 1;
      end = t.a1;
    }
    cands_see_block = (g.K1 < 0) || (k0 < g.K2) || (g.n - kh1 < g.K1);
  }
  t.b0 = t.b1 = end;
  int c_lo = -1, c_hi = -2;
  if (g.n < g.L && cands_see_block) { c_lo = g.n; c_hi = g.L - 1; }
  else if (k1 >= g.n) { c_lo = imax(k0, g.n); c_hi = k1; }
  if (c_hi >= c_lo) {
    t.c0 = imax(c_lo / BN, end);
    t.c1 = imax(c_hi / BN + 1, t.c0);
  } else {
    t.c0 = t.c1 = end;
  }
  return t;
}

// How a block of query rows [w0, w1] relates to a key tile [j0, j1] (j1 may exceed L-1).
enum TileKind { kTileEmpty = 0, kTileFull = 1, kTilePartial = 2 };

// cand_rows: also recognise blocks of candidate rows (all at position n) against history keys as empty or full; without
// it they are reported as partial (for callers whose fast paths assume the distance i - j).
HSTU_HD int classify_tile(const SeqGeom& g, int w0, int w1, int j0, int j1, bool cand_rows = true) {
  if (w0 >= g.L) return kTileEmpty;
  if (w1 < g.n) {                                            // history rows only, all valid
    if (j0 > w1) return kTileEmpty;
    if (g.K1 >= 0 && w0 - j1 >= g.K1 && j0 >= g.K2) return kTileEmpty;
    if (j1 <= w0 && (g.K1 < 0 || w1 - j0 < g.K1 || j1 < g.K2)) return kTileFull;
  } else if (cand_rows && w0 >= g.n && j1 < g.n) {           // candidate rows only (all at position n), history keys only
    if (g.K1 >= 0 && g.n - j1 >= g.K1 && j0 >= g.K2) return kTileEmpty;
    if (w1 < g.L && (g.K1 < 0 || g.n - j0 < g.K1 || j1 < g.K2)) return kTileFull;
  }
  return kTilePartial;
}

}  // namespace hstu
