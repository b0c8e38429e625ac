// Host-side brute-force check of the tile enumeration and classification in hstu_geometry.h
// (the very header the kernels compile).  Built with the host compiler by the CPU test suite.
//   geometry_check(L, M, K1, K2, block_rows, BN) returns 0 when, for one sequence,
//   - every visible (query, key) pair falls in a tile enumerated for its row block (forward / dQ
//     orientation) and for its key block (dK/dV orientation), the ranges are ascending and disjoint,
//   - every enumerated tile holds at least one visible pair (no fully masked tile is scheduled),
//   - classify_tile says Full only if all pairs of the 32x32 block are visible history pairs with
//     distance i - j, and Empty only if none is visible;
//   otherwise a non-zero code naming the violated property.
#include <vector>

#include "hstu_geometry.h"

using namespace hstu;

static int check_ranges(const TileRanges& t) {
  if (t.a0 > t.a1 || t.b0 > t.b1 || t.c0 > t.c1) return 1;
  if (t.a1 > t.b0 && t.b1 > t.b0) return 1;
  if ((t.b1 > t.c0 || t.a1 > t.c0) && t.c1 > t.c0) return 1;
  return 0;
}

extern "C" int geometry_check(int L, int M, int K1, int K2, int block_rows, int BN) {
  const SeqGeom g = {L, L - M, K1, K2};
  const int ntile = (L + BN - 1) / BN;
  for (int orient = 0; orient < 2; ++orient) {
    for (int r0 = 0; r0 < L; r0 += block_rows) {
      const int r1 = imin(r0 + block_rows, L) - 1;
      const TileRanges t = orient == 0 ? tile_ranges(g, r0, r1, BN) : row_tile_ranges(g, r0, r1, BN);
      if (check_ranges(t)) return 10 + orient;
      std::vector<int> listed(ntile + 2, 0), needed(ntile + 2, 0);
      for (int idx = 0; idx < t.count(); ++idx) {
        const int yt = t.at(idx);
        if (yt < 0 || yt >= ntile) return 20 + orient;
        if (listed[yt]) return 30 + orient;
        listed[yt] = 1;
        if (idx > 0 && yt <= t.at(idx - 1)) return 40 + orient;
      }
      for (int x = r0; x <= r1; ++x)
        for (int y = 0; y < L; ++y) {
          int delta;
          const bool vis = orient == 0 ? visible(g, x, y, delta) : visible(g, y, x, delta);
          if (vis) needed[y / BN] = 1;
        }
      for (int yt = 0; yt < ntile; ++yt) {
        if (needed[yt] && !listed[yt]) return 50 + orient;     // a visible pair would be skipped
        if (listed[yt] && !needed[yt]) return 60 + orient;     // a fully masked tile is scheduled
      }
    }
  }
  // classification of 32 x 32 blocks (rows beyond L included, as the kernels see them)
  const int lim = (L + 63) / 32 * 32;
  for (int q0 = 0; q0 < lim; q0 += 32)
    for (int k0 = 0; k0 < lim; k0 += 32) {
      const int kind = classify_tile(g, q0, q0 + 31, k0, k0 + 31);
      int nvis = 0, nbad = 0;
      for (int i = q0; i < q0 + 32; ++i)
        for (int j = k0; j < k0 + 32; ++j) {
          int delta = 0;
          const bool vis = visible(g, i, j, delta);
          nvis += vis;
          const int p = i < g.n ? i : g.n;                       // a candidate row stands at position n
          if (!vis || delta != p - j || i >= L || j >= L) ++nbad;
        }
      if (kind == kTileFull && nbad) return 70;
      if (kind == kTileEmpty && nvis) return 80;
    }
  return 0;
}
