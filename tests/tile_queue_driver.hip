// Host-side check of the tile orders and of the per-XCD queue shares of the persistent kernels.  Built and
// run by tests/test_tile_queue_cpu.py; no GPU is needed (nothing here calls the HIP runtime).
// For every tile count swept and both orders: the entries i < share(y) of the 8 XCDs, decoded with the
// order's map, hand out every tile (tm, tn) exactly once; entries at and beyond share(y) map to no tile;
// 32 consecutive entries of one XCD form a block of at most 4 x 8 neighbouring tiles (what the L2 sharing
// relies on); and dh_split keeps its parts inside the accumulator.
#include <cstdio>
#include <vector>
#include "../paper_2602_05885_amd/csrc/gemm_core.h"
using namespace pg;

static int fails = 0;
#define CHECK(cond, ...) do { if (!(cond)) { if (fails < 20) { printf("FAIL line %d: ", __LINE__); printf(__VA_ARGS__); printf("\n"); } ++fails; } } while (0)

static void sweep(int tiles_m, int tiles_n, int interleaved) {
  TileQueue Q{};
  Q.total = tiles_m * tiles_n; Q.interleaved = interleaved;
  std::vector<int> seen((size_t)Q.total, 0);
  int sum = 0;
  for (int y = 0; y < 8; ++y) {
    const int n = Q.share(y);
    sum += n;
    for (int i = 0; i < n + 3; ++i) {
      int tm = -1, tn = -1;
      const int b = TileQueue::encode(y, i);
      const bool ok = interleaved ? map_tile_interleaved(b, tiles_m, tiles_n, tm, tn) : map_tile(b, tiles_m, tiles_n, tm, tn);
      if (i >= n) { CHECK(!ok, "%dx%d order %d: entry %d of XCD %d beyond its share %d maps to a tile", tiles_m, tiles_n, interleaved, i, y, n); continue; }
      CHECK(ok && tm >= 0 && tm < tiles_m && tn >= 0 && tn < tiles_n, "%dx%d order %d: entry %d of XCD %d -> (%d, %d)", tiles_m, tiles_n, interleaved, i, y, tm, tn);
      if (ok && tm >= 0 && tm < tiles_m && tn >= 0 && tn < tiles_n) ++seen[(size_t)tm * tiles_n + tn];
    }
  }
  CHECK(sum == Q.total, "%dx%d order %d: shares add up to %d of %d", tiles_m, tiles_n, interleaved, sum, Q.total);
  for (int t = 0; t < Q.total; ++t) CHECK(seen[t] == 1, "%dx%d order %d: tile %d handed out %d times", tiles_m, tiles_n, interleaved, t, seen[t]);
  // blocks: entries 32 r .. 32 r + 31 of an XCD span at most 4 tile rows and 8 tile columns
  for (int y = 0; y < 8; ++y)
    for (int i0 = 0; i0 + 32 <= Q.share(y); i0 += 32) {
      int m0 = 1 << 30, m1 = -1, n0 = 1 << 30, n1 = -1;
      for (int i = i0; i < i0 + 32; ++i) {
        int tm, tn;
        if (interleaved) map_tile_interleaved(TileQueue::encode(y, i), tiles_m, tiles_n, tm, tn);
        else map_tile(TileQueue::encode(y, i), tiles_m, tiles_n, tm, tn);
        m0 = imin(m0, tm); m1 = imax(m1, tm); n0 = imin(n0, tn); n1 = imax(n1, tn);
      }
      // a block of the contiguous order may straddle two blocks of the flattened order (its range need not
      // start on a multiple of 32), and ragged edges make blocks narrower and longer: bound the area instead
      if (interleaved && tiles_m % 4 == 0 && tiles_n % 8 == 0 && i0 + 32 <= (Q.total / 256) * 32)
        CHECK(m1 - m0 < 4 && n1 - n0 < 8, "%dx%d: block %d of XCD %d spans %d x %d tiles", tiles_m, tiles_n, i0 / 32, y, m1 - m0 + 1, n1 - n0 + 1);
    }
}

int main() {
  for (int tm = 1; tm <= 70; ++tm)
    for (int tn = 1; tn <= 45; ++tn)
      for (int order = 0; order < 2; ++order) sweep(tm, tn, order);
  for (int order = 0; order < 2; ++order) {     // the shapes the 14B head produces
    sweep(594, 128, order); sweep(89, 20, order); sweep(128, 20, order); sweep(60, 20, order); sweep(594, 512, order);
  }
  for (int n_pad = 256; n_pad <= 65536; n_pad += 256)
    for (int t_cap = n_pad; t_cap <= 65536; t_cap += 4096)
      for (int tiles_n : {1, 2, 16, 20})
        for (int stages : {4, 8, 63, 356, 2374}) {
          const int ks = dh_split(n_pad, t_cap, tiles_n, stages);
          CHECK(ks >= 1 && ks <= 8 && (long long)ks * n_pad <= (long long)imax(t_cap, n_pad) && (ks == 1 || stages / ks >= 8),
                "dh_split(%d, %d, %d, %d) = %d", n_pad, t_cap, tiles_n, stages, ks);
        }
  printf(fails ? "tile queue driver: %d FAILED\n" : "tile queue driver: every tile handed out exactly once (%d failures)\n", fails);
  return fails != 0;
}
