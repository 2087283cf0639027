// Host-side check of the device rule that the residual GEMM (producer) and the RMSNorm (consumer) both evaluate
// from the step's row count: for every row count up to the row limit the producer's workgroups must fit the grid
// the launcher sizes, the slab count must fit the slab buffer, and every K tile of every live output tile must be
// covered by exactly one (tile, split) pair.  Prints "ok <cases>" or the first violation.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#include "../../paper_2605_08862_amd/csrc/common.h"

int main() {
  struct Shape { int N, K, M_max; } shapes[] = {{3584, 18944, 2176}, {3584, 3584, 2176}, {1536, 8960, 4352},
                                                {1536, 1536, 4352}, {8192, 28672, 4352}, {3584, 18944, 700}};
  long cases = 0;
  for (const Shape& sh : shapes) {
    const int cap = 512, n_blocks = (sh.N + 255) / 256, nk = sh.K / 64;
    for (int alt : {0, 128}) {
      const SlabRule rule{0, 96, n_blocks, nk, cap, alt};
      const int tiles_max = (sh.M_max + 95) / 96 * n_blocks;
      const int grid = 8 * (((tiles_max > cap ? tiles_max : cap) + 7) / 8);
      for (int M = 0; M <= sh.M_max; ++M, ++cases) {
        const int bm = rule.tile_rows(M);
        if (bm != 96 && bm != alt) { std::printf("bad tile %d at M=%d\n", bm, M); return 1; }
        const int tiles = (M + bm - 1) / bm * n_blocks, s = rule.slabs(M);
        if (s < 1 || s > kMaxGemmSplit) { std::printf("bad slab count %d at M=%d\n", s, M); return 1; }
        if (s != gemm_adaptive_split(tiles, nk, cap)) { std::printf("producer and consumer disagree at M=%d\n", M); return 1; }
        if ((long)tiles * s > grid) { std::printf("grid %d too small for %d x %d at M=%d\n", grid, tiles, s, M); return 1; }
        if (s > 1 && nk / s < 4) { std::printf("split shorter than four K tiles at M=%d\n", M); return 1; }
        // the K ranges of the splits partition [0, nk)
        int covered = 0, prev_end = 0;
        for (int split = 0; split < s; ++split) {
          const int kt0 = (int)((long)nk * split / s), kt1 = (int)((long)nk * (split + 1) / s);
          if (kt0 != prev_end || kt1 <= kt0) { std::printf("K ranges not contiguous at M=%d\n", M); return 1; }
          covered += kt1 - kt0;
          prev_end = kt1;
        }
        if (covered != nk) { std::printf("K range not covered at M=%d\n", M); return 1; }
      }
    }
  }
  std::printf("ok %ld\n", cases);
  return 0;
}
