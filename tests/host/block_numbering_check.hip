// Host-side check of the update kernels' block numbering: for every launch shape
// in a sweep, each block of C that has to be updated (all of them, or those on and
// below the diagonal) gets exactly one number, number 0 is block (0, 0), and no
// number maps outside the matrix.  Built and run by tests/test_block_numbering.py;
// nothing here touches a GPU.
#include "../../paper_2503_04424_amd/csrc/kernels_update.h"

#include <cstdio>
#include <vector>

using namespace mdet;

int main() {
  long bad = 0, cases = 0;
  for (int tile : {64, 128})
    for (int lower = 0; lower < 2; ++lower)
      for (int nbm = 1; nbm <= 70; ++nbm)
        for (int nbn = 1; nbn <= (lower ? nbm : 40); ++nbn) {
          const int64_t M = (int64_t)nbm * tile - 3, N = (int64_t)nbn * tile - 5;
          const UpdGrid g = update_grid(M, N, lower != 0, tile);
          std::vector<int> seen((size_t)nbm * nbn, 0);
          for (int64_t t = 0; t < 8 * g.per; ++t) {
            int bm = -1, bn = -1;
            if (!update_block_of_number(lower != 0, t, nbm, nbn, g.nsn, g.swl, bm, bn)) continue;
            if (bm < 0 || bn < 0 || bm >= nbm || bn >= nbn) { ++bad; continue; }
            ++seen[(size_t)bm * nbn + bn];
            if (t == 0 && (bm != 0 || bn != 0)) ++bad;
          }
          for (int i = 0; i < nbm; ++i)
            for (int j = 0; j < nbn; ++j) {
              const int want = (!lower || j <= i) ? 1 : 0;
              if (seen[(size_t)i * nbn + j] != want) {
                if (bad < 10)
                  std::printf("tile %d lower %d blocks %d x %d: block (%d, %d) numbered %d times\n", tile,
                              lower, nbm, nbn, i, j, seen[(size_t)i * nbn + j]);
                ++bad;
              }
            }
          ++cases;
        }
  std::printf("shapes %ld bad %ld\n", cases, bad);
  return bad != 0;
}
