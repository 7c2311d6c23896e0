// Host-side replay of every key-row copy the similarity kernel issues for one head, using the kernel's own
// row arithmetic (paper_2505_24133_amd/csrc/gram_index.h).  Prints "ok <copies>" when every row index lies in
// [0, n) and every copy that is later read fetches exactly the rows of its tile; otherwise prints the first
// violation and exits 1.  Usage: gram_bounds_check n parts
#include <cstdio>
#include <cstdlib>

#include "gram_index.h"

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  const int n = std::atoi(argv[1]), parts = std::atoi(argv[2]);
  const int TC = 128;                               // keys per streamed tile (kGramTile)
  const int nct_all = (n + TC - 1) / TC;
  long long copies = 0;
  for (int part = 0; part < parts; ++part) {
    int lo, hi;
    rkv::gram_part_range(part, parts, nct_all, &lo, &hi);
    if (hi <= lo) continue;
    // the part's first tile, clamped form
    for (int row0 = 0; row0 < TC; row0 += 4)
      for (int lane = 0; lane < 64; ++lane) {
        const int r = rkv::gram_copy_row_clamped(hi - 1, TC, row0, lane, n);
        const int want = (hi - 1) * TC + row0 + (lane >> 4);
        ++copies;
        if (r < 0 || r >= n || (want < n && r != want)) {
          std::printf("clamped copy: n=%d parts=%d part=%d tile=%d row0=%d lane=%d -> row %d\n", n, parts, part, hi - 1, row0, lane, r);
          return 1;
        }
      }
    for (int ct = hi - 1; ct >= lo; --ct) {
      const int ctn = rkv::gram_next_tile(ct, lo);
      const bool read_later = ctn < ct;             // the last iteration's copy is never read
      for (int row0 = 0; row0 < TC; row0 += 4)                 // row0 = wave * 4 + jj * 16 over the four waves
        for (int lane = 0; lane < 64; ++lane) {
          const int r = rkv::gram_copy_tile_row0(ctn, TC, n) + rkv::gram_copy_group_row(row0 & 15, TC, n) +
                        rkv::gram_copy_group_row(row0 & ~15, TC, n) + rkv::gram_copy_lane_row(lane, n);
          ++copies;
          if (r < 0 || r >= n || (read_later && r != ctn * TC + row0 + (lane >> 4))) {
            std::printf("unclamped copy: n=%d parts=%d part=%d tile=%d next=%d row0=%d lane=%d -> row %d\n", n, parts, part, ct, ctn,
                        row0, lane, r);
            return 1;
          }
        }
    }
  }
  std::printf("ok %lld\n", copies);
  return 0;
}
