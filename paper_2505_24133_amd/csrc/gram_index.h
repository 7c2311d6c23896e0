// Which key rows the similarity pass fetches, as plain integer functions shared by the kernel and by a
// host-side bounds check (tests/gram_bounds_check.cpp replays every copy of a launch on the CPU and
// asserts that no row index reaches n).  No floating point, no HIP types.
#pragma once

#if defined(__HIPCC__)
#define RKV_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define RKV_HD inline
#endif

namespace rkv {

// Column tiles [lo, hi) that column part `part` of `parts` scans (descending), of nct_all tiles in all.
RKV_HD void gram_part_range(int part, int parts, int nct_all, int* lo, int* hi) {
  *lo = (int)((long long)part * nct_all / parts);
  *hi = (int)((long long)(part + 1) * nct_all / parts);
}

// The tile whose copy is issued while tile `ct` is used.  In the last iteration of a part this is `ct`
// itself: a redundant copy that keeps the copy code free of branches and is never read.
RKV_HD int gram_next_tile(int ct, int ct_lo) { return ct - 1 > ct_lo ? ct - 1 : ct_lo; }

// One wave-wide copy moves four consecutive rows (lane / 16 picks the row).  Clamped form, used for a
// part's first tile (the only one that can reach past n through a real copy): row per lane.
RKV_HD int gram_copy_row_clamped(int ct, int tc, int row0, int lane, int n) {
  const int r = ct * tc + row0 + (lane >> 4);
  return r < n - 1 ? r : n - 1;
}

// Unclamped form, used for every copy issued inside the scan: row = tile row + group row + lane row, the first
// two wave-uniform.  Every copy made this way that is later read lies in a tile that ends at or before n
// (so n >= tc), where all three functions are the identity.  The copy of a part's last iteration is never
// read and can name the head's last, partly filled tile: the tile's first row is pulled back so that the
// tile stays inside [0, n), and a head with fewer than tc candidates reads rows 0 .. min(3, n - 1) only.
RKV_HD int gram_copy_tile_row0(int ct, int tc, int n) {
  int r = ct * tc;
  if (r > n - tc) r = n - tc;
  return r > 0 ? r : 0;
}
RKV_HD int gram_copy_group_row(int row_in_tile, int tc, int n) { return n >= tc ? row_in_tile : 0; }
RKV_HD int gram_copy_lane_row(int lane, int n) {
  const int r = lane >> 4;
  return r < n - 1 ? r : n - 1;
}

}  // namespace rkv
