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

// Unclamped form: a wave-uniform first row plus the lane's row.  Every real copy made this way lies in a
// tile that ends at or before n, where both functions are the identity.  The redundant copy of a part's
// last iteration can name the head's last, partly filled tile; its first row is pulled back so that the
// four rows stay inside [0, n) (their content does not matter).
RKV_HD int gram_copy_first_row(int ct, int tc, int row0, int n) {
  int r = ct * tc + row0;
  if (r > n - 4) r = n - 4;
  return r > 0 ? r : 0;
}
RKV_HD int gram_copy_lane_row(int lane, int n) {
  const int r = lane >> 4;
  return r < n - 1 ? r : n - 1;
}

}  // namespace rkv
