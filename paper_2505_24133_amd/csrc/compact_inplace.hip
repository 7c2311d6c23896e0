// In-place compaction (Alg. 1, gather + concatenate, written back into the cache it reads):
// row r of a head receives row kept[r] of the same head.  The kept list is strictly ascending, so
// kept[r] >= r: rows only move towards the front, and rows in front of the first evicted one do not
// move at all (kept[r] - r is non-decreasing, the first moved row is found by bisection).
//
// One workgroup owns one (head, tensor, column slice) and walks its rows front to back in tiles.
// Within a tile every thread loads its source rows into registers, the workgroup synchronises, and
// only then are the rows written: a tile's sources (rows >= the tile's first row) may be another
// thread's destinations in the same tile, never in an earlier one.  The next tile's sources lie
// behind everything written so far, so their loads are issued before the barrier and overlap the
// stores.  Workgroups never touch each other's bytes.  Pure HBM traffic.
#include <algorithm>

#include "rkv_internal.h"

namespace rkv {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a type the non-temporal builtins accept

constexpr int kIpThreads = 1024;
constexpr int kIpDepth = 4;          // rows per thread and tile

struct InplaceArgs {
  uint16_t* k;
  uint16_t* v;
  const int32_t* kept;
  int H, N, budget, split;           // split = column slices per row (1 or 2)
  KvLayout kl, vl;
};

__global__ __launch_bounds__(kIpThreads) void compact_inplace_kernel(InplaceArgs a) {
  __shared__ int first_moved;
  const int head = blockIdx.x / a.split;
  const int slice = blockIdx.x - head * a.split;
  const int p = head / a.H;
  const int h = head - p * a.H;
  const bool is_v = blockIdx.y != 0;
  const KvLayout lay = is_v ? a.vl : a.kl;
  const int lanes = 16 / a.split;                   // 16-byte pieces of a row handled by this workgroup
  const int t = threadIdx.x;
  const int slot = t / lanes;
  const int piece = t - slot * lanes;
  const int rows_per_pass = kIpThreads / lanes;
  uint16_t* base = (is_v ? a.v : a.k) + (slice * lanes + piece) * 8;
  const int32_t* kept = a.kept + (int64_t)head * a.budget;

  if (t == 0) {
    int lo = 0, hi = a.budget;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (kept[mid] > mid) hi = mid; else lo = mid + 1;
    }
    first_moved = lo;
  }
  __syncthreads();
  const int r_begin = first_moved;
  const int tile = kIpDepth * rows_per_pass;

  // Source indices are fetched one tile ahead of the rows they name, so that the row loads of a tile
  // are issued back to back.  Rows past the end of the list are mapped onto its last entry: their
  // loads read valid memory and their stores are skipped.
  auto load_idx = [&](int r0, int (&src)[kIpDepth]) {
#pragma unroll
    for (int u = 0; u < kIpDepth; ++u) {
      const int r = min(r0 + u * rows_per_pass + slot, a.budget - 1);
      src[u] = kept[r];
    }
  };
  auto load_rows = [&](const int (&src)[kIpDepth], uint4 (&x)[kIpDepth]) {
#pragma unroll
    for (int u = 0; u < kIpDepth; ++u)
      x[u] = *reinterpret_cast<const uint4*>(base + lay.offset(p, h, min(max(src[u], 0), a.N - 1)));
  };

  if (r_begin >= a.budget) return;                  // nothing was evicted in front of the observation rows
  uint4 cur[kIpDepth], nxt[kIpDepth];
  int src[kIpDepth], src_ahead[kIpDepth];
  load_idx(r_begin, src);
  load_rows(src, cur);
  load_idx(r_begin + tile, src);
  for (int r0 = r_begin; r0 < a.budget; r0 += tile) {
    const bool more = r0 + tile < a.budget;         // uniform over the workgroup
    if (more) {
      load_rows(src, nxt);
      load_idx(r0 + 2 * tile, src_ahead);
    }
    // the loaded rows must have arrived in registers before any thread passes the barrier and
    // overwrites one of them: naming the values as operands here makes the wait explicit
#pragma unroll
    for (int u = 0; u < kIpDepth; ++u)
      asm volatile("" ::"v"(cur[u].x), "v"(cur[u].y), "v"(cur[u].z), "v"(cur[u].w) : "memory");
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kIpDepth; ++u) {
      const int r = r0 + u * rows_per_pass + slot;
      if (r < a.budget)      // non-temporal, as in the out-of-place gather: the moved rows are not read again here
        __builtin_nontemporal_store(u32x4{cur[u].x, cur[u].y, cur[u].z, cur[u].w}, reinterpret_cast<u32x4*>(base + lay.offset(p, h, r)));
    }
    if (more) {
#pragma unroll
      for (int u = 0; u < kIpDepth; ++u) {
        cur[u] = nxt[u];
        src[u] = src_ahead[u];
      }
    }
  }
}

}  // namespace

hipError_t launch_compact_inplace(const Plan& pl, void* k, void* v, const int32_t* kept_idx, hipStream_t stream) {
  InplaceArgs a;
  a.k = static_cast<uint16_t*>(k);
  a.v = static_cast<uint16_t*>(v);
  a.kept = kept_idx;
  a.H = pl.H; a.N = pl.N; a.budget = pl.budget;
  a.kl = k_layout(pl); a.vl = v_layout(pl);
  // two 128-byte column slices per row when whole rows would leave compute units without a workgroup
  a.split = (pl.heads * 2 < 512) ? 2 : 1;
  const dim3 grid((unsigned)(pl.heads * a.split), 2);
  hipLaunchKernelGGL(compact_inplace_kernel, grid, dim3(kIpThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rkv
