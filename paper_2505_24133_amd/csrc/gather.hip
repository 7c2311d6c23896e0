// Compaction (Alg. 1, gather + concatenate): out[head][r][:] = in[head][kept[head][r]][:] for K and V
// in one launch.  A row is 256 bytes = 16 lanes x 16 bytes; each thread moves four rows of K and
// of V with all loads issued before the stores.  Pure HBM traffic; the stores are non-temporal (the
// compacted rows are not read again by this step, and keeping them out of the caches is worth 15 % of
// the kernel's time; the same hint on the loads gains nothing and evicts the keys the next step reads).
#include "rkv_internal.h"

namespace rkv {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a type the non-temporal builtins accept

constexpr int kGatherThreads = 256;
constexpr int kRowsPerThread = 4;
constexpr int kRowsPerBlock = (kGatherThreads / 16) * kRowsPerThread;   // 64

struct GatherArgs {
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* kept;
  uint16_t* k_out;
  uint16_t* v_out;
  int H, N, budget, blocks_per_head;
  KvLayout kl, vl;
  int64_t osp, osh, ost;
};

__global__ __launch_bounds__(kGatherThreads) void gather_kernel(GatherArgs a) {
  const int head = blockIdx.x / a.blocks_per_head;
  const int blk = blockIdx.x - head * a.blocks_per_head;
  const int p = head / a.H;
  const int h = head - p * a.H;
  const int c16 = threadIdx.x & 15;
  const int slot = threadIdx.x >> 4;
  const uint16_t* kb = a.k + c16 * 8;
  const uint16_t* vb = a.v + c16 * 8;
  const int32_t* kept = a.kept + (int64_t)head * a.budget;
  u32x4 kr[kRowsPerThread], vr[kRowsPerThread];
  int rows[kRowsPerThread];
#pragma unroll
  for (int m = 0; m < kRowsPerThread; ++m) {
    rows[m] = blk * kRowsPerBlock + m * (kGatherThreads / 16) + slot;
    kr[m] = u32x4{0, 0, 0, 0};
    vr[m] = u32x4{0, 0, 0, 0};
    if (rows[m] < a.budget) {
      int src = kept[rows[m]];
      src = min(max(src, 0), a.N - 1);
      kr[m] = *reinterpret_cast<const u32x4*>(kb + a.kl.offset(p, h, src));
      vr[m] = *reinterpret_cast<const u32x4*>(vb + a.vl.offset(p, h, src));
    }
  }
#pragma unroll
  for (int m = 0; m < kRowsPerThread; ++m) {
    if (rows[m] < a.budget) {
      const int64_t o = p * a.osp + h * a.osh + (int64_t)rows[m] * a.ost + c16 * 8;
      __builtin_nontemporal_store(kr[m], reinterpret_cast<u32x4*>(a.k_out + o));
      __builtin_nontemporal_store(vr[m], reinterpret_cast<u32x4*>(a.v_out + o));
    }
  }
}

}  // namespace

hipError_t launch_gather(const Plan& pl, const void* k, const void* v, const int32_t* kept_idx,
                         void* k_out, void* v_out, hipStream_t stream) {
  GatherArgs a;
  a.k = static_cast<const uint16_t*>(k);
  a.v = static_cast<const uint16_t*>(v);
  a.kept = kept_idx;
  a.k_out = static_cast<uint16_t*>(k_out);
  a.v_out = static_cast<uint16_t*>(v_out);
  a.H = pl.H; a.N = pl.N; a.budget = pl.budget;
  a.blocks_per_head = (pl.budget + kRowsPerBlock - 1) / kRowsPerBlock;
  a.kl = k_layout(pl); a.vl = v_layout(pl);
  a.osp = pl.osp; a.osh = pl.osh; a.ost = pl.ost;
  const dim3 grid((unsigned)((int64_t)pl.heads * a.blocks_per_head));
  hipLaunchKernelGGL(gather_kernel, grid, dim3(kGatherThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rkv
