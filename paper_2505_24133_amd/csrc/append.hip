// Decode-loop bookkeeping around the compression step (Sec. 3.1, App. C.1): a new token's key and
// value rows are written at the end of the cache and its query state into the alpha-slot query cache.
// One thread moves 16 bytes.
#include "rkv_internal.h"

namespace rkv {

namespace {

struct AppendArgs {
  uint16_t* k_cache;
  uint16_t* v_cache;
  uint16_t* q_ring;
  const uint16_t* k_new;
  const uint16_t* v_new;
  const uint16_t* q_new;
  int H, Hq, alpha, pos, slot, kv_rows, q_rows;
  int64_t qsp, qsh, qst;      // strides of the query cache (elements): problem, query head, slot
  KvLayout kl, vl;
};

__global__ __launch_bounds__(256) void append_kernel(AppendArgs a) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  const int row = gid >> 4, c16 = gid & 15;
  if (row < a.kv_rows) {                                   // one row per (problem, kv head)
    const int p = row / a.H, h = row - p * a.H;
    const uint4 kx = *reinterpret_cast<const uint4*>(a.k_new + (int64_t)row * kHeadDim + c16 * 8);
    const uint4 vx = *reinterpret_cast<const uint4*>(a.v_new + (int64_t)row * kHeadDim + c16 * 8);
    *reinterpret_cast<uint4*>(a.k_cache + a.kl.offset(p, h, a.pos) + c16 * 8) = kx;
    *reinterpret_cast<uint4*>(a.v_cache + a.vl.offset(p, h, a.pos) + c16 * 8) = vx;
  } else if (row < a.kv_rows + a.q_rows) {                 // one row per (problem, query head)
    const int qr = row - a.kv_rows;
    const uint4 qx = *reinterpret_cast<const uint4*>(a.q_new + (int64_t)qr * kHeadDim + c16 * 8);
    const int p = qr / a.Hq, hq = qr - p * a.Hq;
    *reinterpret_cast<uint4*>(a.q_ring + p * a.qsp + hq * a.qsh + a.slot * a.qst + c16 * 8) = qx;
  }
}

}  // namespace

hipError_t launch_append(const Plan& pl, void* k_cache, void* v_cache, void* q_ring, const void* k_new,
                         const void* v_new, const void* q_new, int pos, int slot, hipStream_t stream) {
  AppendArgs a;
  a.k_cache = static_cast<uint16_t*>(k_cache);
  a.v_cache = static_cast<uint16_t*>(v_cache);
  a.q_ring = static_cast<uint16_t*>(q_ring);
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.q_new = static_cast<const uint16_t*>(q_new);
  a.H = pl.H; a.Hq = pl.H * pl.G; a.alpha = pl.alpha; a.pos = pos; a.slot = slot;
  a.kv_rows = pl.heads;
  a.q_rows = pl.P * pl.H * pl.G;
  a.qsp = pl.qsp; a.qsh = pl.qsh; a.qst = pl.qst;
  a.kl = k_layout(pl); a.vl = v_layout(pl);
  const int threads = (a.kv_rows + a.q_rows) * 16;
  hipLaunchKernelGGL(append_kernel, dim3((threads + 255) / 256), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace rkv
