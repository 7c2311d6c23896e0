// Measurement aid, not part of the compression path: what the matrix pipe of this chip sustains on the
// instruction the similarity pass is built from.  The published bf16 rate assumes the top clock; under a
// chip-wide stream of v_mfma_f32_32x32x16_bf16 on real data the clock settles well below it, and that
// sustained rate, not the published one, is what the similarity kernel competes with.  The probe issues
// nothing but such MFMAs: every wave holds eight A and eight B fragments cut from the caller's bf16 data
// (so the operand buses toggle as they do in the similarity pass) and accumulates chains of eight.
#include "rkv_internal.h"

namespace rkv {

namespace {

constexpr int kProbeThreads = 256;

__global__ __launch_bounds__(kProbeThreads, 2) void mfma_probe_kernel(const uint16_t* data, float* sink, int chains) {
  // 64 KiB of operands = 4096 fragments of 16 bytes; lanes pick theirs with a stride that spreads them
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int fa = (threadIdx.x * 5 + i * 37 + blockIdx.x * 11) & 4095;
    const int fb = (threadIdx.x * 7 + i * 53 + blockIdx.x * 3 + 2048) & 4095;
    a[i] = *reinterpret_cast<const bf16x8*>(data + fa * 8);
    b[i] = *reinterpret_cast<const bf16x8*>(data + fb * 8);
  }
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  for (int c = 0; c < chains; ++c) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], b[kk], acc, 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) r += acc[i];
  sink[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = r;
}

}  // namespace

}  // namespace rkv

extern "C" rkv_status rkv_probe_mfma(const void* operands, void* sink, int chains, void* stream, int64_t* flops) {
  if (operands == nullptr || sink == nullptr) return RKV_ERR_NULL;
  if (chains < 1 || chains > (1 << 20)) return RKV_ERR_PARAM;
  if (reinterpret_cast<uintptr_t>(operands) % 16 != 0 || reinterpret_cast<uintptr_t>(sink) % 4 != 0) return RKV_ERR_SHAPE;
  const int blocks = 2 * rkv::device_compute_units();
  if ((int64_t)blocks * rkv::kProbeThreads * 4 > (int64_t)RKV_PROBE_SINK_BYTES) return RKV_ERR_WORKSPACE;
  hipLaunchKernelGGL(rkv::mfma_probe_kernel, dim3(blocks), dim3(rkv::kProbeThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint16_t*>(operands), static_cast<float*>(sink), chains);
  if (hipGetLastError() != hipSuccess) return RKV_ERR_HIP;
  if (flops != nullptr) *flops = (int64_t)blocks * (rkv::kProbeThreads / 64) * chains * 8 * (2LL * 32 * 32 * 16);
  return RKV_OK;
}
