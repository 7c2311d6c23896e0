// Internal declarations shared by the HIP translation units of librkv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rkv.h"

namespace rkv {

constexpr int kHeadDim = 128;        // d
constexpr int kChunk = 128;          // keys per workgroup in the key pre-pass
constexpr int kMaxQRows = 64;        // G * alpha rows of observation queries per KV head
constexpr int kGramRows = 384;       // candidate rows per workgroup of the similarity pass (4 waves x 3 row tiles)
constexpr int kGramRowsSkip = 256;   // the same with RKV_FLAG_SKIP_SATURATED (4 waves x 2 row tiles)
constexpr int kGramTile = 128;       // keys per streamed column tile of the similarity pass
constexpr int kGramMaxParts = 16;    // most workgroups that share the column scan of one row block
constexpr int kGramSplitMaxBlocks = 256;   // the scan is split only when all heads have at most this many row blocks
constexpr int kRowBytes = kHeadDim * 2;
constexpr int kLdsRowBytes = kRowBytes + 16;   // padded LDS row: 16-byte fragments of 8 consecutive rows hit distinct banks

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Where row `tok` of (problem p, KV head h) lives: contiguous caches use the three strides; paged
// caches look the page up in the block table (rkv.h describes the layout).
struct KvLayout {
  const int32_t* table;        // nullptr: contiguous
  int page_shift, table_stride;
  int64_t sp, sh, st, spage;   // element strides: problem (contiguous only), head, token, page (paged only)
  __device__ __forceinline__ int64_t offset(int p, int h, int tok) const {
    if (table == nullptr) return p * sp + h * sh + (int64_t)tok * st;
    const int page = table[(int64_t)p * table_stride + (tok >> page_shift)];
    return page * spage + h * sh + (int64_t)(tok & ((1 << page_shift) - 1)) * st;
  }
};

// Derived sizes and the workspace carve-up (all offsets in bytes, 256-byte aligned).
struct Plan {
  int P, H, G, N, n, k_sel, alpha, budget, W, beta;
  int heads;          // P * H
  int chunks;         // ceil(n / kChunk)
  int n_pad;          // chunks * kChunk
  float T, lambda, eps;
  bool skip_saturated;     // RKV_FLAG_SKIP_SATURATED
  bool pool_after_mean;    // RKV_FLAG_POOL_AFTER_MEAN
  bool shared_selection;   // RKV_FLAG_SHARED_SELECTION
  bool recency_transposed; // RKV_FLAG_RECENCY_TRANSPOSED
  bool triangular;         // RKV_FLAG_TRIANGULAR_SCAN
  // Similarity pass: the column scan of every row block is split over `gram_parts` workgroups when
  // there are too few row blocks to fill the machine (beta = 1 only: each part reports the first hit of
  // its own column range and finalize keeps the most recent one).
  int gram_parts;
  int gqa_mode;            // 0: max of the logits, then softmax (Eq. 2-3); 1: softmax, then max; 2: softmax, then mean
  int qrows;               // logit rows kept per head: alpha (mode 0) or G * alpha
  int64_t ksp, ksh, kst;   // key strides (elements)
  int64_t vsp, vsh, vst;   // value strides (elements)
  int64_t osp, osh, ost;   // strides of the compacted outputs (elements)
  int64_t qsp, qsh, qst;   // strides of the observation queries (elements): problem, query head, window slot
  bool paged;              // page_size > 0
  int page_shift, table_stride;
  const int32_t* block_table;
  int64_t kspage, vspage;  // page strides (elements)
  size_t off_kdense;       // bf16  [heads][n_pad][128]       dense copy of the candidate keys (paged caches only)
  size_t off_rnorm;   // float [heads][n_pad]           1 / (|K_i| + eps), 0 for i >= n
  size_t off_upart;   // float [heads][chunks][128]     per-chunk sums of r_i K_i
  size_t off_logit;   // float [heads][qrows][n_pad]    scaled logits (group max in mode 0)
  size_t off_stats;   // float [heads][groups][qrows][2] (max, sum exp) per chunk (groups = chunks), or per
                      //                                 32 keys (groups = 4 * chunks) on the pre-pass's register path
  size_t off_sbar;    // float [heads][n_pad]           mean similarity
  size_t off_imp;     // float [heads][n_pad]           importance (fused path)
  size_t off_red;     // float [heads][n_pad]           redundancy (fused path)
  size_t off_z;       // float [heads][n_pad]           per-head scores Z (shared selection)
  size_t off_credit;  // u64   [heads][n_pad]           forgiven similarity charged to the recent partner, in
                      //                                units of 2^-40 (RKV_FLAG_RECENCY_TRANSPOSED), or the most
                      //                                recent newer partner, row << 32 | similarity bits
                      //                                (RKV_FLAG_TRIANGULAR_SCAN)
  size_t off_pcnt;    // int   [heads][gram_parts][n_pad]    hits found per row and column part (gram_parts > 1)
  size_t off_ppre;    // float [heads][gram_parts][n_pad]    sum of those hits
  size_t off_idx;     // int   [heads][budget]          kept indices when the caller passes none
  size_t total;
};

rkv_status make_plan(const rkv_params* prm, Plan* plan);
int device_compute_units();   // of the current device; cached after the first query

// Kernel launchers (each enqueues on `stream` and returns hipGetLastError()).
// Non-zero (alpha / 2, plus 100 with two query row tiles) when the pre-pass merges the group's heads in
// registers and writes its softmax statistics per 32 keys; 0 when it goes through LDS and writes them
// per chunk of 128 keys.
int prepass_register_path(const Plan& pl);
hipError_t launch_prepass(const Plan& pl, const void* q_obs, const void* k, char* ws, hipStream_t stream);
hipError_t launch_gram(const Plan& pl, const void* k, char* ws, hipStream_t stream);

enum SelectMode : int {
  kModeImportance = 1,   // workspace logits -> importance
  kModeRedundancy = 2,   // workspace mean similarity -> redundancy
  kModeSelect = 4,       // importance, redundancy -> Z, kept indices (per head)
  kModeScore = 8,        // importance, redundancy -> Z in the workspace, no selection
};
hipError_t launch_finalize(const Plan& pl, int mode, char* ws,
                           const float* imp_in, const float* red_in,
                           float* imp_out, float* red_out, float* sbar_out,
                           float* score_out, int32_t* kept_idx, hipStream_t stream);
// One kept list per problem from the head-averaged workspace scores, replicated to every head.
hipError_t launch_shared_select(const Plan& pl, char* ws, int32_t* kept_idx, hipStream_t stream);
hipError_t launch_gather(const Plan& pl, const void* k, const void* v, const int32_t* kept_idx,
                         void* k_out, void* v_out, hipStream_t stream);

// K and V compacted where they lie; kept_idx must be strictly ascending per head.
hipError_t launch_compact_inplace(const Plan& pl, void* k, void* v, const int32_t* kept_idx, hipStream_t stream);

inline KvLayout k_layout(const Plan& pl) {
  return KvLayout{pl.paged ? pl.block_table : nullptr, pl.page_shift, pl.table_stride, pl.ksp, pl.ksh, pl.kst, pl.kspage};
}
inline KvLayout v_layout(const Plan& pl) {
  return KvLayout{pl.paged ? pl.block_table : nullptr, pl.page_shift, pl.table_stride, pl.vsp, pl.vsh, pl.vst, pl.vspage};
}

hipError_t launch_append(const Plan& pl, void* k_cache, void* v_cache, void* q_ring, const void* k_new,
                         const void* v_new, const void* q_new, int pos, int slot, hipStream_t stream);

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Mean similarity of a token (Eq. 6) from its closed-form parts, in ONE fixed sequence of rounded operations
// wherever it is finished (by the similarity kernel itself, or by the finalize kernel when the token's
// column scan was shared by several workgroups), so that the result does not depend on the schedule:
//   closed = r (K_i . u) - (r |K_i|)^2          [row sum of the cosine matrix, diagonal taken off]
//   mean   = (closed - r * forgiven) / n        [forgiven: sum over the forgiven partners of (K_i . K_j) r_j]
__device__ __forceinline__ float mean_sim_closed(float r, float rowdot, float eps) {
  const float self = __fmaf_rn(-eps, r, 1.0f);             // r |K_i| = 1 - eps r
  return __fmaf_rn(r, rowdot, -__fmul_rn(self, self));
}
__device__ __forceinline__ float mean_sim_finish(float closed, float r, float forgiven, int n) {
  return __fdiv_rn(__fmaf_rn(-r, forgiven, closed), (float)n);
}

// Reduction steps between lane l and lane l ^ 16 (or l ^ 32) with the gfx950 row-swap instructions:
// after the swap both lanes of a pair hold (value of the lower lane, value of the upper lane), so
// the two get bit-identical results without a trip through LDS.
__device__ __forceinline__ float pair_sum16(float v) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float pair_sum32(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// max of two floats as ONE v_max_f32.  fmaxf() on values the compiler cannot see the origin of (lane
// exchanges, MFMA results) is preceded by an instruction per operand that quiets signalling NaNs; the
// kernels' inputs hold none, and in the reductions below that tripled the instruction count.
__device__ __forceinline__ float raw_max(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float pair_max16(float v) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return raw_max(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_max32(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return raw_max(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// v + (v of the lane selected by the DPP control), within rows of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  const int x = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
  return v + __int_as_float(x);
}
// max(v, v of the lane selected by the DPP control) as one instruction; the two wait states a DPP read
// needs after the vector instruction that wrote its source travel with it.
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
  static_assert(CTRL == 0xB1 || CTRL == 0x4E || CTRL == 0x141 || CTRL == 0x140, "the four steps of the row reduction");
  float r;
  if constexpr (CTRL == 0xB1) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  else if constexpr (CTRL == 0x4E) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  else if constexpr (CTRL == 0x141) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  else asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_mirror row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  return r;
}
// Reductions over the 32 lanes of each half of the wave (every lane of the half ends with the result):
// four DPP steps inside the rows of 16 lanes, one row swap between the two rows.  The full-wave forms
// add the swap between the halves.  All lanes must be active.
__device__ __forceinline__ float half_wave_max(float v) {
  v = dpp_max<0xB1>(v);     // quad_perm [1,0,3,2]
  v = dpp_max<0x4E>(v);     // quad_perm [2,3,0,1]
  v = dpp_max<0x141>(v);    // row_half_mirror
  v = dpp_max<0x140>(v);    // row_mirror
  return pair_max16(v);
}
__device__ __forceinline__ float half_wave_sum(float v) {
  v = dpp_add<0xB1>(v);
  v = dpp_add<0x4E>(v);
  v = dpp_add<0x141>(v);
  v = dpp_add<0x140>(v);
  return pair_sum16(v);
}
__device__ __forceinline__ float full_wave_max(float v) { return pair_max32(half_wave_max(v)); }
__device__ __forceinline__ float full_wave_sum(float v) { return pair_sum32(half_wave_sum(v)); }

// Inclusive prefix sum over the 64 lanes: shifts by 1, 2, 4, 8 inside the rows of 16 lanes (a lane
// without a source adds 0), then lane 15 of rows 0 and 2 is added to rows 1 and 3, and lane 31 to
// rows 2 and 3.  All lanes must be active.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
  return x;
}

}  // namespace rkv
