// Per-head finalisation, one workgroup per KV head:
//   importance : complete the softmax over all candidates from the pre-pass's per-chunk
//                statistics, 2W-wide sliding max per query row, mean over the alpha rows (Eq. 3-4)
//   redundancy : softmax over the candidates of the mean similarities (Eq. 6)
//   select     : Z = lambda I - (1 - lambda) R (Eq. 7), exact k-th largest by a 4 x 8-bit radix
//                select on order-preserving integer keys held in LDS, ties resolved towards the
//                larger index, kept indices emitted in ascending order by a workgroup prefix scan,
//                followed by the alpha observation rows (Sec. 3.1).
// Two variants follow the paper's pseudo-code (Alg. 1) instead of Eq. 4 / Sec. 3.4: the importance
// may be averaged over the query rows before the pooling, and the selection may be shared by the KV
// heads of a problem (scores averaged over the heads, one workgroup per problem selects).
#include <algorithm>

#include "rkv_internal.h"

namespace rkv {

namespace {

constexpr int kFinThreads = 1024;
constexpr int kFinWaves = kFinThreads / 64;
// LDS floats of the pooling stage.  With many heads two workgroups share a compute unit (74 KB each);
// with at most one head per compute unit a workgroup takes up to 128 KB and stages more columns at once.
constexpr int kMaxPoolFloats = 18944;
constexpr int kMaxPoolFloatsFewHeads = 32768;
static_assert(kMaxPoolFloats >= 16384 + 4 * (kMaxQRows + 1), "room for four columns at the largest supported window");

struct FinArgs {
  const float* logit;    // [heads][rows][n_pad]
  const float* stats;    // [heads][stat_groups][rows][2]
  float* sbar;           // [heads][n_pad]
  const unsigned long long* credit;   // [heads][n_pad] or nullptr: similarity (units of 2^-40) to take off sbar * n
  const float* imp_in;   // [heads][n] (select-only mode)
  const float* red_in;   // [heads][n]
  float* imp_out;        // [heads][n] or nullptr
  float* imp_tmp;        // [heads][n_pad] scratch for the fused path
  float* red_out;        // [heads][n] or nullptr
  float* sbar_out;       // [heads][n] or nullptr
  float* score_out;      // [heads][n] or nullptr
  float* z_tmp;          // [heads][n_pad] scores for the shared selection, or nullptr
  int32_t* kept;         // [heads][budget]
  int n, n_pad, stat_groups, alpha, W, k_sel, budget, pool_floats, pool_rows;
  // similarity rows whose column scan was split over several workgroups: per-part hit counts and
  // running sums, merged here (most recent part first) before the softmax
  const float* rnorm;    // [heads][n_pad]
  const int* part_cnt;   // [heads][parts][n_pad]
  const float* part_pre; // [heads][parts][n_pad]
  int parts;
  const unsigned long long* newer;   // [heads][n_pad] or nullptr: triangular scan, most recent newer partner per token
  int pool_after_mean;
  int rows, G, group_mode;   // rows = logit rows per head: alpha, or G * alpha when group_mode != 0
  float lambda;
};

__device__ __forceinline__ float wave_max(float v) { return full_wave_max(v); }
__device__ __forceinline__ float wave_sum(float v) { return full_wave_sum(v); }
// Workgroup reductions in a fixed order (deterministic); `buf` holds kFinWaves floats.
__device__ float block_sum(float v, float* buf) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = buf[0];
  for (int w = 1; w < kFinWaves; ++w) r += buf[w];
  return r;
}
// Exclusive prefix sum of one uint per thread over the workgroup; also returns the total.
__device__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* buf, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_inclusive_scan(v);
  __syncthreads();
  if (lane == 63) buf[wave] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
  for (int w = 0; w < kFinWaves; ++w) {
    const uint32_t x = buf[w];
    if (w < wave) before += x;
    all += x;
  }
  *total = all;
  return before + inc - v;
}

__device__ __forceinline__ uint32_t order_key(float z) {
  const uint32_t b = __float_as_uint(z);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exact top-k of the n keys held in LDS (equal keys: larger index first).  The k_sel selected indices
// are written in ascending order, followed by n .. n + alpha - 1, to `copies` output lists that lie
// `copy_stride` ints apart.  All threads of the workgroup call this; `keys` must be complete (the
// caller synchronises before the call).  `hist` holds 4 x 256 counters, `sel` 4 x 3 words.
//
// Four 8-bit radix passes find the key of the k-th largest score: each pass counts the digits of the
// keys that match the digits fixed so far (one histogram per pass, all zeroed up front) and the first
// wave alone locates the bin that holds the k-th largest, so a pass costs two workgroup barriers.
__device__ void select_and_emit(const uint32_t* keys, int n, int k_sel, int alpha, int32_t* out, int copies,
                                int64_t copy_stride, uint32_t* hist, uint32_t* scan_buf, uint32_t* sel) {
  const int t = threadIdx.x;
  const int lane = t & 63;
  for (int i = t; i < 4 * 256; i += kFinThreads) hist[i] = 0;
  __syncthreads();
  uint32_t prefix = 0, known = 0, krem = (uint32_t)k_sel, n_equal = 0;
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    uint32_t* h = hist + pass * 256;
    for (int i0 = 0; i0 < n; i0 += kFinThreads) {
      const int i = i0 + t;
      const uint32_t key = (i < n) ? keys[i] : 0u;
      bool live = (i < n) && ((key & known) == prefix);
      const uint32_t digit = (key >> shift) & 255u;
      // scores of one head are often close: count the wave's most common digit with one atomic
      const unsigned long long am = __ballot(live);
      if (am != 0ull) {
        const int first = __builtin_amdgcn_readfirstlane(__ffsll((long long)am) - 1);
        const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, first);
        const unsigned long long same = __ballot(live && digit == d0);
        if (lane == first) atomicAdd(&h[d0], (uint32_t)__popcll(same));
        live = live && (digit != d0);
        if (live) atomicAdd(&h[digit], 1u);
      }
    }
    __syncthreads();
    if (t < 64) {
      // lane l looks at bins 255 - 4l .. 252 - 4l, i.e. the bins in descending order; the bin holding
      // the krem-th largest key is the one whose bins above it hold fewer than krem keys
      const uint32_t b0 = h[255 - 4 * lane], b1 = h[254 - 4 * lane], b2 = h[253 - 4 * lane], b3 = h[252 - 4 * lane];
      const uint32_t mine = (b0 + b1) + (b2 + b3);
      const uint32_t inc = wave_inclusive_scan(mine);
      const uint32_t a0 = inc - mine, a1 = a0 + b0, a2 = a1 + b1, a3 = a2 + b2;
      uint32_t* s3 = sel + pass * 3;
      if (a0 < krem && a1 >= krem) { s3[0] = 255u - 4u * lane; s3[1] = a0; s3[2] = b0; }
      if (a1 < krem && a2 >= krem) { s3[0] = 254u - 4u * lane; s3[1] = a1; s3[2] = b1; }
      if (a2 < krem && a3 >= krem) { s3[0] = 253u - 4u * lane; s3[1] = a2; s3[2] = b2; }
      if (a3 < krem && a3 + b3 >= krem) { s3[0] = 252u - 4u * lane; s3[1] = a3; s3[2] = b3; }
    }
    __syncthreads();
    prefix |= sel[pass * 3] << shift;
    known |= 255u << shift;
    krem -= sel[pass * 3 + 1];
    n_equal = sel[pass * 3 + 2];
  }
  // keys > prefix are all kept; of the n_equal keys == prefix the krem with the largest indices.
  // Each thread owns a run of consecutive candidates, so one workgroup scan orders the output.
  const uint32_t skip_eq = n_equal - krem;
  const int per = (n + kFinThreads - 1) / kFinThreads;
  const int lo = min(t * per, n), hi = min(lo + per, n);
  uint32_t gt = 0, eq = 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t key = keys[i];
    gt += key > prefix ? 1u : 0u;
    eq += key == prefix ? 1u : 0u;
  }
  uint32_t total;
  const uint32_t ex = block_exclusive_scan(gt | (eq << 16), scan_buf, &total);
  uint32_t gt_before = ex & 0xffffu, eq_before = ex >> 16;
  for (int i = lo; i < hi; ++i) {
    const uint32_t key = keys[i];
    const bool is_gt = key > prefix, is_eq = key == prefix;
    if (is_gt || (is_eq && eq_before >= skip_eq)) {
      const uint32_t pos = gt_before + (eq_before > skip_eq ? eq_before - skip_eq : 0u);
      for (int c = 0; c < copies; ++c) out[c * copy_stride + pos] = i;
    }
    gt_before += is_gt ? 1u : 0u;
    eq_before += is_eq ? 1u : 0u;
  }
  for (int r = t; r < alpha; r += kFinThreads)
    for (int c = 0; c < copies; ++c) out[c * copy_stride + k_sel + r] = n + r;
}

constexpr int kModeZ = kModeSelect | kModeScore;     // modes that form the joint score

// PLAIN != 0: the default readings with a window that is a multiple of four wide and an unsplit
// similarity pass; the variants' branches are then compiled out of the instantiation.
// The instantiations for the default readings with the paper's window sizes keep to 64 vector registers, so that two workgroups (eight
// waves per SIMD) share a compute unit when there are many heads; left to itself the register allocator
// takes more for them as soon as unrelated code of the general instantiations changes.
template <int MODE, int PLAIN>
__global__ __launch_bounds__(kFinThreads, PLAIN == 2 ? 8 : 4) void finalize_kernel(FinArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint32_t keys[];   // n_pad order-preserving keys (select mode) / pooling stage
  __shared__ float red[kFinWaves];
  __shared__ uint32_t scan_buf[kFinWaves];
  __shared__ float gmax[kMaxQRows], ginv[kMaxQRows];
  __shared__ uint32_t hist[4 * 256];
  __shared__ uint32_t sel[4 * 3];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int head = blockIdx.x;
  const int n = a.n;
  // PLAIN == 2 additionally fixes the paper's window sizes, alpha = 8 and W = 4, at compile time
  const int alpha = (PLAIN == 2) ? 8 : a.alpha;
  const int W = (PLAIN == 2) ? 4 : a.W;
  const int qrows = PLAIN ? alpha : a.rows;
  const int pool_rows = PLAIN ? alpha : a.pool_rows;
  const int group_mode = PLAIN ? 0 : a.group_mode;
  const bool pool_after_mean = PLAIN ? false : a.pool_after_mean != 0;
  const int sim_parts = PLAIN ? 1 : a.parts;
  const unsigned long long* credit = PLAIN ? nullptr : a.credit;
  const unsigned long long* newer = PLAIN ? nullptr : a.newer;
  const float* lg = a.logit + (int64_t)head * qrows * a.n_pad;
  float* sb = a.sbar + (int64_t)head * a.n_pad;

  // ---- softmax denominators: one wave per query row, lanes over the chunks
  if constexpr ((MODE & kModeImportance) != 0) {
    // the factor 1 / alpha of the mean over the query rows (and 1 / G of the mean over the group's
    // heads, when that is how they are merged) is folded into the softmax normaliser
    const float parts = (float)alpha * (group_mode == 2 ? (float)a.G : 1.0f);
    for (int j = t >> 6; j < qrows; j += kFinWaves) {
      const float* st = a.stats + ((int64_t)head * a.stat_groups * qrows + j) * 2;
      float m = -INFINITY;
      for (int c = lane; c < a.stat_groups; c += 64) m = fmaxf(m, st[(int64_t)c * qrows * 2]);
      m = wave_max(m);
      float den = 0.f;
      for (int c = lane; c < a.stat_groups; c += 64)
        den += st[(int64_t)c * qrows * 2 + 1] * __expf(st[(int64_t)c * qrows * 2] - m);
      den = wave_sum(den);
      if (lane == 0) {
        gmax[j] = m;
        ginv[j] = 1.0f / (den * parts);
      }
    }
  }
  float sinv = 0.f;
  if constexpr ((MODE & kModeRedundancy) != 0) {
    if (sim_parts > 1) {
      // beta = 1 (the only case that is split): the most recent column part that found a hit supplies
      // the forgiven similarity; the slot holds the closed form until now
      for (int i = t; i < n; i += kFinThreads) {
        float forgiven = 0.f;
        for (int p = sim_parts - 1; p >= 0; --p) {
          const int64_t at = ((int64_t)head * sim_parts + p) * a.n_pad + i;
          if (a.part_cnt[at] > 0) {
            forgiven = a.part_pre[at];
            break;
          }
        }
        sb[i] = mean_sim_finish(sb[i], a.rnorm[(int64_t)head * a.n_pad + i], forgiven, n);
      }
    }
    if (newer != nullptr) {
      // triangular scan: a token's most recent partner is the newest token that reported it (the word holds
      // row << 32 | similarity), else the older one its own row met first
      const unsigned long long* nw = newer + (int64_t)head * a.n_pad;
      for (int i = t; i < n; i += kFinThreads) {
        const unsigned long long w = nw[i];
        const float r = a.rnorm[(int64_t)head * a.n_pad + i];
        // the reported similarity is complete (both norms in it): finished as 1 * similarity
        if (w != 0ull) sb[i] = mean_sim_finish(sb[i], 1.0f, __uint_as_float((uint32_t)w), n);
        else sb[i] = mean_sim_finish(sb[i], r, a.part_cnt[(int64_t)head * a.n_pad + i] > 0 ? a.part_pre[(int64_t)head * a.n_pad + i] : 0.f, n);
      }
    }
    if (credit != nullptr) {
      // transposed recency rule: the similarity pass charged the forgiven entries to the recent
      // partner; every thread rewrites the elements it reads again below
      const unsigned long long* cr = credit + (int64_t)head * a.n_pad;
      const float unit = 9.094947017729282e-13f / (float)n;          // 2^-40 / n
      for (int i = t; i < n; i += kFinThreads) sb[i] -= (float)cr[i] * unit;
    }
    // Eq. 6 as it stands: a mean of cosines lies in [-1, 1] (down to -2 with the partner counters taken
    // off), so the exponentials need no shift by the maximum
    float s = 0.f;
    for (int i = t; i < n; i += kFinThreads) s += __expf(sb[i]);
    sinv = 1.0f / block_sum(s, red);
  }
  __syncthreads();

  // ---- importance: the group-max logits are staged in LDS a block of columns at a time (with a halo
  // of W columns, -inf outside [0, n)), so the 2W x alpha window reads per candidate are LDS reads
  float* imp_dst = nullptr;
  if constexpr ((MODE & kModeImportance) != 0) {
    imp_dst = a.imp_out ? a.imp_out + (int64_t)head * n : a.imp_tmp + (int64_t)head * a.n_pad;
    float* pool = reinterpret_cast<float*>(keys);            // the key buffer is not in use yet
    const int win = (W > 0) ? 2 * W : 1;
    const int halo = win - 1;
    // columns per staging block: a multiple of four, leaving room for the window behind the last one
    const int block_cols = (a.pool_floats / pool_rows - win) & ~3;   // >= 4 (checked on the host)
    // W even: four neighbouring candidates share all but three entries of their windows, so one thread
    // serves four candidates from 16-byte LDS reads
    const bool strips = PLAIN || (win >= 4 && (win & 3) == 0);
    for (int cb = 0; cb < n; cb += block_cols) {
      const int cols = min(block_cols, n - cb);
      const int width = cols + halo;
      const int stride = ((cols + 3) & ~3) + win;              // floats per staged row, a multiple of four if `strips`
      const int first = cb - W;                              // column held at pool[j][0]
      if (group_mode != 0) {
        // App. A.2 variants: the attention scores of every query head first (softmax per head), then
        // the max or the mean over the G heads of the group; the staging buffer holds these scores
        // (0 outside [0, n), which never wins a max over scores >= 0)
        for (int j = 0; j < alpha; ++j)
          for (int c = t; c < width; c += kFinThreads) {
            const int col = first + c;
            float pr = 0.f;
            if (col >= 0 && col < n)
              for (int g = 0; g < a.G; ++g) {
                const int row = g * alpha + j;
                const float x = __expf(lg[(int64_t)row * a.n_pad + col] - gmax[row]) * ginv[row];
                pr = (group_mode == 1) ? fmaxf(pr, x) : pr + x;
              }
            pool[j * width + c] = pr;
          }
        __syncthreads();
        if (pool_after_mean) {
          float* avg = pool + alpha * width;
          for (int c = t; c < width; c += kFinThreads) {
            float s = 0.f;
            for (int j = 0; j < alpha; ++j) s += pool[j * width + c];
            avg[c] = s;
          }
          __syncthreads();
          for (int li = t; li < cols; li += kFinThreads) {
            float m = avg[li];
            for (int c = 1; c < win; ++c) m = fmaxf(m, avg[li + c]);
            imp_dst[cb + li] = m;
          }
        } else {
          for (int li = t; li < cols; li += kFinThreads) {
            float imp = 0.f;
            for (int j = 0; j < alpha; ++j) {
              float m = pool[j * width + li];
              for (int c = 1; c < win; ++c) m = fmaxf(m, pool[j * width + li + c]);
              imp += m;
            }
            imp_dst[cb + li] = imp;
          }
        }
        __syncthreads();
        continue;
      }
      // eight query rows x two column slots: sixteen independent loads per thread are in flight
      // before the first LDS store
      for (int c0 = 0; c0 < stride; c0 += 2 * kFinThreads)
      for (int j0 = 0; j0 < alpha; j0 += 8) {
        float v[8][2];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int sl = 0; sl < 2; ++sl) {
            const int c = c0 + t + sl * kFinThreads;
            const int col = first + c;
            v[u][sl] = (j0 + u < alpha && c < width && col >= 0 && col < n)
                           ? lg[(int64_t)(j0 + u) * a.n_pad + col] : -INFINITY;      // -inf also fills width .. stride - 1
          }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int sl = 0; sl < 2; ++sl) {
            const int c = c0 + t + sl * kFinThreads;
            if (j0 + u < alpha && c < stride) pool[(j0 + u) * stride + c] = v[u][sl];
          }
      }
      __syncthreads();
      if (pool_after_mean) {
        // Alg. 1 order: the mean over the query rows of the attention weights first (one extra LDS
        // row; columns outside [0, n) hold exp(-inf) = 0, which never wins a max over weights >= 0
        // because every window holds its own column), then the sliding max of that row
        float* avg = pool + alpha * stride;
        for (int c = t; c < width; c += kFinThreads) {
          float s = 0.f;
          for (int j = 0; j < alpha; ++j) s += __expf(pool[j * stride + c] - gmax[j]) * ginv[j];
          avg[c] = s;
        }
        __syncthreads();
        for (int li = t; li < cols; li += kFinThreads) {
          float m = avg[li];
          for (int c = 1; c < win; ++c) m = fmaxf(m, avg[li + c]);
          imp_dst[cb + li] = m;
        }
        __syncthreads();
        continue;
      }
      if (strips) {
        const int chunks = win >> 2;
        for (int g = t; 4 * g < cols; g += kFinThreads) {
          float imp[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
          for (int j = 0; j < alpha; ++j) {
            // candidates 4g .. 4g+3 of this block: windows [4g + k, 4g + k + win - 1] in staged numbering
            const float4* rowp = reinterpret_cast<const float4*>(pool + j * stride + 4 * g);
            const float4 head4 = rowp[0];
            float inner = head4.w;                               // entries 3 .. win-1 belong to all four windows
            for (int q2 = 1; q2 < chunks; ++q2) {
              const float4 x = rowp[q2];
              inner = fmaxf(inner, fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w)));
            }
            const float4 tail4 = rowp[chunks];
            const float o0 = fmaxf(fmaxf(inner, head4.x), fmaxf(head4.y, head4.z));
            const float o1 = fmaxf(fmaxf(inner, head4.y), fmaxf(head4.z, tail4.x));
            const float o2 = fmaxf(fmaxf(inner, head4.z), fmaxf(tail4.x, tail4.y));
            const float o3 = fmaxf(fmaxf(inner, tail4.x), fmaxf(tail4.y, tail4.z));
            const float gm = gmax[j], gi = ginv[j];
            imp[0] += __expf(o0 - gm) * gi;
            imp[1] += __expf(o1 - gm) * gi;
            imp[2] += __expf(o2 - gm) * gi;
            imp[3] += __expf(o3 - gm) * gi;
          }
#pragma unroll
          for (int k2 = 0; k2 < 4; ++k2)
            if (4 * g + k2 < cols) imp_dst[cb + 4 * g + k2] = imp[k2];
        }
        __syncthreads();
        continue;
      }
      for (int li = t; li < cols; li += kFinThreads) {
        float imp = 0.f;
        // eight query rows at a time: their window reads are independent LDS loads
        for (int j0 = 0; j0 < alpha; j0 += 8) {
          float m[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) m[u] = -INFINITY;
          for (int c = 0; c < win; ++c) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
              if (j0 + u < alpha) m[u] = fmaxf(m[u], pool[(j0 + u) * stride + li + c]);   // window [i - W, i + W - 1]
          }
#pragma unroll
          for (int u = 0; u < 8; ++u)
            if (j0 + u < alpha) imp += __expf(m[u] - gmax[j0 + u]) * ginv[j0 + u];
        }
        imp_dst[cb + li] = imp;
      }
      __syncthreads();
    }
  }

  // ---- per-candidate redundancy and joint score
  for (int i = t; i < n; i += kFinThreads) {
    float imp = 0.f, rd = 0.f;
    if constexpr ((MODE & kModeZ) != 0) {
      if constexpr ((MODE & kModeImportance) != 0) imp = imp_dst[i];
      else imp = a.imp_in[(int64_t)head * n + i];
    }
    if constexpr ((MODE & kModeRedundancy) != 0) {
      const float s = sb[i];
      rd = __expf(s) * sinv;
      if (a.red_out) a.red_out[(int64_t)head * n + i] = rd;
      if (a.sbar_out) a.sbar_out[(int64_t)head * n + i] = s;
    } else if constexpr ((MODE & kModeZ) != 0) {
      rd = a.red_in ? a.red_in[(int64_t)head * n + i] : 0.f;      // no redundancy input: attention-only score
    }
    if constexpr ((MODE & kModeZ) != 0) {
      const float z = a.lambda * imp - (1.0f - a.lambda) * rd;
      if (a.score_out) a.score_out[(int64_t)head * n + i] = z;
      if constexpr ((MODE & kModeScore) != 0) a.z_tmp[(int64_t)head * a.n_pad + i] = z;
      else keys[i] = order_key(z);
    }
  }

  if constexpr ((MODE & kModeSelect) != 0) {
    __syncthreads();
    select_and_emit(keys, n, a.k_sel, alpha, a.kept + (int64_t)head * a.budget, 1, 0, hist, scan_buf, sel);
  }
}

// Shared selection (Alg. 1): one workgroup per problem averages the H per-head scores of each
// candidate (fp32, heads in ascending order) and writes the one kept list into every head's slot.
__global__ __launch_bounds__(kFinThreads) void shared_select_kernel(const float* z, int32_t* kept, int H, int n,
                                                                    int n_pad, int k_sel, int alpha, int budget) {
  extern __shared__ uint32_t keys[];
  __shared__ uint32_t scan_buf[kFinWaves];
  __shared__ uint32_t hist[4 * 256];
  __shared__ uint32_t sel[4 * 3];
  const int p = blockIdx.x;
  const float inv_h = 1.0f / (float)H;
  for (int i = threadIdx.x; i < n; i += kFinThreads) {
    float s = 0.f;
    for (int h = 0; h < H; ++h) s += z[((int64_t)p * H + h) * n_pad + i];
    keys[i] = order_key(s * inv_h);
  }
  __syncthreads();
  select_and_emit(keys, n, k_sel, alpha, kept + (int64_t)p * H * budget, H, budget, hist, scan_buf, sel);
}

template <int MODE, int PLAIN>
hipError_t launch_plain(const FinArgs& a, int heads, size_t lds, hipStream_t stream) {
  // once per kernel instantiation (initialisation of a function-local static is thread-safe)
  static const hipError_t configured = hipFuncSetAttribute(reinterpret_cast<const void*>(&finalize_kernel<MODE, PLAIN>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 32768 * 4);
  if (configured != hipSuccess) return configured;
  hipLaunchKernelGGL((finalize_kernel<MODE, PLAIN>), dim3(heads), dim3(kFinThreads), lds, stream, a);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_mode(const FinArgs& a, int heads, size_t lds, hipStream_t stream) {
  return launch_plain<MODE, 0>(a, heads, lds, stream);
}

}  // namespace

hipError_t launch_finalize(const Plan& pl, int mode, char* ws,
                           const float* imp_in, const float* red_in,
                           float* imp_out, float* red_out, float* sbar_out,
                           float* score_out, int32_t* kept_idx, hipStream_t stream) {
  FinArgs a;
  a.logit = reinterpret_cast<const float*>(ws + pl.off_logit);
  a.stats = reinterpret_cast<const float*>(ws + pl.off_stats);
  a.sbar = reinterpret_cast<float*>(ws + pl.off_sbar);
  a.credit = pl.recency_transposed ? reinterpret_cast<const unsigned long long*>(ws + pl.off_credit) : nullptr;
  a.newer = pl.triangular ? reinterpret_cast<const unsigned long long*>(ws + pl.off_credit) : nullptr;
  a.imp_in = imp_in; a.red_in = red_in;
  a.imp_out = imp_out; a.red_out = red_out; a.sbar_out = sbar_out; a.score_out = score_out;
  a.kept = kept_idx;
  a.n = pl.n; a.n_pad = pl.n_pad; a.stat_groups = pl.chunks * (prepass_register_path(pl) ? 4 : 1); a.alpha = pl.alpha; a.W = pl.W;
  a.k_sel = pl.k_sel; a.budget = pl.budget;
  a.lambda = pl.lambda;
  a.imp_tmp = reinterpret_cast<float*>(ws + pl.off_imp);
  a.z_tmp = reinterpret_cast<float*>(ws + pl.off_z);
  a.pool_after_mean = pl.pool_after_mean ? 1 : 0;
  a.rows = pl.qrows; a.G = pl.G; a.group_mode = pl.gqa_mode;
  a.rnorm = reinterpret_cast<const float*>(ws + pl.off_rnorm);
  a.part_cnt = reinterpret_cast<const int*>(ws + pl.off_pcnt);
  a.part_pre = reinterpret_cast<const float*>(ws + pl.off_ppre);
  a.parts = pl.gram_parts;
  a.pool_rows = pl.alpha + a.pool_after_mean;
  // dynamic LDS: the select keys (n_pad words) and the pooling stage share one region
  size_t words = (mode & kModeSelect) ? (size_t)pl.n_pad : 0;
  a.pool_floats = 0;
  if (mode & kModeImportance) {
    const int win = pl.W > 0 ? 2 * pl.W : 1;
    const size_t want = (size_t)a.pool_rows * (size_t)(pl.n + 3 + win);
    const size_t least = (size_t)a.pool_rows * (size_t)(win + 4); // four columns per block at the very least
    const int cus = device_compute_units();
    const size_t cap = (pl.heads <= cus) ? kMaxPoolFloatsFewHeads : kMaxPoolFloats;
    size_t pool = std::min(std::max(want, least), cap);
    if (pool < least) return hipErrorInvalidValue;                // rejected earlier by make_plan
    a.pool_floats = (int)pool;
    words = std::max(words, pool);
  }
  const size_t lds = words * sizeof(uint32_t);
  // the instantiations without the variants' branches serve the default readings with W a positive
  // multiple of two (other shapes and flags take the general one; only the fused modes are doubled)
  const bool plain_imp = pl.gqa_mode == 0 && !pl.pool_after_mean && pl.W > 0 && (pl.W & 1) == 0;
  const bool plain_red = pl.gram_parts == 1 && !pl.recency_transposed && !pl.triangular;
  const bool paper_window = pl.alpha == 8 && pl.W == 4;
  if (plain_imp && plain_red && mode == (kModeImportance | kModeRedundancy | kModeSelect)) {
    if (paper_window) return launch_plain<kModeImportance | kModeRedundancy | kModeSelect, 2>(a, pl.heads, lds, stream);
    return launch_plain<kModeImportance | kModeRedundancy | kModeSelect, 1>(a, pl.heads, lds, stream);
  }
  if (plain_imp && paper_window && mode == (kModeImportance | kModeSelect))       // attention-only eviction
    return launch_plain<kModeImportance | kModeSelect, 2>(a, pl.heads, lds, stream);
  switch (mode) {
    case kModeImportance: return launch_mode<kModeImportance>(a, pl.heads, lds, stream);
    case kModeRedundancy: return launch_mode<kModeRedundancy>(a, pl.heads, lds, stream);
    case kModeSelect: return launch_mode<kModeSelect>(a, pl.heads, lds, stream);
    case kModeImportance | kModeSelect:
      return launch_mode<kModeImportance | kModeSelect>(a, pl.heads, lds, stream);
    case kModeImportance | kModeRedundancy | kModeSelect:
      return launch_mode<kModeImportance | kModeRedundancy | kModeSelect>(a, pl.heads, lds, stream);
    case kModeScore: return launch_mode<kModeScore>(a, pl.heads, lds, stream);
    case kModeImportance | kModeScore:
      return launch_mode<kModeImportance | kModeScore>(a, pl.heads, lds, stream);
    case kModeImportance | kModeRedundancy | kModeScore:
      return launch_mode<kModeImportance | kModeRedundancy | kModeScore>(a, pl.heads, lds, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_shared_select(const Plan& pl, char* ws, int32_t* kept_idx, hipStream_t stream) {
  static const hipError_t configured = hipFuncSetAttribute(reinterpret_cast<const void*>(&shared_select_kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 32768 * 4);
  if (configured != hipSuccess) return configured;
  hipLaunchKernelGGL(shared_select_kernel, dim3(pl.P), dim3(kFinThreads), (size_t)pl.n_pad * sizeof(uint32_t), stream,
                     reinterpret_cast<const float*>(ws + pl.off_z), kept_idx, pl.H, pl.n, pl.n_pad, pl.k_sel,
                     pl.alpha, pl.budget);
  return hipGetLastError();
}

}  // namespace rkv
