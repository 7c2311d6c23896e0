// Key pre-pass: one read of the candidate keys produces, per chunk of 128 keys,
//   - the inverse norms r_i = 1 / (|K_i|_2 + eps)                      (Eq. 5)
//   - the chunk's share of u = sum_i r_i K_i (used for closed-form row sums of the
//     cosine matrix: sum_j S_ij = r_i K_i . u - S_ii)
//   - the group-max scaled logits of the G*alpha observation query rows (Eq. 2-3, bf16 MFMA,
//     fp32 accumulation) and the chunk's (max, sum exp) per query row for the softmax over
//     all candidates, which the finalize kernel completes.
// HBM-bound: every key byte is read exactly once, coalesced, and staged in LDS.
#include <algorithm>

#include "rkv_internal.h"

namespace rkv {

namespace {

constexpr int kPrepassThreads = 256;
constexpr int kLogitStride = kChunk + 8;   // floats; +8 puts the two half-waves on disjoint banks

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

struct PrepassArgs {
  const uint16_t* q;      // [P, Hq, alpha, d] or nullptr
  const uint16_t* k;
  float* rnorm;
  unsigned long long* credit;   // zeroed here for the similarity pass, or nullptr
  float* upart;
  float* logit;
  float* stats;
  int H, G, alpha, n, n_pad, chunks, items;
  const int32_t* table;       // block table of a paged cache, or nullptr
  int page_shift, table_stride;
  int64_t kspage;
  uint16_t* kdense;           // [heads][n_pad][128] dense copy of the candidate keys (paged caches), or nullptr
  int out_rows, out_groups;   // rows written per key: alpha (max over out_groups = G heads) or G*alpha (out_groups = 1)
  int64_t ksp, ksh, kst;
  int64_t qsp, qsh, qst;      // strides of q (elements): problem, query head, window slot
  float eps, scale;
};

// AH = alpha / 2 selects the register path for the usual window sizes (alpha = 8, 16 or 32): with
// those, the query rows that a lane holds for g = 0 .. G-1 sit AH accumulator registers apart (and in
// the second row tile when G * alpha > 32), so the max over the group and the wave's softmax
// statistics need neither LDS nor a workgroup barrier.  AH = 0 is the general path.
// PAGED: the keys come from a page pool behind a block table and a dense copy of them is written for
// the similarity pass (a separate instantiation, so that the contiguous case carries none of it).
// At least three workgroups per compute unit (one wave of each per SIMD): the variants with two query row
// tiles would otherwise take a few registers too many for a third workgroup, and the kernel lives on the
// number of key chunks in flight.
template <bool HAS_Q, int MT, int AH, bool PAGED>
__global__ __launch_bounds__(kPrepassThreads, 3) void prepass_kernel(PrepassArgs a) {
  // The logit tile reuses the key tile's LDS once every wave has read its key fragments
  // (MT * 32 rows x 136 floats <= 128 rows x 272 bytes), which lets four workgroups share a CU.
  __shared__ __attribute__((aligned(16))) unsigned char ks[kChunk * kLdsRowBytes];
  __shared__ float ured[4][kHeadDim];
  float (*lg)[kLogitStride] = reinterpret_cast<float (*)[kLogitStride]>(ks);
  static_assert(2 * 32 * kLogitStride * sizeof(float) <= sizeof(ks), "logit tile must fit in the key tile");

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int c16 = t & 15;
  const int rbase = t >> 4;

  // Persistent workgroups: each walks over (head, chunk) items.  Four workgroups share a compute unit
  // (128 VGPRs, 37 KB of LDS each), so while one waits for its chunk the others compute; holding the
  // next chunk in registers as well cost a workgroup per compute unit and was slower.
  const uint32_t row_bytes = (uint32_t)a.kst * 2u;
  auto fetch = [&](int hd, int ck, uint4 (&dst)[8]) {
    const int pp = hd / a.H;
    // rows past n repeat row n - 1 (their r is forced to 0 below and their logits are masked)
    if constexpr (PAGED) {
      // paged cache: the 16 rows a thread group fetches together lie in one page (pages hold >= 16 rows)
      const uint16_t* kb = a.k + (hd - pp * a.H) * a.ksh + c16 * 8;
      const int32_t* tb = a.table + (int64_t)pp * a.table_stride;
      const int mask = (1 << a.page_shift) - 1;
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const int grow = min(ck * kChunk + m * 16 + rbase, a.n - 1);
        dst[m] = *reinterpret_cast<const uint4*>(kb + tb[grow >> a.page_shift] * a.kspage + (int64_t)(grow & mask) * a.kst);
      }
    } else {
      const uint16_t* kb = a.k + pp * a.ksp + (hd - pp * a.H) * a.ksh;
      // The chunk's first row goes into the workgroup-uniform base; what is left per thread is a row inside
      // the chunk (pulled back to row n - 1 in a head's last chunk) times the row pitch, a 32-bit offset:
      // rows are at most 65536 bytes apart and a chunk has 128 of them.
      const unsigned char* cb = reinterpret_cast<const unsigned char*>(kb) + (int64_t)ck * kChunk * row_bytes;
      const uint32_t last = (uint32_t)(a.n - 1 - ck * kChunk);
#pragma unroll
      for (int m = 0; m < 8; ++m)
        dst[m] = *reinterpret_cast<const uint4*>(cb + (min((uint32_t)(m * 16 + rbase), last) * row_bytes + (uint32_t)c16 * 16u));
    }
  };
  uint4 regs[8];

  // Walk order (the grid is a multiple of 8 workgroups, dealt round-robin to the 8 XCDs): the workgroups
  // of XCD x take the heads with head % 8 == x, which is where the similarity pass will read their keys
  // again, and take them last head first, so that what this kernel leaves in an XCD's L2 are the heads
  // the similarity pass starts with.
  const int xcd = blockIdx.x & 7;
  const int heads_x = (a.items / a.chunks - xcd + 7) >> 3;
  for (int li = blockIdx.x >> 3; li < heads_x * a.chunks; li += gridDim.x >> 3) {
  const int head = (heads_x - 1 - li / a.chunks) * 8 + xcd;
  const int chunk = li % a.chunks;
  const int p = head / a.H;
  const int h = head - p * a.H;
  const int j0 = chunk * kChunk;
  fetch(head, chunk, regs);
  // the query fragments of this head are requested now and used after the norms: their latency hides
  // behind the first stage (rows past G * alpha repeat the last one; their results are not read)
  bf16x8 qf[MT][8];
  if constexpr (HAS_Q) {
    const int GA = a.G * a.alpha;
    const uint16_t* qbase = a.q + p * a.qsp + (int64_t)h * a.G * a.qsh;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      // query row g * alpha + j of the group: head h * G + g, window slot j
      const int qrow = min(mt * 32 + (lane & 31), GA - 1);
      const int qg = qrow / a.alpha;
      const uint16_t* qr = qbase + qg * a.qsh + (qrow - qg * a.alpha) * a.qst;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const uint4 qv = *reinterpret_cast<const uint4*>(qr + kk * 16 + (lane >> 5) * 8);
        __builtin_memcpy(&qf[mt][kk], &qv, 16);
      }
    }
  }

  // ---- stage the chunk in LDS, norms and the chunk's share of u
  float uacc[8], r8[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) uacc[e] = 0.f;
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    const int row = m * 16 + rbase;
    const int grow = j0 + row;
    const uint4 x = regs[m];
    *reinterpret_cast<uint4*>(ks + row * kLdsRowBytes + c16 * 16) = x;
    const uint32_t w4[4] = {x.x, x.y, x.z, x.w};
    float f[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[2 * e] = __uint_as_float(w4[e] << 16);
      f[2 * e + 1] = __uint_as_float(w4[e] & 0xffff0000u);
    }
    // |K_row|^2: packed bf16 dot products, then a butterfly over the 16 lanes that share the row
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      bf16x2 pr;
      __builtin_memcpy(&pr, &w4[e], 4);
      ss = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ss, false);
    }
    ss = dpp_add<0xB1>(ss);     // quad_perm [1,0,3,2]
    ss = dpp_add<0x4E>(ss);     // quad_perm [2,3,0,1]
    ss = dpp_add<0x141>(ss);    // row_half_mirror
    ss = dpp_add<0x140>(ss);    // row_mirror
    // hardware sqrt / reciprocal (1 ulp each): r enters every score only through products that are
    // compared at 1e-3 relative, and the threshold test tolerates 1e-5 absolute
    const float r = (grow < a.n) ? __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(ss) + a.eps) : 0.f;
    r8[m] = r;
#pragma unroll
    for (int e = 0; e < 8; ++e) uacc[e] = fmaf(r, f[e], uacc[e]);
  }
  if constexpr (PAGED) {
    // paged cache: the similarity pass reads the candidate keys from this dense copy
    uint16_t* kd = a.kdense + ((int64_t)head * a.n_pad + j0 + rbase) * kHeadDim + c16 * 8;
#pragma unroll
    for (int m = 0; m < 8; ++m)
      if (j0 + m * 16 + rbase < a.n) *reinterpret_cast<uint4*>(kd + (int64_t)m * 16 * kHeadDim) = regs[m];
  }
  if (c16 == 0) {
    // one lane per row writes r (0 in the padding up to n_pad) and clears the partner counter
    float* rn = a.rnorm + (int64_t)head * a.n_pad + j0 + rbase;
#pragma unroll
    for (int m = 0; m < 8; ++m) rn[m * 16] = r8[m];
    if (a.credit) {
      unsigned long long* cr = a.credit + (int64_t)head * a.n_pad + j0 + rbase;
#pragma unroll
      for (int m = 0; m < 8; ++m) cr[m * 16] = 0ull;
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) uacc[e] = pair_sum32(pair_sum16(uacc[e]));
  if (lane < 16) {
#pragma unroll
    for (int e = 0; e < 8; ++e) ured[wave][lane * 8 + e] = uacc[e];
  }
  __syncthreads();
  if (t < kHeadDim) {
    const float s = (ured[0][t] + ured[1][t]) + (ured[2][t] + ured[3][t]);
    a.upart[((int64_t)head * a.chunks + chunk) * kHeadDim + t] = s;
  }

  if constexpr (HAS_Q) {
    // ---- logits: A = the G*alpha query rows of this KV head, B = 32 keys per wave
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
    const int lrow = lane & 31;
    const int khalf = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + (wave * 32 + lrow) * kLdsRowBytes + kk * 32 + khalf * 16);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[mt][kk], kf, acc[mt], 0, 0, 0);
    }
    if constexpr (AH > 0) {
      // accumulator element i of row tile mt: key = lane % 32 of this wave's 32 keys, query row
      // g * alpha + j with g = mt * (16 / AH) + i / AH and j = 8 * ((i % AH) / 4) + 4 * (lane / 32) + i % 4
      const int key = j0 + wave * 32 + lrow;
      const bool valid = key < a.n;
      float* lgt = a.logit + (int64_t)head * a.alpha * a.n_pad + key;
      float* st = a.stats + ((int64_t)head * a.chunks * 4 + chunk * 4 + wave) * a.alpha * 2;
      // stage by stage over the lane's AH query rows, so that the cross-lane steps of different rows
      // are in flight together
      float m[AH], mx[AH], e[AH];
#pragma unroll
      for (int i = 0; i < AH; ++i) {
        // scaled first (the scale is positive, so the maximum is the same float): products are known to the
        // compiler as ordinary numbers and the maxima below stay single instructions
        m[i] = acc[0][i] * a.scale;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int iq = 0; iq < 16 / AH; ++iq)
            if (mt * (16 / AH) + iq > 0 && mt * (16 / AH) + iq < a.G) m[i] = fmaxf(m[i], acc[mt][i + iq * AH] * a.scale);
        if (valid) lgt[(int64_t)(8 * (i >> 2) + 4 * khalf + (i & 3)) * a.n_pad] = m[i];
      }
      // (max, sum exp) over the wave's 32 keys of each row
#pragma unroll
      for (int i = 0; i < AH; ++i) mx[i] = half_wave_max(valid ? m[i] : -INFINITY);
#pragma unroll
      for (int i = 0; i < AH; ++i) e[i] = half_wave_sum(valid ? __expf(m[i] - mx[i]) : 0.f);
      if (lrow == 0) {
#pragma unroll
        for (int i = 0; i < AH; ++i) {
          const int j = 8 * (i >> 2) + 4 * khalf + (i & 3);
          *reinterpret_cast<float2*>(st + j * 2) = make_float2(mx[i], e[i]);
        }
      }
    } else {
    __syncthreads();      // all key fragments are in registers: the tile can be overwritten
    // accumulator layout: column (key) = lane % 32, row (query) = 8*(i/4) + 4*(lane/32) + i%4
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int qrow = mt * 32 + 8 * (i >> 2) + 4 * khalf + (i & 3);
        lg[qrow][wave * 32 + lrow] = acc[mt][i] * a.scale;
      }
    __syncthreads();
    // ---- max over the G query heads of the group, per (query position j, key); when the heads are
    // merged after their softmax (App. A.2) every head's row is written as it is (out_groups = 1)
    {
      const int key = t & (kChunk - 1);
      const bool valid = (j0 + key) < a.n;
      for (int j = t >> 7; j < a.out_rows; j += kPrepassThreads / kChunk) {
        float m = lg[j][key];
        for (int g = 1; g < a.out_groups; ++g) m = fmaxf(m, lg[g * a.out_rows + j][key]);
        if (valid) a.logit[((int64_t)head * a.out_rows + j) * a.n_pad + j0 + key] = m;
        lg[j][key] = valid ? m : -INFINITY;      // row j (g = 0) is read by this thread only
      }
    }
    __syncthreads();
    // ---- per-chunk softmax statistics for each written row
    for (int j = wave; j < a.out_rows; j += 4) {
      const float x0 = lg[j][lane], x1 = lg[j][lane + 64];
      const float m = full_wave_max(fmaxf(x0, x1));
      // exp(-inf) = 0 for masked keys; key j0 is always valid
      const float s = full_wave_sum(__expf(x0 - m) + __expf(x1 - m));
      if (lane == 0) {
        float* st = a.stats + (((int64_t)head * a.chunks + chunk) * a.out_rows + j) * 2;
        st[0] = m;
        st[1] = s;
      }
    }
    }  // general path
  }
  __syncthreads();          // the tiles are rewritten by the next item
  }  // items
}

// As many workgroups as stay resident at once (queried once per kernel variant), each walking over
// its share of the items.
template <bool HAS_Q, int MT, int AH, bool PAGED>
void launch_paged(const PrepassArgs& a, hipStream_t stream) {
  static const int res = [] {
    int per_cu = 0;
    const void* fn = reinterpret_cast<const void*>(&prepass_kernel<HAS_Q, MT, AH, PAGED>);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kPrepassThreads, 0) != hipSuccess || per_cu < 1) per_cu = 2;
    return per_cu * device_compute_units();
  }();
  // a multiple of 8 workgroups, at most one per item of the XCD with the most heads
  const int per_xcd = std::max(1, std::min(((a.items / a.chunks + 7) / 8) * a.chunks, res / 8));
  const dim3 grid((unsigned)(8 * per_xcd)), block(kPrepassThreads);
  hipLaunchKernelGGL((prepass_kernel<HAS_Q, MT, AH, PAGED>), grid, block, 0, stream, a);
}

template <bool HAS_Q, int MT, int AH>
void launch_variant(const PrepassArgs& a, hipStream_t stream) {
  if (a.table != nullptr) launch_paged<HAS_Q, MT, AH, true>(a, stream);
  else launch_paged<HAS_Q, MT, AH, false>(a, stream);
}

}  // namespace

int prepass_register_path(const Plan& pl) {
  const bool usual = pl.alpha == 8 || pl.alpha == 16 || pl.alpha == 32;
  if (!usual || pl.gqa_mode != 0) return 0;
  // alpha / 2, plus 100 when the G * alpha query rows need two MFMA row tiles (alpha = 32 then has
  // G = 2, a case left to the general path)
  if (pl.G * pl.alpha <= 32) return pl.alpha / 2;
  return pl.alpha <= 16 ? pl.alpha / 2 + 100 : 0;
}

hipError_t launch_prepass(const Plan& pl, const void* q_obs, const void* k, char* ws, hipStream_t stream) {
  PrepassArgs a;
  a.q = static_cast<const uint16_t*>(q_obs);
  a.k = static_cast<const uint16_t*>(k);
  a.rnorm = reinterpret_cast<float*>(ws + pl.off_rnorm);
  a.upart = reinterpret_cast<float*>(ws + pl.off_upart);
  a.credit = (pl.recency_transposed || pl.triangular) ? reinterpret_cast<unsigned long long*>(ws + pl.off_credit) : nullptr;
  a.logit = reinterpret_cast<float*>(ws + pl.off_logit);
  a.stats = reinterpret_cast<float*>(ws + pl.off_stats);
  a.H = pl.H; a.G = pl.G; a.alpha = pl.alpha; a.n = pl.n; a.n_pad = pl.n_pad; a.chunks = pl.chunks;
  a.out_rows = pl.qrows; a.out_groups = (pl.gqa_mode == 0) ? pl.G : 1;
  a.table = pl.paged ? pl.block_table : nullptr;
  a.page_shift = pl.page_shift; a.table_stride = pl.table_stride; a.kspage = pl.kspage;
  a.kdense = pl.paged ? reinterpret_cast<uint16_t*>(ws + pl.off_kdense) : nullptr;
  a.ksp = pl.ksp; a.ksh = pl.ksh; a.kst = pl.kst;
  a.qsp = pl.qsp; a.qsh = pl.qsh; a.qst = pl.qst;
  a.eps = pl.eps;
  a.scale = 1.0f / sqrtf((float)kHeadDim);
  a.items = pl.heads * pl.chunks;
  const int fast = prepass_register_path(pl);      // alpha / 2, or 0
  if (q_obs == nullptr) launch_variant<false, 1, 0>(a, stream);
  else if (fast == 4) launch_variant<true, 1, 4>(a, stream);
  else if (fast == 8) launch_variant<true, 1, 8>(a, stream);
  else if (fast == 16) launch_variant<true, 1, 16>(a, stream);
  else if (fast == 104) launch_variant<true, 2, 4>(a, stream);
  else if (fast == 108) launch_variant<true, 2, 8>(a, stream);
  else if (pl.G * pl.alpha <= 32) launch_variant<true, 1, 0>(a, stream);
  else launch_variant<true, 2, 0>(a, stream);
  return hipGetLastError();
}

}  // namespace rkv
