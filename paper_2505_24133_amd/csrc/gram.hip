// Redundancy pass (Sec. 3.3): the n x n cosine-similarity matrix of one head's candidate keys
// is formed tile by tile with bf16 MFMA (fp32 accumulation) and consumed in registers; it is
// never written to memory.
//
// What the pass has to extract from the matrix is small: per token i the (up to) beta
// largest-index partners j with S_ij > T and their similarities.  The plain row sums are known
// in closed form from the pre-pass,  sum_{j != i} S_ij = r_i K_i . u - (r_i |K_i|)^2  with
// u = sum_j r_j K_j, so the mean similarity of Eq. 6 is
//     S-bar_i = ( r_i K_i . u - (r_i |K_i|)^2 - sum_{j in forgiven(i)} S_ij ) / n .
// Column tiles are visited in DESCENDING j, so the first beta hits a row meets are its beta
// most recent similar tokens; a row that has met beta hits gets threshold +inf.
//
// Work split: a workgroup owns 64 * NW consecutive rows (each wave 64 rows, held as MFMA A
// fragments in registers for the whole pass) and streams all column tiles (64 keys) of the
// head through double-buffered LDS.  Per 32x32 tile the common-case epilogue is one FMA per
// element (acc * r_j - T / r_i) folded into a running max, then one wave-wide test.
#include "rkv_internal.h"

namespace rkv {

namespace {

constexpr int kTileCols = 64;

struct GramArgs {
  const uint16_t* k;
  const float* rnorm;
  const float* upart;
  float* sbar;
  int H, heads, n, n_pad, chunks, beta, row_blocks;
  int64_t ksp, ksh, kst;
  float T, eps;
};

template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void gram_kernel(GramArgs a) {
  constexpr int NT = NW * 64;
  constexpr int BM = NW * 64;
  constexpr int PIECES = kTileCols * 16;                  // 16-byte pieces per column tile
  constexpr int LPT = (PIECES + NT - 1) / NT;             // pieces per thread

  __shared__ __attribute__((aligned(16))) unsigned char kt[2][kTileCols * kLdsRowBytes];
  __shared__ float rjl[2][kTileCols];
  __shared__ float ul[kHeadDim];
  __shared__ float rowdot[BM];
  __shared__ float sub[BM];
  __shared__ int cnt[BM];

  // Workgroups are dealt round-robin to the 8 XCDs; give every XCD whole heads so that a head's
  // keys are fetched into one L2 only.
  const int b = blockIdx.x;
  const int xcd = b & 7;
  const int q = b >> 3;
  const int head = (q / a.row_blocks) * 8 + xcd;
  const int rb = q % a.row_blocks;
  if (head >= a.heads) return;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int lrow = lane & 31;
  const int half = lane >> 5;
  const int p = head / a.H;
  const int h = head - p * a.H;
  const uint16_t* kbase = a.k + p * a.ksp + h * a.ksh;
  const float* rn = a.rnorm + (int64_t)head * a.n_pad;
  const int n = a.n;
  const int i0 = rb * BM + wave * 64;

  // ---- prologue
  if (t < kHeadDim) {
    const float* up = a.upart + (int64_t)head * a.chunks * kHeadDim + t;
    float s = 0.f;
    for (int c = 0; c < a.chunks; ++c) s += up[(int64_t)c * kHeadDim];
    ul[t] = s;
  }
  for (int i = t; i < BM; i += NT) { sub[i] = 0.f; cnt[i] = 0; }

  bf16x8 af[2][8];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int row = i0 + rt * 32 + lrow;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      uint4 x = make_uint4(0, 0, 0, 0);
      if (row < n) x = *reinterpret_cast<const uint4*>(kbase + (int64_t)row * a.kst + kk * 16 + half * 8);
      __builtin_memcpy(&af[rt][kk], &x, 16);
    }
  }
  float thr[2][16];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = i0 + rt * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
      thr[rt][i] = (row < n && a.beta > 0) ? a.T / rn[row] : INFINITY;
    }
  __syncthreads();
  // K_i . u for the wave's 64 rows (each lane holds half of a row's elements)
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    float s = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf((float)af[rt][kk][e], ul[kk * 16 + half * 8 + e], s);
    s += __shfl_xor(s, 32);
    if (half == 0) rowdot[wave * 64 + rt * 32 + lrow] = s;
  }

  // ---- stream the column tiles, most recent first
  const int nct = (a.beta > 0) ? (n + kTileCols - 1) / kTileCols : 0;
  uint4 stage[LPT];
  float stage_r = 0.f;
  auto load_tile = [&](int ct) {
#pragma unroll
    for (int m = 0; m < LPT; ++m) {
      const int piece = t + m * NT;
      const int row = piece >> 4, c16 = piece & 15;
      const int grow = ct * kTileCols + row;
      stage[m] = make_uint4(0, 0, 0, 0);
      if (piece < PIECES && grow < n)
        stage[m] = *reinterpret_cast<const uint4*>(kbase + (int64_t)grow * a.kst + c16 * 8);
    }
    if (t < kTileCols) {
      const int grow = ct * kTileCols + t;
      stage_r = (grow < n) ? rn[grow] : 0.f;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int m = 0; m < LPT; ++m) {
      const int piece = t + m * NT;
      const int row = piece >> 4, c16 = piece & 15;
      if (piece < PIECES) *reinterpret_cast<uint4*>(kt[buf] + row * kLdsRowBytes + c16 * 16) = stage[m];
    }
    if (t < kTileCols) rjl[buf][t] = stage_r;
  };

  if (nct > 0) {
    load_tile(nct - 1);
    store_tile(0);
  }
  __syncthreads();

  for (int it = 0; it < nct; ++it) {
    const int ct = nct - 1 - it;
    const int buf = it & 1;
    if (it + 1 < nct) load_tile(ct - 1);

#pragma unroll
    for (int s = 1; s >= 0; --s) {
      const int c0 = ct * kTileCols + s * 32;
      bf16x8 bfr[8];
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        bfr[kk] = *reinterpret_cast<const bf16x8*>(kt[buf] + (s * 32 + lrow) * kLdsRowBytes + kk * 32 + half * 16);
      const float rj = rjl[buf][s * 32 + lrow];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rt][kk], bfr[kk], acc, 0, 0, 0);
        // common case: no unsaturated row of this tile has a partner above the threshold
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; i += 2)
          m = fmaxf(m, fmaxf(fmaf(acc[i], rj, -thr[rt][i]), fmaf(acc[i + 1], rj, -thr[rt][i + 1])));
        if (__any(m > 0.f)) {
          // rare case: rank the hits of each row by column (descending) and forgive the first ones
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int rl = wave * 64 + rt * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
            const int row = rb * BM + rl;
            const float tv = acc[i] * rj;
            const bool hit = (tv > thr[rt][i]) && (row != c0 + lrow);
            const unsigned long long mask = __ballot(hit);
            if (mask != 0ull) {
              const uint32_t hm = half ? (uint32_t)(mask >> 32) : (uint32_t)mask;
              if (hm != 0u) {
                const int c = cnt[rl];
                const int room = a.beta - c;
                const int ntake = min((int)__popc(hm), room);
                uint32_t rem = hm;
                float sacc = 0.f;
                for (int z = 0; z < ntake; ++z) {
                  const int src = 31 - __clz(rem);
                  rem &= ~(1u << src);
                  sacc += __shfl(tv, (lane & 32) | src);
                }
                // every lane of the half-wave holds the same values and stores them
                sub[rl] = sub[rl] + sacc;
                cnt[rl] = c + ntake;
                if (c + ntake >= a.beta) thr[rt][i] = INFINITY;
              }
            }
          }
        }
      }
    }

    if (it + 1 < nct) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- closed-form row sums minus the forgiven similarities
  for (int i = t; i < BM; i += NT) {
    const int row = rb * BM + i;
    if (row < n) {
      const float r = rn[row];
      const float self = 1.0f - a.eps * r;               // r_i |K_i| = 1 - eps r_i
      const float total = r * rowdot[i] - self * self - r * sub[i];
      a.sbar[(int64_t)head * a.n_pad + row] = total / (float)n;
    }
  }
}

}  // namespace

hipError_t launch_gram(const Plan& pl, const void* k, char* ws, hipStream_t stream) {
  GramArgs a;
  a.k = static_cast<const uint16_t*>(k);
  a.rnorm = reinterpret_cast<const float*>(ws + pl.off_rnorm);
  a.upart = reinterpret_cast<const float*>(ws + pl.off_upart);
  a.sbar = reinterpret_cast<float*>(ws + pl.off_sbar);
  a.H = pl.H; a.heads = pl.heads; a.n = pl.n; a.n_pad = pl.n_pad; a.chunks = pl.chunks; a.beta = pl.beta;
  a.ksp = pl.ksp; a.ksh = pl.ksh; a.kst = pl.kst;
  a.T = pl.T; a.eps = pl.eps;
  // rows per workgroup: 256 unless 192 wastes fewer padded rows
  const int rb4 = (pl.n + 255) / 256, rb3 = (pl.n + 191) / 192;
  const bool use3 = rb3 * 192 < rb4 * 256;
  a.row_blocks = use3 ? rb3 : rb4;
  const int head_groups = (pl.heads + 7) / 8;
  const dim3 grid((unsigned)((int64_t)head_groups * a.row_blocks * 8));
  if (use3) {
    hipLaunchKernelGGL((gram_kernel<3>), grid, dim3(192), 0, stream, a);
  } else {
    hipLaunchKernelGGL((gram_kernel<4>), grid, dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace rkv
