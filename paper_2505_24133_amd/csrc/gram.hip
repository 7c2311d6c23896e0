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
// Work split: a workgroup owns NW * RT * 32 consecutive rows.  Each wave keeps its RT * 32 rows as
// the MFMA *B* operand in registers for the whole pass, so a lane owns ONE row per row tile and
// the row's state (threshold T / r_i, hits taken, forgiven sum) lives in three registers.  The
// head's keys stream through double-buffered LDS as the MFMA *A* operand in tiles of TC keys,
// copied global -> LDS by the DMA path (no staging registers) into an XOR-swizzled layout that
// the 16-byte fragment reads hit without bank conflicts.  Per 32x32 tile the common-case
// epilogue is one multiply per element folded into a running max, issued in the shadow of the
// next tile's MFMA chain; K_i . u comes from three extra pseudo-keys (u split into bf16 pieces).
#include <algorithm>
#include <type_traits>

#include "rkv_internal.h"

#include "gram_index.h"

namespace rkv {

namespace {

extern __shared__ __attribute__((aligned(1024))) unsigned char gram_lds[];

struct GramArgs {
  const uint16_t* k;
  const float* rnorm;
  const float* upart;
  float* sbar;
  unsigned long long* credit;   // [heads][n_pad] or nullptr: forgiven similarities charged to the partner
  int* part_cnt;                // [heads][parts][n_pad] hits per row found by one column part
  float* part_pre;              // [heads][parts][n_pad] their sum
  int H, heads, n, n_pad, chunks, beta;
  int row_blocks, parts;        // workgroups per head = row_blocks * parts
  int64_t ksp, ksh, kst;
  float T, eps;
};

constexpr int kPseudoBytes = 3 * kRowBytes;     // u as three bf16 pseudo-keys

// 16-byte slot of (row, chunk) inside a tile: rows are 256 bytes, chunks XOR-swizzled by the row, so
// that 16 consecutive rows read at the same chunk fall into 16 different bank groups.
__device__ __forceinline__ int slot_offset(int row, int chunk) { return row * kRowBytes + ((chunk ^ (row & 15)) << 4); }

// One wave-wide DMA copy: lane l fetches 16 bytes at base + voff and the hardware stores them
// at LDS address lds_base + 16 * l.  Issued as inline assembly so that the compiler does not
// serialise later LDS reads of the *other* buffer behind it; completion is awaited explicitly
// (vmcnt) before the barrier that publishes the buffer.  M0 is written here and declared clobbered.
__device__ __forceinline__ void dma16(const void* base, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_base), "v"(voff), "s"(base)
               : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void* base, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2"
               :
               : "s"(lds_base), "v"(voff), "s"(base)
               : "memory", "m0");
}

// Kernel variants (the common one carries none of the others' code):
//   kPlain       one workgroup scans all columns of its rows and writes the mean similarity
//   kSplit       the scan is shared by several workgroups, each reports what it found (beta = 1)
//   kTransposed  forgiven similarities are charged to the recent partner's counter
//   kTriangular  only entries with key < row are looked at (the matrix is symmetric): a row block scans the
//                column tiles up to its own; an entry above T is reported to both of its tokens (beta = 1)
enum GramVariant : int { kPlain = 0, kSplit = 1, kTransposed = 2, kTriangular = 3 };
// SKIP adds the exact shortcut: a row that has met beta partners can gain nothing from the columns still
// to come, so a wave whose rows are all done stops forming tiles, a workgroup whose rows are all done
// leaves the scan, and when the rows still open fit into half as many row tiles as are in use they are
// gathered into the first waves (one row tile each) and the other waves only help copying tiles.

constexpr int kCompactBytes = 3072;             // SKIP: open-row counts of the waves and the records of moved rows

template <int NW, int RT, int TC, int WPS, int VARIANT, bool SKIP, bool B1>
__global__ __launch_bounds__(NW * 64, WPS) void gram_kernel(GramArgs a) {
  // WPS = waves per SIMD the register budget is cut for.  With two row tiles per wave there is room for two
  // sets of key fragments and r_j (the next subtile's are fetched a step ahead); with three row tiles (or
  // three waves per SIMD) one set is kept and refilled fragment by fragment behind the subtile's last chain.
  constexpr int KB = (WPS >= 3 || RT >= 3) ? 1 : 2;
  constexpr int NT = NW * 64;
  constexpr int BM = NW * RT * 32;
  constexpr int NS = TC / 32;                       // 32-key subtiles per tile
  constexpr int LOADS = TC / 4;                     // wave-wide DMA copies per tile (4 rows each)
  static_assert(NW == 2 || NW == 4, "the DMA split assumes 2 or 4 waves");
  static_assert(RT >= 2, "the r_j prefetch needs at least two row tiles per wave");
  static_assert(LOADS % NW == 0, "tile rows must split evenly over the waves");
  // LDS map: [pseudo-keys | tile 0 | tile 1 | r_j of tile 0 | r_j of tile 1 | SKIP: counts, row records]
  constexpr int OFF_TILE = kPseudoBytes;
  constexpr int TILE_SPAN = LOADS * 1024;            // bytes the DMA copies of one tile cover
  constexpr int OFF_RJ = OFF_TILE + 2 * TILE_SPAN;
  constexpr int OFF_CNT = OFF_RJ + 2 * TC * 4;       // two sets of NW open-row counts (by iteration parity)
  constexpr int OFF_REC = OFF_CNT + 64;              // NW * 32 records of 5 words
  static_assert(64 + NW * 32 * 20 <= kCompactBytes && 2 * NW * 4 <= 64, "record area");

  // Workgroups are dealt round-robin to the 8 XCDs; give every XCD whole heads so that a head's
  // keys are fetched into one L2 only.  A head's workgroups (row block x column part) are adjacent.
  const int b = blockIdx.x;
  const int xcd = b & 7;
  const int q = b >> 3;
  const int parts = (VARIANT == kSplit) ? a.parts : 1;
  const int per_head = a.row_blocks * parts;
  const int head = (q / per_head) * 8 + xcd;
  const int rem = q % per_head;
  const int rb = rem / parts;
  const int part = rem - rb * parts;
  if (head >= a.heads) return;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int lrow = lane & 31;
  const int half = lane >> 5;
  const int p = head / a.H;
  const int h = head - p * a.H;
  // the head's key base is workgroup-uniform; pinning it to scalar registers here keeps every DMA
  // address computation below on the scalar unit
  const uint64_t kb64 = (uint64_t)(uintptr_t)(a.k + p * a.ksp + h * a.ksh);
  const uint16_t* kbase = reinterpret_cast<const uint16_t*>(
      ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(kb64 >> 32)) << 32) |
      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)kb64));
  const float* rn = a.rnorm + (int64_t)head * a.n_pad;
  const int n = a.n;
  // Row tiles of this block that hold candidates, dealt to the waves in runs of `rte` tiles: a full block
  // gives every wave RT tiles; a last block with fewer rows gives every wave fewer (its other row tiles
  // stand for rows past n), and the scan below then runs with that many chains per subtile, so the
  // workgroup lives correspondingly shorter.
  const int rtc = min((n - rb * BM + 31) >> 5, NW * RT);
  const int rte = (rtc + NW - 1) / NW;                 // 1 .. RT, the same for every wave of the workgroup
  const int i0 = rb * BM + wave * rte * 32;
  auto tile_row0 = [&](int rt) -> int { return rt < rte ? i0 + rt * 32 : (1 << 20); };   // first row of the wave's row tile rt
  bool active = i0 < n;                              // wave-uniform: does this wave own any candidate row?
  const uint32_t lds0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)gram_lds);   // LDS byte address of the dynamic segment
  const uint32_t row_bytes = (uint32_t)a.kst * 2u;

  // Copy tile `ct` (keys ct*TC ...) and its r_j into buffer `buf`.  Keys past n are read from
  // row n-1 (any finite row will do: their r_j is 0).
  // One wave-wide DMA copy (4 rows) of tile `ct` into buffer `buf`; each wave issues LOADS / NW of them.
  // Only a part's first tile can reach past n through a copy that is read (CLAMP); for the others the row
  // part of the address is wave-uniform and goes into the scalar base, leaving one per-lane offset
  // register.  gram_index.h holds the row arithmetic (and says why no row index reaches n).
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  // chunk that belongs in this lane's LDS slot: rows wave*4 + jj*16 + lane/16 differ by multiples of 16 between
  // the wave's copies, so the swizzle (row & 15) and with it the lane's byte offset is the same for all of them
  const int lane_chunk = (lane & 15) ^ ((wave * 4 + (lane >> 4)) & 15);
  auto issue_rows_clamped = [&](int ct, int buf, int jj) {
    const int row0 = (wave_s + jj * NW) * 4;                   // first of the 4 rows, inside the tile
    const uint32_t dst = lds0 + OFF_TILE + buf * TILE_SPAN + row0 * kRowBytes;
    const int key = gram_copy_row_clamped(ct, TC, row0, lane, n);
    dma16(kbase, (uint32_t)key * row_bytes + (uint32_t)lane_chunk * 16u, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst));
  };
  // Unclamped form, used inside the scan: per tile one scalar source pointer (the wave's first row of the
  // tile) and one scalar LDS address; the wave's copies lie 16 rows apart in both.
  const uint32_t lane_off = (uint32_t)gram_copy_lane_row(lane, n) * row_bytes + (uint32_t)lane_chunk * 16u;
  const uint32_t group_step = (uint32_t)gram_copy_group_row(16, TC, n) * row_bytes;
  auto tile_source = [&](int ct) -> uint64_t {
    const int row = gram_copy_tile_row0(ct, TC, n) + gram_copy_group_row(wave_s * 4, TC, n);
    const uint64_t addr = (uint64_t)(uintptr_t)kbase + (uint64_t)(uint32_t)row * row_bytes;
    // wave-uniform by construction; readfirstlane returns a signed int, so each half is narrowed to
    // uint32_t before widening (a sign-extended low half would overwrite the high half)
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(addr >> 32));
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
    return ((uint64_t)hi << 32) | (uint64_t)lo;
  };
  auto issue_rows = [&](uint64_t src, uint32_t dst, int jj) {
    dma16(reinterpret_cast<const void*>(src + (uint64_t)((uint32_t)jj * group_step)), lane_off,
          dst + (uint32_t)(jj * NW * 4 * kRowBytes));
  };
  auto issue_rj = [&](int ct, int buf) {
    if (wave < TC / 64)
      dma4(rn + ct * TC, (uint32_t)(wave * 64 + lane) * 4u,
           __builtin_amdgcn_readfirstlane(lds0 + OFF_RJ + buf * TC * 4 + wave * 256));
  };
  auto issue_tile = [&](int ct, int buf) {
#pragma unroll
    for (int jj = 0; jj < LOADS / NW; ++jj) issue_rows_clamped(ct, buf, jj);
    issue_rj(ct, buf);
  };
  // this workgroup's share of the column tiles: [ct_lo, ct_hi), scanned from ct_hi - 1 downwards
  const int nct_all = (a.beta > 0) ? (n + TC - 1) / TC : 0;
  int ct_lo, ct_hi;
  gram_part_range(part, parts, nct_all, &ct_lo, &ct_hi);
  if constexpr (VARIANT == kTriangular) {
    // nothing newer than the block's last row is needed: its mirror entry belongs to another row
    ct_hi = min(ct_hi, (min(rb * BM + BM, n) - 1) / TC + 1);
  }
  const int nct = ct_hi - ct_lo;
  const bool split = parts > 1 || VARIANT == kTriangular;   // rows report to the finalize kernel instead of closing their sum
  const bool closing = part == parts - 1;           // the part that also writes the closed-form row sums
  if (nct > 0) issue_tile(ct_hi - 1, 0);

  // ---- prologue: u -> three bf16 pseudo-keys, the wave's rows -> registers.  Every global load of
  // the prologue is issued before anything waits for one of them (one memory latency, not four):
  // rows past n read row n - 1 (their results are never written and their threshold is +inf).
  bf16x8 res[RT][8];
  float thr[RT], sub[RT], rowdot[RT], rni[RT];
  int cnt[RT];
  int rowid[RT];                                     // SKIP: the row a lane works for (-1: none); rows can move
  auto row_of = [&](int rt) -> int {
    if constexpr (SKIP) return rowid[rt];
    else return tile_row0(rt) + lrow;
  };
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int rowc = min(tile_row0(rt) + lrow, n - 1);
    rni[rt] = rn[rowc];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const uint4 x = *reinterpret_cast<const uint4*>(kbase + (int64_t)rowc * a.kst + kk * 16 + half * 8);
      __builtin_memcpy(&res[rt][kk], &x, 16);
    }
  }
  {
    // u = sum of the pre-pass's per-chunk partials, in a fixed order; all threads load in parallel,
    // eight chunks per thread in flight
    constexpr int GROUPS = NT / kHeadDim;
    float* ured = reinterpret_cast<float*>(gram_lds + OFF_TILE + TILE_SPAN);   // tile 1 is not in use yet
    const int e = t & (kHeadDim - 1), grp = t >> 7;
    const float* up = a.upart + (int64_t)head * a.chunks * kHeadDim + e;
    float usum = 0.f;
    for (int c0 = grp; c0 < a.chunks; c0 += 8 * GROUPS) {
      float x[8];
#pragma unroll
      for (int q2 = 0; q2 < 8; ++q2) x[q2] = up[(int64_t)min(c0 + q2 * GROUPS, a.chunks - 1) * kHeadDim];
#pragma unroll
      for (int q2 = 0; q2 < 8; ++q2) x[q2] = (c0 + q2 * GROUPS < a.chunks) ? x[q2] : 0.f;
      usum += ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
    }
    ured[t] = usum;
  }
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int row = tile_row0(rt) + lrow;
    thr[rt] = (row < n && a.beta > 0) ? a.T / rni[rt] : INFINITY;
    sub[rt] = 0.f;
    cnt[rt] = 0;
    rowdot[rt] = 0.f;
    rowid[rt] = row < n ? row : -1;
  }
  __syncthreads();
  if (t < kHeadDim) {
    constexpr int GROUPS = NT / kHeadDim;
    const float* ured = reinterpret_cast<const float*>(gram_lds + OFF_TILE + TILE_SPAN);
    float u = ured[t];
#pragma unroll
    for (int g = 1; g < GROUPS; ++g) u += ured[t + g * kHeadDim];
#pragma unroll
    for (int piece = 0; piece < 3; ++piece) {
      uint32_t bits = __float_as_uint(u);
      bits += 0x7fffu + ((bits >> 16) & 1u);                  // round to nearest even bf16
      const uint16_t hb = (uint16_t)(bits >> 16);
      u -= __uint_as_float((uint32_t)hb << 16);               // exact remainder
      *reinterpret_cast<uint16_t*>(gram_lds + slot_offset(piece, t >> 3) + (t & 7) * 2) = hb;
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // 16-byte A-operand fragments of subtile s: key row lane%32, k-slice (kk, lane/32)
  auto read_k = [&](bf16x8 (&kf)[8], const unsigned char* tile, int s) {
    const int row = s * 32 + lrow;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      kf[kk] = *reinterpret_cast<const bf16x8*>(tile + slot_offset(row, kk * 2 + half));
  };
  // r_j of the 16 keys this lane sees in its accumulator: key = 8*(i/4) + 4*half + i%4
  auto read_rj = [&](float (&rj)[16], const float* rjs, int s) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 v = *reinterpret_cast<const float4*>(rjs + s * 32 + g * 8 + half * 4);
      rj[4 * g] = v.x; rj[4 * g + 1] = v.y; rj[4 * g + 2] = v.z; rj[4 * g + 3] = v.w;
    }
  };
  auto chain = [&](const bf16x8 (&kf)[8], const bf16x8 (&rf)[8]) -> f32x16 {
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], rf[kk], acc, 0, 0, 0);
    return acc;
  };
  // The last chain on a subtile's fragments, single fragment set: as soon as step kk has been issued its
  // fragment register is refilled with the next subtile's, which gives every refill about eight MFMA
  // issue slots before the next subtile's first chain needs it.
  auto chain_refill = [&](bf16x8 (&kf)[8], const bf16x8 (&rf)[8], const unsigned char* tile, int s_next) -> f32x16 {
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    const int row = s_next * 32 + lrow;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], rf[kk], acc, 0, 0, 0);
      kf[kk] = *reinterpret_cast<const bf16x8*>(tile + slot_offset(row, kk * 2 + half));
    }
    return acc;
  };
  // K_i . u = sum of the three pseudo-key columns (accumulator elements 0..2 of lanes with half == 0)
  if (active && closing) {
    bf16x8 pf[8];
    read_k(pf, gram_lds, 0);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const f32x16 acc = chain(pf, res[rt]);
      rowdot[rt] = (acc[2] + acc[1]) + acc[0];
      asm volatile("" : "+v"(rowdot[rt]));       // settle the sum now; the accumulator is dead after this
    }
  }

  // Common-case test of one tile: max over the lane's 16 keys of acc * r_j (compare with T / r_i).
  auto tile_max = [&](const f32x16& acc, const float (&rj)[16]) -> float {
    float m = acc[0] * rj[0];
#pragma unroll
    for (int i = 1; i < 16; i += 3) m = fmaxf(m, fmaxf(acc[i] * rj[i], fmaxf(acc[i + 1] * rj[i + 1], acc[i + 2] * rj[i + 2])));
    return m;
  };
  // Rare case: the row's hits in this tile, ranked by key (descending); forgive the first ones.
  auto tile_hits = [&](const f32x16& acc, const float (&rj)[16], int rt, int c0) {
    const int row = row_of(rt);
    // Accumulator element i holds key c0 + 8*(i/4) + 4*half + i%4.  Masks are built with the bit
    // positions of half 0 (compile-time constants) and shifted by 4*half once.
    float tv[16];
    uint32_t mine0 = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      tv[i] = acc[i] * rj[i];
      if (tv[i] > thr[rt]) mine0 |= 1u << (8 * (i >> 2) + (i & 3));
    }
    uint32_t mine = mine0 << (4 * half);
    const int self = row - c0;                                   // the diagonal, if it is in this tile
    if (self >= 0 && self < 32) mine &= ~(1u << self);
    // the two lanes of a row (l and l ^ 32) exchange their hit masks with a row swap, not through LDS
    const auto both = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    const uint32_t all = both[0] | both[1];
    if (all != 0u) {
      const int room = a.beta - cnt[rt];
      uint32_t rem = all, sel = 0;
      int taken = 0;
      while (rem != 0u && taken < room) {
        const uint32_t bit = 1u << (31 - __clz(rem));
        sel |= bit;
        rem &= ~bit;
        ++taken;
      }
      const uint32_t take0 = (sel & mine) >> (4 * half);
      if (VARIANT == kTransposed) {
        // the other direction of the rule: the similarity leaves the recent partner's sum, not this
        // row's.  Integer atomics (units of 2^-40) keep the total independent of the arrival order.
        const float r_i = rn[row];
        unsigned long long* cr = a.credit + (int64_t)head * a.n_pad + c0 + 4 * half;
#pragma unroll
        for (int i = 15; i >= 0; --i)
          if ((take0 >> (8 * (i >> 2) + (i & 3))) & 1u)
            atomicAdd(cr + 8 * (i >> 2) + (i & 3), (unsigned long long)(tv[i] * r_i * 1099511627776.0f));
      } else {
      // sum of the lane's taken similarities, most recent first: each is fetched by a four-level
      // select on the bits of its accumulator index (usually one per row, often none in this lane)
      float s = 0.f;
      uint32_t left = take0;
      while (left != 0u) {
        const int pos = 31 - __clz(left);                      // bit position = 8*(i/4) + i%4
        left &= ~(1u << pos);
        const bool b0 = pos & 1, b1 = pos & 2, b2 = pos & 8, b3 = pos & 16;
        const float l0 = b0 ? tv[1] : tv[0], l1 = b0 ? tv[3] : tv[2], l2 = b0 ? tv[5] : tv[4], l3 = b0 ? tv[7] : tv[6];
        const float l4 = b0 ? tv[9] : tv[8], l5 = b0 ? tv[11] : tv[10], l6 = b0 ? tv[13] : tv[12], l7 = b0 ? tv[15] : tv[14];
        const float m0 = b1 ? l1 : l0, m1 = b1 ? l3 : l2, m2 = b1 ? l5 : l4, m3 = b1 ? l7 : l6;
        const float n0 = b2 ? m1 : m0, n1 = b2 ? m3 : m2;
        s += b3 ? n1 : n0;
      }
      s = pair_sum32(s);                         // both lanes of the row end with the same sum
      sub[rt] += s;
      }
      cnt[rt] += taken;
      if (cnt[rt] >= a.beta) thr[rt] = INFINITY;
    }
  };
  // Triangular scan (beta = 1): every entry above T with key < row is (a) a candidate for the row's most
  // recent OLDER partner, of which the first one met in the descending scan is kept, and (b) a NEWER partner
  // of the key's token: the largest row index wins a 64-bit atomic maximum (row << 32 | similarity bits; a
  // similarity above T >= 0 is a positive float, whose bit pattern orders like its value).  The row's
  // threshold stays as it is: later entries may still matter to their key.
  auto tile_triangular = [&](const f32x16& acc, const float (&rj)[16], int rt, int c0) {
    const int row = row_of(rt);
    const float r_i = rni[rt];
    int keyl = row - c0 - 4 * half;                          // keys of this lane's numbering below keyl are older than the row
    asm volatile("" : "+v"(keyl));
    float tv[16];
    uint32_t mine0 = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      tv[i] = acc[i] * rj[i];
      if (tv[i] > thr[rt] && 8 * (i >> 2) + (i & 3) < keyl) mine0 |= 1u << (8 * (i >> 2) + (i & 3));
    }
    if (mine0 != 0u) {
      unsigned long long* up = a.credit + (int64_t)head * a.n_pad + c0 + 4 * half;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if ((mine0 >> (8 * (i >> 2) + (i & 3))) & 1u)
          atomicMax(up + 8 * (i >> 2) + (i & 3),
                    ((unsigned long long)(uint32_t)row << 32) | (unsigned long long)__float_as_uint(tv[i] * r_i));
    }
    const uint32_t mine = mine0 << (4 * half);
    const auto both = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    const uint32_t all = both[0] | both[1];
    if (all != 0u && cnt[rt] == 0) {
      const uint32_t top = 1u << (31 - __clz(all));
      float s = 0.f;
      if (mine & top) {
        const int pos = (31 - __clz(all)) - 4 * half;          // bit position = 8*(i/4) + i%4
        const bool b0 = pos & 1, b1 = pos & 2, b2 = pos & 8, b3 = pos & 16;
        const float l0 = b0 ? tv[1] : tv[0], l1 = b0 ? tv[3] : tv[2], l2 = b0 ? tv[5] : tv[4], l3 = b0 ? tv[7] : tv[6];
        const float l4 = b0 ? tv[9] : tv[8], l5 = b0 ? tv[11] : tv[10], l6 = b0 ? tv[13] : tv[12], l7 = b0 ? tv[15] : tv[14];
        const float m0 = b1 ? l1 : l0, m1 = b1 ? l3 : l2, m2 = b1 ? l5 : l4, m3 = b1 ? l7 : l6;
        const float n0 = b2 ? m1 : m0, n1 = b2 ? m3 : m2;
        s = b3 ? n1 : n0;
      }
      sub[rt] = pair_sum32(s);                               // the other lane of the row adds 0
      cnt[rt] = 1;
    }
  };
  // beta = 1 (B1): the row's most recent hit in this tile is all that is wanted.  Within a lane the
  // accumulator elements are in ascending key order, so the last hit met wins; the two lanes of the row
  // then compare keys.  DIAG: the tile holds the row's own key, which is no partner.
  auto tile_first_hit = [&](const f32x16& acc, const float (&rj)[16], int rt, int c0, auto diag) {
    int selfl = row_of(rt) - c0 - 4 * half;                  // own key in this lane's numbering, if it is here
    // keep the 16 comparisons with selfl inside this (rare) path: formed ahead of the scan loop they would
    // occupy 32 scalar registers per row tile for its whole duration
    if constexpr (decltype(diag)::value) asm volatile("" : "+v"(selfl));
    float best = 0.f;
    int bcol = -1;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float tvv = acc[i] * rj[i];
      const int col = 8 * (i >> 2) + (i & 3);
      bool hit = tvv > thr[rt];
      if constexpr (decltype(diag)::value) hit = hit && (col != selfl);
      best = hit ? tvv : best;
      bcol = hit ? col : bcol;
    }
    const int mycol = bcol < 0 ? -1 : bcol + 4 * half;
    const auto cols = __builtin_amdgcn_permlane32_swap((unsigned)mycol, (unsigned)mycol, false, false);
    const auto vals = __builtin_amdgcn_permlane32_swap(__float_as_uint(best), __float_as_uint(best), false, false);
    const bool low = (int)cols[0] > (int)cols[1];
    const int col = low ? (int)cols[0] : (int)cols[1];
    const float val = __uint_as_float(low ? vals[0] : vals[1]);
    if (col >= 0) {
      sub[rt] += val;
      cnt[rt] = 1;
      thr[rt] = INFINITY;
    }
  };
  // Scheduling hint for a block holding one 8-MFMA chain and one tile test (about 24 vector-ALU
  // instructions): issue as 8 x (1 MFMA, 3 VALU) so the test runs in the shadow of the matrix pipe.
  auto interleave = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
    }
  };

  // Closed-form row sum minus the forgiven similarities of the row a lane holds in row tile rt
  auto emit = [&](int rt) {
    const int row = row_of(rt);
    if ((unsigned)row < (unsigned)n) {
      float r;
      if constexpr (SKIP) r = rn[row];                   // rows may have moved between lanes
      else r = rni[rt];                                  // still in the register it was loaded into
      const float closed = mean_sim_closed(r, rowdot[rt], a.eps);
      if (!split) {
        a.sbar[(int64_t)head * a.n_pad + row] = mean_sim_finish(closed, r, sub[rt], n);
      } else {
        // the finalize kernel finishes the mean once every part has reported its hit (beta = 1: the most
        // recent part that found one supplies it); until then the slot holds the closed form
        a.part_cnt[((int64_t)head * parts + part) * a.n_pad + row] = cnt[rt];
        a.part_pre[((int64_t)head * parts + part) * a.n_pad + row] = sub[rt];
        if (closing) a.sbar[(int64_t)head * a.n_pad + row] = closed;
      }
    }
  };

  // ---- stream the tiles, most recent first, from iteration it0 on; RTE = row tiles of the wave that take
  // part (RT, or 1 in a narrow row block and after open rows have been gathered).  Returns the iteration
  // to go on with in the one-row-tile form, or nct when the scan is over.
  int tiles_now = NW * rte;                            // SKIP: row tiles of the workgroup that may hold open rows
  auto scan = [&](auto rte, int it0) __attribute__((always_inline)) -> int {
  constexpr int RTE = decltype(rte)::value;
  for (int it = it0; it < nct; ++it) {
    const int ct = ct_hi - 1 - it;
    const int buf = it & 1;
    // The next tile is copied while this one is used.  The last iteration copies its own tile once more
    // (never read; rows pulled back inside [0, n) if the tile is partly filled) so that the copy needs no
    // branch inside the MFMA/VALU pipeline below.
    const int ctn = gram_next_tile(ct, ct_lo);
    issue_rj(ctn, buf ^ 1);
    const uint64_t next_src = tile_source(ctn);
    const uint32_t next_dst = (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds0 + OFF_TILE + (buf ^ 1) * TILE_SPAN + wave_s * 4 * kRowBytes));
    const unsigned char* tile = gram_lds + OFF_TILE + buf * TILE_SPAN;
    const float* rjs = reinterpret_cast<const float*>(gram_lds + OFF_RJ + buf * TC * 4);

    // Optional exact shortcut: once every row of the wave has met beta hits nothing it could still
    // find changes its result, so the matrix work is skipped (the wave keeps copying tiles).
    bool live = active;
    if constexpr (SKIP) {
      if (live) {
        bool open = false;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) open = open || (thr[rt] != INFINITY);
        live = __any(open);
      }
    }
    if (live) {
    bf16x8 kf[KB][8];
    float rj[KB][16];
    f32x16 acc[2];
    read_k(kf[(NS - 1) % KB], tile, NS - 1);
    read_rj(rj[(NS - 1) % KB], rjs, NS - 1);

    // software pipeline over the NS * RTE tiles of this iteration: chain(q) with test(q - 1)
#pragma unroll
    for (int q2 = 0; q2 <= NS * RTE; ++q2) {
      if (q2 > 0) __builtin_amdgcn_sched_barrier(0);
      if (q2 < NS * RTE) {
        const int s = NS - 1 - q2 / RTE, rt = q2 % RTE;
        if constexpr (KB == 2) {
          // prefetch the next subtile: its key fragments replace those of subtile s + 1 (all chains on
          // them are issued); its r_j replace those of s + 1 one step later, after that subtile's last test
          if (rt == 0 && s > 0) read_k(kf[(s - 1) & 1], tile, s - 1);
          if (RTE > 1 && rt == 1 && s > 0) read_rj(rj[(s - 1) & 1], rjs, s - 1);
          if (RTE == 1 && q2 == 0 && s > 0) read_rj(rj[(s - 1) & 1], rjs, s - 1);   // single row tile: the rest follow the tests
          acc[q2 & 1] = chain(kf[s % KB], res[rt]);
        } else {
          // single fragment set: the subtile's last chain refills the fragments behind itself
          if (rt == RTE - 1 && s > 0) acc[q2 & 1] = chain_refill(kf[0], res[rt], tile, s - 1);
          else acc[q2 & 1] = chain(kf[0], res[rt]);
        }
        // the next tile's DMA copies are spread over the steps instead of stalling the wave up front
        constexpr int PER_STEP = (LOADS / NW + NS * RTE - 1) / (NS * RTE);
#pragma unroll
        for (int d = 0; d < PER_STEP; ++d)
          if (q2 * PER_STEP + d < LOADS / NW) issue_rows(next_src, next_dst, q2 * PER_STEP + d);
      }
      if (q2 > 0) {
        const int qp = q2 - 1;
        const int sp = NS - 1 - qp / RTE, rtp = qp % RTE;
        const float m = tile_max(acc[qp & 1], rj[sp % KB]);
        if (q2 < NS * RTE) interleave();
        if (__any(m > thr[rtp])) {
          if constexpr (VARIANT == kTriangular) {
            tile_triangular(acc[qp & 1], rj[sp % KB], rtp, ct * TC + sp * 32);
          } else if constexpr (B1) {
            const int c0 = ct * TC + sp * 32;
            if (c0 == i0 + rtp * 32) tile_first_hit(acc[qp & 1], rj[sp % KB], rtp, c0, std::true_type{});
            else tile_first_hit(acc[qp & 1], rj[sp % KB], rtp, c0, std::false_type{});
          } else {
            tile_hits(acc[qp & 1], rj[sp % KB], rtp, ct * TC + sp * 32);
          }
        }
        if constexpr (KB == 2 && RTE == 1) {
          // subtile sp's test is done: its r_j registers take those of subtile sp - 2
          if (sp >= 2) read_rj(rj[sp & 1], rjs, sp - 2);
        }
        if constexpr (KB == 1) {
          // the subtile's last test is done: the single r_j set takes those of the next subtile
          if (rtp == RTE - 1 && sp > 0) read_rj(rj[0], rjs, sp - 1);
        }
      }
    }
    } else {
      // a wave without open rows only helps to copy the next tile
#pragma unroll
      for (int jj = 0; jj < LOADS / NW; ++jj) issue_rows(next_src, next_dst, jj);
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if constexpr (!SKIP) {
      __syncthreads();
    } else {
      // open rows of this wave, per row tile (one lane of each row's pair counts)
      int mine = 0;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) mine += __popcll(__ballot(half == 0 && thr[rt] != INFINITY));
      int* cbuf = reinterpret_cast<int*>(gram_lds + OFF_CNT) + (it & 1) * NW;
      if (lane == 0) cbuf[wave] = mine;
      __syncthreads();                                   // also publishes the next tile
      int total = 0, before = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const int c = cbuf[w];
        total += c;
        before += (w < wave) ? c : 0;
      }
      if (total == 0) return nct;                        // nothing the remaining columns could change
      const int need = (total + 31) >> 5;
      if (need <= NW && need * 2 <= tiles_now && it + 1 < nct) {
        // Gather the open rows: rows that are done are written out now, an open row's state goes to a
        // record (slots in wave, row tile, lane order), and wave w takes records 32 w .. 32 w + 31 as its
        // first row tile, fetching those rows' keys again.
        float* rec = reinterpret_cast<float*>(gram_lds + OFF_REC);
        int slot = before;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          const bool open = half == 0 && thr[rt] != INFINITY;
          const unsigned long long ob = __ballot(open);
          if (open) {
            float* r5 = rec + 5 * (slot + __popcll(ob & ((1ull << lane) - 1ull)));
            r5[0] = __int_as_float(rowid[rt]);
            r5[1] = thr[rt];
            r5[2] = sub[rt];
            r5[3] = __int_as_float(cnt[rt]);
            r5[4] = rowdot[rt];
          } else if (half == 0) {
            emit(rt);
          }
          slot += __popcll(ob);
          rowid[rt] = -1;
          thr[rt] = INFINITY;
        }
        __syncthreads();
        const int sl = wave * 32 + lrow;
        active = wave * 32 < total;
        if (sl < total) {
          const float* r5 = rec + 5 * sl;
          rowid[0] = __float_as_int(r5[0]);
          thr[0] = r5[1];
          sub[0] = r5[2];
          cnt[0] = __float_as_int(r5[3]);
          rowdot[0] = r5[4];
#pragma unroll
          for (int kk = 0; kk < 8; ++kk) {
            const uint4 x = *reinterpret_cast<const uint4*>(kbase + (int64_t)rowid[0] * a.kst + kk * 16 + half * 8);
            __builtin_memcpy(&res[0][kk], &x, 16);
          }
        }
        tiles_now = need;
        if constexpr (RTE != 1) return it + 1;           // go on with one row tile per wave
      }
    }
  }
  return nct;
  };   // scan
  // one instantiation of the scan per number of row tiles a wave can hold (the block's rte is uniform)
  auto scan_rte = [&](int it0) __attribute__((always_inline)) -> int {
    if constexpr (RT >= 3) {
      if (rte == 3) return scan(std::integral_constant<int, 3>{}, it0);
    }
    if (rte == 2) return scan(std::integral_constant<int, 2>{}, it0);
    return scan(std::integral_constant<int, 1>{}, it0);
  };
  if constexpr (SKIP) {
    int it = 0;
    if (rte > 1) it = scan_rte(0);
    if (it < nct) scan(std::integral_constant<int, 1>{}, it);
  } else {
    scan_rte(0);
  }

  // ---- closed-form row sums minus the forgiven similarities
  if (half == 0) {
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) emit(rt);
  }
}

template <int NW, int RT, int TC, int WPS, int VARIANT, bool SKIP, bool B1 = false>
hipError_t launch_shape(GramArgs a, const Plan& pl, hipStream_t stream) {
  constexpr int BM = NW * RT * 32;
  constexpr size_t lds = kPseudoBytes + 2 * (size_t)TC * kRowBytes + 2 * (size_t)TC * 4 + (SKIP ? kCompactBytes : 0);
  // once per kernel instantiation (initialisation of a function-local static is thread-safe)
  static const hipError_t configured =
      hipFuncSetAttribute(reinterpret_cast<const void*>(&gram_kernel<NW, RT, TC, WPS, VARIANT, SKIP, B1>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (configured != hipSuccess) return configured;
  static_assert(BM == (SKIP ? kGramRowsSkip : kGramRows) && TC == kGramTile, "the plan's split of the similarity pass assumes this shape");
  const int head_groups = (pl.heads + 7) / 8;
  a.row_blocks = (pl.n + BM - 1) / BM;
  const dim3 grid((unsigned)((int64_t)head_groups * 8 * a.row_blocks * a.parts));
  hipLaunchKernelGGL((gram_kernel<NW, RT, TC, WPS, VARIANT, SKIP, B1>), grid, dim3(NW * 64), lds, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gram(const Plan& pl, const void* k, char* ws, hipStream_t stream) {
  GramArgs a;
  a.k = static_cast<const uint16_t*>(k);
  a.rnorm = reinterpret_cast<const float*>(ws + pl.off_rnorm);
  a.upart = reinterpret_cast<const float*>(ws + pl.off_upart);
  a.sbar = reinterpret_cast<float*>(ws + pl.off_sbar);
  a.credit = (pl.recency_transposed || pl.triangular) ? reinterpret_cast<unsigned long long*>(ws + pl.off_credit) : nullptr;
  a.H = pl.H; a.heads = pl.heads; a.n = pl.n; a.n_pad = pl.n_pad; a.chunks = pl.chunks; a.beta = pl.beta;
  a.ksp = pl.ksp; a.ksh = pl.ksh; a.kst = pl.kst;
  if (pl.paged) {
    // paged cache: the pre-pass left a dense copy of the candidate keys in the workspace
    a.k = reinterpret_cast<const uint16_t*>(ws + pl.off_kdense);
    a.kst = kHeadDim; a.ksh = (int64_t)pl.n_pad * kHeadDim; a.ksp = a.ksh * pl.H;
  }
  a.T = pl.T; a.eps = pl.eps;
  a.row_blocks = 0; a.parts = pl.gram_parts;
  a.part_cnt = reinterpret_cast<int*>(ws + pl.off_pcnt);
  a.part_pre = reinterpret_cast<float*>(ws + pl.off_ppre);
  if (pl.skip_saturated) {
    // (two row tiles per wave: the gathering of open rows needs the registers a third one would take)
    if (a.credit != nullptr) return launch_shape<4, 2, 128, 2, kTransposed, true>(a, pl, stream);
    if (a.parts > 1) return launch_shape<4, 2, 128, 2, kSplit, true>(a, pl, stream);
    return launch_shape<4, 2, 128, 2, kPlain, true>(a, pl, stream);
  }
  if (pl.triangular) return launch_shape<4, 3, 128, 2, kTriangular, false>(a, pl, stream);
  if (a.credit != nullptr) return launch_shape<4, 3, 128, 2, kTransposed, false>(a, pl, stream);
  if (a.parts > 1) return launch_shape<4, 3, 128, 2, kSplit, false>(a, pl, stream);       // split only with beta = 1
  if (pl.beta == 1) return launch_shape<4, 3, 128, 2, kPlain, false, true>(a, pl, stream);
  return launch_shape<4, 3, 128, 2, kPlain, false>(a, pl, stream);
}

}  // namespace rkv
