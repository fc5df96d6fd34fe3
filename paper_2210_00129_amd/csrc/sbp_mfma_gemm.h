// Device code of the two bf16 contractions of the SBP linear backward (paper, eq:backward_fc_sbp):
//   dX tile:  C[j, i] = sum_o dY[row(j), o] W[o, i]          (rows j = kept rows)
//   dW tile:  C[o, i] = sum_j dY[row(j), o] X_k[j, i]        (j = kept rows of one split)
// on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// A block of 4 or 8 wavefronts (2 x 2 or 2 x 4) owns a BM x BN tile and walks the contraction in
// stages of KB = 64 or 32 through a ring of LDS stages filled by asynchronous global -> LDS copies;
// the kept rows of dY are gathered by these copies, so dY_k never exists in memory.  Two LDS tile
// layouts:
//   * "row" tile  [rows][KB]   for an operand whose contraction index is contiguous in memory (dY in
//     dX): MFMA operands are 16-byte LDS reads;
//   * "slow" tile [KB][cols]   for an operand whose contraction index is the slow axis in memory (dY
//     and X_k in dW, W in dX): stored as it lies in memory and read with the transposing LDS read
//     ds_read_b64_tr_b16, which hands every lane 4 consecutive contraction elements of its column.
// This file holds the general engine (any shape, 128 x 128 tiles by default, two blocks per CU) and
// the pieces shared with the large-tile engine of sbp_mfma_big.h.
// The main loop is free of bounds checks: addresses are clamped into the operand (rows or columns
// past the edge compute results that are never stored) and only the last, partial stage zeroes the
// contraction rows past the end.
#ifndef SBP_MFMA_GEMM_H_
#define SBP_MFMA_GEMM_H_

#include <type_traits>

#include "sbp_internal.h"

namespace sbp {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
#define SBP_LDS __attribute__((address_space(3)))
#define SBP_GLB __attribute__((address_space(1)))

static constexpr int NTHREADS = 256;   // threads of the small kernels and of the 4-wavefront GEMM blocks
// A GEMM block has NW = 4 wavefronts (2 x 2 over the tile) or NW = 8 (2 x 4: two wavefronts per SIMD).

// fp32 -> bf16, round to nearest even, two values per instruction (v_cvt_pk_bf16_f32 on gfx950)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ------------------------------------------------------------------------------------------------
// Global -> LDS copies bypass the register file: global_load_lds_dwordx4 moves 16 bytes per lane
// straight into LDS, the 64 lanes of a wavefront filling one contiguous 1 KB block whose base is
// wave-uniform.  Where a piece lands is therefore fixed by the lane number; the swizzles below are
// applied by choosing which global piece each lane fetches.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void async_copy16(const void* g, char* lds_block) {
  __builtin_amdgcn_global_load_lds((SBP_GLB const void*)g, (SBP_LDS void*)lds_block, 16, 0, 0);
}
// wait until at most N of this wavefront's copies are still in flight (they complete in issue order)
template <int N>
__device__ __forceinline__ void wait_async_copies() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// Workgroup barrier that orders LDS traffic only: every wavefront first drains its own LDS reads and
// writes, then meets the others.  Unlike __syncthreads() it does not wait for the asynchronous copies
// still in flight (those are counted by wait_async_copies), so later ring stages stay in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_s_waitcnt(0xc07f);                 // lgkmcnt(0) only; as a builtin the compiler's own wait
  asm volatile("s_barrier" ::: "memory");             // bookkeeping sees it and adds no second wait afterwards
}

// ------------------------------------------------------------------------------------------------
// "row" tile: ROWS rows of KB contraction elements (operand whose contraction index is contiguous in
// memory), swizzled so that the 16-byte operand reads of 32 consecutive rows spread over all 64 banks.
//   KB = 64: 128-byte rows; row m at physical row prow(m) (bits 0 and 3 exchanged), chunk c at slot
//            c ^ (m & 7); a 1 KB block is 8 physical rows.
//   KB = 32:  64-byte rows; chunk c of row m at slot c ^ ((m >> 2) & 3); a 1 KB block is 16 rows.
// Rows past the end are clamped to the last row (their results are never stored); in the tail stage
// chunks past kdim re-read the last chunk (the other operand is zero there).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int prow(int m) { return (m & ~9) | ((m & 1) << 3) | ((m >> 3) & 1); }

template <int ROWS, int NW, int KB>
struct RowTileLoader {
  static constexpr int RPB = KB == 64 ? 8 : 16;         // rows per 1 KB block
  static constexpr int NI = ROWS / RPB / NW;            // blocks per wavefront and stage
  static_assert(NI >= 1 && (KB == 32 || NI % 2 == 0), "block parity trick needs an even block count");
  const uint16_t* rowp[NI];
  int koff[2];                                          // element offset of this lane's chunk in even / odd blocks
  int kdim, blk0;

  __device__ __forceinline__ void init(const uint16_t* src, const int32_t* idx, long long ld, int row0, int nrows,
                                       int kdim_, int lane, int wave) {
    kdim = kdim_;
    blk0 = wave * NI;
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const int q = (blk0 + n) * RPB + (KB == 64 ? (lane >> 3) : (lane >> 2));   // physical row of this lane
      const int m = KB == 64 ? prow(q) : q;                                       // logical row
      const int r = min(row0 + m, nrows - 1);
      const long long g = idx ? (long long)idx[r] : (long long)r;
      rowp[n] = src + g * ld;
    }
    if (KB == 64) {
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int m7 = ((lane >> 3) & 6) | par;          // low bits of the logical row: bit 0 = block parity
        koff[par] = ((lane & 7) ^ m7) * 8;
      }
    } else {
      koff[0] = koff[1] = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
    }
  }
  template <bool TAIL>
  __device__ __forceinline__ void issue(int kbase, char* tile) const {
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      int k = kbase + koff[n & 1];
      if (TAIL) k = min(k, kdim - 8);
      async_copy16(rowp[n] + k, tile + (blk0 + n) * 1024);
    }
  }
  __device__ __forceinline__ void zero_tail(char*, int, int) const {}
};

// per-lane byte offset of the operand fragment rows wbase + 32 f + (lane & 31) in a row tile
template <int KB>
__device__ __forceinline__ int row_tile_lane_off(int wbase, int lane) {
  return KB == 64 ? prow(wbase + (lane & 31)) * 128 : (wbase + (lane & 31)) * 64;
}

template <int F, int KB>
__device__ __forceinline__ void read_row_frags(const char* tile, int lane_off, int ks, int lane, bf16x8_t (&a)[F]) {
  const int sw = KB == 64 ? (lane & 7) : ((lane >> 2) & 3);
  const int ch = ((2 * ks + (lane >> 5)) ^ sw) << 4;
#pragma unroll
  for (int f = 0; f < F; ++f) a[f] = *reinterpret_cast<const bf16x8_t*>(tile + lane_off + f * (32 * KB * 2) + ch);
}

// ------------------------------------------------------------------------------------------------
// "slow" tile: KB contraction rows of COLS bf16, pitch COLS * 2 bytes, stored as in memory except
// that 16-byte chunk c of row k sits at slot c ^ ((k & 3) << 2).  A transposing read of a 16-lane
// group touches 4 consecutive rows x 32 bytes; the swizzle puts those on different banks.
// One 1 KB block = 2 rows (COLS = 256) or 4 rows (COLS = 128).
// Columns past the end are clamped (never stored); contraction rows past kdim are clamped for the
// address and their LDS rows zeroed afterwards (tail stage only).  The row ids of a gathered operand
// come from a table in LDS (rows[k - k0], filled by the caller), so no global load sits between the
// copies.
// ------------------------------------------------------------------------------------------------
template <int COLS, int NW, int KB>
struct SlowTileLoader {
  static constexpr int LPR = COLS / 8;                 // lanes (chunks) per contraction row
  static constexpr int RPI = 64 / LPR;                 // rows per 1 KB block
  static constexpr int NI = KB / RPI / NW;             // blocks per wavefront and stage
  static_assert(NI >= 1 && (RPI == 4 || NI % 2 == 0), "block parity trick needs an even block count");
  static constexpr int PITCH = COLS * 2;
  const uint16_t* src;
  const int* rows;                                     // LDS table of row ids, or nullptr
  long long ld;
  int k0, kdim, blk0, rsub;
  int coff[2];                                         // column (elements) of this lane's chunk in even / odd blocks

  __device__ __forceinline__ void init(const uint16_t* src_, const int* rows_, long long ld_, int col0, int ncols,
                                       int k0_, int kdim_, int lane, int wave) {
    src = src_; rows = rows_; ld = ld_; k0 = k0_; kdim = kdim_;
    blk0 = wave * NI;
    rsub = lane / LPR;
    const int p = lane % LPR;
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int k3 = (RPI * par + rsub) & 3;             // low bits of the row index (blk0 * RPI is a multiple of 4)
      coff[par] = min(col0 + 8 * (p ^ (k3 << 2)), ncols - 8);
    }
  }
  template <bool TAIL>
  __device__ __forceinline__ void issue(int kbase, char* tile) const {
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const int k = kbase + RPI * (blk0 + n) + rsub;
      const long long g = rows ? (long long)rows[k - k0] : (long long)(TAIL ? min(k, kdim - 1) : k);
      async_copy16(src + g * ld + coff[n & 1], tile + (blk0 + n) * 1024);
    }
  }
  // zero the LDS rows kvalid .. KB-1 (contraction rows past the end of the operand)
  __device__ __forceinline__ void zero_tail(char* tile, int kvalid, int t) const {
#pragma unroll
    for (int i = 0; i < KB * LPR / (64 * NW); ++i) {
      const int q = t + 64 * NW * i;
      if (q / LPR >= kvalid) *reinterpret_cast<uint4*>(tile + q * 16) = make_uint4(0, 0, 0, 0);
    }
  }
};

// Per-lane byte offsets for the transposing reads of F fragments (32 columns each) starting at column
// wbase.  In a 16-lane group, lane i addresses row (i >> 2), columns 4 (i & 3) ..; the hardware returns
// to lane j column j of those 4 rows.  Groups 0/1 take columns 0-15 / 16-31, groups 2/3 the next 8 rows.
template <int COLS, int F>
__device__ __forceinline__ void slow_tile_lane_offs(int wbase, int lane, int (&off)[F]) {
  const int g = lane >> 4, i = lane & 15;
  const int k = 8 * (g >> 1) + (i >> 2);
#pragma unroll
  for (int f = 0; f < F; ++f) {
    const int m = wbase + 32 * f + 16 * (g & 1) + 4 * (i & 3);
    off[f] = k * (COLS * 2) + ((((m >> 3)) ^ ((k & 3) << 2)) << 4) + ((m & 7) << 1);
  }
}

template <int COLS, int F>
__device__ __forceinline__ void read_slow_frags(const char* tile, const int (&off)[F], int ks, bf16x8_t (&a)[F]) {
#pragma unroll
  for (int f = 0; f < F; ++f) {
    const char* p = tile + off[f] + ks * 16 * (COLS * 2);
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SBP_LDS s16x4_t*)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SBP_LDS s16x4_t*)(p + 4 * (COLS * 2)));
    a[f] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
}

template <int FM, int FN>
__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[FM][FN]) {
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

// ------------------------------------------------------------------------------------------------
// Stage loop over a ring of NSTAGE LDS buffers: while the MFMAs of stage kt run, the copies of stages
// kt+1 .. kt+NSTAGE-1 are in flight.  One barrier per stage: it publishes the landed stage and retires
// the buffer that the next copies overwrite.  A wavefront's copies complete in issue order, so "stage
// kt has landed" is "at most r * (copies per stage) still in flight", r = stages issued after it.
// ------------------------------------------------------------------------------------------------
template <int NSTAGE, int KB, int A_BYTES, int STAGE, class LA, class LB, class Compute>
__device__ __forceinline__ void stage_loop(char* smem, LA& la, LB& lb, int k0, int kend, int nk, Compute&& compute) {
  static_assert(NSTAGE >= 2 && NSTAGE <= 4, "ring of 2 to 4 stages");
  constexpr int C = LA::NI + LB::NI;               // copies per wavefront and stage
  if (nk <= 0) return;
  const int t = threadIdx.x;
  const bool tail = ((kend - k0) % KB) != 0;
  auto issue = [&](int s) {
    char* buf = smem + (s % NSTAGE) * STAGE;
    const int kbase = k0 + s * KB;
    if (tail && s == nk - 1) {
      la.template issue<true>(kbase, buf);
      lb.template issue<true>(kbase, buf + A_BYTES);
    } else {
      la.template issue<false>(kbase, buf);
      lb.template issue<false>(kbase, buf + A_BYTES);
    }
  };
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nk) issue(s);
  for (int kt = 0; kt < nk; ++kt) {
    char* cur = smem + (kt % NSTAGE) * STAGE;
    const int ahead = min(NSTAGE - 2, nk - 1 - kt);    // stages issued after stage kt
    if (NSTAGE >= 4 && ahead == 2) wait_async_copies<2 * C>();
    else if (NSTAGE >= 3 && ahead == 1) wait_async_copies<C>();
    else wait_async_copies<0>();
    lds_barrier();
    if (tail && kt == nk - 1) {
      const int kvalid = kend - (k0 + kt * KB);
      la.zero_tail(cur, kvalid, t);
      lb.zero_tail(cur + A_BYTES, kvalid, t);
      lds_barrier();
    }
    if (kt + NSTAGE - 1 < nk) issue(kt + NSTAGE - 1);
    compute(cur);
  }
  lds_barrier();
}

// ------------------------------------------------------------------------------------------------
// dX tile: BM kept rows x BN input channels.  The MFMA is issued with the operands exchanged, so a
// lane ends up with 4 consecutive input channels of one kept row: register v of lane l of a 32x32
// tile is C[row l & 31][col 8 (v >> 2) + 4 (l >> 5) + (v & 3)].  The epilogue rounds to bf16, stages
// 64 rows at a time through LDS and writes whole 16-byte pieces of the (scattered) dX rows.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int NW, int KB, int NSTAGE>
__device__ __forceinline__ void dx_tile(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx_in,
                                        const int32_t* __restrict__ idx_out, const uint16_t* __restrict__ W, int K,
                                        int Cin, int Cout, uint16_t* __restrict__ dX, int m0, int n0) {
  constexpr int WGN = NW / 2;                     // wavefront grid: 2 rows x WGN columns
  constexpr int FM = BM / 64, FN = BN / (32 * WGN);
  constexpr int A_BYTES = BM * KB * 2, B_BYTES = BN * KB * 2, STAGE = A_BYTES + B_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = (wave / WGN) * (BM / 2), wn = (wave % WGN) * (BN / WGN);

  RowTileLoader<BM, NW, KB> la;
  SlowTileLoader<BN, NW, KB> lb;
  la.init(dY, idx_in, Cout, m0, K, Cout, lane, __builtin_amdgcn_readfirstlane(wave));
  lb.init(W, nullptr, Cin, n0, Cin, 0, Cout, lane, __builtin_amdgcn_readfirstlane(wave));

  f32x16_t acc[FM][FN];
  zero_acc<FM, FN>(acc);
  const int a_off = row_tile_lane_off<KB>(wm, lane);
  int b_off[FN];
  slow_tile_lane_offs<BN, FN>(wn, lane, b_off);
  const int nk = (Cout + KB - 1) / KB;

  auto compute = [&](const char* cur) {
#pragma unroll
    for (int ks = 0; ks < KB / 16; ++ks) {
      bf16x8_t a[FM], b[FN];
      read_slow_frags<BN, FN>(cur + A_BYTES, b_off, ks, b);
      read_row_frags<FM, KB>(cur, a_off, ks, lane, a);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
  };
  stage_loop<NSTAGE, KB, A_BYTES, STAGE>(smem, la, lb, 0, Cout, nk, compute);

  // epilogue
  constexpr int PITCH = BN * 2 + 16;              // staging row pitch (bytes)
  constexpr int CPR = BN / 8;                     // 16-byte pieces per staged row
  constexpr int RPP = 64 * NW / CPR;              // rows written per pass of the block
  const int pc = t % CPR, pr = t / CPR;
  const bool col_ok = n0 + 8 * pc < Cin;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    {
      char* row = smem + ((wave / WGN) * 32 + (lane & 31)) * PITCH + (wn + 4 * (lane >> 5)) * 2;
#pragma unroll
      for (int jn = 0; jn < FN; ++jn)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2 w;
          w.x = bf16_pack(acc[i][jn][4 * q + 0], acc[i][jn][4 * q + 1]);
          w.y = bf16_pack(acc[i][jn][4 * q + 2], acc[i][jn][4 * q + 3]);
          *reinterpret_cast<uint2*>(row + (32 * jn + 8 * q) * 2) = w;
        }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 64 / RPP; ++p) {
      const int r = pr + p * RPP;                 // staged row: half (r >> 5), row (r & 31)
      const int j = m0 + (r >> 5) * (BM / 2) + 32 * i + (r & 31);
      if (j < K && col_ok) {
        const long long orow = idx_out ? (long long)idx_out[j] : (long long)j;
        *reinterpret_cast<uint4*>(dX + orow * Cin + n0 + 8 * pc) =
            *reinterpret_cast<const uint4*>(smem + r * PITCH + pc * 16);
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// dW tile: BM output channels x BN input channels over the kept rows [j0, j1) of one split, written
// as an fp32 partial.  Register v of lane l of a 32x32 tile is
// C[row 8 (v >> 2) + 4 (l >> 5) + (v & 3)][col l & 31].
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int NW, int KB, int NSTAGE>
__device__ __forceinline__ void dw_tile(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx,
                                        const uint16_t* __restrict__ Xk, int Cin, int Cout, int j0, int j1,
                                        float* __restrict__ part, int m0, int n0) {
  constexpr int WGN = NW / 2;                     // wavefront grid: 2 rows x WGN columns
  constexpr int FM = BM / 64, FN = BN / (32 * WGN);
  constexpr int A_BYTES = BM * KB * 2, B_BYTES = BN * KB * 2, STAGE = A_BYTES + B_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = (wave / WGN) * (BM / 2), wn = (wave % WGN) * (BN / WGN);
  const int nk = (j1 - j0 + KB - 1) / KB;

  // row ids of the split's kept rows (clamped past the end), behind the stage ring
  int* rows = nullptr;
  if (idx) {
    rows = reinterpret_cast<int*>(smem + NSTAGE * STAGE);
    for (int i = t; i < nk * KB; i += 64 * NW) rows[i] = idx[min(j0 + i, j1 - 1)];
    __syncthreads();
  }
  SlowTileLoader<BM, NW, KB> la;
  SlowTileLoader<BN, NW, KB> lb;
  la.init(dY, rows, Cout, m0, Cout, j0, j1, lane, __builtin_amdgcn_readfirstlane(wave));
  lb.init(Xk, nullptr, Cin, n0, Cin, j0, j1, lane, __builtin_amdgcn_readfirstlane(wave));

  f32x16_t acc[FM][FN];
  zero_acc<FM, FN>(acc);
  int a_off[FM], b_off[FN];
  slow_tile_lane_offs<BM, FM>(wm, lane, a_off);
  slow_tile_lane_offs<BN, FN>(wn, lane, b_off);

  auto compute = [&](const char* cur) {
#pragma unroll
    for (int ks = 0; ks < KB / 16; ++ks) {
      bf16x8_t a[FM], b[FN];
      read_slow_frags<BN, FN>(cur + A_BYTES, b_off, ks, b);
      read_slow_frags<BM, FM>(cur, a_off, ks, a);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };
  stage_loop<NSTAGE, KB, A_BYTES, STAGE>(smem, la, lb, j0, j1, nk, compute);

  if (m0 + BM <= Cout && n0 + BN <= Cin) {         // interior tile: no bounds checks
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float* prow_ = part + (long long)(m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * Cin + n0 + wn +
                       (lane & 31);
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) prow_[32 * jn] = acc[i][jn][v];
      }
  } else {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
        for (int jn = 0; jn < FN; ++jn) {
          const int col = n0 + wn + 32 * jn + (lane & 31);
          if (o < Cout && col < Cin) part[(long long)o * Cin + col] = acc[i][jn][v];
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------
// Partial bias gradient of one row slice: dbp[o] = sum_{j in [j0, j1)} dY[row(j), o] for 256 channels
// starting at c0.  Thread (x = t & 31, y = t >> 5) owns 8 channels and every 8th row; the eight row
// lanes are added in a fixed order through LDS.  The slice's row ids are staged in LDS first, so the
// row loads do not wait for index loads and UNR of them are in flight per thread.
// ------------------------------------------------------------------------------------------------
template <int UNR>
__device__ __forceinline__ void colsum_block(char* smem, const uint16_t* __restrict__ dY,
                                             const int32_t* __restrict__ idx, int Cout, int j0, int j1, int c0,
                                             float* __restrict__ dbp) {
  constexpr int CHUNK = 1024;                                 // row ids staged at a time
  float(*red)[32][9] = reinterpret_cast<float(*)[32][9]>(smem);
  int* ids = reinterpret_cast<int*>(smem + sizeof(float) * 8 * 32 * 9);
  const int x = threadIdx.x & 31, y = threadIdx.x >> 5;     // wavefronts past the fourth only keep the barriers company
  const int col = c0 + 8 * x;
  float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int b0 = j0; b0 < j1; b0 += CHUNK) {
    const int n = min(CHUNK, j1 - b0);
    for (int i = threadIdx.x; i < n; i += blockDim.x) ids[i] = idx ? idx[b0 + i] : b0 + i;
    __syncthreads();
    if (col < Cout && y < 8) {
#pragma unroll UNR
      for (int j = y; j < n; j += 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(dY + (long long)ids[j] * Cout + col);
        s[0] += bf16_lo(v.x); s[1] += bf16_hi(v.x); s[2] += bf16_lo(v.y); s[3] += bf16_hi(v.y);
        s[4] += bf16_lo(v.z); s[5] += bf16_hi(v.z); s[6] += bf16_lo(v.w); s[7] += bf16_hi(v.w);
      }
    }
    __syncthreads();
  }
  if (y < 8) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[y][x][e] = s[e];
  }
  __syncthreads();
  if (y == 0 && col < Cout) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float a = 0.f;
#pragma unroll
      for (int yy = 0; yy < 8; ++yy) a += red[yy][x][e];
      dbp[col + e] = a;
    }
  }
}

}  // namespace sbp
#endif
