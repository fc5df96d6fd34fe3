// Device code of the two bf16 contractions of the SBP linear backward (paper, eq:backward_fc_sbp):
//   dX tile:  C[j, i] = sum_o dY[row(j), o] W[o, i]          (rows j = kept rows)
//   dW tile:  C[o, i] = sum_j dY[row(j), o] X_k[j, i]        (j = kept rows of one split)
// on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// A block of 256 threads (2 x 2 wavefronts) owns a BM x BN tile and walks the contraction in stages
// of BK = 64.  Global memory is read in 16-byte pieces into registers NPRE stages ahead and stored to
// a double-buffered LDS stage; the kept rows of dY are gathered by these loads, so dY_k never exists
// in memory.  Two LDS tile layouts:
//   * "row" tile  [rows][BK]   for an operand whose contraction index is contiguous in memory (dY in
//     dX): MFMA operands are 16-byte LDS reads;
//   * "slow" tile [BK][cols]   for an operand whose contraction index is the slow axis in memory (dY
//     and X_k in dW, W in dX): stored as it lies in memory and read with the transposing LDS read
//     ds_read_b64_tr_b16, which hands every lane 4 consecutive contraction elements of its column.
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
typedef float f32x16_t __attribute__((ext_vector_type(16)));
#define SBP_LDS __attribute__((address_space(3)))

static constexpr int BK = 64;          // contraction elements per LDS stage
static constexpr int NTHREADS = 256;   // 4 wavefronts, arranged 2 x 2 over the block tile

__device__ __forceinline__ uint32_t bf16_round(float f) {   // round-to-nearest-even, NaN kept quiet
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi) { return bf16_round(lo) | (bf16_round(hi) << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ------------------------------------------------------------------------------------------------
// "row" tile: ROWS rows of BK bf16 (128 bytes = eight 16-byte chunks).  Row m sits at physical row
// prow(m) (bits 0 and 3 exchanged), its chunk c at slot c ^ (m & 7): the 16-byte operand reads of 32
// consecutive rows and the loader's writes both spread over all 64 banks.
// Rows past the end are clamped to the last row (their results are never stored); in the tail stage
// chunks past kdim re-read the last chunk (the other operand is zero there).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int prow(int m) { return (m & ~9) | ((m & 1) << 3) | ((m >> 3) & 1); }

template <int ROWS, int NPRE>
struct RowTileLoader {
  static constexpr int NI = ROWS / 32;
  const uint16_t* ptr[NI];
  uint4 reg[NPRE][NI];
  int soff[NI];
  int c, kdim;

  __device__ __forceinline__ void init(const uint16_t* src, const int32_t* idx, long long ld, int row0, int nrows,
                                       int kdim_, int t) {
    c = t & 7;
    kdim = kdim_;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = (t >> 3) + 32 * i;        // physical row
      const int m = prow(q);                  // logical row (prow is its own inverse)
      const int r = min(row0 + m, nrows - 1);
      soff[i] = q * 128 + ((c ^ (m & 7)) << 4);
      const long long g = idx ? (long long)idx[r] : (long long)r;
      ptr[i] = src + g * ld;
    }
  }
  template <int S, bool TAIL>
  __device__ __forceinline__ void load(int kbase) {
    int k = kbase + c * 8;
    if (TAIL) k = min(k, kdim - 8);
#pragma unroll
    for (int i = 0; i < NI; ++i) reg[S][i] = *reinterpret_cast<const uint4*>(ptr[i] + k);
  }
  template <int S>
  __device__ __forceinline__ void store(char* buf) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) *reinterpret_cast<uint4*>(buf + soff[i]) = reg[S][i];
  }
};

// per-lane byte offset of the operand fragment rows wbase + 32 f + (lane & 31) in a row tile
__device__ __forceinline__ int row_tile_lane_off(int wbase, int lane) { return prow(wbase + (lane & 31)) * 128; }

template <int F>
__device__ __forceinline__ void read_row_frags(const char* tile, int lane_off, int ks, int lane, bf16x8_t (&a)[F]) {
  const int ch = ((2 * ks + (lane >> 5)) ^ (lane & 7)) << 4;
#pragma unroll
  for (int f = 0; f < F; ++f) a[f] = *reinterpret_cast<const bf16x8_t*>(tile + lane_off + f * 4096 + ch);
}

// ------------------------------------------------------------------------------------------------
// "slow" tile: BK contraction rows of COLS bf16, pitch COLS * 2 bytes, stored as in memory except
// that 16-byte chunk c of row k sits at slot c ^ ((k & 3) << 2).  A transposing read of a 16-lane
// group touches 4 consecutive rows x 32 bytes; the swizzle puts those on different banks.
// Columns past the end are clamped (never stored); contraction rows past kdim are clamped for the
// address and zeroed in the tail stage.  Row ids of a gathered operand are fetched one stage early.
// ------------------------------------------------------------------------------------------------
template <int COLS, int NPRE>
struct SlowTileLoader {
  static constexpr int CPR = COLS / 8;                 // chunks per contraction row
  static constexpr int RSTEP = NTHREADS / CPR;         // rows between a thread's successive chunks (8 or 16)
  static constexpr int NI = BK / RSTEP;                // chunks per thread and stage
  static constexpr int PITCH = COLS * 2;
  const uint16_t* src;
  const int32_t* idx;
  long long ld;
  int kdim, krow, soff0;
  int nrow[NI];                                        // row ids for the next load() of a gathered operand
  uint4 reg[NPRE][NI];

  __device__ __forceinline__ void init(const uint16_t* src_, const int32_t* idx_, long long ld_, int col0, int ncols,
                                       int kdim_, int t) {
    idx = idx_; ld = ld_; kdim = kdim_;
    const int c = t % CPR;
    krow = t / CPR;
    src = src_ + min(col0 + 8 * c, ncols - 8);
    soff0 = krow * PITCH + ((c ^ ((krow & 3) << 2)) << 4);
  }
  // fetch the row ids of the stage starting at kbase (no-op for an operand that is not gathered)
  __device__ __forceinline__ void fetch_rows(int kbase) {
    if (idx) {
#pragma unroll
      for (int i = 0; i < NI; ++i) nrow[i] = idx[min(kbase + krow + RSTEP * i, kdim - 1)];
    }
  }
  template <int S, bool TAIL>
  __device__ __forceinline__ void load(int kbase) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int k = kbase + krow + RSTEP * i;
      const long long g = idx ? (long long)nrow[i] : (long long)(TAIL ? min(k, kdim - 1) : k);
      uint4 v = *reinterpret_cast<const uint4*>(src + g * ld);
      if (TAIL && k >= kdim) v = make_uint4(0, 0, 0, 0);
      reg[S][i] = v;
    }
  }
  template <int S>
  __device__ __forceinline__ void store(char* buf) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) *reinterpret_cast<uint4*>(buf + soff0 + i * RSTEP * PITCH) = reg[S][i];
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
// Generic stage loop.  LA / LB are loaders, READ_A / READ_B fragment readers, MMA the multiply step.
// NPRE = 1: the loads of stage kt+1 are issued before the MFMAs of stage kt and stored after them.
// NPRE = 2: the loads of stage kt+2 are issued before the MFMAs of stage kt, and the registers of
//           stage kt+1 (loaded one iteration earlier) are stored while they run.
// ------------------------------------------------------------------------------------------------
template <int S, bool TAIL, class LA, class LB>
__device__ __forceinline__ void issue_loads(LA& la, LB& lb, int kbase) {
  la.template load<S, TAIL>(kbase);
  lb.template load<S, TAIL>(kbase);
}

template <int NPRE, int A_BYTES, int STAGE, class LA, class LB, class Compute, class Fetch>
__device__ __forceinline__ void stage_loop(char* smem, LA& la, LB& lb, int k0, int nk, bool tail, Compute&& compute,
                                           Fetch&& fetch) {
  // stage s covers contraction rows k0 + s BK ..; `tail` says the last stage is partial
  auto load_stage = [&](auto sel, int s) {
    constexpr int S = decltype(sel)::value;
    if (tail && s == nk - 1) issue_loads<S, true>(la, lb, k0 + s * BK);
    else issue_loads<S, false>(la, lb, k0 + s * BK);
    fetch(la, lb, k0 + (s + 1) * BK);
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  if (nk <= 0) return;
  if constexpr (NPRE == 1) {
    load_stage(I0{}, 0);
    la.template store<0>(smem); lb.template store<0>(smem + A_BYTES);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const char* cur = smem + (kt & 1) * STAGE;
      char* nxt = smem + ((kt + 1) & 1) * STAGE;
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT == 3
      if (kt + 1 < nk) load_stage(I0{}, kt + 1);
#endif
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT != 3
      compute(cur);
#endif
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT != 2
      if (kt + 1 < nk) { la.template store<0>(nxt); lb.template store<0>(nxt + A_BYTES); }
#endif
      __syncthreads();
    }
  } else {
    load_stage(I0{}, 0);
    if (nk > 1) load_stage(I1{}, 1);
    la.template store<0>(smem); lb.template store<0>(smem + A_BYTES);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
      {  // even stage: registers set 0 is free (stored), set 1 holds stage kt+1
        const char* cur = smem;
        char* nxt = smem + STAGE;
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT == 3
        if (kt + 2 < nk) load_stage(I0{}, kt + 2);
#endif
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT != 2
        if (kt + 1 < nk) { la.template store<1>(nxt); lb.template store<1>(nxt + A_BYTES); }
#endif
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT != 3
        compute(cur);
#endif
        __syncthreads();
      }
      if (kt + 1 < nk) {  // odd stage
        const char* cur = smem + STAGE;
        char* nxt = smem;
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT == 3
        if (kt + 3 < nk) load_stage(I1{}, kt + 3);
#endif
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT != 2
        if (kt + 2 < nk) { la.template store<0>(nxt); lb.template store<0>(nxt + A_BYTES); }
#endif
#if !defined(SBP_EXPERIMENT) || SBP_EXPERIMENT != 3
        compute(cur);
#endif
        __syncthreads();
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dX tile: BM kept rows x BN input channels.  The MFMA is issued with the operands exchanged, so a
// lane ends up with 4 consecutive input channels of one kept row: register v of lane l of a 32x32
// tile is C[row l & 31][col 8 (v >> 2) + 4 (l >> 5) + (v & 3)].  The epilogue rounds to bf16, stages
// 64 rows at a time through LDS and writes whole 16-byte pieces of the (scattered) dX rows.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int NPRE>
__device__ __forceinline__ void dx_tile(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx_in,
                                        const int32_t* __restrict__ idx_out, const uint16_t* __restrict__ W, int K,
                                        int Cin, int Cout, uint16_t* __restrict__ dX, int m0, int n0) {
  constexpr int FM = BM / 64, FN = BN / 64;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);

  using LA = RowTileLoader<BM, NPRE>;
  using LB = SlowTileLoader<BN, NPRE>;
  LA la;
  LB lb;
  la.init(dY, idx_in, Cout, m0, K, Cout, t);
  lb.init(W, nullptr, Cin, n0, Cin, Cout, t);

  f32x16_t acc[FM][FN];
  zero_acc<FM, FN>(acc);
  const int a_off = row_tile_lane_off(wm, lane);
  int b_off[FN];
  slow_tile_lane_offs<BN, FN>(wn, lane, b_off);
  const int nk = (Cout + BK - 1) / BK;

  auto compute = [&](const char* cur) {
    bf16x8_t a[2][FM], b[2][FN];
    read_row_frags<FM>(cur, a_off, 0, lane, a[0]);
    read_slow_frags<BN, FN>(cur + A_BYTES, b_off, 0, b[0]);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (ks + 1 < BK / 16) {
        read_row_frags<FM>(cur, a_off, ks + 1, lane, a[(ks + 1) & 1]);
        read_slow_frags<BN, FN>(cur + A_BYTES, b_off, ks + 1, b[(ks + 1) & 1]);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[ks & 1][j], a[ks & 1][i], acc[i][j], 0, 0, 0);
    }
  };
  stage_loop<NPRE, A_BYTES, STAGE>(smem, la, lb, 0, nk, (Cout % BK) != 0, compute, [](LA&, LB&, int) {});

  // epilogue
  constexpr int PITCH = BN * 2 + 16;              // staging row pitch (bytes)
  constexpr int CPR = BN / 8;                     // 16-byte pieces per staged row
  constexpr int RPP = NTHREADS / CPR;             // rows written per pass of the block
  const int pc = t % CPR, pr = t / CPR;
  const bool col_ok = n0 + 8 * pc < Cin;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    {
      char* row = smem + ((wave >> 1) * 32 + (lane & 31)) * PITCH + (wn + 4 * (lane >> 5)) * 2;
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
// C[row 8 (v >> 2) + 4 (l >> 5) + (v & 3)][col l & 31].  Blocks of the first tile column also produce
// the partial bias gradient db[o] = sum_j dY[row(j), o] by multiplying their dY fragments with ones.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int NPRE>
__device__ __forceinline__ void dw_tile(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx,
                                        const uint16_t* __restrict__ Xk, int Cin, int Cout, int j0, int j1,
                                        float* __restrict__ part, float* __restrict__ dbp, int m0, int n0) {
  constexpr int FM = BM / 64, FN = BN / 64;
  constexpr int FD = FM / 2;                       // dY fragments whose row sums this wavefront owns
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * (BN / 2);
  const bool do_db = dbp != nullptr && n0 == 0;    // block-uniform
  const bool upper = (wave & 1) != 0;              // this wavefront owns fragments FD .. 2 FD - 1

  using LA = SlowTileLoader<BM, NPRE>;
  using LB = SlowTileLoader<BN, NPRE>;
  LA la;
  LB lb;
  la.init(dY, idx, Cout, m0, Cout, j1, t);
  lb.init(Xk, nullptr, Cin, n0, Cin, j1, t);
  la.fetch_rows(j0);

  f32x16_t acc[FM][FN];
  zero_acc<FM, FN>(acc);
  f32x16_t accd[FD];
#pragma unroll
  for (int f = 0; f < FD; ++f)
#pragma unroll
    for (int v = 0; v < 16; ++v) accd[f][v] = 0.f;
  bf16x8_t ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  int a_off[FM], b_off[FN];
  slow_tile_lane_offs<BM, FM>(wm, lane, a_off);
  slow_tile_lane_offs<BN, FN>(wn, lane, b_off);
  const int nk = (j1 - j0 + BK - 1) / BK;

  auto compute = [&](const char* cur) {
    bf16x8_t a[2][FM], b[2][FN];
    read_slow_frags<BM, FM>(cur, a_off, 0, a[0]);
    read_slow_frags<BN, FN>(cur + A_BYTES, b_off, 0, b[0]);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (ks + 1 < BK / 16) {
        read_slow_frags<BM, FM>(cur, a_off, ks + 1, a[(ks + 1) & 1]);
        read_slow_frags<BN, FN>(cur + A_BYTES, b_off, ks + 1, b[(ks + 1) & 1]);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
      if (do_db) {
#pragma unroll
        for (int f = 0; f < FD; ++f)
          accd[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(upper ? a[ks & 1][f + FD] : a[ks & 1][f], ones, accd[f],
                                                            0, 0, 0);
      }
    }
  };
  stage_loop<NPRE, A_BYTES, STAGE>(smem, la, lb, j0, nk, ((j1 - j0) % BK) != 0, compute,
                                   [](LA& a, LB&, int kbase) { a.fetch_rows(kbase); });

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
  if (do_db && (lane & 31) == 0) {      // every column of accd holds the row sums; column 0 writes them
#pragma unroll
    for (int f = 0; f < FD; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = m0 + wm + 32 * ((upper ? FD : 0) + f) + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (o < Cout) dbp[o] = accd[f][v];
      }
  }
}

}  // namespace sbp
#endif
