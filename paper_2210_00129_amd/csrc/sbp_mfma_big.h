// Large-tile engine for the two bf16 contractions of the SBP linear backward (paper,
// eq:backward_fc_sbp): 256-wide output tiles, one workgroup of 4 wavefronts per CU, every wavefront
// owning a 128 x 128 quarter of a 256 x 256 tile (16 accumulator blocks of 32 x 32 = 256 accumulator
// registers) or a 64 x 128 quarter of a 128 x 256 dX tile.
//
// Why this shape: at 64 x 64 per wavefront the operand reads from LDS need as many LDS cycles as the
// MFMAs need matrix-core cycles; at 128 x 128 they need half.  With one wavefront per SIMD nothing
// hides a stall, so the instruction stream is laid out by hand:
//   * the contraction runs in stages of 32 through a ring of 4 LDS stages; while stage s is consumed,
//     s + 1 and s + 2 are landing and the copies of s + 3 are being issued;
//   * global -> LDS copies are global_load_lds_dwordx4 with a wave-uniform base and a per-lane 32-bit
//     offset computed once per tile: a stage's copies cost a scalar add and no vector arithmetic;
//   * operand fragments are double-buffered in registers: while the MFMAs of one 16-deep step run,
//     the LDS reads of the next step and then a share of the copies are issued between them, in an
//     order given to the compiler's scheduler group by group (interleave_step);
//   * one barrier per stage, between its two steps: it retires the stage just read and publishes
//     stage s + 1.  The barrier waits for LDS traffic only; copies in flight are counted with
//     s_waitcnt vmcnt.
// LDS tile layouts and their swizzles are those of sbp_mfma_gemm.h ("row" tile for dY in dX, "slow"
// tiles read with ds_read_b64_tr_b16 for everything else).
//
// Limits (checked on the host, the general engine takes the rest): Cout % 32 == 0 (no partial stage
// in dX), row offsets fit 32 bits (M * max(Cin, Cout) * 2 < 2^32), at most 4096 kept rows per dW split.
#ifndef SBP_MFMA_BIG_H_
#define SBP_MFMA_BIG_H_

#include "sbp_mfma_gemm.h"

namespace sbp {
namespace big {

static constexpr int BT = 256;                  // tile edge, rows and columns
static constexpr int KB = 32;                   // contraction elements per stage
static constexpr int NS = 4;                    // ring depth
static constexpr int TILE_BYTES = BT * KB * 2;  // a 256-wide operand tile of a stage
static constexpr int RING = NS * 2 * TILE_BYTES;   // the largest ring (two 256-wide operands): 128 KB
// A tile is BMX x 256 with BMX = 256 (dW, dX), 128 or 64 (dX where too few taller tiles exist to fill the
// chip): FM = BMX / 64 accumulator block rows per wavefront, FM + 4 copies per wavefront and stage.

template <int CPS>
__device__ __forceinline__ void wait_copies_runtime(int stages_in_flight) {   // wave-uniform argument
  if (stages_in_flight >= 3) wait_async_copies<3 * CPS>();
  else if (stages_in_flight == 2) wait_async_copies<2 * CPS>();
  else if (stages_in_flight == 1) wait_async_copies<CPS>();
  else wait_async_copies<0>();
}

// ---- copies of a "row" tile [64 NI rows][32 k]: blocks of 16 rows, NI per wavefront ---------------
template <int NI>
struct RowCopy {
  uint32_t voff[NI];
  __device__ __forceinline__ void init(const int32_t* idx, uint32_t ld_bytes, int row0, int nrows, int lane, int wave) {
    const uint32_t chunk = (uint32_t)(((lane & 3) ^ ((lane >> 4) & 3)) * 16);
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const int r = min(row0 + 16 * (NI * wave + n) + (lane >> 2), nrows - 1);
      const uint32_t g = idx ? (uint32_t)idx[r] : (uint32_t)r;
      voff[n] = g * ld_bytes + chunk;
    }
  }
  __device__ __forceinline__ void issue(const char* base, char* tile, int wave) const {
#pragma unroll
    for (int n = 0; n < NI; ++n) async_copy16(base + voff[n], tile + (NI * wave + n) * 1024);
  }
};

// ---- copies of a "slow" tile [32 k][256 columns]: 16 blocks of 2 rows, 4 per wavefront ----------
struct SlowCopy {
  uint32_t voff[4];   // operand with consecutive rows: (row within the stage) * ld + column bytes
  uint32_t colb[2];   // column bytes of this lane in even / odd blocks
  int kl0;            // row within the stage of block 0 of this wavefront (block n: + 2 n)
  __device__ __forceinline__ void init(uint32_t ld_bytes, int col0, int ncols, int lane, int wave) {
    const int p = lane & 31;
    kl0 = 8 * wave + (lane >> 5);
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int k3 = (2 * par + (lane >> 5)) & 3;
      colb[par] = (uint32_t)(2 * min(col0 + 8 * (p ^ (k3 << 2)), ncols - 8));
    }
#pragma unroll
    for (int n = 0; n < 4; ++n) voff[n] = (uint32_t)(kl0 + 2 * n) * ld_bytes + colb[n & 1];
  }
  __device__ __forceinline__ void issue(const char* base, char* tile, int wave) const {
#pragma unroll
    for (int n = 0; n < 4; ++n) async_copy16(base + voff[n], tile + (4 * wave + n) * 1024);
  }
  // rows clamped to last_row (partial last stage); k0 = first row of the stage
  __device__ __forceinline__ void issue_clamped(const char* src, uint32_t ld_bytes, int k0, int last_row, char* tile,
                                                int wave) const {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const int k = min(k0 + kl0 + 2 * n, last_row);
      async_copy16(src + (size_t)k * ld_bytes + colb[n & 1], tile + (4 * wave + n) * 1024);
    }
  }
};

__device__ __forceinline__ void zero_slow_tail(char* tile, int kvalid, int t) {   // rows kvalid .. 31 of a slow tile
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = t + 256 * i;                       // 16-byte piece; 32 pieces per row
    if ((q >> 5) >= kvalid) *reinterpret_cast<uint4*>(tile + q * 16) = make_uint4(0, 0, 0, 0);
  }
}

// one operand fragment (32 columns x 16 k) of a slow tile: two transposing reads
__device__ __forceinline__ bf16x8_t read_slow1(const char* tile, int off, int ks) {
  const char* p = tile + off + ks * (16 * 512);
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SBP_LDS s16x4_t*)(p));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SBP_LDS s16x4_t*)(p + 4 * 512));
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// The MFMAs of a step run block row by block row (mfma_step below); the fragments are read in the
// order in which they are first needed - b[0], a[0], b[1..3], a[1..] - so that the waits the compiler
// places before each MFMA cover only reads issued long before.
template <bool SWAP, int FM>
__device__ __forceinline__ void mfma_step(f32x16_t (&acc)[FM][4], const bf16x8_t (&a)[FM], const bf16x8_t (&b)[4]) {
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0)
                       : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
}

// Instruction order of a step, given to the scheduler as a pipeline of groups (the code of the step
// is written before the call): NM slots of one MFMA each; the first slots also take two LDS reads
// each until the step's reads are out, the remaining slots share the step's copies evenly.
//   * reads early: the last MFMAs of a step run while the last reads land, so the wait before the
//     barrier (and before the next step's first MFMA) finds them done;
//   * copies spread out: a burst of copies fills the address queue of the memory pipeline and the
//     wavefront - and with it the MFMA stream - stalls at the next copy;
//   * copies after reads, also in program order: the compiler cannot tell the ring's buffers apart
//     and keeps LDS reads and copies in the order in which they are written.
template <int MASK, int N>
__device__ __forceinline__ void sched_group() {
  if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
template <int NM, int NREAD, int NCOPY, int I>
__device__ __forceinline__ void step_slots() {
  constexpr int R = (NREAD + 1) / 2;                 // slots that carry reads
  static_assert(R <= NM && (NCOPY == 0 || R < NM), "a step has room for its reads and copies");
  sched_group<0x008, 1>();
  if constexpr (I < R) {
    sched_group<0x100, (NREAD - 2 * I >= 2 ? 2 : 1)>();
  } else {
    constexpr int C = NM - R, j = I - R;
    sched_group<0x010, (NCOPY * (j + 1)) / C - (NCOPY * j) / C>();
  }
  if constexpr (I + 1 < NM) step_slots<NM, NREAD, NCOPY, I + 1>();
}
template <int NM, int NREAD, int NCOPY>
__device__ __forceinline__ void interleave_step() {
  // (a step of the 64-row dX tile has 4 MFMAs for 9 reads: no room for this pattern, the compiler's own order stands)
  if constexpr ((NREAD + 1) / 2 < NM || ((NREAD + 1) / 2 == NM && NCOPY == 0)) step_slots<NM, NREAD, NCOPY, 0>();
}

// ---- the stage ring ------------------------------------------------------------------------------
// P supplies: prefetch(s) - row ids of stage s into registers (gathered operand only);
// issue_a / issue_b(s, buf, partial) - the copies of the two operands of stage s (issue_a after
// prefetch(s + 1)); read(buf, ks, a, b) - the fragments of step ks; zero_tail(buf, kvalid); SWAP; FM
// (accumulator block rows); STAGE (bytes of a stage); CPA, CPB (copies per wavefront and stage of the
// two operands); NREAD (LDS reads per step); NPRE (LDS reads of a prefetch).
//
// Iteration s consumes stage s in two steps and issues stage s + 3: operand A behind the reads of step
// 0, operand B behind those of step 1.  The barrier between the steps publishes stage s + 1 and
// retires stage s, whose buffer takes stage s + 4 in the next iteration.
template <class P, int CPS>
__device__ __forceinline__ void wait_stage_runtime(bool next2, bool next3a) {   // wave-uniform arguments
  if (next2 && next3a) wait_async_copies<CPS + P::CPA>();
  else if (next2) wait_async_copies<CPS>();
  else wait_async_copies<0>();
}

// the steady state, stages s .. upto - 1: stage s + 3 exists and is not the last one.  EXTRA: with the problem's extra
// work on the fragments of every step (DwProb: the column sums)
template <class P, bool EXTRA>
__device__ __forceinline__ void ring_steady(char* smem, P& pb, int& s, int upto, f32x16_t (&acc)[P::FM][4],
                                            bf16x8_t (&pa)[P::FM], bf16x8_t (&pbf)[4], bf16x8_t (&qa)[P::FM],
                                            bf16x8_t (&qb)[4]) {
  constexpr int STAGE = P::STAGE, CPS = P::CPA + P::CPB, FM = P::FM, NM = 4 * P::FM + P::NEXTRA;
  for (; s < upto; ++s) {
    const char* cur = smem + (s & 3) * STAGE;
    const char* nxt = smem + ((s + 1) & 3) * STAGE;
    char* dst = smem + ((s + 3) & 3) * STAGE;
    pb.prefetch(s + NS);
    pb.read(cur, 1, qa, qb);
    pb.issue_a(s + 3, dst, false);
    mfma_step<P::SWAP, FM>(acc, pa, pbf);
    if constexpr (EXTRA) pb.extra(pa);
    interleave_step<NM, P::NREAD + P::NPRE, P::CPA>();
    wait_async_copies<CPS + P::CPA>();          // stage s + 1 has landed (s + 2 and half of s + 3 may be in flight)
    lds_barrier();
    pb.read(nxt, 0, pa, pbf);
    pb.issue_b(s + 3, dst, false);
    mfma_step<P::SWAP, FM>(acc, qa, qb);
    if constexpr (EXTRA) pb.extra(qa);
    interleave_step<NM, P::NREAD, P::CPB>();
  }
}

// P::PHASED: the extra work runs in the steady stages [pb.extra_begin, pb.extra_end) only (three copies of the steady
// loop, the middle one with it), and in the last NS stages iff pb.extra_drain.
template <class P>
__device__ __forceinline__ void ring_loop(char* smem, P& pb, int nk, bool tail, int kvalid_last,
                                          f32x16_t (&acc)[P::FM][4]) {
  constexpr int STAGE = P::STAGE, CPS = P::CPA + P::CPB, FM = P::FM, NM = 4 * P::FM + P::NEXTRA;
  static_assert(NS == 4, "buffer arithmetic below assumes a ring of four");
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nk) {
      pb.prefetch(s + 1);
      pb.issue_a(s, smem + s * STAGE, tail && s == nk - 1);
      pb.issue_b(s, smem + s * STAGE, tail && s == nk - 1);
    }
  wait_copies_runtime<CPS>(min(NS - 2, nk - 1));
  lds_barrier();
  if (tail && nk == 1) {
    pb.zero_tail(smem, kvalid_last);
    lds_barrier();
  }
  bf16x8_t pa[FM], pbf[4], qa[FM], qb[4];
  pb.read(smem, 0, pa, pbf);

  int s = 0;
  bool drain_extra = true;
  if constexpr (P::PHASED) {
    ring_steady<P, false>(smem, pb, s, min(pb.extra_begin, nk - NS), acc, pa, pbf, qa, qb);
    ring_steady<P, true>(smem, pb, s, min(pb.extra_end, nk - NS), acc, pa, pbf, qa, qb);
    ring_steady<P, false>(smem, pb, s, nk - NS, acc, pa, pbf, qa, qb);
    drain_extra = pb.extra_drain;
  } else {
    ring_steady<P, true>(smem, pb, s, nk - NS, acc, pa, pbf, qa, qb);
  }
  // drain: the same steps with the end of the operand in view
  for (; s < nk; ++s) {
    const char* cur = smem + (s & 3) * STAGE;
    char* nxt = smem + ((s + 1) & 3) * STAGE;
    char* dst = smem + ((s + 3) & 3) * STAGE;
    const bool more = s + 3 < nk, last_partial = tail && s + 3 == nk - 1;
    if (more) pb.prefetch(s + NS);
    pb.read(cur, 1, qa, qb);
    if (more) pb.issue_a(s + 3, dst, last_partial);
    mfma_step<P::SWAP, FM>(acc, pa, pbf);
    if (drain_extra) pb.extra(pa);
    interleave_step<NM, P::NREAD, 0>();
    if (s + 1 < nk) wait_stage_runtime<P, CPS>(s + 2 < nk, more);
    lds_barrier();
    if (tail && s + 1 == nk - 1) {
      pb.zero_tail(nxt, kvalid_last);
      lds_barrier();
    }
    pb.read(nxt, 0, pa, pbf);                   // past the last stage: reads a stale buffer, never used
    if (more) pb.issue_b(s + 3, dst, last_partial);
    mfma_step<P::SWAP, FM>(acc, qa, qb);
    if (drain_extra) pb.extra(qa);
    interleave_step<NM, P::NREAD, 0>();
  }
  lds_barrier();
}

// ---- dX = dY_k W ---------------------------------------------------------------------------------
template <int BMX>
struct DxProb {
  static constexpr bool SWAP = true;            // lane ends with 4 consecutive input channels of one row
  static constexpr int FM = BMX / 64, CPA = FM, CPB = 4, NREAD = FM + 8, NPRE = 0, NEXTRA = 0;
  static constexpr bool PHASED = false;
  __device__ __forceinline__ void extra(const bf16x8_t (&)[FM]) {}
  static constexpr int A_BYTES = BMX * KB * 2, STAGE = A_BYTES + TILE_BYTES;
  RowCopy<FM> ca;
  SlowCopy cb;
  const char* a_src;
  const char* b_src;
  uint32_t b_stride;
  int wave, a_off[2], b_off[4];
  __device__ __forceinline__ void prefetch(int) {}
  __device__ __forceinline__ void issue_a(int s, char* buf, bool) { ca.issue(a_src + (size_t)s * (KB * 2), buf, wave); }
  __device__ __forceinline__ void issue_b(int s, char* buf, bool) {
    cb.issue(b_src + (size_t)s * b_stride, buf + A_BYTES, wave);
  }
  __device__ __forceinline__ bf16x8_t read_a(const char* buf, int ks, int f) const {
    return *reinterpret_cast<const bf16x8_t*>(buf + a_off[ks] + f * (32 * KB * 2));
  }
  __device__ __forceinline__ void read(const char* buf, int ks, bf16x8_t (&a)[FM], bf16x8_t (&b)[4]) const {
    b[0] = read_slow1(buf + A_BYTES, b_off[0], ks);
    a[0] = read_a(buf, ks, 0);
#pragma unroll
    for (int f = 1; f < 4; ++f) b[f] = read_slow1(buf + A_BYTES, b_off[f], ks);
#pragma unroll
    for (int f = 1; f < FM; ++f) a[f] = read_a(buf, ks, f);
  }
  __device__ __forceinline__ void zero_tail(char*, int) const {}
};

template <int BMX>
__device__ __forceinline__ void dx_tile(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx_in,
                                        const int32_t* __restrict__ idx_out, const uint16_t* __restrict__ W, int K,
                                        int Cin, int Cout, uint16_t* __restrict__ dX, int m0, int n0) {
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  constexpr int FM = BMX / 64;
  const int wm = (wave >> 1) * (BMX / 2), wn = (wave & 1) * 128;

  DxProb<BMX> pb;
  pb.wave = wave;
  pb.ca.init(idx_in, (uint32_t)Cout * 2u, m0, K, lane, wave);
  pb.cb.init((uint32_t)Cin * 2u, n0, Cin, lane, wave);
  pb.a_src = reinterpret_cast<const char*>(dY);
  pb.b_src = reinterpret_cast<const char*>(W);
  pb.b_stride = (uint32_t)KB * (uint32_t)Cin * 2u;
  {
    const int row = wm + (lane & 31), sw = (lane >> 2) & 3;
    pb.a_off[0] = row * (KB * 2) + ((((lane >> 5)) ^ sw) << 4);
    pb.a_off[1] = row * (KB * 2) + (((2 + (lane >> 5)) ^ sw) << 4);
  }
  slow_tile_lane_offs<BT, 4>(wn, lane, pb.b_off);
  // output row of every tile row (-1 past the end), behind the ring; published by the ring's barriers
  int* orow = reinterpret_cast<int*>(smem + RING);
  if (t < BMX) orow[t] = m0 + t < K ? (idx_out ? idx_out[m0 + t] : m0 + t) : -1;

  f32x16_t acc[FM][4];
  zero_acc<FM, 4>(acc);
  ring_loop(smem, pb, Cout / KB, false, KB, acc);

  // epilogue: round to bf16, stage up to 128 rows at a time through LDS, write whole 16-byte pieces of the
  // (scattered) rows.  Register v of lane l of block (i, j) is
  // C[row wm + 32 i + (l & 31)][column wn + 32 j + 8 (v >> 2) + 4 (l >> 5) + (v & 3)].
  constexpr int PITCH = BT * 2 + 16;
  constexpr int BPP = FM >= 2 ? 2 : 1;             // accumulator block rows per wavefront and pass
  constexpr int HALF = 32 * BPP;                   // staged rows per half (wavefront row) and pass
  const int pc = t & 31, pr = t >> 5;
  const bool col_ok = n0 + 8 * pc < Cin;
#pragma unroll
  for (int pass = 0; pass < FM / BPP; ++pass) {
#pragma unroll
    for (int ii = 0; ii < BPP; ++ii) {
      const int i = BPP * pass + ii;
      char* row = smem + ((wave >> 1) * HALF + ii * 32 + (lane & 31)) * PITCH + (wn + 4 * (lane >> 5)) * 2;
#pragma unroll
      for (int jn = 0; jn < 4; ++jn)
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
    for (int p = 0; p < 2 * HALF / 8; ++p) {
      const int r = pr + 8 * p;                   // staged row: half r / HALF, block (r % HALF) / 32, row r & 31
      const int o = orow[(r / HALF) * (BMX / 2) + 32 * (BPP * pass + (r % HALF) / 32) + (r & 31)];
      if (o >= 0 && col_ok)
        *reinterpret_cast<uint4*>(dX + (long long)o * Cin + n0 + 8 * pc) =
            *reinterpret_cast<const uint4*>(smem + r * PITCH + pc * 16);
    }
    __syncthreads();
  }
}

// ---- dW partial = dY_k[j0:j1]^T X_k[j0:j1] -----------------------------------------------------------
// DB: the unit also sums the columns of its dY panel (the layer's bias gradient: db[o] = sum_j dY[j][o]) over a part of
// its rows: the units of one tile row and split all hold the same dY panel and share the work, tile column c of n taking
// the c-th of n equal runs of the steady stages and the last column the final stages as well (the sums cost vector
// instructions between the matrix instructions, about a ninth of a stage: left to one tile column they made its units
// the longest of the grid).  Every unit writes one partial per column of its panel.  The sums come from
// the dY fragments that are in registers anyway: lane l of fragment i holds 8 consecutive j of column 32 i + l % 32 (j group
// l / 32), added with four v_dot2_f32_bf16 against (1, 1) into one fp32 sum per fragment row on the vector ALU, which is
// otherwise idle here.  (Summing on the matrix cores - a fifth product with an operand of ones - needs accumulator
// registers beyond the 256 the tile already fills, and the compiler then shuffles accumulators every step.)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
// XT: X_k lies in memory in groups of 8 rows, [row group][channel][8 rows] (one 16-byte piece per channel and group): the
// contraction index is contiguous, a stage is 4 groups x 256 pieces that are copied as they lie (a copy instruction takes
// 64 consecutive pieces of one group) and a fragment is one 16-byte LDS read per lane (lane l: group l / 32 of the step,
// channel l % 32) instead of two transposing reads.
struct GroupCopy {
  uint32_t voff[4];       // this lane's piece of group n of a stage, in bytes from the stage's first group
  __device__ __forceinline__ void init(uint32_t Cin, int col0, int lane, int wave) {
    const uint32_t c = (uint32_t)min(col0 + 64 * wave + lane, (int)Cin - 1);
#pragma unroll
    for (int n = 0; n < 4; ++n) voff[n] = ((uint32_t)n * Cin + c) * 16u;
  }
  // groups g0 .. g0 + 3 of the operand
  __device__ __forceinline__ void issue(const char* src, uint32_t Cin, int g0, char* tile, int wave) const {
    const char* base = src + (size_t)g0 * Cin * 16u;
#pragma unroll
    for (int n = 0; n < 4; ++n) async_copy16(base + voff[n], tile + (n * 256 + 64 * wave) * 16);
  }
  // the same, groups clamped to last_group (partial last stage)
  __device__ __forceinline__ void issue_clamped(const char* src, uint32_t Cin, int g0, int last_group, char* tile, int wave) const {
#pragma unroll
    for (int n = 0; n < 4; ++n)
      async_copy16(src + (size_t)min(g0 + n, last_group) * Cin * 16u + voff[0], tile + (n * 256 + 64 * wave) * 16);
  }
};

template <bool GATHER, bool DB, bool XT = false, int DBH = 0>
struct DwProb {
  static constexpr bool SWAP = false;
  static constexpr int FM = 4, CPA = 4, CPB = 4, STAGE = 2 * TILE_BYTES, NEXTRA = 0;
  static constexpr int NREAD = XT ? 12 : 16, NPRE = GATHER ? 2 : 0;   // the 4 id reads pair up into 2 instructions
  static constexpr bool PHASED = DB;
  int extra_begin, extra_end;   // steady stages in which this unit sums columns
  bool extra_drain;             // ... and whether it does in the final stages
  // The two wavefronts that own the same rows of the tile (and so hold the same dY fragments) share the sums: DBH = 0
  // adds up fragments 0 and 1, DBH = 1 fragments 2 and 3.
  float accdb[DB ? 2 : 1];         // (one running sum per word of a fragment - independent chains - measured 0.7 % slower)
  __device__ __forceinline__ void init_db(int) {
    if constexpr (DB) {
#pragma unroll
      for (int i = 0; i < 2; ++i) accdb[i] = 0.f;
    }
  }
  __device__ __forceinline__ void extra(const bf16x8_t (&a)[4]) {
    if constexpr (DB) {
      const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const u32x4_t w = __builtin_bit_cast(u32x4_t, a[2 * DBH + i]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          unsigned wq = w[q];
          asm("" : "+v"(wq));       // (without this the four words of a fragment were folded into its first one)
          accdb[i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, wq), ones, accdb[i], false);
        }
      }
    }
  }
  SlowCopy ca, cb;
  GroupCopy cg;           // XT: copies of X_k
  int last_group;         // XT: last row group of the split, counted from b_src
  uint32_t cin;
  const char* a_src;      // dY (GATHER) or dY + j0 rows
  const char* b_src;      // X_k + j0 rows (XT: + j0 / 8 row groups)
  const int* rows;        // LDS table: row of dY for kept row j0 + i
  uint32_t a_ld, b_ld, rid[4], rid_next[4];
  int wave, nrows, a_off[4], b_off[4];   // nrows = j1 - j0
  __device__ __forceinline__ void prefetch(int s) {
    if (GATHER) {
#pragma unroll
      for (int n = 0; n < 4; ++n) rid_next[n] = (uint32_t)rows[s * KB + ca.kl0 + 2 * n];
    }
  }
  __device__ __forceinline__ void issue_a(int s, char* buf, bool partial) {
    if (GATHER) {
#pragma unroll
      for (int n = 0; n < 4; ++n) async_copy16(a_src + (rid[n] * a_ld + ca.colb[n & 1]), buf + (4 * wave + n) * 1024);
#pragma unroll
      for (int n = 0; n < 4; ++n) rid[n] = rid_next[n];
    } else if (!partial) {
      ca.issue(a_src + (size_t)s * KB * a_ld, buf, wave);
    } else {
      ca.issue_clamped(a_src, a_ld, s * KB, nrows - 1, buf, wave);
    }
  }
  __device__ __forceinline__ void issue_b(int s, char* buf, bool partial) {
    if constexpr (XT) {
      if (!partial) cg.issue(b_src, cin, s * (KB / 8), buf + TILE_BYTES, wave);
      else cg.issue_clamped(b_src, cin, s * (KB / 8), last_group, buf + TILE_BYTES, wave);
    } else {
      if (!partial) cb.issue(b_src + (size_t)s * KB * b_ld, buf + TILE_BYTES, wave);
      else cb.issue_clamped(b_src, b_ld, s * KB, nrows - 1, buf + TILE_BYTES, wave);
    }
  }
  __device__ __forceinline__ bf16x8_t read_b(const char* buf, int ks, int f) const {
    if constexpr (XT) return *reinterpret_cast<const bf16x8_t*>(buf + TILE_BYTES + b_off[f] + ks * (2 * 256 * 16));
    else return read_slow1(buf + TILE_BYTES, b_off[f], ks);
  }
  __device__ __forceinline__ void read(const char* buf, int ks, bf16x8_t (&a)[4], bf16x8_t (&b)[4]) const {
    b[0] = read_b(buf, ks, 0);
    a[0] = read_slow1(buf, a_off[0], ks);
#pragma unroll
    for (int f = 1; f < 4; ++f) b[f] = read_b(buf, ks, f);
#pragma unroll
    for (int f = 1; f < 4; ++f) a[f] = read_slow1(buf, a_off[f], ks);
  }
  // rows kvalid .. 31 of the last stage: the dY tile is zeroed, so whatever X_k holds there adds nothing (XT: the rows of a
  // partly filled group come from memory, where rows past K are stored as zeros and rows of the next split are finite
  // values of X_k that meet zeros of dY; whole groups past the split are copies of its last group)
  __device__ __forceinline__ void zero_tail(char* buf, int kvalid) const {
    zero_slow_tail(buf, kvalid, threadIdx.x);
    if constexpr (!XT) zero_slow_tail(buf + TILE_BYTES, kvalid, threadIdx.x);
  }
};

template <bool GATHER, bool DB, bool XT, int DBH>
__device__ __forceinline__ void dw_tile_impl(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx,
                                        const uint16_t* __restrict__ Xk, int Cin, int Cout, int j0, int j1,
                                        float* __restrict__ part, int m0, int n0, float* __restrict__ dbp, int db_part,
                                        int db_parts) {
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  const int nrows = j1 - j0;
  const int nk = (nrows + KB - 1) / KB;

  DwProb<GATHER, DB, XT, DBH> pb;
  pb.init_db(lane);
  {
    const int steady = max(nk - NS, 0);
    pb.extra_begin = steady * db_part / db_parts;
    pb.extra_end = steady * (db_part + 1) / db_parts;
    pb.extra_drain = db_part == db_parts - 1;
  }
  pb.wave = wave;
  pb.nrows = nrows;
  pb.a_ld = (uint32_t)Cout * 2u;
  pb.b_ld = (uint32_t)Cin * 2u;
  pb.ca.init(pb.a_ld, m0, Cout, lane, wave);
  pb.cin = (uint32_t)Cin;
  pb.last_group = 0;
  if constexpr (XT) {       // j0 is a multiple of 8 (host)
    pb.cg.init((uint32_t)Cin, n0, lane, wave);
    pb.b_src = reinterpret_cast<const char*>(Xk) + (size_t)(j0 >> 3) * Cin * 16u;
    pb.last_group = ((nrows + 7) >> 3) - 1;
  } else {
    pb.cb.init(pb.b_ld, n0, Cin, lane, wave);
    pb.b_src = reinterpret_cast<const char*>(Xk) + (size_t)j0 * pb.b_ld;
  }
  pb.rows = nullptr;
  if (GATHER) {
    int* rows = reinterpret_cast<int*>(smem + RING);        // one stage more than the split has: ids are read ahead
#pragma unroll 4
    for (int i = t; i < (nk + 1) * KB; i += 256) rows[i] = idx[min(j0 + i, j1 - 1)];
    __syncthreads();
    pb.rows = rows;
    pb.a_src = reinterpret_cast<const char*>(dY);
#pragma unroll
    for (int n = 0; n < 4; ++n) pb.rid[n] = (uint32_t)rows[pb.ca.kl0 + 2 * n];
  } else {
    pb.a_src = reinterpret_cast<const char*>(dY) + (size_t)j0 * pb.a_ld;
  }
  slow_tile_lane_offs<BT, 4>(wm, lane, pb.a_off);
  if constexpr (XT) {
#pragma unroll
    for (int f = 0; f < 4; ++f) pb.b_off[f] = ((lane >> 5) * 256 + wn + 32 * f + (lane & 31)) * 16;
  } else {
    slow_tile_lane_offs<BT, 4>(wn, lane, pb.b_off);
  }

  f32x16_t acc[4][4];
  zero_acc<4, 4>(acc);
  const bool tail = (nrows % KB) != 0;
  ring_loop(smem, pb, nk, tail, nrows - (nk - 1) * KB, acc);

  if constexpr (DB) {
    // lanes l and l + 32 hold the two j groups of column 32 i + l % 32; every wavefront writes the sums of its two fragments
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float both = pb.accdb[i] + __shfl_xor(pb.accdb[i], 32);
      const int o = m0 + wm + 32 * (2 * DBH + i) + (lane & 31);
      if (lane < 32 && o < Cout) dbp[o] = both;
    }
  }
  // register v of lane l of block (i, j) is C[row wm + 32 i + 8 (v >> 2) + 4 (l >> 5) + (v & 3)][col wn + 32 j + (l & 31)]
  if (m0 + BT <= Cout && n0 + BT <= Cin) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float* prow_ = part + (long long)(m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * Cin + n0 + wn +
                       (lane & 31);
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) prow_[32 * jn] = acc[i][jn][v];
      }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) {
          const int col = n0 + wn + 32 * jn + (lane & 31);
          if (o < Cout && col < Cin) part[(long long)o * Cin + col] = acc[i][jn][v];
        }
      }
  }
}

// db_part of db_parts: this unit's share of the column sums (DB)
template <bool GATHER, bool DB = false, bool XT = false>
__device__ __forceinline__ void dw_tile(char* smem, const uint16_t* __restrict__ dY, const int32_t* __restrict__ idx,
                                        const uint16_t* __restrict__ Xk, int Cin, int Cout, int j0, int j1,
                                        float* __restrict__ part, int m0, int n0, float* __restrict__ dbp = nullptr,
                                        int db_part = 0, int db_parts = 1) {
  if constexpr (DB) {
    // (wave-uniform: both versions run the same barriers in the same order)
    if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) & 1)
      dw_tile_impl<GATHER, true, XT, 1>(smem, dY, idx, Xk, Cin, Cout, j0, j1, part, m0, n0, dbp, db_part, db_parts);
    else
      dw_tile_impl<GATHER, true, XT, 0>(smem, dY, idx, Xk, Cin, Cout, j0, j1, part, m0, n0, dbp, db_part, db_parts);
  } else {
    dw_tile_impl<GATHER, false, XT, 0>(smem, dY, idx, Xk, Cin, Cout, j0, j1, part, m0, n0, dbp, 0, 1);
  }
}

}  // namespace big
}  // namespace sbp
#endif
