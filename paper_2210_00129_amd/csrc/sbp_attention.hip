// Backward of scaled dot-product attention on the kept tokens (paper: main text section Design Strategies,
// "How to apply SBP on MHSA?", variant "Drop QKV"; supplement section Gradient Calculation of Attention
// Layers, eq:grad_qkv with the gradient dropout of eq:sbp_sep_on_query / eq:sbp_sep_on_key applied to dropped
// queries AND dropped keys).  Per sample and head, over the kept tokens i, j only:
//   S_ij  = exp(scale q_i.k_j - lse_i)          lse_i: log-sum-exp of the forward over ALL keys
//   dV_j  = sum_i S_ij dA_i
//   dM_ij = S_ij (dA_i.v_j - dA_i.A_i)          the softmax row term sum_l S_il dS_il equals dA_i.A_i (A = S V)
//   dQ_i  = scale sum_j dM_ij k_j,   dK_j = scale sum_i dM_ij q_i
// Two kernels: an MFMA kernel for bf16 (one workgroup per sample and head, all kept tokens of the head in
// LDS) and a plain fp32-arithmetic kernel for fp32 tensors and for sizes beyond the LDS budget.
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "sbp_internal.h"
#include "sbp_mfma_gemm.h"

namespace sbp {

static constexpr float kLog2e = 1.4426950408889634f;

// ------------------------------------------------------------------------------------------------
// plain kernel: an "owner" token per group of d/16 lanes; PHASE 0 owns a key (dK, dV, loop over the
// queries), PHASE 1 owns a query (dQ, loop over the keys).  Sums run in token order: deterministic.
// ------------------------------------------------------------------------------------------------
template <typename T> struct AtIO;
template <> struct AtIO<uint16_t> {
  static __device__ __forceinline__ void load16(const uint16_t* p, float (&v)[16]) {
    const uint4 a = reinterpret_cast<const uint4*>(p)[0], b = reinterpret_cast<const uint4*>(p)[1];
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) { v[2 * i] = bf16_lo(w[i]); v[2 * i + 1] = bf16_hi(w[i]); }
  }
  static __device__ __forceinline__ void store16(uint16_t* p, const float (&v)[16]) {
    uint32_t w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = bf16_pack(v[2 * i], v[2 * i + 1]);
    reinterpret_cast<uint4*>(p)[0] = make_uint4(w[0], w[1], w[2], w[3]);
    reinterpret_cast<uint4*>(p)[1] = make_uint4(w[4], w[5], w[6], w[7]);
  }
};
template <> struct AtIO<float> {
  static __device__ __forceinline__ void load16(const float* p, float (&v)[16]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 a = reinterpret_cast<const float4*>(p)[i];
      v[4 * i] = a.x; v[4 * i + 1] = a.y; v[4 * i + 2] = a.z; v[4 * i + 3] = a.w;
    }
  }
  static __device__ __forceinline__ void store16(float* p, const float (&v)[16]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) reinterpret_cast<float4*>(p)[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
  }
};

__device__ __forceinline__ float dot16(const float (&a)[16], const float (&b)[16]) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s = fmaf(a[i], b[i], s);
  return s;
}
__device__ __forceinline__ float group_sum(float v, int lanes) {   // over `lanes` (1, 2, 4 or 8) adjacent lanes
  for (int m = 1; m < lanes; m <<= 1) v += __shfl_xor(v, m);
  return v;
}

template <typename T, int PHASE>
__global__ void __launch_bounds__(256) attn_bwd_plain_kernel(const T* __restrict__ qkv, const T* __restrict__ A,
                                                              const T* __restrict__ dA, const float* __restrict__ lse,
                                                              int n_k, int h, int d, float scale, T* __restrict__ dqkv) {
  const int cper = d / 16, owners = 256 / cper;
  const int o = blockIdx.x * owners + (int)threadIdx.x / cper, c = (int)threadIdx.x % cper;
  const int head = blockIdx.y, b = blockIdx.z;
  const int tok = min(o, n_k - 1);
  const long long row0 = (long long)b * n_k, ldq = 3LL * h * d, lda = (long long)h * d;
  const int col = head * d + 16 * c;
  const T* q_base = qkv + col;
  const T* k_base = qkv + (long long)h * d + col;
  const T* v_base = qkv + 2LL * h * d + col;
  float own1[16], own2[16], acc1[16], acc2[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc1[i] = acc2[i] = 0.f;
  if (PHASE == 0) {
    AtIO<T>::load16(k_base + (row0 + tok) * ldq, own1);
    AtIO<T>::load16(v_base + (row0 + tok) * ldq, own2);
    for (int t = 0; t < n_k; ++t) {
      float q[16], g[16], a[16];
      AtIO<T>::load16(q_base + (row0 + t) * ldq, q);
      AtIO<T>::load16(dA + (row0 + t) * lda + col, g);
      AtIO<T>::load16(A + (row0 + t) * lda + col, a);
      const float s = group_sum(dot16(q, own1), cper);
      const float dp = group_sum(dot16(g, own2), cper);
      const float delta = group_sum(dot16(g, a), cper);
      const float p = expf(scale * s - lse[(row0 + t) * h + head]);
      const float ds = p * (dp - delta) * scale;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc2[i] = fmaf(p, g[i], acc2[i]);       // dV_j += S_ij dA_i
        acc1[i] = fmaf(ds, q[i], acc1[i]);      // dK_j += scale dM_ij q_i
      }
    }
    if (o < n_k) {
      AtIO<T>::store16(dqkv + (row0 + o) * ldq + (long long)h * d + col, acc1);
      AtIO<T>::store16(dqkv + (row0 + o) * ldq + 2LL * h * d + col, acc2);
    }
  } else {
    float a[16];
    AtIO<T>::load16(q_base + (row0 + tok) * ldq, own1);
    AtIO<T>::load16(dA + (row0 + tok) * lda + col, own2);
    AtIO<T>::load16(A + (row0 + tok) * lda + col, a);
    const float delta = group_sum(dot16(own2, a), cper);
    const float l = lse[(row0 + tok) * h + head];
    for (int t = 0; t < n_k; ++t) {
      float k[16], v[16];
      AtIO<T>::load16(k_base + (row0 + t) * ldq, k);
      AtIO<T>::load16(v_base + (row0 + t) * ldq, v);
      const float s = group_sum(dot16(own1, k), cper);
      const float dp = group_sum(dot16(own2, v), cper);
      const float p = expf(scale * s - l);
      const float ds = p * (dp - delta) * scale;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc1[i] = fmaf(ds, k[i], acc1[i]);   // dQ_i += scale dM_ij k_j
    }
    if (o < n_k) AtIO<T>::store16(dqkv + (row0 + o) * ldq + col, acc1);
  }
}

// ------------------------------------------------------------------------------------------------
// MFMA kernel (bf16).  One workgroup of 4 wavefronts per (sample, head).  LDS: the kept rows of q, k, v
// and dA of the head as [NPAD][D] tiles (rows padded with zeros to a multiple of 32, pitch 2 D + 16
// bytes: 16-byte reads of 16 consecutive rows and the transposing reads hit distinct banks), and the
// per-token tables lse * log2(e) and delta = dA.A.
//
// v_mfma_f32_32x32x16_bf16 register layouts (lane l, u = l >> 5):  A[row l & 31][k 8u .. 8u+7],
// B[k 8u .. 8u+7][col l & 31],  C register v = C[row 8 (v >> 2) + 4u + (v & 3)][col l & 31].
// Phase 1, wavefront = block of 32 keys j, loop over blocks of 32 queries i:
//   S = Q_i K_j^T and dP = dA_i V_j^T   (operands: 16-byte row reads, contraction over the head dim)
//   P = exp2(S c - lse_i),  dS = P (dP - delta_i)          in the C layout: rows i, column j = lane
//   dV_j^T += dA_i^T P,  dK_j^T += Q_i^T dS                 contraction over i: C registers 8 ks .. 8 ks + 7
//     hold rows 16 ks + 4u + (0..3) and 16 ks + 8 + 4u + (0..3) of the lane's column, which is a valid B
//     operand if the A operand lists the same rows: two ds_read_b64_tr_b16 of those 4 + 4 token rows.
// Phase 2, wavefront = block of 32 queries i, loop over blocks of keys j: the transposes S^T = K_j Q_i^T,
//   dP^T = V_j dA_i^T (lse_i and delta_i are then per-lane scalars), dQ_i^T += K_j^T dS^T.
// Recomputing S and dP in phase 2 costs 2 of 7 products and saves every cross-wavefront reduction:
// results are deterministic.  Padded rows are zero, so padded queries add nothing (dA = 0, delta = 0) and
// padded keys add nothing to dQ (k = 0); their own outputs are not stored.
// ------------------------------------------------------------------------------------------------
template <int D>
struct AttnLds {
  static constexpr int PITCH = 2 * D + 16;
  static __host__ __device__ size_t bytes(int npad) { return (size_t)4 * npad * PITCH + (size_t)2 * npad * sizeof(float); }
};

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& c, int ks) {
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = bf16_pack(c[8 * ks + 2 * e], c[8 * ks + 2 * e + 1]);
  return __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
}

// A operand [32 head-dim rows from dcol0][16 tokens]: token rows row0 + 4u + (0..3) and row0 + 8 + 4u + (0..3)
template <int PITCH>
__device__ __forceinline__ bf16x8_t read_tr_tokens(const char* tile, int row0, int dcol0, int lane) {
  const int g = lane >> 4, i = lane & 15;
  const char* p = tile + (row0 + 4 * (g >> 1) + (i >> 2)) * PITCH + (dcol0 + 16 * (g & 1) + 4 * (i & 3)) * 2;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SBP_LDS s16x4_t*)(p));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SBP_LDS s16x4_t*)(p + 8 * PITCH));
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// The LDS image of one (sample, head): four tiles and two tables.
template <int D>
struct AttnTiles {
  static constexpr int PITCH = AttnLds<D>::PITCH;
  char *tq, *tk, *tv, *tg;       // q, k, v, dA
  float *lse_s, *delta_s;        // lse * log2(e), dA.A
  __device__ __forceinline__ void place(char* base, int npad) {
    tq = base;
    tk = tq + npad * PITCH;
    tv = tk + npad * PITCH;
    tg = tv + npad * PITCH;
    lse_s = reinterpret_cast<float*>(tg + npad * PITCH);
    delta_s = lse_s + npad;
  }
};

// Where one (sample, head) lives in global memory.
struct AttnItem {
  const uint16_t *q, *a, *g;     // row 0 of the head's columns in qkv (q third), A and dA
  const float* lse;              // lse[row 0][head]
  uint16_t* o;                   // row 0 of the head's columns in dqkv (dQ third)
};
__device__ __forceinline__ AttnItem attn_item(const uint16_t* qkv, const uint16_t* A, const uint16_t* dA, const float* lse,
                                              uint16_t* dqkv, int b, int head, int n_k, int h, int D) {
  const long long row0 = (long long)b * n_k;
  AttnItem it;
  it.q = qkv + row0 * (3LL * h * D) + head * D;
  it.a = A + row0 * ((long long)h * D) + head * D;
  it.g = dA + row0 * ((long long)h * D) + head * D;
  it.lse = lse + row0 * h + head;
  it.o = dqkv + row0 * (3LL * h * D) + head * D;
  return it;
}

// R rounds of 16-byte pieces per thread (NT threads): piece p = token p / CH, chunk p % CH of q, k, v, dA and A.
template <int D, int R>
struct AttnPieces {
  uint4 q[R], k[R], v[R], g[R], a[R];
  template <int NT>
  __device__ __forceinline__ void load(const AttnItem& it, int p0, int n_k, int h) {
    constexpr int CH = D / 8;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int p = p0 + NT * r, tok = p / CH, ch = p % CH;
      q[r] = k[r] = v[r] = g[r] = a[r] = make_uint4(0, 0, 0, 0);
      if (tok < n_k) {                                   // also false for pieces past the padded tile
        const uint16_t* src = it.q + (long long)tok * (3LL * h * D) + 8 * ch;
        q[r] = *reinterpret_cast<const uint4*>(src);
        k[r] = *reinterpret_cast<const uint4*>(src + (long long)h * D);
        v[r] = *reinterpret_cast<const uint4*>(src + 2LL * h * D);
        g[r] = *reinterpret_cast<const uint4*>(it.g + (long long)tok * ((long long)h * D) + 8 * ch);
        a[r] = *reinterpret_cast<const uint4*>(it.a + (long long)tok * ((long long)h * D) + 8 * ch);
      }
    }
  }
  template <int NT>
  __device__ __forceinline__ void store(const AttnTiles<D>& T, int p0, int npieces) const {
    constexpr int CH = D / 8, PITCH = AttnLds<D>::PITCH;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int p = p0 + NT * r, tok = p / CH, ch = p % CH;
      if (p < npieces) {                                 // uniform per wavefront: npieces is a multiple of 64
        const int off = tok * PITCH + ch * 16;
        *reinterpret_cast<uint4*>(T.tq + off) = q[r];
        *reinterpret_cast<uint4*>(T.tk + off) = k[r];
        *reinterpret_cast<uint4*>(T.tv + off) = v[r];
        *reinterpret_cast<uint4*>(T.tg + off) = g[r];
        const uint32_t gw[4] = {g[r].x, g[r].y, g[r].z, g[r].w}, aw[4] = {a[r].x, a[r].y, a[r].z, a[r].w};
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) s += bf16_lo(gw[e]) * bf16_lo(aw[e]) + bf16_hi(gw[e]) * bf16_hi(aw[e]);
        for (int m = 1; m < CH; m <<= 1) s += __shfl_xor(s, m);
        if (ch == 0) T.delta_s[tok] = s;
      }
    }
  }
};

// dK and dV of 32 keys (one wavefront): the keys' fragments live in registers, the queries come block by block from
// LDS tiles (tq, tg: rows of q and dA; lse_s, delta_s: their tables), any number of tiles one after the other.
template <int D>
struct AttnKeyAcc {
  static constexpr int PITCH = AttnLds<D>::PITCH, KS = D / 16, DB = D / 32;
  f32x16_t dv[DB], dk[DB];
  bf16x8_t kf[KS], vf[KS];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int x = 0; x < DB; ++x)
#pragma unroll
      for (int e = 0; e < 16; ++e) dv[x][e] = dk[x][e] = 0.f;
  }
  // fragments of the keys from LDS tiles (rows row0 .. row0 + 31)
  __device__ __forceinline__ void keys_from_lds(const char* tk, const char* tv, int row0, int lane) {
    const int foff = (row0 + (lane & 31)) * PITCH + 16 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8_t*>(tk + foff + ks * 32);
      vf[ks] = *reinterpret_cast<const bf16x8_t*>(tv + foff + ks * 32);
    }
  }
  // ... or straight from memory: k and v of token `tok` (zeros if valid is false), row pointers of the head's columns
  __device__ __forceinline__ void keys_from_memory(const uint16_t* krow, const uint16_t* vrow, bool valid, int lane) {
    const int u = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 a = make_uint4(0, 0, 0, 0), b = a;
      if (valid) {
        a = *reinterpret_cast<const uint4*>(krow + 16 * ks + 8 * u);
        b = *reinterpret_cast<const uint4*>(vrow + 16 * ks + 8 * u);
      }
      kf[ks] = __builtin_bit_cast(bf16x8_t, a);
      vf[ks] = __builtin_bit_cast(bf16x8_t, b);
    }
  }
  __device__ __forceinline__ void run(const char* tq, const char* tg, const float* lse_s, const float* delta_s, int nblk,
                                      float scale, int lane) {
    const int u = lane >> 5, lrow = lane & 31;
    const int foff = lrow * PITCH + 16 * u;              // 16-byte operand read of row (lane & 31), k chunk 8u
    const float c2 = scale * kLog2e;
    for (int ib = 0; ib < nblk; ++ib) {
      f32x16_t s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = dp[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t qf = *reinterpret_cast<const bf16x8_t*>(tq + ib * 32 * PITCH + foff + ks * 32);
        const bf16x8_t gf = *reinterpret_cast<const bf16x8_t*>(tg + ib * 32 * PITCH + foff + ks * 32);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[ks], s, 0, 0, 0);      // rows i, columns j
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf, vf[ks], dp, 0, 0, 0);
      }
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float4 l4 = *reinterpret_cast<const float4*>(lse_s + ib * 32 + 8 * q4 + 4 * u);
        const float4 d4 = *reinterpret_cast<const float4*>(delta_s + ib * 32 + 8 * q4 + 4 * u);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dl[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = __builtin_amdgcn_exp2f(s[4 * q4 + e] * c2 - lv[e]);
          s[4 * q4 + e] = p;
          dp[4 * q4 + e] = p * (dp[4 * q4 + e] - dl[e]);
        }
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8_t pf = pack8(s, ks), dsf = pack8(dp, ks);
#pragma unroll
        for (int x = 0; x < DB; ++x) {
          const bf16x8_t gt = read_tr_tokens<PITCH>(tg, ib * 32 + 16 * ks, 32 * x, lane);
          const bf16x8_t qt = read_tr_tokens<PITCH>(tq, ib * 32 + 16 * ks, 32 * x, lane);
          dv[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt, pf, dv[x], 0, 0, 0);   // rows head dim, columns j
          dk[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, dsf, dk[x], 0, 0, 0);
        }
      }
    }
  }
  // key j = first key of the block + (lane & 31); out: row 0 of the head's columns in dqkv
  __device__ __forceinline__ void store(uint16_t* __restrict__ out, int j, int n_k, int h, float scale, int lane) const {
    const int u = lane >> 5;
    if (j < n_k) {
      uint16_t* o = out + (long long)j * (3LL * h * D);
#pragma unroll
      for (int x = 0; x < DB; ++x)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int dcol = 32 * x + 8 * q4 + 4 * u;
          uint2 w;
          w.x = bf16_pack(dk[x][4 * q4] * scale, dk[x][4 * q4 + 1] * scale);
          w.y = bf16_pack(dk[x][4 * q4 + 2] * scale, dk[x][4 * q4 + 3] * scale);
          *reinterpret_cast<uint2*>(o + (long long)h * D + dcol) = w;
          w.x = bf16_pack(dv[x][4 * q4], dv[x][4 * q4 + 1]);
          w.y = bf16_pack(dv[x][4 * q4 + 2], dv[x][4 * q4 + 3]);
          *reinterpret_cast<uint2*>(o + 2LL * h * D + dcol) = w;
        }
    }
  }
};

// dQ of 32 queries (one wavefront): the queries' fragments, lse and delta live in registers, the keys come block by
// block from LDS tiles (tk, tv).
template <int D>
struct AttnQueryAcc {
  static constexpr int PITCH = AttnLds<D>::PITCH, KS = D / 16, DB = D / 32;
  f32x16_t dq[DB];
  bf16x8_t qf[KS], gf[KS];
  float l, dl;                   // lse * log2(e) and delta of query (lane & 31)
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int x = 0; x < DB; ++x)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[x][e] = 0.f;
  }
  __device__ __forceinline__ void queries_from_lds(const char* tq, const char* tg, const float* lse_s, const float* delta_s,
                                                   int row0, int lane) {
    const int foff = (row0 + (lane & 31)) * PITCH + 16 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8_t*>(tq + foff + ks * 32);
      gf[ks] = *reinterpret_cast<const bf16x8_t*>(tg + foff + ks * 32);
    }
    l = lse_s[row0 + (lane & 31)];
    dl = delta_s[row0 + (lane & 31)];
  }
  // straight from memory: q, dA, A rows of the token (head's columns) and its lse; zeros if valid is false
  __device__ __forceinline__ void queries_from_memory(const uint16_t* qrow, const uint16_t* grow, const uint16_t* arow,
                                                      const float* lse_tok, bool valid, int lane) {
    const int u = lane >> 5;
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 a = make_uint4(0, 0, 0, 0), b = a, c = a;
      if (valid) {
        a = *reinterpret_cast<const uint4*>(qrow + 16 * ks + 8 * u);
        b = *reinterpret_cast<const uint4*>(grow + 16 * ks + 8 * u);
        c = *reinterpret_cast<const uint4*>(arow + 16 * ks + 8 * u);
      }
      qf[ks] = __builtin_bit_cast(bf16x8_t, a);
      gf[ks] = __builtin_bit_cast(bf16x8_t, b);
      const uint32_t gw[4] = {b.x, b.y, b.z, b.w}, aw[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) part += bf16_lo(gw[e]) * bf16_lo(aw[e]) + bf16_hi(gw[e]) * bf16_hi(aw[e]);
    }
    dl = part + __shfl_xor(part, 32);          // the two halves of every 16 columns lie 32 lanes apart
    l = valid ? *lse_tok * kLog2e : 0.f;
  }
  __device__ __forceinline__ void run(const char* tk, const char* tv, int nblk, float scale, int lane) {
    const int u = lane >> 5, lrow = lane & 31;
    const int foff = lrow * PITCH + 16 * u;
    const float c2 = scale * kLog2e;
    for (int jb = 0; jb < nblk; ++jb) {
      f32x16_t s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = dp[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(tk + jb * 32 * PITCH + foff + ks * 32);
        const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(tv + jb * 32 * PITCH + foff + ks * 32);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);      // rows j, columns i
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, gf[ks], dp, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(s[e] * c2 - l);
        dp[e] = p * (dp[e] - dl);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8_t dsf = pack8(dp, ks);
#pragma unroll
        for (int x = 0; x < DB; ++x) {
          const bf16x8_t kt = read_tr_tokens<PITCH>(tk, jb * 32 + 16 * ks, 32 * x, lane);
          dq[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, dsf, dq[x], 0, 0, 0);   // rows head dim, columns i
        }
      }
    }
  }
  __device__ __forceinline__ void store(uint16_t* __restrict__ out, int i, int n_k, int h, float scale, int lane) const {
    const int u = lane >> 5;
    if (i < n_k) {
      uint16_t* o = out + (long long)i * (3LL * h * D);
#pragma unroll
      for (int x = 0; x < DB; ++x)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint2 w;
          w.x = bf16_pack(dq[x][4 * q4] * scale, dq[x][4 * q4 + 1] * scale);
          w.y = bf16_pack(dq[x][4 * q4 + 2] * scale, dq[x][4 * q4 + 3] * scale);
          *reinterpret_cast<uint2*>(o + 32 * x + 8 * q4 + 4 * u) = w;
        }
    }
  }
};

template <int D>
__device__ __forceinline__ void attn_key_block(const AttnTiles<D>& T, int jb, int nblk, int n_k, int h, float scale,
                                               uint16_t* __restrict__ out, int lane) {
  AttnKeyAcc<D> acc;
  acc.zero();
  acc.keys_from_lds(T.tk, T.tv, jb * 32, lane);
  acc.run(T.tq, T.tg, T.lse_s, T.delta_s, nblk, scale, lane);
  acc.store(out, jb * 32 + (lane & 31), n_k, h, scale, lane);
}

template <int D>
__device__ __forceinline__ void attn_query_block(const AttnTiles<D>& T, int ib, int nblk, int n_k, int h, float scale,
                                                 uint16_t* __restrict__ out, int lane) {
  AttnQueryAcc<D> acc;
  acc.zero();
  acc.queries_from_lds(T.tq, T.tg, T.lse_s, T.delta_s, ib * 32, lane);
  acc.run(T.tk, T.tv, nblk, scale, lane);
  acc.store(out, ib * 32 + (lane & 31), n_k, h, scale, lane);
}

// One (sample, head) per workgroup of 4 wavefronts: load, then the key blocks, then the query blocks.  Any
// number of kept tokens whose tiles fit LDS.
template <int D>
__global__ void __launch_bounds__(256, D == 128 ? 1 : 2) attn_bwd_mfma_kernel(const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ A,
                                                             const uint16_t* __restrict__ dA, const float* __restrict__ lse,
                                                             int n_k, int h, float scale, uint16_t* __restrict__ dqkv) {
  constexpr int CH = D / 8;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int npad = (n_k + 31) & ~31, nblk = npad >> 5;
  AttnTiles<D> T;
  T.place(smem, npad);
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const AttnItem it = attn_item(qkv, A, dA, lse, dqkv, blockIdx.y, blockIdx.x, n_k, h, D);
  const int npieces = npad * CH;
  for (int p0 = t; p0 < npieces; p0 += 4 * 256) {      // four rounds of loads in flight per thread
    AttnPieces<D, 4> pc;
    pc.template load<256>(it, p0, n_k, h);
    pc.template store<256>(T, p0, npieces);
  }
  for (int i = t; i < npad; i += 256) T.lse_s[i] = i < n_k ? it.lse[(long long)i * h] * kLog2e : 0.f;
  __syncthreads();
  for (int jb = wave; jb < nblk; jb += 4) attn_key_block<D>(T, jb, nblk, n_k, h, scale, it.o, lane);
  for (int ib = wave; ib < nblk; ib += 4) attn_query_block<D>(T, ib, nblk, n_k, h, scale, it.o, lane);
}

// ------------------------------------------------------------------------------------------------
// Tiled MFMA kernel: any number of kept tokens.  A workgroup owns a chunk of 128 tokens of one (sample, head) in one of
// two roles: as keys (dK, dV of the chunk: every wavefront holds the k and v fragments of its 32 keys in registers and
// the queries - rows of q and dA, lse, delta - stream through LDS in tiles of 128) or as queries (dQ of the chunk: q,
// dA fragments, lse and delta in registers, the keys - rows of k and v - stream through LDS).  The chunk itself never
// touches LDS, a tile is two [128][D] images (37 KB at D = 64): three workgroups per CU.  Every output element is
// written by exactly one wavefront, sums run in token order: deterministic, no atomics.
// ------------------------------------------------------------------------------------------------
static constexpr int kAttnChunk = 128;

// Rows t0 .. t0 + 127 of one (sample, head) into two LDS images of 128 rows (rows past n_k as zeros).  KEY = true:
// the queries' side (q -> t1, dA -> t2, lse * log2 e and delta = dA.A into the tables); false: the keys' side
// (k -> t1, v -> t2).  The loads are issued before the barrier that retires the images' previous contents.
template <int D, bool KEY>
__device__ __forceinline__ void attn_load_tile(const AttnItem& it, int t0, int n_k, int h, char* t1, char* t2,
                                               float* lse_s, float* delta_s) {
  constexpr int CH = D / 8, PITCH = AttnLds<D>::PITCH, R = kAttnChunk * CH / 256;   // 16-byte pieces per thread, tensor and tile
  const int t = threadIdx.x;
  const long long ldq = 3LL * h * D, lda = (long long)h * D;
  uint4 x1[R], x2[R], x3[KEY ? R : 1];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int p = t + 256 * r, tok = t0 + p / CH, ch = p % CH;
    x1[r] = x2[r] = make_uint4(0, 0, 0, 0);
    if constexpr (KEY) x3[r] = make_uint4(0, 0, 0, 0);
    if (tok < n_k) {
      if constexpr (KEY) {
        x1[r] = *reinterpret_cast<const uint4*>(it.q + tok * ldq + 8 * ch);
        x2[r] = *reinterpret_cast<const uint4*>(it.g + tok * lda + 8 * ch);
        x3[r] = *reinterpret_cast<const uint4*>(it.a + tok * lda + 8 * ch);
      } else {
        x1[r] = *reinterpret_cast<const uint4*>(it.q + tok * ldq + (long long)h * D + 8 * ch);
        x2[r] = *reinterpret_cast<const uint4*>(it.q + tok * ldq + 2LL * h * D + 8 * ch);
      }
    }
  }
  float lv = 0.f;
  if (KEY && t < kAttnChunk && t0 + t < n_k) lv = it.lse[(long long)(t0 + t) * h] * kLog2e;
  __syncthreads();                                        // the previous contents have been consumed
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int p = t + 256 * r, tok = p / CH, ch = p % CH;
    *reinterpret_cast<uint4*>(t1 + tok * PITCH + ch * 16) = x1[r];
    *reinterpret_cast<uint4*>(t2 + tok * PITCH + ch * 16) = x2[r];
    if constexpr (KEY) {
      const uint32_t gw[4] = {x2[r].x, x2[r].y, x2[r].z, x2[r].w}, aw[4] = {x3[r].x, x3[r].y, x3[r].z, x3[r].w};
      float sacc = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) sacc += bf16_lo(gw[e]) * bf16_lo(aw[e]) + bf16_hi(gw[e]) * bf16_hi(aw[e]);
      for (int m = 1; m < CH; m <<= 1) sacc += __shfl_xor(sacc, m);
      if (ch == 0) delta_s[tok] = sacc;
    }
  }
  if (KEY && t < kAttnChunk) lse_s[t] = lv;
}

template <int D, bool KEY>
__device__ __forceinline__ void attn_tiled_body(char* smem, const AttnItem& it, int chunk, int n_k, int h, float scale) {
  constexpr int PITCH = AttnLds<D>::PITCH;
  char* t1 = smem;                                   // rows of q (key role) or k (query role)
  char* t2 = t1 + kAttnChunk * PITCH;                // rows of dA or v
  float* lse_s = reinterpret_cast<float*>(t2 + kAttnChunk * PITCH);
  float* delta_s = lse_s + kAttnChunk;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const long long ldq = 3LL * h * D, lda = (long long)h * D;
  const int own = chunk * kAttnChunk + wave * 32 + (lane & 31);     // this lane's token of the chunk
  const bool own_ok = own < n_k;
  const int own_c = min(own, n_k - 1);
  typename std::conditional<KEY, AttnKeyAcc<D>, AttnQueryAcc<D>>::type acc;
  acc.zero();
  if constexpr (KEY) acc.keys_from_memory(it.q + own_c * ldq + (long long)h * D, it.q + own_c * ldq + 2LL * h * D, own_ok, lane);
  else acc.queries_from_memory(it.q + own_c * ldq, it.g + own_c * lda, it.a + own_c * lda, it.lse + (long long)own_c * h, own_ok, lane);
  const int npad = (n_k + 31) & ~31;
  for (int t0 = 0; t0 < npad; t0 += kAttnChunk) {
    const int rows = min(kAttnChunk, npad - t0);            // rows of this tile (a multiple of 32); rows past n_k are zeros
    attn_load_tile<D, KEY>(it, t0, n_k, h, t1, t2, lse_s, delta_s);
    __syncthreads();
    if constexpr (KEY) acc.run(t1, t2, lse_s, delta_s, rows >> 5, scale, lane);
    else acc.run(t1, t2, rows >> 5, scale, lane);
  }
  acc.store(it.o, own, n_k, h, scale, lane);
}

template <int D>
__global__ void __launch_bounds__(256, D == 128 ? 1 : 3) attn_bwd_tiled_kernel(const uint16_t* __restrict__ qkv, const uint16_t* __restrict__ A,
                                                              const uint16_t* __restrict__ dA, const float* __restrict__ lse,
                                                              int n_k, int h, float scale, int nchunks, uint16_t* __restrict__ dqkv) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const AttnItem it = attn_item(qkv, A, dA, lse, dqkv, blockIdx.z, blockIdx.y, n_k, h, D);
  if ((int)blockIdx.x < nchunks) attn_tiled_body<D, true>(smem, it, blockIdx.x, n_k, h, scale);
  else attn_tiled_body<D, false>(smem, it, blockIdx.x - nchunks, n_k, h, scale);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
static constexpr size_t kAttnMaxLds = 160 * 1024;

static size_t attn_lds_bytes(int n_k, int d) {
  const int npad = (n_k + 31) & ~31;
  return d == 32 ? AttnLds<32>::bytes(npad) : d == 64 ? AttnLds<64>::bytes(npad) : AttnLds<128>::bytes(npad);
}

// 2: tiled MFMA kernel, 1: MFMA kernel with one workgroup per (sample, head), 0: plain kernel
int attention_engine(int32_t n_k, int32_t d, int32_t dtype) {
  if (dtype != SBP_BF16) return 0;
  if (d != 32 && d != 64 && d != 128) return 0;
  const Options opt = options();
  if (opt.attn_mode == 1) return 0;                         // explicit overrides (sbp_set_option "attn" = "plain" | "whole" | "tiled")
  if (opt.attn_mode == 3) return 2;
  const bool fits = attn_lds_bytes(n_k, d) <= kAttnMaxLds;
  return fits ? 1 : 2;
}

template <int D>
static void launch_attn_mfma(const uint16_t* qkv, const uint16_t* A, const uint16_t* dA, const float* lse, int B, int n_k,
                             int h, float scale, uint16_t* dqkv, hipStream_t s) {
  const size_t image = AttnLds<D>::bytes((n_k + 31) & ~31);
  if (image > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_mfma_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)kAttnMaxLds);
  SBP_LAUNCH(SBP_PROF_ATTENTION, s, (attn_bwd_mfma_kernel<D>), dim3(h, B), dim3(256), image, s, qkv, A, dA, lse, n_k, h, scale,
             dqkv);
}

template <int D>
static void launch_attn_tiled(const uint16_t* qkv, const uint16_t* A, const uint16_t* dA, const float* lse, int B, int n_k,
                              int h, float scale, uint16_t* dqkv, hipStream_t s) {
  const size_t lds = (size_t)2 * kAttnChunk * AttnLds<D>::PITCH + (size_t)2 * kAttnChunk * sizeof(float);
  if (lds > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bwd_tiled_kernel<D>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
  const int nchunks = (n_k + kAttnChunk - 1) / kAttnChunk;
  SBP_LAUNCH(SBP_PROF_ATTENTION, s, (attn_bwd_tiled_kernel<D>), dim3(2 * nchunks, h, B), dim3(256), lds, s, qkv, A, dA, lse, n_k, h,
             scale, nchunks, dqkv);
}

template <typename T>
static void launch_attn_plain(const T* qkv, const T* A, const T* dA, const float* lse, int B, int n_k, int h, int d, float scale,
                              T* dqkv, hipStream_t s) {
  const int owners = 256 / (d / 16);
  const dim3 grid((unsigned)ceil_div(n_k, owners), h, B);
  {
    ProfScope scope(SBP_PROF_ATTENTION, s);
    hipLaunchKernelGGL((attn_bwd_plain_kernel<T, 0>), grid, dim3(256), 0, s, qkv, A, dA, lse, n_k, h, d, scale, dqkv);
    hipLaunchKernelGGL((attn_bwd_plain_kernel<T, 1>), grid, dim3(256), 0, s, qkv, A, dA, lse, n_k, h, d, scale, dqkv);
  }
}

int32_t launch_backward_attention(const void* qkv, const void* A, const void* dA, const float* lse, int32_t B, int32_t n_k,
                                  int32_t h, int32_t d, float scale, int32_t dtype, void* dqkv, hipStream_t s) {
  const int engine = attention_engine(n_k, d, dtype);
  if (engine) {
    const uint16_t* q = (const uint16_t*)qkv; const uint16_t* a = (const uint16_t*)A; const uint16_t* g = (const uint16_t*)dA;
    uint16_t* o = (uint16_t*)dqkv;
    if (engine == 2) {
      if (d == 32) launch_attn_tiled<32>(q, a, g, lse, B, n_k, h, scale, o, s);
      else if (d == 64) launch_attn_tiled<64>(q, a, g, lse, B, n_k, h, scale, o, s);
      else launch_attn_tiled<128>(q, a, g, lse, B, n_k, h, scale, o, s);
    } else {
      if (d == 32) launch_attn_mfma<32>(q, a, g, lse, B, n_k, h, scale, o, s);
      else if (d == 64) launch_attn_mfma<64>(q, a, g, lse, B, n_k, h, scale, o, s);
      else launch_attn_mfma<128>(q, a, g, lse, B, n_k, h, scale, o, s);
    }
  } else if (dtype == SBP_BF16) {
    launch_attn_plain<uint16_t>((const uint16_t*)qkv, (const uint16_t*)A, (const uint16_t*)dA, lse, B, n_k, h, d, scale,
                                (uint16_t*)dqkv, s);
  } else {
    launch_attn_plain<float>((const float*)qkv, (const float*)A, (const float*)dA, lse, B, n_k, h, d, scale, (float*)dqkv, s);
  }
  return check_launch("backward_attention");
}

}  // namespace sbp
