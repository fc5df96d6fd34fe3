// Internal declarations shared by the translation units of libsbp (not part of the ABI).
#ifndef SBP_INTERNAL_H_
#define SBP_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "sbp.h"
#include "sbp_fastdiv.h"

namespace sbp {

// Records a formatted message for sbp_last_error() and returns `code`.
int32_t fail(int32_t code, const char* fmt, ...);
// Turns the state left by a kernel launch into a status code.
int32_t check_launch(const char* what);

// Brackets the launches issued during its lifetime with a pair of events when profiling is on.
struct ProfScope {
  ProfScope(int cls, hipStream_t s);
  ~ProfScope();
  int cls_;
  hipStream_t s_;
  void* rec_;
};

// Measurement aid: where the kernels that support it write per-workgroup time stamps (NULL, 0: nowhere).
void timeline_target(unsigned long long** buf, int* capacity_records);

#define SBP_LAUNCH(cls, stream, ...)             \
  do {                                            \
    ::sbp::ProfScope _prof_scope((cls), (stream)); \
    hipLaunchKernelGGL(__VA_ARGS__);              \
  } while (0)

// ---- explicit overrides (sbp_set_option): for tests and sweeps; defaults = everything automatic -------------
struct ShapePlan { int cin, cout, bm, rows_long, n_long, rows_short; };   // cin = 0: every shape
struct Options {
  int  tile_mode = 0;                 // 0 automatic, 1 a tile shape of the general engine, 2 the large-tile engine
  int  tile_bm = 128, tile_bn = 128, tile_nw = 4, tile_kb = 64;
  int  dxbm = 0, splits = 0, dxrows = 0;   // 0 = automatic
  bool order_set = false;
  int  order[3] = {0, 1, 2};
  int  nplans = 0;
  ShapePlan plans[8] = {};
  bool debug_plan = false;
  int  dw_rows = 0;
  bool dw_strips = false;             // depthwise backward: the register-strip kernels instead of the LDS-tiled one
  bool batch_spread = false;          // batched linear backward: units dealt to the XCDs in turn instead of in runs
  bool batch_dynamic = false;         // batched linear backward: units taken from the XCD queues with atomic counters
  int attn_mode = 0;       // attention backward: 0 chosen by size, 1 plain kernel, 2 one workgroup per head where it fits, 3 tiled
  bool dw_separate = false, sampler_no_window = false, sampler_no_masks = false, patch_wide = false;
};
Options options();                    // a snapshot (taken under a lock; safe against a concurrent sbp_set_option)

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- sampler -----------------------------------------------------------------------------
int64_t keep_count_host(const sbp_sample_desc& d);
int32_t launch_sample(const sbp_sample_desc& d, int32_t* idx, int32_t* inv, hipStream_t s);
int32_t launch_sample_batch(const sbp_sample_desc* d, int32_t n, int32_t* const* idx, int32_t* const* inv, hipStream_t s);

// ---- row gather --------------------------------------------------------------------------
int32_t launch_gather_rows(const void* X, const int32_t* idx, int64_t K, int32_t C, int32_t elem_bytes,
                           void* Xk, hipStream_t s);

int32_t launch_gather_rows_batch(const sbp_gather_item* items, int32_t n, int32_t elem_bytes, hipStream_t s);
int32_t launch_kmajor_to_rows(const void* Xt, int64_t K, int32_t C, void* Xrows, hipStream_t s);

// patches of a p x p, stride p down-sampling layer: gather [K, p*p*C] rows / scatter them back with zero fill
int32_t launch_patches(bool scatter, const void* src, const int32_t* idx, const int32_t* inv, int32_t B, int32_t H, int32_t W,
                       int32_t C, int32_t p, int64_t K, int32_t elem_bytes, void* dst, hipStream_t s);

// ---- linear backward ---------------------------------------------------------------------
struct LinearPlan {
  bool   mfma;          // bf16 MFMA path (else plain kernels)
  int    bm_w, bn_w;    // tile of both contractions (rows x columns)
  int    splits;        // split-K factor of the dW contraction
  int    rows_per_split;// kept rows per split (multiple of the k-step)
  int    n_big;         // big engine: the first n_big splits have rows_per_split rows, the others rows_small
  int    rows_small;    // big engine: rows of the short splits that fill the end of the schedule (0: none)
  int    seg_order[3];  // big engine: dispatch order of the unit kinds 0 = dX tiles, 1 = long dW units, 2 = short dW units
  int    nw_w;          // wavefronts per block (4 or 8)
  int    kb;            // contraction elements per LDS stage (64: two stages, 32: four stages)
  bool   big;           // 256 x 256 tiles, one workgroup per CU (sbp_mfma_big.h)
  int    dx_bm;         // rows of a dX tile: big engine 256, or 128 where 256-row tiles are too few; general engine 128, or
                        // 64 (in a ring of three stages) for small layers
  int    db_slices;     // partial sums of db (row slices of the column-sum blocks)
  int    db_slice_rows; // kept rows per db slice
  size_t off_partial;   // fp32 [splits, Cout, Cin]
  size_t off_inv;       // int32 [M]
  size_t off_xrows;     // bf16 [K, Cin]: X_k by rows when it came in the row-group layout and the engine reads rows
  size_t bytes;
};
int32_t check_linear_args(const void* dY, const int32_t* idx, const void* Xk, const void* W, int64_t M, int64_t K,
                          int32_t Cin, int32_t Cout, int32_t dtype, const void* dW, const void* dX, uint32_t flags);
LinearPlan plan_linear(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, uint32_t flags);
int32_t launch_backward_linear(const LinearPlan& p, const void* dY, const int32_t* idx, const int32_t* inv,
                               const void* Xk, const void* W, int64_t M, int64_t K, int32_t Cin, int32_t Cout,
                               int32_t dtype, void* dW, float* db, void* dX, void* ws, uint32_t flags,
                               hipStream_t s);

// several independent layers in one launch
struct BatchLayer {
  int    dx_bm, splits, rows_per_split, db_slices, db_slice_rows;
  bool   direct;        // a single split: the dW unit writes dW itself, nothing to reduce
  size_t off, off_dbp, off_inv;   // workspace: split partials (layer-by-layer mode: the layer's whole workspace), db slices, inverse map
};
struct BatchPlan {
  int    n;
  bool   fused;         // one grid for all layers (else layer by layer)
  BatchLayer lay[SBP_MAX_BATCH_LAYERS];
  size_t off_counters;  // the eight queue counters of the common grid
  size_t bytes;
};
BatchPlan plan_linear_batch(const sbp_linear_layer* layers, int32_t n, int32_t dtype);
int32_t launch_backward_linear_batch(const BatchPlan& p, const sbp_linear_layer* layers, int32_t dtype, void* ws,
                                     hipStream_t s);

// inv[idx[j]] = j (no clearing needed: row m is kept iff 0 <= inv[m] < K and idx[inv[m]] == m), and +0 into
// the rows of out[M][row_bytes] that are not kept (row_bytes a multiple of 2)
void launch_build_inverse(const int32_t* idx, int64_t K, int32_t* inv, hipStream_t s);
void launch_zero_dropped_rows(const int32_t* idx, const int32_t* inv, int64_t K, int64_t M, int64_t row_bytes,
                              void* out, hipStream_t s);

// per-channel layer scale on compact rows: partial sums [ls_blocks(K)][C]
int ls_blocks(int64_t K);
int32_t launch_backward_layerscale(const void* dU, const void* Y, const float* gamma, int64_t K, int32_t C, int32_t dtype,
                                   float* dgamma, void* dY, float* partial, uint32_t flags, hipStream_t s);

// ---- attention backward on the kept tokens -------------------------------------------------------
int attention_engine(int32_t n_k, int32_t d, int32_t dtype);   // 1: matrix-core kernel, 0: plain kernel
int32_t launch_backward_attention(const void* qkv, const void* A, const void* dA, const float* lse, int32_t B, int32_t n_k,
                                  int32_t h, int32_t d, float scale, int32_t dtype, void* dqkv, hipStream_t s);

// ---- row-wise steps between the linear layers ------------------------------------------------
int32_t launch_act_rows(const void* dH, const void* Z, int64_t n, int32_t dtype, int32_t act, bool backward, void* out,
                        hipStream_t s);
struct LnPlan {
  bool   fast;          // one wavefront per row, the row in registers
  int    nblocks;       // blocks = partial sums of dgamma / dbeta
  size_t off_partial;   // fp32 [nblocks, 2, C]
  size_t off_stats;     // fp32 [K, 2] (plain path)
  size_t off_inv;       // int32 [M]
  size_t bytes;
};
LnPlan plan_layernorm(int64_t M, int64_t K, int32_t C, int32_t dtype, uint32_t flags);
int32_t launch_backward_layernorm(const LnPlan& p, const void* dU, const void* Xk, const float* gamma, float eps,
                                  const int32_t* idx, const int32_t* inv, int64_t M, int64_t K, int32_t C,
                                  int32_t dtype, float* dgamma, float* dbeta, void* dX, void* ws, uint32_t flags,
                                  hipStream_t s);

// ---- depthwise backward ------------------------------------------------------------------
struct DwPlan {
  int    tiles_y, tiles_x; // spatial tiles of the dWd/db partial reduction
  int    nparts;           // partial accumulators per (tap, channel)
  size_t off_inv;          // int32 [B*H*W]
  size_t off_partial;      // fp32 [nparts, ks*ks+1, C]
  size_t bytes;
};
DwPlan plan_dwconv(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int64_t K, int32_t dtype);
int32_t launch_backward_dwconv(const DwPlan& p, const void* dY, const int32_t* idx, const int32_t* inv,
                               const void* X, const void* Wd, int32_t B, int32_t H, int32_t W, int32_t C,
                               int32_t ks, int32_t pad, int64_t K, int32_t dtype, float* dWd, float* db,
                               void* dX, void* ws, hipStream_t s);

}  // namespace sbp
#endif
