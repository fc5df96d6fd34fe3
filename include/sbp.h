/*
 * sbp.h -- C ABI of the Stochastic-Backpropagation (SBP) hot path for AMD MI355X (gfx950).
 *
 * SBP (arXiv 2210.00129) runs the full forward pass but back-propagates through a random
 * subset of spatial positions only: per layer it caches just the kept rows of the input
 * activation and computes weight / input gradients from the kept rows of the output
 * gradient (paper, section "Calculation of Linear Layers", equation eq:backward_fc_sbp).
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers (HBM); descriptors are host structs.
 *   - Tensors are dense, row-major, no strides: a [R, C] matrix has leading dimension C.
 *     Feature maps are channels-last, i.e. a [B, H, W, C] map is the [B*H*W, C] matrix.
 *   - The library allocates nothing and frees nothing.  Every buffer, including the
 *     workspace, is owned by the caller and only borrowed until the work enqueued on
 *     `stream` has run.  Inputs are never written; outputs are fully overwritten unless a
 *     flag says otherwise.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; none of them synchronises.
 *   - Every argument is validated on the host BEFORE the first HIP call; a failed
 *     validation enqueues nothing.  Return value: SBP_OK or a negative SBP_ERR_* code;
 *     sbp_last_error() gives a thread-local description of the last failure.
 *   - Weight layout is W[Cout, Cin] (Y = X W^T + b).  The paper writes W as [Cin, Cout];
 *     the quantities are the same with the storage transposed.
 *   - No gradient is rescaled by 1/r (the paper's update rule eq:sbp_formula carries 1/B only).
 */
#ifndef SBP_H_
#define SBP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define SBP_OK              0
#define SBP_ERR_NULL       (-1)  /* a required pointer is NULL */
#define SBP_ERR_SHAPE      (-2)  /* a size is non-positive, inconsistent or overflows int32 row ids */
#define SBP_ERR_RATIO      (-3)  /* keep ratio / kept-slot count out of range */
#define SBP_ERR_DTYPE      (-4)  /* unknown element type */
#define SBP_ERR_CAPACITY   (-5)  /* an output buffer is smaller than what would be written */
#define SBP_ERR_WORKSPACE  (-6)  /* workspace NULL/too small/misaligned */
#define SBP_ERR_HIP        (-7)  /* a HIP launch failed (no device, bad stream, ...) */
#define SBP_ERR_FLAGS      (-8)  /* unknown or unsupported flag / mode */

/* element types of activations and weights */
#define SBP_F32   0   /* fp32 storage, fp32 accumulate */
#define SBP_BF16  1   /* bf16 storage, fp32 accumulate (MFMA) */

/* sampler modes */
#define SBP_GRID_PER_CELL 0  /* independent draw in every cell */
#define SBP_GRID_SHARED   1  /* one slot permutation shared by all cells of a sample (regular lattice) */
/* The paper's other strategy, "random mask sampling": per sample exactly round-half-up(k/4 * H*W) (>= 1) of
 * the grid positions, a uniformly random subset without grid structure (those with the smallest hashed keys;
 * ties by position).  idx order: sample-major, prefix rows, kept positions ascending.  cell must be 2. */
#define SBP_RANDOM_MASK   2
/* Temporal subsets (the special case on the temporal dimension cited under eq:sbp_formula): the rows of a
 * sample are P prefix rows and H frames of W positions each; of every `cell` (2..4) consecutive frames k
 * (1..cell) are kept whole, drawn independently per cell; a partial last cell of c' frames keeps
 * round-half-up(k*c'/cell) (>= 1).  idx order: sample-major, prefix rows, kept frames ascending. */
#define SBP_TEMPORAL      3

#define SBP_MAX_BATCH_LAYERS 8   /* most layers / tensors one batched call takes */

/* flags of sbp_backward_linear */
#define SBP_FLAG_DY_COMPACT     1u  /* dY is already compact: [K, Cout], row j belongs to idx[j] */
#define SBP_FLAG_DX_COMPACT     2u  /* write dX compact: [K, Cin], no scatter, no zero rows */
#define SBP_FLAG_ACCUMULATE_DW  4u  /* dW += and db += instead of overwrite */
#define SBP_FLAG_DW_OUT_BF16    8u  /* sbp_backward_linear: dW is bf16 [Cout, Cin]: the fp32 sum rounded once */
#define SBP_FLAG_XK_KMAJOR     16u  /* sbp_backward_linear: X_k is in the row-group layout SBP_LAYOUT_KMAJOR (bf16 only) */

/* Layouts of a cached tensor X_k (the kept rows of a layer input, written by sbp_forward_cache_batch, read by the
 * linear backward for dW = dY_k^T X_k, whose contraction runs over the kept rows):
 *   SBP_LAYOUT_ROWS    [K, C] row-major: X_k[j][c] at element j * C + c
 *   SBP_LAYOUT_KMAJOR  [ceil(K / 8), C, 8]: X_k[j][c] at element ((j / 8) * C + c) * 8 + j % 8, i.e. the 8 rows of a
 *                      group side by side for every channel (one 16-byte piece per channel and group of rows), rows
 *                      K .. 8 ceil(K / 8) - 1 stored as +0.  8 ceil(K / 8) * C elements.  bf16 with C % 8 == 0 only.
 *                      The contraction index is then contiguous in memory, as the matrix cores want their operands:
 *                      the dW units read X_k from LDS with plain 16-byte reads instead of transposing reads. */
#define SBP_LAYOUT_ROWS   0
#define SBP_LAYOUT_KMAJOR 1

/*
 * One draw of a grid-wise keep-set (paper, "How to sample the gradient keep mask?": a
 * structured sample drawn afresh every step).  The paper gives no algorithm; the reading
 * implemented here: the H x W map of each sample is tiled into 2x2 cells and k of the 4
 * slots of every cell are kept (k = round(4 r)); partial cells on an odd edge with c valid
 * slots keep max(1, round(k c / 4)) of them.  cell = 3 or 4 tiles the map into 3x3 or 4x4 cells and keeps k of
 * the 9 or 16 slots (keep ratios k/9, k/16; edge cells with v valid slots keep max(1, round(k v / cell^2))).
 * The draw is a pure function of (seed, stream_id, sample, cell): a SplitMix64-based counter hash, no state.
 * Rows are numbered b*(P + H*W) + p for the P always-kept prefix rows of sample b (the
 * ViT class token) and b*(P + H*W) + P + y*W + x for grid position (y, x).
 */
typedef struct sbp_sample_desc {
  int32_t  B;          /* samples in the batch, >= 1 */
  int32_t  P;          /* always-kept prefix rows per sample, >= 0 */
  int32_t  H, W;       /* grid, >= 1 each */
  int32_t  cell;       /* cell edge: 2 (the default), 3 or 4 in the grid modes; 2 for SBP_RANDOM_MASK; SBP_TEMPORAL: frames per cell, 2..4 */
  int32_t  k;          /* kept slots per full cell, 1..cell^2 (SBP_TEMPORAL: kept frames per cell, 1..cell) */
  int32_t  mode;       /* SBP_GRID_PER_CELL, SBP_GRID_SHARED, SBP_RANDOM_MASK or SBP_TEMPORAL */
  int32_t  per_sample; /* 1: every sample draws its own mask; 0: one mask for the batch */
  uint64_t seed;       /* run seed */
  uint64_t stream_id;  /* caller's (step, layer) counter: a new value gives a new mask */
} sbp_sample_desc;

/* Host only.  Text for a status code; never NULL. */
const char* sbp_status_string(int32_t status);
/* Host only.  Thread-local description of the last failed call on this thread ("" if none). */
const char* sbp_last_error(void);

/* Host only.  Kept slots per cell for keep ratio r: round-half-up(r*cell*cell), clamped to
 * [1, cell*cell].  Returns SBP_ERR_RATIO if r is not in (0, 1], SBP_ERR_SHAPE if cell is not 2, 3 or 4. */
int32_t sbp_k_from_ratio(double r, int32_t cell);

/* Host only.  Number of kept rows K of a draw (closed form), or a negative SBP_ERR_* code.
 * The keep ratio of the paper is K / (B*(P+H*W)). */
int64_t sbp_keep_count(const sbp_sample_desc* desc);

/*
 * Step "sample keep-set".  Writes the kept row ids, int32, into idx[0..K) in canonical
 * order: sample-major; inside a sample the P prefix rows, then (grid modes) the cells in row-major cell
 * order, and inside a cell the kept slots in ascending slot number cell*(y%cell) + (x%cell); the other modes
 * write ascending row ids.
 *   idx          device, out, capacity idx_capacity elements (>= K else SBP_ERR_CAPACITY)
 *   inv          device, out, [B*(P+H*W)] or NULL: inv[row] = position of row in idx, -1 if dropped
 */
int32_t sbp_sample_indices(const sbp_sample_desc* desc, int32_t* idx, int64_t idx_capacity,
                           int32_t* inv, void* stream);

/*
 * Several draws in one call (a training step draws the keep-sets of all its blocks or layers at once): draw i is
 * sbp_sample_indices(&descs[i], idx[i], idx_capacity[i], inv ? inv[i] : NULL).  Draws of the 2 x 2 grid sampler
 * share launches (16 draws each); the other modes run one by one.  descs, idx, idx_capacity, inv are HOST arrays of n
 * entries (idx[i], inv[i] device pointers; inv or single inv[i] may be NULL); 1 <= n <= 4096.
 */
int32_t sbp_sample_indices_batch(const sbp_sample_desc* descs, int32_t n, int32_t* const* idx,
                                 const int64_t* idx_capacity, int32_t* const* inv, void* stream);

/*
 * Step "forward cache" (paper, section "Calculation of Linear Layers": of the layer input only the kept
 * rows are retained for the backward pass):
 * X_k[j, :] = X[idx[j], :] for j in [0, K).
 *   X      device, in,  [M, C] of `dtype`
 *   idx    device, in,  [K] row ids in [0, M), unique (caller's contract; any unique list is legal)
 *   X_k    device, out, [K, C] of `dtype`
 */
int32_t sbp_forward_cache(const void* X, const int32_t* idx, int64_t M, int64_t K, int32_t C,
                          int32_t dtype, void* X_k, void* stream);

/*
 * Step "forward cache" for several tensors in one call (the inputs of all linear layers of a block): item i is
 * sbp_forward_cache(X, idx, M, K, C, dtype, X_k).  Rows whose byte length is a multiple of 16 (16-byte aligned
 * tensors) are served by ONE launch; otherwise the items run one after the other.  1 <= n <= SBP_MAX_BATCH_LAYERS.
 * layout = SBP_LAYOUT_KMAJOR writes X_k in the row-group layout (bf16, C % 8 == 0, 16-byte aligned tensors; else
 * SBP_ERR_FLAGS); items of one call that share a layout share a launch.
 */
typedef struct sbp_gather_item {
  const void*    X;       /* [M, C] */
  const int32_t* idx;     /* [K] */
  void*          X_k;     /* [K, C] out ([ceil(K / 8), C, 8] with SBP_LAYOUT_KMAJOR) */
  int64_t        M, K;
  int32_t        C;
  int32_t        layout;  /* SBP_LAYOUT_ROWS (0) or SBP_LAYOUT_KMAJOR */
} sbp_gather_item;
int32_t sbp_forward_cache_batch(const sbp_gather_item* items, int32_t n, int32_t dtype, void* stream);

/* Host only.  Bytes of workspace sbp_backward_linear needs for these sizes (0 on invalid sizes). */
size_t sbp_backward_linear_workspace(int64_t M, int64_t K, int32_t Cin, int32_t Cout,
                                     int32_t dtype, uint32_t flags);

/*
 * Host only.  Which kernels sbp_backward_linear runs for these sizes (a report for logs and
 * benchmarks; the results do not depend on it): SBP_ENGINE_PLAIN (fp32, or channel counts that are
 * not multiples of 8), SBP_ENGINE_MFMA (128 x 128 tiles), SBP_ENGINE_MFMA_LARGE (256-wide tiles, one
 * workgroup per CU); -1 on invalid sizes.  If split_count is not NULL it receives the number of
 * fp32 partial sums of dW that the reduction adds.
 */
#define SBP_ENGINE_PLAIN 0
#define SBP_ENGINE_MFMA 1
#define SBP_ENGINE_MFMA_LARGE 2
int32_t sbp_backward_linear_engine(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype,
                                   uint32_t flags, int32_t* split_count);

/*
 * Steps "gather dY", "dW", "db", "dX" (paper, eq:backward_fc_sbp with every dropped term
 * removed):
 *   dW[o, i] = sum_j dY[idx[j], o] * X_k[j, i]           fp32, [Cout, Cin]
 *   db[o]    = sum_j dY[idx[j], o]                       fp32, [Cout]
 *   dX[idx[j], :] = dY[idx[j], :] * W ; every other row of dX is +0.0     `dtype`, [M, Cin]
 * Sums are accumulated in fp32; bf16 outputs are rounded once (round-to-nearest-even).
 * The result is deterministic (no floating-point atomics).
 *   dY     device, in,  [M, Cout] (only rows in idx are read) or [K, Cout] with SBP_FLAG_DY_COMPACT
 *   idx    device, in,  [K] unique row ids in [0, M)
 *   inv    device, in,  [M] inverse map of idx, or NULL: then it is built in the workspace by one more
 *                       small kernel.  Only used to zero-fill dX.  ONE contract for every call of this
 *                       library that takes an inverse map (this one, sbp_backward_dwconv,
 *                       sbp_backward_layernorm, sbp_scatter_patches): inv[idx[j]] = j for the kept rows
 *                       and -1 for every dropped row, i.e. what sbp_sample_indices writes.
 *   X_k    device, in,  [K, Cin] rows cached by sbp_forward_cache (may be NULL if dW is NULL); with
 *                       SBP_FLAG_XK_KMAJOR in the row-group layout written by sbp_forward_cache_batch (bf16, Cin % 8
 *                       == 0 and a 16-byte aligned X_k, else SBP_ERR_FLAGS): the large-tile engine reads it as it
 *                       is, every other engine first copies it back to rows in the workspace
 *   W      device, in,  [Cout, Cin]                       (may be NULL if dX is NULL)
 *   dW, db, dX   device, out; each may be NULL to skip that output.  dW is fp32, or bf16 with
 *                SBP_FLAG_DW_OUT_BF16 (the same fp32 sum, rounded to nearest even once; together with
 *                SBP_FLAG_ACCUMULATE_DW the old bf16 values are added in fp32 and the sum rounded again);
 *                db is fp32 either way
 *   workspace    device, 256-byte aligned, at least sbp_backward_linear_workspace(...) bytes;
 *                contents on entry are irrelevant, contents on exit are unspecified
 * Channel counts that are multiples of 8 take the MFMA path for SBP_BF16; any other shape
 * and SBP_F32 take a plain (slower) kernel -- never an error.
 */
int32_t sbp_backward_linear(const void* dY, const int32_t* idx, const int32_t* inv, const void* X_k,
                            const void* W,
                            int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype,
                            void* dW, float* db, void* dX,
                            void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Several linear layers in one call (paper, eq:backward_fc_sbp per layer; the benchmark configuration asks for
 * the "per-block backward of all four linears" of a transformer block).  Every layer is described as in
 * sbp_backward_linear (same argument meaning, flags and outputs); all layers share `dtype`.  The layers must be
 * independent: no layer's dY may be another's dX or alias any output of the call.  (A chain of dependent layers
 * can still hand the weight gradients of a block to one call with dX = NULL - they need only each layer's dY and
 * X_k - after running the dX of the critical path layer by layer; on the ViT-Base block that was measured slower
 * than one full sbp_backward_linear call per layer, whose launch overlaps a layer's dX tiles with its dW units.)
 * bf16 layers within the large-tile engine's limits (Cin % 8 == 0, Cout % 32 == 0, M * max(Cin, Cout) < 2^31,
 * K >= 1, 16-byte aligned tensors) that are at least 256 channels wide with K >= 1024 run as ONE grid whose
 * units - dX tiles, dW units (which also sum db), zero-fill blocks of all layers - are laid out in one queue
 * per XCD, longest first, plus one reduction launch for all split sums; a batch with any other layer runs
 * layer by layer, exactly as n calls of sbp_backward_linear would.  A layer whose dW
 * needs a single split (up to 7936 kept rows) writes dW directly (no partial sums; the reduction launch then
 * adds only the db partials, one per tile column of dW).  Results per layer equal those of
 * sbp_backward_linear up to the summation order of dW / db (bit-identical on exactly representable inputs).
 *   layers     host array of n descriptors, 1 <= n <= SBP_MAX_BATCH_LAYERS; read during the call only
 *   workspace  device, 256-byte aligned, sbp_backward_linear_batch_workspace(layers, n, dtype) bytes (the
 *              query looks at sizes, flags and at which of inv / dW / db / dX are NULL, not at the addresses)
 */
typedef struct sbp_linear_layer {
  const void*    dY;      /* [M, Cout], or [K, Cout] with SBP_FLAG_DY_COMPACT */
  const int32_t* idx;     /* [K] */
  const int32_t* inv;     /* [M] or NULL */
  const void*    X_k;     /* [K, Cin] */
  const void*    W;       /* [Cout, Cin] */
  int64_t        M, K;
  int32_t        Cin, Cout;
  void*          dW;      /* [Cout, Cin] fp32 (bf16 with SBP_FLAG_DW_OUT_BF16) or NULL */
  float*         db;      /* [Cout] or NULL */
  void*          dX;      /* [M, Cin] ([K, Cin] with SBP_FLAG_DX_COMPACT) or NULL */
  uint32_t       flags;   /* SBP_FLAG_* as for sbp_backward_linear */
  uint32_t       reserved;/* 0 */
} sbp_linear_layer;
size_t sbp_backward_linear_batch_workspace(const sbp_linear_layer* layers, int32_t n, int32_t dtype);
int32_t sbp_backward_linear_batch(const sbp_linear_layer* layers, int32_t n, int32_t dtype,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * sbp_backward_linear for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as sbp_backward_linear without `workspace` / `workspace_bytes`: the partial sums of the dW splits, the
 * db slices and the inverse row map live in a fixed array of SBP_STATIC_SCRATCH_BYTES in device memory that
 * belongs to the library (one per GPU, held from the library's first use on that GPU until the process ends;
 * its address is looked up once per device, on the first call with that device current).  The call allocates
 * and frees nothing.  Sizes that need more scratch than that (sbp_backward_linear_workspace(...) >
 * SBP_STATIC_SCRATCH_BYTES) are refused with SBP_ERR_CAPACITY before anything is enqueued; every layer of the
 * ViT / ConvNeXt workloads this library is measured on fits.  All calls on one GPU share the array: two calls
 * that may overlap in time on that GPU (different streams, or graph branches) race; calls on one stream are
 * ordered and safe.  Nothing in the array has to be cleared between calls (every element read was written by
 * the same call first).  sbp_static_scratch_bytes() returns SBP_STATIC_SCRATCH_BYTES (host only).
 */
#define SBP_STATIC_SCRATCH_BYTES (48u << 20)
size_t sbp_static_scratch_bytes(void);
int32_t sbp_backward_linear_static(const void* dY, const int32_t* idx, const int32_t* inv, const void* X_k,
                                   const void* W,
                                   int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype,
                                   void* dW, float* db, void* dX, uint32_t flags, void* stream);

/* Host only.  Bytes of workspace sbp_backward_dwconv needs (0 on invalid sizes). */
size_t sbp_backward_dwconv_workspace(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks,
                                     int64_t K, int32_t dtype, uint32_t flags);

/*
 * Step "depthwise conv backward on kept outputs" (paper, eq:conv_grad_layer_before_sbp with
 * dY set to zero at dropped positions; exact because the gradient arriving from an SBP
 * pointwise layer is zero there, eq:conv_grad_layer_before_sbp_chain).  Depthwise, stride 1,
 * zero padding `pad`, forward Y[b,y,x,c] = sum_{u,v} X[b,y+u-pad,x+v-pad,c] * Wd[u,v,c]:
 *   dWd[u,v,c] = sum_{(b,y,x) kept} dY[b,y,x,c] * X[b,y+u-pad,x+v-pad,c]      fp32, [ks,ks,C]
 *   db[c]      = sum_{(b,y,x) kept} dY[b,y,x,c]                               fp32, [C]
 *   dX[b,y,x,c]= sum_{u,v} [ (b,y-u+pad,x-v+pad) kept ] dY[..] * Wd[u,v,c]    `dtype`, dense
 *   dY   device, in, [B,H,W,C]; only kept positions are read
 *   idx  device, in, [K] kept flat positions b*H*W + y*W + x, unique
 *   inv  device, in, [B*H*W] inverse map of idx (position in idx, -1 = dropped: the contract stated at
 *        sbp_backward_linear) or NULL (then built in the workspace)
 *   X    device, in, [B,H,W,C] FULL input of the layer (a k>1 conv needs the neighbours); required
 *        whenever dWd or db is requested (SBP_ERR_NULL otherwise)
 *   Wd   device, in, [ks,ks,C]
 *   dWd, db, dX  device, out; each may be NULL
 * ks must be odd and <= 7, pad = ks/2.
 */
int32_t sbp_backward_dwconv(const void* dY, const int32_t* idx, const int32_t* inv,
                            const void* X, const void* Wd,
                            int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int32_t pad,
                            int64_t K, int32_t dtype,
                            float* dWd, float* db, void* dX,
                            void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Down-sampling layers: a convolution with kernel p x p and stride p (paper, section "Calculation of
 * Convolutional Layers": for a stride not smaller than the kernel the neighbour effects vanish and the
 * layer behaves like a point-wise one; ConvNeXt applies SBP to its 2 x 2, stride 2 down-sampling
 * layers).  idx holds kept OUTPUT positions b*Ho*Wo + yo*Wo + xo (Ho = H / p, Wo = W / p; a sampler
 * draw on the Ho x Wo grid).  The layer then is sbp_backward_linear on patch rows:
 *   sbp_forward_cache_patches   X_k[j, (dy*p + dx)*C + c] = X[b, p*yo + dy, p*xo + dx, c]   [K, p*p*C]
 *   sbp_backward_linear         with M = B*Ho*Wo, Cin = p*p*C, W viewed as [Cout, p*p*C] (= [Cout, p, p, C]),
 *                               SBP_FLAG_DX_COMPACT: dW, db and the compact gradient rows dXp_k [K, p*p*C]
 *   sbp_scatter_patches         dX[b, y, x, :] = the piece of dXp_k that belongs to input pixel (y, x) if its
 *                               output position is kept, +0.0 otherwise                          [B, H, W, C]
 *   X, dX   device, [B, H, W, C] of `dtype`, H and W multiples of p, 1 <= p <= 8
 *   inv     device, in, [B*Ho*Wo] inverse of idx (as written by sbp_sample_indices) or NULL: then it is built
 *           in the workspace (sbp_scatter_patches_workspace bytes, 256-byte aligned; may be NULL if inv is given)
 */
int32_t sbp_forward_cache_patches(const void* X, const int32_t* idx, int32_t B, int32_t H, int32_t W,
                                  int32_t C, int32_t p, int64_t K, int32_t dtype, void* X_k, void* stream);
size_t sbp_scatter_patches_workspace(int32_t B, int32_t H, int32_t W, int32_t p);
int32_t sbp_scatter_patches(const void* dXp_k, const int32_t* idx, const int32_t* inv, int32_t B, int32_t H,
                            int32_t W, int32_t C, int32_t p, int64_t K, int32_t dtype, void* dX,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * Row-wise steps between the linear layers, on compact rows (paper, Alg. alg:sbp_impl: "an arbitrary
 * operation f" sees the kept rows with gradient and the dropped rows without; with one keep-set shared
 * by a stack of layers the kept / dropped split passes through the chain unchanged,
 * eq:backward_fc2_sbp_same_drop_loc).  With SBP_FLAG_DX_COMPACT / SBP_FLAG_DY_COMPACT on the linear
 * layers around them, a whole MLP branch runs its backward on [K, .] rows and only its last step
 * scatters to [M, .] and zero-fills.
 *
 * Activation, act = SBP_ACT_GELU (exact GELU, z * Phi(z), the ViT / ConvNeXt MLP activation):
 *   sbp_act_forward_rows    H_k  = gelu(Z_k)                  recomputes the second layer's input from the
 *                                                             cached kept rows of the pre-activation
 *   sbp_act_backward_rows   dZ_k = dH_k * gelu'(Z_k),  gelu'(z) = Phi(z) + z phi(z)
 *   Z_k, dH_k  device, in,  [K, C] of `dtype`;   H_k, dZ_k  device, out, [K, C] of `dtype`
 *   (dZ_k may be the same buffer as dH_k: every element is read before it is written).
 * fp32 arithmetic; bf16 outputs are rounded once (round-to-nearest-even).
 */
#define SBP_ACT_GELU 0
int32_t sbp_act_forward_rows(const void* Z_k, int64_t K, int32_t C, int32_t dtype, int32_t act,
                             void* H_k, void* stream);
int32_t sbp_act_backward_rows(const void* dH_k, const void* Z_k, int64_t K, int32_t C, int32_t dtype,
                              int32_t act, void* dZ_k, void* stream);

/*
 * Backward of the per-channel layer scale U = gamma * Y (the last step of a ConvNeXt block's branch) on the kept
 * rows (paper, Alg. alg:sbp_impl with f = the scale; kept rows through f with gradient, dropped rows without):
 *   dY_k = dU_k * gamma,     dgamma[c] = sum over the kept rows j of dU_k[j, c] * Y_k[j, c]
 *   dU_k, Y_k  device, in,  [K, C] of `dtype` (compact: gather the kept rows of the block output's gradient with
 *              sbp_forward_cache; Y_k is the cached kept rows of the scale's input)
 *   gamma      device, in,  fp32 [C];   dgamma  device, out, fp32 [C] or NULL;   dY_k  device, out, [K, C] or NULL
 *              (dY_k may be dU_k: every element is read before it is written)
 *   workspace  sbp_backward_layerscale_workspace(K, C) bytes, 256-byte aligned (partial sums of dgamma)
 *   flags      SBP_FLAG_ACCUMULATE_DW: dgamma += instead of overwrite; nothing else
 * fp32 arithmetic, dgamma summed in a fixed order (deterministic); bf16 outputs rounded once.
 */
size_t sbp_backward_layerscale_workspace(int64_t K, int32_t C);
int32_t sbp_backward_layerscale(const void* dU_k, const void* Y_k, const float* gamma, int64_t K, int32_t C,
                                int32_t dtype, float* dgamma, void* dY_k, void* workspace, size_t workspace_bytes,
                                uint32_t flags, void* stream);

/*
 * Backward of scaled dot-product attention on the kept tokens: the variant "Drop QKV" that the paper picks
 * for image transformers (main text, section Design Strategies, "How to apply SBP on MHSA?"; supplement,
 * section Gradient Calculation of Attention Layers: eq:attention, eq:grad_qkv, and the gradient dropout on
 * the attention map M of eq:sbp_sep_on_query / eq:sbp_sep_on_key, carried over to dropped keys and values).
 * The forward is the ordinary attention over all n tokens of a sample; in the backward every entry of dM
 * whose query or key token is dropped is zero, the kept entries are exact, and dQ, dK, dV are produced at
 * the kept tokens only.  Per sample b and head a, with i, j running over the n_k kept tokens:
 *   S_ij  = exp(scale * q_i.k_j - lse_i)
 *   dV_j  = sum_i S_ij dA_i
 *   dM_ij = S_ij * (dA_i.v_j - dA_i.A_i)      (the softmax row term sum_l S_il dS_il over ALL keys l equals
 *                                              dA_i.A_i because A_i = sum_l S_il v_l)
 *   dQ_i  = scale * sum_j dM_ij k_j           dK_j = scale * sum_i dM_ij q_i
 * (of the two forms of dQ the supplement prints, the shape-consistent one).  Every sample keeps the same
 * number n_k of tokens (the samplers of this library do); all tensors hold kept tokens only, sample-major:
 * row b * n_k + t is the t-th kept token of sample b, i.e. the rows sbp_forward_cache gathers.
 *   qkv_k   device, in,  [B*n_k, 3*h*d] of `dtype`: kept rows of the qkv projection's output, q | k | v thirds,
 *           each third head-major [h, d]
 *   A_k     device, in,  [B*n_k, h*d]  kept rows of the attention output (the proj layer's cached input)
 *   dA_k    device, in,  [B*n_k, h*d]  gradient of the attention output at the kept rows (the proj layer's
 *           backward with SBP_FLAG_DX_COMPACT writes exactly this)
 *   lse_k   device, in,  [B*n_k, h] fp32: natural-log sum over ALL n keys of exp(scale * q_i.k_l), kept queries
 *   dqkv_k  device, out, [B*n_k, 3*h*d] of `dtype`: dQ | dK | dV in the layout of qkv_k; it is the compact
 *           dY (SBP_FLAG_DY_COMPACT) of the qkv projection's backward
 *   d       head dimension: 16, 32, 64 or 128.   scale: usually 1/sqrt(d).
 * All pointers 16-byte aligned.  fp32 arithmetic and accumulation; in bf16 the probabilities S and dM are
 * rounded to bf16 before the second products (matrix cores), outputs rounded once.  Deterministic.
 * sbp_backward_attention_engine (host only) reports which kernel serves a size: 1 = matrix-core kernel with one
 * workgroup per (sample, head) (bf16, d in {32, 64, 128}, the kept tokens of one head fit LDS: n_k <= 256 at
 * d = 64), 2 = matrix-core kernel tiled over chunks of 128 tokens (bf16, d in {32, 64, 128}, any n_k),
 * 0 = plain kernel (fp32, d = 16).
 */
int32_t sbp_backward_attention_engine(int32_t n_k, int32_t d, int32_t dtype);
int32_t sbp_backward_attention(const void* qkv_k, const void* A_k, const void* dA_k, const float* lse_k,
                               int32_t B, int32_t n_k, int32_t h, int32_t d, float scale, int32_t dtype,
                               void* dqkv_k, void* stream);

/* Host only.  Bytes of workspace sbp_backward_layernorm needs (0 on invalid sizes). */
size_t sbp_backward_layernorm_workspace(int64_t M, int64_t K, int32_t C, int32_t dtype, uint32_t flags);

/*
 * Backward of U = LayerNorm(X) * gamma + beta (normalisation over the C channels of a row, biased
 * variance, `eps` inside the square root) restricted to the kept rows:
 *   per kept row j:  xhat = (x - mean(x)) / sqrt(var(x) + eps),  g = dU_k[j] * gamma,
 *                    dX[idx[j], :] = (g - mean(g) - xhat * mean(g * xhat)) / sqrt(var(x) + eps)
 *   every other row of dX is +0.0;   dgamma = sum_j dU_k[j] * xhat_j,   dbeta = sum_j dU_k[j]
 *   dU_k   device, in,  [K, C] of `dtype` (compact: the output of the linear backward with
 *                       SBP_FLAG_DX_COMPACT)
 *   X_k    device, in,  [K, C] kept rows of the LayerNorm input (sbp_forward_cache); mean and variance
 *                       are recomputed from them in fp32
 *   gamma  device, in,  [C] fp32
 *   idx, inv            as for sbp_backward_linear (inv may be NULL; unused with SBP_FLAG_DX_COMPACT)
 *   dgamma, dbeta  device, out, [C] fp32 (added to with SBP_FLAG_ACCUMULATE_DW); dX device, out,
 *                       [M, C] of `dtype`, or [K, C] with SBP_FLAG_DX_COMPACT; each may be NULL
 *   workspace           device, 256-byte aligned, sbp_backward_layernorm_workspace(...) bytes
 * Deterministic (fixed summation order, no floating-point atomics).
 */
int32_t sbp_backward_layernorm(const void* dU_k, const void* X_k, const float* gamma, float eps,
                               const int32_t* idx, const int32_t* inv, int64_t M, int64_t K, int32_t C,
                               int32_t dtype, float* dgamma, float* dbeta, void* dX,
                               void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * Explicit overrides for tests and parameter sweeps (not a step of the method).  The library reads no
 * environment variable; by default every choice below is automatic.  name = NULL restores all defaults;
 * value = NULL clears one override.  Process-wide, thread-safe (calls in flight use the snapshot they took);
 * results never depend on these beyond the summation order of dW / db.  Returns SBP_ERR_FLAGS for an unknown
 * name or a value that is not valid for it (nothing changes then).
 *   "tile"      "big" (large-tile engine wherever its limits allow) | "128x128x4x64" | "128x128x4x32" |
 *               "256x256x8x64" | "256x256x8x32" | "256x256x4x64" | "256x256x4x32" (general engine: rows x
 *               columns x wavefronts x stage length)
 *   "dxbm"      64 | 128 | 256: rows of a dX tile of the large-tile engine;  "dxrows"  64 | 128: general engine
 *   "splits"    number of equal dW splits of the large-tile engine
 *   "plan", "plan_<Cin>x<Cout>"   "bm,rows_long,n_long,rows_short": a whole schedule of the large-tile engine
 *               for every shape / one shape (ignored where it does not fit the kept-row count)
 *   "order"     "a,b,c", a permutation of 0,1,2: dispatch order of the kinds of workgroups
 *   "dw_rows"   rows per strip of the depthwise kernels;  "dw_separate"  "1": dX and dWd as two launches
 *   "attn"      "plain": attention backward without the matrix cores | "whole": one workgroup per (sample, head)
 *               where its tokens fit LDS | "tiled": chunks of 128 tokens per workgroup, at any size
 *   "sampler_no_window", "sampler_no_masks", "patch_wide", "debug_plan"   "1" | "0"
 *   "batch_spread"  "1": batched linear call deals its units to the XCDs in turn (no neighbour affinity)
 *   "batch_dynamic" "1": batched linear call fetches units through one counter per XCD instead of static queues
 *   "dw_strips"     "1": depthwise backward with the register-strip kernels instead of the LDS-tiled one
 */
int32_t sbp_set_option(const char* name, const char* value);

/*
 * Measurement aid (not a step of the method; for benchmarks only).  While enabled, every kernel
 * launch of the library is bracketed by a pair of HIP events on the caller's stream; this is the
 * one place where the library creates HIP objects (the events, destroyed again by the read call).
 * sbp_profile_read waits for the recorded events, adds the elapsed times of the kernels of class
 * `which` to *total_ms and their number to *launches (host pointers), and forgets all records when
 * which == SBP_PROF_RESET.  Not thread-safe; do not enable under graph capture.
 */
#define SBP_PROF_SAMPLE      0
#define SBP_PROF_GATHER      1
#define SBP_PROF_DW_GEMM     2   /* dW contraction (MFMA) */
#define SBP_PROF_DX_GEMM     3   /* dX contraction (MFMA) */
#define SBP_PROF_REDUCE      4   /* split reduction of dW / db */
#define SBP_PROF_COLSUM      5   /* db column sums */
#define SBP_PROF_ZERO_ROWS   6   /* marking kept rows + zero-filling dropped rows of dX */
#define SBP_PROF_DWCONV_DX   7
#define SBP_PROF_DWCONV_DW   8
#define SBP_PROF_OTHER       9
#define SBP_PROF_ATTENTION  10   /* attention backward on the kept tokens */
#define SBP_PROF_NCLASSES   11
#define SBP_PROF_RESET     (-1)
int32_t sbp_profile_enable(int32_t on);
/*
 * Measurement aid: per-workgroup time stamps of the batched linear backward.  While `records` (device memory,
 * 8 x uint64 per unit of work, capacity_records units; NULL switches it off) is set, every unit of
 * sbp_backward_linear_batch's common grid with a number below the capacity writes
 *   [0] start and [1] end on the 100 MHz constant clock, [2] start and [3] end on the shader clock,
 *   [4] kind | layer << 8 | unit << 16   (kind 0 dX tile, 1 dW unit, 3 zero-fill block, 4 column-sum block)
 *   [5] queue (XCD) the unit was planned on | XCD that ran it << 8 | workgroup << 16
 * The caller owns the buffer and zeroes it.  Not thread-safe.
 */
int32_t sbp_profile_timeline(void* records, int64_t capacity_records);
int32_t sbp_profile_read(int32_t which, double* total_ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* SBP_H_ */
