// C ABI of libsbp: host-side validation, then kernel launches.  Every argument check runs
// before the first HIP call so that error paths need no device.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cmath>
#include <mutex>
#include <vector>

#include <string>

#include "sbp_internal.h"

namespace sbp {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int32_t check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SBP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return SBP_OK;
}

// ---- explicit overrides -------------------------------------------------------------------------
static std::mutex g_opt_mutex;
static Options g_opt;
Options options() {
  std::lock_guard<std::mutex> lock(g_opt_mutex);
  return g_opt;
}

static bool parse_flag(const char* v, bool* out) {
  if (!v || !std::strcmp(v, "0") || !std::strcmp(v, "")) { *out = false; return true; }
  if (!std::strcmp(v, "1")) { *out = true; return true; }
  return false;
}

// Applies one override to `o`; false if the name is unknown or the value is not valid for it.
static bool apply_option(Options& o, const char* name, const char* v) {
  const std::string n(name);
  if (n == "tile") {
    if (!v) { o.tile_mode = 0; return true; }
    if (!std::strcmp(v, "big")) { o.tile_mode = 2; return true; }
    int a = 0, b = 0, w = 4, k = 64;
    if (std::sscanf(v, "%dx%dx%dx%d", &a, &b, &w, &k) < 2) return false;
    const bool ok = ((a == 256 && b == 256 && (w == 8 || w == 4)) || (a == 128 && b == 128 && w == 4)) && (k == 32 || k == 64);
    if (!ok) return false;
    o.tile_mode = 1; o.tile_bm = a; o.tile_bn = b; o.tile_nw = w; o.tile_kb = k;
    return true;
  }
  if (n == "dxbm" || n == "dxrows" || n == "splits" || n == "dw_rows") {
    int x = v ? std::atoi(v) : 0;
    if (v && x <= 0) return false;
    if (n == "dxbm") { if (x && x != 64 && x != 128 && x != 256) return false; o.dxbm = x; }
    else if (n == "dxrows") { if (x && x != 64 && x != 128) return false; o.dxrows = x; }
    else if (n == "splits") { if (x > 4096) return false; o.splits = x; }
    else { if (x > 4096) return false; o.dw_rows = x; }
    return true;
  }
  if (n == "order") {
    if (!v) { o.order_set = false; return true; }
    int q[3];
    if (std::sscanf(v, "%d,%d,%d", &q[0], &q[1], &q[2]) != 3) return false;
    for (int i = 0; i < 3; ++i) if ((unsigned)q[i] > 2u) return false;
    if ((1 << q[0] | 1 << q[1] | 1 << q[2]) != 7) return false;          // a permutation of 0, 1, 2
    o.order_set = true;
    for (int i = 0; i < 3; ++i) o.order[i] = q[i];
    return true;
  }
  if (n.rfind("plan", 0) == 0) {                                        // "plan" or "plan_<Cin>x<Cout>"
    int cin = 0, cout = 0;
    if (n != "plan" && (std::sscanf(name, "plan_%dx%d", &cin, &cout) != 2 || cin < 1 || cout < 1)) return false;
    int slot = -1;
    for (int i = 0; i < o.nplans; ++i) if (o.plans[i].cin == cin && o.plans[i].cout == cout) slot = i;
    if (!v) {
      if (slot >= 0) o.plans[slot] = o.plans[--o.nplans];
      return true;
    }
    int bm = 0, A = 0, nb = 0, a = 0;
    if (std::sscanf(v, "%d,%d,%d,%d", &bm, &A, &nb, &a) != 4) return false;
    if ((bm != 64 && bm != 128 && bm != 256) || A < 64 || A % 64 || nb < 1 || a < 0 || a % 64 || a > A) return false;
    if (slot < 0) { if (o.nplans == 8) return false; slot = o.nplans++; }
    o.plans[slot] = ShapePlan{cin, cout, bm, A, nb, a};
    return true;
  }
  if (n == "attn") {
    if (!v) { o.attn_mode = 0; return true; }
    const int m = !std::strcmp(v, "plain") ? 1 : !std::strcmp(v, "whole") ? 2 : !std::strcmp(v, "tiled") ? 3 : -1;
    if (m < 0) return false;
    o.attn_mode = m;
    return true;
  }
  bool* flag = n == "debug_plan" ? &o.debug_plan : n == "dw_separate" ? &o.dw_separate
             : n == "sampler_no_window" ? &o.sampler_no_window : n == "sampler_no_masks" ? &o.sampler_no_masks
             : n == "patch_wide" ? &o.patch_wide : n == "batch_dynamic" ? &o.batch_dynamic
             : n == "batch_spread" ? &o.batch_spread : n == "dw_strips" ? &o.dw_strips
             : nullptr;
  if (!flag) return false;
  return parse_flag(v, flag);
}

// ---- measurement aid --------------------------------------------------------------------------
struct ProfRec { int cls; hipEvent_t a, b; };
static bool g_prof_on = false;
static std::vector<ProfRec>* g_prof = nullptr;

ProfScope::ProfScope(int cls, hipStream_t s) : cls_(cls), s_(s), rec_(nullptr) {
  if (!g_prof_on) return;
  if (!g_prof) g_prof = new std::vector<ProfRec>();
  ProfRec r{cls, nullptr, nullptr};
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, s);
  g_prof->push_back(r);
  rec_ = reinterpret_cast<void*>(g_prof->size());   // index + 1
}
ProfScope::~ProfScope() {
  if (!rec_) return;
  (void)hipEventRecord((*g_prof)[reinterpret_cast<size_t>(rec_) - 1].b, s_);
}

static unsigned long long* g_timeline = nullptr;
static int g_timeline_cap = 0;
void timeline_target(unsigned long long** buf, int* capacity_records) {
  *buf = g_timeline;
  *capacity_records = g_timeline_cap;
}

static int32_t validate_desc(const sbp_sample_desc* d) {
  if (!d) return fail(SBP_ERR_NULL, "sample descriptor is NULL");
  if (d->B < 1 || d->P < 0 || d->H < 1 || d->W < 1)
    return fail(SBP_ERR_SHAPE, "bad geometry B=%d P=%d H=%d W=%d", d->B, d->P, d->H, d->W);
  if (d->mode == SBP_TEMPORAL) {
    if (d->cell < 2 || d->cell > 4) return fail(SBP_ERR_SHAPE, "temporal cell must be 2..4 frames, got %d", d->cell);
    if (d->k < 1 || d->k > d->cell) return fail(SBP_ERR_RATIO, "k must be in 1..cell, got %d", d->k);
  } else if (d->mode == SBP_RANDOM_MASK) {
    if (d->cell != 2) return fail(SBP_ERR_SHAPE, "cell must be 2, got %d", d->cell);
    if (d->k < 1 || d->k > 4) return fail(SBP_ERR_RATIO, "k must be in 1..4, got %d", d->k);
  } else {
    if (d->cell < 2 || d->cell > 4) return fail(SBP_ERR_SHAPE, "cell must be 2, 3 or 4, got %d", d->cell);
    if (d->k < 1 || d->k > d->cell * d->cell) return fail(SBP_ERR_RATIO, "k must be in 1..cell^2, got %d", d->k);
  }
  if (d->mode != SBP_GRID_PER_CELL && d->mode != SBP_GRID_SHARED && d->mode != SBP_RANDOM_MASK && d->mode != SBP_TEMPORAL)
    return fail(SBP_ERR_FLAGS, "unknown sampler mode %d", d->mode);
  if (d->per_sample != 0 && d->per_sample != 1)
    return fail(SBP_ERR_FLAGS, "per_sample must be 0 or 1, got %d", d->per_sample);
  int64_t rows = (int64_t)d->B * ((int64_t)d->P + (int64_t)d->H * d->W);
  if (rows > INT32_MAX) return fail(SBP_ERR_SHAPE, "B*(P+H*W)=%lld exceeds int32 row ids", (long long)rows);
  return SBP_OK;
}

static int elem_bytes(int32_t dtype) { return dtype == SBP_F32 ? 4 : dtype == SBP_BF16 ? 2 : 0; }

}  // namespace sbp

using namespace sbp;

extern "C" {

const char* sbp_status_string(int32_t st) {
  switch (st) {
    case SBP_OK: return "ok";
    case SBP_ERR_NULL: return "null pointer";
    case SBP_ERR_SHAPE: return "bad shape";
    case SBP_ERR_RATIO: return "bad keep ratio";
    case SBP_ERR_DTYPE: return "bad dtype";
    case SBP_ERR_CAPACITY: return "output capacity too small";
    case SBP_ERR_WORKSPACE: return "bad workspace";
    case SBP_ERR_HIP: return "HIP error";
    case SBP_ERR_FLAGS: return "bad flags";
    default: return "unknown status";
  }
}

const char* sbp_last_error(void) { return g_err; }

int32_t sbp_k_from_ratio(double r, int32_t cell) {
  if (cell < 2 || cell > 4) return fail(SBP_ERR_SHAPE, "cell must be 2, 3 or 4, got %d", cell);
  if (!(r > 0.0 && r <= 1.0)) return fail(SBP_ERR_RATIO, "keep ratio %g not in (0,1]", r);
  int32_t n = cell * cell;
  int32_t k = (int32_t)std::floor(r * n + 0.5);
  return k < 1 ? 1 : (k > n ? n : k);
}

int64_t sbp_keep_count(const sbp_sample_desc* d) {
  int32_t st = validate_desc(d);
  if (st != SBP_OK) return st;
  return keep_count_host(*d);
}

int32_t sbp_sample_indices(const sbp_sample_desc* d, int32_t* idx, int64_t idx_capacity, int32_t* inv,
                           void* stream) {
  int32_t st = validate_desc(d);
  if (st != SBP_OK) return st;
  if (!idx) return fail(SBP_ERR_NULL, "idx is NULL");
  int64_t K = keep_count_host(*d);
  if (idx_capacity < K)
    return fail(SBP_ERR_CAPACITY, "idx capacity %lld < K=%lld", (long long)idx_capacity, (long long)K);
  return launch_sample(*d, idx, inv, (hipStream_t)stream);
}

int32_t sbp_sample_indices_batch(const sbp_sample_desc* descs, int32_t n, int32_t* const* idx, const int64_t* idx_capacity,
                                 int32_t* const* inv, void* stream) {
  if (!descs || !idx || !idx_capacity) return fail(SBP_ERR_NULL, "descs, idx or idx_capacity is NULL");
  if (n < 1 || n > 4096) return fail(SBP_ERR_SHAPE, "need 1 <= n <= 4096 draws, got %d", n);
  for (int i = 0; i < n; ++i) {
    int32_t st = validate_desc(&descs[i]);
    if (st != SBP_OK) return st;
    if (!idx[i]) return fail(SBP_ERR_NULL, "idx[%d] is NULL", i);
    const int64_t K = keep_count_host(descs[i]);
    if (idx_capacity[i] < K)
      return fail(SBP_ERR_CAPACITY, "idx[%d] capacity %lld < K=%lld", i, (long long)idx_capacity[i], (long long)K);
  }
  return launch_sample_batch(descs, n, idx, inv, (hipStream_t)stream);
}

int32_t sbp_forward_cache(const void* X, const int32_t* idx, int64_t M, int64_t K, int32_t C, int32_t dtype,
                          void* Xk, void* stream) {
  int eb = elem_bytes(dtype);
  if (!eb) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (M < 1 || M > INT32_MAX || C < 1) return fail(SBP_ERR_SHAPE, "bad shape M=%lld C=%d", (long long)M, C);
  if (K < 0 || K > M) return fail(SBP_ERR_SHAPE, "need 0 <= K <= M, got K=%lld M=%lld", (long long)K, (long long)M);
  if (K == 0) return SBP_OK;   // nothing to gather (empty tensors may have NULL storage)
  if (!X || !idx || !Xk) return fail(SBP_ERR_NULL, "X, idx and X_k must be non-NULL");
  return launch_gather_rows(X, idx, K, C, eb, Xk, (hipStream_t)stream);
}

static int32_t validate_linear(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, uint32_t flags) {
  if (!elem_bytes(dtype)) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (flags & ~(SBP_FLAG_DY_COMPACT | SBP_FLAG_DX_COMPACT | SBP_FLAG_ACCUMULATE_DW | SBP_FLAG_DW_OUT_BF16 | SBP_FLAG_XK_KMAJOR))
    return fail(SBP_ERR_FLAGS, "unknown flags 0x%x", flags);
  if ((flags & SBP_FLAG_XK_KMAJOR) && (dtype != SBP_BF16 || Cin % 8 != 0))
    return fail(SBP_ERR_FLAGS, "SBP_FLAG_XK_KMAJOR needs bf16 and Cin %% 8 == 0 (dtype %d, Cin %d)", dtype, Cin);
  if (M < 1 || M > INT32_MAX || Cin < 1 || Cout < 1)
    return fail(SBP_ERR_SHAPE, "bad shape M=%lld Cin=%d Cout=%d", (long long)M, Cin, Cout);
  if (K < 0 || K > M) return fail(SBP_ERR_SHAPE, "need 0 <= K <= M, got K=%lld M=%lld", (long long)K, (long long)M);
  if ((int64_t)Cin * Cout > INT32_MAX) return fail(SBP_ERR_SHAPE, "Cin*Cout too large");
  return SBP_OK;
}

int32_t sbp_forward_cache_batch(const sbp_gather_item* items, int32_t n, int32_t dtype, void* stream) {
  int eb = elem_bytes(dtype);
  if (!eb) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (!items) return fail(SBP_ERR_NULL, "items is NULL");
  if (n < 1 || n > SBP_MAX_BATCH_LAYERS) return fail(SBP_ERR_SHAPE, "need 1 <= n <= %d items, got %d", SBP_MAX_BATCH_LAYERS, n);
  for (int i = 0; i < n; ++i) {
    const sbp_gather_item& g = items[i];
    if (g.layout != SBP_LAYOUT_ROWS && g.layout != SBP_LAYOUT_KMAJOR) return fail(SBP_ERR_FLAGS, "item %d: unknown layout %d", i, g.layout);
    if (g.layout == SBP_LAYOUT_KMAJOR && (dtype != SBP_BF16 || g.C % 8 != 0 || (uintptr_t)g.X % 16 || (uintptr_t)g.X_k % 16))
      return fail(SBP_ERR_FLAGS, "item %d: SBP_LAYOUT_KMAJOR needs bf16, C %% 8 == 0 and 16-byte aligned tensors", i);
    if (g.M < 1 || g.M > INT32_MAX || g.C < 1) return fail(SBP_ERR_SHAPE, "item %d: bad shape M=%lld C=%d", i, (long long)g.M, g.C);
    if (g.K < 0 || g.K > g.M) return fail(SBP_ERR_SHAPE, "item %d: need 0 <= K <= M, got K=%lld M=%lld", i, (long long)g.K, (long long)g.M);
    if (g.K > 0 && (!g.X || !g.idx || !g.X_k)) return fail(SBP_ERR_NULL, "item %d: X, idx and X_k must be non-NULL", i);
  }
  return launch_gather_rows_batch(items, n, eb, (hipStream_t)stream);
}

}  // extern "C"

namespace sbp {
// Host-side argument checks shared by the entry points of the linear backward (sizes, flags, required pointers).
int32_t check_linear_args(const void* dY, const int32_t* idx, const void* Xk, const void* W, int64_t M, int64_t K,
                          int32_t Cin, int32_t Cout, int32_t dtype, const void* dW, const void* dX, uint32_t flags) {
  int32_t st = validate_linear(M, K, Cin, Cout, dtype, flags);
  if (st != SBP_OK) return st;
  if (!dY) return fail(SBP_ERR_NULL, "dY is NULL");
  bool need_idx = !((flags & SBP_FLAG_DY_COMPACT) && ((flags & SBP_FLAG_DX_COMPACT) || !dX));
  if (need_idx && !idx && K > 0) return fail(SBP_ERR_NULL, "idx is NULL");
  if (dW && !Xk && K > 0) return fail(SBP_ERR_NULL, "X_k is NULL but dW is requested");
  if (dX && !W) return fail(SBP_ERR_NULL, "W is NULL but dX is requested");
  if ((flags & SBP_FLAG_XK_KMAJOR) && ((uintptr_t)Xk % 16)) return fail(SBP_ERR_FLAGS, "SBP_FLAG_XK_KMAJOR needs a 16-byte aligned X_k");
  return SBP_OK;
}
}  // namespace sbp

extern "C" {

size_t sbp_backward_linear_workspace(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype,
                                     uint32_t flags) {
  if (validate_linear(M, K, Cin, Cout, dtype, flags) != SBP_OK) return 0;
  return plan_linear(M, K, Cin, Cout, dtype, flags).bytes;
}

int32_t sbp_backward_linear_engine(int64_t M, int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, uint32_t flags,
                                   int32_t* split_count) {
  if (validate_linear(M, K, Cin, Cout, dtype, flags) != SBP_OK) return -1;
  const LinearPlan p = plan_linear(M, K, Cin, Cout, dtype, flags);
  if (split_count) *split_count = p.splits;
  return !p.mfma ? SBP_ENGINE_PLAIN : (p.big ? SBP_ENGINE_MFMA_LARGE : SBP_ENGINE_MFMA);
}

int32_t sbp_backward_linear(const void* dY, const int32_t* idx, const int32_t* inv, const void* Xk, const void* W,
                            int64_t M,
                            int64_t K, int32_t Cin, int32_t Cout, int32_t dtype, void* dW, float* db,
                            void* dX, void* ws, size_t ws_bytes, uint32_t flags, void* stream) {
  int32_t st = check_linear_args(dY, idx, Xk, W, M, K, Cin, Cout, dtype, dW, dX, flags);
  if (st != SBP_OK) return st;
  LinearPlan p = plan_linear(M, K, Cin, Cout, dtype, flags);
  if (p.bytes) {
    if (!ws) return fail(SBP_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", p.bytes);
    if (ws_bytes < p.bytes) return fail(SBP_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", ws_bytes, p.bytes);
    if ((uintptr_t)ws % 256) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  }
  if (!dW && !db && !dX) return SBP_OK;
  return launch_backward_linear(p, dY, idx, inv, Xk, W, M, K, Cin, Cout, dtype, dW, db, dX, ws, flags,
                                (hipStream_t)stream);
}

static int32_t check_batch(const sbp_linear_layer* layers, int32_t n, int32_t dtype) {
  if (!layers) return fail(SBP_ERR_NULL, "layers is NULL");
  if (n < 1 || n > SBP_MAX_BATCH_LAYERS) return fail(SBP_ERR_SHAPE, "need 1 <= n <= %d layers, got %d", SBP_MAX_BATCH_LAYERS, n);
  for (int i = 0; i < n; ++i) {
    const sbp_linear_layer& l = layers[i];
    if (l.reserved) return fail(SBP_ERR_FLAGS, "layer %d: reserved field must be 0", i);
    int32_t st = check_linear_args(l.dY, l.idx, l.X_k, l.W, l.M, l.K, l.Cin, l.Cout, dtype, l.dW, l.dX, l.flags);
    if (st != SBP_OK) return st;
  }
  return SBP_OK;
}

size_t sbp_backward_linear_batch_workspace(const sbp_linear_layer* layers, int32_t n, int32_t dtype) {
  if (!layers || n < 1 || n > SBP_MAX_BATCH_LAYERS || !elem_bytes(dtype)) return 0;
  for (int i = 0; i < n; ++i)
    if (validate_linear(layers[i].M, layers[i].K, layers[i].Cin, layers[i].Cout, dtype, layers[i].flags) != SBP_OK) return 0;
  return plan_linear_batch(layers, n, dtype).bytes;
}

int32_t sbp_backward_linear_batch(const sbp_linear_layer* layers, int32_t n, int32_t dtype, void* ws, size_t ws_bytes,
                                  void* stream) {
  int32_t st = check_batch(layers, n, dtype);
  if (st != SBP_OK) return st;
  const BatchPlan p = plan_linear_batch(layers, n, dtype);
  if (p.bytes) {
    if (!ws) return fail(SBP_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", p.bytes);
    if (ws_bytes < p.bytes) return fail(SBP_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", ws_bytes, p.bytes);
    if ((uintptr_t)ws % 256) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  }
  return launch_backward_linear_batch(p, layers, dtype, ws, (hipStream_t)stream);
}

static int32_t validate_dw(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int32_t pad, int64_t K,
                           int32_t dtype, uint32_t flags) {
  if (!elem_bytes(dtype)) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (flags) return fail(SBP_ERR_FLAGS, "unknown flags 0x%x", flags);
  if (B < 1 || H < 1 || W < 1 || C < 1) return fail(SBP_ERR_SHAPE, "bad shape B=%d H=%d W=%d C=%d", B, H, W, C);
  if (ks < 1 || ks > 7 || (ks & 1) == 0) return fail(SBP_ERR_SHAPE, "kernel size must be odd and <= 7, got %d", ks);
  if (pad != ks / 2) return fail(SBP_ERR_SHAPE, "pad must be ks/2=%d, got %d", ks / 2, pad);
  int64_t Mpos = (int64_t)B * H * W;
  if (Mpos > INT32_MAX) return fail(SBP_ERR_SHAPE, "B*H*W exceeds int32 row ids");
  if (K < 0 || K > Mpos) return fail(SBP_ERR_SHAPE, "need 0 <= K <= B*H*W, got K=%lld", (long long)K);
  return SBP_OK;
}

static int32_t validate_patches(int32_t B, int32_t H, int32_t W, int32_t C, int32_t p, int64_t K, int32_t dtype) {
  if (!elem_bytes(dtype)) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (p < 1 || p > 8) return fail(SBP_ERR_SHAPE, "patch size %d not in [1, 8]", p);
  if (B < 1 || H < 1 || W < 1 || C < 1 || H % p || W % p)
    return fail(SBP_ERR_SHAPE, "bad shape B=%d H=%d W=%d C=%d for patch size %d", B, H, W, C, p);
  if ((int64_t)B * H * W > INT32_MAX) return fail(SBP_ERR_SHAPE, "B*H*W too large");
  const int64_t Mo = (int64_t)B * (H / p) * (W / p);
  if (K < 0 || K > Mo) return fail(SBP_ERR_SHAPE, "need 0 <= K <= B*Ho*Wo, got K=%lld", (long long)K);
  return SBP_OK;
}

int32_t sbp_forward_cache_patches(const void* X, const int32_t* idx, int32_t B, int32_t H, int32_t W, int32_t C, int32_t p,
                                  int64_t K, int32_t dtype, void* Xk, void* stream) {
  int32_t st = validate_patches(B, H, W, C, p, K, dtype);
  if (st != SBP_OK) return st;
  if (K == 0) return SBP_OK;
  if (!X || !idx || !Xk) return fail(SBP_ERR_NULL, "X, idx or X_k is NULL");
  return launch_patches(false, X, idx, nullptr, B, H, W, C, p, K, elem_bytes(dtype), Xk, static_cast<hipStream_t>(stream));
}

size_t sbp_scatter_patches_workspace(int32_t B, int32_t H, int32_t W, int32_t p) {
  if (p < 1 || p > 8 || B < 1 || H < 1 || W < 1 || H % p || W % p) return 0;
  return align_up((size_t)B * (H / p) * (W / p) * sizeof(int32_t), 256);
}

int32_t sbp_scatter_patches(const void* dXp, const int32_t* idx, const int32_t* inv, int32_t B, int32_t H, int32_t W,
                            int32_t C, int32_t p, int64_t K, int32_t dtype, void* dX, void* ws, size_t ws_bytes,
                            void* stream) {
  int32_t st = validate_patches(B, H, W, C, p, K, dtype);
  if (st != SBP_OK) return st;
  if (!dX) return fail(SBP_ERR_NULL, "dX is NULL");
  if (K > 0 && (!dXp || !idx)) return fail(SBP_ERR_NULL, "dXp_k or idx is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!inv) {
    const size_t need = sbp_scatter_patches_workspace(B, H, W, p);
    if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) % 256) != 0)
      return fail(SBP_ERR_WORKSPACE, "workspace missing, misaligned or smaller than %zu bytes", need);
    launch_build_inverse(idx, K, static_cast<int32_t*>(ws), s);
    inv = static_cast<const int32_t*>(ws);
  }
  return launch_patches(true, dXp, idx, inv, B, H, W, C, p, K, elem_bytes(dtype), dX, s);
}

static int32_t validate_rows(int64_t K, int32_t C, int32_t dtype) {
  if (!elem_bytes(dtype)) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (K < 0 || C < 1 || K > INT32_MAX) return fail(SBP_ERR_SHAPE, "bad shape K=%lld C=%d", (long long)K, C);
  return SBP_OK;
}

int32_t sbp_act_forward_rows(const void* Zk, int64_t K, int32_t C, int32_t dtype, int32_t act, void* Hk, void* stream) {
  int32_t st = validate_rows(K, C, dtype);
  if (st != SBP_OK) return st;
  if (act != SBP_ACT_GELU) return fail(SBP_ERR_FLAGS, "unknown activation %d", act);
  if (K == 0) return SBP_OK;
  if (!Zk || !Hk) return fail(SBP_ERR_NULL, "Z_k or H_k is NULL");
  return launch_act_rows(nullptr, Zk, K * (int64_t)C, dtype, act, false, Hk, static_cast<hipStream_t>(stream));
}

int32_t sbp_act_backward_rows(const void* dHk, const void* Zk, int64_t K, int32_t C, int32_t dtype, int32_t act,
                              void* dZk, void* stream) {
  int32_t st = validate_rows(K, C, dtype);
  if (st != SBP_OK) return st;
  if (act != SBP_ACT_GELU) return fail(SBP_ERR_FLAGS, "unknown activation %d", act);
  if (K == 0) return SBP_OK;
  if (!dHk || !Zk || !dZk) return fail(SBP_ERR_NULL, "dH_k, Z_k or dZ_k is NULL");
  return launch_act_rows(dHk, Zk, K * (int64_t)C, dtype, act, true, dZk, static_cast<hipStream_t>(stream));
}

size_t sbp_backward_layerscale_workspace(int64_t K, int32_t C) {
  if (K < 0 || K > INT32_MAX || C < 1) return 0;
  return align_up((size_t)ls_blocks(K) * C * sizeof(float), 256);
}

int32_t sbp_backward_layerscale(const void* dUk, const void* Yk, const float* gamma, int64_t K, int32_t C, int32_t dtype,
                                float* dgamma, void* dYk, void* ws, size_t ws_bytes, uint32_t flags, void* stream) {
  int32_t st = validate_rows(K, C, dtype);
  if (st != SBP_OK) return st;
  if (flags & ~SBP_FLAG_ACCUMULATE_DW) return fail(SBP_ERR_FLAGS, "unknown flags 0x%x", flags);
  if (!dgamma && !dYk) return SBP_OK;
  if (K > 0 && (!dUk || !Yk || !gamma)) return fail(SBP_ERR_NULL, "dU_k, Y_k or gamma is NULL");
  const size_t need = sbp_backward_layerscale_workspace(K, C);
  if (dgamma && K > 0 && (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) % 256) != 0))
    return fail(SBP_ERR_WORKSPACE, "workspace missing, misaligned or smaller than %zu bytes", need);
  return launch_backward_layerscale(dUk, Yk, gamma, K, C, dtype, dgamma, dYk, static_cast<float*>(ws), flags,
                                    static_cast<hipStream_t>(stream));
}

static int32_t validate_attention(int32_t B, int32_t n_k, int32_t h, int32_t d, int32_t dtype) {
  if (!elem_bytes(dtype)) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (B < 1 || n_k < 0 || h < 1) return fail(SBP_ERR_SHAPE, "bad shape B=%d n_k=%d h=%d", B, n_k, h);
  if (d != 16 && d != 32 && d != 64 && d != 128) return fail(SBP_ERR_SHAPE, "head dimension %d is not 16, 32, 64 or 128", d);
  if ((int64_t)B * n_k > INT32_MAX || (int64_t)h * d * 3 > INT32_MAX || h > 65535 || B > 65535)
    return fail(SBP_ERR_SHAPE, "B=%d n_k=%d h=%d d=%d overflows the row / grid range", B, n_k, h, d);
  return SBP_OK;
}

int32_t sbp_backward_attention_engine(int32_t n_k, int32_t d, int32_t dtype) {
  if (validate_attention(1, n_k, 1, d, dtype) != SBP_OK) return -1;
  return attention_engine(n_k, d, dtype);
}

int32_t sbp_backward_attention(const void* qkv_k, const void* A_k, const void* dA_k, const float* lse_k, int32_t B,
                               int32_t n_k, int32_t h, int32_t d, float scale, int32_t dtype, void* dqkv_k,
                               void* stream) {
  int32_t st = validate_attention(B, n_k, h, d, dtype);
  if (st != SBP_OK) return st;
  if (!(scale == scale) || scale <= 0.f) return fail(SBP_ERR_SHAPE, "scale must be positive");
  if (n_k == 0) return SBP_OK;
  if (!qkv_k || !A_k || !dA_k || !lse_k || !dqkv_k) return fail(SBP_ERR_NULL, "qkv_k, A_k, dA_k, lse_k or dqkv_k is NULL");
  if (((uintptr_t)qkv_k | (uintptr_t)A_k | (uintptr_t)dA_k | (uintptr_t)dqkv_k) & 15)
    return fail(SBP_ERR_SHAPE, "tensors must be 16-byte aligned");
  return launch_backward_attention(qkv_k, A_k, dA_k, lse_k, B, n_k, h, d, scale, dtype, dqkv_k,
                                   static_cast<hipStream_t>(stream));
}

static int32_t validate_layernorm(int64_t M, int64_t K, int32_t C, int32_t dtype, uint32_t flags) {
  if (!elem_bytes(dtype)) return fail(SBP_ERR_DTYPE, "unknown dtype %d", dtype);
  if (flags & ~(SBP_FLAG_DX_COMPACT | SBP_FLAG_ACCUMULATE_DW)) return fail(SBP_ERR_FLAGS, "unknown flags 0x%x", flags);
  if (M < 1 || M > INT32_MAX || C < 1) return fail(SBP_ERR_SHAPE, "bad shape M=%lld C=%d", (long long)M, C);
  if (K < 0 || K > M) return fail(SBP_ERR_SHAPE, "need 0 <= K <= M, got K=%lld M=%lld", (long long)K, (long long)M);
  return SBP_OK;
}

size_t sbp_backward_layernorm_workspace(int64_t M, int64_t K, int32_t C, int32_t dtype, uint32_t flags) {
  if (validate_layernorm(M, K, C, dtype, flags) != SBP_OK) return 0;
  return plan_layernorm(M, K, C, dtype, flags).bytes;
}

int32_t sbp_backward_layernorm(const void* dUk, const void* Xk, const float* gamma, float eps, const int32_t* idx,
                               const int32_t* inv, int64_t M, int64_t K, int32_t C, int32_t dtype, float* dgamma,
                               float* dbeta, void* dX, void* ws, size_t ws_bytes, uint32_t flags, void* stream) {
  int32_t st = validate_layernorm(M, K, C, dtype, flags);
  if (st != SBP_OK) return st;
  if (!(eps >= 0.f)) return fail(SBP_ERR_SHAPE, "eps must be >= 0");
  if (!dgamma && !dbeta && !dX) return SBP_OK;
  if (K > 0 && (!dUk || !Xk || !gamma)) return fail(SBP_ERR_NULL, "dU_k, X_k or gamma is NULL");
  if (dX && !(flags & SBP_FLAG_DX_COMPACT) && !idx && K > 0) return fail(SBP_ERR_NULL, "idx is NULL");
  const LnPlan p = plan_layernorm(M, K, C, dtype, flags);
  if (!ws || ws_bytes < p.bytes || (reinterpret_cast<uintptr_t>(ws) % 256) != 0)
    return fail(SBP_ERR_WORKSPACE, "workspace missing, misaligned or smaller than %zu bytes", p.bytes);
  return launch_backward_layernorm(p, dUk, Xk, gamma, eps, idx, inv, M, K, C, dtype, dgamma, dbeta, dX, ws, flags,
                                   static_cast<hipStream_t>(stream));
}

size_t sbp_backward_dwconv_workspace(int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks, int64_t K,
                                     int32_t dtype, uint32_t flags) {
  if (validate_dw(B, H, W, C, ks, ks / 2, K, dtype, flags) != SBP_OK) return 0;
  return plan_dwconv(B, H, W, C, ks, K, dtype).bytes;
}

int32_t sbp_backward_dwconv(const void* dY, const int32_t* idx, const int32_t* inv, const void* X,
                            const void* Wd, int32_t B, int32_t H, int32_t W, int32_t C, int32_t ks,
                            int32_t pad, int64_t K, int32_t dtype, float* dWd, float* db, void* dX, void* ws,
                            size_t ws_bytes, uint32_t flags, void* stream) {
  int32_t st = validate_dw(B, H, W, C, ks, pad, K, dtype, flags);
  if (st != SBP_OK) return st;
  if (!dY) return fail(SBP_ERR_NULL, "dY is NULL");
  if ((dWd || db) && !idx && K > 0) return fail(SBP_ERR_NULL, "idx is NULL but dWd / db is requested");
  if (dX && !idx && !inv && K > 0) return fail(SBP_ERR_NULL, "idx and inv are both NULL");
  if ((dWd || db) && !X) return fail(SBP_ERR_NULL, "X is NULL but dWd / db is requested");
  if (dX && !Wd) return fail(SBP_ERR_NULL, "Wd is NULL but dX is requested");
  DwPlan p = plan_dwconv(B, H, W, C, ks, K, dtype);
  if (!ws) return fail(SBP_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", p.bytes);
  if (ws_bytes < p.bytes) return fail(SBP_ERR_WORKSPACE, "workspace %zu bytes < %zu needed", ws_bytes, p.bytes);
  if ((uintptr_t)ws % 256) return fail(SBP_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (!dWd && !db && !dX) return SBP_OK;
  return launch_backward_dwconv(p, dY, idx, inv, X, Wd, B, H, W, C, ks, pad, K, dtype, dWd, db, dX, ws,
                                (hipStream_t)stream);
}

int32_t sbp_set_option(const char* name, const char* value) {
  std::lock_guard<std::mutex> lock(g_opt_mutex);
  if (!name) {                 // back to the defaults
    g_opt = Options{};
    return SBP_OK;
  }
  Options o = g_opt;
  if (!apply_option(o, name, value))
    return fail(SBP_ERR_FLAGS, "unknown option or invalid value: %s = %s", name, value ? value : "(unset)");
  g_opt = o;
  return SBP_OK;
}

int32_t sbp_profile_enable(int32_t on) {
  g_prof_on = on != 0;
  return SBP_OK;
}

int32_t sbp_profile_timeline(void* records, int64_t capacity_records) {
  if (capacity_records < 0 || capacity_records > INT32_MAX) return fail(SBP_ERR_SHAPE, "bad record capacity");
  if (records && ((uintptr_t)records & 7)) return fail(SBP_ERR_SHAPE, "records must be 8-byte aligned");
  g_timeline = records && capacity_records ? static_cast<unsigned long long*>(records) : nullptr;
  g_timeline_cap = g_timeline ? (int)capacity_records : 0;
  return SBP_OK;
}

int32_t sbp_profile_read(int32_t which, double* total_ms, int64_t* launches) {
  if (which != SBP_PROF_RESET && (which < 0 || which >= SBP_PROF_NCLASSES))
    return fail(SBP_ERR_FLAGS, "unknown kernel class %d", which);
  if (which != SBP_PROF_RESET && (!total_ms || !launches)) return fail(SBP_ERR_NULL, "output pointer is NULL");
  if (!g_prof) return SBP_OK;
  if (which == SBP_PROF_RESET) {
    for (auto& r : *g_prof) {
      (void)hipEventSynchronize(r.b);
      (void)hipEventDestroy(r.a);
      (void)hipEventDestroy(r.b);
    }
    g_prof->clear();
    return SBP_OK;
  }
  for (auto& r : *g_prof) {
    if (r.cls != which) continue;
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess)
      return fail(SBP_ERR_HIP, "event timing failed");
    *total_ms += ms;
    *launches += 1;
  }
  return SBP_OK;
}

}  // extern "C"
