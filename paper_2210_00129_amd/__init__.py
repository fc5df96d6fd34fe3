"""MI355X-native hot path of Stochastic Backpropagation (SBP, arXiv 2210.00129).

Thin Python binding over the C-ABI library libsbp.so (hand-written HIP kernels for gfx950).
The functions below carry the names of the library's entry points and only marshal
arguments: torch provides device memory and the current stream, every step of the path
runs in the library's kernels.  There is no fallback: without the built library, or
without a GPU for the compute calls, they raise.

    idx, inv = sample_indices(B, P, H, W, k, seed, stream_id)     # draw the keep-set
    X_k      = forward_cache(X, idx)                              # cache kept rows only
    dW, db, dX = backward_linear(dY, idx, X_k, W)                 # token-subset backward
    dWd, db, dX = backward_dwconv(dY, idx, X, Wd)                 # depthwise 7x7, kept outputs
"""
from __future__ import annotations

import torch

from . import _lib
from ._lib import GatherItem, LinearLayer, SampleDesc, SbpError  # noqa: F401

F32, BF16 = 0, 1
GRID_PER_CELL, GRID_SHARED, RANDOM_MASK, TEMPORAL = 0, 1, 2, 3
FLAG_DY_COMPACT, FLAG_DX_COMPACT, FLAG_ACCUMULATE_DW, FLAG_DW_OUT_BF16, FLAG_XK_KMAJOR = 1, 2, 4, 8, 16
LAYOUT_ROWS, LAYOUT_KMAJOR = 0, 1

_DTYPES = {torch.float32: F32, torch.bfloat16: BF16}


def _dtype_code(t: torch.Tensor) -> int:
    try:
        return _DTYPES[t.dtype]
    except KeyError:
        raise TypeError(f"unsupported dtype {t.dtype}; use float32 or bfloat16") from None


def _dev(t, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in GPU memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def make_desc(B, P, H, W, k, seed, stream_id, mode=GRID_PER_CELL, per_sample=True, cell=2) -> SampleDesc:
    """cell: 2 for the grid and random modes; TEMPORAL: frames per cell (H = frames, W = positions per frame)."""
    return SampleDesc(int(B), int(P), int(H), int(W), int(cell), int(k), int(mode), int(bool(per_sample)),
                      int(seed) & 0xFFFFFFFFFFFFFFFF, int(stream_id) & 0xFFFFFFFFFFFFFFFF)


def k_from_ratio(r: float, cell: int = 2) -> int:
    """Kept slots per 2x2 cell for keep ratio r (host only)."""
    return _lib.check(_lib.lib().sbp_k_from_ratio(float(r), int(cell)))


def keep_count(B, P, H, W, k, mode=GRID_PER_CELL, per_sample=True, cell=2) -> int:
    """Number of kept rows K of a draw (host only, closed form)."""
    d = make_desc(B, P, H, W, k, 0, 0, mode, per_sample, cell)
    return _lib.check(_lib.lib().sbp_keep_count(d))


def sample_indices(B, P, H, W, k, seed, stream_id, mode=GRID_PER_CELL, per_sample=True, want_inv=False,
                   device="cuda", idx_out=None, inv_out=None, cell=2):
    """Draws the keep-set on the GPU; returns (idx [K] int32, inv [B*(P+H*W)] int32 or None)."""
    d = make_desc(B, P, H, W, k, seed, stream_id, mode, per_sample, cell)
    K = _lib.check(_lib.lib().sbp_keep_count(d))
    dev = torch.device(device)
    idx = idx_out if idx_out is not None else torch.empty(K, dtype=torch.int32, device=dev)
    inv = inv_out
    if inv is None and want_inv:
        inv = torch.empty(B * (P + H * W), dtype=torch.int32, device=dev)
    _lib.check(_lib.lib().sbp_sample_indices(d, _dev(idx, "idx"), idx.numel(), _dev(inv, "inv"),
                                             _stream(idx.device)))
    return idx, inv


def sample_indices_batch(descs, idx_list, inv_list=None):
    """Several draws in one call: descs = SampleDesc objects (make_desc), idx_list / inv_list = preallocated int32
    tensors on the GPU (inv_list or single entries may be None)."""
    import ctypes
    n = len(descs)
    arr = (SampleDesc * n)(*descs)
    idx_p = (ctypes.c_void_p * n)(*[_dev(t, "idx") for t in idx_list])
    cap = (ctypes.c_int64 * n)(*[t.numel() for t in idx_list])
    inv_p = None
    if inv_list is not None:
        inv_p = (ctypes.c_void_p * n)(*[_dev(t, "inv") for t in inv_list])
    _lib.check(_lib.lib().sbp_sample_indices_batch(arr, n, idx_p, cap, inv_p, _stream(idx_list[0].device)))
    return idx_list, inv_list


def forward_cache(X: torch.Tensor, idx: torch.Tensor, out=None) -> torch.Tensor:
    """X_k = X[idx] (rows), the only part of the layer input kept for the backward pass."""
    if X.dim() != 2:
        raise ValueError("X must be [M, C]")
    M, C = X.shape
    K = idx.numel()
    Xk = out if out is not None else torch.empty((K, C), dtype=X.dtype, device=X.device)
    _lib.check(_lib.lib().sbp_forward_cache(_dev(X, "X"), _dev(idx, "idx"), M, K, C, _dtype_code(X),
                                            _dev(Xk, "X_k"), _stream(X.device)))
    return Xk


def forward_cache_batch(Xs, idxs, outs=None, layout=LAYOUT_ROWS):
    """X_k = X[idx] for several tensors in one call (one launch where every row is a multiple of 16 bytes).
    layout = LAYOUT_KMAJOR writes [ceil(K / 8), C, 8] (groups of 8 kept rows side by side per channel, zero padded)."""
    n = len(Xs)
    if outs is None:
        if layout == LAYOUT_KMAJOR:
            outs = [torch.empty(((i.numel() + 7) // 8, X.shape[1], 8), dtype=X.dtype, device=X.device) for X, i in zip(Xs, idxs)]
        else:
            outs = [torch.empty((i.numel(), X.shape[1]), dtype=X.dtype, device=X.device) for X, i in zip(Xs, idxs)]
    items = (GatherItem * n)(*[GatherItem(_dev(X, "X"), _dev(i, "idx"), _dev(o, "X_k"), X.shape[0], i.numel(), X.shape[1], layout)
                               for X, i, o in zip(Xs, idxs, outs)])
    _lib.check(_lib.lib().sbp_forward_cache_batch(items, n, _dtype_code(Xs[0]), _stream(Xs[0].device)))
    return outs


def backward_linear_workspace(M, K, Cin, Cout, dtype_code, flags=0) -> int:
    return int(_lib.lib().sbp_backward_linear_workspace(M, K, Cin, Cout, dtype_code, flags))


ENGINE_NAMES = {0: "plain", 1: "mfma", 2: "mfma_large"}


def backward_linear_engine(M, K, Cin, Cout, dtype_code, flags=0):
    """(engine name, dW split count) that sbp_backward_linear uses for these sizes."""
    import ctypes
    n = ctypes.c_int32(0)
    e = int(_lib.lib().sbp_backward_linear_engine(M, K, Cin, Cout, dtype_code, flags, ctypes.byref(n)))
    if e < 0:
        raise ValueError("invalid sizes")
    return ENGINE_NAMES[e], int(n.value)


def backward_linear(dY, idx, X_k, W, M=None, flags=0, want=("dW", "db", "dX"), dW=None, db=None, dX=None,
                    workspace=None, inv=None):
    """SBP backward of Y = X W^T + b on the kept rows.  Returns (dW fp32 - bf16 with FLAG_DW_OUT_BF16 -, db fp32, dX)."""
    Cout, Cin = W.shape
    K = idx.numel() if idx is not None else dY.shape[0]
    if M is None:
        if flags & FLAG_DY_COMPACT:
            raise ValueError("M is required when dY is compact")
        M = dY.shape[0]
    code = _dtype_code(W)
    dev = W.device
    if "dW" in want and dW is None:
        dW = torch.empty((Cout, Cin), dtype=torch.bfloat16 if flags & FLAG_DW_OUT_BF16 else torch.float32, device=dev)
    if dW is not None and dW.dtype != (torch.bfloat16 if flags & FLAG_DW_OUT_BF16 else torch.float32):
        raise ValueError("dW must be bfloat16 with FLAG_DW_OUT_BF16 and float32 without")
    if "db" in want and db is None:
        db = torch.empty((Cout,), dtype=torch.float32, device=dev)
    if "dX" in want and dX is None:
        rows = K if (flags & FLAG_DX_COMPACT) else M
        dX = torch.empty((rows, Cin), dtype=W.dtype, device=dev)
    need = backward_linear_workspace(M, K, Cin, Cout, code, flags)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _lib.check(_lib.lib().sbp_backward_linear(
        _dev(dY, "dY"), _dev(idx, "idx"), _dev(inv, "inv"), _dev(X_k, "X_k"), _dev(W, "W"), M, K, Cin, Cout, code,
        _dev(dW, "dW"), _dev(db, "db"), _dev(dX, "dX"), _dev(workspace, "workspace"), workspace.numel(),
        flags, _stream(dev)))
    return dW, db, dX


def make_layer(dY, idx, X_k, W, M, dW=None, db=None, dX=None, flags=0, inv=None) -> LinearLayer:
    """One sbp_linear_layer descriptor from tensors (outputs preallocated by the caller; None skips one)."""
    Cout, Cin = W.shape
    K = idx.numel() if idx is not None else dY.shape[0]
    return LinearLayer(_dev(dY, "dY"), _dev(idx, "idx"), _dev(inv, "inv"), _dev(X_k, "X_k"), _dev(W, "W"), int(M), int(K),
                       int(Cin), int(Cout), _dev(dW, "dW"), _dev(db, "db"), _dev(dX, "dX"), int(flags), 0)


def backward_linear_batch_workspace(descs, dtype_code) -> int:
    arr = (LinearLayer * len(descs))(*descs)
    return int(_lib.lib().sbp_backward_linear_batch_workspace(arr, len(descs), dtype_code))


def backward_linear_batch(layers, workspace=None, want=("dW", "db", "dX")):
    """SBP backward of several independent layers in one call.  layers: dicts with dY, idx, X_k, W, M and
    optionally flags, inv, dW, db, dX (preallocated outputs); outputs named in `want` are allocated when absent.
    Returns a list of (dW, db, dX)."""
    descs, outs = [], []
    code = None
    for l in layers:
        W = l["W"]
        Cout, Cin = W.shape
        flags = l.get("flags", 0)
        idx = l["idx"]
        K = idx.numel()
        M = l["M"]
        dev = W.device
        code = _dtype_code(W)
        dW, db, dX = l.get("dW"), l.get("db"), l.get("dX")
        if "dW" in want and dW is None:
            dW = torch.empty((Cout, Cin), dtype=torch.bfloat16 if flags & FLAG_DW_OUT_BF16 else torch.float32, device=dev)
        if "db" in want and db is None:
            db = torch.empty((Cout,), dtype=torch.float32, device=dev)
        if "dX" in want and dX is None:
            dX = torch.empty((K if flags & FLAG_DX_COMPACT else M, Cin), dtype=W.dtype, device=dev)
        descs.append(make_layer(l["dY"], idx, l["X_k"], W, M, dW, db, dX, flags, l.get("inv")))
        outs.append((dW, db, dX))
    arr = (LinearLayer * len(descs))(*descs)
    need = int(_lib.lib().sbp_backward_linear_batch_workspace(arr, len(descs), code))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=layers[0]["W"].device)
    _lib.check(_lib.lib().sbp_backward_linear_batch(arr, len(descs), code, _dev(workspace, "workspace"), workspace.numel(),
                                                    _stream(layers[0]["W"].device)))
    return outs


def static_scratch_bytes() -> int:
    return int(_lib.lib().sbp_static_scratch_bytes())


def backward_linear_static(dY, idx, X_k, W, dW, db, dX, M, flags=0, inv=None):
    """sbp_backward_linear_static: the caller passes inputs and (preallocated) outputs only; the workspace is the
    library's own fixed device array.  Any of dW, db, dX may be None."""
    Cout, Cin = W.shape
    K = idx.numel() if idx is not None else dY.shape[0]
    _lib.check(_lib.lib().sbp_backward_linear_static(
        _dev(dY, "dY"), _dev(idx, "idx"), _dev(inv, "inv"), _dev(X_k, "X_k"), _dev(W, "W"), M, K, Cin, Cout,
        _dtype_code(W), _dev(dW, "dW"), _dev(db, "db"), _dev(dX, "dX"), flags, _stream(W.device)))
    return dW, db, dX


def forward_cache_patches(X, idx, p, out=None):
    """Rows [K, p*p*C]: the p x p input patch of X [B, H, W, C] under every kept output position."""
    B, H, W, C = X.shape
    K = idx.numel()
    Xk = out if out is not None else torch.empty((K, p * p * C), dtype=X.dtype, device=X.device)
    _lib.check(_lib.lib().sbp_forward_cache_patches(_dev(X, "X"), _dev(idx, "idx"), B, H, W, C, p, K, _dtype_code(X),
                                                    _dev(Xk, "X_k"), _stream(X.device)))
    return Xk


def scatter_patches(dXp_k, idx, shape, p, inv=None, out=None):
    """dX [B, H, W, C] from the compact gradient rows [K, p*p*C] of a down-sampling layer (zeros elsewhere)."""
    B, H, W, C = shape
    K = idx.numel()
    dX = out if out is not None else torch.empty((B, H, W, C), dtype=dXp_k.dtype, device=dXp_k.device)
    ws = None
    nbytes = 0
    if inv is None:
        nbytes = int(_lib.lib().sbp_scatter_patches_workspace(B, H, W, p))
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dXp_k.device)
    _lib.check(_lib.lib().sbp_scatter_patches(_dev(dXp_k, "dXp_k"), _dev(idx, "idx"), _dev(inv, "inv"), B, H, W, C, p, K,
                                              _dtype_code(dXp_k), _dev(dX, "dX"), _dev(ws, "workspace"),
                                              ws.numel() if ws is not None else 0, _stream(dXp_k.device)))
    return dX


ACT_GELU = 0


def act_forward_rows(Z_k, out=None, act=ACT_GELU):
    """H_k = gelu(Z_k) on compact kept rows [K, C]."""
    K, C = Z_k.shape
    if out is None:
        out = torch.empty_like(Z_k)
    _lib.check(_lib.lib().sbp_act_forward_rows(_dev(Z_k, "Z_k"), K, C, _dtype_code(Z_k), act, _dev(out, "H_k"),
                                               _stream(Z_k.device)))
    return out


def act_backward_rows(dH_k, Z_k, out=None, act=ACT_GELU):
    """dZ_k = dH_k * gelu'(Z_k) on compact kept rows [K, C] (out may be dH_k)."""
    K, C = Z_k.shape
    if out is None:
        out = torch.empty_like(Z_k)
    _lib.check(_lib.lib().sbp_act_backward_rows(_dev(dH_k, "dH_k"), _dev(Z_k, "Z_k"), K, C, _dtype_code(Z_k), act,
                                                _dev(out, "dZ_k"), _stream(Z_k.device)))
    return out


def backward_layernorm_workspace(M, K, C, dtype_code, flags=0) -> int:
    return int(_lib.lib().sbp_backward_layernorm_workspace(M, K, C, dtype_code, flags))


def backward_layernorm(dU_k, X_k, gamma, eps, idx, M, inv=None, flags=0, want=("dgamma", "dbeta", "dX"),
                       dgamma=None, dbeta=None, dX=None, workspace=None):
    """LayerNorm backward on the kept rows.  dU_k, X_k: [K, C]; gamma fp32 [C].  Returns (dgamma, dbeta, dX)."""
    K, C = X_k.shape
    code = _dtype_code(X_k)
    dev = X_k.device
    if "dgamma" in want and dgamma is None:
        dgamma = torch.empty((C,), dtype=torch.float32, device=dev)
    if "dbeta" in want and dbeta is None:
        dbeta = torch.empty((C,), dtype=torch.float32, device=dev)
    if "dX" in want and dX is None:
        dX = torch.empty((K if (flags & FLAG_DX_COMPACT) else M, C), dtype=X_k.dtype, device=dev)
    need = backward_layernorm_workspace(M, K, C, code, flags)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _lib.check(_lib.lib().sbp_backward_layernorm(
        _dev(dU_k, "dU_k"), _dev(X_k, "X_k"), _dev(gamma, "gamma"), float(eps), _dev(idx, "idx"), _dev(inv, "inv"),
        M, K, C, code, _dev(dgamma, "dgamma"), _dev(dbeta, "dbeta"), _dev(dX, "dX"), _dev(workspace, "workspace"),
        workspace.numel(), flags, _stream(dev)))
    return dgamma, dbeta, dX


def backward_layerscale(dU_k, Y_k, gamma, flags=0, want=("dgamma", "dY"), dgamma=None, dY=None, workspace=None):
    """Per-channel layer scale backward on the kept rows.  dU_k, Y_k: [K, C]; gamma fp32 [C].  Returns (dgamma, dY_k)."""
    K, C = Y_k.shape
    dev = Y_k.device
    if "dgamma" in want and dgamma is None:
        dgamma = torch.empty((C,), dtype=torch.float32, device=dev)
    if "dY" in want and dY is None:
        dY = torch.empty_like(dU_k)
    need = int(_lib.lib().sbp_backward_layerscale_workspace(K, C))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _lib.check(_lib.lib().sbp_backward_layerscale(
        _dev(dU_k, "dU_k"), _dev(Y_k, "Y_k"), _dev(gamma, "gamma"), K, C, _dtype_code(Y_k), _dev(dgamma, "dgamma"),
        _dev(dY, "dY_k"), _dev(workspace, "workspace"), workspace.numel(), flags, _stream(dev)))
    return dgamma, dY


def backward_dwconv_workspace(B, H, W, C, ks, K, dtype_code, flags=0) -> int:
    return int(_lib.lib().sbp_backward_dwconv_workspace(B, H, W, C, ks, K, dtype_code, flags))


def backward_dwconv(dY, idx, X, Wd, inv=None, want=("dWd", "db", "dX"), dWd=None, db=None, dX=None,
                    workspace=None):
    """Depthwise-conv backward on the kept output positions.  dY, X: [B,H,W,C]; Wd: [ks,ks,C]."""
    B, H, W, C = dY.shape
    ks = Wd.shape[0]
    K = idx.numel()
    code = _dtype_code(dY)
    dev = dY.device
    if "dWd" in want and dWd is None:
        dWd = torch.empty((ks, ks, C), dtype=torch.float32, device=dev)
    if "db" in want and db is None:
        db = torch.empty((C,), dtype=torch.float32, device=dev)
    if "dX" in want and dX is None:
        dX = torch.empty((B, H, W, C), dtype=dY.dtype, device=dev)
    need = backward_dwconv_workspace(B, H, W, C, ks, K, code, 0)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _lib.check(_lib.lib().sbp_backward_dwconv(
        _dev(dY, "dY"), _dev(idx, "idx"), _dev(inv, "inv"), _dev(X, "X"), _dev(Wd, "Wd"), B, H, W, C, ks, ks // 2,
        K, code, _dev(dWd, "dWd"), _dev(db, "db"), _dev(dX, "dX"), _dev(workspace, "workspace"),
        workspace.numel(), 0, _stream(dev)))
    return dWd, db, dX


def backward_attention_engine(n_k, d, dtype_code) -> str:
    """Which kernel serves an attention backward of n_k kept tokens per sample: 'mfma' (one workgroup per head),
    'mfma_tiled' (chunks of 128 tokens) or 'plain'."""
    e = int(_lib.lib().sbp_backward_attention_engine(n_k, d, dtype_code))
    if e < 0:
        raise ValueError(_lib.lib().sbp_last_error().decode())
    return {1: "mfma", 2: "mfma_tiled"}.get(e, "plain")


def backward_attention(qkv_k, A_k, dA_k, lse_k, B, h, d, scale, out=None):
    """Attention backward on the kept tokens ("Drop QKV").  qkv_k: [B*n_k, 3*h*d]; A_k, dA_k: [B*n_k, h*d];
    lse_k: fp32 [B*n_k, h].  Returns dqkv_k [B*n_k, 3*h*d] (dQ | dK | dV)."""
    rows = qkv_k.shape[0]
    if rows % B:
        raise ValueError("rows of qkv_k must be B * n_k")
    n_k = rows // B
    if out is None:
        out = torch.empty_like(qkv_k)
    _lib.check(_lib.lib().sbp_backward_attention(
        _dev(qkv_k, "qkv_k"), _dev(A_k, "A_k"), _dev(dA_k, "dA_k"), _dev(lse_k, "lse_k"), B, n_k, h, d, float(scale),
        _dtype_code(qkv_k), _dev(out, "dqkv_k"), _stream(qkv_k.device)))
    return out


def set_option(name=None, value=None) -> None:
    """Explicit override for tests and sweeps (see sbp_set_option in include/sbp.h); name=None restores the defaults."""
    _lib.check(_lib.lib().sbp_set_option(None if name is None else str(name).encode(),
                                         None if value is None else str(value).encode()))


class options:
    """Context manager: sets overrides for the duration of a block, then restores the defaults for those names."""
    def __init__(self, **kv):
        self.kv = kv

    def __enter__(self):
        for k, v in self.kv.items():
            set_option(k, v)
        return self

    def __exit__(self, *exc):
        for k in self.kv:
            set_option(k, None)


PROF_CLASSES = ("sample", "gather", "dw_gemm", "dx_gemm", "reduce", "colsum", "zero_rows", "dwconv_dx",
                "dwconv_dw", "other", "attention")


def profile_enable(on: bool) -> None:
    """Benchmark aid: bracket every kernel launch of the library with HIP events."""
    _lib.check(_lib.lib().sbp_profile_enable(1 if on else 0))


def profile_timeline(records=None) -> None:
    """Benchmark aid: per-workgroup time stamps of the batched linear backward into `records` (int64 tensor
    [n, 8] on the GPU, zeroed by the caller); None switches it off."""
    if records is None:
        _lib.check(_lib.lib().sbp_profile_timeline(None, 0))
    else:
        _lib.check(_lib.lib().sbp_profile_timeline(_dev(records, "records"), records.shape[0]))


def profile_read(reset: bool = True) -> dict:
    """Per kernel class: (total milliseconds, launches) recorded since the last reset."""
    import ctypes
    out = {}
    for i, name in enumerate(PROF_CLASSES):
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _lib.check(_lib.lib().sbp_profile_read(i, ctypes.byref(ms), ctypes.byref(n)))
        out[name] = (ms.value, n.value)
    if reset:
        _lib.check(_lib.lib().sbp_profile_read(-1, None, None))
    return out
