"""Plain CPU oracle of the Stochastic-Backpropagation (SBP) hot path.

TEST INFRASTRUCTURE.  Slow, fp64, obviously-correct write-out of what the paper
defines; it is imported only by tests, the smoke check and the benchmark's
cpu_baseline leg, never by the product path, and it shares no code with the HIP
kernels.

What follows the paper and what is this repository's own reading:

* ``backward_linear`` is the definition in the paper's section "Calculation of
  Linear Layers": the split of the backward pass into kept and dropped index
  sets (the equation labelled ``eq:backward_fc_sbp``) with every dropped term
  removed, i.e. dX_drop = 0 and dW = X_keep^T dX_{i+1}^keep.  The paper stores
  W as [C_in, C_out]; here W is [C_out, C_in] (Y = X W^T + b), so the same
  quantities read dW = dY_k^T X_k and dX_k = dY_k W.  The paper omits the
  bias; db = column sum of the kept rows of dY follows from the same split.
  No 1/r rescaling: the update rule (``eq:sbp_formula``) carries only 1/B,
  which belongs to the loss.
* ``backward_dwconv`` is the ordinary convolution backward of the section
  "Calculation of Convolutional Layers" (``eq:conv_grad_layer_before_sbp``)
  applied to dY with its dropped positions set to zero, for a depthwise
  kernel.  dX is dense (the paper's remark (a): dropped inputs still receive
  gradient from kept neighbours).
* ``forward_cache`` keeps only the kept rows of the layer input ("only caches a
  subset of the feature maps").
* ``sample_indices``: the paper only names "grid-wise mask sampling" and shows a
  figure.  The reading taken here: tile the H x W map into 2x2 cells and keep
  k = round(4 r) of the four slots of every cell, drawn from a counter-based
  integer hash of (seed, stream, sample, cell).  The hash constants and the
  canonical order of the index list are this repository's own specification:
  PARITY UNPINNED by the paper for the generator itself (the mixer is pinned to
  the published SplitMix64 sequence, the structure to the properties the paper
  states: fixed keep ratio per cell, equal visiting frequency of every
  position).  Cells of 3 x 3 and 4 x 4 slots (keep ratios k/9 and k/16) follow
  the same construction: a permutation of the cell's slots from the hash (the
  hash scaled to [0, slots!) by a 64 x 64 -> high 64 bit product, Lehmer
  decoded), the k slots of smallest rank kept, edge cells with v valid slots
  keeping max(1, round-half-up(k v / slots)) of them.
* ``act_forward_rows`` / ``act_backward_rows`` / ``backward_layernorm``: the
  paper's implementation (Alg. ``alg:sbp_impl``) wraps "an arbitrary operation
  f": the kept rows go through f with gradient, the dropped rows without, and
  with one keep-set shared by a stack of layers the kept / dropped split passes
  through the chain unchanged (``eq:backward_fc2_sbp_same_drop_loc``).  For a
  row-wise f (GELU, LayerNorm) that is the ordinary backward of f on the kept
  rows, zero on the dropped rows, parameter gradients summed over the kept
  rows only.  GELU is the exact form x Phi(x) used by ViT and ConvNeXt.
  ``backward_layerscale`` is the same for ConvNeXt's per-channel layer scale
  U = gamma * Y at the end of the block's branch.
* ``backward_downsample`` / ``forward_cache_patches``: a convolution whose stride
  is at least its kernel size (the p x p, stride p down-sampling layers of
  ConvNeXt).  The paper's section "Calculation of Convolutional Layers" notes
  that for s >= k the neighbour effects vanish and the layer behaves like a
  point-wise one: every kept output position owns its own p x p patch of inputs.
  The oracle writes the convolution backward out position by position.
* ``backward_attention``: the supplement's section "Gradient Calculation of
  Attention Layers" applies the gradient dropout to the attention map M
  (``eq:sbp_attn_drop_query`` .. ``eq:sbp_sep_on_key``) and writes the case
  "drop on the query" out; the main text (section Design Strategies, "How to
  apply SBP on MHSA?") picks "Drop QKV" for image transformers and leaves its
  derivation to the reader.  The reading taken here: the forward is the
  ordinary full attention; in the backward every entry of dM whose query OR key
  token is dropped is set to zero, the kept entries keep their exact value
  (``eq:grad_qkv`` with the ordinary softmax derivative over the whole row),
  and the gradients of Q, K and V are taken at the kept tokens only (zero at the
  dropped ones).  dA arrives with zero rows at the dropped tokens (the chain
  rule effect of the section "Chain Rule Effect of Transformer Blocks").
  Of the two forms of dQ the supplement prints, the shape-consistent one is
  used: dQ = dM K / sqrt(d), dK = dM^T Q / sqrt(d).
"""
from __future__ import annotations

import numpy as np

GRID_PER_CELL = 0  # independent draw in every 2x2 cell
GRID_SHARED = 1    # one slot permutation shared by all cells of a sample
RANDOM_MASK = 2    # uniformly random subset of the grid positions of a sample (the paper's "random mask sampling")
TEMPORAL = 3       # whole frames: k of every `cell` consecutive frames (the temporal special case the paper cites)

_MASK64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def mix64(z: int) -> int:
    """SplitMix64 output function (Steele, Lea, Flood 2014) on a 64-bit word."""
    z &= _MASK64
    z = ((z ^ (z >> 30)) * _C1) & _MASK64
    z = ((z ^ (z >> 27)) * _C2) & _MASK64
    return z ^ (z >> 31)


def _absorb(h: int, v: int) -> int:
    return mix64((h + v + _GAMMA) & _MASK64)


def k_from_ratio(r: float, cell: int = 2) -> int:
    """Kept slots per cell for keep ratio r: round-half-up(r * cell^2), at least 1."""
    if not (0.0 < r <= 1.0):
        raise ValueError("keep ratio must be in (0, 1]")
    n = cell * cell
    k = int(np.floor(r * n + 0.5))
    return max(1, min(n, k))


def _k_partial(k: int, c: int) -> int:
    """Kept slots of an edge cell with c (1 or 2) valid slots: round-half-up(k*c/4), >= 1."""
    return max(1, (k * c + 2) // 4)


def keep_count(B: int, P: int, H: int, W: int, k: int) -> int:
    """Closed-form number of kept rows for a draw (keep ratio r = K / (B*(P+H*W)))."""
    full = (H // 2) * (W // 2)
    edge2 = (W % 2) * (H // 2) + (H % 2) * (W // 2)
    corner = (H % 2) * (W % 2)
    return B * (P + k * full + _k_partial(k, 2) * edge2 + _k_partial(k, 1) * corner)


def _slot_ranks(h: int):
    """Rank (0..3) of each of the four slots in the permutation drawn from hash h.

    p in [0, 24) is taken from the top 32 bits of h by multiply-shift and decoded
    as a Lehmer code: digit d_t picks the d_t-th of the slots not yet placed.
    """
    p = ((h >> 32) * 24) >> 32
    digits = (p // 6, (p % 6) // 2, p % 2, 0)
    remaining = [0, 1, 2, 3]
    rank = [0, 0, 0, 0]
    for t, d in enumerate(digits):
        s = remaining.pop(d)
        rank[s] = t
    return rank


def sample_indices(B, P, H, W, k, seed, stream_id, mode=GRID_PER_CELL, per_sample=True):
    """Grid-wise keep-set at k kept slots per 2x2 cell.

    Returns int32 flat row ids into the [B*(P+H*W)] row space, in canonical
    order: sample-major; inside a sample the P prefix rows (always kept), then
    the cells in row-major cell order, and inside a cell the kept slots in
    ascending slot number s = 2*(y%2) + (x%2).
    """
    if not (1 <= k <= 4):
        raise ValueError("k must be in 1..4")
    N = P + H * W
    ch, cw = (H + 1) // 2, (W + 1) // 2
    base = _absorb(_absorb(0, seed), stream_id)
    out = []
    for b in range(B):
        hb = _absorb(base, b if per_sample else 0)
        out.extend(b * N + p for p in range(P))
        for cy in range(ch):
            for cx in range(cw):
                cell = 0 if mode == GRID_SHARED else cy * cw + cx
                rank = _slot_ranks(_absorb(hb, cell))
                valid = [s for s in range(4)
                         if 2 * cy + (s >> 1) < H and 2 * cx + (s & 1) < W]
                kc = k if len(valid) == 4 else _k_partial(k, len(valid))
                chosen = sorted(sorted(valid, key=lambda s: rank[s])[:kc])
                for s in chosen:
                    y, x = 2 * cy + (s >> 1), 2 * cx + (s & 1)
                    out.append(b * N + P + y * W + x)
    return np.asarray(out, dtype=np.int32)


def _factorial(n: int) -> int:
    f = 1
    for i in range(2, n + 1):
        f *= i
    return f


def _k_partial_cell(k: int, valid: int, slots: int) -> int:
    """Kept slots of an edge cell with `valid` of `slots` slots inside the map: round-half-up(k*valid/slots), >= 1."""
    return max(1, (2 * k * valid + slots) // (2 * slots))


def keep_count_cells(B: int, P: int, H: int, W: int, k: int, cell: int) -> int:
    """Number of kept rows of sample_indices_cells (closed form)."""
    n = cell * cell
    fh, fw, rh, rw = H // cell, W // cell, H % cell, W % cell
    total = k * fh * fw
    if rw:
        total += fh * _k_partial_cell(k, cell * rw, n)
    if rh:
        total += fw * _k_partial_cell(k, rh * cell, n)
    if rh and rw:
        total += _k_partial_cell(k, rh * rw, n)
    return B * (P + total)


def _slot_ranks_cells(h: int, n: int):
    """Rank of each of the n slots in the permutation drawn from the 64-bit hash h: p = floor(h * n! / 2^64),
    Lehmer decoded (digit t, most significant first, picks the d_t-th of the slots not yet placed)."""
    p = (h * _factorial(n)) >> 64
    remaining = list(range(n))
    rank = [0] * n
    for t in range(n):
        f = _factorial(n - 1 - t)
        d, p = divmod(p, f)
        rank[remaining.pop(d)] = t
    return rank


def sample_indices_cells(B, P, H, W, k, cell, seed, stream_id, mode=GRID_PER_CELL, per_sample=True):
    """Grid-wise keep-set with cells of cell x cell slots (cell = 3 or 4), k of the cell^2 slots of every cell kept:
    keep ratio k / cell^2.  Same hash chain and canonical order as sample_indices (sample-major; prefix rows; cells
    row-major; inside a cell the kept slots ascending, slot s = cell * (y % cell) + (x % cell))."""
    n = cell * cell
    if cell not in (3, 4) or not (1 <= k <= n):
        raise ValueError("need cell in (3, 4) and 1 <= k <= cell^2")
    N = P + H * W
    ch, cw = -(-H // cell), -(-W // cell)
    base = _absorb(_absorb(0, seed), stream_id)
    out = []
    for b in range(B):
        hb = _absorb(base, b if per_sample else 0)
        out.extend(b * N + p for p in range(P))
        for cy in range(ch):
            for cx in range(cw):
                c = 0 if mode == GRID_SHARED else cy * cw + cx
                rank = _slot_ranks_cells(_absorb(hb, c), n)
                valid = [s for s in range(n) if cell * cy + s // cell < H and cell * cx + s % cell < W]
                kc = k if len(valid) == n else _k_partial_cell(k, len(valid), n)
                for s in sorted(sorted(valid, key=lambda q: rank[q])[:kc]):
                    out.append(b * N + P + (cell * cy + s // cell) * W + cell * cx + s % cell)
    return np.asarray(out, dtype=np.int32)


def random_keep_count(H: int, W: int, k: int) -> int:
    """Kept grid positions per sample of the random mask at ratio k/4: round-half-up(k*H*W/4), >= 1."""
    return max(1, (k * H * W + 2) // 4)


def sample_indices_random(B, P, H, W, k, seed, stream_id, per_sample=True):
    """Random mask sampling (section "Design Strategies", "How to sample the gradient keep mask?"): per sample
    a uniformly random subset of exactly round(k/4 * H*W) grid positions, no grid structure.

    This repository's construction (the paper gives none): every position p draws the key
    absorb(h_sample, p) from the counter hash; the positions with the smallest (key, p) are kept.
    Canonical order: sample-major, the P prefix rows, then the kept positions in ascending order.
    """
    if not (1 <= k <= 4):
        raise ValueError("k must be in 1..4")
    N = P + H * W
    n_keep = random_keep_count(H, W, k)
    base = _absorb(_absorb(0, seed), stream_id)
    out = []
    for b in range(B):
        hb = _absorb(base, b if per_sample else 0)
        keys = [(_absorb(hb, p), p) for p in range(H * W)]
        kept = sorted(p for _, p in sorted(keys)[:n_keep])
        out.extend(b * N + p for p in range(P))
        out.extend(b * N + P + p for p in kept)
    return np.asarray(out, dtype=np.int32)


def temporal_keep_frames(T: int, c: int, k: int) -> int:
    """Kept frames per sample: k of every full cell of c frames, round-half-up(k*c'/c) >= 1 of a tail of c' frames."""
    tail = T % c
    return k * (T // c) + (max(1, (2 * k * tail + c) // (2 * c)) if tail else 0)


def sample_indices_temporal(B, P, T, HW, c, k, seed, stream_id, per_sample=True):
    """Temporal subsets (the special case on the temporal dimension that the paper cites under eq:sbp_formula):
    the rows of a sample are P prefix rows and T frames of HW positions; of every c consecutive frames k are kept
    whole.  Inside a cell frame s draws the key absorb(h_cell, s); the frames with the smallest (key, s) are kept.
    Canonical order: sample-major, prefix rows, then kept frames ascending, positions ascending.
    """
    if not (2 <= c <= 4 and 1 <= k <= c):
        raise ValueError("need 2 <= c <= 4 and 1 <= k <= c")
    N = P + T * HW
    base = _absorb(_absorb(0, seed), stream_id)
    out = []
    for b in range(B):
        hb = _absorb(base, b if per_sample else 0)
        out.extend(b * N + p for p in range(P))
        for cell in range((T + c - 1) // c):
            frames = [f for f in range(cell * c, min(T, cell * c + c))]
            kc = k if len(frames) == c else max(1, (2 * k * len(frames) + c) // (2 * c))
            hc = _absorb(hb, cell)
            ranked = sorted(frames, key=lambda f: (_absorb(hc, f - cell * c), f))
            for f in sorted(ranked[:kc]):
                out.extend(b * N + P + f * HW + p for p in range(HW))
    return np.asarray(out, dtype=np.int32)


def inverse_map(idx, M):
    """inv[m] = position of row m in idx, or -1 for a dropped row."""
    inv = np.full(M, -1, dtype=np.int32)
    inv[np.asarray(idx, dtype=np.int64)] = np.arange(len(idx), dtype=np.int32)
    return inv


def forward_cache(X, idx):
    """X_k[j, :] = X[idx[j], :] -- the only activation kept for the backward pass."""
    X = np.asarray(X)
    return X[np.asarray(idx, dtype=np.int64)].copy()


def backward_linear(dY, idx, X_k, W, M):
    """SBP backward of Y = X W^T + b restricted to the kept rows Z = set(idx).

    dY [M, Cout] (only rows in idx are read), X_k [K, Cin] = X[idx], W [Cout, Cin].
    Returns (dW [Cout, Cin], db [Cout], dX [M, Cin]) in fp64:
      dW[o, i] = sum_{m in Z} dY[m, o] X[m, i]
      db[o]    = sum_{m in Z} dY[m, o]
      dX[m, :] = dY[m, :] W for m in Z, +0.0 elsewhere.
    """
    idx = np.asarray(idx, dtype=np.int64)
    dY = np.asarray(dY, dtype=np.float64)
    X_k = np.asarray(X_k, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dY_k = dY[idx]
    dW = dY_k.T @ X_k
    db = dY_k.sum(axis=0)
    dX = np.zeros((M, W.shape[1]), dtype=np.float64)
    dX[idx] = dY_k @ W
    return dW, db, dX


def backward_dwconv(dY, idx, X, Wd, pad):
    """Backward of a depthwise conv (stride 1, zero padding) with dY zeroed off the keep-set.

    Forward: Y[b,y,x,c] = sum_{u,v} X[b, y+u-pad, x+v-pad, c] Wd[u,v,c] (+ bias).
    dY, X [B,H,W,C] (channels last), Wd [ks,ks,C], idx = kept flat positions in
    [0, B*H*W).  Returns (dWd [ks,ks,C], db [C], dX [B,H,W,C]) in fp64.
    """
    dY = np.asarray(dY, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    B, H, Wi, C = dY.shape
    ks = Wd.shape[0]
    mask = np.zeros(B * H * Wi, dtype=np.float64)
    mask[np.asarray(idx, dtype=np.int64)] = 1.0
    g = dY * mask.reshape(B, H, Wi, 1)
    Xp = np.zeros((B, H + 2 * pad, Wi + 2 * pad, C), dtype=np.float64)
    Xp[:, pad:pad + H, pad:pad + Wi, :] = X
    dXp = np.zeros_like(Xp)
    dWd = np.zeros((ks, ks, C), dtype=np.float64)
    for u in range(ks):
        for v in range(ks):
            dWd[u, v, :] = (g * Xp[:, u:u + H, v:v + Wi, :]).sum(axis=(0, 1, 2))
            dXp[:, u:u + H, v:v + Wi, :] += g * Wd[u, v, :]
    db = g.sum(axis=(0, 1, 2))
    dX = dXp[:, pad:pad + H, pad:pad + Wi, :].copy()
    return dWd, db, dX


# ---------------------------------------------------------------------------------------------
# Row-wise operations between the linear layers, on the kept rows only (Alg. alg:sbp_impl with a
# row-wise f; chain rule with a shared keep-set, eq:backward_fc2_sbp_same_drop_loc).
# ---------------------------------------------------------------------------------------------
def _phi_cdf(z):
    from scipy.special import erf          # library primitive: the error function, fp64
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0)))


def gelu(z):
    """Exact GELU: z * Phi(z), Phi the standard normal distribution function."""
    z = np.asarray(z, dtype=np.float64)
    return z * _phi_cdf(z)


def gelu_grad(z):
    """d/dz [z Phi(z)] = Phi(z) + z phi(z), phi the standard normal density."""
    z = np.asarray(z, dtype=np.float64)
    return _phi_cdf(z) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def act_forward_rows(Z_k):
    """H_k = gelu(Z_k) on the cached kept rows of the pre-activation."""
    return gelu(Z_k)


def act_backward_rows(dH_k, Z_k):
    """dZ_k = dH_k * gelu'(Z_k): backward of the activation on the kept rows."""
    return np.asarray(dH_k, dtype=np.float64) * gelu_grad(Z_k)


def layernorm_rows(X_k, gamma, beta, eps):
    """Row-wise LayerNorm (biased variance), for the pins."""
    X_k = np.asarray(X_k, dtype=np.float64)
    mu = X_k.mean(axis=1, keepdims=True)
    var = ((X_k - mu) ** 2).mean(axis=1, keepdims=True)
    return (X_k - mu) / np.sqrt(var + eps) * gamma + beta


def backward_layernorm(dU_k, X_k, gamma, eps, idx, M):
    """Backward of U = LayerNorm(X) * gamma + beta restricted to the kept rows.

    dU_k [K, C]: gradient at the kept rows of U; X_k [K, C]: the kept rows of X.
    Returns dX [M, C] (zero off the keep-set), dgamma [C], dbeta [C].
    Per kept row, with xhat = (x - mean) / sqrt(var + eps) and g = dU * gamma:
    dx = (g - mean(g) - xhat * mean(g * xhat)) / sqrt(var + eps).
    """
    dU_k = np.asarray(dU_k, dtype=np.float64)
    X_k = np.asarray(X_k, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    K, C = X_k.shape
    dX = np.zeros((M, C), dtype=np.float64)
    dgamma = np.zeros(C, dtype=np.float64)
    dbeta = np.zeros(C, dtype=np.float64)
    for j in range(K):
        x = X_k[j]
        mu = x.mean()
        var = ((x - mu) ** 2).mean()
        rstd = 1.0 / np.sqrt(var + eps)
        xhat = (x - mu) * rstd
        g = dU_k[j] * gamma
        dX[idx[j]] = (g - g.mean() - xhat * (g * xhat).mean()) * rstd
        dgamma += dU_k[j] * xhat
        dbeta += dU_k[j]
    return dX, dgamma, dbeta


# ---------------------------------------------------------------------------------------------
# Down-sampling convolution, kernel p x p, stride p (section "Calculation of Convolutional Layers",
# the case s >= k): Y[b, yo, xo, o] = sum_{dy, dx, c} X[b, p yo + dy, p xo + dx, c] Wc[o, dy, dx, c] + bias[o].
# ---------------------------------------------------------------------------------------------
def backward_layerscale(dU_k, Y_k, gamma):
    """Backward of the per-channel scale U = gamma * Y on the kept rows (Alg. alg:sbp_impl with f = the scale):
    dY_k = dU_k * gamma, dgamma = sum over the kept rows of dU_k * Y_k (dropped rows contribute nothing)."""
    dU_k = np.asarray(dU_k, dtype=np.float64)
    Y_k = np.asarray(Y_k, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    return dU_k * gamma[None, :], (dU_k * Y_k).sum(axis=0)


def forward_cache_patches(X, idx, p):
    """Rows [K, p*p*C]: the p x p input patch under every kept output position, (dy, dx, c) order."""
    X = np.asarray(X)
    B, H, W, C = X.shape
    Ho, Wo = H // p, W // p
    out = np.zeros((len(idx), p * p * C), dtype=X.dtype)
    for j, f in enumerate(np.asarray(idx, dtype=np.int64)):
        b, rem = divmod(int(f), Ho * Wo)
        yo, xo = divmod(rem, Wo)
        out[j] = X[b, p * yo:p * yo + p, p * xo:p * xo + p, :].reshape(-1)
    return out


def backward_downsample(dY, idx, X, Wc, p):
    """Backward of the p x p, stride p convolution with dY zero off the kept output positions.

    dY [B, Ho, Wo, Cout]; idx: kept flat output positions b*Ho*Wo + yo*Wo + xo; X [B, H, W, C] with
    H = p Ho, W = p Wo; Wc [Cout, p, p, C].  Returns dWc [Cout, p, p, C], db [Cout], dX [B, H, W, C]
    (zero outside the patches of the kept outputs, exact inside).
    """
    dY = np.asarray(dY, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    Wc = np.asarray(Wc, dtype=np.float64)
    B, Ho, Wo, Cout = dY.shape
    dWc = np.zeros_like(Wc)
    db = np.zeros(Cout, dtype=np.float64)
    dX = np.zeros_like(X)
    for f in np.asarray(idx, dtype=np.int64):
        b, rem = divmod(int(f), Ho * Wo)
        yo, xo = divmod(rem, Wo)
        g = dY[b, yo, xo]                                   # [Cout]
        db += g
        for dy in range(p):
            for dx in range(p):
                x = X[b, p * yo + dy, p * xo + dx]          # [C]
                dWc[:, dy, dx, :] += np.outer(g, x)
                dX[b, p * yo + dy, p * xo + dx] = g @ Wc[:, dy, dx, :]
    return dWc, db, dX


def attention_scores(Q, K, scale):
    """M = Q K^T * scale and S = softmax(M) over the keys, per sample and head (``eq:attention``).

    Q, K: [B, n, h, d].  Returns M, S: [B, h, n, n].
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, n, h, d = Q.shape
    M = np.empty((B, h, n, n))
    S = np.empty((B, h, n, n))
    for b in range(B):
        for a in range(h):
            m = (Q[b, :, a, :] @ K[b, :, a, :].T) * scale
            e = np.exp(m - m.max(axis=1, keepdims=True))
            M[b, a] = m
            S[b, a] = e / e.sum(axis=1, keepdims=True)
    return M, S


def backward_attention(dA_k, Q, K, V, keep, scale):
    """Backward of scaled dot-product attention with the gradient dropout on the attention map
    ("Drop QKV": section Design Strategies; supplement ``eq:grad_qkv``, ``eq:sbp_sep_on_query``,
    ``eq:sbp_sep_on_key`` carried over to dropped keys and values).

    Q, K, V : [B, n, h, d]  the full forward tensors of one attention layer
    keep    : [B, n_k]      kept token positions of every sample (ascending)
    dA_k    : [B, n_k, h, d] gradient of the attention output at the kept tokens (zero elsewhere)
    Returns dQ_k, dK_k, dV_k : [B, n_k, h, d], the gradients at the kept tokens (zero elsewhere).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dA_k = np.asarray(dA_k, dtype=np.float64)
    keep = np.asarray(keep)
    B, n, h, d = Q.shape
    n_k = keep.shape[1]
    _, S = attention_scores(Q, K, scale)
    dQ_k = np.zeros((B, n_k, h, d))
    dK_k = np.zeros((B, n_k, h, d))
    dV_k = np.zeros((B, n_k, h, d))
    for b in range(B):
        kp = keep[b]
        for a in range(h):
            dA = np.zeros((n, d))
            dA[kp] = dA_k[b, :, a, :]                       # dA^drop = 0
            dS = dA @ V[b, :, a, :].T                       # from A = S V
            s = S[b, a]
            dM = s * (dS - (s * dS).sum(axis=1, keepdims=True))   # softmax derivative, whole rows
            mask = np.zeros((n, n))
            mask[np.ix_(kp, kp)] = 1.0
            dM = dM * mask                                  # dM^drop = 0: dropped query or dropped key
            dQ = (dM @ K[b, :, a, :]) * scale
            dK = (dM.T @ Q[b, :, a, :]) * scale
            dV = s.T @ dA
            dQ_k[b, :, a, :] = dQ[kp]
            dK_k[b, :, a, :] = dK[kp]
            dV_k[b, :, a, :] = dV[kp]                       # V's gradient is taken at the kept tokens only
    return dQ_k, dK_k, dV_k
