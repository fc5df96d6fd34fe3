"""Pins of the oracle's down-sampling convolution backward (kernel p, stride p, kept output positions):
the library's strided convolution differentiated by torch on a masked gradient, and the reduction to the
linear-layer oracle on patch rows that the paper's remark on s >= k describes."""
import numpy as np
import pytest
import torch

import oracle


def _case(B, Ho, Wo, C, Cout, p, K, seed):
    g = np.random.default_rng(seed)
    X = g.standard_normal((B, p * Ho, p * Wo, C))
    Wc = g.standard_normal((Cout, p, p, C)) * 0.3
    dY = g.standard_normal((B, Ho, Wo, Cout))
    idx = np.sort(g.choice(B * Ho * Wo, size=K, replace=False))
    return X, Wc, dY, idx


@pytest.mark.parametrize("p", [2, 4, 1])
def test_backward_downsample_is_autograd_of_the_strided_convolution_on_a_masked_gradient(p):
    B, Ho, Wo, C, Cout, K = 2, 3, 5, 4, 6, 11
    X, Wc, dY, idx = _case(B, Ho, Wo, C, Cout, p, K, 3 + p)
    xt = torch.from_numpy(X).permute(0, 3, 1, 2).contiguous().requires_grad_(True)          # NCHW
    wt = torch.from_numpy(Wc).permute(0, 3, 1, 2).contiguous().requires_grad_(True)         # [Cout, C, p, p]
    bt = torch.zeros(Cout, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.conv2d(xt, wt, bt, stride=p)                                   # [B, Cout, Ho, Wo]
    mask = np.zeros(B * Ho * Wo); mask[idx] = 1.0
    gm = torch.from_numpy(dY * mask.reshape(B, Ho, Wo, 1)).permute(0, 3, 1, 2)
    (y * gm).sum().backward()
    dWc, db, dX = oracle.backward_downsample(dY, idx, X, Wc, p)
    assert np.allclose(dX, xt.grad.permute(0, 2, 3, 1).numpy(), atol=1e-12)
    assert np.allclose(dWc, wt.grad.permute(0, 2, 3, 1).numpy(), atol=1e-12)
    assert np.allclose(db, bt.grad.numpy(), atol=1e-12)


def test_backward_downsample_reduces_to_the_linear_oracle_on_patch_rows():
    p, B, Ho, Wo, C, Cout, K = 2, 2, 4, 3, 5, 7, 9
    X, Wc, dY, idx = _case(B, Ho, Wo, C, Cout, p, K, 17)
    dWc, db, dX = oracle.backward_downsample(dY, idx, X, Wc, p)
    Xp = oracle.forward_cache_patches(X, idx, p)                                            # [K, p*p*C]
    M = B * Ho * Wo
    rW, rb, rXp = oracle.backward_linear(dY.reshape(M, Cout), idx, Xp, Wc.reshape(Cout, -1), M)
    assert np.allclose(dWc.reshape(Cout, -1), rW, atol=1e-12) and np.allclose(db, rb, atol=1e-12)
    # un-patchify the kept rows of the linear oracle's dX
    ref = np.zeros_like(X)
    for j, f in enumerate(idx):
        b, rem = divmod(int(f), Ho * Wo); yo, xo = divmod(rem, Wo)
        ref[b, p * yo:p * yo + p, p * xo:p * xo + p, :] = rXp[f].reshape(p, p, C)
    assert np.allclose(dX, ref, atol=1e-12)
    # inputs under dropped outputs get exactly zero, inputs under kept outputs the exact gradient
    kept_in = np.zeros((B, p * Ho, p * Wo), dtype=bool)
    for f in idx:
        b, rem = divmod(int(f), Ho * Wo); yo, xo = divmod(rem, Wo)
        kept_in[b, p * yo:p * yo + p, p * xo:p * xo + p] = True
    assert np.all(dX[~kept_in] == 0)
    full = oracle.backward_downsample(dY, np.arange(M), X, Wc, p)[2]
    assert np.allclose(dX[kept_in], full[kept_in], atol=1e-12)


def test_forward_cache_patches_layout():
    X = np.arange(2 * 4 * 6 * 3).reshape(2, 4, 6, 3)
    rows = oracle.forward_cache_patches(X, np.array([0, 4, 11]), 2)       # Ho, Wo = 2, 3
    assert rows.shape == (3, 12)
    assert np.array_equal(rows[0], np.concatenate([X[0, 0, 0], X[0, 0, 1], X[0, 1, 0], X[0, 1, 1]]))
    assert np.array_equal(rows[1], np.concatenate([X[0, 2, 2], X[0, 2, 3], X[0, 3, 2], X[0, 3, 3]]))   # (b=0, yo=1, xo=1)
    assert np.array_equal(rows[2], np.concatenate([X[1, 2, 4], X[1, 2, 5], X[1, 3, 4], X[1, 3, 5]]))   # (b=1, yo=1, xo=2)
