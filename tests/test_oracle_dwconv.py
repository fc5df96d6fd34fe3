"""Pins for the oracle's depthwise-conv backward on kept output positions.

The paper's convolution backward (eq:conv_grad_layer_before_sbp) with dY zeroed at
dropped positions: checked against torch's conv2d autograd on the CPU, a brute
force loop nest, and a hand case (one kept position stamps the kernel into dX).
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _case(B, H, W, C, ks, seed):
    X, Wd, dY = si.dwconv_case(B, H, W, C, ks, seed, "f32")
    return si.to_f64(X), si.to_f64(Wd), si.to_f64(dY)


def _brute(dY, keep, X, Wd, pad):
    B, H, W, C = dY.shape
    ks = Wd.shape[0]
    dWd = np.zeros_like(Wd)
    db = np.zeros(C)
    dX = np.zeros_like(X)
    for b in range(B):
        for y in range(H):
            for x in range(W):
                if not keep[b, y, x]:
                    continue
                for c in range(C):
                    g = dY[b, y, x, c]
                    db[c] += g
                    for u in range(ks):
                        for v in range(ks):
                            yy, xx = y + u - pad, x + v - pad
                            if 0 <= yy < H and 0 <= xx < W:
                                dWd[u, v, c] += g * X[b, yy, xx, c]
                                dX[b, yy, xx, c] += g * Wd[u, v, c]
    return dWd, db, dX


@pytest.mark.parametrize("ks,pad", [(7, 3), (3, 1)])
def test_matches_brute_force(ks, pad):
    B, H, W, C = 2, 6, 6, 3
    X, Wd, dY = _case(B, H, W, C, ks, 1)
    idx = oracle.sample_indices(B, 0, H, W, 2, seed=1, stream_id=0)
    keep = np.zeros(B * H * W, dtype=bool)
    keep[idx] = True
    want = _brute(dY, keep.reshape(B, H, W), X, Wd, pad)
    got = oracle.backward_dwconv(dY, idx, X, Wd, pad)
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k", [1, 2, 4])
def test_matches_conv2d_autograd_on_masked_dY(k):
    B, H, W, C, ks, pad = 2, 10, 8, 5, 7, 3
    X, Wd, dY = _case(B, H, W, C, ks, 2)
    idx = oracle.sample_indices(B, 0, H, W, k, seed=2, stream_id=7)
    mask = np.zeros(B * H * W)
    mask[idx] = 1
    g = dY * mask.reshape(B, H, W, 1)
    tX = torch.tensor(X).permute(0, 3, 1, 2).contiguous().requires_grad_(True)       # NCHW
    tW = torch.tensor(Wd).permute(2, 0, 1).unsqueeze(1).contiguous().requires_grad_(True)  # [C,1,ks,ks]
    tb = torch.zeros(C, dtype=torch.float64, requires_grad=True)
    Y = torch.nn.functional.conv2d(tX, tW, tb, stride=1, padding=pad, groups=C)
    Y.backward(torch.tensor(g).permute(0, 3, 1, 2).contiguous())
    dWd, db, dX = oracle.backward_dwconv(dY, idx, X, Wd, pad)
    np.testing.assert_allclose(dWd, tW.grad.squeeze(1).permute(1, 2, 0).numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dX, tX.grad.permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)


def test_single_kept_position_stamps_the_kernel():
    # One kept output at (4,5): dX is dY * Wd placed so that tap (u,v) lands on (4+u-3, 5+v-3)
    # (the 180-degree rotation of the paper's formula is this index reversal), and dWd is the
    # 7x7 window of X around the position times dY.
    B, H, W, C, ks, pad = 1, 9, 11, 2, 7, 3
    X, Wd, dY = _case(B, H, W, C, ks, 3)
    y0, x0 = 4, 5
    idx = np.array([y0 * W + x0], dtype=np.int32)
    dWd, db, dX = oracle.backward_dwconv(dY, idx, X, Wd, pad)
    g = dY[0, y0, x0]
    want_dX = np.zeros_like(X)
    want_dX[0, y0 - 3:y0 + 4, x0 - 3:x0 + 4, :] = Wd * g
    np.testing.assert_allclose(dX, want_dX, rtol=1e-14, atol=0)
    np.testing.assert_allclose(dWd, X[0, y0 - 3:y0 + 4, x0 - 3:x0 + 4, :] * g, rtol=1e-14, atol=0)
    np.testing.assert_array_equal(db, g)


def test_corner_position_uses_zero_padding():
    B, H, W, C, ks, pad = 1, 8, 8, 1, 7, 3
    X, Wd, dY = _case(B, H, W, C, ks, 4)
    idx = np.array([0], dtype=np.int32)        # top-left corner kept
    dWd, db, dX = oracle.backward_dwconv(dY, idx, X, Wd, pad)
    g = dY[0, 0, 0, 0]
    assert np.all(dWd[:3, :, 0] == 0) and np.all(dWd[:, :3, 0] == 0)
    np.testing.assert_allclose(dWd[3:, 3:, 0], X[0, :4, :4, 0] * g, rtol=1e-14)
    np.testing.assert_allclose(dX[0, :4, :4, 0], Wd[3:, 3:, 0] * g, rtol=1e-14)
    assert np.all(dX[0, 4:, :, 0] == 0) and np.all(dX[0, :, 4:, 0] == 0)


def test_dropped_positions_of_dY_are_ignored_and_dX_is_dense():
    B, H, W, C, ks, pad = 1, 8, 8, 2, 7, 3
    X, Wd, dY = _case(B, H, W, C, ks, 5)
    idx = oracle.sample_indices(B, 0, H, W, 2, seed=5, stream_id=0)
    a = oracle.backward_dwconv(dY, idx, X, Wd, pad)
    dY2 = dY.reshape(-1, C).copy()
    dropped = np.setdiff1d(np.arange(B * H * W), idx)
    dY2[dropped] = 1e5
    b = oracle.backward_dwconv(dY2.reshape(dY.shape), idx, X, Wd, pad)
    for u, v in zip(a, b):
        np.testing.assert_array_equal(u, v)
    # remark (a) of the paper: dropped inputs still receive gradient from kept neighbours
    assert np.all(a[2].reshape(-1, C)[dropped] != 0)


def test_full_keep_equals_plain_depthwise_backward():
    B, H, W, C, ks, pad = 1, 6, 7, 2, 7, 3
    X, Wd, dY = _case(B, H, W, C, ks, 6)
    idx = np.arange(B * H * W, dtype=np.int32)
    got = oracle.backward_dwconv(dY, idx, X, Wd, pad)
    want = _brute(dY, np.ones((B, H, W), dtype=bool), X, Wd, pad)
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, rtol=1e-12, atol=1e-12)
