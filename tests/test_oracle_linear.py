"""Pins for the oracle's linear / pointwise-conv SBP backward.

Each test ties the oracle to something other than itself: a hand-computed case,
an independent brute-force loop, torch.autograd on the CPU, or an identity the
paper states (dropped rows are zero, the weight gradient splits additively over
kept and dropped rows, keep-sets propagate / intersect through stacked layers).
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _brute_full(dY, X, W):
    """Textbook full backprop of Y = X W^T + b by explicit loops (paper: eq:backward_fc)."""
    M, Cout = dY.shape
    Cin = X.shape[1]
    dW = np.zeros((Cout, Cin))
    db = np.zeros(Cout)
    dX = np.zeros((M, Cin))
    for m in range(M):
        for o in range(Cout):
            db[o] += dY[m, o]
            for i in range(Cin):
                dW[o, i] += dY[m, o] * X[m, i]
                dX[m, i] += dY[m, o] * W[o, i]
    return dW, db, dX


def _case(M, Cin, Cout, seed):
    X, W, dY = si.linear_case(M, Cin, Cout, seed, "f32")
    return si.to_f64(X), si.to_f64(W), si.to_f64(dY)


def test_hand_computed_2x2():
    # One sample, 2x2 grid (4 rows), Cin = Cout = 2, rows 1 and 2 kept.  Values worked by hand.
    X = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float64)
    W = np.array([[1, -1], [2, 0.5]], dtype=np.float64)          # [Cout, Cin]
    dY = np.array([[1, 0], [0, 1], [2, -1], [1, 1]], dtype=np.float64)
    idx = np.array([1, 2], dtype=np.int32)
    dW, db, dX = oracle.backward_linear(dY, idx, oracle.forward_cache(X, idx), W, 4)
    np.testing.assert_array_equal(dW, [[10, 12], [-2, -2]])
    np.testing.assert_array_equal(db, [2, 0])
    np.testing.assert_array_equal(dX, [[0, 0], [2, 0.5], [0, -2.5], [0, 0]])


def test_hand_computed_order_of_idx_matters_only_for_cache():
    X = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float64)
    W = np.array([[1, -1], [2, 0.5]], dtype=np.float64)
    dY = np.array([[1, 0], [0, 1], [2, -1], [1, 1]], dtype=np.float64)
    idx = np.array([2, 1], dtype=np.int32)
    Xk = oracle.forward_cache(X, idx)
    np.testing.assert_array_equal(Xk, [[5, 6], [3, 4]])
    dW, db, dX = oracle.backward_linear(dY, idx, Xk, W, 4)
    np.testing.assert_array_equal(dW, [[10, 12], [-2, -2]])
    np.testing.assert_array_equal(dX, [[0, 0], [2, 0.5], [0, -2.5], [0, 0]])


def test_full_keep_equals_brute_force_backprop():
    M, Cin, Cout = 12, 5, 7
    X, W, dY = _case(M, Cin, Cout, 1)
    idx = np.arange(M, dtype=np.int32)
    dW, db, dX = oracle.backward_linear(dY, idx, oracle.forward_cache(X, idx), W, M)
    bW, bb, bX = _brute_full(dY, X, W)
    np.testing.assert_allclose(dW, bW, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(db, bb, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dX, bX, rtol=1e-13, atol=1e-13)


def test_full_keep_equals_autograd():
    M, Cin, Cout = 40, 9, 6
    X, W, dY = _case(M, Cin, Cout, 2)
    tX = torch.tensor(X, requires_grad=True)
    tW = torch.tensor(W, requires_grad=True)
    tb = torch.zeros(Cout, dtype=torch.float64, requires_grad=True)
    Y = torch.nn.functional.linear(tX, tW, tb)
    Y.backward(torch.tensor(dY))
    idx = np.arange(M, dtype=np.int32)
    dW, db, dX = oracle.backward_linear(dY, idx, X, W, M)
    np.testing.assert_allclose(dW, tW.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX, tX.grad.numpy(), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("r", [0.25, 0.5, 0.75])
def test_subset_equals_full_backprop_on_kept_rows_alone(r):
    B, H, Wd_, Cin, Cout = 2, 6, 8, 5, 4
    M = B * H * Wd_
    X, W, dY = _case(M, Cin, Cout, 3)
    k = oracle.k_from_ratio(r)
    idx = oracle.sample_indices(B, 0, H, Wd_, k, seed=5, stream_id=1)
    dW, db, dX = oracle.backward_linear(dY, idx, oracle.forward_cache(X, idx), W, M)
    # the sub-problem made of the kept rows only, by autograd
    tX = torch.tensor(X[idx], requires_grad=True)
    tW = torch.tensor(W, requires_grad=True)
    tb = torch.zeros(Cout, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.linear(tX, tW, tb).backward(torch.tensor(dY[idx]))
    np.testing.assert_allclose(dW, tW.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX[idx], tX.grad.numpy(), rtol=1e-12, atol=1e-12)
    # kept rows carry the exact full-backprop gradient; dropped rows are +0.0 bit for bit
    _, _, fX = _brute_full(dY, X, W)
    np.testing.assert_allclose(dX[idx], fX[idx], rtol=1e-12, atol=1e-12)
    dropped = np.setdiff1d(np.arange(M), idx)
    assert dropped.size == M - idx.size
    assert np.all(dX[dropped].view(np.uint64) == 0)


def test_dropped_rows_ignore_their_dY():
    # dY at dropped rows must not leak into any output.
    M, Cin, Cout = 16, 3, 4
    X, W, dY = _case(M, Cin, Cout, 4)
    idx = np.array([0, 3, 4, 9, 15], dtype=np.int32)
    a = oracle.backward_linear(dY, idx, X[idx], W, M)
    dY2 = dY.copy()
    dropped = np.setdiff1d(np.arange(M), idx)
    dY2[dropped] = 1e6
    b = oracle.backward_linear(dY2, idx, X[idx], W, M)
    for u, v in zip(a, b):
        np.testing.assert_array_equal(u, v)


def test_weight_gradient_splits_additively_bit_exact_on_integers():
    # dW_full = dW(Z) + dW(complement Z); exact on small integers whatever the summation order.
    M, Cin, Cout = 64, 8, 8
    X = si.to_f64(si.small_ints((M, Cin), -4, 4, 11, "f32"))
    W = si.to_f64(si.small_ints((Cout, Cin), -4, 4, 12, "f32"))
    dY = si.to_f64(si.small_ints((M, Cout), -4, 4, 13, "f32"))
    idx = oracle.sample_indices(1, 0, 8, 8, 2, seed=1, stream_id=0)
    comp = np.setdiff1d(np.arange(M), idx).astype(np.int32)
    full = np.arange(M, dtype=np.int32)
    wa, ba, xa = oracle.backward_linear(dY, idx, X[idx], W, M)
    wb, bb, xb = oracle.backward_linear(dY, comp, X[comp], W, M)
    wf, bf, xf = oracle.backward_linear(dY, full, X, W, M)
    np.testing.assert_array_equal(wa + wb, wf)
    np.testing.assert_array_equal(ba + bb, bf)
    np.testing.assert_array_equal(xa + xb, xf)
    assert np.any(wa != wf)


def test_no_rescaling_by_keep_ratio():
    # eq:sbp_formula carries 1/B only: summing fewer rows must shrink db, not rescale it.
    M, C = 8, 2
    dY = np.ones((M, C))
    X = np.ones((M, C))
    W = np.eye(C)
    idx = np.array([0, 1, 2, 3], dtype=np.int32)
    dW, db, dX = oracle.backward_linear(dY, idx, X[idx], W, M)
    np.testing.assert_array_equal(db, [4, 4])
    np.testing.assert_array_equal(dW, np.full((C, C), 4.0))


def test_same_mask_propagates_through_two_layers():
    # eq:backward_fc2_sbp_same_drop_loc: with one keep-set for both layers, running the second
    # backward on compact rows equals running it on the scattered (zero-filled) gradient.
    M, C0, C1, C2 = 32, 4, 6, 5
    X0, W0, _ = _case(M, C0, C1, 5)
    X1, W1, dY2 = _case(M, C1, C2, 6)
    idx = oracle.sample_indices(2, 0, 4, 4, 2, seed=9, stream_id=3)
    _, _, dX1 = oracle.backward_linear(dY2, idx, X1[idx], W1, M)
    dW0_a, db0_a, dX0_a = oracle.backward_linear(dX1, idx, X0[idx], W0, M)
    # closed form of the paper: dW_{i-1} = X_{i-1}^keep^T dX_{i+1}^keep W_i^T  (our layout: W1, W0)
    g = dY2[idx] @ W1
    np.testing.assert_allclose(dW0_a, g.T @ X0[idx], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX0_a[idx], g @ W0, rtol=1e-12, atol=1e-12)
    dropped = np.setdiff1d(np.arange(M), idx)
    assert np.all(dX0_a[dropped] == 0)


def test_different_masks_give_intersection():
    # eq:keep_indices_intersect / eq:backward_fc2_sbp_different_drop_loc
    M, C0, C1, C2 = 32, 4, 6, 5
    X0, W0, _ = _case(M, C0, C1, 7)
    X1, W1, dY2 = _case(M, C1, C2, 8)
    z_hi = oracle.sample_indices(2, 0, 4, 4, 2, seed=1, stream_id=1)
    z_lo = oracle.sample_indices(2, 0, 4, 4, 2, seed=1, stream_id=2)
    both = np.intersect1d(z_hi, z_lo).astype(np.int32)
    assert 0 < both.size < z_hi.size
    _, _, dX1 = oracle.backward_linear(dY2, z_hi, X1[z_hi], W1, M)
    dW0, db0, dX0 = oracle.backward_linear(dX1, z_lo, X0[z_lo], W0, M)
    # single run over the intersection with the un-dropped upstream gradient
    g_full = dY2 @ W1
    dW0_i, db0_i, dX0_i = oracle.backward_linear(g_full, both, X0[both], W0, M)
    np.testing.assert_allclose(dW0, dW0_i, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db0, db0_i, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dX0, dX0_i, rtol=1e-12, atol=1e-12)


def test_forward_cache_is_row_gather():
    X = np.arange(20, dtype=np.float64).reshape(5, 4)
    idx = np.array([4, 0, 2], dtype=np.int32)
    np.testing.assert_array_equal(oracle.forward_cache(X, idx), X[[4, 0, 2]])
    inv = oracle.inverse_map(idx, 5)
    np.testing.assert_array_equal(inv, [1, -1, 2, -1, 0])
