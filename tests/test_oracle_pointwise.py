"""Pins of the oracle's row-wise steps (GELU, LayerNorm on the kept rows): closed forms, finite
differences of the forward definitions, and reverse-mode differentiation by torch (CPU, fp64) of the
effect of the paper's wrapper (Alg. alg:sbp_impl: gradient flows through the kept rows of f only) -- none
of which share a formula with the oracle's backward code."""
import math

import numpy as np
import pytest
import torch

import oracle


def _sbp_f(f, inputs, keep, drop, out_cols):
    # What Alg. alg:sbp_impl achieves, expressed differently: the full forward result everywhere, with the
    # gradient path cut under the dropped rows (a row mask picks between f(x) and its detached copy).
    full = f(inputs)
    assert full.shape[1] == out_cols
    kept = torch.zeros(inputs.shape[0], dtype=torch.bool)
    kept[keep] = True
    assert not kept[drop].any()
    return torch.where(kept[:, None], full, full.detach())


def _case(M, C, K, seed):
    g = np.random.default_rng(seed)
    idx = np.sort(g.choice(M, size=K, replace=False))
    drop = np.setdiff1d(np.arange(M), idx)
    return g, idx, drop


def test_gelu_closed_forms():
    assert oracle.gelu(0.0) == 0.0
    assert oracle.gelu_grad(0.0) == 0.5
    x = np.linspace(-6, 6, 241)
    # z Phi(z) - (-z) Phi(-z) = z (Phi(z) + Phi(-z)) = z
    assert np.allclose(oracle.gelu(x) - oracle.gelu(-x), x, atol=1e-15)
    # gelu'(z) + gelu'(-z) = Phi(z) + Phi(-z) = 1
    assert np.allclose(oracle.gelu_grad(x) + oracle.gelu_grad(-x), 1.0, atol=1e-15)
    assert abs(oracle.gelu(10.0) - 10.0) < 1e-20 and abs(oracle.gelu(-10.0)) < 1e-20
    # a tabulated value of the normal distribution function: Phi(1) = 0.841344746068543
    assert abs(oracle.gelu(1.0) - 0.841344746068543) < 1e-14
    # the minimum of z Phi(z) lies where Phi(z) + z phi(z) = 0, near z = -0.7517916
    assert abs(oracle.gelu_grad(-0.751791524693564)) < 1e-9


def test_gelu_matches_library_and_finite_differences():
    x = np.linspace(-5, 5, 1001)
    assert np.allclose(oracle.gelu(x), torch.nn.functional.gelu(torch.from_numpy(x)).numpy(), atol=1e-14)
    h = 1e-5
    fd = (oracle.gelu(x + h) - oracle.gelu(x - h)) / (2 * h)
    assert np.max(np.abs(fd - oracle.gelu_grad(x))) < 1e-9


def test_act_backward_rows_is_autograd_of_the_wrapped_activation():
    M, C, K = 40, 12, 17
    g, idx, drop = _case(M, C, K, 3)
    Z = torch.from_numpy(g.standard_normal((M, C)) * 2).requires_grad_(True)
    G = torch.from_numpy(g.standard_normal((M, C)))
    out = _sbp_f(torch.nn.functional.gelu, Z, torch.from_numpy(idx), torch.from_numpy(drop), C)
    (out * G).sum().backward()
    ref = Z.grad.numpy()
    got = oracle.act_backward_rows(G.numpy()[idx], Z.detach().numpy()[idx])
    assert np.allclose(got, ref[idx], atol=1e-13)
    assert np.all(ref[drop] == 0)                     # dropped rows carry no gradient
    assert np.allclose(oracle.act_forward_rows(Z.detach().numpy()[idx]), out.detach().numpy()[idx], atol=1e-14)


@pytest.mark.parametrize("C,eps", [(16, 1e-5), (7, 1e-6), (96, 1e-5)])
def test_backward_layernorm_is_autograd_of_the_wrapped_layernorm(C, eps):
    M, K = 30, 13
    g, idx, drop = _case(M, C, K, 5 + C)
    X = torch.from_numpy(g.standard_normal((M, C)) * 1.5 + 0.3).requires_grad_(True)
    gamma = torch.from_numpy(g.standard_normal(C) * 0.5 + 1.0).requires_grad_(True)
    beta = torch.from_numpy(g.standard_normal(C) * 0.1).requires_grad_(True)
    G = torch.from_numpy(g.standard_normal((M, C)))
    f = lambda x: torch.nn.functional.layer_norm(x, (C,), gamma, beta, eps)
    out = _sbp_f(f, X, torch.from_numpy(idx), torch.from_numpy(drop), C)
    (out * G).sum().backward()
    dX, dgamma, dbeta = oracle.backward_layernorm(G.numpy()[idx], X.detach().numpy()[idx], gamma.detach().numpy(), eps, idx, M)
    assert np.allclose(dX, X.grad.numpy(), atol=1e-12)
    assert np.all(dX[drop] == 0)
    assert np.allclose(dgamma, gamma.grad.numpy(), atol=1e-12)
    assert np.allclose(dbeta, beta.grad.numpy(), atol=1e-12)
    # the forward used for the pins is the library's
    assert np.allclose(oracle.layernorm_rows(X.detach().numpy()[idx], gamma.detach().numpy(), beta.detach().numpy(), eps),
                       out.detach().numpy()[idx], atol=1e-13)


def test_backward_layernorm_invariants_and_finite_differences():
    C, K, M, eps = 24, 5, 9, 1e-5
    g, idx, _ = _case(M, C, K, 11)
    Xk = g.standard_normal((K, C)); gamma = g.standard_normal(C) + 1.0; dU = g.standard_normal((K, C))
    dX, dgamma, dbeta = oracle.backward_layernorm(dU, Xk, gamma, eps, idx, M)
    # LayerNorm ignores a constant added to a row: its gradient rows sum to zero
    assert np.allclose(dX[idx].sum(axis=1), 0, atol=1e-13)
    assert np.allclose(dbeta, dU.sum(axis=0), atol=1e-13)
    # directional finite difference of sum(dU * LN(X)) along a random direction
    D = g.standard_normal((K, C)); h = 1e-6
    beta = np.zeros(C)
    f = lambda X_: np.sum(dU * oracle.layernorm_rows(X_, gamma, beta, eps))
    fd = (f(Xk + h * D) - f(Xk - h * D)) / (2 * h)
    assert abs(fd - np.sum(dX[idx] * D)) < 1e-7 * max(1.0, abs(fd))
    # a scaled copy of the row scales the gradient by 1/scale (eps negligible): homogeneity of degree -1
    dX2, _, _ = oracle.backward_layernorm(dU, 3.0 * Xk, gamma, 0.0, idx, M)
    dX1, _, _ = oracle.backward_layernorm(dU, Xk, gamma, 0.0, idx, M)
    assert np.allclose(dX2, dX1 / 3.0, atol=1e-12)


def test_mlp_branch_chain_with_one_keep_set_is_autograd_of_the_wrapped_layers():
    # LayerNorm -> fc1 -> GELU -> fc2, every layer wrapped as in Alg. alg:sbp_impl with the same keep-set:
    # composing the oracle's steps on compact rows must give autograd's gradients
    M, C, Hd, K = 26, 10, 20, 11
    g, idx, drop = _case(M, C, K, 21)
    ki, di = torch.from_numpy(idx), torch.from_numpy(drop)
    X = torch.from_numpy(g.standard_normal((M, C))).requires_grad_(True)
    gamma = torch.from_numpy(g.standard_normal(C) * 0.3 + 1).requires_grad_(True)
    beta = torch.from_numpy(g.standard_normal(C) * 0.1).requires_grad_(True)
    W1 = torch.from_numpy(g.standard_normal((Hd, C)) * 0.4).requires_grad_(True); b1 = torch.from_numpy(g.standard_normal(Hd) * 0.1).requires_grad_(True)
    W2 = torch.from_numpy(g.standard_normal((C, Hd)) * 0.4).requires_grad_(True); b2 = torch.from_numpy(g.standard_normal(C) * 0.1).requires_grad_(True)
    G = torch.from_numpy(g.standard_normal((M, C)))
    eps = 1e-5
    U = _sbp_f(lambda x: torch.nn.functional.layer_norm(x, (C,), gamma, beta, eps), X, ki, di, C)
    Z = _sbp_f(lambda u: u @ W1.t() + b1, U, ki, di, Hd)
    Hh = _sbp_f(torch.nn.functional.gelu, Z, ki, di, Hd)
    Y = _sbp_f(lambda h: h @ W2.t() + b2, Hh, ki, di, C)
    (Y * G).sum().backward()
    # the same on compact rows with the oracle
    Uk, Zk = U.detach().numpy()[idx], Z.detach().numpy()[idx]
    Hk = oracle.act_forward_rows(Zk)
    dW2, db2, dH = oracle.backward_linear(G.numpy(), idx, Hk, W2.detach().numpy(), M)
    dZk = oracle.act_backward_rows(dH[idx], Zk)
    dZ_full = np.zeros((M, Hd)); dZ_full[idx] = dZk
    dW1, db1, dU = oracle.backward_linear(dZ_full, idx, Uk, W1.detach().numpy(), M)
    dX, dgamma, dbeta = oracle.backward_layernorm(dU[idx], X.detach().numpy()[idx], gamma.detach().numpy(), eps, idx, M)
    for got, ref in ((dW2, W2.grad), (db2, b2.grad), (dW1, W1.grad), (db1, b1.grad), (dX, X.grad), (dgamma, gamma.grad), (dbeta, beta.grad)):
        assert np.allclose(got, ref.numpy(), atol=1e-11)


def test_backward_layerscale_is_autograd_of_the_wrapped_scale_and_closed_forms():
    M, C, K = 37, 11, 15
    g, idx, drop = _case(M, C, K, 21)
    Y = torch.tensor(g.normal(size=(M, C)), requires_grad=True)
    gamma = torch.tensor(g.normal(size=C) * 0.3 + 1.0, requires_grad=True)
    G = np.zeros((M, C)); G[idx] = g.normal(size=(K, C))          # the gradient arrives with zero rows at dropped positions
    out = _sbp_f(lambda y: y * gamma, Y, idx, drop, C)
    (out * torch.tensor(G)).sum().backward()
    dY_k, dgamma = oracle.backward_layerscale(G[idx], Y.detach().numpy()[idx], gamma.detach().numpy())
    np.testing.assert_allclose(dY_k, Y.grad.numpy()[idx], rtol=1e-13, atol=1e-15)
    assert np.all(Y.grad.numpy()[drop] == 0)
    np.testing.assert_allclose(dgamma, gamma.grad.numpy(), rtol=1e-12, atol=1e-14)
    # closed forms: gamma = 1 passes the gradient through; rows of ones count the kept rows
    dY1, dg1 = oracle.backward_layerscale(np.ones((K, C)), np.ones((K, C)), np.ones(C))
    assert np.all(dY1 == 1.0) and np.all(dg1 == K)
    # a planted mistake (dgamma taken against the gradient instead of the input) differs
    assert not np.allclose((G[idx] * G[idx]).sum(0), dgamma)
