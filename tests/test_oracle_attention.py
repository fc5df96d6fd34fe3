"""Pins of the attention-backward oracle (gradient dropout on the attention map, "Drop QKV").

The oracle is checked against things other than itself:
  * with every token kept it must equal the library's autograd of softmax attention;
  * with dropped tokens it must equal the library's autograd of the FULL attention whose gradient
    of the attention map is multiplied by the keep mask on its way back (a hook on M) and whose
    output gradient is zero at the dropped tokens;
  * an element-by-element evaluation of the defining sums on a tiny case;
  * structure: a key nobody kept contributes nothing, the kept entries of dM are those of the
    exact backward, the row sums of the exact dM vanish;
  * planted mistakes (transposed dK, a dropped softmax row term, a row sum over kept keys only)
    are caught by the same comparisons.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


def _case(B, n, h, d, n_k, seed):
    qkv, dA = si.attention_case(B, n, h, d, seed, "f32")
    x = si.to_f64(qkv).reshape(B, n, 3, h, d)
    Q, K, V = x[:, :, 0], x[:, :, 1], x[:, :, 2]
    rng = np.random.default_rng(seed)
    keep = np.stack([np.sort(rng.choice(n, size=n_k, replace=False)) for _ in range(B)])
    dA_full = si.to_f64(dA).reshape(B, n, h, d)
    dA_k = np.stack([dA_full[b, keep[b]] for b in range(B)])
    return Q, K, V, keep, dA_k


def _autograd_masked(Q, K, V, keep, dA_k, scale):
    """Library autograd through the full attention with the keep mask applied to the gradient of M."""
    B, n, h, d = Q.shape
    q = torch.tensor(Q).permute(0, 2, 1, 3).clone().requires_grad_(True)
    k = torch.tensor(K).permute(0, 2, 1, 3).clone().requires_grad_(True)
    v = torch.tensor(V).permute(0, 2, 1, 3).clone().requires_grad_(True)
    mask = torch.zeros(B, 1, n, n, dtype=torch.float64)
    G = torch.zeros(B, h, n, d, dtype=torch.float64)
    for b in range(B):
        kp = torch.tensor(keep[b])
        mask[b, 0][kp[:, None], kp[None, :]] = 1.0
        G[b][:, kp, :] = torch.tensor(dA_k[b]).permute(1, 0, 2)
    m = torch.matmul(q, k.transpose(-1, -2)) * scale
    m.register_hook(lambda g: g * mask)
    a = torch.matmul(torch.softmax(m, dim=-1), v)
    (a * G).sum().backward()
    out = []
    for t in (q.grad, k.grad, v.grad):
        t = t.permute(0, 2, 1, 3).numpy()
        out.append(t)
    return out


@pytest.mark.parametrize("B,n,h,d", [(2, 17, 3, 8), (1, 50, 2, 64)])
def test_all_kept_equals_library_autograd(B, n, h, d):
    Q, K, V, keep, dA_k = _case(B, n, h, d, n, 5)
    scale = 1.0 / math.sqrt(d)
    dQ, dK, dV = oracle.backward_attention(dA_k, Q, K, V, keep, scale)
    q = torch.tensor(Q, requires_grad=True)
    k = torch.tensor(K, requires_grad=True)
    v = torch.tensor(V, requires_grad=True)
    a = torch.nn.functional.scaled_dot_product_attention(q.permute(0, 2, 1, 3), k.permute(0, 2, 1, 3), v.permute(0, 2, 1, 3))
    (a.permute(0, 2, 1, 3) * torch.tensor(dA_k)).sum().backward()
    for got, ref in ((dQ, q.grad), (dK, k.grad), (dV, v.grad)):
        np.testing.assert_allclose(got, ref.numpy(), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("B,n,h,d,n_k", [(2, 17, 3, 8, 9), (2, 50, 2, 64, 25), (1, 33, 1, 32, 1)])
def test_dropped_tokens_equal_autograd_with_masked_map_gradient(B, n, h, d, n_k):
    Q, K, V, keep, dA_k = _case(B, n, h, d, n_k, 11)
    scale = 1.0 / math.sqrt(d)
    dQ, dK, dV = oracle.backward_attention(dA_k, Q, K, V, keep, scale)
    gq, gk, gv = _autograd_masked(Q, K, V, keep, dA_k, scale)
    for b in range(B):
        kp = keep[b]
        drop = np.setdiff1d(np.arange(n), kp)
        np.testing.assert_allclose(dQ[b], gq[b, kp], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dK[b], gk[b, kp], rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dV[b], gv[b, kp], rtol=1e-10, atol=1e-12)     # V's gradient: kept rows are taken
        assert np.all(gq[b, drop] == 0) and np.all(gk[b, drop] == 0)             # dropped queries / keys get nothing


def test_tiny_case_element_by_element():
    B, n, h, d, n_k = 1, 5, 1, 3, 3
    Q, K, V, keep, dA_k = _case(B, n, h, d, n_k, 3)
    scale = 0.7
    dQ, dK, dV = oracle.backward_attention(dA_k, Q, K, V, keep, scale)
    kp = list(keep[0])
    q, k, v = Q[0, :, 0], K[0, :, 0], V[0, :, 0]
    S = [[0.0] * n for _ in range(n)]
    for i in range(n):
        e = [math.exp(scale * sum(q[i][c] * k[j][c] for c in range(d))) for j in range(n)]
        z = sum(e)
        S[i] = [x / z for x in e]
    dA = {kp[a]: dA_k[0, a, 0] for a in range(n_k)}
    dQe = np.zeros((n_k, d)); dKe = np.zeros((n_k, d)); dVe = np.zeros((n_k, d))
    for a, i in enumerate(kp):
        dS_row = [sum(dA[i][c] * v[l][c] for c in range(d)) for l in range(n)]      # all keys
        delta = sum(S[i][l] * dS_row[l] for l in range(n))
        for bb, j in enumerate(kp):
            dM = S[i][j] * (dS_row[j] - delta)
            for c in range(d):
                dQe[a, c] += scale * dM * k[j][c]
                dKe[bb, c] += scale * dM * q[i][c]
                dVe[bb, c] += S[i][j] * dA[i][c]
    np.testing.assert_allclose(dQ[0, :, 0], dQe, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dK[0, :, 0], dKe, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dV[0, :, 0], dVe, rtol=1e-12, atol=1e-14)


def test_row_term_identity_and_structure():
    """The softmax row term sum_l S_il dS_il equals dA_i . A_i (A = S V): the kept-only form of the
    backward (what a kernel can compute from kept tensors and the forward's row statistics) is the
    same function.  Also: the scores are a softmax (rows sum to one)."""
    B, n, h, d, n_k = 2, 21, 2, 16, 10
    Q, K, V, keep, dA_k = _case(B, n, h, d, n_k, 7)
    scale = 1.0 / math.sqrt(d)
    M, S = oracle.attention_scores(Q, K, scale)
    np.testing.assert_allclose(S.sum(-1), 1.0, rtol=0, atol=1e-13)
    dQ, dK, dV = oracle.backward_attention(dA_k, Q, K, V, keep, scale)
    for b in range(B):
        kp = keep[b]
        for a in range(h):
            lse = np.log(np.exp(M[b, a]).sum(-1))
            A = S[b, a] @ V[b, :, a]
            Qk, Kk, Vk, Ak = Q[b, kp, a], K[b, kp, a], V[b, kp, a], A[kp]
            Skk = np.exp(Qk @ Kk.T * scale - lse[kp][:, None])
            dA = dA_k[b, :, a]
            dM = Skk * (dA @ Vk.T - (dA * Ak).sum(-1, keepdims=True))
            np.testing.assert_allclose(dQ[b, :, a], dM @ Kk * scale, rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(dK[b, :, a], dM.T @ Qk * scale, rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(dV[b, :, a], Skk.T @ dA, rtol=1e-10, atol=1e-12)


def test_planted_mistakes_are_caught():
    B, n, h, d, n_k = 1, 19, 2, 8, 9
    Q, K, V, keep, dA_k = _case(B, n, h, d, n_k, 13)
    scale = 1.0 / math.sqrt(d)
    gq, gk, gv = _autograd_masked(Q, K, V, keep, dA_k, scale)
    kp = keep[0]
    _, S = oracle.attention_scores(Q, K, scale)

    def variant(kind):
        outs = []
        for a in range(h):
            s = S[0, a]
            dA = np.zeros((n, d)); dA[kp] = dA_k[0, :, a]
            dS = dA @ V[0, :, a].T
            if kind == "row_sum_over_kept_keys":
                row = (s[:, kp] * dS[:, kp]).sum(1, keepdims=True)
            elif kind == "no_row_term":
                row = 0.0
            else:
                row = (s * dS).sum(1, keepdims=True)
            dM = s * (dS - row)
            mask = np.zeros((n, n)); mask[np.ix_(kp, kp)] = 1
            dM = dM * mask
            dK = (dM @ Q[0, :, a] if kind == "dk_not_transposed" else dM.T @ Q[0, :, a]) * scale
            dQ = dM @ K[0, :, a] * scale
            outs.append((dQ[kp], dK[kp]))
        return outs

    for kind in ("row_sum_over_kept_keys", "no_row_term", "dk_not_transposed"):
        outs = variant(kind)
        bad = any(not np.allclose(outs[a][0], gq[0, kp, a], rtol=1e-8, atol=1e-10) or
                  not np.allclose(outs[a][1], gk[0, kp, a], rtol=1e-8, atol=1e-10) for a in range(h))
        assert bad, kind
    outs = variant("exact")
    for a in range(h):
        np.testing.assert_allclose(outs[a][0], gq[0, kp, a], rtol=1e-10, atol=1e-12)
