"""GPU parity of the row-wise steps between the linear layers (activation, LayerNorm backward on the
kept rows) and of a whole MLP branch run on compact rows, against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si
from gpu_util import TOL_BF16_TIGHT, TOL_F32, bits, f64, nerr

pytestmark = pytest.mark.gpu


def _tol(dtype):
    return TOL_F32 if dtype == "f32" else TOL_BF16_TIGHT


# ------------------------------------------------------------------ activation
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(6336, 3072), (197, 768), (33, 20), (5, 7), (1, 1), (1000, 8)])
def test_act_forward_and_backward_rows(shape, dtype):
    K, C = shape
    Z = si.normal((K, C), 2.0, 11, dtype)              # pre-activations over several standard deviations
    dH = si.normal((K, C), 1.0, 12, dtype)
    H = sbp.act_forward_rows(Z.cuda())
    dZ = sbp.act_backward_rows(dH.cuda(), Z.cuda())
    torch.cuda.synchronize()
    assert nerr(f64(H), oracle.act_forward_rows(si.to_f64(Z))) <= _tol(dtype)
    assert nerr(f64(dZ), oracle.act_backward_rows(si.to_f64(dH), si.to_f64(Z))) <= _tol(dtype)


def test_act_tails_extremes_in_place_and_empty():
    # values where erf saturates, exact zeros, signed zero, and the in-place form of the backward
    z = torch.tensor([[-40.0, -9.0, -3.0, -0.75, -0.0, 0.0, 0.75, 3.0, 9.0, 40.0, 1e-30, -1e-30]], dtype=torch.float32)
    g = torch.full_like(z, 2.0)
    H = sbp.act_forward_rows(z.cuda())
    buf = g.cuda().clone()
    out = sbp.act_backward_rows(buf, z.cuda(), out=buf)
    assert out.data_ptr() == buf.data_ptr()
    torch.cuda.synchronize()
    assert np.allclose(f64(H), oracle.gelu(z.double().numpy()), atol=2e-6, rtol=1e-6)
    assert np.allclose(f64(out), 2.0 * oracle.gelu_grad(z.double().numpy()), atol=2e-6, rtol=1e-6)
    assert float(H[0, 0]) == 0.0 and float(H[0, -3]) == 40.0          # saturated ends are exact
    e = torch.empty((0, 16), dtype=torch.bfloat16, device="cuda")
    assert sbp.act_forward_rows(e).shape == (0, 16)
    assert sbp.act_backward_rows(e, e).shape == (0, 16)


# ------------------------------------------------------------------ LayerNorm backward
def _ln_case(M, K, C, dtype, seed):
    g = np.random.default_rng(seed)
    idx = np.sort(g.choice(M, size=K, replace=False)).astype(np.int32)
    X = si.normal((M, C), 1.5, seed + 1, dtype) + 0.25
    X = X.to(si.torch_dtype(dtype))
    dU = si.normal((K, C), 1.0, seed + 2, dtype)
    gamma = (si.normal((C,), 0.3, seed + 3, "f32") + 1.0).float()
    return idx, X, dU, gamma


def _check_ln(M, K, C, dtype, seed, flags=0, inv_mode=None, eps=1e-5):
    idx, X, dU, gamma = _ln_case(M, K, C, dtype, seed)
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    inv = None
    if inv_mode:
        inv_np = oracle.inverse_map(idx, M)
        if inv_mode == "garbage":
            junk = np.random.default_rng(2).integers(-5, K + 5, size=M).astype(np.int32)
            inv_np = np.where(inv_np >= 0, inv_np, junk).astype(np.int32)
        inv = torch.from_numpy(inv_np).cuda()
    dgamma, dbeta, dX = sbp.backward_layernorm(dU.cuda(), Xk, gamma.cuda(), eps, idxd, M, inv=inv, flags=flags)
    torch.cuda.synchronize()
    rX, rg, rb = oracle.backward_layernorm(si.to_f64(dU), si.to_f64(X)[idx], gamma.double().numpy(), eps, idx, M)
    assert nerr(f64(dgamma), rg) <= TOL_F32
    assert nerr(f64(dbeta), rb) <= TOL_F32
    if flags & sbp.FLAG_DX_COMPACT:
        assert dX.shape == (K, C)
        assert nerr(f64(dX), rX[idx]) <= _tol(dtype)
    elif C == 1:
        # one channel: x - mean(x) = 0, the exact gradient is 0 and rstd = eps^-1/2 = 316 multiplies the
        # rounding residue of g - mean(g): an absolute bound takes the place of the normalised one
        assert np.all(rX == 0) and np.max(np.abs(f64(dX))) <= 64 * 2.0 ** -24 * 316 * 4
    else:
        assert nerr(f64(dX), rX) <= _tol(dtype)
        dropped = np.setdiff1d(np.arange(M), idx)
        assert np.all(bits(dX)[dropped] == 0), "dropped rows of dX must be +0.0 bit for bit"


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("C", [768, 192, 96, 8, 1024, 1032, 4096, 4104, 20, 7, 1])
def test_backward_layernorm_channel_counts(C, dtype):
    # multiples of 8 up to 4096 take the one-wavefront-per-row kernel (1, 2, 4 or 8 groups per lane),
    # everything else the plain kernels
    _check_ln(M=300, K=157, C=C, dtype=dtype, seed=C)


@pytest.mark.parametrize("K", [0, 1, 3, 8, 9, 300])
def test_backward_layernorm_row_counts(K):
    _check_ln(M=300, K=K, C=64, dtype="bf16", seed=40 + K)


@pytest.mark.parametrize("inv_mode", [None, "sampler", "garbage"])
@pytest.mark.parametrize("flags", [0, sbp.FLAG_DX_COMPACT])
def test_backward_layernorm_inverse_map_and_compact_output(flags, inv_mode):
    _check_ln(M=1000, K=431, C=192, dtype="bf16", seed=7, flags=flags, inv_mode=inv_mode)


def test_backward_layernorm_vit_base_full_size_accumulate_and_determinism():
    B, P, H, W, C = 64, 1, 14, 14, 768
    M = B * (P + H * W)
    idx = oracle.sample_indices(B, P, H, W, 2, 3, 4)
    K = idx.size
    X = si.normal((M, C), 1.0, 1, "bf16"); dU = si.normal((K, C), 1.0, 2, "bf16")
    gamma = (si.normal((C,), 0.2, 3, "f32") + 1.0).float()
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    a = sbp.backward_layernorm(dU.cuda(), Xk, gamma.cuda(), 1e-6, idxd, M)
    b = sbp.backward_layernorm(dU.cuda(), Xk, gamma.cuda(), 1e-6, idxd, M)
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    rX, rg, rb = oracle.backward_layernorm(si.to_f64(dU), si.to_f64(X)[idx], gamma.double().numpy(), 1e-6, idx, M)
    assert nerr(f64(a[0]), rg) <= TOL_F32 and nerr(f64(a[1]), rb) <= TOL_F32 and nerr(f64(a[2]), rX) <= TOL_BF16_TIGHT
    # accumulate: the parameter gradients are added to what the buffers hold
    dg = torch.full((C,), 2.0, device="cuda"); db = torch.full((C,), -1.0, device="cuda")
    sbp.backward_layernorm(dU.cuda(), Xk, gamma.cuda(), 1e-6, idxd, M, flags=sbp.FLAG_ACCUMULATE_DW, dgamma=dg, dbeta=db,
                           want=("dgamma", "dbeta"))
    assert nerr(f64(dg), rg + 2.0) <= TOL_F32 and nerr(f64(db), rb - 1.0) <= TOL_F32


# ------------------------------------------------------------------ a whole MLP branch on compact rows
@pytest.mark.parametrize("geom", [(4, 1, 14, 14, 64, 256), (16, 1, 14, 14, 768, 3072)])
def test_mlp_branch_backward_on_compact_rows(geom):
    # LayerNorm -> fc1 -> GELU -> fc2 with one keep-set (eq:backward_fc2_sbp_same_drop_loc): cached are the
    # kept rows of x, of u = LN(x) and of z = fc1(u); the backward runs [K, .] -> [K, .] and scatters once
    B, P, H, W, C, Hd = geom
    M = B * (P + H * W)
    idx = oracle.sample_indices(B, P, H, W, 2, 9, 9)
    K = idx.size
    Xf = si.normal((M, C), 1.0, 1, "bf16")
    gamma = (si.normal((C,), 0.2, 2, "f32") + 1.0).float(); beta = si.normal((C,), 0.1, 3, "f32").float()
    W1 = si.normal((Hd, C), C ** -0.5, 4, "bf16"); b1 = si.normal((Hd,), 0.1, 5, "f32")
    W2 = si.normal((C, Hd), Hd ** -0.5, 6, "bf16")
    dY = si.normal((M, C), 1.0, 7, "bf16")
    eps = 1e-6
    # forward on the CPU in fp64 from the stored values, rounded to bf16 where the model would store them
    x64 = si.to_f64(Xf)
    U = torch.from_numpy(oracle.layernorm_rows(x64, gamma.double().numpy(), beta.double().numpy(), eps)).to(torch.bfloat16)
    Z = torch.from_numpy(si.to_f64(U) @ si.to_f64(W1).T + b1.double().numpy()).to(torch.bfloat16)
    idxd = torch.from_numpy(idx).cuda()
    inv = torch.from_numpy(oracle.inverse_map(idx, M)).cuda()
    Xk, Uk, Zk = (sbp.forward_cache(t.cuda(), idxd) for t in (Xf, U, Z))

    # GPU: compact pipeline
    Hk = sbp.act_forward_rows(Zk)
    dW2, db2, dHk = sbp.backward_linear(dY.cuda(), idxd, Hk, W2.cuda(), M=M, flags=sbp.FLAG_DX_COMPACT, inv=inv)
    dZk = sbp.act_backward_rows(dHk, Zk, out=dHk)
    dW1, db1, dUk = sbp.backward_linear(dZk, idxd, Uk, W1.cuda(), M=M, flags=sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT, inv=inv)
    dgamma, dbeta, dX = sbp.backward_layernorm(dUk, Xk, gamma.cuda(), eps, idxd, M, inv=inv)
    torch.cuda.synchronize()

    # oracle: the same chain; each step starts from the GPU's stored (bf16) result of the step before, so every
    # comparison tests one step at the tolerance of one rounding
    Hk_ref = oracle.act_forward_rows(si.to_f64(Z)[idx])
    assert nerr(f64(Hk), Hk_ref) <= TOL_BF16_TIGHT
    rW2, rb2, rH = oracle.backward_linear(si.to_f64(dY), idx, f64(Hk), si.to_f64(W2), M)
    assert nerr(f64(dW2), rW2) <= TOL_F32 and nerr(f64(db2), rb2) <= TOL_F32
    # dHk was overwritten in place by dZk: check the product of the two steps against the oracle's
    rZk = oracle.act_backward_rows(rH[idx], si.to_f64(Z)[idx])
    assert nerr(f64(dZk), rZk) <= 2 * TOL_BF16_TIGHT                       # two roundings: dH_k, then dZ_k
    dZ_full = np.zeros((M, Hd)); dZ_full[idx] = f64(dZk)
    rW1, rb1, rU = oracle.backward_linear(dZ_full, idx, si.to_f64(U)[idx], si.to_f64(W1), M)
    assert nerr(f64(dW1), rW1) <= TOL_F32 and nerr(f64(db1), rb1) <= TOL_F32
    assert nerr(f64(dUk), rU[idx]) <= TOL_BF16_TIGHT
    rX, rg, rbeta = oracle.backward_layernorm(f64(dUk), x64[idx], gamma.double().numpy(), eps, idx, M)
    assert nerr(f64(dgamma), rg) <= TOL_F32 and nerr(f64(dbeta), rbeta) <= TOL_F32
    assert nerr(f64(dX), rX) <= TOL_BF16_TIGHT
    dropped = np.setdiff1d(np.arange(M), idx)
    assert np.all(bits(dX)[dropped] == 0)

    # the pipeline that scatters after every layer gives the same bits
    _, _, dH_full = sbp.backward_linear(dY.cuda(), idxd, Hk, W2.cuda(), M=M, inv=inv)
    dZ_s = sbp.act_backward_rows(dH_full[idxd.long()].contiguous(), Zk)
    assert torch.equal(dZ_s, dZk)
    dZ_scat = torch.zeros((M, Hd), dtype=torch.bfloat16, device="cuda"); dZ_scat[idxd.long()] = dZ_s
    dW1s, db1s, dU_full = sbp.backward_linear(dZ_scat, idxd, Uk, W1.cuda(), M=M, inv=inv)
    assert torch.equal(dW1s, dW1) and torch.equal(db1s, db1) and torch.equal(dU_full[idxd.long()], dUk)


# ------------------------------------------------------------------ layer scale
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(8400, 512), (6336, 768), (33, 24), (17, 7), (1, 1), (5000, 8)])
def test_backward_layerscale_matches_oracle(shape, dtype):
    K, C = shape
    dU = si.normal((K, C), 1.0, 31, dtype)
    Y = si.normal((K, C), 1.0, 32, dtype)
    gamma = (si.normal((C,), 0.1, 33, "f32") + 0.5).float()
    dg, dY = sbp.backward_layerscale(dU.cuda(), Y.cuda(), gamma.cuda())
    torch.cuda.synchronize()
    rY, rg = oracle.backward_layerscale(si.to_f64(dU), si.to_f64(Y), si.to_f64(gamma))
    assert nerr(f64(dY), rY) <= _tol(dtype)
    assert nerr(f64(dg), rg) <= TOL_F32


def test_backward_layerscale_in_place_accumulate_empty_and_exact():
    K, C = 300, 64
    dU = si.small_ints((K, C), -3, 3, 41, "bf16").cuda()
    Y = si.small_ints((K, C), -3, 3, 42, "bf16").cuda()
    gamma = torch.full((C,), 2.0, device="cuda")
    ref_Y, ref_g = oracle.backward_layerscale(si.to_f64(dU), si.to_f64(Y), si.to_f64(gamma))
    buf = dU.clone()
    dg = torch.ones(C, device="cuda")
    out_g, out_Y = sbp.backward_layerscale(buf, Y, gamma, flags=sbp.FLAG_ACCUMULATE_DW, dgamma=dg, dY=buf)   # in place, dgamma +=
    torch.cuda.synchronize()
    assert out_Y.data_ptr() == buf.data_ptr()
    assert np.array_equal(f64(out_Y), ref_Y) and np.array_equal(f64(out_g), ref_g + 1.0)      # small integers: exact
    e = torch.empty((0, C), dtype=torch.bfloat16, device="cuda")
    g0, y0 = sbp.backward_layerscale(e, e, gamma)
    torch.cuda.synchronize()
    assert y0.shape == (0, C) and np.all(f64(g0) == 0)
