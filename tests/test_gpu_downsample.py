"""GPU parity of the down-sampling layer path (kernel p, stride p convolution on kept output positions):
patch gather, linear backward on patch rows, patch scatter with zero fill, against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si
from gpu_util import TOL_BF16_TIGHT, TOL_F32, bits, f64, nerr

pytestmark = pytest.mark.gpu


def _keep(B, Ho, Wo, k, seed):
    return oracle.sample_indices(B, 0, Ho, Wo, k, seed, 31)


@pytest.mark.parametrize("wide", [False, True])
@pytest.mark.parametrize("dtype,C", [("bf16", 128), ("bf16", 8), ("bf16", 3), ("f32", 5), ("f32", 64)])
@pytest.mark.parametrize("p", [2, 4, 1])
def test_patch_gather_and_scatter_are_bit_exact(p, dtype, C, wide):
    # wide: the kernels with 64-bit unit numbers, which otherwise only tensors of 2^32 units and more would reach
    sbp.set_option("patch_wide", int(wide))
    try:
        _patch_gather_and_scatter(p, dtype, C)
    finally:
        sbp.set_option("patch_wide", None)


def _patch_gather_and_scatter(p, dtype, C):
    B, Ho, Wo = 3, 6, 10
    H, W = p * Ho, p * Wo
    X = si.normal((B, H, W, C), 1.0, 7, dtype)
    idx = _keep(B, Ho, Wo, 2, 5)
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache_patches(X.cuda(), idxd, p)
    ref = oracle.forward_cache_patches(bits(X), idx, p)
    assert np.array_equal(bits(Xk), ref)
    # scatter the same rows back: kept patches return, everything else is +0
    for inv in (None, torch.from_numpy(oracle.inverse_map(idx, B * Ho * Wo)).cuda()):
        back = sbp.scatter_patches(Xk, idxd, (B, H, W, C), p, inv=inv)
        want = np.zeros_like(bits(X))
        for f in idx:
            b, rem = divmod(int(f), Ho * Wo); yo, xo = divmod(rem, Wo)
            want[b, p * yo:p * yo + p, p * xo:p * xo + p] = bits(X)[b, p * yo:p * yo + p, p * xo:p * xo + p]
        assert np.array_equal(bits(back), want)


def test_patch_steps_empty_and_full_keep_sets():
    B, Ho, Wo, C, p = 2, 4, 4, 16, 2
    X = si.normal((B, 2 * Ho, 2 * Wo, C), 1.0, 3, "bf16").cuda()
    none = torch.empty(0, dtype=torch.int32, device="cuda")
    assert sbp.forward_cache_patches(X, none, p).shape == (0, 4 * C)
    z = sbp.scatter_patches(torch.empty((0, 4 * C), dtype=torch.bfloat16, device="cuda"), none, X.shape, p)
    assert np.all(bits(z) == 0)
    every = torch.arange(B * Ho * Wo, dtype=torch.int32, device="cuda")
    back = sbp.scatter_patches(sbp.forward_cache_patches(X, every, p), every, X.shape, p)
    assert torch.equal(back, X)


@pytest.mark.parametrize("geom", [(2, 6, 10, 16, 32, 2, "bf16"), (1, 5, 7, 24, 40, 2, "f32"), (2, 3, 4, 8, 16, 4, "bf16"),
                                  (2, 100, 168, 128, 256, 2, "bf16")])
def test_downsample_layer_backward(geom):
    B, Ho, Wo, C, Cout, p, dtype = geom
    H, W = p * Ho, p * Wo
    X = si.normal((B, H, W, C), 1.0, 11, dtype)
    Wc = si.normal((Cout, p, p, C), (p * p * C) ** -0.5, 12, dtype)
    dY = si.normal((B, Ho, Wo, Cout), 1.0, 13, dtype)
    idx = _keep(B, Ho, Wo, 2, 17)
    K, Mo = idx.size, B * Ho * Wo
    idxd = torch.from_numpy(idx).cuda()
    inv = torch.from_numpy(oracle.inverse_map(idx, Mo)).cuda()
    Xk = sbp.forward_cache_patches(X.cuda(), idxd, p)
    dW, db, dXp = sbp.backward_linear(dY.cuda().reshape(Mo, Cout), idxd, Xk, Wc.cuda().reshape(Cout, p * p * C), M=Mo,
                                      flags=sbp.FLAG_DX_COMPACT, inv=inv)
    dX = sbp.scatter_patches(dXp, idxd, (B, H, W, C), p, inv=inv)
    torch.cuda.synchronize()
    rW, rb, rX = oracle.backward_downsample(si.to_f64(dY), idx, si.to_f64(X), si.to_f64(Wc), p)
    assert nerr(f64(dW).reshape(Cout, p, p, C), rW) <= TOL_F32
    assert nerr(f64(db), rb) <= TOL_F32
    assert nerr(f64(dX), rX) <= (TOL_F32 if dtype == "f32" else TOL_BF16_TIGHT)
    # input pixels under dropped outputs (exact gradient all zero) hold +0.0 bit for bit
    assert np.count_nonzero(bits(dX)[np.all(rX == 0, axis=-1)]) == 0
