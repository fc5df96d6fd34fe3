"""GPU parity of the row-group layout of the cached rows (SBP_LAYOUT_KMAJOR / SBP_FLAG_XK_KMAJOR): the cache written by
sbp_forward_cache_batch is compared bit for bit with the layout's definition, and the linear backward that reads it
with the oracle and, bit for bit, with the same call on the row-major cache (the layout changes how X_k reaches the
matrix cores, not the order of any sum)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si
from gpu_util import TOL_BF16_TIGHT, TOL_F32, bits, f64, nerr

pytestmark = pytest.mark.gpu
KM = sbp.FLAG_XK_KMAJOR


def _kmajor_reference(Xk_rows):
    """[K, C] -> [ceil(K / 8), C, 8] with zero rows appended: element (j, c) at [j // 8, c, j % 8]."""
    K, C = Xk_rows.shape
    G = (K + 7) // 8
    pad = torch.zeros((G * 8, C), dtype=Xk_rows.dtype)
    pad[:K] = Xk_rows
    return pad.view(G, 8, C).permute(0, 2, 1).contiguous()


@pytest.mark.parametrize("B,P,H,W,C,k", [(3, 1, 14, 14, 192, 2), (2, 0, 9, 7, 8, 1), (5, 1, 14, 14, 776, 3), (1, 0, 2, 2, 64, 1),
                                         (64, 1, 14, 14, 768, 2)])
def test_forward_cache_in_row_groups_is_the_layout_definition(B, P, H, W, C, k):
    M = B * (P + H * W)
    X = si.normal((M, C), 1.0, 7, "bf16")
    idx_np = oracle.sample_indices(B, P, H, W, k, 3, 9)
    idx = torch.from_numpy(idx_np).cuda()
    (Xt,) = sbp.forward_cache_batch([X.cuda()], [idx], layout=sbp.LAYOUT_KMAJOR)
    torch.cuda.synchronize()
    ref = _kmajor_reference(X[torch.from_numpy(idx_np).long()])
    assert Xt.shape == ref.shape
    assert np.array_equal(bits(Xt), bits(ref))           # padding rows are +0 bit for bit


def test_forward_cache_batch_mixes_layouts_per_call_via_two_calls_and_shares_a_launch_per_layout():
    # four tensors of a block in one call, all in row groups: equal to four single calls
    B, P, H, W = 4, 1, 14, 14
    M = B * (P + H * W)
    idx_np = oracle.sample_indices(B, P, H, W, 2, 5, 1)
    idx = torch.from_numpy(idx_np).cuda()
    Xs = [si.normal((M, C), 1.0, 20 + i, "bf16") for i, C in enumerate((64, 256, 72, 1024))]
    outs = sbp.forward_cache_batch([x.cuda() for x in Xs], [idx] * 4, layout=sbp.LAYOUT_KMAJOR)
    torch.cuda.synchronize()
    for x, o in zip(Xs, outs):
        assert np.array_equal(bits(o), bits(_kmajor_reference(x[torch.from_numpy(idx_np).long()])))


def _case(B, P, H, W, Cin, Cout, k, seed, ints=False):
    M = B * (P + H * W)
    if ints:
        X = si.small_ints((M, Cin), -2, 2, seed, "bf16"); Wt = si.small_ints((Cout, Cin), -2, 2, seed + 1, "bf16")
        dY = si.small_ints((M, Cout), -2, 2, seed + 2, "bf16")
    else:
        X, Wt, dY = si.linear_case(M, Cin, Cout, seed, "bf16")
    idx = oracle.sample_indices(B, P, H, W, k, seed, 77)
    return M, X, Wt, dY, idx


def _both_layouts(M, X, Wt, dY, idx_np, flags=0, opts=None):
    idx = torch.from_numpy(idx_np).cuda()
    Xd, dYd, Wd = X.cuda(), dY.cuda(), Wt.cuda()
    (Xr,) = sbp.forward_cache_batch([Xd], [idx])
    (Xt,) = sbp.forward_cache_batch([Xd], [idx], layout=sbp.LAYOUT_KMAJOR)
    dY_in = dYd[idx.long()].contiguous() if flags & sbp.FLAG_DY_COMPACT else dYd
    with sbp.options(**(opts or {})):
        rows = sbp.backward_linear(dY_in, idx, Xr, Wd, M=M, flags=flags)
        grp = sbp.backward_linear(dY_in, idx, Xt, Wd, M=M, flags=flags | KM)
    torch.cuda.synchronize()
    return rows, grp


@pytest.mark.parametrize("shape,opts", [
    ((16, 1, 14, 14, 320, 288, 2), dict(tile="big")),                 # large-tile engine, ragged tiles, partial last stage
    ((16, 1, 14, 14, 512, 256, 3), dict(tile="big", splits=5)),       # several splits, each starting on a row group
    ((16, 1, 14, 14, 264, 160, 1), dict(tile="big", dxbm=64)),
    ((64, 1, 14, 14, 768, 768, 2), dict()),                           # ViT-Base proj at full size, the engine chosen by itself
    ((6, 1, 14, 14, 192, 768, 2), dict()),                            # general engine: the cache is copied back to rows first
    ((3, 0, 9, 7, 72, 40, 2), dict()),
])
def test_linear_backward_reads_row_groups(shape, opts):
    B, P, H, W, Cin, Cout, k = shape
    M, X, Wt, dY, idx = _case(B, P, H, W, Cin, Cout, k, 31)
    rows, grp = _both_layouts(M, X, Wt, dY, idx, opts=opts)
    rW, rb, rX = oracle.backward_linear(si.to_f64(dY), idx, si.to_f64(X)[idx], si.to_f64(Wt), M)
    assert nerr(f64(grp[0]), rW) <= TOL_F32
    assert nerr(f64(grp[1]), rb) <= TOL_F32
    assert nerr(f64(grp[2]), rX) <= TOL_BF16_TIGHT
    for a, b in zip(rows, grp):                     # same products, same order of every sum
        assert np.array_equal(bits(a), bits(b))


@pytest.mark.parametrize("flags", [sbp.FLAG_DY_COMPACT, sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT, sbp.FLAG_DW_OUT_BF16])
def test_row_groups_with_compact_gradients_and_bf16_dw_on_integers(flags):
    # exactly representable inputs: every partial sum is exact, so the result must equal the oracle's bit for bit
    M, X, Wt, dY, idx = _case(16, 1, 14, 14, 320, 288, 2, 41, ints=True)
    rows, grp = _both_layouts(M, X, Wt, dY, idx, flags=flags, opts=dict(tile="big"))
    rW, rb, rX = oracle.backward_linear(si.to_f64(dY), idx, si.to_f64(X)[idx], si.to_f64(Wt), M)
    if flags & sbp.FLAG_DW_OUT_BF16:       # the exact sum, rounded once to bf16
        assert np.array_equal(f64(grp[0]), f64(torch.from_numpy(rW).to(torch.bfloat16)))
    else:
        assert np.array_equal(f64(grp[0]), rW)
    assert np.array_equal(f64(grp[1]), rb)
    assert np.array_equal(f64(grp[2]), rX[idx] if flags & sbp.FLAG_DX_COMPACT else rX)


@pytest.mark.parametrize("forced", [True, False])
def test_batched_call_reads_row_groups(forced):
    shapes = [(64, 1, 14, 14, 768, 2304, 2), (64, 1, 14, 14, 768, 768, 2)] if not forced else \
             [(16, 1, 14, 14, 320, 288, 3), (16, 1, 14, 14, 288, 320, 2), (6, 1, 14, 14, 264, 160, 1)]
    layers_r, layers_g, cases = [], [], []
    for i, sh in enumerate(shapes):
        M, X, Wt, dY, idx_np = _case(*sh, seed=50 + i)
        idx = torch.from_numpy(idx_np).cuda()
        Xd = X.cuda()
        (Xr,) = sbp.forward_cache_batch([Xd], [idx])
        (Xt,) = sbp.forward_cache_batch([Xd], [idx], layout=sbp.LAYOUT_KMAJOR)
        common = dict(dY=dY.cuda(), idx=idx, W=Wt.cuda(), M=M)
        layers_r.append(dict(common, X_k=Xr, flags=0))
        layers_g.append(dict(common, X_k=Xt, flags=KM))
        cases.append((M, X, Wt, dY, idx_np))
    with sbp.options(**({"tile": "big"} if forced else {})):
        out_r = sbp.backward_linear_batch(layers_r)
        out_g = sbp.backward_linear_batch(layers_g)
    torch.cuda.synchronize()
    for (M, X, Wt, dY, idx_np), r, g in zip(cases, out_r, out_g):
        rW, rb, rX = oracle.backward_linear(si.to_f64(dY), idx_np, si.to_f64(X)[idx_np], si.to_f64(Wt), M)
        assert nerr(f64(g[0]), rW) <= TOL_F32
        assert nerr(f64(g[1]), rb) <= TOL_F32
        assert nerr(f64(g[2]), rX) <= TOL_BF16_TIGHT
        for a, b in zip(r, g):
            assert np.array_equal(bits(a), bits(b))
