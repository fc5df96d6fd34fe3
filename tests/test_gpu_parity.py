"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Index work must be bit-exact; gradients within 1e-5 (fp32 outputs) / 2e-2 (bf16 outputs)
of max|reference|, with a tighter bound derived from one bf16 rounding also enforced."""
import numpy as np
import pytest
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si
from gpu_util import TOL_BF16, TOL_BF16_TIGHT, TOL_F32, bits, check_linear, f64, nerr

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ sampler
@pytest.mark.parametrize("geom", [(2, 0, 4, 4), (2, 0, 14, 14), (64, 1, 14, 14), (3, 1, 5, 7), (1, 2, 3, 3),
                                  (2, 1, 1, 6), (1, 0, 1, 1), (2, 0, 50, 84), (2, 0, 100, 168)])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_sampler_bit_exact(geom, k):
    B, P, H, W = geom
    for mode in (sbp.GRID_PER_CELL, sbp.GRID_SHARED):
        for per_sample in (True, False):
            seed, stream = 12345 + k, 1000 * k + mode
            idx, inv = sbp.sample_indices(B, P, H, W, k, seed, stream, mode=mode, per_sample=per_sample,
                                          want_inv=True)
            want = oracle.sample_indices(B, P, H, W, k, seed, stream, mode=mode, per_sample=per_sample)
            assert np.array_equal(idx.cpu().numpy(), want)
            assert np.array_equal(inv.cpu().numpy(), oracle.inverse_map(want, B * (P + H * W)))


def test_sampler_full_size_detection_map_and_extreme_seeds():
    B, P, H, W, k = 2, 0, 200, 336, 2
    for seed, stream in [(0, 0), (2**64 - 1, 2**63 + 11)]:
        idx, _ = sbp.sample_indices(B, P, H, W, k, seed, stream)
        want = oracle.sample_indices(B, P, H, W, k, seed, stream)
        assert idx.numel() == 67200
        assert np.array_equal(idx.cpu().numpy(), want)


def test_sampler_golden_vectors():
    from test_oracle_sampler import _read_golden
    for (B, P, H, W, k, mode, ps, seed, stream), want in _read_golden():
        idx, _ = sbp.sample_indices(B, P, H, W, k, seed, stream, mode=mode, per_sample=bool(ps))
        assert np.array_equal(idx.cpu().numpy(), want)


@pytest.mark.parametrize("geom", [(2, 1, 14, 14), (64, 1, 14, 14), (3, 0, 5, 7), (1, 2, 1, 1), (2, 0, 100, 168), (5, 0, 17, 15)])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_random_mask_sampler_bit_exact(geom, k):
    B, P, H, W = geom
    ref = oracle.sample_indices_random(B, P, H, W, k, 11, 12)
    idx, inv = sbp.sample_indices(B, P, H, W, k, 11, 12, mode=sbp.RANDOM_MASK, want_inv=True)
    assert idx.numel() == sbp.keep_count(B, P, H, W, k, mode=sbp.RANDOM_MASK) == ref.size
    assert np.array_equal(idx.cpu().numpy(), ref)
    assert np.array_equal(inv.cpu().numpy(), oracle.inverse_map(ref, B * (P + H * W)))
    one = sbp.sample_indices(B, P, H, W, k, 11, 12, mode=sbp.RANDOM_MASK, per_sample=False)[0]
    assert np.array_equal(one.cpu().numpy(), oracle.sample_indices_random(B, P, H, W, k, 11, 12, per_sample=False))


@pytest.mark.parametrize("window,masks", [(True, True), (False, True), (True, False)])
def test_random_mask_sampler_large_maps_window_and_full_select(window, masks):
    # maps above 2048 positions: the select over a window of keys around the expected threshold, and (window switched
    # off) the full select that stands behind it; the ordered write-out from keep masks in LDS (also beyond 64 KB of
    # LDS: the 300 x 400 map) and (masks switched off) the chunked loop that stands behind it; several seeds, all keep
    # ratios, the detection-size map among them
    with sbp.options(sampler_no_window=int(not window), sampler_no_masks=int(not masks)):
        for (B, P, H, W), seeds in (((2, 0, 200, 336), ((0, 1),)), ((3, 1, 50, 84), ((5, 6), (2**64 - 1, 7), (123, 2**40))),
                                    ((1, 2, 300, 400), ((3, 4),))):
            for k in (1, 2, 3, 4):
                for seed, stream in seeds:
                    ref = oracle.sample_indices_random(B, P, H, W, k, seed, stream)
                    idx, inv = sbp.sample_indices(B, P, H, W, k, seed, stream, mode=sbp.RANDOM_MASK, want_inv=True)
                    torch.cuda.synchronize()
                    assert np.array_equal(idx.cpu().numpy(), ref)
                    assert np.array_equal(inv.cpu().numpy(), oracle.inverse_map(ref, B * (P + H * W)))


@pytest.mark.parametrize("c,k", [(2, 1), (2, 2), (3, 2), (4, 1), (4, 3)])
@pytest.mark.parametrize("geom", [(2, 1, 8, 196), (3, 0, 9, 5), (1, 0, 1, 7), (2, 2, 10, 49), (2, 0, 16, 3136)])
def test_temporal_sampler_bit_exact(geom, c, k):
    B, P, T, HW = geom
    ref = oracle.sample_indices_temporal(B, P, T, HW, c, k, 21, 22)
    idx, inv = sbp.sample_indices(B, P, T, HW, k, 21, 22, mode=sbp.TEMPORAL, want_inv=True, cell=c)
    assert idx.numel() == sbp.keep_count(B, P, T, HW, k, mode=sbp.TEMPORAL, cell=c) == ref.size
    assert np.array_equal(idx.cpu().numpy(), ref)
    assert np.array_equal(inv.cpu().numpy(), oracle.inverse_map(ref, B * (P + T * HW)))


def test_other_samplers_feed_the_linear_backward():
    # a random mask and a temporal subset are keep lists like any other: cache + backward against the oracle
    for ref in (oracle.sample_indices_random(4, 1, 14, 14, 2, 3, 4), oracle.sample_indices_temporal(2, 0, 8, 98, 4, 2, 3, 4)):
        M = 4 * 197 if ref.size == 4 * 99 else 2 * 8 * 98
        X, W, dY = si.linear_case(M, 64, 128, 9, "bf16")
        check_linear(X, W, dY, ref, "bf16")


# ------------------------------------------------------------------ forward cache
@pytest.mark.parametrize("dtype,C", [("f32", 64), ("bf16", 192), ("bf16", 768), ("bf16", 20), ("f32", 7), ("bf16", 3)])
def test_forward_cache_bit_exact(dtype, C):
    B, P, H, W = 4, 1, 14, 14
    M = B * (P + H * W)
    X = si.normal((M, C), 1.0, 5, dtype)
    idx_np = oracle.sample_indices(B, P, H, W, 2, 3, 4)
    idx = torch.from_numpy(idx_np).cuda()
    Xk = sbp.forward_cache(X.cuda(), idx)
    want = oracle.forward_cache(bits(X), idx_np)
    assert np.array_equal(bits(Xk), want)


def test_forward_cache_arbitrary_unique_rows_and_empty():
    M, C = 1000, 128
    X = si.normal((M, C), 1.0, 6, "bf16")
    rng = np.random.default_rng(0)
    idx_np = rng.permutation(M)[:333].astype(np.int32)
    Xk = sbp.forward_cache(X.cuda(), torch.from_numpy(idx_np).cuda())
    assert np.array_equal(bits(Xk), bits(X)[idx_np])
    empty = sbp.forward_cache(X.cuda(), torch.empty(0, dtype=torch.int32, device="cuda"))
    assert empty.shape == (0, C)


# ------------------------------------------------------------------ linear backward
def _grid_case(B, P, H, W, Cin, Cout, k, dtype, seed):
    M = B * (P + H * W)
    X, Wt, dY = si.linear_case(M, Cin, Cout, seed, dtype)
    idx = oracle.sample_indices(B, P, H, W, k, seed, 1000 + seed)
    return X, Wt, dY, idx


def test_linear_fp32_config():
    # B=2, 14x14 tokens, 64 -> 256, r = 0.5, seed 0
    X, W, dY, idx = _grid_case(2, 0, 14, 14, 64, 256, 2, "f32", 0)
    assert idx.size == 196
    check_linear(X, W, dY, idx, "f32")


@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(192, 768), (768, 192), (128, 512), (512, 128), (72, 200), (8, 8), (264, 136)])
def test_linear_bf16_mfma_tiles_and_ragged_tails(shape, k):
    Cin, Cout = shape
    # 6 samples of 1 + 14x14 tokens: K spans several 128-row tiles with a ragged tail
    X, W, dY, idx = _grid_case(6, 1, 14, 14, Cin, Cout, k, "bf16", 10 + k)
    check_linear(X, W, dY, idx, "bf16")


def _env(**kv):
    """Explicit overrides of the library's choices (sbp_set_option) for the duration of a block."""
    names = {"SBP_TILE": "tile", "SBP_DXBM": "dxbm", "SBP_SPLITS": "splits", "SBP_DXROWS": "dxrows", "SBP_ORDER": "order",
             "SBP_DW_SEPARATE": "dw_separate"}
    return sbp.options(**{names[k]: v for k, v in kv.items()})


@pytest.mark.parametrize("dx_rows", [256, 128, 64])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", [(192, 768), (768, 192), (512, 128), (72, 224), (8, 32), (264, 160)])
def test_linear_large_tile_engine_forced_on_ragged_shapes(shape, k, dx_rows):
    # the 256-wide engine on shapes it would not pick: partial tiles in every dimension, a partial last
    # stage in the dW contraction (K not a multiple of 32), one or several splits
    Cin, Cout = shape
    X, W, dY, idx = _grid_case(6, 1, 14, 14, Cin, Cout, k, "bf16", 20 + k)
    with _env(SBP_TILE="big", SBP_DXBM=dx_rows):
        check_linear(X, W, dY, idx, "bf16")


@pytest.mark.parametrize("splits", [1, 2, 5, 13])
@pytest.mark.parametrize("flags", [0, sbp.FLAG_DY_COMPACT, sbp.FLAG_DX_COMPACT, sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT])
def test_linear_large_tile_engine_splits_and_compact_flags(splits, flags):
    X, W, dY, idx = _grid_case(16, 1, 14, 14, 320, 288, 3, "bf16", 33)     # K = 16 * 148 = 2368 = 74 stages of 32
    assert idx.size == 2368
    with _env(SBP_TILE="big", SBP_SPLITS=splits):
        check_linear(X, W, dY, idx, "bf16", flags=flags)


@pytest.mark.parametrize("K", [1, 31, 32, 33, 95, 129, 257])
def test_linear_large_tile_engine_short_contractions(K):
    # fewer stages than the ring is deep, with and without a partial last stage
    g = np.random.default_rng(K)
    M, Cin, Cout = 300, 264, 96
    idx = np.sort(g.choice(M, size=K, replace=False)).astype(np.int32)
    X = si.normal((M, Cin), 1.0, 5, "bf16"); W = si.normal((Cout, Cin), 0.05, 6, "bf16"); dY = si.normal((M, Cout), 1.0, 7, "bf16")
    with _env(SBP_TILE="big"):
        check_linear(X, W, dY, idx, "bf16")
    with _env(SBP_TILE="big", SBP_DXBM=128):
        check_linear(X, W, dY, idx, "bf16")
    with _env(SBP_TILE="big", SBP_DXBM=64):
        check_linear(X, W, dY, idx, "bf16")


@pytest.mark.parametrize("K", [7936, 7937, 7999])
@pytest.mark.parametrize("flags", [0, sbp.FLAG_DY_COMPACT])
def test_linear_large_tile_engine_longest_split(K, flags):
    # 7936 kept rows are the longest single split (their row ids fill the LDS beside the ring); one more makes two splits
    g = np.random.default_rng(K)
    M, Cin, Cout = 9000, 264, 320
    idx = np.sort(g.choice(M, size=K, replace=False)).astype(np.int32)
    X = si.normal((M, Cin), 1.0, 15, "bf16"); W = si.normal((Cout, Cin), 0.05, 16, "bf16"); dY = si.normal((M, Cout), 1.0, 17, "bf16")
    with _env(SBP_TILE="big", SBP_SPLITS=1):
        assert sbp.backward_linear_engine(M, K, Cin, Cout, sbp.BF16) == ("mfma_large", 1 if K <= 7936 else 2)
        check_linear(X, W, dY, idx, "bf16", flags=flags)


@pytest.mark.parametrize("order", ["0,1,2", "0,2,1", "1,0,2", "1,2,0", "2,0,1", "2,1,0"])
def test_linear_general_engine_every_segment_order(order):
    # the 128-tile engine lays its three kinds of workgroups (dX tiles, dW units, zero-fill / column-sum blocks) in
    # the grid longest first; every order gives the same gradients (ragged tiles, several splits, scatter with zero fill)
    X, W, dY, idx = _grid_case(6, 1, 14, 14, 200, 136, 2, "bf16", 41)
    with _env(SBP_TILE="128x128x4x64", SBP_ORDER=order):
        check_linear(X, W, dY, idx, "bf16")
        check_linear(X, W, dY, idx, "bf16", flags=sbp.FLAG_DX_COMPACT)


@pytest.mark.parametrize("k", [1, 2, 4])
@pytest.mark.parametrize("shape", [(192, 768), (768, 192), (72, 200), (8, 8), (264, 136)])
def test_linear_general_engine_short_dx_tiles(shape, k):
    # dX tiles of 64 rows in a ring of three stages (what small layers get by themselves), forced on ragged shapes
    # with one to many stages of the contraction
    Cin, Cout = shape
    X, W, dY, idx = _grid_case(6, 1, 14, 14, Cin, Cout, k, "bf16", 50 + k)
    with _env(SBP_TILE="128x128x4x64", SBP_DXROWS=64):
        check_linear(X, W, dY, idx, "bf16")
        check_linear(X, W, dY, idx, "bf16", flags=sbp.FLAG_DX_COMPACT | sbp.FLAG_DY_COMPACT)


def test_linear_engines_agree_bit_for_bit_on_integers():
    # exact arithmetic: whichever engine, tile height or split count runs, the results are the same bits
    B, P, H, W_, Cin, Cout = 8, 1, 14, 14, 320, 288
    M = B * (P + H * W_)
    X = si.small_ints((M, Cin), -2, 2, 1, "bf16"); Wt = si.small_ints((Cout, Cin), -2, 2, 2, "bf16")
    dY = si.small_ints((M, Cout), -2, 2, 3, "bf16")
    idx = torch.from_numpy(oracle.sample_indices(B, P, H, W_, 2, 5, 9)).cuda()
    Xk = sbp.forward_cache(X.cuda(), idx)
    outs = []
    for env in (dict(SBP_TILE="128x128x4x64"), dict(SBP_TILE="128x128x4x64", SBP_DXROWS=64),
                dict(SBP_TILE="big", SBP_DXBM=256, SBP_SPLITS=1),
                dict(SBP_TILE="big", SBP_DXBM=128, SBP_SPLITS=4), dict(SBP_TILE="big", SBP_DXBM=64, SBP_SPLITS=2)):
        with _env(**env):
            outs.append([bits(t) if t.dtype == torch.bfloat16 else f64(t) for t in sbp.backward_linear(dY.cuda(), idx, Xk, Wt.cuda())])
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("inv_mode", ["sampler", "garbage"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_linear_with_caller_supplied_inverse_map(inv_mode, dtype):
    X, W, dY, idx = _grid_case(5, 1, 14, 14, 192, 320, 2, dtype, 17)
    check_linear(X, W, dY, idx, dtype, inv_mode=inv_mode)


def test_linear_single_outputs():
    # each output on its own (the launch then carries only that kind of work)
    X, W, dY, idx = _grid_case(4, 1, 14, 14, 128, 256, 2, "bf16", 19)
    M = X.shape[0]
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    full = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda())
    for i, name in enumerate(("dW", "db", "dX")):
        one = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda(), want=(name,))
        assert [o is not None for o in one] == [j == i for j in range(3)]
        assert np.array_equal(bits(one[i]), bits(full[i]))


@pytest.mark.parametrize("shape", [(20, 36), (7, 5), (64, 30)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_linear_plain_path_odd_channels(shape, dtype):
    Cin, Cout = shape
    X, W, dY, idx = _grid_case(3, 1, 6, 6, Cin, Cout, 2, dtype, 21)
    check_linear(X, W, dY, idx, dtype)


@pytest.mark.parametrize("flags", [sbp.FLAG_DY_COMPACT, sbp.FLAG_DX_COMPACT, sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_linear_compact_flags(flags, dtype):
    X, W, dY, idx = _grid_case(4, 1, 14, 14, 192, 256, 2, dtype, 31)
    check_linear(X, W, dY, idx, dtype, flags=flags)


def test_linear_vit_tiny_mlp_full_size():
    # B=64, 197 tokens, 192 -> 768 -> 192, r = 0.5, fresh mask per layer
    for (Cin, Cout, seed) in [(192, 768, 41), (768, 192, 42)]:
        X, W, dY, idx = _grid_case(64, 1, 14, 14, Cin, Cout, 2, "bf16", seed)
        assert idx.size == 6336
        check_linear(X, W, dY, idx, "bf16")


@pytest.mark.parametrize("name,Cin,Cout", [("qkv", 768, 2304), ("proj", 768, 768), ("fc1", 768, 3072), ("fc2", 3072, 768)])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_linear_vit_base_full_size(name, Cin, Cout, k):
    X, W, dY, idx = _grid_case(64, 1, 14, 14, Cin, Cout, k, "bf16", 50 + k)
    assert idx.size == [3200, 6336, 9472, 12608][k - 1]
    check_linear(X, W, dY, idx, "bf16", check_cache=(k == 2))


@pytest.mark.parametrize("geom", [(200, 336, 128, 512), (200, 336, 512, 128), (100, 168, 256, 1024), (100, 168, 1024, 256)])
def test_linear_convnext_detection_full_size(geom):
    H, W, Cin, Cout = geom
    X, Wt, dY, idx = _grid_case(2, 0, H, W, Cin, Cout, 2, "bf16", 61)
    check_linear(X, Wt, dY, idx, "bf16", check_cache=False)


@pytest.mark.parametrize("k", [1, 2, 4])
@pytest.mark.parametrize("shape", [(512, 2048), (2048, 512)])
def test_linear_convnext_stage3_pointwise_full_size(shape, k):
    # the two pointwise convs of the stage-3 block: B = 2, 50 x 84 map, 512 -> 2048 -> 512, r = 0.25 / 0.5 / 1
    # (eq:backward_fc_sbp), with whatever engine and splits the library picks for these sizes
    Cin, Cout = shape
    X, Wt, dY, idx = _grid_case(2, 0, 50, 84, Cin, Cout, k, "bf16", 70 + k)
    assert idx.size == {1: 2100, 2: 4200, 4: 8400}[k]
    check_linear(X, Wt, dY, idx, "bf16", check_cache=(k == 2))


def test_linear_integer_inputs_are_bit_exact():
    # small integers: every product and partial sum is exact in fp32, so any summation order must
    # reproduce the oracle bit for bit, and the kept / dropped halves must add up to full backprop
    B, P, H, W, Cin, Cout = 4, 0, 8, 8, 64, 128
    M = B * H * W
    X = si.small_ints((M, Cin), -3, 3, 1, "bf16")
    Wt = si.small_ints((Cout, Cin), -3, 3, 2, "bf16")
    dY = si.small_ints((M, Cout), -3, 3, 3, "bf16")
    idx = oracle.sample_indices(B, P, H, W, 2, 7, 7)
    comp = np.setdiff1d(np.arange(M), idx).astype(np.int32)
    outs = []
    for z in (idx, comp, np.arange(M, dtype=np.int32)):
        zi = torch.from_numpy(z).cuda()
        Xk = sbp.forward_cache(X.cuda(), zi)
        dW, db, dX = sbp.backward_linear(dY.cuda(), zi, Xk, Wt.cuda())
        rW, rb, rX = oracle.backward_linear(si.to_f64(dY), z, si.to_f64(X)[z], si.to_f64(Wt), M)
        assert np.array_equal(f64(dW), rW) and np.array_equal(f64(db), rb) and np.array_equal(f64(dX), rX)
        outs.append((f64(dW), f64(db), f64(dX)))
    for a, b, full in zip(*outs):
        assert np.array_equal(a + b, full)


def test_linear_dropped_rows_of_dY_are_never_used():
    X, W, dY, idx = _grid_case(4, 1, 14, 14, 128, 128, 2, "bf16", 71)
    M = X.shape[0]
    dropped = np.setdiff1d(np.arange(M), idx)
    dY2 = dY.clone()
    dY2[torch.from_numpy(dropped)] = float("nan")
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    a = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda())
    b = sbp.backward_linear(dY2.cuda(), idxd, Xk, W.cuda())
    for u, v in zip(a, b):
        assert np.array_equal(bits(u), bits(v))


def test_linear_nothing_kept_and_everything_kept():
    M, Cin, Cout = 300, 64, 96
    X, W, dY = si.linear_case(M, Cin, Cout, 81, "bf16")
    empty = torch.empty(0, dtype=torch.int32, device="cuda")
    Xk = torch.empty((0, Cin), dtype=torch.bfloat16, device="cuda")
    dW, db, dX = sbp.backward_linear(dY.cuda(), empty, Xk, W.cuda())
    assert np.all(bits(dW) == 0) and np.all(bits(db) == 0) and np.all(bits(dX) == 0)
    check_linear(X, W, dY, np.arange(M, dtype=np.int32), "bf16")


def test_linear_accumulate_flag():
    X, W, dY, idx = _grid_case(2, 1, 14, 14, 64, 128, 2, "bf16", 91)
    M = X.shape[0]
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    dW0 = torch.full((128, 64), 2.0, dtype=torch.float32, device="cuda")
    db0 = torch.full((128,), -1.0, dtype=torch.float32, device="cuda")
    dW, db, _ = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda(), flags=sbp.FLAG_ACCUMULATE_DW, dW=dW0, db=db0)
    rW, rb, _ = oracle.backward_linear(si.to_f64(dY), idx, si.to_f64(X)[idx], si.to_f64(W), M)
    assert nerr(f64(dW), rW + 2.0) <= TOL_F32 and nerr(f64(db), rb - 1.0) <= TOL_F32


@pytest.mark.parametrize("case", ["large_tile", "general", "general_many_splits", "plain_f32", "plain_odd"])
def test_linear_bf16_weight_gradient(case):
    # FLAG_DW_OUT_BF16: dW leaves as bf16 = the fp32 sum rounded to nearest even once, on every engine and through
    # every form of the split reduction; db and dX are untouched by the flag.  With FLAG_ACCUMULATE_DW the old bf16
    # values are added in fp32 and the sum is rounded again.
    B, Cin, Cout, dtype, env = {"large_tile": (16, 320, 288, "bf16", dict(SBP_TILE="big", SBP_SPLITS=3)),
                                "general": (6, 200, 136, "bf16", dict(SBP_TILE="128x128x4x64")),
                                "general_many_splits": (24, 64, 128, "bf16", {}),
                                "plain_f32": (3, 24, 40, "f32", {}),
                                "plain_odd": (3, 7, 5, "bf16", {})}[case]
    X, W, dY, idx = _grid_case(B, 1, 14, 14, Cin, Cout, 2, dtype, 97)
    M = X.shape[0]
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    with _env(**env):
        dW32, db32, dX32 = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda())
        dW16, db16, dX16 = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda(), flags=sbp.FLAG_DW_OUT_BF16)
        assert dW16.dtype == torch.bfloat16
        assert np.array_equal(bits(dW16), bits(dW32.to(torch.bfloat16)))          # one rounding of the same sum
        assert np.array_equal(bits(db16), bits(db32)) and np.array_equal(bits(dX16), bits(dX32))
        rW, _, _ = oracle.backward_linear(si.to_f64(dY), idx, si.to_f64(X)[idx], si.to_f64(W), M)
        assert nerr(f64(dW16), rW) <= TOL_BF16_TIGHT
        old = torch.full((Cout, Cin), 0.5, dtype=torch.bfloat16, device="cuda")
        acc, _, _ = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda(), flags=sbp.FLAG_DW_OUT_BF16 | sbp.FLAG_ACCUMULATE_DW,
                                        dW=old, want=("dW",))
        assert np.array_equal(bits(acc), bits((dW32 + 0.5).to(torch.bfloat16)))
    # nothing kept: zeros of the right type
    empty = torch.empty(0, dtype=torch.int32, device="cuda")
    z, _, _ = sbp.backward_linear(dY.cuda(), empty, Xk[:0], W.cuda(), flags=sbp.FLAG_DW_OUT_BF16, want=("dW", "db"))
    assert z.dtype == torch.bfloat16 and np.all(bits(z) == 0)


def test_linear_is_deterministic():
    X, W, dY, idx = _grid_case(8, 1, 14, 14, 256, 256, 2, "bf16", 95)
    idxd = torch.from_numpy(idx).cuda()
    Xk = sbp.forward_cache(X.cuda(), idxd)
    a = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda())
    b = sbp.backward_linear(dY.cuda(), idxd, Xk, W.cuda())
    for u, v in zip(a, b):
        assert np.array_equal(bits(u), bits(v))


def test_two_layer_chain_same_mask_compact():
    # eq:backward_fc2_sbp_same_drop_loc: one keep-set for both layers of an MLP; the gradient
    # stays compact between them and is scattered once at the end
    B, P, H, W, C0, C1, C2 = 4, 1, 14, 14, 64, 256, 64
    M = B * (P + H * W)
    X0, W0, _ = si.linear_case(M, C0, C1, 101, "bf16")
    X1, W1, dY2 = si.linear_case(M, C1, C2, 102, "bf16")
    idx = oracle.sample_indices(B, P, H, W, 2, 5, 5)
    idxd = torch.from_numpy(idx).cuda()
    X0k, X1k = sbp.forward_cache(X0.cuda(), idxd), sbp.forward_cache(X1.cuda(), idxd)
    dW1, db1, g = sbp.backward_linear(dY2.cuda(), idxd, X1k, W1.cuda(), flags=sbp.FLAG_DX_COMPACT)
    dW0, db0, dX0 = sbp.backward_linear(g, idxd, X0k, W0.cuda(), M=M, flags=sbp.FLAG_DY_COMPACT)
    # oracle: same chain through the full-size zero-filled gradient, with the GPU's bf16 rounding of g
    rW1, rb1, rg = oracle.backward_linear(si.to_f64(dY2), idx, si.to_f64(X1)[idx], si.to_f64(W1), M)
    assert nerr(f64(g), rg[idx]) <= TOL_BF16_TIGHT
    g_full = np.zeros((M, C1))
    g_full[idx] = f64(g)
    rW0, rb0, rX0 = oracle.backward_linear(g_full, idx, si.to_f64(X0)[idx], si.to_f64(W0), M)
    assert nerr(f64(dW0), rW0) <= TOL_F32 and nerr(f64(db0), rb0) <= TOL_F32
    assert nerr(f64(dX0), rX0) <= TOL_BF16_TIGHT
    dropped = np.setdiff1d(np.arange(M), idx)
    assert np.all(bits(dX0)[dropped] == 0)


def test_two_layer_chain_different_masks_is_the_intersection():
    # eq:keep_indices_intersect / eq:backward_fc2_sbp_different_drop_loc: layer 2 (later in the forward) drops with
    # mask Z2 and hands a full-size, zero-filled gradient to layer 1, which drops with its own mask Z1.  Layer 1's
    # weight gradient and input gradient then come from the rows in both sets only: one oracle run on the
    # intersection, fed with the exact gradient rows, must agree.
    B, P, H, W, C0, C1, C2 = 6, 1, 14, 14, 128, 256, 192
    M = B * (P + H * W)
    X0, W0, _ = si.linear_case(M, C0, C1, 201, "bf16")
    X1, W1, dY2 = si.linear_case(M, C1, C2, 202, "bf16")
    z1 = oracle.sample_indices(B, P, H, W, 2, 5, 11)
    z2 = oracle.sample_indices(B, P, H, W, 3, 5, 12)
    both = np.intersect1d(z1, z2).astype(np.int32)
    assert 0 < both.size < min(z1.size, z2.size)
    z1d, z2d = torch.from_numpy(z1).cuda(), torch.from_numpy(z2).cuda()
    X0k, X1k = sbp.forward_cache(X0.cuda(), z1d), sbp.forward_cache(X1.cuda(), z2d)
    _, _, g = sbp.backward_linear(dY2.cuda(), z2d, X1k, W1.cuda())            # [M, C1], zero off Z2
    dW0, db0, dX0 = sbp.backward_linear(g, z1d, X0k, W0.cuda())                 # Z1 applied to that gradient
    torch.cuda.synchronize()
    # oracle: layer 2 on Z2 (exact rows), then layer 1 on the intersection alone
    _, _, rg = oracle.backward_linear(si.to_f64(dY2), z2, si.to_f64(X1)[z2], si.to_f64(W1), M)
    assert nerr(f64(g), rg) <= TOL_BF16_TIGHT
    g_gpu = f64(g)                                                           # the rounded gradient layer 1 really saw
    rW0, rb0, rX0 = oracle.backward_linear(g_gpu, both, si.to_f64(X0)[both], si.to_f64(W0), M)
    assert nerr(f64(dW0), rW0) <= TOL_F32 and nerr(f64(db0), rb0) <= TOL_F32
    assert nerr(f64(dX0), rX0) <= TOL_BF16_TIGHT
    off = np.setdiff1d(np.arange(M), both)
    assert np.all(f64(dX0)[off] == 0), "rows outside the intersection carry no gradient"
    assert np.all(bits(dX0)[np.setdiff1d(np.arange(M), z1)] == 0)
    # and against the oracle's own two-mask chain from the unrounded gradient (bf16 bar: g was rounded once)
    qW0, _, qX0 = oracle.backward_linear(rg, z1, si.to_f64(X0)[z1], si.to_f64(W0), M)
    assert nerr(f64(dW0), qW0) <= TOL_BF16_TIGHT and nerr(f64(dX0), qX0) <= 2 * TOL_BF16_TIGHT


# ------------------------------------------------------------------ depthwise backward
def _check_dw(B, H, W, C, ks, k, dtype, seed, use_inv):
    X, Wd, dY = si.dwconv_case(B, H, W, C, ks, seed, dtype)
    idx_np = oracle.sample_indices(B, 0, H, W, k, seed, 77)
    idx = torch.from_numpy(idx_np).cuda()
    inv = torch.from_numpy(oracle.inverse_map(idx_np, B * H * W)).cuda() if use_inv else None
    dWd, db, dX = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv)
    rWd, rb, rX = oracle.backward_dwconv(si.to_f64(dY), idx_np, si.to_f64(X), si.to_f64(Wd), ks // 2)
    assert nerr(f64(dWd), rWd) <= TOL_F32
    assert nerr(f64(db), rb) <= TOL_F32
    assert nerr(f64(dX), rX) <= (TOL_F32 if dtype == "f32" else TOL_BF16_TIGHT)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("k", [1, 2, 4])
def test_dwconv_small(dtype, k):
    _check_dw(2, 10, 12, 64, 7, k, dtype, 111, use_inv=(k == 2))


@pytest.mark.parametrize("geom", [(1, 7, 9, 24, 7), (2, 5, 5, 8, 3), (1, 3, 20, 130, 7), (1, 16, 16, 6, 5)])
def test_dwconv_odd_shapes(geom):
    B, H, W, C, ks = geom
    _check_dw(B, H, W, C, ks, 2, "bf16", 121, use_inv=False)


@pytest.mark.parametrize("k", [1, 2, 4])
def test_dwconv_convnext_stage3_full_size(k):
    _check_dw(2, 50, 84, 512, 7, k, "bf16", 131, use_inv=True)


@pytest.mark.parametrize("geom", [(2, 50, 84, 512, 7), (1, 7, 9, 24, 7), (2, 5, 5, 8, 3)])
def test_dwconv_one_launch_two_launches_and_single_outputs_agree(geom):
    # the register-strip kernels (what channel counts that are not multiples of 8 get; forced here): dX and the weight
    # gradient normally share one launch; the two kernels on their own (switch, or a caller that wants only one of the
    # outputs) give the same dX bit for bit and the same sums up to their order
    B, H, W, C, ks = geom
    X, Wd, dY = si.dwconv_case(B, H, W, C, ks, 151, "bf16")
    idx_np = oracle.sample_indices(B, 0, H, W, 2, 151, 78)
    idx = torch.from_numpy(idx_np).cuda()
    inv = torch.from_numpy(oracle.inverse_map(idx_np, B * H * W)).cuda()
    with sbp.options(dw_strips=1):
        both = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv)
        with _env(SBP_DW_SEPARATE=1):
            two = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv)
        only_dx = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv, want=("dX",))
        only_w = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv, want=("dWd", "db"))
    assert np.array_equal(bits(both[2]), bits(two[2])) and np.array_equal(bits(both[2]), bits(only_dx[2]))
    rWd, rb, rX = oracle.backward_dwconv(si.to_f64(dY), idx_np, si.to_f64(X), si.to_f64(Wd), ks // 2)
    for got in (both, two, only_w):
        assert nerr(f64(got[0]), rWd) <= TOL_F32 and nerr(f64(got[1]), rb) <= TOL_F32
    assert nerr(f64(both[2]), rX) <= TOL_BF16_TIGHT


@pytest.mark.parametrize("geom", [(2, 50, 84, 512, 7), (1, 7, 9, 24, 7), (2, 5, 5, 8, 3), (1, 33, 70, 40, 7), (3, 4, 100, 72, 3),
                                  (1, 1, 1, 8, 7), (2, 19, 9, 264, 7)])
@pytest.mark.parametrize("k", [1, 2, 4])
def test_dwconv_lds_tiled_kernel_and_single_outputs(geom, k):
    # the LDS-tiled kernel (bf16, channel counts that are multiples of 8): ragged tiles in rows, columns and channel
    # slabs, maps smaller than a tile, every keep ratio; a caller that wants only dX or only the weight gradient gets
    # the same values bit for bit
    B, H, W, C, ks = geom
    X, Wd, dY = si.dwconv_case(B, H, W, C, ks, 161, "bf16")
    idx_np = oracle.sample_indices(B, 0, H, W, k, 161, 79)
    idx = torch.from_numpy(idx_np).cuda()
    inv = torch.from_numpy(oracle.inverse_map(idx_np, B * H * W)).cuda()
    full = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv)
    rWd, rb, rX = oracle.backward_dwconv(si.to_f64(dY), idx_np, si.to_f64(X), si.to_f64(Wd), ks // 2)
    assert nerr(f64(full[0]), rWd) <= TOL_F32 and nerr(f64(full[1]), rb) <= TOL_F32
    assert nerr(f64(full[2]), rX) <= TOL_BF16_TIGHT
    only_dx = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), inv=inv, want=("dX",))
    only_w = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda(), want=("dWd", "db"))        # inverse map built inside
    assert np.array_equal(bits(only_dx[2]), bits(full[2]))
    assert np.array_equal(f64(only_w[0]), f64(full[0])) and np.array_equal(f64(only_w[1]), f64(full[1]))
    # dropped gradient values are never used
    dY2 = dY.clone().view(-1, C)
    dY2[torch.from_numpy(np.setdiff1d(np.arange(B * H * W), idx_np))] = float("nan")
    again = sbp.backward_dwconv(dY2.view(B, H, W, C).cuda(), idx, X.cuda(), Wd.cuda(), inv=inv)
    for u, v in zip(again, full):
        assert np.array_equal(bits(u), bits(v))


def test_dwconv_single_kept_position_stamps_kernel():
    B, H, W, C, ks = 1, 9, 11, 64, 7
    X, Wd, dY = si.dwconv_case(B, H, W, C, ks, 141, "f32")
    y0, x0 = 4, 5
    idx = torch.tensor([y0 * W + x0], dtype=torch.int32, device="cuda")
    dWd, db, dX = sbp.backward_dwconv(dY.cuda(), idx, X.cuda(), Wd.cuda())
    g = f64(dY)[0, y0, x0]
    want = np.zeros((B, H, W, C))
    want[0, y0 - 3:y0 + 4, x0 - 3:x0 + 4] = f64(Wd) * g
    assert nerr(f64(dX), want) <= TOL_F32
    assert nerr(f64(dWd), f64(X)[0, y0 - 3:y0 + 4, x0 - 3:x0 + 4] * g) <= TOL_F32
    assert nerr(f64(db), g) <= TOL_F32


def test_convnext_block_chain():
    # pw2 backward -> pw1 backward (scattered, zero rows) -> depthwise backward on kept outputs
    B, H, W, C, E = 2, 12, 16, 64, 256
    M = B * H * W
    idx_np = oracle.sample_indices(B, 0, H, W, 2, 9, 9)
    idx = torch.from_numpy(idx_np).cuda()
    Xd, Wdw, _ = si.dwconv_case(B, H, W, C, 7, 151, "bf16")
    X1, W1, _ = si.linear_case(M, C, E, 152, "bf16")
    X2, W2, dY = si.linear_case(M, E, C, 153, "bf16")
    X1k, X2k = sbp.forward_cache(X1.cuda(), idx), sbp.forward_cache(X2.cuda(), idx)
    _, _, g2 = sbp.backward_linear(dY.cuda(), idx, X2k, W2.cuda(), flags=sbp.FLAG_DX_COMPACT)
    _, _, g1 = sbp.backward_linear(g2, idx, X1k, W1.cuda(), M=M, flags=sbp.FLAG_DY_COMPACT)
    dWd, db, dX = sbp.backward_dwconv(g1.view(B, H, W, C), idx, Xd.cuda(), Wdw.cuda())
    # oracle on the GPU's own (rounded) intermediate so that only the depthwise step is compared
    rWd, rb, rX = oracle.backward_dwconv(f64(g1).reshape(B, H, W, C), idx_np, si.to_f64(Xd), si.to_f64(Wdw), 3)
    assert nerr(f64(dWd), rWd) <= TOL_F32 and nerr(f64(db), rb) <= TOL_F32
    assert nerr(f64(dX), rX) <= TOL_BF16_TIGHT
    # since g1 is zero off the keep-set, a dense depthwise backward of g1 gives the same result
    full = np.arange(M, dtype=np.int32)
    fWd, fb, fX = oracle.backward_dwconv(f64(g1).reshape(B, H, W, C), full, si.to_f64(Xd), si.to_f64(Wdw), 3)
    assert np.array_equal(fWd, rWd) and np.array_equal(fX, rX)


@pytest.mark.parametrize("geom", [(2, 1, 14, 14, 4, 3), (64, 1, 14, 14, 8, 4), (2, 0, 200, 336, 4, 4), (2, 0, 50, 84, 5, 3),
                                  (3, 2, 7, 10, 9, 3), (1, 0, 1, 1, 3, 4), (2, 0, 5, 11, 2, 4), (1, 0, 13, 9, 16, 4)])
@pytest.mark.parametrize("mode", ["per_cell", "shared"])
def test_sampler_with_larger_cells_bit_exact(geom, mode):
    B, P, H, W, k, cell = geom
    m = sbp.GRID_SHARED if mode == "shared" else sbp.GRID_PER_CELL
    om = oracle.GRID_SHARED if mode == "shared" else oracle.GRID_PER_CELL
    for seed, stream, ps in ((0, 0, True), (7, 123456789, True), (2**64 - 1, 5, False)):
        idx, inv = sbp.sample_indices(B, P, H, W, k, seed, stream, mode=m, per_sample=ps, want_inv=True, cell=cell)
        torch.cuda.synchronize()
        ref = oracle.sample_indices_cells(B, P, H, W, k, cell, seed, stream, mode=om, per_sample=ps)
        got = idx.cpu().numpy()
        assert np.array_equal(got, ref)
        want_inv = np.full(B * (P + H * W), -1, dtype=np.int32)
        want_inv[ref] = np.arange(len(ref), dtype=np.int32)
        assert np.array_equal(inv.cpu().numpy(), want_inv)
