"""GPU parity of the attention backward on the kept tokens ("Drop QKV") against the fp64 oracle, through
the C ABI.  The forward (attention output and the row log-sum-exp over all keys) is the model's, computed
by the library routines of the input module; the oracle gets the full q, k, v and the keep sets, the HIP
path only the kept rows."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si
from gpu_util import TOL_BF16, TOL_F32, f64, nerr

pytestmark = pytest.mark.gpu


def _keep_sets(B, n, n_k, seed):
    g = np.random.default_rng(seed)
    return np.stack([np.sort(g.choice(n, size=n_k, replace=False)) for _ in range(B)])


def _run(B, n, h, d, keep, dtype, seed, scale=None):
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    n_k = keep.shape[1]
    qkv, dA = si.attention_case(B, n, h, d, seed, dtype)
    A64, lse64 = si.attention_forward(qkv, B, n, h, d, scale)
    tdt = si.torch_dtype(dtype)
    A = A64.to(tdt)                                   # a forward stores its output in the model's type
    lse = lse64.to(torch.float32)
    rows = torch.from_numpy((np.arange(B)[:, None] * n + keep).reshape(-1)).long()
    dA_k = dA[rows].contiguous()
    out = sbp.backward_attention(qkv[rows].contiguous().cuda(), A[rows].contiguous().cuda(), dA_k.cuda(),
                                 lse[rows].contiguous().cuda(), B, h, d, scale)
    torch.cuda.synchronize()
    x = si.to_f64(qkv).reshape(B, n, 3, h, d)
    ref = oracle.backward_attention(si.to_f64(dA_k).reshape(B, n_k, h, d), x[:, :, 0], x[:, :, 1], x[:, :, 2], keep, scale)
    got = f64(out).reshape(B, n_k, 3, h, d)
    return [nerr(got[:, :, i], ref[i]) for i in range(3)]


CASES = [  # B, n, h, d, n_k
    (2, 197, 3, 64, 99),      # ViT at r = 0.5: 4 blocks of 32 with a ragged tail
    (1, 197, 2, 64, 197),     # everything kept: 7 blocks
    (2, 50, 2, 64, 1),        # a single kept token
    (2, 70, 2, 64, 32),       # exactly one block
    (1, 70, 1, 64, 33),
    (1, 300, 1, 64, 256),     # the largest size of the matrix-core kernel at d = 64
    (1, 300, 1, 64, 257),     # one more: tiled over chunks of 128 tokens (three chunks, the last with one token)
    (1, 600, 2, 64, 512),     # four full chunks
    (1, 1100, 1, 64, 1024),
    (1, 400, 1, 32, 390),
    (1, 300, 1, 128, 161),
    (2, 120, 3, 32, 100),
    (1, 140, 2, 128, 100),
    (2, 40, 2, 16, 21),       # d = 16: plain kernel
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,n,h,d,n_k", CASES)
def test_attention_backward_matches_oracle(B, n, h, d, n_k, dtype):
    errs = _run(B, n, h, d, _keep_sets(B, n, n_k, 5), dtype, 3)
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    assert max(errs) <= tol, errs


def test_engine_choice():
    assert sbp.backward_attention_engine(99, 64, sbp.BF16) == "mfma"
    assert sbp.backward_attention_engine(256, 64, sbp.BF16) == "mfma"
    assert sbp.backward_attention_engine(257, 64, sbp.BF16) == "mfma_tiled"
    assert sbp.backward_attention_engine(4096, 128, sbp.BF16) == "mfma_tiled"
    assert sbp.backward_attention_engine(99, 64, sbp.F32) == "plain"
    assert sbp.backward_attention_engine(99, 16, sbp.BF16) == "plain"


def test_plain_kernel_on_bf16_matches_oracle():
    with sbp.options(attn="plain"):
        assert sbp.backward_attention_engine(99, 64, sbp.BF16) == "plain"
        errs = _run(2, 197, 3, 64, _keep_sets(2, 197, 99, 7), "bf16", 9)
    assert sbp.backward_attention_engine(99, 64, sbp.BF16) == "mfma"
    assert max(errs) <= TOL_BF16, errs


def test_grid_sampler_keep_sets_and_other_scale():
    # keep sets as the library's sampler draws them (class token + 2x2 grid cells), a non-default scale
    B, P, H, W, h, d = 3, 1, 14, 14, 2, 64
    n = P + H * W
    idx = sbp.sample_indices(B, P, H, W, 2, 17, 4)[0].cpu().numpy().astype(np.int64)
    n_k = idx.size // B
    keep = (idx.reshape(B, n_k) - np.arange(B)[:, None] * n)
    assert keep.min() >= 0 and keep.max() < n
    errs = _run(B, n, h, d, keep, "bf16", 21, scale=0.09)
    assert max(errs) <= TOL_BF16, errs


def test_bench_size_vit_base():
    # the size bench.py times: B = 64, 12 heads of 64, 99 of 197 tokens kept
    B, n, h, d, n_k = 64, 197, 12, 64, 99
    errs = _run(B, n, h, d, _keep_sets(B, n, n_k, 1), "bf16", 2)
    assert max(errs) <= TOL_BF16, errs


def test_feeds_the_qkv_linear_backward():
    # dqkv_k is the compact dY of the qkv projection: its backward from these rows equals the oracle's
    B, n, h, d, n_k, C = 2, 50, 2, 64, 25, 64
    keep = _keep_sets(B, n, n_k, 3)
    scale = 1.0 / math.sqrt(d)
    qkv, dA = si.attention_case(B, n, h, d, 4, "bf16")
    A64, lse64 = si.attention_forward(qkv, B, n, h, d, scale)
    rows_np = (np.arange(B)[:, None] * n + keep).reshape(-1)
    rows = torch.from_numpy(rows_np).long()
    X, Wt, _ = si.linear_case(B * n, C, 3 * h * d, 6, "bf16")
    dqkv = sbp.backward_attention(qkv[rows].contiguous().cuda(), A64.to(torch.bfloat16)[rows].contiguous().cuda(),
                                  dA[rows].contiguous().cuda(), lse64.float()[rows].contiguous().cuda(), B, h, d, scale)
    idx = torch.from_numpy(rows_np.astype(np.int32)).cuda()
    Xk = sbp.forward_cache(X.cuda(), idx)
    dW, db, dX = sbp.backward_linear(dqkv, idx, Xk, Wt.cuda(), M=B * n, flags=sbp.FLAG_DY_COMPACT)
    torch.cuda.synchronize()
    dY_full = np.zeros((B * n, 3 * h * d))
    dY_full[rows_np] = f64(dqkv)                      # the same rounded rows the kernel consumed
    rW, rb, rX = oracle.backward_linear(dY_full, rows_np, si.to_f64(X)[rows_np], si.to_f64(Wt), B * n)
    assert nerr(f64(dW), rW) <= TOL_F32 and nerr(f64(db), rb) <= TOL_F32 and nerr(f64(dX), rX) <= TOL_BF16


def test_empty_and_errors():
    e = torch.empty((0, 3 * 2 * 64), dtype=torch.bfloat16, device="cuda")
    a = torch.empty((0, 2 * 64), dtype=torch.bfloat16, device="cuda")
    l = torch.empty((0, 2), dtype=torch.float32, device="cuda")
    assert sbp.backward_attention(e, a, a, l, 1, 2, 64, 0.125).shape == (0, 384)
    q = torch.zeros((4, 3 * 2 * 24), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(Exception):
        sbp.backward_attention(q, q[:, :48], q[:, :48], torch.zeros((4, 2), device="cuda"), 1, 2, 24, 0.2)   # d = 24


@pytest.mark.parametrize("B,n,h,d,n_k", [(2, 197, 3, 64, 99), (1, 197, 2, 64, 197), (2, 50, 2, 64, 1), (1, 70, 1, 64, 33),
                                         (1, 300, 1, 64, 256), (2, 120, 3, 32, 100), (1, 140, 2, 128, 100)])
def test_tiled_kernel_at_sizes_the_single_workgroup_kernel_also_serves(B, n, h, d, n_k):
    # the two matrix-core kernels do the same products on the same rounded probabilities: both within the bar, and
    # close to each other
    keep = _keep_sets(B, n, n_k, 11)
    with sbp.options(attn="tiled"):
        assert sbp.backward_attention_engine(n_k, d, sbp.BF16) == "mfma_tiled"
        errs = _run(B, n, h, d, keep, "bf16", 13)
    assert max(errs) <= TOL_BF16, errs
    with sbp.options(attn="whole"):
        assert sbp.backward_attention_engine(n_k, d, sbp.BF16) == "mfma"
        errs_w = _run(B, n, h, d, keep, "bf16", 13)
    assert max(errs_w) <= TOL_BF16, errs_w
