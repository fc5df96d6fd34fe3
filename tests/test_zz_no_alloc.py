"""The entry point that allocates nothing (sbp_backward_linear_static, for callers that cannot call hipMalloc):
called through the C ABI with preallocated outputs, it must give what sbp_backward_linear gives with a caller's
workspace - same kernels, same plan, so the same bits - and match the CPU oracle to the usual bars; twice in a
row on one GPU, the second call smaller, so that whatever the first call left in the library's fixed scratch
array cannot leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si
from gpu_util import TOL_BF16_TIGHT, TOL_F32, bits, f64, nerr
from paper_2210_00129_amd import _lib

pytestmark = pytest.mark.gpu


def _case(B, Cin, Cout, k, seed):
    P, H, W = 1, 14, 14
    M = B * (P + H * W)
    X, Wt, dY = si.linear_case(M, Cin, Cout, seed, "bf16")
    idx = oracle.sample_indices(B, P, H, W, k, seed, 3000 + seed)
    return M, X, Wt, dY, idx


def _run_both(M, X, Wt, dY, idx_np, flags=0):
    L = _lib.lib()
    dev = "cuda"
    Cout, Cin = Wt.shape
    K = idx_np.size
    idx = torch.from_numpy(idx_np).to(dev)
    Xd, Wd, dYd = X.to(dev), Wt.to(dev), dY.to(dev)
    Xk = sbp.forward_cache(Xd, idx)
    inv = torch.from_numpy(oracle.inverse_map(idx_np, M)).to(dev)
    rows = K if flags & sbp.FLAG_DX_COMPACT else M
    dY_in = dYd[idx.long()].contiguous() if flags & sbp.FLAG_DY_COMPACT else dYd
    # reference: the existing entry point with a workspace of the caller's
    rW, rb, rX = sbp.backward_linear(dY_in, idx, Xk, Wd, M=M, flags=flags, inv=inv)
    # the static entry point: outputs preallocated (poisoned), nothing but pointers and sizes cross the ABI
    dW = torch.full((Cout, Cin), float("nan"), dtype=torch.float32, device=dev)
    db = torch.full((Cout,), float("nan"), dtype=torch.float32, device=dev)
    dX = torch.full((rows, Cin), float("nan"), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = L.sbp_backward_linear_static(dY_in.data_ptr(), idx.data_ptr(), inv.data_ptr(), Xk.data_ptr(), Wd.data_ptr(), M, K,
                                      Cin, Cout, sbp.BF16, dW.data_ptr(), db.data_ptr(), dX.data_ptr(), flags,
                                      torch.cuda.current_stream().cuda_stream)
    assert st == 0, L.sbp_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for got, ref in ((dW, rW), (db, rb), (dX, rX)):
        assert np.array_equal(bits(got), bits(ref))
    oW, ob, oX = oracle.backward_linear(si.to_f64(dY), idx_np, si.to_f64(X)[idx_np], si.to_f64(Wt), M)
    assert nerr(f64(dW), oW) <= TOL_F32 and nerr(f64(db), ob) <= TOL_F32
    assert nerr(f64(dX), oX[idx_np] if flags & sbp.FLAG_DX_COMPACT else oX) <= TOL_BF16_TIGHT
    if not flags & sbp.FLAG_DX_COMPACT:
        assert np.all(bits(dX)[np.setdiff1d(np.arange(M), idx_np)] == 0)


def test_static_entry_point_two_calls_in_a_row_second_smaller():
    assert sbp.static_scratch_bytes() == 48 << 20
    # first call: a ViT-Base-size layer on the large-tile engine (several dW splits: about 27 MB of the scratch array)
    _run_both(*_case(64, 768, 3072, 2, 5))
    # second call, smaller in every dimension, on the general engine, leaving most of the first call's partial sums
    # in the array behind its own
    _run_both(*_case(6, 192, 136, 1, 6))
    # and once more with compact rows on both sides (no inverse map in the scratch array at all)
    _run_both(*_case(6, 192, 136, 3, 7), flags=sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT)


def test_static_entry_point_refuses_sizes_beyond_its_scratch_array():
    L = _lib.lib()
    M, K, Cin, Cout = 65536, 65536, 4096, 4096
    assert sbp.backward_linear_workspace(M, K, Cin, Cout, sbp.BF16) > sbp.static_scratch_bytes()
    p = ctypes.c_void_p(4096)
    st = L.sbp_backward_linear_static(p, p, None, p, p, M, K, Cin, Cout, sbp.BF16, p, p, p, 0, None)
    assert st == -5 and b"static buffer" in L.sbp_last_error()
