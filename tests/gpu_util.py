"""Helpers shared by the GPU parity tests: run the HIP path through the binding, the oracle on
the same stored values, and compare with the error measure the acceptance bar is written in."""
import numpy as np
import torch

import oracle
import paper_2210_00129_amd as sbp
import synth_inputs as si

# max |gpu - ref| / max |ref| bars
TOL_F32 = 1e-5          # fp32 outputs (fp32 path, and dW / db of the bf16 path: fp32 accumulators)
TOL_BF16 = 2e-2         # bf16 outputs, stated bar
TOL_BF16_TIGHT = 4.1e-3 # one RNE rounding to bf16 (8 significant bits) is <= 2^-8 = 3.9e-3 of the value's magnitude


def nerr(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got))
    denom = np.max(np.abs(ref))
    if denom == 0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / denom)


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def bits(t):
    """Raw storage of a tensor as unsigned integers (for bitwise-zero checks)."""
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()


def check_linear(X, W, dY, idx_np, dtype, flags=0, check_cache=True, inv_mode=None):
    """Runs cache + backward on the GPU and the oracle; returns the three normalised errors."""
    M = X.shape[0]
    dev = "cuda"
    idx = torch.from_numpy(np.ascontiguousarray(idx_np)).to(dev)
    Xd, Wd_, dYd = X.to(dev), W.to(dev), dY.to(dev)
    Xk = sbp.forward_cache(Xd, idx)
    if check_cache:
        assert np.array_equal(bits(Xk), bits(X[torch.from_numpy(idx_np).long()]))
    dY_in = dYd
    if flags & sbp.FLAG_DY_COMPACT:
        dY_in = dYd[idx.long()].contiguous()
    inv = None
    if inv_mode is not None:
        # the inverse map a caller may hand over: exact where rows are kept, -1 ("sampler") or
        # arbitrary numbers ("garbage") where they are dropped
        inv_np = oracle.inverse_map(idx_np, M)
        if inv_mode == "garbage":
            rng = np.random.default_rng(1)
            junk = rng.integers(-5, max(len(idx_np), 1) + 5, size=M).astype(np.int32)
            inv_np = np.where(inv_np >= 0, inv_np, junk).astype(np.int32)
        inv = torch.from_numpy(inv_np).to(dev)
    dW, db, dX = sbp.backward_linear(dY_in, idx, Xk, Wd_, M=M, flags=flags, inv=inv)
    torch.cuda.synchronize()
    rW, rb, rX = oracle.backward_linear(si.to_f64(dY), idx_np, si.to_f64(X)[idx_np], si.to_f64(W), M)
    out_tol = TOL_F32 if dtype == "f32" else TOL_BF16_TIGHT
    eW, eb = nerr(f64(dW), rW), nerr(f64(db), rb)
    if flags & sbp.FLAG_DX_COMPACT:
        eX = nerr(f64(dX), rX[idx_np])
    else:
        eX = nerr(f64(dX), rX)
        dropped = np.setdiff1d(np.arange(M), idx_np)
        assert np.all(bits(dX)[dropped] == 0), "dropped rows of dX must be +0.0 bit for bit"
    assert eW <= TOL_F32, ("dW", eW)
    assert eb <= TOL_F32, ("db", eb)
    assert eX <= out_tol, ("dX", eX)
    return eW, eb, eX
