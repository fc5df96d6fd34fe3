"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before touching the GPU (none of these calls launches a kernel)."""
import ctypes
import os
import re

import pytest

import oracle
import paper_2210_00129_amd as sbp
from paper_2210_00129_amd import _lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "sbp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sbp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) == 32
    handle = ctypes.CDLL(_lib.LIB_PATH)
    for n in names:
        assert hasattr(handle, n), n
    assert sorted(_lib.PROTOTYPES) == names


def test_status_strings():
    L = _lib.lib()
    assert L.sbp_status_string(0) == b"ok"
    for code in range(-8, 0):
        assert L.sbp_status_string(code) not in (b"", b"ok", b"unknown status")
    assert L.sbp_status_string(-99) == b"unknown status"


@pytest.mark.parametrize("r", [0.05, 0.125, 0.25, 0.3, 0.375, 0.5, 0.62, 0.75, 0.875, 0.9, 1.0])
def test_k_from_ratio_matches_oracle(r):
    assert sbp.k_from_ratio(r) == oracle.k_from_ratio(r)


def test_k_from_ratio_rejects_bad_input():
    for r in (0.0, -0.5, 1.01, float("nan")):
        with pytest.raises(sbp.SbpError) as e:
            sbp.k_from_ratio(r)
        assert e.value.status == -3
    with pytest.raises(sbp.SbpError) as e:
        sbp.k_from_ratio(0.5, cell=5)
    assert e.value.status == -2
    assert sbp.k_from_ratio(0.5, cell=3) == oracle.k_from_ratio(0.5, 3) == 5      # round-half-up(4.5)
    assert sbp.k_from_ratio(0.25, cell=4) == oracle.k_from_ratio(0.25, 4) == 4


@pytest.mark.parametrize("geom", [(2, 0, 14, 14), (64, 1, 14, 14), (2, 0, 200, 336), (2, 0, 5, 7), (1, 2, 3, 3),
                                  (3, 1, 1, 6), (1, 0, 1, 1), (2, 0, 50, 84), (2, 0, 800, 1333)])
def test_keep_count_matches_oracle(geom):
    B, P, H, W = geom
    for k in (1, 2, 3, 4):
        assert sbp.keep_count(B, P, H, W, k) == oracle.keep_count(B, P, H, W, k)


@pytest.mark.parametrize("geom", [(2, 1, 14, 14), (2, 0, 200, 336), (2, 0, 5, 7), (1, 2, 3, 3), (3, 1, 1, 6), (1, 0, 1, 1),
                                  (2, 0, 50, 84), (1, 0, 13, 9)])
def test_keep_count_of_larger_cells_matches_oracle(geom):
    B, P, H, W = geom
    for cell, ks in ((3, (1, 4, 5, 9)), (4, (1, 4, 8, 16))):
        for k in ks:
            assert sbp.keep_count(B, P, H, W, k, cell=cell) == oracle.keep_count_cells(B, P, H, W, k, cell)


def _desc(**kw):
    base = dict(B=2, P=0, H=4, W=4, k=2, seed=0, stream_id=0)
    base.update(kw)
    d = sbp.make_desc(base["B"], base["P"], base["H"], base["W"], base["k"], base["seed"], base["stream_id"])
    for f in ("cell", "mode", "per_sample"):
        if f in kw:
            setattr(d, f, kw[f])
    return d


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), -2), (dict(P=-1), -2), (dict(H=0), -2), (dict(W=0), -2), (dict(cell=5), -2), (dict(cell=1), -2), (dict(cell=3, k=10), -3), (dict(cell=3, mode=2), -2),
    (dict(k=0), -3), (dict(k=5), -3), (dict(mode=7), -8), (dict(per_sample=2), -8),
    (dict(B=70000, H=200, W=200), -2),
])
def test_keep_count_rejects_bad_descriptor(kw, status):
    assert _lib.lib().sbp_keep_count(_desc(**kw)) == status
    assert _lib.lib().sbp_last_error() != b""


def test_sample_indices_argument_errors():
    L = _lib.lib()
    d = _desc()
    assert L.sbp_sample_indices(None, 16, 100, None, None) == -1
    assert L.sbp_sample_indices(d, None, 100, None, None) == -1
    assert L.sbp_sample_indices(d, 4096, 15, None, None) == -5      # K = 16
    assert b"capacity" in L.sbp_last_error()


def test_forward_cache_argument_errors():
    L = _lib.lib()
    p = 4096  # never dereferenced: validation fails first
    assert L.sbp_forward_cache(None, p, 10, 5, 8, 1, p, None) == -1
    assert L.sbp_forward_cache(p, None, 10, 5, 8, 1, p, None) == -1
    assert L.sbp_forward_cache(p, p, 10, 5, 8, 1, None, None) == -1
    assert L.sbp_forward_cache(p, p, 10, 5, 8, 9, p, None) == -4
    assert L.sbp_forward_cache(p, p, 0, 0, 8, 1, p, None) == -2
    assert L.sbp_forward_cache(p, p, 10, 11, 8, 1, p, None) == -2
    assert L.sbp_forward_cache(p, p, 10, 5, 0, 1, p, None) == -2
    assert L.sbp_forward_cache(p, p, 10, 0, 8, 1, p, None) == 0     # nothing to gather


def test_backward_linear_argument_errors():
    L = _lib.lib()
    p = 4096
    ws = L.sbp_backward_linear_workspace(100, 50, 64, 128, 1, 0)
    assert ws > 0 and ws % 256 == 0
    args = dict(dY=p, idx=p, Xk=p, W=p, M=100, K=50, Cin=64, Cout=128, dtype=1, dW=p, db=p, dX=p, ws=p * 4,
                ws_bytes=ws, flags=0)

    def call(**kw):
        a = dict(args)
        a.update(kw)
        return L.sbp_backward_linear(a["dY"], a["idx"], None, a["Xk"], a["W"], a["M"], a["K"], a["Cin"], a["Cout"],
                                     a["dtype"], a["dW"], a["db"], a["dX"], a["ws"], a["ws_bytes"], a["flags"], None)

    assert call(dY=None) == -1
    assert call(idx=None) == -1
    assert call(Xk=None) == -1
    assert call(W=None) == -1
    assert call(dtype=5) == -4
    assert call(K=101) == -2
    assert call(M=0) == -2
    assert call(Cin=0) == -2
    assert call(flags=64) == -8
    # the row-group layout of X_k exists for bf16 with Cin % 8 == 0 and a 16-byte aligned X_k only
    assert call(flags=16, dtype=0) == -8
    assert call(flags=16, Cin=60) == -8
    assert call(flags=16, Xk=p + 8) == -8
    assert L.sbp_backward_linear_workspace(100, 50, 64, 128, 1, 16) >= ws + 50 * 64 * 2   # room to copy X_k back to rows
    assert call(ws=None) == -6
    assert call(ws_bytes=ws - 1) == -6
    assert call(ws=p * 4 + 8) == -6
    assert call(dW=None, db=None, dX=None) == 0                     # nothing requested, nothing launched
    assert L.sbp_backward_linear_workspace(100, 500, 64, 128, 1, 0) == 0
    # compact dX needs no inverse map: smaller workspace
    assert L.sbp_backward_linear_workspace(100, 50, 64, 128, 1, 2) < ws


def test_backward_linear_engine_report_and_plan():
    # host logic of the plan: which kernels a shape gets, and how many partial sums of dW
    assert sbp.backward_linear_engine(100, 50, 64, 128, sbp.F32)[0] == "plain"
    assert sbp.backward_linear_engine(100, 50, 60, 36, sbp.BF16)[0] == "plain"          # channels not multiples of 8
    assert sbp.backward_linear_engine(12608, 6336, 192, 768, sbp.BF16)[0] == "mfma"     # narrower than a 256 tile
    for Cin, Cout in [(768, 2304), (768, 768), (768, 3072), (3072, 768)]:               # ViT-Base layers, r = 0.5
        name, splits = sbp.backward_linear_engine(12608, 6336, Cin, Cout, sbp.BF16)
        assert name == "mfma_large" and 2 <= splits <= 24
        # the workspace holds that many fp32 copies of dW (+ db partials + the inverse map)
        assert sbp.backward_linear_workspace(12608, 6336, Cin, Cout, sbp.BF16) >= splits * Cin * Cout * 4
    assert sbp.backward_linear_engine(12608, 6336, 768, 2320, sbp.BF16)[0] == "mfma"    # Cout not a multiple of 32
    assert sbp.backward_linear_engine(4200, 500, 512, 512, sbp.BF16)[0] == "mfma"       # too few kept rows
    with pytest.raises(ValueError):
        sbp.backward_linear_engine(100, 500, 64, 128, sbp.BF16)
    # the bf16 weight gradient is a property of the last step only: same plan, same workspace
    assert sbp.backward_linear_workspace(12608, 6336, 768, 768, sbp.BF16, sbp.FLAG_DW_OUT_BF16) == \
        sbp.backward_linear_workspace(12608, 6336, 768, 768, sbp.BF16)
    assert sbp.backward_linear_workspace(12608, 6336, 768, 768, sbp.BF16, 32) == 0      # unknown flag
    # rows of dY that byte offsets of 32 bits cannot reach: the general engine takes the shape
    assert sbp.backward_linear_engine(1 << 20, 1 << 19, 4096, 4096, sbp.BF16)[0] == "mfma"


def test_other_sampler_modes_counts_and_errors():
    for (B, P, H, W) in [(2, 1, 14, 14), (3, 0, 5, 7), (1, 0, 1, 1), (2, 0, 100, 168)]:
        for k in (1, 2, 3, 4):
            assert sbp.keep_count(B, P, H, W, k, mode=sbp.RANDOM_MASK) == B * (P + oracle.random_keep_count(H, W, k))
    for (B, P, T, HW) in [(2, 1, 8, 196), (3, 0, 9, 5), (1, 0, 1, 7), (2, 0, 10, 3)]:
        for c in (2, 3, 4):
            for k in range(1, c + 1):
                assert sbp.keep_count(B, P, T, HW, k, mode=sbp.TEMPORAL, cell=c) == B * (P + oracle.temporal_keep_frames(T, c, k) * HW)
    L = _lib.lib()
    assert L.sbp_keep_count(sbp.make_desc(2, 0, 8, 4, 1, 0, 0, mode=sbp.TEMPORAL, cell=5)) == -2
    assert L.sbp_keep_count(sbp.make_desc(2, 0, 8, 4, 4, 0, 0, mode=sbp.TEMPORAL, cell=3)) == -3
    assert L.sbp_keep_count(sbp.make_desc(2, 0, 8, 4, 2, 0, 0, mode=sbp.RANDOM_MASK, cell=3)) == -2
    assert L.sbp_keep_count(sbp.make_desc(2, 0, 8, 4, 2, 0, 0, mode=4)) == -8


def test_patch_steps_argument_errors():
    L = _lib.lib()
    p = 4096
    assert L.sbp_forward_cache_patches(p, p, 2, 8, 8, 16, 3, 10, 1, p, None) == -2      # H not a multiple of p
    assert L.sbp_forward_cache_patches(p, p, 2, 8, 8, 16, 9, 10, 1, p, None) == -2
    assert L.sbp_forward_cache_patches(p, p, 2, 8, 8, 16, 2, 33, 1, p, None) == -2      # K > B*Ho*Wo = 32
    assert L.sbp_forward_cache_patches(None, p, 2, 8, 8, 16, 2, 10, 1, p, None) == -1
    assert L.sbp_forward_cache_patches(p, p, 2, 8, 8, 16, 2, 10, 4, p, None) == -4
    assert L.sbp_forward_cache_patches(None, None, 2, 8, 8, 16, 2, 0, 1, None, None) == 0
    assert L.sbp_scatter_patches_workspace(2, 8, 8, 2) == 256                           # 32 output positions
    assert L.sbp_scatter_patches_workspace(2, 8, 8, 3) == 0
    assert L.sbp_scatter_patches(p, p, None, 2, 8, 8, 16, 2, 10, 1, p, None, 0, None) == -6   # no inv, no workspace
    assert L.sbp_scatter_patches(p, p, None, 2, 8, 8, 16, 2, 10, 1, None, p, 256, None) == -1
    assert L.sbp_scatter_patches(None, p, p, 2, 8, 8, 16, 2, 10, 1, p, None, 0, None) == -1


def test_rowwise_steps_argument_errors():
    L = _lib.lib()
    p = 4096
    assert L.sbp_act_forward_rows(p, 10, 8, 7, 0, p, None) == -4
    assert L.sbp_act_forward_rows(p, 10, 8, 1, 3, p, None) == -8
    assert L.sbp_act_forward_rows(None, 10, 8, 1, 0, p, None) == -1
    assert L.sbp_act_forward_rows(p, -1, 8, 1, 0, p, None) == -2
    assert L.sbp_act_forward_rows(None, 0, 8, 1, 0, None, None) == 0            # nothing to do
    assert L.sbp_act_backward_rows(p, None, 10, 8, 1, 0, p, None) == -1
    assert L.sbp_act_backward_rows(p, p, 10, 0, 1, 0, p, None) == -2
    ws = L.sbp_backward_layernorm_workspace(100, 50, 64, 1, 0)
    assert ws > 0 and ws % 256 == 0
    assert L.sbp_backward_layernorm_workspace(100, 50, 64, 1, 2) < ws            # compact dX: no inverse map
    assert L.sbp_backward_layernorm_workspace(100, 500, 64, 1, 0) == 0
    assert L.sbp_backward_layernorm_workspace(100, 50, 64, 1, 1) == 0            # dU is always compact: no such flag

    def ln(dU=p, Xk=p, gamma=p, eps=1e-5, idx=p, M=100, K=50, C=64, dtype=1, dg=p, db=p, dX=p, w=p * 4, wb=ws, flags=0):
        return L.sbp_backward_layernorm(dU, Xk, gamma, eps, idx, None, M, K, C, dtype, dg, db, dX, w, wb, flags, None)

    assert ln(dU=None) == -1 and ln(Xk=None) == -1 and ln(gamma=None) == -1 and ln(idx=None) == -1
    assert ln(dtype=9) == -4 and ln(K=101) == -2 and ln(C=0) == -2 and ln(flags=1) == -8
    assert ln(eps=-1.0) == -2
    assert ln(w=None) == -6 and ln(wb=ws - 1) == -6 and ln(w=p * 4 + 16) == -6
    assert ln(dg=None, db=None, dX=None) == 0


def test_backward_attention_argument_errors_and_engine():
    L = _lib.lib()
    p = ctypes.c_void_p(256)     # never dereferenced: validation comes first and enqueues nothing

    def call(B=2, n_k=10, h=3, d=64, scale=0.125, dtype=1, q=p, a=p, g=p, l=p, o=p):
        return L.sbp_backward_attention(q, a, g, l, B, n_k, h, d, scale, dtype, o, None)

    assert call(dtype=7) == -4
    assert call(B=0) == -2 and call(h=0) == -2 and call(n_k=-1) == -2
    assert call(d=48) == -2 and call(d=256) == -2
    assert call(scale=0.0) == -2 and call(scale=float("nan")) == -2
    assert call(n_k=0, q=None, a=None, g=None, l=None, o=None) == 0          # nothing kept: nothing to do
    assert call(q=None) == -1 and call(l=None) == -1 and call(o=None) == -1
    assert call(a=ctypes.c_void_p(260)) == -2                                # alignment
    assert L.sbp_backward_attention_engine(99, 64, 1) == 1                   # bf16: matrix-core kernel
    assert L.sbp_backward_attention_engine(256, 64, 1) == 1 and L.sbp_backward_attention_engine(257, 64, 1) == 2   # beyond one LDS image: tiled
    assert L.sbp_backward_attention_engine(128, 128, 1) == 1 and L.sbp_backward_attention_engine(129, 128, 1) == 2
    assert L.sbp_backward_attention_engine(99, 64, 0) == 0 and L.sbp_backward_attention_engine(99, 16, 1) == 0
    assert L.sbp_backward_attention_engine(99, 48, 1) == -1


def test_backward_layerscale_argument_errors():
    L = _lib.lib()
    p = ctypes.c_void_p(256)
    need = L.sbp_backward_layerscale_workspace(100, 64)
    assert need >= 7 * 64 * 4 and need % 256 == 0 and L.sbp_backward_layerscale_workspace(-1, 64) == 0

    def call(K=100, C=64, dtype=1, dU=p, Y=p, gamma=p, dg=p, dY=p, ws=p, wb=need, flags=0):
        return L.sbp_backward_layerscale(dU, Y, gamma, K, C, dtype, dg, dY, ws, wb, flags, None)

    assert call(dtype=9) == -4 and call(K=-1) == -2 and call(C=0) == -2
    assert call(flags=2) == -8
    assert call(dU=None) == -1 and call(gamma=None) == -1
    assert call(ws=None) == -6 and call(wb=need - 1) == -6 and call(ws=ctypes.c_void_p(260)) == -6
    assert call(dg=None, dY=None) == 0                                      # nothing asked for


def test_backward_dwconv_argument_errors():
    L = _lib.lib()
    p = 4096
    ws = L.sbp_backward_dwconv_workspace(2, 8, 8, 16, 7, 64, 1, 0)
    assert ws > 0

    def call(dY=p, idx=p, inv=None, X=p, Wd=p, B=2, H=8, W=8, C=16, ks=7, pad=3, K=64, dtype=1, dWd=p, db=p,
             dX=p, wsp=p * 4, wsb=ws, flags=0):
        return L.sbp_backward_dwconv(dY, idx, inv, X, Wd, B, H, W, C, ks, pad, K, dtype, dWd, db, dX, wsp, wsb,
                                     flags, None)

    assert call(dY=None) == -1
    assert call(idx=None) == -1
    assert call(X=None) == -1
    assert call(X=None, dWd=None) == -1                 # db alone also reads X's positions: rejected on the host
    assert call(Wd=None) == -1
    assert call(ks=4) == -2
    assert call(ks=9, pad=4) == -2
    assert call(pad=2) == -2
    assert call(K=200) == -2
    assert call(dtype=3) == -4
    assert call(flags=1) == -8
    assert call(wsp=None) == -6
    assert call(wsb=16) == -6
    assert call(dWd=None, db=None, dX=None) == 0


def test_set_option_validates_names_and_values_and_changes_the_plan():
    L = _lib.lib()
    try:
        assert L.sbp_set_option(b"no_such_option", b"1") == -8
        assert L.sbp_set_option(b"tile", b"96x96") == -8
        assert L.sbp_set_option(b"dxbm", b"100") == -8
        # the dispatch order must be a permutation of 0, 1, 2: repeated or out-of-range kinds are refused here, on
        # the host, and never reach a kernel
        for bad in (b"0,0,0", b"0,1,3", b"1,2", b"-1,0,1", b"2,2,1"):
            assert L.sbp_set_option(b"order", bad) == -8
        assert L.sbp_set_option(b"order", b"2,0,1") == 0
        assert L.sbp_set_option(b"plan", b"128,100,1,0") == -8           # rows not a multiple of 64
        assert L.sbp_set_option(b"plan_768x2304", b"128,2112,3,0") == 0
        # the engine report follows an override and returns to the automatic choice when it is cleared
        auto = sbp.backward_linear_engine(4 * 197, 4 * 99, 64, 128, sbp.BF16)
        assert auto[0] == "mfma"
        sbp.set_option("tile", "big")
        sbp.set_option("splits", 3)
        assert sbp.backward_linear_engine(4 * 197, 4 * 99, 64, 128, sbp.BF16) == ("mfma_large", 3)
        sbp.set_option("splits", None)
        # a forced engine on a size its schedule search cannot serve falls back to equal legal splits (never a
        # split length of zero): 70000 kept rows need at least 9 splits of at most 7936 rows
        eng, n = sbp.backward_linear_engine(140000, 70000, 64, 128, sbp.BF16)
        assert eng == "mfma_large" and n >= 9
        # a split holds at most 7936 kept rows (their row ids sit in LDS): one more row forces a second split
        sbp.set_option("splits", 1)
        assert sbp.backward_linear_engine(9000, 7936, 256, 256, sbp.BF16) == ("mfma_large", 1)
        assert sbp.backward_linear_engine(9000, 7937, 256, 256, sbp.BF16) == ("mfma_large", 2)
        sbp.set_option("splits", None)
        sbp.set_option("tile", None)
        assert sbp.backward_linear_engine(4 * 197, 4 * 99, 64, 128, sbp.BF16) == auto
        ws_auto = sbp.backward_linear_workspace(12608, 6336, 768, 2304, sbp.BF16)
        sbp.set_option("plan_768x2304", "128,1088,6,0")
        assert sbp.backward_linear_engine(12608, 6336, 768, 2304, sbp.BF16) == ("mfma_large", 6)
        assert sbp.backward_linear_workspace(12608, 6336, 768, 2304, sbp.BF16) != ws_auto
    finally:
        assert L.sbp_set_option(None, None) == 0
    assert sbp.backward_linear_workspace(12608, 6336, 768, 2304, sbp.BF16) == ws_auto


def test_library_reads_no_environment_variable():
    src = os.path.join(ROOT, "paper_2210_00129_amd", "csrc")
    for name in os.listdir(src):
        assert "getenv" not in open(os.path.join(src, name)).read(), name


def test_binding_refuses_cpu_tensors():
    import torch
    X = torch.zeros(4, 8)
    idx = torch.zeros(2, dtype=torch.int32)
    with pytest.raises(ValueError):
        sbp.forward_cache(X, idx)


def test_fast_division_of_the_streaming_kernels_is_exact(tmp_path):
    # the kernels turn flat element numbers into (row, column) with a multiply and a shift; the same header compiled
    # for the host must agree with the compiler's division on edge values and a pseudo-random sample
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    exe = str(tmp_path / "fastdiv_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-I", os.path.join(here, "..", "paper_2210_00129_amd", "csrc"),
                    os.path.join(here, "fastdiv_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    assert out.startswith("ok "), out


def test_forward_cache_batch_rejects_bad_layouts():
    L = _lib.lib()
    p = 4096

    def call(layout, dtype=1, C=64, X=p, Xk=p):
        items = (_lib.GatherItem * 1)(_lib.GatherItem(X, p, Xk, 100, 50, C, layout))
        return L.sbp_forward_cache_batch(items, 1, dtype, None)

    assert call(2) == -8 and call(-1) == -8
    assert call(1, dtype=0) == -8            # row groups: bf16 only
    assert call(1, C=60) == -8
    assert call(1, X=p + 8) == -8 and call(1, Xk=p + 2) == -8
