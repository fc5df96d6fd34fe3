#!/usr/bin/env python3
"""Benchmark of the SBP hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vit_base] [--ratio 0.5]

One "step" is one pass of the whole path over one synthetic batch of the workload: for every
block, draw a fresh grid-wise keep-set, cache the kept input rows of every linear layer
(forward side), then run the token-subset backward (dW, db, dX) of every linear layer; workloads
with a depthwise conv add its kept-position backward.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

value = useful contraction work (4 K Cin Cout flop per linear, + 4 ks^2 K C for the depthwise
conv) of a step divided by the step's wall time, everything included.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "SBP backward TFLOP/s at keep r=0.5 + speedup vs r=1 on one MI355X"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vit_base")
    ap.add_argument("--ratio", type=float, default=0.5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements of the other workloads")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--per-layer", action="store_true",
                    help="one cache call and one backward call per layer instead of one batched call per block")
    ap.add_argument("--xk-layout", choices=["rows", "kmajor"], default="rows",
                    help="layout of the cached rows X_k in the batched call pattern: [K, C] or groups of 8 rows [K/8, C, 8]")
    ap.add_argument("--set", action="append", default=[], metavar="NAME=VALUE",
                    help="an explicit override of the library's choices (sbp_set_option), for sweeps")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="workload for rocprofv3 --pmc runs: a calibration copy of known size, then one cold pass of a block")
    ap.add_argument("--summarize-pmc", nargs="+", metavar="DIR",
                    help="print per-kernel means of the counters in rocprofv3 output directories and exit (no GPU needed)")
    ap.add_argument("--timeline", action="store_true",
                    help="per-workgroup time stamps of the last batched backward launch of a step, summarised per kind of unit")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed region at the chosen ratio (for profiler runs: no r=1 leg, no event pass)")
    ap.add_argument("--rowwise-only", action="store_true",
                    help="only the side measurements of the row-wise steps, the down-sampling layer and the samplers")
    ap.add_argument("--attention-only", action="store_true",
                    help="only the attention-backward side measurement (for profiler runs)")
    return ap.parse_args()


class LinearLayer:
    """Device buffers and pre-marshalled library calls of one linear layer of one block."""

    def __init__(self, sbp, torch, L, shape, M, Kmax, dtype, src, ws, stream):
        self.Cin, self.Cout = shape.Cin, shape.Cout
        X, W, dY = src
        self.X, self.W, self.dY = X.clone(), W.clone(), dY.clone()     # own memory per block
        self.Xk = torch.empty((Kmax + 8, self.Cin), dtype=X.dtype, device="cuda")   # (+ 8: room for a padded last row group)
        self.code = sbp.BF16 if dtype == "bf16" else sbp.F32
        self.M = M
        self.L = L
        self.ws = ws
        self.stream = stream

    def bind_outputs(self, dW, db, dX):
        self.dW, self.db, self.dX = dW, db, dX

    def cache(self, idx_ptr, K):
        return self.L.sbp_forward_cache(self.X.data_ptr(), idx_ptr, self.M, K, self.Cin, self.code,
                                        self.Xk.data_ptr(), self.stream)

    def backward_dx(self, idx_ptr, inv_ptr, K):
        """only the input gradient (the critical path of a chain of dependent layers)"""
        return self.L.sbp_backward_linear(self.dY.data_ptr(), idx_ptr, inv_ptr, None, self.W.data_ptr(), self.M,
                                          K, self.Cin, self.Cout, self.code, None, None,
                                          self.dX.data_ptr(), self.ws.data_ptr(), self.ws.numel(), 0, self.stream)

    def backward(self, idx_ptr, inv_ptr, K):
        return self.L.sbp_backward_linear(self.dY.data_ptr(), idx_ptr, inv_ptr, self.Xk.data_ptr(), self.W.data_ptr(), self.M,
                                          K, self.Cin, self.Cout, self.code, self.dW.data_ptr(), self.db.data_ptr(),
                                          self.dX.data_ptr(), self.ws.data_ptr(), self.ws.numel(), 0, self.stream)


class Job:
    """All buffers of a workload and a step() that enqueues one pass of the path."""

    def __init__(self, wl, torch, sbp, si, batched=True, kmajor=False):
        from paper_2210_00129_amd import _lib
        self.wl, self.torch, self.sbp = wl, torch, sbp
        self.batched = batched
        self.kmajor = bool(kmajor and batched and wl.dtype == "bf16" and all(s.Cin % 8 == 0 for s in wl.linears))
        self.L = _lib.lib()
        self.check = _lib.check
        self.stream = torch.cuda.current_stream().cuda_stream
        M = wl.M
        self.M = M
        self.code = sbp.BF16 if wl.dtype == "bf16" else sbp.F32
        ws_bytes = 256
        for s in wl.linears:
            for k in (1, 2, 3, 4):
                K = sbp.keep_count(wl.B, wl.P, wl.H, wl.W, k)
                ws_bytes = max(ws_bytes, sbp.backward_linear_workspace(M, K, s.Cin, s.Cout, self.code, 0))
        if wl.dw_channels:
            ws_bytes = max(ws_bytes, sbp.backward_dwconv_workspace(wl.B, wl.H, wl.W, wl.dw_channels, 7, M, self.code, 0))
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        self.idx = torch.empty(M, dtype=torch.int32, device="cuda")
        self.inv = torch.empty(M, dtype=torch.int32, device="cuda")   # the sampler's inverse map rides along
        # one seeded CPU draw per layer shape, copied into separate device buffers for every block so
        # that successive blocks do not hit each other's data in the 256 MB last-level cache
        srcs = [tuple(t.cuda() for t in si.linear_case(M, s.Cin, s.Cout, 100 + i, wl.dtype))
                for i, s in enumerate(wl.linears)]
        self.blocks = []
        for _ in range(wl.blocks):
            self.blocks.append([LinearLayer(sbp, torch, self.L, s, M, M, wl.dtype, srcs[i], self.ws, self.stream)
                                for i, s in enumerate(wl.linears)])
        del srcs
        # outputs are shared by all blocks (a training loop hands them to the optimizer / previous layer)
        tdt = si.torch_dtype(wl.dtype)
        outs = [(torch.empty((s.Cout, s.Cin), dtype=torch.float32, device="cuda"),
                 torch.empty((s.Cout,), dtype=torch.float32, device="cuda"),
                 torch.empty((M, s.Cin), dtype=tdt, device="cuda")) for s in wl.linears]
        for blk in self.blocks:
            for lay, o in zip(blk, outs):
                lay.bind_outputs(*o)
        self.outs = outs
        if wl.dw_channels:
            C = wl.dw_channels
            self.dw_in = [tuple(t.cuda() for t in si.dwconv_case(wl.B, wl.H, wl.W, C, 7, 200 + b, wl.dtype))
                          for b in range(wl.blocks)]
            self.dw_out = (torch.empty((7, 7, C), dtype=torch.float32, device="cuda"),
                           torch.empty((C,), dtype=torch.float32, device="cuda"),
                           torch.empty((wl.B, wl.H, wl.W, C), dtype=tdt, device="cuda"))
        self.desc = sbp.make_desc(wl.B, wl.P, wl.H, wl.W, 2, 0, 0)
        self.step_no = 0
        # batched calls: per block one array of layer descriptors (backward order) and one of gather items,
        # marshalled once; set_ratio fills in K
        # (every block has its own keep list there: the masks of a whole step are drawn by one call at its start)
        self.batch_args = []
        self.batch_args_w = []
        self.chained = False
        nb = len(self.blocks)
        self.idx_b = [torch.empty(M, dtype=torch.int32, device="cuda") for _ in range(nb)]
        self.inv_b = [torch.empty(M, dtype=torch.int32, device="cuda") for _ in range(nb)]
        for b, blk in enumerate(self.blocks):
            ip, vp = self.idx_b[b].data_ptr(), self.inv_b[b].data_ptr()
            lays = (_lib.LinearLayer * len(blk))(*[
                _lib.LinearLayer(l.dY.data_ptr(), ip, vp, l.Xk.data_ptr(), l.W.data_ptr(), M, 0,
                                 l.Cin, l.Cout, l.dW.data_ptr(), l.db.data_ptr(), l.dX.data_ptr(), sbp.FLAG_XK_KMAJOR if self.kmajor else 0, 0)
                for l in reversed(blk)])
            items = (_lib.GatherItem * len(blk))(*[
                _lib.GatherItem(l.X.data_ptr(), ip, l.Xk.data_ptr(), M, 0, l.Cin, sbp.LAYOUT_KMAJOR if self.kmajor else 0) for l in blk])
            # chained pattern: the weight gradients of the block in one call, no dX
            lays_w = (_lib.LinearLayer * len(blk))(*[
                _lib.LinearLayer(l.dY.data_ptr(), ip, vp, l.Xk.data_ptr(), l.W.data_ptr(), M, 0,
                                 l.Cin, l.Cout, l.dW.data_ptr(), l.db.data_ptr(), None, sbp.FLAG_XK_KMAJOR if self.kmajor else 0, 0)
                for l in reversed(blk)])
            self.batch_args.append((lays, items))
            self.batch_args_w.append(lays_w)
        self.descs = (_lib.SampleDesc * nb)(*[sbp.make_desc(wl.B, wl.P, wl.H, wl.W, 2, 0, 0) for _ in range(nb)])
        self.idx_ptrs = (ctypes.c_void_p * nb)(*[t.data_ptr() for t in self.idx_b])
        self.inv_ptrs = (ctypes.c_void_p * nb)(*[t.data_ptr() for t in self.inv_b])
        self.idx_caps = (ctypes.c_int64 * nb)(*[M] * nb)
        self.ws_batch = None

    def set_ratio(self, r):
        self.k = self.sbp.k_from_ratio(r)
        self.desc.k = self.k
        self.K = self.sbp.keep_count(self.wl.B, self.wl.P, self.wl.H, self.wl.W, self.k)
        need = 256
        for lays, items in self.batch_args:
            for i in range(len(lays)):
                lays[i].K = self.K
                items[i].K = self.K
            need = max(need, int(self.L.sbp_backward_linear_batch_workspace(lays, len(lays), self.code)))
        for lays in self.batch_args_w:
            for i in range(len(lays)):
                lays[i].K = self.K
            need = max(need, int(self.L.sbp_backward_linear_batch_workspace(lays, len(lays), self.code)))
        if self.ws_batch is None or self.ws_batch.numel() < need:
            self.ws_batch = self.torch.empty(need, dtype=self.torch.uint8, device="cuda")

    def flops_per_step(self):
        f = sum(4.0 * self.K * s.Cin * s.Cout for s in self.wl.linears)
        if self.wl.dw_channels:
            f += 4.0 * 49 * self.K * self.wl.dw_channels
        return f * self.wl.blocks

    def step(self):
        L, check = self.L, self.check
        idx_ptr, K = self.idx.data_ptr(), self.K
        inv_ptr = self.inv.data_ptr() if self.inv is not None else None
        self.step_no += 1
        if self.batched:                                            # fresh masks for every block and step, drawn at once
            for b in range(len(self.blocks)):
                self.descs[b].k = self.k
                self.descs[b].stream_id = self.step_no * 1000 + b
            check(L.sbp_sample_indices_batch(self.descs, len(self.blocks), self.idx_ptrs, self.idx_caps, self.inv_ptrs, self.stream))
        for b, blk in enumerate(self.blocks):
            if self.batched:
                idx_ptr, inv_ptr = self.idx_b[b].data_ptr(), self.inv_b[b].data_ptr()
            else:
                self.desc.stream_id = self.step_no * 1000 + b      # fresh mask for every block and step
                check(L.sbp_sample_indices(ctypes.byref(self.desc), idx_ptr, self.M, inv_ptr, self.stream))
            if self.batched and self.chained:
                # a chain of dependent layers: dX layer by layer (the critical path), then all weight gradients of the block at once
                lays, items = self.batch_args[b]
                check(L.sbp_forward_cache_batch(items, len(items), self.code, self.stream))
                for lay in reversed(blk):
                    check(lay.backward_dx(idx_ptr, inv_ptr, K))
                lw = self.batch_args_w[b]
                check(L.sbp_backward_linear_batch(lw, len(lw), self.code, self.ws_batch.data_ptr(), self.ws_batch.numel(), self.stream))
            elif self.batched:
                lays, items = self.batch_args[b]
                check(L.sbp_forward_cache_batch(items, len(items), self.code, self.stream))   # forward side: the kept rows
                check(L.sbp_backward_linear_batch(lays, len(lays), self.code, self.ws_batch.data_ptr(),
                                                  self.ws_batch.numel(), self.stream))          # backward side
            else:
                for lay in blk:                                     # forward side: keep only the kept rows
                    check(lay.cache(idx_ptr, K))
                for lay in reversed(blk):                           # backward side
                    check(lay.backward(idx_ptr, inv_ptr, K))
            if self.wl.dw_channels:
                X, Wd, dY = self.dw_in[b]
                dWd, db, dX = self.dw_out
                wl = self.wl
                check(L.sbp_backward_dwconv(dY.data_ptr(), idx_ptr, inv_ptr, X.data_ptr(), Wd.data_ptr(), wl.B, wl.H,
                                            wl.W, wl.dw_channels, 7, 3, K, self.code, dWd.data_ptr(), db.data_ptr(),
                                            dX.data_ptr(), self.ws.data_ptr(), self.ws.numel(), 0, self.stream))

    def time_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        ev[0].record()
        for i in range(steps):
            self.step()
            ev[i + 1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
        self.last_stats = {"mean_ms": round(ev[0].elapsed_time(ev[steps]) / steps, 4), "median_ms": round(per[steps // 2], 4),
                           "min_ms": round(per[0], 4), "max_ms": round(per[-1], 4)}
        return max(ev[0].elapsed_time(ev[steps]) / steps, 0.0), wall

    def kernel_breakdown(self, steps):
        """Second pass with every launch bracketed by HIP events: per-class average durations."""
        sbp, torch = self.sbp, self.torch
        torch.cuda.synchronize()
        sbp.profile_read(reset=True)
        sbp.profile_enable(True)
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        sbp.profile_enable(False)
        return sbp.profile_read(reset=True)

    def algorithmic_bytes_per_step(self):
        """Bytes the method itself must move: kept rows in, gradients out (dX at full size)."""
        s_ = 2 if self.wl.dtype == "bf16" else 4
        K, M = self.K, self.M
        total = 4 * K                                                       # idx written by the sampler
        for s in self.wl.linears:
            total += 2 * K * s.Cin * s_ + 4 * K                             # cache gather
            total += s_ * (K * s.Cout + K * s.Cin + s.Cout * s.Cin + M * s.Cin) + 4 * s.Cout * s.Cin + 4 * s.Cout + 4 * K
        if self.wl.dw_channels:
            C = self.wl.dw_channels
            total += s_ * (K * C + 2 * M * C) + 49 * C * (s_ + 4)
        return total * self.wl.blocks


def timeline_report(job, torch, sbp, wl):
    """Device-clock time stamps of every workgroup of one linear_multi_kernel launch inside a step (the last block's):
    per layer and kind of unit the start times and durations, the shader clock the long units ran at, and how busy
    the 256 CUs were."""
    import numpy as np
    for _ in range(3):
        job.step()
    torch.cuda.synchronize()
    rec = torch.zeros((8192, 8), dtype=torch.int64, device="cuda")
    sbp.profile_timeline(rec)
    job.step()
    torch.cuda.synchronize()
    sbp.profile_timeline(None)
    t = rec.cpu().numpy()
    used = t[:, 0] > 0
    n = int(used.sum())
    t = t[:np.nonzero(used)[0].max() + 1]
    base = t[used[:len(t)], 0].min()
    kind, layer = t[:, 4] & 0xff, (t[:, 4] >> 8) & 0xff
    s = (t[:, 0] - base) / 100.0
    tiles = t[:, 1] > 0
    e = np.where(tiles, (t[:, 1] - base) / 100.0, s)
    d = e - s
    names = [x.name for x in reversed(wl.linears)]
    kn = {0: "dX tile", 1: "dW unit", 2: "dW unit (short)", 3: "zero fill", 4: "column sums"}
    out = {"workgroups": n, "span_us": round(float(e.max()), 1), "segments": []}
    xcd, ran_on = t[:, 5] & 0xff, (t[:, 5] >> 8) & 0xff      # queue the unit was planned on, XCD that ran it
    keys = sorted({(int(layer[i]), int(kind[i])) for i in range(len(t)) if used[i]}, key=lambda lk: float(np.min(s[(layer == lk[0]) & (kind == lk[1]) & used[:len(t)]])))
    for lay, kd in keys:
        sl = (layer == lay) & (kind == kd) & used[:len(t)]
        seg = {"layer": names[lay] if lay < len(names) else lay, "kind": kn[kd], "workgroups": int(sl.sum()),
               "xcds": sorted(int(v) for v in set(xcd[sl])), "run_elsewhere": int((xcd[sl] != ran_on[sl]).sum()),
               "start_us": [round(float(f(s[sl])), 1) for f in (np.min, np.median, np.max)]}
        if True:
            seg["duration_us"] = [round(float(f(d[sl])), 1) for f in (np.min, np.median, np.max)]
            seg["end_max_us"] = round(float(e[sl].max()), 1)
            cyc = (t[sl, 3] - t[sl, 2]).astype(np.float64)
            seg["shader_mhz_median"] = round(float(np.median(cyc / np.maximum(d[sl], 1e-3))), 0)
            # the same per XCD that ran the units (every XCD has a clock of its own): [units, median us, median MHz]
            seg["by_xcd"] = {int(x): [int((sl & (ran_on == x)).sum()), round(float(np.median(d[sl & (ran_on == x)])), 1),
                                      round(float(np.median(cyc[ran_on[sl] == x] / np.maximum(d[sl & (ran_on == x)], 1e-3))), 0)]
                             for x in sorted(int(v) for v in set(ran_on[sl]))}
        out["segments"].append(seg)
    out["cu_busy_frac"] = round(float(d[tiles].sum() / (256.0 * e.max())), 3)
    out["cu_busy_frac_tiles_only"] = round(float(d[tiles & (kind <= 2)].sum() / (256.0 * e.max())), 3)
    out["per_xcd_last_end_us"] = [round(float(e[(ran_on == x) & used[:len(t)]].max()), 1) for x in range(8)]
    return out


COPY_BYTES = 256 * 1024 * 1024           # the calibration copy reads 256 MiB and writes 256 MiB


def traffic_probe(wl, ratio, torch, sbp, si, kmajor=False):
    """Workload of the counter runs (rocprofv3 --pmc <counters> -- python3 bench.py --traffic-probe): a plain device
    copy of known size (what FETCH_SIZE / WRITE_SIZE read for a known number of bytes), then, on buffers pushed out of
    the last-level cache before every call, one block of the workload through the batched calls, the same layers
    through the per-layer calls, and the depthwise backward where the workload has one."""
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    flush = torch.empty(768 * 1024 * 1024, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        dst.copy_(src)
    k = sbp.k_from_ratio(ratio)
    idx, inv = sbp.sample_indices(wl.B, wl.P, wl.H, wl.W, k, 0, 1, want_inv=True)
    layers = []
    for i, s in enumerate(wl.linears):
        X, W, dY = (t.cuda() for t in si.linear_case(wl.M, s.Cin, s.Cout, 100 + i, wl.dtype))
        layers.append(dict(X=X, W=W, dY=dY))
    for rep in range(2):                                   # the second pass is the one to read (code and plans warm)
        flush.fill_(0)
        if kmajor:                                         # the cached rows in groups of 8 rows, as the batched call can read them
            Xkt = sbp.forward_cache_batch([l["X"] for l in layers], [idx] * len(layers), layout=sbp.LAYOUT_KMAJOR)
            flush.fill_(0)
            sbp.backward_linear_batch([dict(dY=l["dY"], idx=idx, inv=inv, X_k=xk, W=l["W"], M=wl.M, flags=sbp.FLAG_XK_KMAJOR)
                                       for l, xk in zip(layers, Xkt)])
            flush.fill_(0)
        Xks = sbp.forward_cache_batch([l["X"] for l in layers], [idx] * len(layers))
        flush.fill_(0)
        sbp.backward_linear_batch([dict(dY=l["dY"], idx=idx, inv=inv, X_k=xk, W=l["W"], M=wl.M) for l, xk in zip(layers, Xks)])
        for l, xk in zip(layers, Xks):
            flush.fill_(0)
            sbp.forward_cache(l["X"], idx, out=xk)
            flush.fill_(0)
            sbp.backward_linear(l["dY"], idx, xk, l["W"], inv=inv)
        if wl.dw_channels:
            X, Wd, dY = (t.cuda() for t in si.dwconv_case(wl.B, wl.H, wl.W, wl.dw_channels, 7, 200, wl.dtype))
            flush.fill_(0)
            sbp.backward_dwconv(dY, idx, X, Wd, inv=inv)
    torch.cuda.synchronize()
    print(json.dumps({"traffic_probe": wl.name, "keep_ratio": ratio, "K": idx.numel()}))


def summarize_pmc(dirs):
    """Per kernel and counter: dispatches, mean and last value over the *counter_collection.csv files under `dirs`;
    FETCH_SIZE / WRITE_SIZE (KiB) are also scaled by what the same counter read for the calibration copy."""
    import csv
    import glob
    vals = {}
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                vals.setdefault((row["Counter_Name"], row["Kernel_Name"][:72]), []).append(float(row["Counter_Value"]))
    factor = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        cands = [(max(v), k) for (c, k), v in vals.items() if c == counter and "copy" in k.lower()]
        if cands:
            reading, k = max(cands)
            factor[counter] = COPY_BYTES / (reading * 1024.0)
            print(f"calibration {counter}: copy kernel '{k[:50]}' reads {reading:.0f} KiB for {COPY_BYTES} bytes -> factor {factor[counter]:.4f}")
    for (counter, kernel), v in sorted(vals.items(), key=lambda kv: (kv[0][1], kv[0][0])):
        if not any(t in kernel for t in ("sbp::", "copy")):
            continue
        line = f"{kernel:72s} {counter:32s} n={len(v):4d} mean={sum(v) / len(v):16.1f} last={v[-1]:16.1f}"
        if counter in factor:
            line += f"  calibrated last = {v[-1] * 1024 * factor[counter] / 1e6:9.2f} MB"
        print(line)


def measured_traffic(name):
    """HBM-side bytes per launch of the dominant kernel, as measured with rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE and written down in profiles/ (bench.py cannot run the profiler on itself)."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH"):
                return int(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(wl, r, seconds, si):
    """The fp64 oracle, as it stands, on the host cores: whole blocks of the same workload, one after the other,
    until the time budget (about 15 s) is used."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    k = oracle.k_from_ratio(r)
    M = wl.M
    data = [tuple(si.to_f64(t) for t in si.linear_case(M, s.Cin, s.Cout, 100 + i, wl.dtype))
            for i, s in enumerate(wl.linears)]
    dwd = None
    if wl.dw_channels:
        dwd = tuple(si.to_f64(t) for t in si.dwconv_case(wl.B, wl.H, wl.W, wl.dw_channels, 7, 200, wl.dtype))
    flops, blocks, t0 = 0.0, 0, time.perf_counter()
    while blocks == 0 or time.perf_counter() - t0 < seconds:      # whole blocks, fresh mask each, until the budget is used
        idx = oracle.sample_indices(wl.B, wl.P, wl.H, wl.W, k, 0, 1000 + blocks)
        K = idx.size
        for (X, W, dY), s in zip(data, wl.linears):
            Xk = oracle.forward_cache(X, idx)
            oracle.backward_linear(dY, idx, Xk, W, M)
            flops += 4.0 * K * s.Cin * s.Cout
        if dwd is not None:
            oracle.backward_dwconv(dwd[2], idx, dwd[0], dwd[1], 3)
            flops += 4.0 * 49 * K * wl.dw_channels
        blocks += 1
    dt = time.perf_counter() - t0
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{blocks} block(s) of {wl.name} ({blocks / wl.blocks:.1f} steps of {wl.blocks} blocks) at r={r} "
                      f"(fp64 numpy oracle incl. its python sampler), {dt:.1f} s"}


def attainable_tflops(flops, algorithmic_bytes):
    """Ceiling of a whole step by the two published peaks: the matrix cores, or the step's intensity (flop per
    algorithmic byte, gathers and zero-filled rows included) times the HBM rate, whichever is lower."""
    return min(PEAK_BF16_TFLOPS, flops / algorithmic_bytes * PEAK_HBM_GBS / 1e3)


def ratio_entry(job, ms):
    tf = job.flops_per_step() / ms / 1e9
    ceiling = attainable_tflops(job.flops_per_step(), job.algorithmic_bytes_per_step())
    return {"K": job.K, "ms_per_step": round(ms, 4), "median_ms": job.last_stats["median_ms"], "min_ms": job.last_stats["min_ms"],
            "tflops": round(tf, 2), "algorithmic_gbs": round(job.algorithmic_bytes_per_step() / ms / 1e6, 1),
            "attainable_tflops": round(ceiling, 1), "frac_of_attainable": round(tf / ceiling, 4)}


def measure_extra(name, r, torch, sbp, si, steps=10, warmup=3, ratios=None):
    """A workload's step at several keep ratios (the batched calls; buffers of a step exceed the last-level cache only
    for the larger workloads: every block has its own tensors, see Job)."""
    wl = si.WORKLOADS[name]
    job = Job(wl, torch, sbp, si)
    out = {"workload": name}
    for rr in (ratios or (r, 1.0)):
        job.set_ratio(rr)
        ms, _ = job.time_steps(steps, warmup)
        out[f"r{rr:g}"] = ratio_entry(job, ms)
    out["speedup_vs_r1"] = round(out["r1"]["ms_per_step"] / out[f"r{r:g}"]["ms_per_step"], 3)
    out["ideal_flop_ratio_vs_r1"] = round(out["r1"]["K"] / out[f"r{r:g}"]["K"], 3)
    del job
    torch.cuda.empty_cache()
    return out


PEAK_VALU_TFLOPS = 78.6        # fp32 vector ALU without packed instructions: 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz


def measure_dwconv(torch, sbp, si, iters=40, warmup=5):
    """The depthwise 7 x 7 backward on kept outputs alone (ConvNeXt stage 3: 2 x 50 x 84 x 512) at r = 0.25 / 0.5 / 1:
    eight rotating tensor sets (8 x 26 MB: the last-level cache holds them - the map is small - so these are
    cache-resident numbers); algorithmic bytes s (K C + 2 M C) + 49 C (s + 4), flops 4 * 49 K C."""
    B, H, W, C = 2, 50, 84, 512
    M = B * H * W
    out = {"workload": f"depthwise 7x7 backward, map {B}x{H}x{W}x{C} (cache-resident: 8 rotating sets of 26 MB)", "ratios": {}}
    sets = []
    for i in range(8):
        X, Wd, dY = (t.cuda() for t in si.dwconv_case(B, H, W, C, 7, 300 + i, "bf16"))
        sets.append((X, Wd, dY, torch.empty_like(X), torch.empty((7, 7, C), device="cuda"), torch.empty(C, device="cuda")))
    from paper_2210_00129_amd import _lib
    L = _lib.lib()
    stream = torch.cuda.current_stream().cuda_stream
    for r in (0.25, 0.5, 1.0):
        k = sbp.k_from_ratio(r)
        idx, inv = sbp.sample_indices(B, 0, H, W, k, 0, 1, want_inv=True)
        K = idx.numel()
        ws = torch.empty(sbp.backward_dwconv_workspace(B, H, W, C, 7, K, sbp.BF16), dtype=torch.uint8, device="cuda")

        def run(i):
            X, Wd, dY, dX, dWd, db = sets[i % 8]
            _lib.check(L.sbp_backward_dwconv(dY.data_ptr(), idx.data_ptr(), inv.data_ptr(), X.data_ptr(), Wd.data_ptr(), B, H, W, C,
                                             7, 3, K, sbp.BF16, dWd.data_ptr(), db.data_ptr(), dX.data_ptr(), ws.data_ptr(),
                                             ws.numel(), 0, stream))
        for i in range(warmup):
            run(i)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record()
        for i in range(iters):
            run(i)
            ev[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(iters))
        us = ev[0].elapsed_time(ev[iters]) * 1e3 / iters
        nbytes = 2 * (K * C + 2 * M * C) + 49 * C * 6
        flops = 4.0 * 49 * K * C
        out["ratios"][f"r{r:g}"] = {"K": K, "us": round(us, 2), "median_us": round(per[iters // 2], 2), "min_us": round(per[0], 2),
                                    "algorithmic_mb": round(nbytes / 1e6, 2), "gbs": round(nbytes / us / 1e3, 1),
                                    "frac_of_hbm_peak": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4),
                                    "tflops": round(flops / us / 1e6, 2),
                                    "frac_of_fp32_valu_peak": round(flops / us / 1e6 / PEAK_VALU_TFLOPS, 4)}
    return out


def copy_same_size_us(torch, nbytes, iters=50, warmup=6):
    """A plain device copy that moves `nbytes` in total (half read, half written), timed like the kernels it is compared
    with: what the box gives a streaming kernel of this size (small tensors do not reach the rate of a 1 GB copy)."""
    n = max(int(nbytes) // 2, 256)
    bufs = [(torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1), torch.empty(n, dtype=torch.uint8, device="cuda")) for _ in range(6)]
    for i in range(warmup):
        bufs[i % 6][1].copy_(bufs[i % 6][0])
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        bufs[i % 6][1].copy_(bufs[i % 6][0])
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def measure_mlp_branch(torch, sbp, si, r, iters=20, warmup=5, model="vit_base", C=768, Hd=3072, row_wise=True):
    """Backward of one ViT MLP branch (LayerNorm -> fc1 -> GELU -> fc2, one keep-set) on compact rows with a
    single final scatter, against the same kernels scattering to full size after every linear layer; plus the
    row-wise kernels on their own against the HBM roofline."""
    wl = si.WORKLOADS[model]
    M = wl.B * (wl.P + wl.H * wl.W)
    k = sbp.k_from_ratio(r)
    idx, inv = sbp.sample_indices(wl.B, wl.P, wl.H, wl.W, k, 0, 1, want_inv=True)
    K = idx.numel()
    nset = 4                                              # rotate buffer sets: 4 x ~150 MB defeats the last-level cache
    sets = []
    for i in range(nset):
        t = lambda shape, std, seed: si.normal(shape, std, 300 + 10 * i + seed, "bf16").cuda()
        sets.append(dict(Xk=t((K, C), 1.0, 0), Uk=t((K, C), 1.0, 1), Zk=t((K, Hd), 1.5, 2), dY=t((M, C), 1.0, 3),
                         W1=t((Hd, C), C ** -0.5, 4), W2=t((C, Hd), Hd ** -0.5, 5),
                         gamma=torch.ones(C, device="cuda"), Hk=torch.empty((K, Hd), dtype=torch.bfloat16, device="cuda"),
                         dHk=torch.empty((K, Hd), dtype=torch.bfloat16, device="cuda"),
                         dHf=torch.empty((M, Hd), dtype=torch.bfloat16, device="cuda"),
                         dUk=torch.empty((K, C), dtype=torch.bfloat16, device="cuda"),
                         dUf=torch.empty((M, C), dtype=torch.bfloat16, device="cuda"),
                         dX=torch.empty((M, C), dtype=torch.bfloat16, device="cuda"),
                         dW1=torch.empty((Hd, C), device="cuda"), db1=torch.empty(Hd, device="cuda"),
                         dW2=torch.empty((C, Hd), device="cuda"), db2=torch.empty(C, device="cuda"),
                         dg=torch.empty(C, device="cuda"), dbt=torch.empty(C, device="cuda")))
    ws_bytes = max(sbp.backward_linear_workspace(M, K, Hd, C, sbp.BF16), sbp.backward_linear_workspace(M, K, C, Hd, sbp.BF16),
                   sbp.backward_layernorm_workspace(M, K, C, sbp.BF16))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    CF = sbp.FLAG_DX_COMPACT
    CB = sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT

    def compact(b):
        sbp.act_forward_rows(b["Zk"], out=b["Hk"])
        sbp.backward_linear(b["dY"], idx, b["Hk"], b["W2"], M=M, flags=CF, inv=inv, dW=b["dW2"], db=b["db2"], dX=b["dHk"], workspace=ws)
        sbp.act_backward_rows(b["dHk"], b["Zk"], out=b["dHk"])
        sbp.backward_linear(b["dHk"], idx, b["Uk"], b["W1"], M=M, flags=CB, inv=inv, dW=b["dW1"], db=b["db1"], dX=b["dUk"], workspace=ws)
        sbp.backward_layernorm(b["dUk"], b["Xk"], b["gamma"], 1e-6, idx, M, inv=inv, dgamma=b["dg"], dbeta=b["dbt"], dX=b["dX"], workspace=ws)

    def scattered(b):
        sbp.act_forward_rows(b["Zk"], out=b["Hk"])
        sbp.backward_linear(b["dY"], idx, b["Hk"], b["W2"], M=M, inv=inv, dW=b["dW2"], db=b["db2"], dX=b["dHf"], workspace=ws)
        sbp.forward_cache(b["dHf"], idx, out=b["dHk"])                   # the row-wise step gathers its input again
        sbp.act_backward_rows(b["dHk"], b["Zk"], out=b["dHk"])
        sbp.backward_linear(b["dHk"], idx, b["Uk"], b["W1"], M=M, flags=sbp.FLAG_DY_COMPACT, inv=inv, dW=b["dW1"], db=b["db1"], dX=b["dUf"], workspace=ws)
        sbp.forward_cache(b["dUf"], idx, out=b["dUk"])
        sbp.backward_layernorm(b["dUk"], b["Xk"], b["gamma"], 1e-6, idx, M, inv=inv, dgamma=b["dg"], dbeta=b["dbt"], dX=b["dX"], workspace=ws)

    def timed(fn, n=iters):
        for i in range(warmup):
            fn(sets[i % nset])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(sets[i % nset])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    flops = 2 * 4.0 * K * C * Hd
    ms_c, ms_s = timed(compact), timed(scattered)
    kern = {}
    for name, fn, nbytes in () if not row_wise else (
            ("act_forward_rows", lambda b: sbp.act_forward_rows(b["Zk"], out=b["Hk"]), 2 * K * Hd * 2),
            ("act_backward_rows", lambda b: sbp.act_backward_rows(b["dHk"], b["Zk"], out=b["dHk"]), 3 * K * Hd * 2),
            ("backward_layernorm", lambda b: sbp.backward_layernorm(b["dUk"], b["Xk"], b["gamma"], 1e-6, idx, M, inv=inv,
                                                                    dgamma=b["dg"], dbeta=b["dbt"], dX=b["dX"], workspace=ws),
             (2 * K * C + M * C) * 2 + 3 * C * 4 + 8 * K),
            ("backward_layerscale", lambda b: sbp.backward_layerscale(b["dUk"], b["Xk"], b["gamma"], dgamma=b["dg"], dY=b["dUk"],
                                                                      workspace=ws),
             3 * K * C * 2 + 2 * C * 4)):
        ms = timed(fn, 50)
        cp = copy_same_size_us(torch, nbytes)
        kern[name] = {"us": round(ms * 1e3, 2), "algorithmic_mb": round(nbytes / 1e6, 2),
                      "gbs": round(nbytes / ms / 1e6, 1), "frac_of_hbm_peak": round(nbytes / ms / 1e6 / 8000.0, 4),
                      "copy_same_size_us": round(cp, 2), "frac_of_copy_same_size": round(cp / (ms * 1e3), 3)}
    out = {"workload": f"{model} MLP branch backward (LayerNorm, fc1 {C}->{Hd}, GELU, fc2 {Hd}->{C}), K={K} of M={M}",
           "compact_ms": round(ms_c, 4), "scatter_every_layer_ms": round(ms_s, 4), "speedup": round(ms_s / ms_c, 3),
           "tflops_compact": round(flops / ms_c / 1e9, 1)}
    if row_wise:
        out["row_wise_kernels"] = kern
    return out


def measure_downsample(torch, sbp, si, r, iters=20, warmup=5):
    """Backward of a ConvNeXt down-sampling layer (2 x 2, stride 2 convolution, 128 -> 256 channels on a
    2 x 200 x 336 detection map) on kept output positions: patch gather, linear backward on patch rows, patch scatter."""
    B, H, W, C, Cout, p = 2, 200, 336, 128, 256, 2
    Ho, Wo = H // p, W // p
    Mo = B * Ho * Wo
    k = sbp.k_from_ratio(r)
    idx, inv = sbp.sample_indices(B, 0, Ho, Wo, k, 0, 1, want_inv=True)
    K = idx.numel()
    nset = 6
    sets = []
    for i in range(nset):
        t = lambda shape, std, seed: si.normal(shape, std, 500 + 10 * i + seed, "bf16").cuda()
        sets.append(dict(X=t((B, H, W, C), 1.0, 0), dY=t((Mo, Cout), 1.0, 1), Wc=t((Cout, p * p * C), (p * p * C) ** -0.5, 2),
                         Xk=torch.empty((K, p * p * C), dtype=torch.bfloat16, device="cuda"),
                         dXp=torch.empty((K, p * p * C), dtype=torch.bfloat16, device="cuda"),
                         dX=torch.empty((B, H, W, C), dtype=torch.bfloat16, device="cuda"),
                         dW=torch.empty((Cout, p * p * C), device="cuda"), db=torch.empty(Cout, device="cuda")))
    ws = torch.empty(sbp.backward_linear_workspace(Mo, K, p * p * C, Cout, sbp.BF16, sbp.FLAG_DX_COMPACT), dtype=torch.uint8, device="cuda")

    def gather(b): sbp.forward_cache_patches(b["X"], idx, p, out=b["Xk"])
    def linear(b): sbp.backward_linear(b["dY"], idx, b["Xk"], b["Wc"], M=Mo, flags=sbp.FLAG_DX_COMPACT, inv=inv, dW=b["dW"], db=b["db"], dX=b["dXp"], workspace=ws)
    def scatter(b): sbp.scatter_patches(b["dXp"], idx, (B, H, W, C), p, inv=inv, out=b["dX"])
    def layer(b): gather(b); linear(b); scatter(b)

    def timed(fn, n=iters):
        for i in range(warmup):
            fn(sets[i % nset])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(sets[i % nset])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    flops = 4.0 * K * p * p * C * Cout
    ms = timed(layer)
    out = {"workload": f"convnext down-sampling layer 2x2/2, {C}->{Cout}, map {B}x{H}x{W}, K={K} of {Mo} output positions",
           "ms": round(ms, 4), "tflops": round(flops / ms / 1e9, 1), "kernels": {}}
    for name, fn, nbytes in (("forward_cache_patches", gather, 2 * K * p * p * C * 2 + 4 * K),
                             ("backward_linear(patch rows)", linear, None),
                             ("scatter_patches", scatter, (K * p * p * C + B * H * W * C) * 2 + 4 * Mo + 4 * K)):
        m = timed(fn, 50)
        out["kernels"][name] = {"us": round(m * 1e3, 2)}
        if nbytes:
            cp = copy_same_size_us(torch, nbytes)
            out["kernels"][name].update({"algorithmic_mb": round(nbytes / 1e6, 2), "gbs": round(nbytes / m / 1e6, 1),
                                         "frac_of_hbm_peak": round(nbytes / m / 1e6 / 8000.0, 4),
                                         "copy_same_size_us": round(cp, 2), "frac_of_copy_same_size": round(cp / (m * 1e3), 3)})
    return out


def measure_attention(torch, sbp, si, iters=30, warmup=6):
    """Attention backward on the kept tokens ("Drop QKV") at the ViT-Base sizes: 64 samples, 12 heads of 64, 99 of
    197 tokens kept (r = 0.5) and all 197 (r = 1).  Six rotating input sets; algorithmic bytes = kept rows of qkv,
    A, dA read once, lse read, dqkv written; flops = the five products of the backward (10 n_k^2 d per head)."""
    import math
    B0, h, d = 64, 12, 64
    out = {"workload": f"vit_base attention core backward, B={B0}, {h} heads of {d} (long: B=8, 1024 kept tokens)", "sizes": {}}
    for tag, n_k, B in (("r0.5", 99, B0), ("r1", 197, B0), ("long", 1024, 8)):
        K = B * n_k
        sets = []
        for i in range(6):
            qkv, dA = si.attention_case(B, n_k, h, d, 700 + i, "bf16")
            sets.append((qkv.cuda(), si.normal((K, h * d), 0.2, 800 + i, "bf16").cuda(), dA.cuda(),
                         torch.full((K, h), 5.5, dtype=torch.float32, device="cuda"),
                         torch.empty((K, 3 * h * d), dtype=torch.bfloat16, device="cuda")))
        sc = 1.0 / math.sqrt(d)
        for i in range(warmup):
            b = sets[i % 6]
            sbp.backward_attention(b[0], b[1], b[2], b[3], B, h, d, sc, out=b[4])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            b = sets[i % 6]
            sbp.backward_attention(b[0], b[1], b[2], b[3], B, h, d, sc, out=b[4])
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / iters * 1e3
        nbytes = K * h * d * 2 * 8 + K * h * 4
        flops = 10.0 * B * h * n_k * n_k * d
        out["sizes"][tag] = {"n_k": n_k, "us": round(us, 2), "engine": sbp.backward_attention_engine(n_k, d, sbp.BF16),
                             "algorithmic_mb": round(nbytes / 1e6, 2), "gbs": round(nbytes / us / 1e3, 1),
                             "frac_of_hbm_peak": round(nbytes / us / 1e3 / 8000.0, 4), "tflops": round(flops / us / 1e6, 1)}
    out["speedup_vs_r1"] = round(out["sizes"]["r1"]["us"] / out["sizes"]["r0.5"]["us"], 3)
    return out


def measure_ceilings(torch, sbp, si, iters=10):
    """What this library's own kernels reach on this machine where nothing of SBP is in the way: the row gather with
    every row kept, in order (a plain copy of 512 MB), and the linear backward with every row kept on compact
    operands of a large square layer (two plain dense bf16 GEMMs, 16384 x 4096 x 4096)."""
    out = {}
    M, C = 65536, 4096
    X = torch.empty((M, C), dtype=torch.bfloat16, device="cuda").normal_()
    Y = torch.empty_like(X)
    idx = torch.arange(M, dtype=torch.int32, device="cuda")
    def timed(fn, n):
        for _ in range(3): fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n): fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    ms = timed(lambda: sbp.forward_cache(X, idx, out=Y), iters)
    out["stream_copy"] = {"kernel": "gather_rows_vec16, identity keep list", "mb": round(2 * M * C * 2 / 1e6, 1),
                          "us": round(ms * 1e3, 1), "gbs": round(2 * M * C * 2 / ms / 1e6, 1),
                          "frac_of_hbm_peak": round(2 * M * C * 2 / ms / 1e6 / PEAK_HBM_GBS, 4)}
    ms = timed(lambda: Y.copy_(X), iters)                 # the runtime's own device-to-device copy of the same 512 MiB
    out["device_copy"] = {"kernel": "hipMemcpy device to device (torch copy_)", "mb": round(2 * M * C * 2 / 1e6, 1),
                          "us": round(ms * 1e3, 1), "gbs": round(2 * M * C * 2 / ms / 1e6, 1),
                          "frac_of_hbm_peak": round(2 * M * C * 2 / ms / 1e6 / PEAK_HBM_GBS, 4)}
    del X, Y
    K, Cin, Cout = 16384, 4096, 4096
    dY = torch.empty((K, Cout), dtype=torch.bfloat16, device="cuda").normal_()
    Xk = torch.empty((K, Cin), dtype=torch.bfloat16, device="cuda").normal_()
    W = torch.empty((Cout, Cin), dtype=torch.bfloat16, device="cuda").normal_(0, 0.02)
    flags = sbp.FLAG_DY_COMPACT | sbp.FLAG_DX_COMPACT
    dW = torch.empty((Cout, Cin), dtype=torch.float32, device="cuda")
    dX = torch.empty((K, Cin), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(sbp.backward_linear_workspace(K, K, Cin, Cout, sbp.BF16, flags), dtype=torch.uint8, device="cuda")
    idx = idx[:K].contiguous()
    ms = timed(lambda: sbp.backward_linear(dY, idx, Xk, W, M=K, flags=flags, want=("dW", "dX"), dW=dW, dX=dX, workspace=ws), iters)
    tf = 4.0 * K * Cin * Cout / ms / 1e9
    out["dense_gemm_pair"] = {"kernel": "sbp_backward_linear, r = 1, compact operands, 16384 x 4096 x 4096",
                              "us": round(ms * 1e3, 1), "tflops": round(tf, 1),
                              "frac_of_bf16_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
    # for scale only (not part of the product, which calls no vendor GEMM): what the vendor's GEMM library reaches on this
    # box for the same two dense products through torch.matmul, bf16 in, bf16 out
    try:
        dWv = torch.empty((Cout, Cin), dtype=torch.bfloat16, device="cuda")

        def vendor():
            torch.matmul(dY.t(), Xk, out=dWv)
            torch.matmul(dY, W, out=dX)
        msv = timed(vendor, iters)
        tfv = 4.0 * K * Cin * Cout / msv / 1e9
        out["vendor_gemm_pair"] = {"kernel": "torch.matmul (vendor GEMM library), the same two dense products, bf16 outputs",
                                   "us": round(msv * 1e3, 1), "tflops": round(tfv, 1),
                                   "frac_of_bf16_mfma_peak": round(tfv / PEAK_BF16_TFLOPS, 4)}
        out["dense_gemm_pair"]["frac_of_vendor_gemm_pair"] = round(tf / tfv, 3)
        del dWv
    except Exception as e:   # the measurement is context, never a reason to fail the run
        out["vendor_gemm_pair"] = {"error": str(e)[:200]}
    del dY, Xk, W, dW, dX, ws
    torch.cuda.empty_cache()
    return out


def measure_samplers(torch, sbp, si):
    """One draw (keep list + inverse map) of every sampler mode on the ViT-Base batch and on a detection map."""
    out = {}
    for tag, (B, P, H, W) in (("vit_base 64x(1+14x14)", (64, 1, 14, 14)), ("detection 2x200x336", (2, 0, 200, 336))):
        M = B * (P + H * W)
        idx = torch.empty(M, dtype=torch.int32, device="cuda")
        inv = torch.empty(M, dtype=torch.int32, device="cuda")
        res = {}
        for name, kw in (("grid", dict(mode=sbp.GRID_PER_CELL)), ("grid 4x4 cells, 8 of 16", dict(mode=sbp.GRID_PER_CELL, cell=4, k=8)),
                         ("random_mask", dict(mode=sbp.RANDOM_MASK)),
                         ("temporal(8 frames, 2 of 4)", dict(mode=sbp.TEMPORAL, cell=4))):
            kw = dict(kw)
            k = kw.pop("k", 2)
            if name.startswith("temporal"):
                if (H * W) % 8:
                    continue
                geom = (B, P, 8, H * W // 8)
            else:
                geom = (B, P, H, W)
            for i in range(3):
                sbp.sample_indices(*geom, k, 0, i, idx_out=idx, inv_out=inv, **kw)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(50):
                sbp.sample_indices(*geom, k, 0, 10 + i, idx_out=idx, inv_out=inv, **kw)
            e1.record()
            torch.cuda.synchronize()
            res[name] = {"us": round(e0.elapsed_time(e1) / 50 * 1e3, 2)}
        out[tag] = res
    return out


def main():
    args = parse()
    if args.summarize_pmc:
        summarize_pmc(args.summarize_pmc)
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this path has no multi-GPU leg (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2210_00129_amd as sbp
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    for kv in args.set:
        name, _, value = kv.partition("=")
        sbp.set_option(name, value)
    if args.attention_only:
        print(json.dumps({"attention_drop_qkv": measure_attention(torch, sbp, si)}))
        return
    if args.rowwise_only:
        print(json.dumps({"mlp_branch_compact": measure_mlp_branch(torch, sbp, si, args.ratio),
                          "downsample_layer": measure_downsample(torch, sbp, si, args.ratio),
                          "sampler_modes": measure_samplers(torch, sbp, si)}))
        return
    wl = si.WORKLOADS[args.workload]
    if args.traffic_probe:
        traffic_probe(wl, args.ratio, torch, sbp, si, kmajor=args.xk_layout == "kmajor")
        return
    job = Job(wl, torch, sbp, si, batched=not args.per_layer, kmajor=args.xk_layout == "kmajor")

    job.set_ratio(args.ratio)
    if args.timeline:
        print(json.dumps(timeline_report(job, torch, sbp, wl)))
        return
    ms, wall_ms = job.time_steps(args.steps, args.warmup)
    main_stats = dict(job.last_stats)
    flops = job.flops_per_step()
    value = flops / ms / 1e9                       # TFLOP/s
    bytes_step = job.algorithmic_bytes_per_step()
    K_r = job.K
    if args.main_only:
        print(json.dumps({"metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "ms_per_step": round(ms, 4),
                          "steps": args.steps, "warmup": args.warmup, "config": {"workload": wl.name,
                                                                                 "keep_ratio": args.ratio}}))
        return
    prof = job.kernel_breakdown(max(2, min(args.steps, 5)))

    # dominant kernel and its roofline
    # the bf16 path issues ONE launch per linear layer (dW tiles + dX tiles + db + zero-fill), recorded
    # under "dw_gemm"; separate dX launches exist only on the plain fp32 path
    fused = prof["dx_gemm"][1] == 0
    gemm_flops = {"dw_gemm": 4.0 if fused else 2.0, "dx_gemm": 2.0}
    per_launch = {}
    layers_per_launch = len(wl.linears) if job.batched else 1        # a batched call serves a whole block in one launch
    for cls in ("dw_gemm", "dx_gemm"):
        tot_ms, n = prof[cls]
        if n:
            fl = sum(gemm_flops[cls] * K_r * s.Cin * s.Cout for s in wl.linears) / len(wl.linears) * layers_per_launch
            per_launch[cls] = (tot_ms / n, fl)
    dom = max(per_launch, key=lambda c: prof[c][0]) if per_launch else None
    roofline = None
    if dom:
        avg_ms, fl = per_launch[dom]
        achieved = fl / avg_ms / 1e9
        # which kernel the library runs for these layers (one fused launch per layer on the bf16 path)
        engines = sorted({sbp.backward_linear_engine(job.M, K_r, s.Cin, s.Cout, job.code)[0] for s in wl.linears})
        kname = {"mfma_large": "linear_big_kernel", "mfma": "linear_bwd_kernel", "plain": "plain_dw_kernel"}
        kernel = " / ".join(kname[e] for e in engines) + (" (dW + dX tiles, zero fill, db sums: one launch per layer)" if fused else "")
        if job.batched and engines == ["mfma_large"]:
            kernel = f"linear_multi_kernel (dX tiles, dW units, zero fill, db sums of the {len(wl.linears)} layers of a block: one launch per block)"
        profile_file = "linear_multi_kernel_vit_base_r0.5.md" if job.batched else "linear_big_kernel_vit_base_r0.5.md"
        roofline = {"bound": "mfma", "kernel": kernel if fused else dom, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": measured_traffic(profile_file)
                    if (wl.name == "vit_base" and args.ratio == 0.5 and engines == ["mfma_large"]) else None,
                    "avg_launch_us": round(avg_ms * 1e3, 2),
                    "flops_per_launch": fl}
        # layers whose intensity lies under the ridge of the two peaks are priced against HBM instead
        s_b = 2 if wl.dtype == "bf16" else 4
        by = sum(s_b * (K_r * s.Cout + K_r * s.Cin + s.Cout * s.Cin + wl.M * s.Cin) + 4 * s.Cout * s.Cin + 4 * s.Cout + 4 * K_r
                 for s in wl.linears) / len(wl.linears) * layers_per_launch
        if fused and fl / by < PEAK_BF16_TFLOPS * 1e3 / PEAK_HBM_GBS:
            gbs = by / avg_ms / 1e6
            roofline.update({"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes_per_launch": by,
                             "mfma_tflops": round(achieved, 2)})
    breakdown = {c: {"ms_per_step": round(v[0] / max(2, min(args.steps, 5)), 4), "launches": v[1]}
                 for c, v in prof.items() if v[1]}

    # same kernels at r = 1, and the other keep ratios of the workload's configuration
    sweep = {f"r{args.ratio:g}": None}
    job.set_ratio(1.0)
    ms_full, _ = job.time_steps(max(3, args.steps // 2), 2)
    sweep["r1"] = ratio_entry(job, ms_full)
    for rr in (0.25, 0.75):
        if rr != args.ratio:
            job.set_ratio(rr)
            ms_r, _ = job.time_steps(max(3, args.steps // 2), 2)
            sweep[f"r{rr:g}"] = ratio_entry(job, ms_r)
    job.set_ratio(args.ratio)
    job.last_stats = main_stats
    sweep[f"r{args.ratio:g}"] = ratio_entry(job, ms)
    for v in sweep.values():
        v["speedup_vs_r1"] = round(ms_full / v["ms_per_step"], 3)
        v["ideal_flop_ratio_vs_r1"] = round(wl.M / v["K"], 3)
    # the same step with one cache call and one backward call per layer (the four-call ABI of the method) / batched
    job.batched = not job.batched
    ms_other, _ = job.time_steps(max(3, args.steps // 2), 2)
    other_mode = {"calls": "one sbp_forward_cache_batch + one sbp_backward_linear_batch per block" if job.batched
                  else "one sbp_forward_cache + one sbp_backward_linear per layer",
                  "ms_per_step": round(ms_other, 4), "tflops": round(flops / ms_other / 1e9, 2)}
    job.batched = not job.batched
    chained_mode = None
    if job.batched and not job.kmajor:
        # a chain of dependent layers (a real training step): the input gradients layer by layer, the weight gradients
        # of the block in one batched call
        job.chained = True
        ms_ch, _ = job.time_steps(max(3, args.steps // 2), 2)
        job.chained = False
        chained_mode = {"calls": "one sbp_forward_cache_batch per block, one sbp_backward_linear (dX only) per layer, "
                                 "one sbp_backward_linear_batch (dW, db of the block) per block",
                        "ms_per_step": round(ms_ch, 4), "tflops": round(flops / ms_ch / 1e9, 2)}
    s_ = 2 if wl.dtype == "bf16" else 4
    cached = sum(K_r * s.Cin * s_ + 4 * K_r for s in wl.linears)
    full = sum(wl.M * s.Cin * s_ for s in wl.linears)

    result = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "median_ms_per_step": main_stats["median_ms"],
        "min_ms_per_step": main_stats["min_ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B}, {wl.N} tokens, {wl.blocks} blocks x "
                               f"{[(s.name, s.Cin, s.Cout) for s in wl.linears]}, grid-wise 2x2 keep r={args.ratio}",
                   "keep_ratio": args.ratio, "K": K_r, "M": wl.M},
        "speedup_vs_r1": round(ms_full / ms, 3), "ms_per_step_r1": round(ms_full, 4),
        "ideal_flop_ratio_vs_r1": round(wl.M / K_r, 3),
        "host_wall_ms_per_step": round(wall_ms, 4),
        "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "algorithmic_gbs": round(bytes_step / ms / 1e6, 1),
        "attainable_tflops": round(attainable_tflops(flops, bytes_step), 1),
        "frac_of_attainable": round(value / attainable_tflops(flops, bytes_step), 4),
        "activation_memory_saving": round(1.0 - cached / full, 4),
        "calls": "one sbp_sample_indices_batch per step, one sbp_forward_cache_batch + one sbp_backward_linear_batch per block" if job.batched
                 else "one sbp_forward_cache + one sbp_backward_linear per layer",
        "other_call_pattern": other_mode,
        "chained_call_pattern": chained_mode,
        "keep_ratio_sweep": sweep,
        "kernel_breakdown": breakdown,
        "roofline": roofline,
    }
    del job
    torch.cuda.empty_cache()
    if not args.no_extras:
        extras = []
        for name in ("vit_tiny_mlp", "convnext_det_s1", "convnext_det_s2", "convnext_s3_block"):
            if name != wl.name:
                extras.append(measure_extra(name, args.ratio, torch, sbp, si,
                                            ratios=(0.25, 0.5, 1.0) if name == "convnext_s3_block" else None))
        result["other_workloads"] = extras
        result["dwconv_backward"] = measure_dwconv(torch, sbp, si)
        result["mlp_branch_compact"] = measure_mlp_branch(torch, sbp, si, args.ratio)
        result["mlp_branch_compact_vit_tiny"] = measure_mlp_branch(torch, sbp, si, args.ratio, model="vit_tiny_mlp", C=192, Hd=768,
                                                                   row_wise=False)
        result["downsample_layer"] = measure_downsample(torch, sbp, si, args.ratio)
        result["sampler_modes"] = measure_samplers(torch, sbp, si)
        result["attention_drop_qkv"] = measure_attention(torch, sbp, si)
        result["measured_ceilings"] = measure_ceilings(torch, sbp, si)
        result["frac_of_own_dense_gemm"] = round(value / result["measured_ceilings"]["dense_gemm_pair"]["tflops"], 4)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, args.ratio, args.cpu_seconds, si)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
