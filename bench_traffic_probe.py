#!/usr/bin/env python3
"""HBM-traffic probe for the roofline's `traffic` field.

Run it twice under rocprofv3, once per counter (the two do not fit one pass):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d prof_out/pmc_fetch -- python3 bench_traffic_probe.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d prof_out/pmc_write -- python3 bench_traffic_probe.py
    python3 bench_traffic_probe.py --summarize prof_out/pmc_fetch prof_out/pmc_write

(`--workload NAME` after the script name takes another workload of synth_inputs.WORKLOADS than ViT-Base.)
The workload: a plain device-to-device copy of known size (the calibration: what the counter reads
for a known number of bytes), then one SBP linear backward per ViT-Base layer shape at r = 0.5 and one
forward-cache gather, on fresh buffers larger than the last-level cache between launches.
The summary prints, per kernel, the mean counter value per dispatch (KiB), the calibration factor
(known copy bytes / counter reading) and the calibrated bytes.
"""
from __future__ import annotations

import csv
import glob
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

COPY_BYTES = 256 * 1024 * 1024           # read 256 MiB, write 256 MiB per copy launch


def workload(name="vit_base"):
    import torch
    import paper_2210_00129_amd as sbp
    import synth_inputs as si

    torch.cuda.set_device(0)
    wl = si.WORKLOADS[name]
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    flush = torch.empty(768 * 1024 * 1024, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        dst.copy_(src)
    idx, inv = sbp.sample_indices(wl.B, wl.P, wl.H, wl.W, 2, 0, 1, want_inv=True)
    K = idx.numel()
    for s in wl.linears:
        X = torch.randn(wl.M, s.Cin, device="cuda").bfloat16()
        W = (torch.randn(s.Cout, s.Cin, device="cuda") * 0.02).bfloat16()
        dY = torch.randn(wl.M, s.Cout, device="cuda").bfloat16()
        flush.fill_(0)                                    # push earlier data out of the last-level cache
        Xk = sbp.forward_cache(X, idx)
        flush.fill_(0)
        sbp.backward_linear(dY, idx, Xk, W, inv=inv)
    torch.cuda.synchronize()
    print("probe done: K =", K)


def summarize(dirs):
    vals = {}
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                key = (row["Counter_Name"], row["Kernel_Name"][:70])
                vals.setdefault(key, []).append(float(row["Counter_Value"]))
    factor = {}
    # calibration: the copy kernel is torch's elementwise copy; take the dispatches with the largest reading
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        cands = [(max(v), k) for (c, k), v in vals.items() if c == counter and "copy" in k.lower()]
        if cands:
            reading, k = max(cands)
            factor[counter] = COPY_BYTES / (reading * 1024.0)
            print(f"calibration {counter}: copy kernel '{k[:50]}' reads {reading:.0f} KiB for {COPY_BYTES} bytes -> factor {factor[counter]:.4f}")
    for (counter, kernel), v in sorted(vals.items()):
        if not any(t in kernel for t in ("sbp::", "copy")):
            continue
        mean = sum(v) / len(v)
        fac = factor.get(counter, 1.0)
        print(f"{counter:10s} {kernel:70s} n={len(v):3d} mean={mean:12.1f} KiB  calibrated={mean * 1024 * fac / 1e6:10.2f} MB")


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "--summarize":
        summarize(sys.argv[2:])
    elif len(sys.argv) > 2 and sys.argv[1] == "--workload":     # e.g. --workload convnext_det_s1
        workload(sys.argv[2])
    else:
        workload()
