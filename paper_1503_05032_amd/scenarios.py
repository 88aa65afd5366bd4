"""Iteration-based scenarios (Section 5.5, Table 3): what converting CSR -> CSR5
costs and when it pays off against staying in CSR.

    python -m paper_1503_05032_amd.scenarios [--workloads 1,2,3,4,5]

Per workload: time of one CSR5 SpMV, of the conversion (workspace supplied, no
host check), of the best CSR row-block baseline (CSR-scalar, CSR-vector with 2..64
lanes per row), the preprocessing-to-SpMV ratio T_pre / T_spmv and the speedup
n*T_csr / (T_pre + n*T_csr5) for n = 50 and 500 iterations.  Needs a GPU.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def _time(torch, fn, reps):
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    best = 1e30
    for _ in range(3):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps)
    return best


def measure(a, reps=50, sigma=0):
    """Returns a dict of times in ms and the derived Table-3 quantities."""
    import torch
    from . import binding as B
    dev = torch.device("cuda:0")
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col0 = torch.from_numpy(a.col_idx).to(dev)
    val0 = torch.from_numpy(a.val).to(dev)
    x = torch.from_numpy(a.x).to(dev)
    y = torch.empty(max(a.m, 1), dtype=torch.float64, device=dev)
    reps = reps if a.nnz < 50_000_000 else max(10, reps // 4)
    # CSR baselines on the untouched arrays
    t_csr = {"scalar": _time(torch, lambda: B.csr5_baseline_csr_scalar(a.m, row_ptr, col0, val0, x, y), reps)}
    for lanes in (2, 4, 8, 16, 32, 64):
        t_csr[f"vector{lanes}"] = _time(
            torch, lambda: B.csr5_baseline_csr_vector(a.m, a.nnz, row_ptr, col0, val0, x, y, lanes_per_row=lanes), reps)
    best_csr = min(t_csr, key=t_csr.get)
    # conversion (fresh copies each time; the copies are outside the timed region)
    sigma = sigma or B.csr5_sigma_auto(a.nnz, a.m)
    ws = torch.empty(B.csr5_workspace_bytes(a.m, a.nnz, sigma), dtype=torch.uint8, device=dev)
    col, val = col0.clone(), val0.clone()
    conv = []
    h = None
    for _ in range(5):
        if h is not None:
            B.csr5_free(h)
        col.copy_(col0)
        val.copy_(val0)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        h = B.csr5_convert_ex(a.m, a.n, a.nnz, row_ptr, col, val, sigma=sigma, workspace=ws,
                              flags=B.CSR5_FLAG_NO_HOST_CHECK)
        e1.record()
        torch.cuda.synchronize()
        conv.append(e0.elapsed_time(e1))
    t_pre = float(np.median(conv))
    assert B.csr5_status(h) & 3 == 0              # the handle learns which launches the matrix needs
    t_csr5 = _time(torch, lambda: B.csr5_spmv_ex(h, x, y), reps)
    B.csr5_free(h)
    tc = t_csr[best_csr]
    out = {
        "workload": a.name, "nnz": a.nnz, "sigma": sigma,
        "t_csr5_ms": t_csr5, "t_pre_ms": t_pre, "t_csr_ms": tc, "best_csr": best_csr,
        "csr_all_ms": t_csr,
        "pre_to_spmv": t_pre / t_csr5,
        "speedup_isolated": tc / t_csr5,
    }
    for n in (50, 500):
        out[f"speedup_n{n}"] = n * tc / (t_pre + n * t_csr5)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workloads", default="1,2,3,4,5,6")
    ap.add_argument("--json", default=None)
    args = ap.parse_args()
    from . import binding as B
    from . import workloads as wl
    B.load()
    rows = []
    print(f"{'workload':26s} {'nnz':>10s} {'sig':>3s} {'CSR5 ms':>9s} {'conv ms':>8s} {'pre/spmv':>8s} "
          f"{'best CSR':>9s} {'CSR ms':>9s} {'x iso':>6s} {'x n=50':>7s} {'x n=500':>8s}")
    for tok in args.workloads.split(","):
        a = wl.config(int(tok))
        r = measure(a)
        rows.append(r)
        print(f"{r['workload']:26s} {r['nnz']:10d} {r['sigma']:3d} {r['t_csr5_ms']:9.5f} {r['t_pre_ms']:8.4f} "
              f"{r['pre_to_spmv']:8.2f} {r['best_csr']:>9s} {r['t_csr_ms']:9.5f} {r['speedup_isolated']:6.2f} "
              f"{r['speedup_n50']:7.2f} {r['speedup_n500']:8.2f}", flush=True)
    if args.json:
        json.dump(rows, open(args.json, "w"))


if __name__ == "__main__":
    sys.exit(main())
