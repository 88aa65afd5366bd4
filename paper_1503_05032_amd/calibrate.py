"""sigma calibration for the current GPU (Section 3.2: the bounds <r, s, t, u> of the
nnz/row -> sigma rule are hardware constants "obtained through some simple
benchmarks"; Section 5.4 / Figure 9: auto-tuned sigma against the best sigma).

    python -m paper_1503_05032_amd.calibrate [--sigmas 4..48] [--workloads 1,2,3,4,5,probes,bigprobes]

For every matrix it converts at each sigma, times csr5_spmv (HIP events around
back-to-back calls) and prints one table row per matrix: nnz/row, the best
sigma, the time at the library's automatic sigma and the loss against the best.
The probe matrices have fixed row lengths 1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 64,
128, 256, 512, 2048 (banded random columns), which is what the rule is a function
of, at about 8 M nonzeros ("probes": fewer tiles than the chip holds wavefronts
for) and, for a few lengths, at about 60 M ("bigprobes"); "sizeprobes" are rows of
8 and 27 entries at 8 to 40 M nonzeros, for the size below which the smaller
tile wins.
Needs a GPU.  Results are facts about the machine, not parity items.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def probe_matrix(row_len, nnz_target=8_000_000, seed=100):
    """Square matrix whose rows all have `row_len` entries, banded random columns."""
    from . import workloads as wl
    rng = np.random.default_rng(seed + row_len)
    m = max(64, nnz_target // row_len)
    n = max(m, 4 * row_len)
    width = max(4 * row_len, 64)
    rows = np.repeat(np.arange(m, dtype=np.int64), row_len)
    cols = (rows * n // m + rng.integers(0, width, size=rows.shape[0])) % n
    lens, c = wl._dedupe_sorted(rows, cols, m, n)
    val = rng.uniform(-1, 1, size=c.shape[0])
    x = rng.uniform(-1, 1, size=n)
    return wl._finish(m, n, lens, c, val, x, f"probe_len{row_len}")


def time_spmv(B, torch, h, x, y, reps):
    for _ in range(10):
        B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    best = 1e30
    for _ in range(3):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            B.csr5_spmv_ex(h, x, y)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / reps)
    return best


def sweep(a, sigmas, reps=100):
    import torch
    from . import binding as B
    dev = torch.device("cuda:0")
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col0 = torch.from_numpy(a.col_idx).to(dev)
    val0 = torch.from_numpy(a.val).to(dev)
    x = torch.from_numpy(a.x).to(dev)
    y = torch.empty(a.m, dtype=torch.float64, device=dev)
    out = {}
    for sg in sigmas:
        col, val = col0.clone(), val0.clone()
        ws = torch.empty(B.csr5_workspace_bytes(a.m, a.nnz, sg), dtype=torch.uint8, device=dev)
        h = B.csr5_convert_ex(a.m, a.n, a.nnz, row_ptr, col, val, sigma=sg, workspace=ws,
                              flags=B.CSR5_FLAG_NO_HOST_CHECK)
        assert B.csr5_status(h) & 3 == 0          # the handle learns which launches the matrix needs
        out[sg] = time_spmv(B, torch, h, x, y, reps)
        B.csr5_free(h)
        del col, val, ws
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sigmas", default="4..48")
    ap.add_argument("--workloads", default="1,2,3,4,5,6,probes")
    ap.add_argument("--reps", type=int, default=100)
    ap.add_argument("--json", default=None, help="also write the raw timings here")
    args = ap.parse_args()
    if ".." in args.sigmas:
        lo, hi = args.sigmas.split("..")
        sigmas = list(range(int(lo), int(hi) + 1))
    else:
        sigmas = [int(v) for v in args.sigmas.split(",")]

    from . import binding as B
    from . import workloads as wl
    B.load()
    mats = []
    for tok in args.workloads.split(","):
        if tok == "probes":
            mats += [probe_matrix(L) for L in (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 64, 128, 256, 512, 2048)]
        elif tok == "sizeprobes":      # where the small-matrix rule (sigma 8 below 12288 tiles) should end
            for L in (8, 27):
                for mn in (8, 12, 16, 20, 24, 30, 40):
                    a = probe_matrix(L, nnz_target=mn * 1_000_000)
                    a.name = f"size{mn}M_" + a.name
                    mats.append(a)
        elif tok == "bigprobes":
            for L in (1, 2, 4, 8, 12, 32, 128):
                a = probe_matrix(L, nnz_target=60_000_000)
                a.name = "big_" + a.name
                mats.append(a)
        else:
            mats.append(wl.config(int(tok)))
    raw = {}
    print(f"{'matrix':28s} {'nnz':>10s} {'nnz/row':>8s} {'best':>5s} {'ms@best':>9s} {'auto':>5s} {'ms@auto':>9s} {'loss%':>6s}")
    losses = []
    for a in mats:
        t = sweep(a, sigmas, reps=args.reps if a.nnz < 50_000_000 else max(10, args.reps // 5))
        raw[a.name] = {"nnz": a.nnz, "m": a.m, "ms": t}
        best = min(t, key=t.get)
        auto = B.csr5_sigma_auto(a.nnz, a.m)
        t_auto = t.get(auto)
        if t_auto is None:
            t_auto = sweep(a, [auto], reps=args.reps)[auto]
        loss = 100.0 * (t_auto / t[best] - 1.0)
        losses.append(loss)
        print(f"{a.name:28s} {a.nnz:10d} {a.nnz / max(a.m, 1):8.2f} {best:5d} {t[best]:9.5f} {auto:5d} "
              f"{t_auto:9.5f} {loss:6.2f}", flush=True)
    print(f"average loss of the automatic sigma against the best: {np.mean(losses):.2f} %")
    if args.json:
        json.dump(raw, open(args.json, "w"))


if __name__ == "__main__":
    sys.exit(main())
