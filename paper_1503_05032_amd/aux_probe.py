"""What the two ways of adding cross-tile sums through the auxiliary array cost
(Section 4), on the current GPU.

    python -m paper_1503_05032_amd.aux_probe

A matrix with a tile that starts too far into a row for the look-behind sends
the sums of the rows that span tiles through the auxiliary array.  They are added
either by a second small kernel or inside the tile kernel (the tile groups meet
per row, see csr5_spmv in the header); the library picks by size.  This probe
times both on matrices of several kinds and sizes, by fixing the choice with the
conversion flags CSR5_FLAG_AUX_TWO_KERNELS and CSR5_FLAG_AUX_ONE_KERNEL, and says
which one the library picks by itself.

Needs a GPU.  Results are facts about the machine, not parity items.
"""
from __future__ import annotations

import sys

import numpy as np


def spmv_us(a, sigma, flags, reps=200):
    """Whole SpMV, mean of `reps` back-to-back calls, best of three series (us);
    also whether a second kernel ran, and the number of tiles."""
    import torch
    from . import binding as B
    dev = torch.device("cuda:0")
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col = torch.from_numpy(a.col_idx).to(dev)
    val = torch.from_numpy(a.val).to(dev)
    x = torch.from_numpy(a.x).to(dev)
    y = torch.empty(a.m, dtype=torch.float64, device=dev)
    h = B.csr5_convert_ex(a.m, a.n, a.nnz, row_ptr, col, val, sigma=sigma, flags=flags)
    info = B.csr5_get_info(h)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for _ in range(20):
            B.csr5_spmv_ex(h, x, y)
        best = 1e30
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                B.csr5_spmv_ex(h, x, y)
            e1.record()
            stream.synchronize()
            best = min(best, e0.elapsed_time(e1) / reps)
        _, ms_second = B.csr5_spmv_profile(h, x, y, 50)
    stream.synchronize()
    B.csr5_free(h)
    return best * 1e3, ms_second > 1e-3, info["sigma"], info["p"]


def main():
    from . import binding as B
    from . import workloads as wl
    B.load()
    rows = lambda length, count, n: wl.from_row_lengths(np.full(count, length), n, seed=1, name=f"rows of {length}")
    cases = [("dense 2000 x 2000", lambda: wl.dense(2000), 0)]
    cases += [(f"power-law, scale {s}", (lambda s=s: wl.config(3, scale=s)), 0) for s in (0.12, 0.25, 0.5, 1.0)]
    cases += [(f"lp_rect, scale {s}", (lambda s=s: wl.config(4, scale=s)), 0) for s in (0.1, 0.25, 0.9)]
    cases += [(f"rows of 701", (lambda c=c: rows(701, c, 60000)), 16) for c in (2900, 5800, 8700, 30000)]
    cases += [(f"rows of 2000", (lambda c=c: rows(2000, c, 100000)), 16) for c in (1000, 3000, 4000)]
    cases += [(f"rows of 200", (lambda c=c: rows(200, c, 60000)), 8) for c in (10000, 20000, 30000, 50000)]
    print(f"{'matrix':24s} {'nnz':>10s} {'sigma':>5s} {'tiles':>7s} {'two kernels us':>15s} {'one kernel us':>14s} {'library picks':>14s}")
    for name, make, sigma in cases:
        a = make()
        two, second2, sg, p = spmv_us(a, sigma, B.CSR5_FLAG_AUX_TWO_KERNELS)
        one, second1, _, _ = spmv_us(a, sigma, B.CSR5_FLAG_AUX_ONE_KERNEL)
        _, second0, _, _ = spmv_us(a, sigma, B.CSR5_FLAG_NONE, reps=20)
        assert second2 and not second1, (name, second2, second1)     # the flags did what they say
        print(f"{name:24s} {a.nnz:10d} {sg:5d} {p:7d} {two:15.2f} {one:14.2f} {'two' if second0 else 'one':>14s}", flush=True)


if __name__ == "__main__":
    sys.exit(main())
