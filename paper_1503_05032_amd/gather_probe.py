"""What a scattered gather of x costs the tile kernel on the current GPU.

    python -m paper_1503_05032_amd.gather_probe

Matrices with uniformly random columns (the structure of the rectangular and the
large mixed workload) are bound by the gathers x[col_idx[k]] of the per-column
loop of Algorithm 8, not by the tile stream.  Two tables say by what exactly:

1. x size.  The rectangular workload's generator with the number of columns
   varied (1.5 M rows, about 33.7 M nonzeros throughout): gathers per second as
   x grows from 8 MB to 2 GB, i.e. from "mostly in the L2s" through "in the
   memory-side cache" to "in HBM only".
2. Granularity.  One million rows of 16 entries in 16 different random 128-byte
   lines of a 512 MB x, then the same rows with a second (or three more) entries
   added in the same line: same 32-byte sector, other sector of the same 64-byte
   half, other half; and, for comparison, with a second entry in a different line.
   If the memory system moved less than a line per gather, an entry in another
   sector of the line would cost like a new line.

Needs a GPU.  Results are facts about the machine, not parity items.
"""
from __future__ import annotations

import sys

import numpy as np


def line_matrix(m, per_row, n, partners=(), far=False, seed=5):
    """`per_row` entries per row in different random 128-byte lines of x (16
    doubles), plus for every entry its partners `column ^ k` for k in `partners`
    (same line), plus with `far` one entry half of x away (another line)."""
    from . import workloads as wl
    rng = np.random.default_rng(seed)
    c0 = rng.integers(0, n // 16, size=(m, per_row)).astype(np.int64) * 16 + rng.integers(0, 16, size=(m, per_row))
    parts = [c0] + [c0 ^ k for k in partners] + ([(c0 + n // 2) % n] if far else [])
    cols = np.sort(np.concatenate(parts, axis=1), axis=1)
    k = cols.shape[1]
    rows = np.repeat(np.arange(m, dtype=np.int64), k)
    lens, c = wl._dedupe_sorted(rows, cols.reshape(-1), m, n)
    val = rng.uniform(-1.0, 1.0, size=c.shape[0])
    x = rng.uniform(-1.0, 1.0, size=n)
    return wl._finish(m, n, lens, c, val, x, "lines"), m * per_row * (2 if far else 1)


def tile_kernel_ms(a, reps=30):
    """Mean duration of the tile kernel at sigma = 16 (best of three series)."""
    import torch
    from . import binding as B
    dev = torch.device("cuda:0")
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col = torch.from_numpy(a.col_idx).to(dev)
    val = torch.from_numpy(a.val).to(dev)
    x = torch.from_numpy(a.x).to(dev)
    y = torch.empty(a.m, dtype=torch.float64, device=dev)
    h = B.csr5_convert_ex(a.m, a.n, a.nnz, row_ptr, col, val, sigma=16)
    B.csr5_status(h)
    for _ in range(5):
        B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    best = min(B.csr5_spmv_profile(h, x, y, reps)[0] for _ in range(3))
    B.csr5_free(h)
    return best


def main():
    from . import binding as B
    from . import workloads as wl
    B.load()
    print("1. x size (rectangular workload's generator, 1.5 M rows)")
    print(f"{'columns':>11s} {'x MB':>7s} {'nnz':>10s} {'tile kernel us':>15s} {'G gathers/s':>12s} {'x 128 B, TB/s':>14s}")
    for n in (1_000_000, 4_000_000, 16_000_000, 32_000_000, 64_000_000, 128_000_000, 256_000_000):
        a = wl.lp_rect(n=n)
        ms = tile_kernel_ms(a)
        print(f"{n:11d} {n * 8 / 1e6:7.0f} {a.nnz:10d} {ms * 1e3:15.1f} {a.nnz / ms / 1e6:12.1f} "
              f"{a.nnz * 128 / ms / 1e9:14.2f}", flush=True)
    print()
    print("2. granularity (1 M rows, 16 random lines of a 512 MB x per row)")
    print(f"{'entries per line':42s} {'nnz':>10s} {'tile kernel us':>15s} {'G lines/s':>10s}")
    m, per_row, n = 1_000_000, 16, 64_000_000
    for name, partners, far in (("one", (), False),
                                ("two, same 32-byte sector", (1,), False),
                                ("two, other sector of the same 64 bytes", (4,), False),
                                ("two, other 64-byte half", (8,), False),
                                ("four, one per 32-byte sector", (4, 8, 12), False),
                                ("one, and one in a line half of x away", (), True)):
        a, lines = line_matrix(m, per_row, n, partners, far)
        ms = tile_kernel_ms(a)
        print(f"{name:42s} {a.nnz:10d} {ms * 1e3:15.1f} {lines / ms / 1e6:10.1f}", flush=True)


if __name__ == "__main__":
    sys.exit(main())
