"""Seeded synthetic matrix too large to build on the host: 2^31 nonzeros and more,
generated with torch directly in GPU memory (it is there for device memory and
random numbers; none of the method's arithmetic lives here).

`huge_mixed` is the 64-bit-index workload: the structure of the `mixed_large`
configuration (moderately long rows of varying length, a few per cent of empty
rows, a handful of rows that span thousands of tiles) at sixteen times the size.
At scale 1 it has 6.4 M rows and about 2.2e9 nonzeros (27 GB of val + col_idx).
The columns of a row form a band that starts at the diagonal (stride 2 with a
pseudo-random 0/1 jitter, wrapping at n), so the columns of a row are distinct.  A small `scale` gives the same structure in a size
that also fits a CPU tensor, for the tests of the generator itself.
"""
from __future__ import annotations

import torch

LONG_ROWS = 5              # rows of about n/2 entries
EMPTY_FRACTION = 0.03
LEN_LO, LEN_HI = 200, 520  # ordinary rows: uniform in [LEN_LO, LEN_HI)
CHUNK = 1 << 27            # entries generated per step (bounds the temporaries to a few GB)


def huge_mixed(device="cuda:0", scale=1.0, seed=20150503):
    """Returns dict(m, n, nnz, row_ptr int64[m+1], col_idx int32[nnz], val float64[nnz],
    x float64[n], name) with every tensor on `device`."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    m = max(64, int(6_400_000 * scale))
    n = m
    lens = torch.randint(LEN_LO, LEN_HI, (m,), generator=g, device=dev, dtype=torch.int64)
    lens[torch.rand(m, generator=g, device=dev) < EMPTY_FRACTION] = 0
    long_rows = torch.randint(0, m, (LONG_ROWS,), generator=g, device=dev)
    lens[long_rows] = torch.randint(n // 2 - n // 16, n // 2, (LONG_ROWS,), generator=g, device=dev,
                                    dtype=torch.int64)
    row_ptr = torch.zeros(m + 1, dtype=torch.int64, device=dev)
    torch.cumsum(lens, 0, out=row_ptr[1:])
    nnz = int(row_ptr[-1].item())
    col_idx = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)[:nnz]
    val = torch.empty(max(nnz, 1), dtype=torch.float64, device=dev)[:nnz]
    for e0 in range(0, nnz, CHUNK):
        e1 = min(nnz, e0 + CHUNK)
        e = torch.arange(e0, e1, dtype=torch.int64, device=dev)
        r = torch.searchsorted(row_ptr, e, right=True) - 1          # owning row of every entry
        k = e - row_ptr[r]                                          # position inside the row
        jitter = ((e * 2654435761) >> 7) & 1
        col_idx[e0:e1] = ((r + 2 * k + jitter) % n).to(torch.int32)
        val[e0:e1] = torch.rand(e1 - e0, generator=g, device=dev, dtype=torch.float64) * 2 - 1
        del e, r, k, jitter
    x = torch.rand(n, generator=g, device=dev, dtype=torch.float64) * 2 - 1
    return dict(m=m, n=n, nnz=nnz, row_ptr=row_ptr, col_idx=col_idx, val=val, x=x,
                name=f"huge_mixed(scale={scale})")
