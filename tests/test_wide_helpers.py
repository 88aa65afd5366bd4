"""CPU tests around the 64-bit index variant: the device-side generator (at a
scale that fits the host) and the stand-alone-tile reference the large GPU test
relies on, checked against the oracle's conversion of the whole matrix."""
import numpy as np

import oracle
from paper_1503_05032_amd import workloads_device as wd

from gpu_util import tile_reference


def _small():
    A = wd.huge_mixed("cpu", scale=0.002)
    return A, A["row_ptr"].numpy(), A["col_idx"].numpy(), A["val"].numpy()


def test_generator_structure_and_reproducibility():
    A, rp, col, val = _small()
    m, n, nnz = A["m"], A["n"], A["nnz"]
    assert rp.dtype == np.int64 and rp[0] == 0 and rp[-1] == nnz and np.all(np.diff(rp) >= 0)
    lens = np.diff(rp)
    assert 0.01 < (lens == 0).mean() < 0.06
    assert np.sort(lens)[-wd.LONG_ROWS] >= n // 2 - n // 16          # the long rows are there
    body = lens[(lens > 0) & (lens < wd.LEN_HI)]
    assert body.min() >= wd.LEN_LO and abs(body.mean() - (wd.LEN_LO + wd.LEN_HI) / 2) < 10
    assert col.min() >= 0 and col.max() < n and np.all(np.abs(val) <= 1)
    for r in np.concatenate([np.arange(50), np.argsort(lens)[-2:]]):   # distinct columns inside a row
        c = col[rp[r]:rp[r + 1]]
        assert np.unique(c).shape[0] == c.shape[0]
    B = wd.huge_mixed("cpu", scale=0.002)
    assert np.array_equal(B["col_idx"].numpy(), col) and np.array_equal(B["val"].numpy(), val)
    # at full scale the matrix needs the 64-bit variant: mean row length times the row count
    assert lens.mean() * 6_400_000 > 2**31


def test_stand_alone_tile_reference_equals_whole_matrix_oracle():
    A, rp, col, val = _small()
    m, n, nnz = A["m"], A["n"], A["nnz"]
    for sigma in (16, 5, 40):
        T = 64 * sigma
        ref = oracle.convert(m, n, nnz, rp.astype(np.int32), col, val, 64, sigma)
        td = ref.tile_desc.reshape(ref.pc, ref.W * 64)
        marked = 0
        for t in range(ref.pc):
            lo, hi = t * T, (t + 1) * T
            r0, one = tile_reference(rp, m, n, t, T, sigma, col[lo:hi], val[lo:hi])
            assert r0 == ref.tile_ptr[t] & 0x7fffffff
            assert bool(one.tile_ptr[0] >> 31) == bool(ref.tile_ptr[t] >> 31)
            assert np.array_equal(one.tile_desc, td[t])
            if ref.tile_ptr[t] >> 31:
                marked += 1
                assert np.array_equal(one.empty_offset,
                                      ref.empty_offset[ref.empty_offset_ptr[t]:ref.empty_offset_ptr[t + 1]])
            assert np.array_equal(one.col_idx, ref.col_idx[lo:hi])
            assert np.array_equal(one.val, ref.val[lo:hi])
        assert marked > 10
