"""CPU checks of the seeded input generators: structure (sorted distinct columns,
index ranges), the shape statistics the documentation quotes, and reproducibility."""
import hashlib

import numpy as np
import pytest

from paper_1503_05032_amd import workloads as wl


def check_structure(a):
    assert a.row_ptr.dtype == np.int32 and a.col_idx.dtype == np.int32 and a.val.dtype == np.float64
    assert a.row_ptr.shape == (a.m + 1,) and a.row_ptr[0] == 0 and a.row_ptr[-1] == a.nnz
    lens = np.diff(a.row_ptr.astype(np.int64))
    assert np.all(lens >= 0)
    assert a.col_idx.shape == (a.nnz,) and a.val.shape == (a.nnz,) and a.x.shape == (a.n,)
    if a.nnz:
        assert a.col_idx.min() >= 0 and a.col_idx.max() < a.n
        if getattr(a, "sorted_distinct", True):
            inc = np.diff(a.col_idx.astype(np.int64)) > 0
            starts = np.zeros(a.nnz, dtype=bool)
            starts[a.row_ptr[:-1][lens > 0]] = True
            assert np.all(inc | starts[1:]), "columns must be sorted and distinct inside every row"
    assert np.all(np.isfinite(a.val)) and np.all(np.isfinite(a.x))


def digest(a):
    h = hashlib.sha256()
    for arr in (a.row_ptr, a.col_idx, a.val, a.x):
        h.update(np.ascontiguousarray(arr).tobytes())
    return h.hexdigest()


def test_tiny_uniform():
    a = wl.config(1)
    check_structure(a)
    assert (a.m, a.n, a.nnz) == (2000, 2000, 20510)
    lens = np.diff(a.row_ptr)
    assert lens.max() == 20 and (lens == 0).sum() == 89
    assert digest(a) == digest(wl.config(1))


def test_stencil_small_and_full_nnz_formula():
    a = wl.stencil27(g=12, seed=1)
    check_structure(a)
    assert a.nnz == (3 * 12 - 2) ** 3
    lens = np.diff(a.row_ptr)
    assert lens.min() == 8 and lens.max() == 27
    # every row holds its diagonal, value 26
    for r in (0, 5, 700, a.m - 1):
        seg = slice(a.row_ptr[r], a.row_ptr[r + 1])
        k = np.nonzero(a.col_idx[seg] == r)[0]
        assert k.size == 1 and a.val[seg][k[0]] == 26.0
    off = a.val[a.val != 26.0]
    assert np.all(np.abs(off + 1.0) <= 0.01)
    # symmetric pattern
    rows = np.repeat(np.arange(a.m), lens)
    fwd = set(zip(rows[:5000].tolist(), a.col_idx[:5000].tolist()))
    allp = set(zip(rows.tolist(), a.col_idx.tolist()))
    assert all((c, r) in allp for r, c in fwd)


@pytest.mark.parametrize("cfg,scale", [(3, 0.02), (4, 0.02), (5, 0.01), (8, 0.05)])
def test_scaled_irregular_workloads(cfg, scale):
    a = wl.config(cfg, scale=scale)
    check_structure(a)
    lens = np.diff(a.row_ptr)
    if cfg == 3:
        assert lens.min() >= 1 and 6.0 < lens.mean() < 11.0
        assert (a.col_idx < 16).mean() > 0.15            # preferential toward low ids
        assert lens.max() > 1000
    if cfg == 4:
        assert 0.27 < (lens == 0).mean() < 0.33
        assert lens.max() > 1000
    if cfg == 8:      # same row model with a quarter of the dense rows: 12 M nonzeros at full size
        assert 0.27 < (lens == 0).mean() < 0.33
        assert 6.5 < lens.mean() < 9.0 and lens.max() > 1000
    if cfg == 5:
        assert lens.min() >= 1 and 12.0 < lens.mean() < 22.0
    assert digest(a) == digest(wl.config(cfg, scale=scale))


def test_dense_matrix_of_the_paper():
    a = wl.dense(200)
    check_structure(a)
    assert a.nnz == 200 * 200 and np.all(np.diff(a.row_ptr) == 200)
    assert wl.config(6).nnz == 4_000_000                  # Table 2, r1: 2K x 2K, 4.0M


def test_edge_case_catalogue():
    T = 64 * 4
    cases = wl.edge_cases(T)
    names = [c.name for c in cases]
    assert len(set(names)) == len(names)
    for a in cases:
        check_structure(a)
    by = {c.name: c for c in cases}
    assert by["all_empty"].nnz == 0
    assert by["one_long_row"].m == 1 and by["one_long_row"].nnz > 3 * T
    assert by["exact_two_tiles"].nnz == 2 * T
    assert by["less_than_one_tile"].nnz < T


def test_structured_case_catalogue():
    T = 64 * 4
    cases = wl.structured_cases(T)
    by = {c.name.split("_")[0]: c for c in cases}
    for a in cases:
        check_structure(a)
        assert digest(a) == digest({c.name: c for c in wl.structured_cases(T)}[a.name])
    arrow = by["arrowhead"]
    lens = np.diff(arrow.row_ptr)
    assert lens[0] == arrow.n and np.all(lens[1:] == 2) and arrow.nnz > 4 * T
    band = by["band7"]
    assert np.diff(band.row_ptr).max() == 7 and np.diff(band.row_ptr).min() == 4
    tri = by["upper"]
    assert np.array_equal(np.diff(tri.row_ptr), np.arange(tri.n, 0, -1)) and tri.nnz > T
    rep = by["unsorted"]
    assert not rep.sorted_distinct
    r = np.repeat(np.arange(rep.m), np.diff(rep.row_ptr))
    assert np.unique(np.stack([r, rep.col_idx]), axis=1).shape[1] < rep.nnz          # it does repeat entries



def test_measured_traffic_file_is_well_formed():
    """bench.py's roofline.traffic comes from a tracked summary of offline rocprofv3
    runs: every line names workload, sigma, dtype, the two counters, the commit it
    was measured at and the kernel; bench.py's reader scales them as documented."""
    import os
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import bench
    assert os.path.exists(bench.TRAFFIC_FILE)
    seen = set()
    for line in open(bench.TRAFFIC_FILE):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        assert len(f) == 7, line
        w, sigma, dtype = int(f[0]), int(f[1]), f[2]
        fetch, write = float(f[3]), float(f[4])
        assert 1 <= w <= 8 and 1 <= sigma <= 48 and dtype in ("f64", "f32")
        assert fetch > 0 and write > 0 and len(f[5]) >= 7 and f[6].startswith("k_spmv<")
        t = bench.measured_traffic(w, sigma, dtype, 1.0)
        assert t["bytes"] == int((2.0 * fetch + write) * 1024) and t["measured_at_commit"] == f[5]
        seen.add(w)
    assert {2, 3, 4, 5}.issubset(seen)                 # every configuration with a traffic-bound kernel
    assert bench.measured_traffic(2, 16, "f64", 2.0) is None          # a size sweep has no stored figure
    assert bench.measured_traffic(2, 7, "f64", 1.0) is None
