"""GPU parity of the 64-bit index variant (csr5l_convert_ex; Section 3.3 mentions a
64-bit tile_ptr).  On matrices the oracle can convert whole, every array is
compared bit by bit as for the 32-bit variant.  On a matrix of more than 2^31
nonzeros, generated in GPU memory, sampled tiles and rows are checked against
the oracle one by one, and the rest through properties that hold at any size."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from paper_1503_05032_amd import binding as B
from paper_1503_05032_amd import workloads as wl
from paper_1503_05032_amd import workloads_device as wd

from gpu_util import DeviceCsr, check_format, check_spmv, convert, tile_reference

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("sigma", [1, 4, 16, 33, 48])
def test_wide_edge_cases(sigma):
    for a in wl.edge_cases(64 * sigma):
        say("wide edge", sigma, a.name, a.m, a.n, a.nnz)
        d = DeviceCsr(a, wide=True)
        h = convert(d, sigma=sigma)
        check_format(d, h, (a.name, sigma))
        check_spmv(d, h, (a.name, sigma))
        B.csr5_to_csr(h)
        torch.cuda.synchronize()
        if a.nnz:
            assert np.array_equal(d.col_idx.cpu().numpy(), a.col_idx)
            assert np.array_equal(d.val.cpu().numpy(), a.val)
        B.csr5_free(h)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_wide_full_size_configs(cfg):
    a = wl.config(cfg)
    say("wide", a.stats())
    d = DeviceCsr(a, wide=True)
    h = convert(d, sigma=0)
    check_format(d, h, f"wide config{cfg}")
    check_spmv(d, h, f"wide config{cfg}")
    B.csr5_free(h)


def test_wide_and_narrow_handles_are_told_apart():
    a = wl.config(1)
    dn, dw = DeviceCsr(a), DeviceCsr(a, wide=True)
    hn, hw = convert(dn), convert(dw)
    assert B.csr5_get_arrays(hw, check=False) == B.CSR5_EINVAL
    assert B.csr5l_get_arrays(hn, check=False) == B.CSR5_EINVAL
    assert set(B.csr5l_get_arrays(hw)) == set(B.csr5_get_arrays(hn))
    # a wide handle made without a workspace, through the blocking path
    d2 = DeviceCsr(a, wide=True)
    h2 = convert(d2, use_workspace=False)
    check_format(d2, h2, "wide malloc")
    check_spmv(d2, h2, "wide malloc")
    # blocking path refuses a bad row_ptr and restores CSR order
    d3 = DeviceCsr(a, wide=True)
    d3.row_ptr[a.m // 2] = a.nnz + 5
    rc, h3 = B.csr5l_convert_ex(a.m, a.n, a.nnz, d3.row_ptr, d3.col_idx, d3.val, check=False)
    assert rc == B.CSR5_EINVAL and not h3
    assert np.array_equal(d3.col_idx.cpu().numpy(), a.col_idx)
    for h in (hn, hw, h2):
        B.csr5_free(h)


# --------------------------------------------------------------------------
# more than 2^31 nonzeros
# --------------------------------------------------------------------------
def test_wide_more_than_2g_nonzeros():
    free, _ = torch.cuda.mem_get_info()
    if free < 90 * 2**30:
        pytest.skip("needs about 80 GB of GPU memory")
    dev = torch.device("cuda:0")
    t_start = time.time()
    A = wd.huge_mixed(dev)
    m, n, nnz = A["m"], A["n"], A["nnz"]
    say("generated", A["name"], "m", m, "nnz", nnz, f"{time.time() - t_start:.1f}s")
    assert nnz > 2**31
    row_ptr_d, col, val, x = A["row_ptr"], A["col_idx"], A["val"], A["x"]
    col0, val0 = col.clone(), val.clone()               # CSR order, kept for the checks
    row_ptr = row_ptr_d.cpu().numpy()
    lens = np.diff(row_ptr)

    sigma = B.csr5_sigma_auto(nnz, m)
    T = 64 * sigma
    p, pc = (nnz + T - 1) // T, nnz // T
    assert B.csr5_workspace_bytes(m, 2**31 - 1, sigma) > 0
    ws = torch.empty(B.csr5l_workspace_bytes(m, nnz, sigma), dtype=torch.uint8, device=dev)
    h = B.csr5l_convert_ex(m, n, nnz, row_ptr_d, col, val, sigma=sigma, workspace=ws,
                           flags=B.CSR5_FLAG_NO_HOST_CHECK)
    st = B.csr5_status(h)
    say("converted, sigma", sigma, "tiles", p, "status", st)
    assert st & 3 == 0
    info = B.csr5_get_info(h)
    assert (info["p"], info["p_complete"], info["sigma"]) == (p, pc, sigma)
    W = info["desc_words_per_lane"]

    # ---- tile_ptr, every tile: the definition (Algorithm 4) as a property
    tp = B.csr5_read_array(h, B.CSR5_ARRAY_TILE_PTR, wide=True)
    assert tp.dtype == np.uint64 and tp.shape[0] == p + 1
    rows = (tp & np.uint64(2**63 - 1)).astype(np.int64)
    dirty = (tp >> np.uint64(63)).astype(bool)
    bnd = np.arange(p + 1, dtype=np.int64) * T
    assert np.all(rows <= m)
    assert np.all(row_ptr[rows] <= bnd)                                   # the row starts at or before the boundary
    nxt = np.minimum(rows + 1, m)
    assert np.all((row_ptr[nxt] > bnd) | (rows >= m))                     # and the next one after it
    assert rows[p] == m and not dirty[p]
    # empty-row flag: some empty row in [tile_ptr[t], min(tile_ptr[t+1], m-1)]
    n_empty_before = np.concatenate([[0], np.cumsum(lens == 0)])          # empty rows among rows < r
    last = np.minimum(rows[1:], m - 1)
    want_dirty = (n_empty_before[last + 1] - n_empty_before[rows[:-1]]) > 0
    assert np.array_equal(dirty[:-1], want_dirty)
    assert bool(st & B.CSR5_STATUS_HAS_DIRTY) == bool(want_dirty.any())
    say("tile_ptr ok; marked tiles", int(want_dirty.sum()))

    # ---- empty_offset_ptr, every tile: running count of the marked tiles' segments
    eop = B.csr5_read_array(h, B.CSR5_ARRAY_EMPTY_OFFSET_PTR, wide=True)
    assert eop.dtype == np.int64 and eop[0] == 0 and np.all(np.diff(eop) >= 0)
    assert np.all((np.diff(eop) > 0) == want_dirty[:pc])
    eo = B.csr5_read_array(h, B.CSR5_ARRAY_EMPTY_OFFSET)
    assert eo.shape[0] == eop[pc]
    td = B.csr5_read_array(h, B.CSR5_ARRAY_TILE_DESC).reshape(pc, W * 64)

    # ---- sampled tiles against the oracle, one by one
    rng = np.random.default_rng(7)
    long_rows = np.argsort(lens)[-wd.LONG_ROWS:]
    sample = set([0, 1, pc - 1, pc - 2]) | set(rng.integers(0, pc, 120).tolist())
    sample |= set(np.nonzero(want_dirty[:pc])[0][rng.integers(0, int(want_dirty[:pc].sum()), 40)].tolist())
    for r in long_rows:                                  # first, inner and last tile of every long row
        t0, t1 = int(row_ptr[r] // T), int((row_ptr[r + 1] - 1) // T)
        sample |= {t0, (t0 + t1) // 2, min(t1, pc - 1)}
    sample |= {int(2**31 // T) - 1, int(2**31 // T), int(2**31 // T) + 1}   # around entry 2^31
    sample = sorted(t for t in sample if 0 <= t < pc)
    for t in sample:
        lo, hi = t * T, (t + 1) * T
        r0, ref = tile_reference(row_ptr, m, n, t, T, sigma, col0[lo:hi].cpu().numpy(), val0[lo:hi].cpu().numpy())
        assert r0 == rows[t], t
        assert bool(ref.tile_ptr[0] >> 31) == bool(dirty[t]), t
        assert np.array_equal(td[t], ref.tile_desc), ("tile_desc", t)
        if dirty[t]:
            assert np.array_equal(eo[eop[t]:eop[t + 1]], ref.empty_offset), ("empty_offset", t)
        assert np.array_equal(col[lo:hi].cpu().numpy(), ref.col_idx), ("col_idx", t)
        assert np.array_equal(val[lo:hi].cpu().numpy().view(np.uint64), ref.val.view(np.uint64)), ("val", t)
    say("sampled tiles ok:", len(sample))
    if pc * T < nnz:                                     # the incomplete tile stays in CSR order
        assert torch.equal(col[pc * T:], col0[pc * T:]) and torch.equal(val[pc * T:], val0[pc * T:])

    # ---- SpMV
    y = torch.full((m,), float("nan"), dtype=torch.float64, device=dev)
    B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    # sampled rows against the oracle (Algorithm 1), one small CSR matrix of just those rows
    rows_s = set(rng.integers(0, m, 300).tolist()) | set(long_rows.tolist()) | {0, m - 1}
    rows_s |= set(rows[rng.integers(0, p, 100)].tolist())             # rows cut by a tile boundary
    rows_s |= set(np.nonzero(lens == 0)[0][:20].tolist())
    rows_s = np.array(sorted(r for r in rows_s if r < m), dtype=np.int64)
    cs = [col0[row_ptr[r]:row_ptr[r + 1]].cpu().numpy() for r in rows_s]
    vs = [val0[row_ptr[r]:row_ptr[r + 1]].cpu().numpy() for r in rows_s]
    rp_s = np.concatenate([[0], np.cumsum(lens[rows_s])]).astype(np.int32)
    y_ref, s_ref = oracle.csr_spmv(len(rows_s), rp_s, np.concatenate(cs), np.concatenate(vs), x.cpu().numpy())
    y_s = y[torch.from_numpy(rows_s).to(dev)].cpu().numpy()
    err = np.abs(y_s - y_ref)
    assert np.all(err <= 1e-12 * s_ref + 1e-300), (rows_s[np.argmax(err - 1e-12 * s_ref)], err.max())
    say("sampled rows ok:", len(rows_s), "worst err/sum|ax|", float((err / np.maximum(s_ref, 1e-300)).max()))
    # every row: rows without nonzeros are exactly 0; the others agree with a row-wise
    # sum formed by torch on the untouched copy (a consistency check over all rows;
    # the claim of parity rests on the oracle-checked samples above)
    y_t = torch.empty(m, dtype=torch.float64, device=dev)
    s_t = torch.empty(m, dtype=torch.float64, device=dev)
    ROWS = 400_000                                       # rows per step: about 1.4e8 entries
    for ra in range(0, m, ROWS):
        rb = min(m, ra + ROWS)
        ea, eb = int(row_ptr[ra]), int(row_ptr[rb])
        prod = val0[ea:eb] * x[col0[ea:eb].long()]
        off = row_ptr_d[ra:rb + 1] - ea
        y_t[ra:rb] = torch.segment_reduce(prod, "sum", offsets=off, unsafe=True)
        s_t[ra:rb] = torch.segment_reduce(prod.abs(), "sum", offsets=off, unsafe=True)
        torch.cuda.synchronize()
        say("  rows", ra, "..", rb, "summed by torch")
        del prod, off
    assert bool(((y - y_t).abs() <= 1e-12 * s_t + 1e-300).all())
    assert bool((y[torch.from_numpy(lens == 0).to(dev)] == 0).all())
    say("all rows consistent")

    # ---- a few timed SpMVs, for the record
    for _ in range(2):
        B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / 5 * 1e3
    say(f"spmv {ms:.3f} ms  = {2 * nnz / ms / 1e6:.1f} GFLOP/s, {12.86 * nnz / ms / 1e6:.0f} GB/s of the byte model")

    # ---- back to CSR, bit-exact
    B.csr5_to_csr(h)
    torch.cuda.synchronize()
    for e0 in range(0, nnz, 1 << 29):
        e1 = min(nnz, e0 + (1 << 29))
        assert torch.equal(col[e0:e1], col0[e0:e1]) and torch.equal(val[e0:e1], val0[e0:e1])
    B.csr5_free(h)
    say(f"done in {time.time() - t_start:.1f}s")


def test_int32_variant_at_its_largest_size():
    """nnz = 2^31 - 1 through the 32-bit entry points: the first rows of the large
    matrix, the last row cut so that the count is exact.  1023 entries follow the
    last complete tile, so the incomplete-tile path works right below the top of
    the index range."""
    free, _ = torch.cuda.mem_get_info()
    if free < 90 * 2**30:
        pytest.skip("needs about 80 GB of GPU memory")
    dev = torch.device("cuda:0")
    A = wd.huge_mixed(dev)
    nnz = 2**31 - 1
    rp64 = A["row_ptr"]
    m = int(torch.searchsorted(rp64, torch.tensor([nnz], device=dev), right=True).item())   # rows 0..m-1 start at or before nnz
    rp64 = rp64[:m + 1].clone()
    rp64[m] = nnz                                        # the last row ends where int32 ends
    if int(rp64[m - 1].item()) == nnz:
        m -= 1
        rp64 = rp64[:m + 1]
    n = A["n"]
    row_ptr_d = rp64.to(torch.int32)
    col, val, x = A["col_idx"][:nnz].clone(), A["val"][:nnz].clone(), A["x"]
    col0, val0 = A["col_idx"], A["val"]                 # CSR order (the clones get transposed)
    row_ptr = row_ptr_d.cpu().numpy()
    lens = np.diff(row_ptr.astype(np.int64))
    say("m", m, "nnz", nnz, "last row length", int(lens[-1]))
    sigma = 16
    T = 64 * sigma
    p, pc = (nnz + T - 1) // T, nnz // T
    assert nnz - pc * T == 1023
    ws = torch.empty(B.csr5_workspace_bytes(m, nnz, sigma), dtype=torch.uint8, device=dev)
    h = B.csr5_convert_ex(m, n, nnz, row_ptr_d, col, val, sigma=sigma, workspace=ws)     # blocking, with the checks
    assert B.csr5_status(h) & 3 == 0
    tp = B.csr5_read_array(h, B.CSR5_ARRAY_TILE_PTR)
    rows = (tp & np.uint32(0x7fffffff)).astype(np.int64)
    bnd = np.arange(p + 1, dtype=np.int64) * T
    assert rows[p] == m and np.all(row_ptr[rows] <= bnd)
    assert np.all((row_ptr[np.minimum(rows + 1, m)] > bnd) | (rows >= m))
    rng = np.random.default_rng(3)
    td = B.csr5_read_array(h, B.CSR5_ARRAY_TILE_DESC).reshape(pc, -1)
    rp_wide = row_ptr.astype(np.int64)
    for t in sorted(set(rng.integers(0, pc, 40).tolist()) | {0, pc - 1, pc - 2}):
        lo, hi = t * T, (t + 1) * T
        r0, ref = tile_reference(rp_wide, m, n, t, T, sigma, col0[lo:hi].cpu().numpy(), val0[lo:hi].cpu().numpy())
        assert r0 == rows[t] and np.array_equal(td[t], ref.tile_desc), t
        assert np.array_equal(col[lo:hi].cpu().numpy(), ref.col_idx), t
    y = torch.full((m,), float("nan"), dtype=torch.float64, device=dev)
    B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    rows_s = np.unique(np.concatenate([rng.integers(0, m, 200), np.arange(m - 40, m), np.argsort(lens)[-3:], [0]]))
    cs = np.concatenate([col0[row_ptr[r]:row_ptr[r + 1]].cpu().numpy() for r in rows_s])
    vs = np.concatenate([val0[row_ptr[r]:row_ptr[r + 1]].cpu().numpy() for r in rows_s])
    rp_s = np.concatenate([[0], np.cumsum(lens[rows_s])]).astype(np.int32)
    y_ref, s_ref = oracle.csr_spmv(len(rows_s), rp_s, cs, vs, x.cpu().numpy())
    err = np.abs(y[torch.from_numpy(rows_s).to(dev)].cpu().numpy() - y_ref)
    assert np.all(err <= 1e-12 * s_ref + 1e-300)
    assert bool((y[torch.from_numpy(lens == 0).to(dev)] == 0).all()) and not bool(torch.isnan(y).any())
    # the CSR baselines at the same size (their entry counters also run up to 2^31 - 1)
    yb = torch.full((m,), float("nan"), dtype=torch.float64, device=dev)
    B.csr5_to_csr(h)
    B.csr5_baseline_csr_vector(m, nnz, row_ptr_d, col, val, x, yb)
    torch.cuda.synchronize()
    assert bool(((y - yb).abs() <= 1e-6 * (y.abs() + 1)).all())
    assert torch.equal(col, col0[:nnz])
    B.csr5_free(h)


def test_largest_row_count():
    """m = 2^31 - 2 rows, nearly all of them empty: the row-parallel conversion
    kernels and the zero-fill of the fix-up run over 2^31 threads / rows."""
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2**30:
        pytest.skip("needs about 40 GB of GPU memory")
    dev = torch.device("cuda:0")
    m, n, sigma = 2**31 - 2, 4096, 4
    T = 64 * sigma
    rng = np.random.default_rng(5)
    live = np.unique(np.concatenate([[0, 1, 5, 1000, 2**20, 2**30 - 1, 2**30, m - 2, m - 1],
                                     rng.integers(0, m, 60), m - 1 - rng.integers(0, 5000, 20)]))
    lens_live = rng.integers(1, 300, live.shape[0])
    lens_live[3] = 5 * T + 7                                   # one row over several tiles
    nnz = int(lens_live.sum())
    row_ptr_d = torch.zeros(m + 1, dtype=torch.int32, device=dev)
    for r, L in zip(live.tolist(), lens_live.tolist()):         # row_ptr[k] = entries in rows < k
        row_ptr_d[r + 1:] += L
    say("m", m, "nnz", nnz, "rows with nonzeros", live.shape[0])
    col_h = np.concatenate([np.sort(rng.choice(n, L, replace=False)) for L in lens_live]).astype(np.int32)
    val_h = rng.uniform(-1, 1, nnz)
    x_h = rng.uniform(-1, 1, n)
    col, val, x = (torch.from_numpy(a).to(dev) for a in (col_h, val_h, x_h))
    y = torch.full((m,), float("nan"), dtype=torch.float64, device=dev)
    h = B.csr5_convert_ex(m, n, nnz, row_ptr_d, col, val, sigma=sigma)       # hipMalloc inside, blocking checks
    st = B.csr5_status(h)
    assert st & 3 == 0 and st & B.CSR5_STATUS_HAS_EMPTY_ROWS and st & B.CSR5_STATUS_HAS_DIRTY
    say("converted")
    row_ptr = row_ptr_d.cpu().numpy()
    say("row_ptr on the host")
    ref = oracle.convert(m, n, nnz, row_ptr, col_h, val_h, 64, sigma)
    say("oracle converted")
    for which, want in ((B.CSR5_ARRAY_TILE_PTR, ref.tile_ptr), (B.CSR5_ARRAY_TILE_DESC, ref.tile_desc),
                        (B.CSR5_ARRAY_EMPTY_OFFSET_PTR, ref.empty_offset_ptr),
                        (B.CSR5_ARRAY_EMPTY_OFFSET, ref.empty_offset)):
        assert np.array_equal(B.csr5_read_array(h, which), want), which
    assert np.array_equal(col.cpu().numpy(), ref.col_idx)
    B.csr5_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    say("spmv done")
    # the rows with nonzeros against Algorithm 1 on a matrix of just those rows; every other row exactly 0
    rp_s = np.concatenate([[0], np.cumsum(lens_live)]).astype(np.int32)
    y_ref, s_ref = oracle.csr_spmv(live.shape[0], rp_s, col_h, val_h, x_h)
    y_live = y[torch.from_numpy(live).to(dev)].cpu().numpy()
    assert np.all(np.abs(y_live - y_ref) <= 1e-12 * s_ref + 1e-300)
    assert not bool(torch.isnan(y).any())
    assert int((y != 0).sum().item()) == int((y_live != 0).sum())
    B.csr5_free(h)
