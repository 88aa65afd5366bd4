"""GPU parity: the HIP library (through its C ABI) against the CPU oracle.
Format arrays bit-exact; y within 1e-12 * sum_j|a_ij x_j| + 1e-300 per row."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_1503_05032_amd import binding as B
from paper_1503_05032_amd import workloads as wl

from gpu_util import DeviceCsr, check_format, check_spmv, convert, second_kernel_ms

pytestmark = pytest.mark.gpu

SIGMAS_EDGE = [1, 4, 7, 16, 20, 32, 33, 46, 48]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("sigma", SIGMAS_EDGE)
def test_edge_cases(sigma):
    T = 64 * sigma
    for a in wl.edge_cases(T):
        say("edge", sigma, a.name, a.m, a.n, a.nnz)
        d = DeviceCsr(a)
        h = convert(d, sigma=sigma)
        check_format(d, h, (a.name, sigma))
        check_spmv(d, h, (a.name, sigma))
        B.csr5_to_csr(h)
        torch.cuda.synchronize()
        if a.nnz:
            assert np.array_equal(d.col_idx.cpu().numpy(), a.col_idx), (a.name, "to_csr col")
            assert np.array_equal(d.val.cpu().numpy(), a.val), (a.name, "to_csr val")
        B.csr5_free(h)


@pytest.mark.parametrize("sigma", list(range(1, 49)))
def test_every_sigma_small(sigma):
    a = wl.tiny_uniform(m=1500, n=1200, max_len=25, seed=sigma)
    say("sigma", sigma, a.nnz)
    d = DeviceCsr(a)
    h = convert(d, sigma=sigma)
    check_format(d, h, ("tiny", sigma))
    check_spmv(d, h, ("tiny", sigma))
    B.csr5_free(h)


def test_config1_auto_sigma_and_plain_convert():
    a = wl.config(1)
    d = DeviceCsr(a)
    say("config1 via csr5_convert", a.stats())
    h = B.csr5_convert(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val)     # hipMalloc path, auto sigma
    info = B.csr5_get_info(h)
    assert info["sigma"] == B.csr5_sigma_auto(a.nnz, a.m)
    check_format(d, h, "config1")
    check_spmv(d, h, "config1")
    # a second x through the same handle, and the non-_ex entry point
    x2 = np.random.default_rng(9).uniform(-1, 1, size=a.n)
    check_spmv(d, h, "config1-x2", x=x2)
    d.y.fill_(float("nan"))
    B.csr5_spmv(h, d.x, d.y)
    torch.cuda.synchronize()
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, x2)
    assert np.all(np.abs(d.y.cpu().numpy() - y_ref) <= 1e-12 * s + 1e-300)
    B.csr5_free(h)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 6, 8])
def test_full_size_configs(cfg):
    say("generating config", cfg)
    a = wl.config(cfg)
    say(a.stats())
    d = DeviceCsr(a)
    h = convert(d, sigma=0)
    say("converted; sigma", B.csr5_get_info(h)["sigma"])
    check_format(d, h, f"config{cfg}")
    say("format ok")
    worst = check_spmv(d, h, f"config{cfg}")
    say("spmv ok, worst err/sum|ax| =", worst)
    B.csr5_free(h)


@pytest.mark.parametrize("sigma,wide", [(4, False), (2, True)])
def test_many_marked_tiles(sigma, wide):
    """More than 65536 tiles, a third of them holding empty rows: the layout of
    empty_offset is then scanned by many workgroups instead of one."""
    a = wl.config(4)
    d = DeviceCsr(a, wide=wide)
    h = convert(d, sigma=sigma)
    info = B.csr5_get_info(h)
    say("tiles", info["p"], "empty_offset_len", info["empty_offset_len"])
    assert info["p_complete"] > 65536 and info["empty_offset_len"] > 0
    check_format(d, h, ("many marked tiles", sigma, wide))
    check_spmv(d, h, ("many marked tiles", sigma, wide))
    B.csr5_free(h)


def test_workspace_and_malloc_paths_agree():
    a = wl.config(3, scale=0.02)
    d1, d2 = DeviceCsr(a), DeviceCsr(a)
    h1 = convert(d1, sigma=12, use_workspace=True, flags=B.CSR5_FLAG_NO_HOST_CHECK)
    h2 = convert(d2, sigma=12, use_workspace=False)
    for which in range(4):
        assert np.array_equal(B.csr5_read_array(h1, which), B.csr5_read_array(h2, which))
    check_format(d1, h1, "ws")
    check_spmv(d1, h1, "ws")
    check_spmv(d2, h2, "malloc")
    B.csr5_free(h1)
    B.csr5_free(h2)


def test_error_paths():
    a = wl.tiny_uniform(m=300, n=300, seed=1)
    d = DeviceCsr(a)
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val, sigma=49, check=False)
    assert rc == B.CSR5_ERANGE and not h
    rc, h = B.csr5_convert_ex(-1, a.n, a.nnz, d.row_ptr, d.col_idx, d.val, check=False)
    assert rc == B.CSR5_EINVAL and not h
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, None, d.col_idx, d.val, check=False)
    assert rc == B.CSR5_EINVAL and not h
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, None, d.val, check=False)
    assert rc == B.CSR5_EINVAL and not h
    # nnz that does not match row_ptr[m]: caught by the device-side check of the last row
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz - 1, d.row_ptr, d.col_idx, d.val, check=False)
    assert rc == B.CSR5_EINVAL and not h
    assert np.array_equal(d.col_idx.cpu().numpy(), a.col_idx) and np.array_equal(d.val.cpu().numpy(), a.val)
    # row_ptr[0] != 0
    d0 = DeviceCsr(a)
    d0.row_ptr[0] = 1
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, d0.row_ptr, d0.col_idx, d0.val, check=False)
    assert rc == B.CSR5_EINVAL and not h
    assert np.array_equal(d0.col_idx.cpu().numpy(), a.col_idx)
    # workspace too small
    ws = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val, sigma=4, workspace=ws, check=False)
    assert rc == B.CSR5_ENOMEM and not h
    assert B.csr5_spmv(None, d.x, d.y, check=False) == B.CSR5_EINVAL
    assert B.csr5_free(None) == B.CSR5_OK
    # decreasing row_ptr in the middle
    rp = a.row_ptr.copy()
    rp[100], rp[101] = rp[101] + 3, rp[100]
    d2 = DeviceCsr(a)
    d2.row_ptr = torch.from_numpy(rp).to("cuda:0")
    # (a) blocking variant: refused, col_idx / val back in CSR order
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, d2.row_ptr, d2.col_idx, d2.val, sigma=4, check=False)
    assert rc == B.CSR5_EINVAL and not h
    assert np.array_equal(d2.col_idx.cpu().numpy(), a.col_idx)
    assert np.array_equal(d2.val.cpu().numpy(), a.val)
    # (b) asynchronous variant: a handle, the verdict in the status word, SpMV touches nothing
    h = B.csr5_convert_ex(a.m, a.n, a.nnz, d2.row_ptr, d2.col_idx, d2.val, sigma=4,
                          flags=B.CSR5_FLAG_NO_HOST_CHECK)
    d2.y.fill_(123.0)
    B.csr5_spmv(h, d2.x, d2.y)
    torch.cuda.synchronize()
    assert np.all(d2.y.cpu().numpy() == 123.0)
    assert B.csr5_status(h) & B.CSR5_STATUS_BAD_ROW_PTR
    B.csr5_free(h)
    # a column index out of range
    ci = a.col_idx.copy()
    ci[77] = a.n + 5
    d3 = DeviceCsr(a)
    d3.col_idx = torch.from_numpy(ci).to("cuda:0")
    rc, h = B.csr5_convert_ex(a.m, a.n, a.nnz, d3.row_ptr, d3.col_idx, d3.val, sigma=4, check=False)
    assert rc == B.CSR5_EINVAL and not h
    assert np.array_equal(d3.col_idx.cpu().numpy(), ci)
    h = B.csr5_convert_ex(a.m, a.n, a.nnz, d3.row_ptr, d3.col_idx, d3.val, sigma=4,
                          flags=B.CSR5_FLAG_NO_HOST_CHECK)
    assert B.csr5_status(h) & B.CSR5_STATUS_BAD_COL_IDX
    d3.y.fill_(123.0)
    B.csr5_spmv(h, d3.x, d3.y)
    torch.cuda.synchronize()
    assert np.all(d3.y.cpu().numpy() == 123.0)      # nothing gathered, nothing stored
    B.csr5_free(h)


def test_repeatability_within_tolerance():
    a = wl.config(4, scale=0.02)
    d = DeviceCsr(a)
    h = convert(d, sigma=0)
    ys = []
    for _ in range(3):
        check_spmv(d, h, "repeat")
        ys.append(d.y.cpu().numpy().copy())
    _, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    assert np.all(np.abs(ys[0] - ys[1]) <= 2e-12 * s + 1e-300)
    assert np.all(np.abs(ys[0] - ys[2]) <= 2e-12 * s + 1e-300)
    B.csr5_free(h)


def _check_y(y, a, label):
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    err = np.abs(y - y_ref)
    bad = np.nonzero(~(err <= 1e-12 * s + 1e-300))[0]
    assert bad.size == 0, (label, int(bad.size), int(bad[0]))


def test_csr_baselines_match_oracle():
    """CSR-scalar and CSR-vector (Section 2.2.1) on the untouched CSR arrays."""
    mats = wl.edge_cases(64 * 4) + [wl.config(1), wl.config(3, scale=0.01), wl.config(4, scale=0.01)]
    for a in mats:
        if a.m == 0:
            continue
        say("baseline", a.name, a.m, a.nnz)
        d = DeviceCsr(a)
        d.y.fill_(float("nan"))
        B.csr5_baseline_csr_scalar(a.m, d.row_ptr, d.col_idx, d.val, d.x, d.y)
        torch.cuda.synchronize()
        _check_y(d.y.cpu().numpy()[:a.m], a, (a.name, "scalar"))
        for lanes in (0, 2, 4, 8, 16, 32, 64):
            d.y.fill_(float("nan"))
            B.csr5_baseline_csr_vector(a.m, a.nnz, d.row_ptr, d.col_idx, d.val, d.x, d.y, lanes_per_row=lanes)
            torch.cuda.synchronize()
            _check_y(d.y.cpu().numpy()[:a.m], a, (a.name, "vector", lanes))
    assert B.csr5_baseline_csr_vector(5, 5, d.row_ptr, d.col_idx, d.val, d.x, d.y, lanes_per_row=3,
                                      check=False) == B.CSR5_EINVAL


@pytest.mark.parametrize("kind", ["carry_array", "look_behind"])
def test_side_stream_and_graph_replay(kind):
    """csr5_spmv_ex only enqueues kernels: it runs on any stream and can be
    captured into a HIP graph; every replay must equal the eager result.  Both
    ways of forming cross-tile sums: through the auxiliary array (a matrix with
    long rows; at this size inside the tile kernel, whose meeting words and
    counters every replay must find at rest) and by look-behind."""
    if kind == "carry_array":
        a = wl.config(4, scale=0.02)       # has empty rows, long rows and an incomplete tile
    else:
        a = wl.config(2, scale=0.03)       # 27-point stencil: every row is finished by the tile it ends in
    d = DeviceCsr(a)
    h = convert(d, sigma=0)
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        d.y.fill_(float("nan"))
        B.csr5_spmv_ex(h, d.x, d.y)          # binding passes the current (= side) stream
    side.synchronize()
    assert np.all(np.abs(d.y.cpu().numpy()[:a.m] - y_ref) <= 1e-12 * s + 1e-300)
    # graph capture + replays with the eager path in between
    xs = [np.random.default_rng(k).standard_normal(a.n) for k in range(3)]
    xg = d.x.clone()
    yg = torch.empty_like(d.y)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.csr5_spmv_ex(h, xg, yg)
    for k, xk in enumerate(xs):
        xg.copy_(torch.from_numpy(xk))
        yg.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = yg.cpu().numpy()[:a.m].copy()
        check_spmv(d, h, ("eager", k), x=xk)                 # eager work between replays
        yk, sk = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, xk)
        assert np.all(np.abs(got - yk) <= 1e-12 * sk + 1e-300), ("replay", k)
    B.csr5_free(h)


@pytest.mark.parametrize("sigma", [4, 16, 33])
@pytest.mark.parametrize("wide", [False, True])
def test_structured_cases(sigma, wide):
    """Arrowhead, band, dense diagonal blocks, dense triangle, unsorted rows with
    repeated column indices."""
    for a in wl.structured_cases(64 * sigma):
        say("structured", sigma, wide, a.name, a.m, a.n, a.nnz)
        d = DeviceCsr(a, wide=wide)
        h = convert(d, sigma=sigma)
        check_format(d, h, (a.name, sigma))
        check_spmv(d, h, (a.name, sigma))
        B.csr5_free(h)


def test_conversion_in_a_graph():
    """With a workspace and CSR5_FLAG_NO_HOST_CHECK the conversion only enqueues
    kernels (no allocation, no memset, no wait), so conversion + SpMV can be
    captured together; every replay converts the restored CSR arrays again."""
    a = wl.config(4, scale=0.03)
    d = DeviceCsr(a)
    col0, val0 = d.col_idx.clone(), d.val.clone()
    sigma = 12
    ws = torch.empty(B.csr5_workspace_bytes(a.m, a.nnz, sigma), dtype=torch.uint8, device="cuda:0")
    yg = torch.empty_like(d.y)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        d.col_idx.copy_(col0)
        d.val.copy_(val0)
        h = B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val, sigma=sigma, workspace=ws,
                              flags=B.CSR5_FLAG_NO_HOST_CHECK)
        B.csr5_spmv_ex(h, d.x, yg)
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    for k in range(3):
        ws.fill_(0xAB)                                   # the replay must rebuild everything
        yg.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.all(np.abs(yg.cpu().numpy()[:a.m] - y_ref) <= 1e-12 * s + 1e-300), ("replay", k)
        check_format(d, h, ("graph", k))
    B.csr5_free(h)


@pytest.mark.parametrize("wide,seed,cases", [(False, 2024, 40), (True, 2025, 30), (False, 7, 60)])
def test_random_matrices(wide, seed, cases):
    """Randomised parity: mixed row-length distributions (empty runs, short rows,
    a few rows longer than a tile), random shapes and sigma; 32- and 64-bit indices."""
    rng = np.random.default_rng(seed)
    for case in range(cases):
        sigma = int(rng.integers(1, 49))
        T = 64 * sigma
        m = int(rng.integers(1, 3000))
        n = int(rng.integers(1, 5000))
        kind = case % 4
        if kind == 0:
            lens = rng.geometric(0.2, size=m) - 1
        elif kind == 1:
            lens = rng.integers(0, 4, size=m) * (rng.random(m) < 0.5)
        elif kind == 2:
            lens = rng.integers(0, 30, size=m)
            lens[rng.integers(0, m, size=3)] = rng.integers(T, 3 * T + 2, size=3)
        else:
            lens = np.zeros(m, dtype=np.int64)
            idx = rng.integers(0, m, size=max(1, m // 50))
            lens[idx] = rng.integers(1, 2 * T, size=idx.size)
        a = wl.from_row_lengths(lens, n, seed=seed + case, name=f"random{case}")
        say("random", case, "sigma", sigma, a.m, a.n, a.nnz)
        d = DeviceCsr(a, wide=wide)
        h = convert(d, sigma=sigma, use_workspace=bool(case % 2))
        check_format(d, h, (a.name, sigma))
        check_spmv(d, h, (a.name, sigma))
        B.csr5_free(h)


# ---------------------------------------------------------------- single precision
TOL32 = 1e-5      # depth of any addition chain <= sigma + 6 + 6 + a few (<= 64): 64 * 2^-24 = 3.8e-6


def _run32(a, sigma):
    dev = torch.device("cuda:0")
    val32 = a.val.astype(np.float32)
    x32 = a.x.astype(np.float32)
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col = torch.from_numpy(a.col_idx).to(dev) if a.nnz else torch.zeros(4, dtype=torch.int32, device=dev)
    val = torch.from_numpy(val32).to(dev) if a.nnz else torch.zeros(4, dtype=torch.float32, device=dev)
    x = torch.from_numpy(x32).to(dev) if a.n else torch.zeros(1, dtype=torch.float32, device=dev)
    y = torch.full((max(a.m, 1),), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty(B.csr5_workspace_bytes(a.m, a.nnz, sigma), dtype=torch.uint8, device=dev)
    h = B.csr5s_convert_ex(a.m, a.n, a.nnz, row_ptr, col, val, sigma=sigma, workspace=ws)
    info = B.csr5_get_info(h)
    ref = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, val32.astype(np.float64), 64, info["sigma"])
    assert np.array_equal(B.csr5_read_array(h, B.CSR5_ARRAY_TILE_PTR), ref.tile_ptr)
    assert np.array_equal(B.csr5_read_array(h, B.CSR5_ARRAY_TILE_DESC), ref.tile_desc)
    assert np.array_equal(B.csr5_read_array(h, B.CSR5_ARRAY_EMPTY_OFFSET_PTR), ref.empty_offset_ptr)
    assert np.array_equal(B.csr5_read_array(h, B.CSR5_ARRAY_EMPTY_OFFSET), ref.empty_offset)
    if a.nnz:
        assert np.array_equal(col.cpu().numpy(), ref.col_idx)
        assert np.array_equal(val.cpu().numpy().astype(np.float64), ref.val)     # bit-exact in float
    B.csr5s_spmv_ex(h, x, y)
    torch.cuda.synchronize()
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, val32.astype(np.float64), x32.astype(np.float64))
    got = y.cpu().numpy()[:a.m].astype(np.float64)
    bad = np.nonzero(~(np.abs(got - y_ref) <= TOL32 * s + 1e-30))[0]
    assert bad.size == 0, (a.name, sigma, int(bad.size), int(bad[0]), got[bad[0]], y_ref[bad[0]], s[bad[0]])
    assert np.all(got[np.diff(a.row_ptr) == 0] == 0.0)
    # the double-precision calls refuse a single-precision handle: the binding by the
    # tensors' type, the library (given raw addresses) by the handle's
    with pytest.raises(ValueError):
        B.csr5_spmv_ex(h, x, y, check=False)
    assert B.csr5_spmv_ex(h, x.data_ptr(), y.data_ptr(), check=False) == B.CSR5_EINVAL
    B.csr5_to_csr(h)
    torch.cuda.synchronize()
    if a.nnz:
        assert np.array_equal(col.cpu().numpy(), a.col_idx)
        assert np.array_equal(val.cpu().numpy(), val32)
    B.csr5_free(h)


@pytest.mark.parametrize("sigma", [4, 16, 33, 48])
def test_single_precision_edge_cases(sigma):
    for a in wl.edge_cases(64 * sigma):
        if a.name == "wide_values":
            continue                      # 16 decades of magnitudes do not fit single precision's range of sums
        say("f32 edge", sigma, a.name)
        _run32(a, sigma)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_single_precision_full_size(cfg):
    a = wl.config(cfg)
    say("f32", a.stats())
    _run32(a, 0)


def test_profile_helper_leaves_y_correct():
    """csr5_spmv_profile launches each kernel many times in a row and then runs one
    full SpMV: durations are positive and y is A*x afterwards."""
    a = wl.config(4, scale=0.02)
    d = DeviceCsr(a)
    h = convert(d, sigma=0)
    d.y.fill_(float("nan"))
    ms_tiles, ms_fixup = B.csr5_spmv_profile(h, d.x, d.y, reps=20)
    torch.cuda.synchronize()
    assert 0 < ms_tiles < 10 and 0 <= ms_fixup < 10      # (no second kernel for this matrix: its series is empty)
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    assert np.all(np.abs(d.y.cpu().numpy()[:a.m] - y_ref) <= 1e-12 * s + 1e-300)
    B.csr5_free(h)


@pytest.mark.parametrize("row_len,one_kernel", [(32, True), (33, True), (34, True), (96, True), (160, True), (161, True),
                                                (163, False), (701, False)])
def test_row_lengths_around_the_look_behind_limits(row_len, one_kernel):
    """Every row has `row_len` entries, at three tile heights (workgroups of four
    and of two tiles).  Up to 161 entries per row the tile kernel completes the
    rows that cross tiles by re-reading their heads; with 163 (a prime, and more
    workgroups than that: every offset into a row occurs at a workgroup's first
    tile) some such tile starts more than 160 entries into a row and the sums go
    through the auxiliary array, inside the same kernel at this size.
    Either way y is the oracle's and there is no second kernel."""
    m = 40_000 // row_len * 64 + 37
    a = wl.from_row_lengths(np.full(m, row_len), 5 * row_len + 1000, seed=row_len, name=f"rows{row_len}")
    for sigma in (8, 16, 24):
        d = DeviceCsr(a)
        h = convert(d, sigma=sigma)
        say("row length", row_len, "sigma", sigma, a.m, a.nnz)
        check_format(d, h, (a.name, sigma))
        check_spmv(d, h, (a.name, sigma))
        ms_second = second_kernel_ms(h, d.x, d.y)
        assert ms_second < 1e-3, (row_len, sigma, ms_second, one_kernel)
        _check_y(d.y.cpu().numpy()[:a.m], a, ("after profile", row_len, sigma))
        B.csr5_free(h)


def test_stencil_beyond_the_far_record_limit():
    """A 27-point stencil with more than 28 million nonzeros: its look-behind
    records hold the near part only (a different record stride), the SpMV is
    still one kernel, format and result are the oracle's."""
    a = wl.stencil27(g=104)
    assert a.nnz > 28_000_000
    d = DeviceCsr(a)
    h = convert(d, sigma=16)
    say("stencil 104^3", a.nnz)
    check_format(d, h, (a.name, 16))
    check_spmv(d, h, (a.name, 16))
    ms_second = second_kernel_ms(h, d.x, d.y)
    assert ms_second < 1e-3, ms_second
    _check_y(d.y.cpu().numpy()[:a.m], a, "after profile")
    B.csr5_free(h)


@pytest.mark.parametrize("sigma", [8, 16, 24])
def test_single_precision_long_heads(sigma):
    """Rows of 100 entries in single precision: the look-behind reads the far part
    of the records (4-byte values in 8-byte slots), the SpMV is one kernel."""
    a = wl.from_row_lengths(np.full(9000, 100), 3000, seed=77, name="rows100")
    _run32(a, sigma)
    dev = torch.device("cuda:0")
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col = torch.from_numpy(a.col_idx).to(dev)
    val = torch.from_numpy(a.val.astype(np.float32)).to(dev)
    x = torch.from_numpy(a.x.astype(np.float32)).to(dev)
    y = torch.empty(a.m, dtype=torch.float32, device=dev)
    h = B.csr5s_convert_ex(a.m, a.n, a.nnz, row_ptr, col, val, sigma=sigma)
    _, ms_second = B.csr5s_spmv_profile(h, x, y, reps=50)
    torch.cuda.synchronize()
    assert ms_second < 1e-3, ms_second
    B.csr5_free(h)


@pytest.mark.parametrize("f32", [False, True])
def test_bound_call_is_the_same_call(f32):
    """binding.csr5_spmv_bound marshals once and then only makes the C call: the
    result is csr5_spmv_ex's, bit for bit, on a matrix without atomics in its sums."""
    a = wl.config(2, scale=0.05)
    dev = torch.device("cuda:0")
    dt, npdt = (torch.float32, np.float32) if f32 else (torch.float64, np.float64)
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col = torch.from_numpy(a.col_idx).to(dev)
    val = torch.from_numpy(a.val.astype(npdt)).to(dev)
    x = torch.from_numpy(a.x.astype(npdt)).to(dev)
    y1 = torch.full((a.m,), float("nan"), dtype=dt, device=dev)
    y2 = torch.full((a.m,), float("nan"), dtype=dt, device=dev)
    conv, spmv = (B.csr5s_convert_ex, B.csr5s_spmv_ex) if f32 else (B.csr5_convert_ex, B.csr5_spmv_ex)
    h = conv(a.m, a.n, a.nnz, row_ptr, col, val)
    spmv(h, x, y1)
    call = B.csr5_spmv_bound(h, x, y2)
    call()
    call()
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val.astype(npdt).astype(np.float64),
                               a.x.astype(npdt).astype(np.float64))
    assert np.all(np.abs(y2.cpu().numpy().astype(np.float64) - y_ref) <= (TOL32 if f32 else 1e-12) * s + 1e-30)
    with pytest.raises(ValueError):
        B.csr5_spmv_bound(h, x, y2[:a.m - 1])
    B.csr5_free(h)


@pytest.mark.parametrize("sigma,f32", [(16, False), (7, False), (48, False), (16, True)])
def test_stream_floor_reads_only_and_stays_inside_y(sigma, f32):
    """csr5_stream_floor times a bare read of the tile streams, with and without
    the rows of y.  It must leave the matrix alone (an SpMV afterwards is still
    the oracle's), write nothing outside the m entries of y, refuse a y that is
    too short, and not be slower than the tile kernel by more than timing noise."""
    a = wl.config(2, scale=0.2)
    dev = torch.device("cuda:0")
    dt, npdt = (torch.float32, np.float32) if f32 else (torch.float64, np.float64)
    row_ptr = torch.from_numpy(a.row_ptr).to(dev)
    col = torch.from_numpy(a.col_idx).to(dev)
    val = torch.from_numpy(a.val.astype(npdt)).to(dev)
    x = torch.from_numpy(a.x.astype(npdt)).to(dev)
    y = torch.full((a.m,), float("nan"), dtype=dt, device=dev)
    conv, spmv, profile = ((B.csr5s_convert_ex, B.csr5s_spmv_ex, B.csr5s_spmv_profile) if f32 else
                           (B.csr5_convert_ex, B.csr5_spmv_ex, B.csr5_spmv_profile))
    h = conv(a.m, a.n, a.nnz, row_ptr, col, val, sigma=sigma)
    scratch = torch.full((a.m + 64,), 7.0, dtype=dt, device=dev)
    say("stream floor", sigma, "f32" if f32 else "f64")
    read_ms, read_write_ms = B.csr5_stream_floor(h, scratch, reps=20)
    torch.cuda.synchronize()
    assert 0 < read_ms < 10 and 0 < read_write_ms < 10
    assert bool(torch.all(scratch[a.m:] == 7.0))
    with pytest.raises(B.Csr5Error):
        B.csr5_stream_floor(h, scratch[:a.m - 1], reps=1)
    tiles_ms, _ = profile(h, x, y, reps=20)
    assert read_write_ms < 1.5 * tiles_ms + 0.005, (read_write_ms, tiles_ms)     # (measured first, possibly at idle clocks)
    y.fill_(float("nan"))
    spmv(h, x, y)
    torch.cuda.synchronize()
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val.astype(npdt).astype(np.float64),
                               a.x.astype(npdt).astype(np.float64))
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - y_ref) <= (TOL32 if f32 else 1e-12) * s + 1e-30)
    B.csr5_free(h)


@pytest.mark.parametrize("sigma", [4, 16, 40])
def test_non_finite_x_stays_in_its_rows(sigma):
    """An infinite or NaN entry of x must reach exactly the rows that reference its
    column: segment sums are formed directly, not as differences of tile-wide
    prefix sums (the hazard of taking Algorithm 6 literally)."""
    a = wl.from_row_lengths(np.random.default_rng(sigma).integers(0, 40, size=1500), 600, seed=sigma, name="nonfinite")
    x = a.x.copy()
    x[7] = np.inf
    x[300] = -np.inf
    x[451] = np.nan
    d = DeviceCsr(a)
    h = convert(d, sigma=sigma)
    d.x = torch.from_numpy(x).to("cuda:0")
    d.y.fill_(0.0)
    B.csr5_spmv_ex(h, d.x, d.y)
    torch.cuda.synchronize()
    y = d.y.cpu().numpy()[:a.m]
    with np.errstate(invalid="ignore", over="ignore"):
        y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, x)
    fin = np.isfinite(y_ref)
    assert 50 < (~fin).sum() < a.m - 50                       # both kinds of rows are present
    assert np.all(np.isfinite(y[fin])) and np.all(np.abs(y[fin] - y_ref[fin]) <= 1e-12 * s[fin] + 1e-300)
    assert np.array_equal(np.isnan(y[~fin]), np.isnan(y_ref[~fin]))
    inf_rows = ~fin & ~np.isnan(y_ref)
    assert np.array_equal(y[inf_rows], y_ref[inf_rows])        # same signed infinity
    B.csr5_free(h)


@pytest.mark.parametrize("kind", ["short_rows", "long_rows", "empty_rows", "no_nonzeros"])
def test_launch_set_before_and_after_status(kind):
    """Which kernels an SpMV launches depends on what the host knows about the
    matrix: everything until it has read the conversion's status word, only what
    the matrix needs afterwards (no second kernel when no tile starts more than 32
    entries into a row, no zero-filling workgroups without empty rows).  Both
    must give the oracle's y."""
    rng = np.random.default_rng(5)
    if kind == "short_rows":          # every row is completed by the tile it ends in
        a = wl.from_row_lengths(rng.integers(1, 33, size=6000), 5000, seed=1, name=kind)
    elif kind == "long_rows":         # rows longer than several tiles: carries
        lens = rng.integers(1, 30, size=3000)
        lens[[7, 1500, 2999]] = [5000, 1300, 2100]
        a = wl.from_row_lengths(lens, 9000, seed=2, name=kind)
    elif kind == "empty_rows":
        a = wl.from_row_lengths(rng.integers(0, 3, size=20000) * rng.integers(0, 30, size=20000), 7000, seed=3, name=kind)
    else:
        a = wl.from_row_lengths(np.zeros(1000, dtype=np.int64), 50, seed=4, name=kind)
    for sigma in (4, 16, 37):
        d = DeviceCsr(a)
        ws = torch.empty(B.csr5_workspace_bytes(a.m, a.nnz, sigma), dtype=torch.uint8, device="cuda:0")
        h = B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val, sigma=sigma, workspace=ws,
                              flags=B.CSR5_FLAG_NO_HOST_CHECK)
        say(kind, sigma, "nnz", a.nnz)
        check_spmv(d, h, (kind, sigma, "status unknown"))
        assert B.csr5_status(h) & 3 == 0
        check_spmv(d, h, (kind, sigma, "status known"))
        check_format(d, h, (kind, sigma))
        B.csr5_free(h)



def test_no_rows_and_no_columns():
    """m = 0 is a valid matrix (CSR5_OK, nothing to compute); so is a matrix
    without columns, which can hold no nonzero."""
    dev = torch.device("cuda:0")
    rp0 = torch.zeros(1, dtype=torch.int32, device=dev)
    dummy_c = torch.zeros(4, dtype=torch.int32, device=dev)
    dummy_v = torch.zeros(8, dtype=torch.float64, device=dev)
    y = torch.full((4,), 5.0, dtype=torch.float64, device=dev)
    for ws_on in (False, True):
        ws = None
        if ws_on:
            ws = torch.empty(B.csr5_workspace_bytes(0, 0, 0), dtype=torch.uint8, device=dev)
        h = B.csr5_convert_ex(0, 7, 0, rp0, dummy_c, dummy_v, workspace=ws)          # m = 0, n > 0
        info = B.csr5_get_info(h)
        assert info["p"] == 0 and info["p_complete"] == 0 and info["empty_offset_len"] == 0
        assert B.csr5_status(h) & 3 == 0
        assert B.csr5_spmv_ex(h, dummy_v, y) == B.CSR5_OK
        assert B.csr5_spmv_static(h, dummy_v, y) == B.CSR5_OK
        torch.cuda.synchronize()
        assert np.all(y.cpu().numpy() == 5.0)                 # no row: nothing written
        assert B.csr5_to_csr(h) == B.CSR5_OK
        B.csr5_free(h)
    h = B.csr5_convert(0, 0, 0, rp0, None, None)              # m = n = nnz = 0 through the plain entry point
    assert B.csr5_spmv(h, None, None) == B.CSR5_OK
    B.csr5_free(h)
    # n = 0 and nnz = 0 with rows: every row is empty, y = 0
    a = wl.from_row_lengths(np.zeros(777, dtype=np.int64), 0, seed=1, name="no_columns")
    assert a.n == 0 and a.nnz == 0
    d = DeviceCsr(a)
    for use_ws in (True, False):
        h = convert(d, use_workspace=use_ws)
        check_format(d, h, "no columns")
        check_spmv(d, h, "no columns")
        assert np.all(d.y.cpu().numpy()[:a.m] == 0.0)
        B.csr5_free(h)
    # nnz > 0 needs rows and columns
    rc, h = B.csr5_convert_ex(0, 5, 3, rp0, dummy_c, dummy_v, check=False)
    assert rc == B.CSR5_EINVAL and not h
    rp6 = torch.tensor([0, 1, 2, 3, 3, 3], dtype=torch.int32, device=dev)
    rc, h = B.csr5_convert_ex(5, 0, 3, rp6, dummy_c, dummy_v, check=False)
    assert rc == B.CSR5_EINVAL and not h


@pytest.mark.parametrize("cfg", [3, 4])
def test_plain_convert_on_full_size_irregular(cfg):
    """csr5_convert (blocking, hipMalloc inside, automatic sigma, default stream) on
    a full-size irregular configuration."""
    a = wl.config(cfg)
    d = DeviceCsr(a)
    h = B.csr5_convert(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val)
    say("config", cfg, B.csr5_get_info(h))
    check_format(d, h, f"plain convert config{cfg}")
    check_spmv(d, h, f"plain convert config{cfg}")
    B.csr5_free(h)


@pytest.mark.parametrize("offset", [1, 2, 3])
def test_col_idx_view_at_an_odd_offset(offset):
    """col_idx and val may be views into larger arrays: a col_idx base that is
    only 4-byte aligned is read entry by entry instead of sixteen bytes at a time."""
    for a, sigma in ((wl.config(4, scale=0.02), 16), (wl.tiny_uniform(m=900, n=700, seed=3), 5),
                     (wl.config(2, scale=0.01), 0)):
        d = DeviceCsr(a)
        big_c = torch.full((a.nnz + 8,), -7, dtype=torch.int32, device="cuda:0")
        big_v = torch.full((a.nnz + 8,), float("nan"), dtype=torch.float64, device="cuda:0")
        assert big_c.data_ptr() % 16 == 0
        big_c[offset:offset + a.nnz] = d.col_idx
        big_v[offset:offset + a.nnz] = d.val
        d.col_idx = big_c[offset:offset + a.nnz]
        d.val = big_v[offset:offset + a.nnz]
        assert d.col_idx.data_ptr() % 16 == 4 * offset
        h = convert(d, sigma=sigma)
        say("offset", offset, a.name, B.csr5_get_info(h)["sigma"])
        check_format(d, h, ("offset view", offset))
        check_spmv(d, h, ("offset view", offset))
        B.csr5_to_csr(h)
        torch.cuda.synchronize()
        assert np.array_equal(d.col_idx.cpu().numpy(), a.col_idx) and np.array_equal(d.val.cpu().numpy(), a.val)
        # nothing outside the view was touched
        assert int((big_c[:offset] != -7).sum()) == 0 and int((big_c[offset + a.nnz:] != -7).sum()) == 0
        assert bool(torch.isnan(big_v[:offset]).all()) and bool(torch.isnan(big_v[offset + a.nnz:]).all())
        B.csr5_free(h)


def test_two_handles_on_two_streams():
    """Two matrices, two handles, SpMVs of both in flight at the same time on two
    streams (every handle has its own auxiliary array): both results are the
    oracle's, whatever the interleaving."""
    a1, a2 = wl.config(3, scale=0.05), wl.config(4, scale=0.05)
    d1, d2 = DeviceCsr(a1), DeviceCsr(a2)
    h1, h2 = convert(d1, sigma=0), convert(d2, sigma=8)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    ys1 = [torch.full_like(d1.y, float("nan")) for _ in range(6)]
    ys2 = [torch.full_like(d2.y, float("nan")) for _ in range(6)]
    for k in range(6):                       # enqueue alternately, no waiting in between
        B.csr5_spmv_ex(h1, d1.x, ys1[k], stream=s1)
        B.csr5_spmv_ex(h2, d2.x, ys2[k], stream=s2)
    s1.synchronize()
    s2.synchronize()
    for k in range(6):
        _check_y(ys1[k].cpu().numpy()[:a1.m], a1, ("stream 1", k))
        _check_y(ys2[k].cpu().numpy()[:a2.m], a2, ("stream 2", k))
    B.csr5_free(h1)
    B.csr5_free(h2)



def test_binding_refuses_wrong_types_and_short_arrays():
    """A tensor of the wrong element type or length would make a kernel leave its
    array; the binding refuses it on the host before anything is launched."""
    a = wl.tiny_uniform(m=300, n=200, seed=2)
    d = DeviceCsr(a)
    with pytest.raises(ValueError):
        B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr.long(), d.col_idx, d.val)          # int64 row_ptr
    with pytest.raises(ValueError):
        B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val.float())         # float32 val
    with pytest.raises(ValueError):
        B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr[:-1], d.col_idx, d.val)            # short row_ptr
    with pytest.raises(ValueError):
        B.csr5_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx[:-1], d.val)            # short col_idx
    with pytest.raises(ValueError):
        B.csr5l_convert_ex(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val)                # int32 row_ptr, wide entry point
    h = convert(d, sigma=4)
    assert B.csr5_get_shape(h) == (a.m, a.n)
    with pytest.raises(ValueError):
        B.csr5_spmv_ex(h, d.x[:-1], d.y)                                                # short x
    with pytest.raises(ValueError):
        B.csr5_spmv_ex(h, d.x, d.y[:a.m - 1])                                           # short y
    with pytest.raises(ValueError):
        B.csr5_spmv_ex(h, d.x.float(), d.y)
    check_spmv(d, h, "after refusals")
    B.csr5_free(h)


def test_one_handle_on_two_streams():
    """Up to four SpMVs of ONE handle may be in flight at once (the handle takes its
    four auxiliary arrays in turn): two streams, two calls each, different x, then
    a synchronisation, several rounds.  A matrix with long rows, so that every call
    really uses its auxiliary array."""
    a = wl.config(4, scale=0.05)
    d = DeviceCsr(a)
    h = convert(d, sigma=8)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    rng = np.random.default_rng(3)
    xs = [rng.standard_normal(a.n) for _ in range(4)]
    xd = [torch.from_numpy(x).to("cuda:0") for x in xs]
    refs = [oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, x) for x in xs]
    torch.cuda.synchronize()
    for rnd in range(5):
        ys = [torch.full_like(d.y, float("nan")) for _ in range(4)]
        B.csr5_spmv_ex(h, xd[0], ys[0], stream=s1)
        B.csr5_spmv_ex(h, xd[1], ys[1], stream=s2)
        B.csr5_spmv_ex(h, xd[2], ys[2], stream=s1)
        B.csr5_spmv_ex(h, xd[3], ys[3], stream=s2)
        s1.synchronize()
        s2.synchronize()
        for k in range(4):
            y_ref, s = refs[k]
            got = ys[k].cpu().numpy()[:a.m]
            bad = np.nonzero(~(np.abs(got - y_ref) <= 1e-12 * s + 1e-300))[0]
            assert bad.size == 0, (rnd, k, int(bad.size), int(bad[0]))
    B.csr5_free(h)


@pytest.mark.parametrize("wide,seed,longest", [(False, 31, 33), (True, 32, 33), (False, 33, 161), (True, 34, 161)])
def test_random_short_row_matrices_take_one_kernel(wide, seed, longest):
    """Matrices whose rows have at most 161 entries, so that no tile can start more
    than 160 entries into a row (33 and 32: the part of the previous tile's record
    that a workgroup's first tile always reads): for 8 <= sigma <= 32 their SpMV is
    the tile kernel alone (the profile helper reports no second kernel), whatever
    the mix of empty rows, and its result is the oracle's."""
    rng = np.random.default_rng(seed)
    for case in range(24):
        sigma = int(rng.integers(8, 33))
        m = int(rng.integers(200, 6000))
        n = int(rng.integers(40 if longest < 40 else 200, 8000))
        top = int(rng.integers(1, longest + 1))
        lens = rng.integers(0, top + 1, size=m)
        if case % 3 == 0:
            lens *= rng.random(m) < 0.5                      # many empty rows
        if case % 3 == 1:
            lens = np.maximum(lens, 1)                       # none
        a = wl.from_row_lengths(lens, n, seed=seed * 100 + case, name=f"short{case}")
        say("short rows", case, "sigma", sigma, a.m, a.n, a.nnz, "max len", int(np.diff(a.row_ptr).max()) if a.m else 0)
        d = DeviceCsr(a, wide=wide)
        h = convert(d, sigma=sigma)                          # blocking: the handle knows the matrix
        check_format(d, h, (a.name, sigma))
        check_spmv(d, h, (a.name, sigma))
        if not wide and a.m:
            ms_second = second_kernel_ms(h, d.x, d.y)
            assert ms_second < 1e-3, ("a second kernel was launched", ms_second)   # 50 launches of it would take 2 us each
            _check_y(d.y.cpu().numpy()[:a.m], a, ("after profile", case))
        B.csr5_free(h)


def _group_cases(sigma):
    """Row-length lists that put rows in every position relative to the groups of
    tiles (workgroups of the tile kernel: 4 tiles up to sigma 16, 2 up to 32)."""
    T = 64 * sigma
    G = T * (4 if sigma <= 16 else 2)
    rng = np.random.default_rng(sigma)
    mix = rng.choice([0, 0, 1, 2, 5, 30, 200, T - 1, T, T + 1, G - 1, G, G + 1, 2 * G + 17, 3 * G], size=60)
    return {
        "ends_on_a_group_boundary": [G // 2, G // 2 + G, 7, 3],
        "starts_with_a_group": [G, 2 * G, 5, G - 5, G + 9],
        "four_groups": [10, 3 * G, 10, 1],
        "one_row_and_a_tail": [5 * G + 77],
        "into_the_tail_from_a_partial_group": [G + T - 9, 40],
        "into_the_tail_across_groups": [11, 2 * G + T + 5],
        "last_entry_of_a_group": [G - 1, 2, G + 1, 2 * G - 2, 1, 1],
        "neighbours": [G - 3, 6, G - 3, G + 6, 3 * G - 6, 2, 2 * G],
        "empty_rows_between": [0, G + 5, 0, 0, 3, 0, 2 * G, 0, T + 1, 0],
        "mixed": list(mix),
    }


@pytest.mark.parametrize("sigma", [8, 16, 24, 32])
def test_rows_across_groups_of_tiles_in_one_kernel(sigma):
    """Matrices of this size that need the auxiliary array get their cross-tile sums
    inside the tile kernel: rows that end on, start with, or run across the
    boundaries of the tile groups, rows that reach the incomplete tile, rows of
    two groups (one exchange) and of more (counted).  y is the oracle's on every
    one of several calls in a row (the meeting words and counters must come back
    to rest), in double and in single precision, and no second kernel runs."""
    for k, (name, lens) in enumerate(_group_cases(sigma).items()):
        lens = np.asarray(lens, dtype=np.int64)
        a = wl.from_row_lengths(lens, int(lens.max()) + 100, seed=sigma, name=name)
        d = DeviceCsr(a, wide=(k % 2 == 1))      # every other case through the 64-bit index variant
        h = convert(d, sigma=sigma)
        say("groups", sigma, name, a.m, a.nnz, "wide" if d.wide else "")
        check_format(d, h, (name, sigma))
        rng = np.random.default_rng(1)
        for call in range(3):
            check_spmv(d, h, (name, sigma, call), x=rng.standard_normal(a.n))
        ms_second = second_kernel_ms(h, d.x, d.y)
        assert ms_second < 1e-3, (name, sigma, ms_second)
        check_spmv(d, h, (name, sigma, "after profile"))
        B.csr5_free(h)
        if not d.wide:
            _run32(a, sigma)


def test_the_empty_pattern_of_the_meeting_words_as_a_value():
    """The one-launch path marks a free meeting word with a particular NaN.  A part
    that is that very NaN (x holds it, and a NaN operand's payload survives
    multiplication and addition) must not be mistaken for it: the rows that use it
    are NaN, the others are the oracle's, and so is everything on the next call."""
    sigma = 16
    G = 64 * sigma * 4
    lens = np.array([G - 5, 700, G + 40, 3 * G, 9, 2 * G, 12], dtype=np.int64)
    a = wl.from_row_lengths(lens, 4 * G, seed=3, name="payload")
    d = DeviceCsr(a)
    h = convert(d, sigma=sigma)
    x = a.x.copy()
    poison = np.array([0xfff8c5125eaf0001], dtype=np.uint64).view(np.float64)[0]
    hit = a.col_idx[a.row_ptr[1] + 3], a.col_idx[a.row_ptr[3] + 5 * G // 2]
    x[list(hit)] = poison
    d.x = torch.from_numpy(x).to("cuda:0")
    d.y.fill_(0.0)
    B.csr5_spmv_ex(h, d.x, d.y)
    torch.cuda.synchronize()
    y = d.y.cpu().numpy()[:a.m]
    with np.errstate(invalid="ignore"):
        y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, x)
    nan_rows = np.isnan(y_ref)
    assert nan_rows[1] and nan_rows[3] and 2 <= nan_rows.sum() < a.m
    assert np.array_equal(np.isnan(y), nan_rows)
    assert np.all(np.abs(y[~nan_rows] - y_ref[~nan_rows]) <= 1e-12 * s[~nan_rows] + 1e-300)
    for call in range(2):
        check_spmv(d, h, ("payload", "clean call", call), x=a.x)
    B.csr5_free(h)


def test_beyond_the_one_kernel_sizes_the_second_kernel_runs():
    """Rows of 701 entries: up to 6144 tiles the sums cross inside the tile kernel,
    beyond that (long rows on average) the second kernel adds them.  Same y."""
    for rows, second in ((6000, False), (12000, True)):
        a = wl.from_row_lengths(np.full(rows, 701), 60000, seed=rows, name=f"r701x{rows}")
        d = DeviceCsr(a)
        h = convert(d, sigma=16)
        assert (B.csr5_get_info(h)["p"] > 6144) == second
        check_spmv(d, h, (a.name,))
        ms_second = second_kernel_ms(h, d.x, d.y)
        assert (ms_second > 1e-3) == second, (rows, ms_second)
        _check_y(d.y.cpu().numpy()[:a.m], a, ("after profile", rows))
        B.csr5_free(h)


def test_flags_that_fix_the_form_of_the_auxiliary_array_path():
    """CSR5_FLAG_AUX_TWO_KERNELS and CSR5_FLAG_AUX_ONE_KERNEL (measurement aids)
    override the size rule, in both directions; y is the oracle's either way, and
    a matrix that does not use the auxiliary array is not affected."""
    small = wl.from_row_lengths(np.full(3000, 701), 60000, seed=2, name="small")       # rule: one kernel
    large = wl.from_row_lengths(np.full(12000, 701), 60000, seed=3, name="large")      # rule: two
    short = wl.from_row_lengths(np.full(20000, 20), 5000, seed=4, name="short")        # look-behind
    for a, by_rule in ((small, False), (large, True), (short, False)):
        for flags, second in ((B.CSR5_FLAG_NONE, by_rule), (B.CSR5_FLAG_AUX_TWO_KERNELS, a is not short),
                              (B.CSR5_FLAG_AUX_ONE_KERNEL, False)):
            d = DeviceCsr(a)
            h = convert(d, sigma=16, flags=flags)
            say("aux form", a.name, flags)
            check_spmv(d, h, (a.name, flags))
            ms_second = second_kernel_ms(h, d.x, d.y)
            assert (ms_second > 1e-3) == second, (a.name, flags, ms_second)
            check_spmv(d, h, (a.name, flags, "again"))
            B.csr5_free(h)


@pytest.mark.parametrize("kind", ["look_behind", "auxiliary_array_one_kernel"])
def test_one_kernel_forms_add_in_a_fixed_order(kind):
    """Both one-kernel forms add the parts of a row in an order that does not depend
    on which wavefront finishes first: repeated calls give the same bits.  (No
    incomplete tile here: rows cut by the 64-entry chunks inside it are added with
    LDS atomics, and so are rows the second kernel sums with several wavefronts.)"""
    rng = np.random.default_rng(11)
    T = 64 * 16
    if kind == "look_behind":
        lens = rng.integers(1, 34, size=120_000)
    else:
        lens = np.where(rng.random(20_000) < 0.01, rng.integers(200, 30_000, size=20_000), rng.integers(0, 30, size=20_000))
    lens[-1] += (-int(lens.sum())) % T
    a = wl.from_row_lengths(lens, 40_000, seed=12, name=kind)
    assert a.nnz % T == 0
    d = DeviceCsr(a)
    h = convert(d, sigma=16)
    check_spmv(d, h, (kind,))
    ms_second = second_kernel_ms(h, d.x, d.y)
    assert ms_second < 1e-3
    first = None
    for call in range(8):
        d.y.fill_(float("nan"))
        B.csr5_spmv_ex(h, d.x, d.y)
        torch.cuda.synchronize()
        if first is None:
            first = d.y.clone()
        assert torch.equal(first.view(torch.int64), d.y.view(torch.int64)), (kind, call)
    _check_y(first.cpu().numpy()[:a.m], a, (kind, "bits"))
    B.csr5_free(h)


@pytest.mark.parametrize("seed,cases", [(5000, 150), (77000, 150)])
def test_random_matrices_with_rows_across_tile_groups(seed, cases):
    """Random small matrices in which rows of every length up to several groups of
    tiles are mixed with short and empty ones, at random tile heights 8..32, in
    both index widths: the auxiliary-array path inside the tile kernel.  Two calls
    with different x on every handle."""
    for case in range(cases):
        rng = np.random.default_rng(seed + case)
        sigma = int(rng.integers(8, 33))
        T = 64 * sigma
        G = T * (4 if sigma <= 16 else 2)
        m = int(rng.integers(1, 400))
        kind = case % 5
        base = rng.integers(0, 40, size=m)
        if kind == 0:
            lens = np.where(rng.random(m) < 0.1, rng.integers(150, 4 * G, size=m), base)
        elif kind == 1:
            lens = np.where(rng.random(m) < 0.3, rng.integers(G - 3, G + 4, size=m), base)
        elif kind == 2:
            lens = np.where(rng.random(m) < 0.2, rng.integers(1, 6, size=m) * G + rng.integers(-2, 3, size=m), base)
        elif kind == 3:
            lens = np.where(rng.random(m) < 0.3, rng.integers(T - 2, 3 * T, size=m), np.where(rng.random(m) < 0.5, 0, base))
        else:
            lens = rng.integers(100, 6 * T, size=m)
        lens = np.maximum(lens, 0)
        n = int(max(lens.max(), 200)) + int(rng.integers(0, 500))
        a = wl.from_row_lengths(lens, n, seed=seed + case, name=f"groups{case}")
        d = DeviceCsr(a, wide=bool(case % 2))
        say("case", case, "kind", kind, "sigma", sigma, "m", a.m, "nnz", a.nnz, "wide", d.wide)
        h = convert(d, sigma=sigma)
        for call in range(2):
            check_spmv(d, h, (a.name, sigma, call), x=rng.standard_normal(a.n))
        B.csr5_free(h)
