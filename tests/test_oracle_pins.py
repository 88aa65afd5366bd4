"""Pins for the CPU oracle: each part is checked against something other than
itself -- brute force on small inputs, closed forms, invariants, and the facts
the paper's text states about its 8x8 example (tests/golden/fig4_like.txt).
No GPU needed."""
import math
import os

import numpy as np
import pytest

import oracle
from paper_1503_05032_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SHAPES = [(4, 4), (8, 5), (32, 16), (64, 4), (64, 16), (64, 20), (64, 48)]


def coo_rows(a):
    return np.repeat(np.arange(a.m, dtype=np.int64), np.diff(a.row_ptr.astype(np.int64)))


def small_cases(T):
    return wl.edge_cases(T) + wl.structured_cases(T) + [wl.tiny_uniform(m=300, n=200, max_len=12, seed=5)]


# ----------------------------------------------------------------- Algorithm 1
def test_spmv_dense_bruteforce():
    rng = np.random.default_rng(0)
    for m, n in [(1, 1), (7, 5), (33, 64), (64, 64)]:
        dense = rng.uniform(-1, 1, size=(m, n)) * (rng.random((m, n)) < 0.3)
        lens = (dense != 0).sum(1)
        rp = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        r, c = np.nonzero(dense)
        x = rng.uniform(-1, 1, size=n)
        y, s = oracle.csr_spmv(m, rp, c.astype(np.int32), dense[r, c], x)
        # dense brute force, plain Python accumulation over ALL columns
        for i in range(m):
            acc = math.fsum(dense[i, j] * x[j] for j in range(n))
            mag = math.fsum(abs(dense[i, j] * x[j]) for j in range(n))
            assert abs(y[i] - acc) <= 4e-16 * mag + 1e-300
            assert abs(s[i] - mag) <= 4e-16 * mag * n + 1e-300


def test_spmv_identity_and_permutation_exact():
    a = wl.identity(257)
    y, _ = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    assert np.array_equal(y, a.x)
    a = wl.permutation(300, seed=3)
    y, _ = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    assert np.array_equal(y, a.x[a.col_idx])      # one entry per row: y[i] = x[perm[i]]


def test_spmv_ones_gives_row_sums_and_empty_rows_zero():
    a = wl.tiny_uniform(m=500, n=300, seed=11)
    y, _ = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, np.ones(a.n))
    for i in range(a.m):
        seg = a.val[a.row_ptr[i]:a.row_ptr[i + 1]]
        assert abs(y[i] - math.fsum(seg)) <= 1e-15 * np.abs(seg).sum()
        if seg.size == 0:
            assert y[i] == 0.0
    e = wl.from_row_lengths([0] * 20, 9)
    y, s = oracle.csr_spmv(e.m, e.row_ptr, e.col_idx, e.val, e.x)
    assert np.all(y == 0) and np.all(s == 0)


def test_spmv_single_long_row_is_dot():
    a = wl.from_row_lengths([5000], 8000, seed=2)
    y, s = oracle.csr_spmv(1, a.row_ptr, a.col_idx, a.val, a.x)
    exact = math.fsum(float(v) * float(a.x[c]) for v, c in zip(a.val, a.col_idx))
    assert abs(y[0] - exact) <= 1e-13 * s[0]


def test_spmv_uses_column_indices_not_positions():
    # transposed-operand mistake would survive symmetric tests; this one is asymmetric
    rp = np.array([0, 1, 2], dtype=np.int32)
    y, _ = oracle.csr_spmv(2, rp, np.array([2, 0], dtype=np.int32), np.array([2.0, 3.0]),
                           np.array([10.0, 100.0, 1000.0]))
    assert y.tolist() == [2000.0, 30.0]


# ----------------------------------------------------------------- Algorithm 4
@pytest.mark.parametrize("omega,sigma", SHAPES)
def test_tile_ptr_bruteforce(omega, sigma):
    T = omega * sigma
    for a in small_cases(T):
        tp = oracle.tile_ptr(a.m, a.nnz, a.row_ptr, omega, sigma)
        p = -(-a.nnz // T)
        assert tp.shape[0] == p + 1
        rows = coo_rows(a)
        raw = tp & 0x7FFFFFFF
        for t in range(p + 1):
            exp = rows[t * T] if t * T < a.nnz else a.m       # row that owns nonzero t*T
            assert raw[t] == exp, (a.name, t)
        assert np.all(np.diff(raw.astype(np.int64)) >= 0)
        assert raw[p] == a.m and not (tp[p] & 0x80000000)
        # dirty flag: literal definition, inclusive row range, clamped at m-1
        lens = np.diff(a.row_ptr)
        for t in range(p):
            lo, hi = int(raw[t]), min(int(raw[t + 1]), a.m - 1)
            exp_dirty = bool((lens[lo:hi + 1] == 0).any())
            assert bool(tp[t] & 0x80000000) == exp_dirty, (a.name, t)


def test_tile_ptr_no_empty_rows_means_no_flag():
    a = wl.from_row_lengths(np.random.default_rng(1).integers(1, 30, size=500), 1000)
    tp = oracle.tile_ptr(a.m, a.nnz, a.row_ptr, 64, 4)
    assert not (tp & 0x80000000).any()


def test_negative_zero_tile_ptr():
    # Section 3.3: first tile starts in row 0 and holds an empty row -> 1000...0
    a = [c for c in wl.edge_cases(64 * 4) if c.name == "negative_zero_tile_ptr"][0]
    tp = oracle.tile_ptr(a.m, a.nnz, a.row_ptr, 64, 4)
    assert tp[0] == 0x80000000


# ---------------------------------------------------- golden: Figure-4-like case
def _gold():
    paper, derived, lens = {}, {}, None
    for line in open(os.path.join(GOLD, "fig4_like.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "row_lengths":
            lens = [int(v) for v in f[1:]]
        elif f[0] == "paper":
            paper[f[1]] = [int(v) for v in f[2:]]
        elif f[0] == "derived":
            derived[f[1]] = [int(v) for v in f[2:]]
    return lens, paper, derived


def test_paper_example_facts():
    lens, paper, derived = _gold()
    assert len(lens) == 8 and sum(lens) == 34
    a = wl.from_row_lengths(lens, 8, seed=0)
    c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, 4, 4)
    assert [c5.p] == paper["num_tiles"]
    assert [c5.pc] == paper["num_complete_tiles"]
    assert [a.nnz - c5.pc * 16] == paper["incomplete_tile_size"]
    assert [int(c5.tile_ptr[1] & 0x7FFFFFFF)] == paper["tile_ptr_1"]
    assert [int(c5.bit_flag[0].sum())] == paper["tile0_num_true"]
    assert [int(c5.tile_ptr[0] >> 31)] == paper["tile0_dirty"]
    assert [int(c5.empty_offset_ptr[1] - c5.empty_offset_ptr[0])] == paper["tile0_empty_offset_len"]
    assert c5.seg_offset[0].tolist() == paper["tile0_seg_offset"]
    assert c5.bit_flag[0, 2].sum() == 0                      # "the 3rd column" has no TRUE
    assert [int(c5.bit_flag[1, 0].sum())] == paper["tile1_col0_num_true"]
    assert [int(c5.y_offset[1, 1])] == paper["tile1_y_offset_1"]
    assert [int(c5.y_offset[1, 3])] == paper["tile1_y_offset_3"]
    # hand-derived values for this matrix
    assert c5.tile_ptr.tolist() == derived["tile_ptr"]
    assert c5.y_offset[0].tolist() == derived["tile0_y_offset"]
    assert c5.empty_offset[:4].tolist() == derived["tile0_empty_offset"]
    assert c5.y_offset[1].tolist() == derived["tile1_y_offset"]
    assert c5.seg_offset[1].tolist() == derived["tile1_seg_offset"]
    assert c5.empty_offset.shape[0] == 4                     # tile 1 is not dirty


# ------------------------------------------- bit_flag / y_offset / seg_offset
@pytest.mark.parametrize("omega,sigma", SHAPES)
def test_descriptor_bruteforce_and_row_reconstruction(omega, sigma):
    T = omega * sigma
    for a in small_cases(T):
        c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, omega, sigma)
        rows = coo_rows(a)
        lens = np.diff(a.row_ptr)
        starts = set(int(v) for v in a.row_ptr[:-1][lens > 0])
        for t in range(c5.pc):
            row0 = int(c5.tile_ptr[t] & 0x7FFFFFFF)
            dirty = bool(c5.tile_ptr[t] >> 31)
            eo = c5.empty_offset[c5.empty_offset_ptr[t]:c5.empty_offset_ptr[t + 1]]
            nflag = 0
            ntrue_prev_cols = 0
            for i in range(omega):
                assert c5.y_offset[t, i] == ntrue_prev_cols, (a.name, t, i)
                col_true = 0
                for j in range(sigma):
                    k = t * T + i * sigma + j                # CSR position of entry (i, j)
                    exp = 1 if (k in starts or (i == 0 and j == 0)) else 0
                    assert c5.bit_flag[t, i, j] == exp, (a.name, t, i, j)
                    nflag += exp
                    col_true += exp
                    seg = nflag - 1
                    # row-reconstruction invariant
                    got = row0 + (int(eo[seg]) if dirty else seg)
                    assert got == rows[k], (a.name, t, i, j)
                ntrue_prev_cols += col_true
            # seg_offset from its verbal definition (Section 3.4)
            has = c5.bit_flag[t].any(axis=1)
            for i in range(omega):
                if has[i]:
                    k = i + 1
                    while k < omega and not has[k]:
                        k += 1
                    assert c5.seg_offset[t, i] == k - i - 1
                else:
                    assert c5.seg_offset[t, i] == 0
            if dirty:
                assert eo.shape[0] == nflag and eo[0] == 0
                assert np.all(np.diff(eo) > 0)
            else:
                assert eo.shape[0] == 0
        assert c5.empty_offset_ptr[0] == 0
        assert c5.empty_offset_ptr[c5.pc] == c5.empty_offset.shape[0]


def test_closed_forms():
    omega, sigma = 64, 16
    T = omega * sigma
    # one long row: only the forced flag; column 0 absorbs all 63 others
    a = wl.from_row_lengths([2 * T + 5], 3 * T)
    c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, omega, sigma)
    for t in range(2):
        assert c5.bit_flag[t].sum() == 1 and c5.bit_flag[t, 0, 0] == 1
        assert np.all(c5.y_offset[t] == [0] + [1] * (omega - 1))
        assert c5.seg_offset[t].tolist() == [omega - 1] + [0] * (omega - 1)
    # all rows of length sigma: one flag per column, in row 0
    a = wl.from_row_lengths([sigma] * (2 * omega), 500)
    c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, omega, sigma)
    for t in range(2):
        assert np.all(c5.bit_flag[t, :, 0] == 1) and c5.bit_flag[t].sum() == omega
        assert c5.y_offset[t].tolist() == list(range(omega))
        assert np.all(c5.seg_offset[t] == 0)
        assert c5.tile_ptr[t] == t * omega
    # all rows of length 1: every flag set
    a = wl.from_row_lengths([1] * (2 * T), 500)
    c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, omega, sigma)
    assert c5.bit_flag.all()
    assert c5.y_offset[1].tolist() == [i * sigma for i in range(omega)]
    assert c5.tile_ptr.tolist() == [0, T, 2 * T]


# ----------------------------------------------------------------- Section 3.5
def test_packing_size_closed_form():
    assert oracle.desc_bits(32, 16) == 30                  # 9 + 5 + 16, as printed
    assert oracle.desc_words(32, 16) == 1
    extra = 32 * 4 / (32 * 16 * 12)                        # omega words vs 12-byte entries
    assert abs(extra - 0.0208) < 1e-3                      # "around 2%"
    assert oracle.desc_bits(64, 16) == 32 and oracle.desc_words(64, 16) == 1
    assert oracle.desc_words(64, 17) == 2 and oracle.desc_words(64, 46) == 2
    assert oracle.desc_words(64, 47) == 3


@pytest.mark.parametrize("omega,sigma", SHAPES)
def test_pack_unpack_roundtrip(omega, sigma):
    a = wl.tiny_uniform(m=400, n=300, max_len=9, seed=3)
    c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, omega, sigma)
    W = c5.W
    sbits = (omega - 1).bit_length()
    ybits = (omega * sigma - 1).bit_length()
    assert W == -(-(sigma + sbits + ybits) // 32)
    td = c5.tile_desc.reshape(c5.pc, W, omega)
    for t in range(c5.pc):
        for i in range(omega):
            word = 0
            for k in range(W):
                word |= int(td[t, k, i]) << (32 * k)
            flags = [(word >> j) & 1 for j in range(sigma)]
            assert flags == c5.bit_flag[t, i].tolist()
            assert (word >> sigma) & ((1 << sbits) - 1) == c5.seg_offset[t, i]
            assert (word >> (sigma + sbits)) & ((1 << ybits) - 1) == c5.y_offset[t, i]
            assert word >> (sigma + sbits + ybits) == 0


# ----------------------------------------------------------------- Section 3.1
@pytest.mark.parametrize("omega,sigma", SHAPES)
def test_transpose(omega, sigma):
    T = omega * sigma
    a = wl.from_row_lengths([7] * ((2 * T + 31) // 7 + 1), 1000, seed=1)
    ct, vt = oracle.transpose(a.nnz, omega, sigma, a.col_idx, a.val)
    pc = a.nnz // T
    assert pc >= 2
    for t in range(pc):
        blk_c = a.col_idx[t * T:(t + 1) * T].reshape(omega, sigma)     # [i][j] row-major
        blk_v = a.val[t * T:(t + 1) * T].reshape(omega, sigma)
        assert np.array_equal(ct[t * T:(t + 1) * T].reshape(sigma, omega), blk_c.T)
        assert np.array_equal(vt[t * T:(t + 1) * T].reshape(sigma, omega), blk_v.T)
    assert np.array_equal(ct[pc * T:], a.col_idx[pc * T:])
    assert np.array_equal(vt[pc * T:], a.val[pc * T:])
    # pairs stay together
    pairs_in = sorted(zip(a.col_idx.tolist(), a.val.tolist()))
    assert pairs_in == sorted(zip(ct.tolist(), vt.tolist()))


# ----------------------------------------------------------------- Section 3.2
def test_sigma_rule_paper_constants():
    r, s, t, u = 4, 32, 256, 4            # the constants printed for one of the GPUs
    m = 1000
    assert oracle.sigma_rule(3 * m, m, r, s, t, u) == 4
    assert oracle.sigma_rule(4 * m, m, r, s, t, u) == 4
    assert oracle.sigma_rule(10 * m, m, r, s, t, u) == 10
    assert oracle.sigma_rule(32 * m, m, r, s, t, u) == 32
    assert oracle.sigma_rule(100 * m, m, r, s, t, u) == 32
    assert oracle.sigma_rule(256 * m, m, r, s, t, u) == 32
    assert oracle.sigma_rule(257 * m, m, r, s, t, u) == 4
    assert oracle.sigma_rule(0, 0, r, s, t, u) == 4
    assert oracle.sigma_rule(6 * m, m, 4, 7, 256, 4) == 6   # the other printed set
    assert oracle.sigma_rule(9 * m, m, 4, 7, 256, 4) == 7


# ------------------------------------------------- Algorithm 8 over the format
@pytest.mark.parametrize("omega,sigma", SHAPES)
def test_csr5_spmv_equals_algorithm1(omega, sigma):
    T = omega * sigma
    for a in small_cases(T):
        c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, omega, sigma)
        y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
        y5 = oracle.csr5_spmv(c5, a.x)
        # Algorithm 6 subtracts prefix sums taken over the whole tile, so its
        # error scales with the tile's magnitude, not the row's
        scale = s.max() if s.size else 0.0
        assert np.all(np.abs(y5 - y_ref) <= 1e-12 * scale + 1e-300), a.name
        if a.name != "wide_values":
            assert np.all(np.abs(y5 - y_ref) <= 1e-12 * s + 1e-300 + 1e-13 * scale), a.name


def test_csr5_spmv_mid_size():
    a = wl.config(3, scale=0.01)
    for sigma in (4, 16, 32):
        c5 = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, 64, sigma)
        y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
        y5 = oracle.csr5_spmv(c5, a.x)
        assert np.all(np.abs(y5 - y_ref) <= 1e-12 * s + 1e-300)


def test_all_cores_variant_is_bit_identical():
    """The OpenMP loop of the benchmark's all-cores figure sums every row exactly as Algorithm 1 does."""
    a = wl.config(3, scale=0.01)
    y1, s1 = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    y2, s2, threads = oracle.csr_spmv_all_cores(a.m, a.row_ptr, a.col_idx, a.val, a.x)
    assert threads >= 1
    assert np.array_equal(y1.view(np.uint64), y2.view(np.uint64))
    assert np.array_equal(s1.view(np.uint64), s2.view(np.uint64))
