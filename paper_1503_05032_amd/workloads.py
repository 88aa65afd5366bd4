"""Seeded synthetic sparse matrices (CSR, int32 indices, fp64 values) and dense x.

This module only *draws inputs*: row lengths, column indices, values and the
vector x.  It holds none of the CSR5 method's arithmetic (no tile, descriptor or
SpMV code) so that both the CPU oracle's tests and the HIP path's tests can use
the same inputs without sharing any implementation.

The paper evaluates on matrices of the University of Florida collection
(Section 5.2, Table 2); those are not available offline, so the five workloads
here reproduce the *shape statistics* of its regular group (tightly clustered
row lengths) and irregular group (power-law / a few huge rows / empty rows).

Every generator returns a `Csr` whose columns are sorted and distinct inside a
row.  All randomness comes from `numpy.random.default_rng(seed)` (PCG64).
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np


@dataclass
class Csr:
    """CSR matrix (Section 2.1): row_ptr int32[m+1], col_idx int32[nnz], val fp64[nnz]."""

    m: int
    n: int
    row_ptr: np.ndarray
    col_idx: np.ndarray
    val: np.ndarray
    x: np.ndarray
    name: str = ""

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])

    def stats(self) -> dict:
        ln = np.diff(self.row_ptr.astype(np.int64))
        return {
            "name": self.name, "m": self.m, "n": self.n, "nnz": self.nnz,
            "row_len_min": int(ln.min()) if self.m else 0,
            "row_len_avg": float(ln.mean()) if self.m else 0.0,
            "row_len_max": int(ln.max()) if self.m else 0,
            "empty_rows": int((ln == 0).sum()),
        }


def _finish(m, n, lens, cols, val, x, name) -> Csr:
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    assert row_ptr[-1] == cols.shape[0] == val.shape[0]
    assert row_ptr[-1] < 2 ** 31
    return Csr(m, n, row_ptr.astype(np.int32), np.ascontiguousarray(cols, dtype=np.int32),
               np.ascontiguousarray(val, dtype=np.float64),
               np.ascontiguousarray(x, dtype=np.float64), name)


def _dedupe_sorted(rows: np.ndarray, cols: np.ndarray, m: int, n: int):
    """Sort (row, col) pairs, drop duplicates; returns (lens[m], cols sorted by row then col).

    `rows` must already be non-decreasing (pairs are generated row by row).
    """
    key = rows.astype(np.int64) * np.int64(n) + cols.astype(np.int64)
    key.sort()
    if key.size:
        keep = np.empty(key.size, dtype=bool)
        keep[0] = True
        np.not_equal(key[1:], key[:-1], out=keep[1:])
        key = key[keep]
    r = key // np.int64(n)
    c = key - r * np.int64(n)
    lens = np.bincount(r, minlength=m).astype(np.int64)
    return lens, c.astype(np.int32)


# --------------------------------------------------------------------------
# config 1: tiny uniform
# --------------------------------------------------------------------------
def tiny_uniform(m=2000, n=2000, max_len=20, seed=0) -> Csr:
    """Row lengths uniform in {0..max_len} (about 1/(max_len+1) rows empty), columns
    drawn without replacement, values and x uniform in [-1, 1]."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, max_len + 1, size=m).astype(np.int64)
    lens = np.minimum(lens, n)
    cols = np.empty(int(lens.sum()), dtype=np.int32)
    o = 0
    for i in range(m):
        k = int(lens[i])
        if k:
            cols[o:o + k] = np.sort(rng.choice(n, size=k, replace=False))
            o += k
    val = rng.uniform(-1.0, 1.0, size=o)
    x = rng.uniform(-1.0, 1.0, size=n)
    return _finish(m, n, lens, cols, val, x, f"tiny_uniform_{m}x{n}")


# --------------------------------------------------------------------------
# config 2: 27-point stencil on a g^3 grid
# --------------------------------------------------------------------------
def stencil27(g=100, seed=1) -> Csr:
    """3-D 27-point stencil, grid points numbered x-fastest; boundary rows are
    truncated (8..27 entries).  Centre 26.0, neighbours -1.0 + U[-0.01, 0.01];
    x ~ U[0, 1].  nnz = (3g-2)^3."""
    rng = np.random.default_rng(seed)
    m = g * g * g
    idx = np.arange(m, dtype=np.int64)
    ix, iy, iz = idx % g, (idx // g) % g, idx // (g * g)
    # Offsets in increasing column order: dz slowest, dx fastest.
    valid = []
    offs = []
    for dz in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                ok = ((ix + dx >= 0) & (ix + dx < g) & (iy + dy >= 0) & (iy + dy < g)
                      & (iz + dz >= 0) & (iz + dz < g))
                valid.append(ok)
                offs.append(dx + dy * g + dz * g * g)
    valid = np.stack(valid, axis=1)            # [m, 27]
    offs = np.asarray(offs, dtype=np.int64)
    lens = valid.sum(axis=1).astype(np.int64)
    colmat = idx[:, None] + offs[None, :]
    cols = colmat[valid]                        # row-major flatten keeps column order
    centre = np.broadcast_to(offs[None, :] == 0, valid.shape)[valid]
    nnz = cols.shape[0]
    assert nnz == (3 * g - 2) ** 3
    val = -1.0 + rng.uniform(-0.01, 0.01, size=nnz)
    val[centre] = 26.0
    x = rng.uniform(0.0, 1.0, size=m)
    return _finish(m, m, lens, cols.astype(np.int32), val, x, f"stencil27_{g}")


# --------------------------------------------------------------------------
# config 3: power-law
# --------------------------------------------------------------------------
def _zipf_distinct_row(rng, target, n, a_col):
    """Distinct columns of one long power-law row, drawn in the "many draws" limit.

    Drawing N times from Zipf(a) over {1..n} and dropping duplicates keeps
    column k with probability 1 - exp(-tau * k^-a) (tau = N / zeta-normaliser),
    independently of the other columns to a very good approximation.  tau is
    chosen so that the expected number of distinct columns equals `target`
    (closed form of the sum for n -> infinity, minus the part beyond n).  The
    head (where the probability is not small) is drawn column by column; the
    far tail, where the probability is ~ tau * k^-a, as a Poisson process.
    Returns sorted distinct 0-based columns."""
    from math import gamma
    g = gamma(1.0 - 1.0 / a_col)                    # a=1.5: Gamma(1/3)
    pw = 1.0 / a_col                                # distinct(tau) ~ g * tau^(1/a)
    tail_c = 1.0 / (a_col - 1.0)                    # integral_n^inf k^-a dk = tail_c * n^(1-a)

    def expected(tau):
        return g * tau ** pw - tau * tail_c * n ** (1.0 - a_col)
    lo, hi = 1.0, 1.0
    while expected(hi) < target and hi < 1e18:
        hi *= 2.0
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if expected(mid) < target:
            lo = mid
        else:
            hi = mid
    tau = 0.5 * (lo + hi)
    K = int(min(n, max(64, 8.0 * tau ** pw)))       # beyond K the keep-probability is < 8^-a
    k = np.arange(1, K + 1, dtype=np.float64)
    keep = rng.random(K) < -np.expm1(-tau * k ** (-a_col))
    head = np.nonzero(keep)[0]                      # 0-based columns
    if K < n:
        e = 1.0 - a_col                             # cumulative intensity tau*tail_c*(K^e - k^e)
        lam_max = tau * tail_c * (K ** e - float(n) ** e)
        cnt = rng.poisson(lam_max)
        s = np.sort(rng.random(cnt)) * lam_max
        kk = (K ** e - s / (tau * tail_c)) ** (1.0 / e)
        tail = np.unique(np.clip(np.ceil(kk).astype(np.int64), K + 1, n)) - 1
        return np.concatenate([head, tail]).astype(np.int32)
    return head.astype(np.int32)


def _first_distinct(rng, targets, n, a_col):
    """For every row r: the first targets[r] DISTINCT values of a stream of
    (Zipf(a_col) - 1) mod n draws ("draw until the row has its length").
    Vectorised: draw a batch per row, keep first occurrences in draw order, repeat
    for the rows that are still short.  Returns (lens, cols), cols sorted inside
    each row."""
    m = targets.shape[0]
    nn = np.int64(n)
    have = np.empty(0, dtype=np.int64)               # accepted keys row*n + col
    need = targets.copy()
    for it in range(200):
        todo = np.nonzero(need > 0)[0]
        if todo.size == 0:
            break
        nd = need[todo]
        draws = np.where((it == 0) & (nd == 1), 1, np.ceil(1.7 * nd).astype(np.int64) + 2 + 2 * it)
        rows = np.repeat(todo, draws)
        new = rows * nn + (rng.zipf(a_col, size=rows.shape[0]) - 1) % n
        if have.size:
            mask = np.zeros(m, dtype=bool)
            mask[todo] = True
            ex = have[mask[have // nn]]              # what the unfinished rows already hold
        else:
            ex = have
        cand = np.concatenate([ex, new])
        uniq, first = np.unique(cand, return_index=True)
        fresh = first >= ex.shape[0]                 # values the row did not have yet
        uniq, first = uniq[fresh], first[fresh]
        urow = uniq // nn
        order = np.lexsort((first, urow))            # by row, then by draw order
        uniq, urow = uniq[order], urow[order]
        start = np.searchsorted(urow, urow, side="left")
        rank = np.arange(urow.shape[0]) - start
        acc = uniq[rank < need[urow]]
        have = np.concatenate([have, acc])
        need = need - np.bincount(acc // nn, minlength=m)
    have.sort()
    r = have // nn
    c = have - r * nn
    return np.bincount(r, minlength=m).astype(np.int64), c.astype(np.int32)


def powerlaw(m=2_000_000, a_len=2.0, a_col=1.5, max_len=200_000, long_above=256, seed=2) -> Csr:
    """Square power-law matrix.  Row length = clip(Zipf(a_len), 1, max_len) (mean
    about 8).  Columns are preferential toward low ids: the row's entries are the
    first `length` distinct values of a stream of (Zipf(a_col) - 1) mod n draws,
    sorted.  A row longer than `long_above` would need an astronomical number of
    draws, so it is drawn directly as the distinct set such a stream converges to
    (_zipf_distinct_row: expected length = the target).  Values and x ~ U[0, 1]."""
    rng = np.random.default_rng(seed)
    n = m
    max_len = min(max_len, n)
    target = np.clip(rng.zipf(a_len, size=m), 1, max_len).astype(np.int64)
    long_rows = np.nonzero(target > long_above)[0]
    short_t = target.copy()
    short_t[long_rows] = 0
    lens, c = _first_distinct(rng, short_t, n, a_col)
    if long_rows.size:
        start = np.zeros(m + 1, dtype=np.int64)
        np.cumsum(lens, out=start[1:])
        pieces = []
        prev = 0
        for r in long_rows:
            got = _zipf_distinct_row(rng, int(target[r]), n, a_col)
            pieces.append(c[start[prev]:start[r]])
            pieces.append(got)
            lens[r] = got.size
            prev = r + 1
        pieces.append(c[start[prev]:])
        c = np.concatenate(pieces)
    nnz = c.shape[0]
    val = rng.uniform(0.0, 1.0, size=nnz)
    x = rng.uniform(0.0, 1.0, size=n)
    return _finish(m, n, lens, c, val, x, f"powerlaw_{m}")


# --------------------------------------------------------------------------
# config 4: rectangular LP / circuit-like
# --------------------------------------------------------------------------
def lp_rect(m=1_500_000, n=4_000_000, empty_frac=0.30, geo_mean=4.0, dense_frac=0.001,
            dense_len=20_000, seed=3) -> Csr:
    """`empty_frac` of the rows are empty, `dense_frac` have `dense_len` entries,
    the rest have geometric lengths with mean `geo_mean`.  Uniform columns
    (duplicates dropped), values and x ~ N(0, 1)."""
    rng = np.random.default_rng(seed)
    dense_len = min(dense_len, n)
    u = rng.random(m)
    lens_t = rng.geometric(1.0 / geo_mean, size=m).astype(np.int64)
    lens_t = np.minimum(lens_t, n)
    lens_t[u < empty_frac] = 0
    lens_t[u >= 1.0 - dense_frac] = dense_len
    rows = np.repeat(np.arange(m, dtype=np.int64), lens_t)
    cols = rng.integers(0, n, size=rows.shape[0])
    lens, c = _dedupe_sorted(rows, cols, m, n)
    nnz = c.shape[0]
    val = rng.standard_normal(nnz)
    x = rng.standard_normal(n)
    return _finish(m, n, lens, c, val, x, f"lp_rect_{m}x{n}")


# --------------------------------------------------------------------------
# config 5: large mixed
# --------------------------------------------------------------------------
def mixed_large(m=8_000_000, band=5000, p_band=0.8, mu=2.5, sg=1.5, seed=4,
                chunk_rows=1_000_000) -> Csr:
    """Each row independently: with probability `p_band` a length uniform in
    {8..16} with columns within +-band of the diagonal (clipped to [0, n)), else
    a length floor(lognormal(mu, sg)) clipped to [1, n] with uniform columns.
    Duplicates inside a row are dropped.  Values and x ~ U[-1, 1].  Generated in
    row chunks to bound memory."""
    rng = np.random.default_rng(seed)
    n = m
    lens_all, cols_all = [], []
    for r0 in range(0, m, chunk_rows):
        r1 = min(m, r0 + chunk_rows)
        k = r1 - r0
        is_band = rng.random(k) < p_band
        lb = rng.integers(8, 17, size=k).astype(np.int64)
        ll = np.clip(np.floor(rng.lognormal(mu, sg, size=k)), 1, n).astype(np.int64)
        lt = np.where(is_band, lb, ll)
        rows = np.repeat(np.arange(k, dtype=np.int64), lt)
        rb = np.repeat(is_band, lt)
        tot = rows.shape[0]
        cu = rng.integers(0, n, size=tot)
        cb = rows + r0 + rng.integers(-band, band + 1, size=tot)
        np.clip(cb, 0, n - 1, out=cb)
        cols = np.where(rb, cb, cu)
        lens, c = _dedupe_sorted(rows, cols, k, n)
        lens_all.append(lens)
        cols_all.append(c)
    lens = np.concatenate(lens_all)
    c = np.concatenate(cols_all)
    nnz = c.shape[0]
    val = rng.uniform(-1.0, 1.0, size=nnz)
    x = rng.uniform(-1.0, 1.0, size=n)
    return _finish(m, n, lens, c, val, x, f"mixed_large_{m}")


# --------------------------------------------------------------------------
# the one matrix of the paper's suite that is fully specified in its text
# --------------------------------------------------------------------------
def dense(n=2000, seed=5) -> Csr:
    """Dense n x n matrix stored in CSR (Table 2, matrix r1 "Dense": 2K x 2K,
    4.0 M nonzeros, 2K per row; the only suite matrix that does not come from a
    collection).  Values and x ~ U[-1, 1]."""
    rng = np.random.default_rng(seed)
    lens = np.full(n, n, dtype=np.int64)
    cols = np.tile(np.arange(n, dtype=np.int32), n)
    val = rng.uniform(-1.0, 1.0, size=n * n)
    x = rng.uniform(-1.0, 1.0, size=n)
    return _finish(n, n, lens, cols, val, x, f"dense_{n}")


# --------------------------------------------------------------------------
# registry of the five headline workloads and their scaled-down versions
# --------------------------------------------------------------------------
def config(i: int, scale: float = 1.0) -> Csr:
    """Workload i in 1..5 (6 = the paper's dense 2K x 2K matrix, 8 = the smaller
    variant of workload 4; 7 lives in workloads_device) at full size
    (scale=1) or shrunk (scale<1 reduces the number of rows; the per-row
    distributions are unchanged)."""
    if i == 1:
        return tiny_uniform()
    if i == 2:
        g = max(4, int(round(100 * scale ** (1.0 / 3.0))))
        return stencil27(g=g)
    if i == 3:
        m = max(1000, int(2_000_000 * scale))
        return powerlaw(m=m, max_len=min(200_000, m))
    if i == 4:
        m = max(1000, int(1_500_000 * scale))
        nn = max(2000, int(4_000_000 * scale))
        return lp_rect(m=m, n=nn, dense_len=min(20_000, nn // 4))
    if i == 5:
        m = max(20_000, int(8_000_000 * scale))
        return mixed_large(m=m, band=min(5000, m // 4), chunk_rows=1_000_000)
    if i == 6:                      # extra: the paper's own dense matrix
        return dense(max(64, int(round(2000 * scale ** 0.5))))
    if i == 8:                      # extra: config 4 with 0.026 % dense rows, which meets its stated "~12 M" nonzeros
        m = max(1000, int(1_500_000 * scale))
        nn = max(2000, int(4_000_000 * scale))
        a = lp_rect(m=m, n=nn, dense_frac=0.00026, dense_len=min(20_000, nn // 4))
        a.name += "_b"
        return a
    raise ValueError(i)


# --------------------------------------------------------------------------
# small structured / degenerate matrices for pins and edge-case parity
# --------------------------------------------------------------------------
def from_row_lengths(lens, n, seed=0, name="custom", value_kind="uniform") -> Csr:
    """Matrix with the given row lengths, uniform distinct sorted columns."""
    rng = np.random.default_rng(seed)
    lens = np.minimum(np.asarray(lens, dtype=np.int64), n)
    m = lens.shape[0]
    tot = int(lens.sum())
    cols = np.empty(tot, dtype=np.int32)
    o = 0
    for i in range(m):
        k = int(lens[i])
        if k == 0:
            continue
        if k > n // 2:
            pick = np.sort(rng.permutation(n)[:k])
        else:
            pick = np.unique(rng.integers(0, n, size=k))
            while pick.size < k:
                pick = np.unique(np.concatenate([pick, rng.integers(0, n, size=k - pick.size)]))
        cols[o:o + k] = pick
        o += k
    if value_kind == "uniform":
        val = rng.uniform(-1.0, 1.0, size=tot)
    elif value_kind == "wide":       # magnitudes spread over many decades
        val = rng.uniform(-1.0, 1.0, size=tot) * 10.0 ** rng.integers(-8, 9, size=tot)
    else:
        raise ValueError(value_kind)
    x = rng.uniform(-1.0, 1.0, size=n)
    return _finish(m, n, lens, cols, val, x, name)


def identity(n) -> Csr:
    rng = np.random.default_rng(n)
    return _finish(n, n, np.ones(n, dtype=np.int64), np.arange(n, dtype=np.int32),
                   np.ones(n), rng.uniform(-1, 1, size=n), f"identity_{n}")


def permutation(n, seed=0) -> Csr:
    rng = np.random.default_rng(seed)
    perm = rng.permutation(n).astype(np.int32)
    return _finish(n, n, np.ones(n, dtype=np.int64), perm, np.ones(n),
                   rng.uniform(-1, 1, size=n), f"permutation_{n}")


def edge_cases(T: int, seed: int = 7) -> list:
    """Degenerate and boundary-straddling matrices for a tile of T = omega*sigma
    nonzeros: no nonzeros, fewer than one tile, exact multiples of a tile, one
    long row over several tiles, empty rows at the head / tail / between tiles,
    rows shorter than sigma, identity, permutation."""
    rng = np.random.default_rng(seed)
    out = []
    out.append(from_row_lengths([0] * 37, 50, seed, "all_empty"))
    out.append(from_row_lengths([5], 40, seed, "one_short_row"))
    out.append(from_row_lengths([T // 2, 0, 3], 2 * T, seed, "less_than_one_tile"))
    out.append(from_row_lengths([3 * T + 17], 4 * T, seed, "one_long_row"))
    out.append(from_row_lengths([T], T + 5, seed, "exactly_one_tile_one_row"))
    out.append(from_row_lengths([T // 4] * 8, T, seed, "exact_two_tiles"))
    out.append(from_row_lengths([0, 0, 0, 2 * T + 3, 0, 0, 5, 0, 0, 0], 3 * T, seed, "empties_head_tail"))
    # a row ends exactly on a tile boundary, followed by empty rows, then more rows
    out.append(from_row_lengths([T - 7, 7, 0, 0, 0, T // 2, T // 2, 0, 9], 2 * T, seed, "empties_at_tile_boundary"))
    out.append(from_row_lengths(np.ones(2 * T + 11, dtype=np.int64), 3 * T, seed, "all_len1"))
    out.append(from_row_lengths(rng.integers(0, 3, size=3 * T), 4 * T, seed, "len0to2"))
    out.append(from_row_lengths(rng.integers(0, 40, size=400), 3000, seed, "len0to39"))
    out.append(from_row_lengths([1, 2 * T, 1, 0, T + T // 2, 0, 0, 4, 3 * T, 2], 5 * T, seed, "long_rows_mixed"))
    out.append(from_row_lengths(rng.integers(0, 40, size=300), 2000, seed, "wide_values", value_kind="wide"))
    # dirty first tile whose first row is row 0  ("-0" tile pointer, Section 3.3)
    out.append(from_row_lengths([4, 0, T, 3], 2 * T, seed, "negative_zero_tile_ptr"))
    out.append(identity(T + 13))
    out.append(permutation(2 * T + 1, seed))
    return out


def structured_cases(T: int, seed: int = 11) -> list:
    """Classic sparsity structures, sized around a tile of T nonzeros: arrowhead
    (dense first row and column plus the diagonal), a band, dense diagonal blocks,
    a dense upper triangle, and a matrix whose rows hold unsorted, repeated column
    indices (a legal CSR matrix: repeated entries add up)."""
    rng = np.random.default_rng(seed)
    out = []

    def from_coo(m, n, rows, cols, name, sort=True):
        rows = np.asarray(rows, dtype=np.int64)
        cols = np.asarray(cols, dtype=np.int64)
        order = np.lexsort((cols, rows)) if sort else np.argsort(rows, kind="stable")
        rows, cols = rows[order], cols[order]
        lens = np.bincount(rows, minlength=m)
        val = rng.uniform(-1, 1, size=rows.shape[0])
        x = rng.uniform(-1, 1, size=n)
        return _finish(m, n, lens, cols, val, x, name)

    n = T + T // 2 + 3                                   # arrowhead: about 4.5 T nonzeros
    i = np.arange(1, n)
    out.append(from_coo(n, n, np.concatenate([np.zeros(n, np.int64), i, i]),
                        np.concatenate([np.arange(n), np.zeros(n - 1, np.int64), i]), f"arrowhead_{n}"))
    n = T // 2 + 7                                       # band of half-width 3
    r = np.repeat(np.arange(n), 7)
    c = r + np.tile(np.arange(-3, 4), n)
    keep = (c >= 0) & (c < n)
    out.append(from_coo(n, n, r[keep], c[keep], f"band7_{n}"))
    b, nb = 24, max(2, (2 * T) // (24 * 24) + 1)         # dense 24 x 24 blocks on the diagonal
    n = b * nb
    r = np.repeat(np.arange(n), b)
    c = (r // b) * b + np.tile(np.arange(b), n)
    out.append(from_coo(n, n, r, c, f"blockdiag{b}_{n}"))
    n = int(np.ceil(np.sqrt(2.0 * (T + T // 3))))        # dense upper triangle, a bit more than T nonzeros
    r, c = np.triu_indices(n)
    out.append(from_coo(n, n, r, c, f"upper_triangle_{n}"))
    m, n = 200, 97                                       # unsorted columns with repeats
    lens = rng.integers(0, 30, size=m)
    r = np.repeat(np.arange(m), lens)
    c = rng.integers(0, n, size=r.shape[0])
    a = from_coo(m, n, r, c, "unsorted_repeated_columns", sort=False)
    a.sorted_distinct = False
    out.append(a)
    return out
