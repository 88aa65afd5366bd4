"""CPU oracle for CSR5 -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over `csr5_oracle.c` (plain sequential C written from the
paper's definitions).  Only `tests/`, the smoke entry and the benchmark's
`cpu_baseline` leg may import this package; the product (the HIP library and
its Python binding) never does, and this package imports nothing of the
product.

Every function takes and returns NumPy arrays; nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csr5_oracle.c")
_SO = os.path.join(_HERE, "libcsr5_oracle.so")
_lib = None

DIRTY = 0x80000000


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math).  Returns the .so path."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC])
        os.replace(tmp, _SO)
    return _SO


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_tiles.restype = C.c_int64
        _lib.oracle_num_tiles.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        _lib.oracle_num_complete_tiles.restype = C.c_int64
        _lib.oracle_num_complete_tiles.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        _lib.oracle_desc_bits.restype = C.c_int32
        _lib.oracle_desc_bits.argtypes = [C.c_int32, C.c_int32]
        _lib.oracle_desc_words.restype = C.c_int32
        _lib.oracle_desc_words.argtypes = [C.c_int32, C.c_int32]
        _lib.oracle_sigma_rule.restype = C.c_int32
        _lib.oracle_sigma_rule.argtypes = [C.c_int64, C.c_int64] + [C.c_int32] * 4
        for name in ("oracle_csr_spmv", "oracle_tile_ptr", "oracle_bit_flag", "oracle_y_seg_offset",
                     "oracle_pack_desc", "oracle_empty_offset", "oracle_transpose",
                     "oracle_csr5_spmv"):
            getattr(_lib, name).restype = None
        _lib.oracle_csr_spmv_all_cores.restype = C.c_int32
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def csr_spmv(m, row_ptr, col_idx, val, x):
    """Algorithm 1.  Returns (y, abs_sum) with abs_sum[i] = sum_j |a_ij x_j|."""
    row_ptr, col_idx, val, x = _i32(row_ptr), _i32(col_idx), _f64(val), _f64(x)
    y = np.empty(m, dtype=np.float64)
    s = np.empty(m, dtype=np.float64)
    lib().oracle_csr_spmv(C.c_int32(m), _p(row_ptr, C.c_int32), _p(col_idx, C.c_int32),
                          _p(val, C.c_double), _p(x, C.c_double), _p(y, C.c_double),
                          _p(s, C.c_double))
    return y, s


def csr_spmv_all_cores(m, row_ptr, col_idx, val, x):
    """Algorithm 1 with the rows shared among the host's cores (OpenMP); the same
    values as csr_spmv.  Returns (y, abs_sum, threads used)."""
    row_ptr, col_idx, val, x = _i32(row_ptr), _i32(col_idx), _f64(val), _f64(x)
    y = np.empty(m, dtype=np.float64)
    s = np.empty(m, dtype=np.float64)
    nt = lib().oracle_csr_spmv_all_cores(C.c_int32(m), _p(row_ptr, C.c_int32), _p(col_idx, C.c_int32),
                                         _p(val, C.c_double), _p(x, C.c_double), _p(y, C.c_double),
                                         _p(s, C.c_double))
    return y, s, int(nt)


def num_tiles(nnz, omega, sigma):
    return int(lib().oracle_num_tiles(nnz, omega, sigma))


def num_complete_tiles(nnz, omega, sigma):
    return int(lib().oracle_num_complete_tiles(nnz, omega, sigma))


def desc_bits(omega, sigma):
    return int(lib().oracle_desc_bits(omega, sigma))


def desc_words(omega, sigma):
    return int(lib().oracle_desc_words(omega, sigma))


def sigma_rule(nnz, m, r, s, t, u):
    return int(lib().oracle_sigma_rule(nnz, m, r, s, t, u))


def tile_ptr(m, nnz, row_ptr, omega, sigma):
    """Algorithm 4.  uint32[p+1], top bit = tile holds an empty row."""
    row_ptr = _i32(row_ptr)
    p = num_tiles(nnz, omega, sigma)
    out = np.zeros(p + 1, dtype=np.uint32)
    lib().oracle_tile_ptr(C.c_int32(m), C.c_int32(nnz), _p(row_ptr, C.c_int32),
                          C.c_int32(omega), C.c_int32(sigma), _p(out, C.c_uint32))
    return out


def bit_flag(m, nnz, row_ptr, omega, sigma):
    """Section 3.4.  uint8[pc, omega, sigma] (column i, row j)."""
    row_ptr = _i32(row_ptr)
    pc = num_complete_tiles(nnz, omega, sigma)
    out = np.zeros((pc, omega, sigma), dtype=np.uint8)
    lib().oracle_bit_flag(C.c_int32(m), C.c_int32(nnz), _p(row_ptr, C.c_int32),
                          C.c_int32(omega), C.c_int32(sigma), _p(out, C.c_uint8))
    return out


def y_seg_offset(bf):
    """Algorithm 5.  Returns (y_offset, seg_offset), int32[pc, omega] each."""
    bf = np.ascontiguousarray(bf, dtype=np.uint8)
    pc, omega, sigma = bf.shape
    yo = np.zeros((pc, omega), dtype=np.int32)
    so = np.zeros((pc, omega), dtype=np.int32)
    lib().oracle_y_seg_offset(C.c_int64(pc), C.c_int32(omega), C.c_int32(sigma),
                              _p(bf, C.c_uint8), _p(yo, C.c_int32), _p(so, C.c_int32))
    return yo, so


def pack_desc(bf, yo, so):
    """Section 3.5.  uint32[pc * W * omega]."""
    bf = np.ascontiguousarray(bf, dtype=np.uint8)
    pc, omega, sigma = bf.shape
    W = desc_words(omega, sigma)
    out = np.zeros(pc * W * omega, dtype=np.uint32)
    yo, so = _i32(yo), _i32(so)
    lib().oracle_pack_desc(C.c_int64(pc), C.c_int32(omega), C.c_int32(sigma), _p(bf, C.c_uint8),
                           _p(yo, C.c_int32), _p(so, C.c_int32), _p(out, C.c_uint32))
    return out


def empty_offset(m, nnz, row_ptr, omega, sigma, tptr, bf):
    """Algorithm 7.  Returns (empty_offset_ptr int32[pc+1], empty_offset int32[E])."""
    row_ptr = _i32(row_ptr)
    bf = np.ascontiguousarray(bf, dtype=np.uint8)
    tptr = np.ascontiguousarray(tptr, dtype=np.uint32)
    pc = num_complete_tiles(nnz, omega, sigma)
    eop = np.zeros(pc + 1, dtype=np.int32)
    args = [C.c_int32(m), C.c_int32(nnz), _p(row_ptr, C.c_int32), C.c_int32(omega),
            C.c_int32(sigma), _p(tptr, C.c_uint32), _p(bf, C.c_uint8), _p(eop, C.c_int32)]
    lib().oracle_empty_offset(*args, None)
    eo = np.zeros(max(int(eop[pc]), 1), dtype=np.int32)
    lib().oracle_empty_offset(*args, _p(eo, C.c_int32))
    return eop, eo[:int(eop[pc])]


def transpose(nnz, omega, sigma, col_idx, val):
    """Section 3.1 tile transposition (out of place)."""
    col_idx, val = _i32(col_idx), _f64(val)
    co = np.empty_like(col_idx)
    vo = np.empty_like(val)
    lib().oracle_transpose(C.c_int32(nnz), C.c_int32(omega), C.c_int32(sigma),
                           _p(col_idx, C.c_int32), _p(val, C.c_double),
                           _p(co, C.c_int32), _p(vo, C.c_double))
    return co, vo


@dataclass
class Csr5:
    """All five groups of CSR5 data plus the unpacked descriptor parts."""
    m: int
    n: int
    nnz: int
    omega: int
    sigma: int
    p: int
    pc: int
    W: int
    row_ptr: np.ndarray
    tile_ptr: np.ndarray
    tile_desc: np.ndarray
    empty_offset_ptr: np.ndarray
    empty_offset: np.ndarray
    col_idx: np.ndarray        # tile-transposed
    val: np.ndarray            # tile-transposed
    bit_flag: np.ndarray
    y_offset: np.ndarray
    seg_offset: np.ndarray


def convert(m, n, nnz, row_ptr, col_idx, val, omega, sigma) -> Csr5:
    """CSR -> CSR5, the steps of Sections 3.3-3.5 in the paper's order."""
    tp = tile_ptr(m, nnz, row_ptr, omega, sigma)
    bf = bit_flag(m, nnz, row_ptr, omega, sigma)
    yo, so = y_seg_offset(bf)
    td = pack_desc(bf, yo, so)
    eop, eo = empty_offset(m, nnz, row_ptr, omega, sigma, tp, bf)
    ct, vt = transpose(nnz, omega, sigma, col_idx, val)
    return Csr5(m, n, nnz, omega, sigma, num_tiles(nnz, omega, sigma),
                num_complete_tiles(nnz, omega, sigma), desc_words(omega, sigma),
                _i32(row_ptr), tp, td, eop, eo, ct, vt, bf, yo, so)


def csr5_spmv(a: Csr5, x):
    """Algorithm 8 run sequentially over the CSR5 arrays."""
    x = _f64(x)
    y = np.empty(a.m, dtype=np.float64)
    eo = a.empty_offset if a.empty_offset.size else np.zeros(1, dtype=np.int32)
    td = a.tile_desc if a.tile_desc.size else np.zeros(1, dtype=np.uint32)
    lib().oracle_csr5_spmv(C.c_int32(a.m), C.c_int32(a.nnz), _p(a.row_ptr, C.c_int32),
                           C.c_int32(a.omega), C.c_int32(a.sigma), _p(a.tile_ptr, C.c_uint32),
                           _p(td, C.c_uint32), _p(a.empty_offset_ptr, C.c_int32),
                           _p(eo, C.c_int32), _p(a.col_idx, C.c_int32), _p(a.val, C.c_double),
                           _p(x, C.c_double), _p(y, C.c_double))
    return y
