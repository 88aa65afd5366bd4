"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and its pure-host entry points agree with the oracle."""
import ctypes
import os
import re

import pytest

import oracle
from paper_1503_05032_amd import binding as B
from paper_1503_05032_amd import build as libbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        libbuild.build(verbose=False)
    return B.load()


def test_header_symbols_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "csr5.h")).read()
    declared = set(re.findall(r"\b(csr5[sl]?_[a-z_0-9]+)\s*\(", hdr))
    declared -= {"csr5_handle_s"}
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def test_header_is_plain_c_and_links(lib, tmp_path):
    """The boundary is a C ABI: a C99 program that includes the header compiles
    without warnings, links against the library, and its host-only calls work
    without a GPU."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    src = tmp_path / "use_csr5.c"
    src.write_text("""
#include <stdio.h>
#include <string.h>
#include "csr5.h"
int main(void) {
    csr5_handle_t h = NULL;
    if (csr5_sigma_auto(27000000, 1000000) <= 0) return 1;
    if (csr5_workspace_bytes(1000, 26000, 16) == 0) return 2;
    if (csr5_workspace_bytes(-1, 10, 4) != 0) return 3;
    if (strcmp(csr5_strerror(CSR5_OK), "ok") != 0) return 4;
    if (csr5_convert_ex(-1, 1, 0, NULL, NULL, NULL, 0, NULL, 0, NULL, CSR5_FLAG_NONE, &h) != CSR5_EINVAL) return 5;
    if (h != NULL) return 6;
    if (csr5_free(NULL) != CSR5_OK) return 7;
    printf("%d %d\\n", CSR5_OMEGA, CSR5_SIGMA_MAX);
    return 0;
}
""")
    exe = tmp_path / "use_csr5"
    libdir = os.path.dirname(B.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
           str(src), "-o", str(exe), "-L", libdir, "-l:" + os.path.basename(B.LIB_PATH), "-Wl,-rpath," + libdir,
           "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True, stdin=subprocess.DEVNULL, timeout=120)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, stdin=subprocess.DEVNULL, timeout=60)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.split() == ["64", "48"]


def test_sigma_rule_matches_paper_shape(lib):
    # The library's rule is the four-way map of Section 3.2 with its own constants.
    # Recover them from its behaviour on a matrix large enough that the
    # small-matrix clamp is inactive, and compare with the oracle's rule.
    m = 40_000_000
    vals = [B.csr5_sigma_auto(q * m, m) for q in range(1, 400)]
    r, s, u = vals[0], max(vals), vals[-1]
    t = 256
    for q in range(1, 400):
        assert vals[q - 1] == oracle.sigma_rule(q * m, m, r, s, t, u), q
    assert B.csr5_sigma_auto(0, 0) == r
    assert all(B.CSR5_SIGMA_MIN <= v <= B.CSR5_SIGMA_MAX for v in vals)
    # small-matrix clamp: fewer than 12288 tiles  ->  sigma 8  (only up to t nonzeros per row)
    assert B.csr5_sigma_auto(12 * 1000, 1000) == 8
    big = 12288 * 64 * r
    assert B.csr5_sigma_auto(big, big // 12) == r
    assert B.csr5_sigma_auto(big - 1, big // 12) == 8
    assert B.csr5_sigma_auto(1000 * 1000, 1000) == u


def test_workspace_bytes(lib):
    assert B.csr5_workspace_bytes(-1, 10, 4) == 0
    assert B.csr5_workspace_bytes(10, 10, 49) == 0
    m, nnz, sigma = 1000, 26000, 16
    T = 64 * sigma
    p, pc = -(-nnz // T), nnz // T
    W = oracle.desc_words(64, sigma)
    need = (p + 1) * 4 + pc * W * 64 * 4 + (pc + 1) * 4 + min(m + pc, pc * T) * 4 + 4 * (p + 1) * 8 + 4
    need += 4 * (-(-pc // 4) + 1) * (8 + 4)    # one-launch SpMV (8 <= sigma <= 32, up to 32768 tiles): a meeting word and a counter per group of 4 tiles (+ the incomplete one), four times
    need += (p + 1) * 8                    # ... and per tile the groups of tiles its first row touches
    need += -(-pc // 4) * 160 * (4 + 8)    # copy of the last 160 entries of every 4th tile and of the last (8 <= sigma <= 16)
    need += (p + 1) * 4                    # per tile: how far into its first row it starts
    need += 8192 * 4                       # conversion scratch: one word per workgroup of the tile_ptr kernel
    got = B.csr5_workspace_bytes(m, nnz, sigma)
    assert need <= got <= need + 23 * 256
    # two tiles per workgroup from sigma 17 to 32: a copy for every 2nd tile
    T24 = 64 * 24
    p24, pc24 = -(-nnz // T24), nnz // T24
    need24 = ((p24 + 1) * 4 + pc24 * oracle.desc_words(64, 24) * 64 * 4 + (pc24 + 1) * 4 + min(m + pc24, pc24 * T24) * 4
              + 4 * ((p24 + 1) * 8 + (-(-pc24 // 2) + 1) * (8 + 4)) + (p24 + 1) * 8 + 4 + -(-pc24 // 2) * 160 * (4 + 8) + (p24 + 1) * 4 + 8192 * 4)
    assert need24 <= B.csr5_workspace_bytes(m, nnz, 24) <= need24 + 23 * 256
    # beyond 28 million nonzeros the copies hold 32 entries
    mb, nb = 3_000_000, 40_000_000
    Tb = 64 * 16
    pb, pcb = -(-nb // Tb), nb // Tb
    needb = ((pb + 1) * 4 + pcb * 64 * 4 + (pcb + 1) * 4 + min(mb + pcb, pcb * Tb) * 4 + 4 * (pb + 1) * 8 + 4
             + -(-pcb // 4) * 32 * (4 + 8) + (pb + 1) * 4 + 8192 * 4)
    # ... and beyond 32768 tiles the SpMV always takes two kernels: no meeting words, counters or groups
    assert needb <= B.csr5_workspace_bytes(mb, nb, 16) <= needb + 14 * 256
    # no such copy below sigma 8
    p4, pc4 = -(-nnz // 256), nnz // 256
    need4 = (p4 + 1) * 4 + pc4 * 64 * 4 + (pc4 + 1) * 4 + min(m + pc4, pc4 * 256) * 4 + 4 * (p4 + 1) * 8 + 4 + (p4 + 1) * 4 + 8192 * 4
    assert need4 <= B.csr5_workspace_bytes(m, nnz, 4) <= need4 + 12 * 256


def test_host_side_argument_errors(lib):
    # these return before any HIP call
    rc, h = B.csr5_convert_ex(-1, 1, 0, 0, 0, 0, check=False, stream=0)
    assert rc == B.CSR5_EINVAL and not h
    rc, h = B.csr5_convert_ex(1, 1, 0, 0, 0, 0, check=False, stream=0)
    assert rc == B.CSR5_EINVAL and not h
    assert B.csr5_free(None) == B.CSR5_OK
    assert B.csr5_strerror(B.CSR5_ERANGE).startswith("sigma out of range")
    # flag bits nobody defined, and the two measurement flags that contradict each other (dummy aligned addresses)
    for flags in (8, 1 << 31, B.CSR5_FLAG_AUX_TWO_KERNELS | B.CSR5_FLAG_AUX_ONE_KERNEL):
        rc, h = B.csr5_convert_ex(10, 10, 20, 256, 256, 256, sigma=16, flags=flags, check=False, stream=0)
        assert rc == B.CSR5_EINVAL and not h
    hdr = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "csr5.h")).read()
    for name in ("CSR5_FLAG_NO_HOST_CHECK", "CSR5_FLAG_AUX_TWO_KERNELS", "CSR5_FLAG_AUX_ONE_KERNEL"):
        assert int(re.search(r"#define\s+" + name + r"\s+(\d+)u", hdr).group(1)) == getattr(B, name)


def test_wide_variant_limits(lib):
    # 8-byte tile_ptr and empty_offset_ptr entries
    m, nnz, sigma = 1000, 26000, 16
    T = 64 * sigma
    p, pc = -(-nnz // T), nnz // T
    W = oracle.desc_words(64, sigma)
    need = (p + 1) * 8 + pc * W * 64 * 4 + (pc + 1) * 8 + min(m + pc, pc * T) * 4 + 4 * (p + 1) * 8 + 4
    need += -(-pc // 4) * 160 * (4 + 8) + (p + 1) * 4 + 8192 * 4
    need += 4 * (-(-pc // 4) + 1) * (8 + 4) + (p + 1) * 8    # one-launch SpMV: meeting words and counters per group of tiles, groups per row
    got = B.csr5l_workspace_bytes(m, nnz, sigma)
    assert need <= got <= need + 23 * 256
    # beyond 2^31 nonzeros; the limit is the number of tiles (2^26 - 5)
    assert B.csr5l_workspace_bytes(6_400_000, 2_300_000_000, 16) > 2_300_000_000 // 1024 * 64 * 4
    most = (2**26 - 5) * 64 * 16
    assert B.csr5l_workspace_bytes(1000, most, 16) > 0
    assert B.csr5l_workspace_bytes(1000, most + 1, 16) == 0
    assert B.csr5l_workspace_bytes(1000, most, 15) == 0
    # the conversion refuses such a matrix before touching any pointer (dummy addresses)
    rc, h = B.csr5l_convert_ex(1000, 1000, most + 1, 256, 256, 256, sigma=16, check=False, stream=0)
    assert rc == B.CSR5_ERANGE and not h
    rc, h = B.csr5_convert_ex(2**31 - 1, 1000, 100, 256, 256, 256, sigma=16, check=False, stream=0)
    assert rc == B.CSR5_ERANGE and not h          # m + 1 must fit 32 bits
    assert B.csr5_workspace_bytes(2**31 - 2, 100, 16) > 0
    rc, h = B.csr5l_convert_ex(1000, 1000, 100, 260, 256, 256, sigma=16, check=False, stream=0)
    assert rc == B.CSR5_EINVAL and not h          # int64 row_ptr must be 8-byte aligned
