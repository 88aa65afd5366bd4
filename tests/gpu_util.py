"""Helpers shared by the GPU parity tests: run the HIP library through its
binding on a workloads.Csr and compare against the CPU oracle."""
import numpy as np
import torch

import oracle
from paper_1503_05032_amd import binding as B

TOL_REL = 1e-12      # |y_gpu - y_ref| <= TOL_REL * sum_j |a_ij x_j| + TOL_ABS   (per row)
TOL_ABS = 1e-300


class DeviceCsr:
    def __init__(self, a, wide=False):
        dev = torch.device("cuda:0")
        self.a = a
        self.wide = wide            # 64-bit index variant: int64 row_ptr, csr5l_ entry points
        self.row_ptr = torch.from_numpy(a.row_ptr.astype(np.int64) if wide else a.row_ptr).to(dev)
        self.col_idx = torch.from_numpy(a.col_idx).to(dev) if a.nnz else torch.zeros(1, dtype=torch.int32, device=dev)
        self.val = torch.from_numpy(a.val).to(dev) if a.nnz else torch.zeros(1, dtype=torch.float64, device=dev)
        self.x = torch.from_numpy(a.x).to(dev) if a.n else torch.zeros(1, dtype=torch.float64, device=dev)
        self.y = torch.full((max(a.m, 1),), float("nan"), dtype=torch.float64, device=dev)


def convert(d, sigma=0, use_workspace=True, flags=B.CSR5_FLAG_NONE):
    a = d.a
    ws = None
    if use_workspace:
        nbytes = (B.csr5l_workspace_bytes if d.wide else B.csr5_workspace_bytes)(a.m, a.nnz, sigma)
        assert nbytes > 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        assert ws.data_ptr() % 256 == 0
    h = (B.csr5l_convert_ex if d.wide else B.csr5_convert_ex)(a.m, a.n, a.nnz, d.row_ptr, d.col_idx, d.val, sigma=sigma, workspace=ws,
                          flags=flags)
    d.workspace = ws
    return h


def check_format(d, h, label=""):
    """Bit-exact comparison of every CSR5 array with the oracle's."""
    a = d.a
    info = B.csr5_get_info(h)
    assert info["omega"] == 64
    sigma = info["sigma"]
    ref = oracle.convert(a.m, a.n, a.nnz, a.row_ptr, a.col_idx, a.val, 64, sigma)
    assert info["p"] == ref.p and info["p_complete"] == ref.pc, label
    assert info["desc_words_per_lane"] == ref.W, label
    st = B.csr5_status(h)
    assert st & 3 == 0 and st < 16, (label, st)        # no error bit, nothing but the four documented bits
    tp = B.csr5_read_array(h, B.CSR5_ARRAY_TILE_PTR, wide=d.wide)
    if d.wide:      # same row indices, flag in bit 63 instead of bit 31, nothing in between
        assert tp.dtype == np.uint64 and not ((tp >> np.uint64(31)) & np.uint64(0xffffffff)).any(), label
        tp = ((tp & np.uint64(0x7fffffff)) | ((tp >> np.uint64(63)) << np.uint64(31))).astype(np.uint32)
    assert np.array_equal(tp, ref.tile_ptr), (label, "tile_ptr", _first_diff(tp, ref.tile_ptr))
    assert bool(st & B.CSR5_STATUS_HAS_DIRTY) == bool((ref.tile_ptr >> 31).any()), label
    td = B.csr5_read_array(h, B.CSR5_ARRAY_TILE_DESC)
    assert np.array_equal(td, ref.tile_desc), (label, "tile_desc", _first_diff(td, ref.tile_desc))
    eop = B.csr5_read_array(h, B.CSR5_ARRAY_EMPTY_OFFSET_PTR, wide=d.wide)
    assert eop.dtype == (np.int64 if d.wide else np.int32)
    assert np.array_equal(eop, ref.empty_offset_ptr), (label, "empty_offset_ptr", _first_diff(eop, ref.empty_offset_ptr))
    assert info["empty_offset_len"] == ref.empty_offset.shape[0], label
    eo = B.csr5_read_array(h, B.CSR5_ARRAY_EMPTY_OFFSET)
    assert np.array_equal(eo, ref.empty_offset), (label, "empty_offset", _first_diff(eo, ref.empty_offset))
    if a.nnz:
        col = d.col_idx.cpu().numpy()
        val = d.val.cpu().numpy()
        assert np.array_equal(col, ref.col_idx), (label, "col_idx", _first_diff(col, ref.col_idx))
        assert np.array_equal(val.view(np.uint64), ref.val.view(np.uint64)), (label, "val")
    return ref


def _first_diff(a, b):
    if a.shape != b.shape:
        return ("shape", a.shape, b.shape)
    k = np.nonzero(a != b)[0]
    return None if k.size == 0 else (int(k[0]), int(a[k[0]]), int(b[k[0]]), int(k.size))


def check_spmv(d, h, label="", x=None):
    a = d.a
    if x is not None:
        d.x = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    xh = d.x.cpu().numpy()[:a.n] if a.n else np.zeros(0)
    d.y.fill_(float("nan"))
    B.csr5_spmv_ex(h, d.x, d.y)
    torch.cuda.synchronize()
    y = d.y.cpu().numpy()[:a.m]
    y_ref, s = oracle.csr_spmv(a.m, a.row_ptr, a.col_idx, a.val, xh)
    err = np.abs(y - y_ref)
    tol = TOL_REL * s + TOL_ABS
    bad = np.nonzero(~(err <= tol))[0]          # also catches NaN
    assert bad.size == 0, (label, "rows out of tolerance", int(bad.size), int(bad[0]),
                           float(y[bad[0]]), float(y_ref[bad[0]]), float(s[bad[0]]))
    empty = np.diff(a.row_ptr) == 0
    assert np.all(y[empty] == 0.0), (label, "empty rows must be exactly zero")
    return float((err / np.maximum(s, 1e-300)).max()) if a.m else 0.0


def tile_reference(row_ptr, m, n, t, T, sigma, col_tile, val_tile):
    """The oracle's conversion of the stand-alone matrix that consists of tile t's
    entries: rows tile_ptr[t] .. (last row that starts before the tile ends), row
    boundaries clipped to the tile.  Its only tile has the descriptor, the
    empty-row flag, the empty_offset entries and the transposed arrays that tile
    t has inside the big matrix (the forced first flag is what makes the two
    agree when the tile starts in the middle of a row)."""
    lo, hi = t * T, (t + 1) * T
    r0 = int(np.searchsorted(row_ptr, lo, side="right")) - 1
    r1 = int(np.searchsorted(row_ptr, hi, side="right")) - 1
    r_end = r1 - 1 if row_ptr[min(r1, m)] == hi else r1
    rp = (np.clip(row_ptr[r0:r_end + 2], lo, hi) - lo).astype(np.int32)
    assert rp[0] == 0 and rp[-1] == T
    ref = oracle.convert(r_end - r0 + 1, n, T, rp, col_tile, val_tile, 64, sigma)
    return r0, ref


def second_kernel_ms(h, x, y, reps=100):
    """Mean duration per call of the SpMV's second kernel (ms), 0 when none is
    launched: the smaller of two series, so that a hiccup of the host between the
    two event records of an empty series is not taken for a kernel (a launched
    second kernel takes about 3e-3 ms per call, an empty series about 1e-4)."""
    best = min(B.csr5_spmv_profile(h, x, y, reps=reps)[1] for _ in range(2))
    torch.cuda.synchronize()
    return best

