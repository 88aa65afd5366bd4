"""ctypes binding of libcsr5 (include/csr5.h).  Argument marshalling only: every
step of the conversion and of the SpMV runs in the library's HIP kernels.

Functions carry the C names.  Array arguments are torch tensors on the GPU (or
raw integer device addresses); PyTorch is used for device memory and streams
only.  A non-zero return code raises Csr5Error unless check=False.

The shared library must have been built (paper_1503_05032_amd/build.py); there
is no fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcsr5.so")

CSR5_OK, CSR5_EINVAL, CSR5_ENOMEM, CSR5_EHIP, CSR5_ERANGE = 0, -1, -2, -3, -4
CSR5_OMEGA, CSR5_SIGMA_MIN, CSR5_SIGMA_MAX = 64, 1, 48
CSR5_STATIC_SCRATCH_BYTES = 4 << 20
CSR5_STATIC_MAX_TILES = CSR5_STATIC_SCRATCH_BYTES // 8 - 1
CSR5_FLAG_NONE, CSR5_FLAG_NO_HOST_CHECK = 0, 1
CSR5_FLAG_AUX_TWO_KERNELS, CSR5_FLAG_AUX_ONE_KERNEL = 2, 4
CSR5_STATUS_BAD_ROW_PTR, CSR5_STATUS_BAD_COL_IDX, CSR5_STATUS_HAS_DIRTY = 1, 2, 4
CSR5_STATUS_HAS_EMPTY_ROWS = 8
CSR5_ARRAY_TILE_PTR, CSR5_ARRAY_TILE_DESC, CSR5_ARRAY_EMPTY_OFFSET_PTR, CSR5_ARRAY_EMPTY_OFFSET = 0, 1, 2, 3

# every symbol include/csr5.h declares
SYMBOLS = [
    "csr5_sigma_auto", "csr5_workspace_bytes", "csr5_convert", "csr5_convert_ex", "csr5_spmv",
    "csr5_spmv_ex", "csr5_spmv_static", "csr5_spmv_profile", "csr5_stream_floor", "csr5_to_csr", "csr5_free", "csr5_status", "csr5_get_info",
    "csr5_get_shape", "csr5_get_arrays",
    "csr5_read_array", "csr5_strerror", "csr5_baseline_csr_scalar", "csr5_baseline_csr_vector",
    "csr5s_convert_ex", "csr5s_spmv_ex", "csr5s_spmv_profile",
    "csr5l_workspace_bytes", "csr5l_convert_ex", "csr5l_get_arrays",
]


class Csr5Error(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {csr5_strerror(code)} ({code})")


_lib = None


def load():
    """Loads libcsr5.so.  torch is imported first so that the library binds to
    the HIP runtime torch already brought into the process."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           f"`python {os.path.join(_PKG, 'build.py')}` (there is no fallback)")
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_size_t
    lib.csr5_sigma_auto.restype = i32
    lib.csr5_sigma_auto.argtypes = [i64, i64]
    lib.csr5_workspace_bytes.restype = sz
    lib.csr5_workspace_bytes.argtypes = [i32, i32, i32]
    lib.csr5_convert.restype = C.c_int
    lib.csr5_convert.argtypes = [i32, i32, i32, vp, vp, vp, C.POINTER(vp)]
    lib.csr5_convert_ex.restype = C.c_int
    lib.csr5_convert_ex.argtypes = [i32, i32, i32, vp, vp, vp, i32, vp, sz, vp, u32, C.POINTER(vp)]
    lib.csr5s_convert_ex.restype = C.c_int
    lib.csr5s_convert_ex.argtypes = [i32, i32, i32, vp, vp, vp, i32, vp, sz, vp, u32, C.POINTER(vp)]
    lib.csr5l_workspace_bytes.restype = sz
    lib.csr5l_workspace_bytes.argtypes = [i32, i64, i32]
    lib.csr5l_convert_ex.restype = C.c_int
    lib.csr5l_convert_ex.argtypes = [i32, i32, i64, vp, vp, vp, i32, vp, sz, vp, u32, C.POINTER(vp)]
    lib.csr5l_get_arrays.restype = C.c_int
    lib.csr5l_get_arrays.argtypes = [vp] + [C.POINTER(vp)] * 4
    lib.csr5s_spmv_ex.restype = C.c_int
    lib.csr5s_spmv_ex.argtypes = [vp, vp, vp, vp]
    lib.csr5s_spmv_profile.restype = C.c_int
    lib.csr5s_spmv_profile.argtypes = [vp, vp, vp, vp, C.c_int, C.POINTER(C.c_float)]
    lib.csr5_spmv.restype = C.c_int
    lib.csr5_spmv.argtypes = [vp, vp, vp]
    lib.csr5_spmv_ex.restype = C.c_int
    lib.csr5_spmv_ex.argtypes = [vp, vp, vp, vp]
    lib.csr5_spmv_static.restype = C.c_int
    lib.csr5_spmv_static.argtypes = [vp, vp, vp, vp]
    lib.csr5_spmv_profile.restype = C.c_int
    lib.csr5_spmv_profile.argtypes = [vp, vp, vp, vp, C.c_int, C.POINTER(C.c_float)]
    lib.csr5_stream_floor.restype = C.c_int
    lib.csr5_stream_floor.argtypes = [vp, vp, C.c_size_t, vp, C.c_int, C.POINTER(C.c_float)]
    lib.csr5_to_csr.restype = C.c_int
    lib.csr5_to_csr.argtypes = [vp, vp]
    lib.csr5_free.restype = C.c_int
    lib.csr5_free.argtypes = [vp]
    lib.csr5_status.restype = C.c_int
    lib.csr5_status.argtypes = [vp, C.POINTER(u32)]
    lib.csr5_get_info.restype = C.c_int
    lib.csr5_get_info.argtypes = [vp] + [C.POINTER(i32)] * 6
    lib.csr5_get_shape.restype = C.c_int
    lib.csr5_get_shape.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    lib.csr5_get_arrays.restype = C.c_int
    lib.csr5_get_arrays.argtypes = [vp] + [C.POINTER(vp)] * 4
    lib.csr5_read_array.restype = C.c_int
    lib.csr5_read_array.argtypes = [vp, C.c_int, vp, sz]
    lib.csr5_baseline_csr_scalar.restype = C.c_int
    lib.csr5_baseline_csr_scalar.argtypes = [i32, vp, vp, vp, vp, vp, vp]
    lib.csr5_baseline_csr_vector.restype = C.c_int
    lib.csr5_baseline_csr_vector.argtypes = [i32, i32, vp, vp, vp, vp, vp, i32, vp]
    lib.csr5_strerror.restype = C.c_char_p
    lib.csr5_strerror.argtypes = [C.c_int]
    _lib = lib
    return lib


def _ptr(t):
    """Device address of a torch tensor (or pass an int / None through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t or None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return t.data_ptr() or None


_DTYPES: dict = {}      # filled on first use (torch is imported by load())


def _arr(t, dtypes, min_numel, name):
    """Device address of a torch tensor after checking what the library cannot
    check: element type and length.  A wrong one would make a kernel read or
    write outside the tensor, so it is refused here, on the host.  Integers
    (raw device addresses) and None pass through unchecked."""
    if t is None or isinstance(t, int):
        return _ptr(t)
    if not _DTYPES:
        import torch
        _DTYPES.update({"i32": torch.int32, "i64": torch.int64, "f64": torch.float64, "f32": torch.float32,
                        "u8": torch.uint8})
    if not any(t.dtype is _DTYPES[d] for d in dtypes):
        raise ValueError(f"{name}: expected dtype {' or '.join(dtypes)}, got {t.dtype}")
    if t.numel() < min_numel:
        raise ValueError(f"{name}: needs at least {min_numel} elements, has {t.numel()}")
    return _ptr(t)


def _csr_args(m, n, nnz, row_ptr, col_idx, val, index, value):
    return (_arr(row_ptr, [index], m + 1, "row_ptr"), _arr(col_idx, ["i32"], nnz, "col_idx"),
            _arr(val, [value], nnz, "val"))


def _stream(s):
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


def _chk(rc, where, check):
    if check and rc != CSR5_OK:
        raise Csr5Error(rc, where)
    return rc


def csr5_strerror(code):
    return load().csr5_strerror(int(code)).decode()


def csr5_sigma_auto(nnz, m):
    return int(load().csr5_sigma_auto(int(nnz), int(m)))


def csr5_workspace_bytes(m, nnz, sigma=0):
    return int(load().csr5_workspace_bytes(int(m), int(nnz), int(sigma)))


def csr5_convert(m, n, nnz, row_ptr, col_idx, val, check=True):
    """Returns the handle (an integer).  Uses the default stream and hipMalloc."""
    h = C.c_void_p()
    rc = load().csr5_convert(m, n, nnz, *_csr_args(m, n, nnz, row_ptr, col_idx, val, "i32", "f64"), C.byref(h))
    _chk(rc, "csr5_convert", check)
    return h.value if check else (rc, h.value)


def csr5_convert_ex(m, n, nnz, row_ptr, col_idx, val, sigma=0, workspace=None, stream=None,
                    flags=CSR5_FLAG_NONE, check=True):
    """`workspace` is a torch uint8 GPU tensor (or None -> hipMalloc inside)."""
    h = C.c_void_p()
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().csr5_convert_ex(m, n, nnz, *_csr_args(m, n, nnz, row_ptr, col_idx, val, "i32", "f64"), int(sigma),
                                _arr(workspace, ["u8"], 0, "workspace"), wsb, _stream(stream), int(flags), C.byref(h))
    _chk(rc, "csr5_convert_ex", check)
    return h.value if check else (rc, h.value)


def csr5s_convert_ex(m, n, nnz, row_ptr, col_idx, val, sigma=0, workspace=None, stream=None,
                     flags=CSR5_FLAG_NONE, check=True):
    """Single precision: `val` is a float32 GPU tensor."""
    h = C.c_void_p()
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().csr5s_convert_ex(m, n, nnz, *_csr_args(m, n, nnz, row_ptr, col_idx, val, "i32", "f32"), int(sigma),
                                 _arr(workspace, ["u8"], 0, "workspace"), wsb, _stream(stream), int(flags), C.byref(h))
    _chk(rc, "csr5s_convert_ex", check)
    return h.value if check else (rc, h.value)


def csr5l_workspace_bytes(m, nnz, sigma=0):
    return int(load().csr5l_workspace_bytes(int(m), int(nnz), int(sigma)))


def csr5l_convert_ex(m, n, nnz, row_ptr, col_idx, val, sigma=0, workspace=None, stream=None,
                     flags=CSR5_FLAG_NONE, check=True):
    """64-bit index variant: `row_ptr` is an int64 GPU tensor, nnz may exceed 2^31."""
    h = C.c_void_p()
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().csr5l_convert_ex(m, n, int(nnz), *_csr_args(m, n, nnz, row_ptr, col_idx, val, "i64", "f64"), int(sigma),
                                 _arr(workspace, ["u8"], 0, "workspace"), wsb, _stream(stream), int(flags), C.byref(h))
    _chk(rc, "csr5l_convert_ex", check)
    return h.value if check else (rc, h.value)


def csr5l_get_arrays(h, check=True):
    """Device addresses of a 64-bit-index handle's arrays."""
    v = [C.c_void_p() for _ in range(4)]
    rc = _chk(load().csr5l_get_arrays(h, *[C.byref(a) for a in v]), "csr5l_get_arrays", check)
    if rc != CSR5_OK:
        return rc
    return dict(zip(["tile_ptr", "tile_desc", "empty_offset_ptr", "empty_offset"], [a.value for a in v]))


_shapes: dict = {}      # handle -> (m, n), so that an SpMV call costs no extra library call


def _xy(h, x, y, value):
    """x and y of an SpMV: element type of the entry point, at least n and m elements."""
    if not h:
        m, n = 0, 0
    else:
        mn = _shapes.get(h)
        if mn is None:
            mn = _shapes[h] = csr5_get_shape(h)
        m, n = mn
    return _arr(x, [value], n, "x"), _arr(y, [value], m, "y")


def csr5_get_shape(h):
    """(m, n) of the handle's matrix."""
    m, n = C.c_int32(), C.c_int32()
    _chk(load().csr5_get_shape(h, C.byref(m), C.byref(n)), "csr5_get_shape", True)
    return m.value, n.value


def csr5s_spmv_ex(h, x, y, stream=None, check=True):
    return _chk(load().csr5s_spmv_ex(h, *_xy(h, x, y, "f32"), _stream(stream)), "csr5s_spmv_ex", check)


def csr5s_spmv_profile(h, x, y, reps, stream=None):
    ms = (C.c_float * 2)()
    _chk(load().csr5s_spmv_profile(h, *_xy(h, x, y, "f32"), _stream(stream), int(reps), ms),
         "csr5s_spmv_profile", True)
    return float(ms[0]), float(ms[1])


def csr5_spmv(h, x, y, check=True):
    return _chk(load().csr5_spmv(h, *_xy(h, x, y, "f64")), "csr5_spmv", check)


def csr5_spmv_ex(h, x, y, stream=None, check=True):
    return _chk(load().csr5_spmv_ex(h, *_xy(h, x, y, "f64"), _stream(stream)), "csr5_spmv_ex", check)


def csr5_spmv_bound(h, x, y, stream=None):
    """csr5_spmv_ex (csr5s_spmv_ex for float32 tensors) with its arguments checked
    and marshalled once: returns a function of no arguments that makes the call,
    for loops that repeat one SpMV.  The tensors must stay alive and in place."""
    import torch
    f32 = not isinstance(x, int) and x is not None and x.dtype is torch.float32
    fn = load().csr5s_spmv_ex if f32 else load().csr5_spmv_ex
    where = "csr5s_spmv_ex" if f32 else "csr5_spmv_ex"
    args = (h,) + _xy(h, x, y, "f32" if f32 else "f64") + (_stream(stream),)

    def call():
        rc = fn(*args)
        if rc != CSR5_OK:
            raise Csr5Error(rc, where)
    return call


def csr5_spmv_static(h, x, y, stream=None, check=True):
    """csr5_spmv_ex without any allocation: the cross-tile array is the library's static one."""
    return _chk(load().csr5_spmv_static(h, *_xy(h, x, y, "f64"), _stream(stream)), "csr5_spmv_static", check)


def csr5_spmv_profile(h, x, y, reps, stream=None):
    """Mean kernel durations in ms: (tile kernel, carry fix-up)."""
    ms = (C.c_float * 2)()
    _chk(load().csr5_spmv_profile(h, *_xy(h, x, y, "f64"), _stream(stream), int(reps), ms),
         "csr5_spmv_profile", True)
    return float(ms[0]), float(ms[1])


def csr5_stream_floor(h, y, reps, stream=None):
    """Mean durations in ms of a bare read of the handle's tile streams: (reads only,
    reads plus the rows of y).  y (a handle-typed scratch vector) is overwritten."""
    ms = (C.c_float * 2)()
    _chk(load().csr5_stream_floor(h, _arr(y, ["f64", "f32"], 0, "y"), y.numel() * y.element_size(), _stream(stream),
                                  int(reps), ms), "csr5_stream_floor", True)
    return float(ms[0]), float(ms[1])


def csr5_to_csr(h, stream=None, check=True):
    return _chk(load().csr5_to_csr(h, _stream(stream)), "csr5_to_csr", check)


def csr5_free(h, check=True):
    _shapes.pop(h, None)
    return _chk(load().csr5_free(h), "csr5_free", check)


def csr5_status(h):
    st = C.c_uint32()
    _chk(load().csr5_status(h, C.byref(st)), "csr5_status", True)
    return st.value


def csr5_get_info(h):
    """dict(omega, sigma, p, p_complete, desc_words_per_lane, empty_offset_len)."""
    v = [C.c_int32() for _ in range(6)]
    _chk(load().csr5_get_info(h, *[C.byref(a) for a in v]), "csr5_get_info", True)
    keys = ["omega", "sigma", "p", "p_complete", "desc_words_per_lane", "empty_offset_len"]
    return {k: a.value for k, a in zip(keys, v)}


def csr5_get_arrays(h, check=True):
    """Device addresses: dict(tile_ptr, tile_desc, empty_offset_ptr, empty_offset)."""
    v = [C.c_void_p() for _ in range(4)]
    rc = _chk(load().csr5_get_arrays(h, *[C.byref(a) for a in v]), "csr5_get_arrays", check)
    if rc != CSR5_OK:
        return rc
    return dict(zip(["tile_ptr", "tile_desc", "empty_offset_ptr", "empty_offset"], [a.value for a in v]))


def csr5_baseline_csr_scalar(m, row_ptr, col_idx, val, x, y, stream=None, check=True):
    nnz = 0
    return _chk(load().csr5_baseline_csr_scalar(m, _arr(row_ptr, ["i32"], m + 1, "row_ptr"), _arr(col_idx, ["i32"], nnz, "col_idx"),
                                                _arr(val, ["f64"], nnz, "val"), _arr(x, ["f64"], 0, "x"), _arr(y, ["f64"], m, "y"),
                                                _stream(stream)), "csr5_baseline_csr_scalar", check)


def csr5_baseline_csr_vector(m, nnz, row_ptr, col_idx, val, x, y, lanes_per_row=0, stream=None, check=True):
    return _chk(load().csr5_baseline_csr_vector(m, nnz, *_csr_args(m, 0, nnz, row_ptr, col_idx, val, "i32", "f64"),
                                                _arr(x, ["f64"], 0, "x"), _arr(y, ["f64"], m, "y"),
                                                int(lanes_per_row), _stream(stream)),
                "csr5_baseline_csr_vector", check)


def csr5_read_array(h, which, wide=False):
    """Host copy (NumPy) of one of the handle's arrays; wide=True for a handle
    made by csr5l_convert_ex (8-byte tile_ptr and empty_offset_ptr entries)."""
    info = csr5_get_info(h)
    count, dtype = {
        CSR5_ARRAY_TILE_PTR: (info["p"] + 1, np.uint64 if wide else np.uint32),
        CSR5_ARRAY_TILE_DESC: (info["p_complete"] * info["desc_words_per_lane"] * CSR5_OMEGA, np.uint32),
        CSR5_ARRAY_EMPTY_OFFSET_PTR: (info["p_complete"] + 1, np.int64 if wide else np.int32),
        CSR5_ARRAY_EMPTY_OFFSET: (info["empty_offset_len"], np.int32),
    }[which]
    out = np.empty(count, dtype=dtype)
    _chk(load().csr5_read_array(h, which, out.ctypes.data_as(C.c_void_p), out.nbytes),
         "csr5_read_array", True)
    return out
