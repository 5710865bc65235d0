"""Python binding of libhbp (MI355X / gfx950 Hash-based Partition SpMV).

Argument marshalling only: every step of the path runs in the HIP kernels behind the C ABI
declared in ``include/hbp.h``.  PyTorch supplies device memory and the stream.  There is no
CPU fallback: if the built library is missing, loading it raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhbp.so")

HBP_OK = 0
HBP_FLAG_VALIDATE = 1
HBP_FLAG_NO_REORDER = 2
HBP_FLAG_KEY_LENGTH = 4
HBP_FLAG_PAPER_SCHEDULE = 8
HBP_FLAG_BLOCK_SHIFT = 16
HBP_FLAG_KEEP_KEYS = 32

ARRAY_IDS = {
    "blk_bm": 0, "blk_bn": 1, "slot_ptr": 2, "blk_group_ptr": 3, "col_blk_ptr": 4, "stripe_ptr": 5,
    "stripe_blk": 6, "group_ptr": 7, "group_slot": 8, "row_local": 9, "seg_len": 10, "col_local": 11,
    "data": 12, "add_sign": 13, "partial": 14, "col_group_ptr": 15, "comp_lo": 16,
    "fixed_start": 17, "fixed_col": 18, "unit_ptr": 19, "unit_stripe": 20, "unit_k": 21, "multi_stripes": 22,
    "group_rounds": 23, "comp_col": 24, "slot_key": 25, "blk_shift": 26,
}
ARRAY_DTYPES = {
    "blk_bm": "int32", "blk_bn": "int32", "slot_ptr": "int32", "blk_group_ptr": "int32", "col_blk_ptr": "int32",
    "stripe_ptr": "int32", "stripe_blk": "int32", "group_ptr": "int32", "group_slot": "int32",
    "row_local": "uint16", "seg_len": "uint16", "col_local": "uint16", "data": "float32", "add_sign": "int32",
    "partial": "float32", "col_group_ptr": "int32", "comp_lo": "int32",
    "fixed_start": "int32", "fixed_col": "int32",
    "unit_ptr": "int32", "unit_stripe": "int32", "unit_k": "int32", "multi_stripes": "int32",
    "group_rounds": "int32", "comp_col": "int32", "slot_key": "uint32", "blk_shift": "int32",
}
# every symbol include/hbp.h declares
EXPORTED_SYMBOLS = (
    "hbp_default_params", "hbp_build", "hbp_spmv", "hbp_free", "hbp_get_info", "hbp_export", "hbp_spmv_timed",
    "hbp_csr_spmv", "hbp_status_string", "hbp_last_hip_error",
    "hbp_build_f64", "hbp_spmv_f64", "hbp_spmv_timed_f64", "hbp_csr_spmv_f64", "hbp_release_workspace", "hbp_hash_keys",
    "hbp_spmv_static_scratch",
)


class hbp_params_t(ctypes.Structure):
    _fields_ = [("rows_per_block", ctypes.c_int32), ("cols_per_block", ctypes.c_int32), ("group_width", ctypes.c_int32),
                ("num_workers", ctypes.c_int32), ("fixed_fraction_q8", ctypes.c_int32), ("hash_shift", ctypes.c_int32),
                ("claim_chunk", ctypes.c_int32), ("threads_per_worker", ctypes.c_int32),
                ("rounds_per_batch", ctypes.c_int32), ("slot_weight", ctypes.c_int32), ("group_weight", ctypes.c_int32),
                ("combine_unit_slots", ctypes.c_int32), ("round_weight", ctypes.c_int32), ("heavy_group_rounds", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("column_weight", ctypes.c_int32)]


class hbp_info_t(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("rows_per_block", ctypes.c_int32), ("cols_per_block", ctypes.c_int32), ("group_width", ctypes.c_int32),
                ("hash_shift", ctypes.c_int32), ("hash_b", ctypes.c_int32),
                ("row_blocks", ctypes.c_int64), ("col_blocks", ctypes.c_int64),
                ("blocks", ctypes.c_int64), ("slots", ctypes.c_int64), ("groups", ctypes.c_int64),
                ("num_workers", ctypes.c_int32), ("fixed_fraction_q8", ctypes.c_int32), ("claim_chunk", ctypes.c_int32),
                ("threads_per_worker", ctypes.c_int32), ("rounds_per_batch", ctypes.c_int32),
                ("slot_weight", ctypes.c_int32), ("group_weight", ctypes.c_int32), ("combine_unit_slots", ctypes.c_int32),
                ("heavy_group_rounds", ctypes.c_int32), ("round_weight", ctypes.c_int32), ("column_weight", ctypes.c_int32),
                ("combine_units", ctypes.c_int64), ("split_row_blocks", ctypes.c_int64), ("value_bytes", ctypes.c_int32),
                ("first_ticket_block", ctypes.c_int64), ("bytes_layout", ctypes.c_int64), ("bytes_spmv_part", ctypes.c_int64), ("bytes_combine", ctypes.c_int64),
                ("build_ms", ctypes.c_double)]


class HbpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {hbp_status_string(status)} (status {status}, hip error {lib().hbp_last_hip_error()})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_08860_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU fallback")
        # PyTorch ships its own HIP runtime (same soname as the system one).  It has to be in
        # the process before libhbp.so is loaded, so that both share one runtime and device
        # pointers from torch tensors are valid in the library's calls.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.hbp_default_params.argtypes = [ctypes.POINTER(hbp_params_t)]
        L.hbp_build.argtypes = [vp, vp, vp, i64, i64, ctypes.POINTER(hbp_params_t), vp, ctypes.POINTER(vp)]
        L.hbp_spmv.argtypes = [vp, vp, vp, vp]
        L.hbp_free.argtypes = [vp]
        L.hbp_get_info.argtypes = [vp, ctypes.POINTER(hbp_info_t)]
        L.hbp_export.argtypes = [vp, ctypes.c_int, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.hbp_spmv_timed.argtypes = [vp, vp, vp, vp, ctypes.c_int] + [ctypes.POINTER(ctypes.c_float)] * 3
        L.hbp_csr_spmv.argtypes = [ctypes.c_int, vp, vp, vp, vp, vp, i64, vp]
        L.hbp_build_f64.argtypes = L.hbp_build.argtypes
        L.hbp_spmv_f64.argtypes = L.hbp_spmv.argtypes
        L.hbp_spmv_static_scratch.argtypes = L.hbp_spmv.argtypes
        L.hbp_spmv_timed_f64.argtypes = L.hbp_spmv_timed.argtypes
        L.hbp_csr_spmv_f64.argtypes = L.hbp_csr_spmv.argtypes
        L.hbp_status_string.argtypes = [ctypes.c_int]
        L.hbp_status_string.restype = ctypes.c_char_p
        L.hbp_last_hip_error.argtypes = []
        L.hbp_release_workspace.argtypes = []
        L.hbp_hash_keys.argtypes = [vp, i64, i32, i32, vp, vp]
        for name in EXPORTED_SYMBOLS:
            if name not in ("hbp_status_string",):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != HBP_OK:
        raise HbpError(status, where)


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return int(getattr(stream, "cuda_stream", stream))


def _dev_i32(t, what):
    import torch
    assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous(), f"{what}: contiguous int32 CUDA tensor required"
    return t.data_ptr()


def _dev_f32(t, what):
    import torch
    assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous(), f"{what}: contiguous float32 CUDA tensor required"
    return t.data_ptr()


def _dev_f64(t, what):
    import torch
    assert t.is_cuda and t.dtype == torch.float64 and t.is_contiguous(), f"{what}: contiguous float64 CUDA tensor required"
    return t.data_ptr()


def hbp_status_string(status: int) -> str:
    return lib().hbp_status_string(int(status)).decode()


def hbp_default_params() -> hbp_params_t:
    p = hbp_params_t()
    _check(lib().hbp_default_params(ctypes.byref(p)), "hbp_default_params")
    return p


def _build(f64: bool, csr_ptr, csr_col, csr_val, n_rows, n_cols, params, stream, overrides) -> int:
    p = params if params is not None else hbp_default_params()
    for k, v in overrides.items():
        if k == "validate":
            p.flags = (p.flags | HBP_FLAG_VALIDATE) if v else (p.flags & ~HBP_FLAG_VALIDATE)
        elif k == "no_reorder":
            p.flags = (p.flags | HBP_FLAG_NO_REORDER) if v else (p.flags & ~HBP_FLAG_NO_REORDER)
        elif k == "key_length":
            p.flags = (p.flags | HBP_FLAG_KEY_LENGTH) if v else (p.flags & ~HBP_FLAG_KEY_LENGTH)
        elif k == "paper_schedule":
            p.flags = (p.flags | HBP_FLAG_PAPER_SCHEDULE) if v else (p.flags & ~HBP_FLAG_PAPER_SCHEDULE)
        elif k == "block_shift":
            p.flags = (p.flags | HBP_FLAG_BLOCK_SHIFT) if v else (p.flags & ~HBP_FLAG_BLOCK_SHIFT)
        elif k == "keep_keys":
            p.flags = (p.flags | HBP_FLAG_KEEP_KEYS) if v else (p.flags & ~HBP_FLAG_KEEP_KEYS)
        else:
            if not hasattr(p, k):
                raise TypeError(f"hbp_params_t has no field {k}")
            setattr(p, k, v)
    assert csr_ptr.numel() == n_rows + 1
    assert csr_col.numel() == csr_val.numel()
    out = ctypes.c_void_p()
    fn, val = (lib().hbp_build_f64, _dev_f64(csr_val, "csr_val")) if f64 else (lib().hbp_build, _dev_f32(csr_val, "csr_val"))
    _check(fn(_dev_i32(csr_ptr, "csr_ptr"), _dev_i32(csr_col, "csr_col"), val,
              int(n_rows), int(n_cols), ctypes.byref(p), _stream_ptr(stream), ctypes.byref(out)), "hbp_build_f64" if f64 else "hbp_build")
    return out.value


def hbp_build(csr_ptr, csr_col, csr_val, n_rows: int, n_cols: int, params: hbp_params_t | None = None, stream=None,
              **overrides) -> int:
    """CSR (device tensors, float32 values) -> handle.  ``overrides`` set fields of hbp_params_t by name
    (``validate=``, ``no_reorder=``, ``key_length=``, ``paper_schedule=``, ``block_shift=`` and ``keep_keys=True/False``
    set the flags)."""
    return _build(False, csr_ptr, csr_col, csr_val, n_rows, n_cols, params, stream, overrides)


def hbp_build_f64(csr_ptr, csr_col, csr_val, n_rows: int, n_cols: int, params: hbp_params_t | None = None, stream=None,
                  **overrides) -> int:
    """hbp_build for float64 values; the handle goes with the ``_f64`` calls."""
    return _build(True, csr_ptr, csr_col, csr_val, n_rows, n_cols, params, stream, overrides)


def hbp_spmv(handle: int, x, y, stream=None) -> None:
    info = hbp_get_info(handle)
    assert x.numel() == info.n_cols and y.numel() == info.n_rows
    _check(lib().hbp_spmv(handle, _dev_f32(x, "x"), _dev_f32(y, "y"), _stream_ptr(stream)), "hbp_spmv")


def hbp_spmv_static_scratch(handle: int, x, y, stream=None) -> None:
    """hbp_spmv with the call's intermediates in the library's fixed scratch array (no allocation anywhere)."""
    info = hbp_get_info(handle)
    assert x.numel() == info.n_cols and y.numel() == info.n_rows
    _check(lib().hbp_spmv_static_scratch(handle, _dev_f32(x, "x"), _dev_f32(y, "y"), _stream_ptr(stream)), "hbp_spmv_static_scratch")


def hbp_spmv_f64(handle: int, x, y, stream=None) -> None:
    info = hbp_get_info(handle)
    assert x.numel() == info.n_cols and y.numel() == info.n_rows
    _check(lib().hbp_spmv_f64(handle, _dev_f64(x, "x"), _dev_f64(y, "y"), _stream_ptr(stream)), "hbp_spmv_f64")


def hbp_spmv_timed(handle: int, x, y, iters: int, stream=None):
    """(ms SpMV-part kernel, ms combine kernel, ms whole call), averaged over ``iters`` calls."""
    a, b, c = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _check(lib().hbp_spmv_timed(handle, _dev_f32(x, "x"), _dev_f32(y, "y"), _stream_ptr(stream), int(iters),
                                ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "hbp_spmv_timed")
    return a.value, b.value, c.value


def hbp_spmv_timed_f64(handle: int, x, y, iters: int, stream=None):
    a, b, c = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    _check(lib().hbp_spmv_timed_f64(handle, _dev_f64(x, "x"), _dev_f64(y, "y"), _stream_ptr(stream), int(iters),
                                    ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "hbp_spmv_timed_f64")
    return a.value, b.value, c.value


def hbp_free(handle: int) -> None:
    _check(lib().hbp_free(handle), "hbp_free")


def hbp_get_info(handle: int) -> hbp_info_t:
    info = hbp_info_t()
    _check(lib().hbp_get_info(handle, ctypes.byref(info)), "hbp_get_info")
    return info


def hbp_export(handle: int, name: str):
    """One layout array as a numpy array (host copy)."""
    import numpy as np
    which = ARRAY_IDS[name]
    nbytes = ctypes.c_size_t()
    _check(lib().hbp_export(handle, which, None, 0, ctypes.byref(nbytes)), "hbp_export")
    dt = np.dtype(ARRAY_DTYPES[name])
    if name in ("data", "partial") and hbp_get_info(handle).value_bytes == 8:
        dt = np.dtype("float64")
    out = np.empty(nbytes.value // dt.itemsize, dtype=dt)
    if nbytes.value:
        _check(lib().hbp_export(handle, which, out.ctypes.data, out.nbytes, ctypes.byref(nbytes)), "hbp_export")
    return out


def hbp_csr_spmv(kind: int, csr_ptr, csr_col, csr_val, x, y, stream=None) -> None:
    """In-repo CSR baseline: kind 0 = thread per row, 1 = wavefront per row, 2/4/8/16/32 = that many lanes per row."""
    _check(lib().hbp_csr_spmv(int(kind), _dev_i32(csr_ptr, "csr_ptr"), _dev_i32(csr_col, "csr_col"),
                              _dev_f32(csr_val, "csr_val"), _dev_f32(x, "x"), _dev_f32(y, "y"),
                              csr_ptr.numel() - 1, _stream_ptr(stream)), "hbp_csr_spmv")


def hbp_csr_spmv_f64(kind: int, csr_ptr, csr_col, csr_val, x, y, stream=None) -> None:
    _check(lib().hbp_csr_spmv_f64(int(kind), _dev_i32(csr_ptr, "csr_ptr"), _dev_i32(csr_col, "csr_col"),
                                  _dev_f64(csr_val, "csr_val"), _dev_f64(x, "x"), _dev_f64(y, "y"),
                                  csr_ptr.numel() - 1, _stream_ptr(stream)), "hbp_csr_spmv_f64")


def hbp_hash_keys(n, a: int, rows_per_block: int, stream=None):
    """The device's hash key (Section 3.2) of every length in ``n`` (uint32/int32 CUDA tensor) -> int32 CUDA tensor."""
    import torch
    assert n.is_cuda and n.dtype == torch.int32 and n.is_contiguous()
    out = torch.empty_like(n)
    _check(lib().hbp_hash_keys(n.data_ptr(), n.numel(), int(a), int(rows_per_block), out.data_ptr(), _stream_ptr(stream)),
           "hbp_hash_keys")
    return out


def hbp_release_workspace() -> None:
    """Gives back the scratch memory hbp_build keeps between builds."""
    _check(lib().hbp_release_workspace(), "hbp_release_workspace")
