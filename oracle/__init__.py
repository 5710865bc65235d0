"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this package.  It imports nothing from the HIP binding, and the HIP binding
imports nothing from here.

``hbp_oracle.c`` holds what the paper defines (Algorithm 1, the hash, the compact-layout builder,
Algorithm 3's walk and the combine); ``hbp_oracle_schedule.c`` holds the schedule of Section 3.3
(the paper's own sentence as one mode, this build's weighted ranges as the other) and the work
units of the combine part; ``hbp_literal.py`` holds the paper's literal layout for tiny inputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("hbp_oracle.c", "hbp_oracle_schedule.c")]
_DEPS = _SRCS + [os.path.join(_HERE, "hbp_oracle.h")]
_LIB = os.path.join(_HERE, "libhbp_oracle.so")

ARRAYS = {  # name -> (id in oracle_hbp_copy, dtype)
    "blk_bm": (0, np.int32), "blk_bn": (1, np.int32), "slot_ptr": (2, np.int32),
    "blk_group_ptr": (3, np.int32), "col_blk_ptr": (4, np.int32), "stripe_ptr": (5, np.int32),
    "stripe_blk": (6, np.int32), "group_ptr": (7, np.int32), "group_slot": (8, np.int32),
    "row_local": (9, np.uint16), "seg_len": (10, np.uint16), "col_local": (11, np.uint16),
    "data": (12, np.float32), "add_sign": (13, np.int32), "col_group_ptr": (14, np.int32),
    "comp_lo": (15, np.int32), "fixed_start": (16, np.int32), "fixed_col": (17, np.int32),
    "unit_ptr": (18, np.int32), "unit_stripe": (19, np.int32), "unit_k": (20, np.int32), "multi_stripes": (21, np.int32),
    "group_rounds": (22, np.int32), "comp_col": (23, np.int32), "slot_key": (24, np.uint32), "blk_shift": (25, np.int32),
}
DIMS = ("n_rows", "n_cols", "nnz", "R", "C", "W", "a", "NBR", "NBC", "B", "S", "G", "P", "fixed_q8", "U", "NM",
        "first_ticket_block")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, single-threaded)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _DEPS):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", *_SRCS, "-o", _LIB])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        lib.oracle_csr_spmv_f64.argtypes = [vp, vp, vp, vp, i64, vp, vp]
        lib.oracle_csr_spmv_f64.restype = None
        lib.oracle_csr_spmv_f64_d.argtypes = [vp, vp, vp, vp, i64, vp, vp]
        lib.oracle_csr_spmv_f64_d.restype = None
        lib.oracle_hash_key.argtypes = [ctypes.c_uint32, i32, i32]
        lib.oracle_hash_key.restype = ctypes.c_uint32
        lib.oracle_hash_keys.argtypes = [vp, i64, i32, i32, vp]
        lib.oracle_hash_keys.restype = None
        lib.oracle_sample_shift.argtypes = [vp, vp, i64, i32]
        lib.oracle_sample_shift.restype = i32
        lib.oracle_hbp_build.argtypes = [vp, vp, vp, i32, i64, i64, i32, i32, i32, i32]
        lib.oracle_hbp_build.restype = vp
        lib.oracle_hbp_schedule.argtypes = [vp, i64, i32, i32, i32, i32, i32, i32]
        lib.oracle_hbp_schedule.restype = i32
        lib.oracle_hbp_units.argtypes = [vp, i32]
        lib.oracle_hbp_units.restype = i32
        lib.oracle_hbp_free.argtypes = [vp]
        lib.oracle_hbp_free.restype = None
        lib.oracle_hbp_dims.argtypes = [vp, vp]
        lib.oracle_hbp_dims.restype = None
        lib.oracle_hbp_copy.argtypes = [vp, i32, vp]
        lib.oracle_hbp_copy.restype = i64
        lib.oracle_hbp_spmv.argtypes = [vp, vp, vp, vp, vp]
        lib.oracle_hbp_spmv.restype = None
        lib.oracle_hbp_to_coo.argtypes = [vp, vp, vp, vp]
        lib.oracle_hbp_to_coo.restype = None
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def csr_spmv_f64(ptr, col, val, x):
    """(y_ref, s_abs): fp64 CSR SpMV by the plain definition and the per-row sum of
    absolute products."""
    n_rows = len(ptr) - 1
    y = np.empty(n_rows, dtype=np.float64)
    s = np.empty(n_rows, dtype=np.float64)
    assert val.dtype == x.dtype and val.dtype in (np.float32, np.float64)
    fn = _load().oracle_csr_spmv_f64 if val.dtype == np.float32 else _load().oracle_csr_spmv_f64_d
    fn(_p(ptr), _p(col), _p(val), _p(x), n_rows, _p(y), _p(s))
    return y, s


def hash_key(n: int, a: int, R: int) -> int:
    return int(_load().oracle_hash_key(int(n), int(a), int(R)))


def hash_keys(n: np.ndarray, a: int, R: int) -> np.ndarray:
    """hash_key of every length in ``n`` (uint32)."""
    n = np.ascontiguousarray(n, dtype=np.uint32)
    out = np.empty_like(n)
    _load().oracle_hash_keys(_p(n), len(n), int(a), int(R), _p(out))
    return out


def sample_shift(ptr, col, n_rows: int, C: int) -> int:
    return int(_load().oracle_sample_shift(_p(ptr), _p(col), int(n_rows), int(C)))


class OracleHbp:
    """The compact HBP layout built by the C oracle; arrays are numpy copies."""

    def __init__(self, ptr, col, val, n_rows, n_cols, R=512, C=4096, W=64, hash_shift=-1,
                 num_workers=1, fixed_q8=128, slot_weight=1, unit_slots=16384, round_weight=0, group_weight=0, column_weight=0,
                 paper_schedule=False):
        """hash_shift: 0..12 given, -1 sampled, -2 no reorder, -3 length as key, -4 one shift per block.
        paper_schedule: Section 3.3 read literally (equal block counts, one ticket counter)."""
        lib = _load()
        assert val.dtype in (np.float32, np.float64)
        self.value_dtype = val.dtype
        self._h = lib.oracle_hbp_build(_p(ptr), _p(col), _p(val), int(val.dtype.itemsize), int(n_rows), int(n_cols), int(R), int(C), int(W),
                                       int(hash_shift))
        if not self._h:
            raise ValueError("oracle_hbp_build rejected the parameters")
        if lib.oracle_hbp_schedule(self._h, int(num_workers), int(fixed_q8), int(slot_weight), int(round_weight), int(group_weight),
                                   int(column_weight), 1 if paper_schedule else 0) != 0 or lib.oracle_hbp_units(self._h, int(unit_slots)) != 0:
            lib.oracle_hbp_free(self._h)
            self._h = None
            raise ValueError("oracle schedule parameters rejected")
        dims = np.zeros(len(DIMS), dtype=np.int64)
        lib.oracle_hbp_dims(self._h, _p(dims))
        for k, v in zip(DIMS, dims):
            setattr(self, k, int(v))
        self._cache = {}

    def array(self, name: str) -> np.ndarray:
        if name not in self._cache:
            which, dt = ARRAYS[name]
            if name == "data":
                dt = self.value_dtype
            lib = _load()
            nbytes = lib.oracle_hbp_copy(self._h, which, None)
            out = np.empty(nbytes // np.dtype(dt).itemsize, dtype=dt)
            if nbytes:
                lib.oracle_hbp_copy(self._h, which, _p(out))
            self._cache[name] = out
        return self._cache[name]

    def spmv(self, x, with_abs=False):
        """(y, partial) through the layout (Algorithm 3 walk + combine), fp64; with_abs adds the per-slot
        sums of absolute products."""
        partial = np.zeros(max(self.S, 1), dtype=np.float64)
        mag = np.zeros(max(self.S, 1), dtype=np.float64)
        y = np.zeros(self.n_rows, dtype=np.float64)
        assert x.dtype == self.value_dtype
        _load().oracle_hbp_spmv(self._h, _p(x), _p(partial), _p(y), _p(mag) if with_abs else None)
        if with_abs:
            return y, partial[: self.S], mag[: self.S]
        return y, partial[: self.S]

    def to_coo(self):
        rows = np.full(max(self.nnz, 1), -1, dtype=np.int64)
        cols = np.full(max(self.nnz, 1), -1, dtype=np.int64)
        vals = np.zeros(max(self.nnz, 1), dtype=self.value_dtype)
        _load().oracle_hbp_to_coo(self._h, _p(rows), _p(cols), _p(vals))
        return rows[: self.nnz], cols[: self.nnz], vals[: self.nnz]

    def close(self):
        if self._h:
            _load().oracle_hbp_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
