"""Seeded generators for the five benchmark configurations and small test inputs.

All randomness comes from ``numpy.random.default_rng(seed)`` (PCG64).  The five
named configurations use ``seed = 8860 + config number``; ``scale`` shrinks a
configuration to a size a CPU test can finish in seconds while keeping its
structure (stencil shape, template reuse, R-MAT skew, lognormal row lengths).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class CsrMatrix:
    """A CSR matrix plus the dense vector it is multiplied with."""

    name: str
    n_rows: int
    n_cols: int
    ptr: np.ndarray  # int32, n_rows + 1
    col: np.ndarray  # int32, nnz, strictly ascending inside each row
    val: np.ndarray  # float32 (float64 after widen_to_f64), nnz
    x: np.ndarray  # same type as val, n_cols

    @property
    def nnz(self) -> int:
        return int(self.ptr[-1])

    def check(self) -> None:
        """Structural self-check of the generator output (not of the method)."""
        assert self.ptr.dtype == np.int32 and self.col.dtype == np.int32
        assert self.val.dtype == self.x.dtype and self.val.dtype in (np.float32, np.float64)
        assert self.ptr.shape == (self.n_rows + 1,) and self.ptr[0] == 0
        assert self.col.shape == (self.nnz,) and self.val.shape == (self.nnz,)
        assert self.x.shape == (self.n_cols,)
        assert np.all(np.diff(self.ptr) >= 0)
        if self.nnz:
            assert self.col.min() >= 0 and self.col.max() < self.n_cols
            inc = np.diff(self.col.astype(np.int64)) > 0
            # a non-increase is only allowed where a new row starts
            starts = np.zeros(self.nnz, dtype=bool)
            p = self.ptr[:-1][np.diff(self.ptr) > 0]
            starts[p] = True
            assert np.all(inc | starts[1:])


def _from_sorted_keys(name, n_rows, n_cols, keys, shift, rng, val_kind, x_rng=None):
    """Build a CSR matrix from sorted unique int64 keys ``row << shift | col``."""
    rows = (keys >> shift).astype(np.int64)
    col = (keys & ((1 << shift) - 1)).astype(np.int32)
    counts = np.bincount(rows, minlength=n_rows)
    ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=ptr[1:])
    assert ptr[-1] < 2**31
    nnz = int(ptr[-1])
    if val_kind == "normal":
        val = rng.standard_normal(nnz, dtype=np.float32)
    elif val_kind == "unit_open_closed":  # uniform on (0, 1]
        val = (1.0 - rng.random(nnz, dtype=np.float32)).astype(np.float32)
    else:
        raise ValueError(val_kind)
    x = rng.uniform(-1.0, 1.0, n_cols).astype(np.float32)
    return CsrMatrix(name, n_rows, n_cols, ptr.astype(np.int32), col, val, x)


def laplacian_2d(side: int = 64, seed: int = 8861) -> CsrMatrix:
    """5-point Laplacian on a side x side grid: 4 on the diagonal, -1 off it,
    plus uniform[-0.01, 0.01] noise on every stored entry."""
    rng = np.random.default_rng(seed)
    n = side * side
    r = np.arange(n, dtype=np.int64)
    gy, gx = r // side, r % side
    offs = [(-1, 0), (0, -1), (0, 0), (0, 1), (1, 0)]  # ascending column order
    cols = np.empty((n, 5), dtype=np.int64)
    mask = np.empty((n, 5), dtype=bool)
    base = np.empty((n, 5), dtype=np.float32)
    for k, (dy, dx) in enumerate(offs):
        yy, xx = gy + dy, gx + dx
        mask[:, k] = (yy >= 0) & (yy < side) & (xx >= 0) & (xx < side)
        cols[:, k] = yy * side + xx
        base[:, k] = 4.0 if (dy == 0 and dx == 0) else -1.0
    ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(mask.sum(axis=1), out=ptr[1:])
    col = cols[mask].astype(np.int32)
    val = base[mask] + rng.uniform(-0.01, 0.01, int(ptr[-1])).astype(np.float32)
    x = rng.uniform(-1.0, 1.0, n).astype(np.float32)
    return CsrMatrix(f"laplace2d_{side}", n, n, ptr.astype(np.int32), col, val.astype(np.float32), x)


def stencil_27pt(side: int = 128, seed: int = 8862) -> CsrMatrix:
    """27-point stencil on a side^3 grid; values uniform[-1, 1], diagonal 27."""
    rng = np.random.default_rng(seed)
    n = side**3
    r = np.arange(n, dtype=np.int32)
    gz, gy, gx = r // (side * side), (r // side) % side, r % side
    cols = np.empty((n, 27), dtype=np.int32)
    mask = np.empty((n, 27), dtype=bool)
    k = 0
    for dz in (-1, 0, 1):
        mz = (gz + dz >= 0) & (gz + dz < side)
        for dy in (-1, 0, 1):
            my = mz & (gy + dy >= 0) & (gy + dy < side)
            for dx in (-1, 0, 1):
                mask[:, k] = my & (gx + dx >= 0) & (gx + dx < side)
                cols[:, k] = r + (dz * side * side + dy * side + dx)
                k += 1
    ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(mask.sum(axis=1), out=ptr[1:])
    col = cols[mask]
    nnz = int(ptr[-1])
    val = rng.uniform(-1.0, 1.0, nnz).astype(np.float32)
    diag = np.empty((n, 27), dtype=bool)
    diag[:] = False
    diag[:, 13] = True
    val[diag[mask]] = 27.0
    del cols, mask, diag
    x = rng.uniform(-1.0, 1.0, n).astype(np.float32)
    return CsrMatrix(f"stencil27_{side}", n, n, ptr.astype(np.int32), col, val, x)


def row_template(log2_n: int = 20, n_templates: int = 1024, row_len: int = 32,
                 p_resample: float = 0.1, seed: int = 8863) -> CsrMatrix:
    """Rows copy one of ``n_templates`` sorted column patterns, with each column
    resampled with probability ``p_resample``; template ids are a shuffled
    balanced assignment; duplicates merged; values N(0, 1)."""
    rng = np.random.default_rng(seed)
    n = 1 << log2_n
    tmpl = rng.integers(0, n, size=(n_templates, row_len), dtype=np.int64)
    tid = rng.permutation(np.arange(n, dtype=np.int64) % n_templates)
    cols = tmpl[tid]  # n x row_len
    resample = rng.random((n, row_len), dtype=np.float32) < p_resample
    fresh = rng.integers(0, n, size=(n, row_len), dtype=np.int64)
    cols = np.where(resample, fresh, cols)
    del resample, fresh
    keys = (np.arange(n, dtype=np.int64)[:, None] << log2_n) | cols
    del cols
    keys = np.unique(keys.ravel())
    return _from_sorted_keys(f"rowtemplate_2^{log2_n}", n, n, keys, log2_n, rng, "normal")


def rmat(log2_n: int = 22, avg_degree: int = 16, probs=(0.57, 0.19, 0.19, 0.05),
         seed: int = 8864) -> CsrMatrix:
    """R-MAT adjacency: avg_degree * n edge draws, duplicates merged, values in (0, 1]."""
    rng = np.random.default_rng(seed)
    n = 1 << log2_n
    m = avg_degree * n
    a, b, c, _ = probs
    keys = np.zeros(m, dtype=np.int64)
    for level in range(log2_n):
        u = rng.random(m, dtype=np.float32)
        row_bit = u >= np.float32(a + b)                       # quadrants c, d
        col_bit = ((u >= np.float32(a)) & ~row_bit) | (u >= np.float32(a + b + c))  # quadrants b, d
        bitpos = log2_n - 1 - level
        keys |= row_bit.astype(np.int64) << (log2_n + bitpos)
        keys |= col_bit.astype(np.int64) << bitpos
    keys = np.unique(keys)
    return _from_sorted_keys(f"rmat_2^{log2_n}", n, n, keys, log2_n, rng, "unit_open_closed")


def lognormal_rect(n_rows: int = 4_000_000, n_cols: int = 1_000_000, mu: float = 2.5,
                   sigma: float = 1.2, cap: int = 10_000, seed: int = 8865) -> CsrMatrix:
    """Row lengths min(floor(lognormal(mu, sigma)), cap); columns uniform (drawn
    with replacement, duplicates merged); values N(0, 1)."""
    rng = np.random.default_rng(seed)
    lens = np.minimum(np.floor(rng.lognormal(mu, sigma, n_rows)), min(cap, n_cols)).astype(np.int64)
    total = int(lens.sum())
    shift = max(1, int(n_cols - 1).bit_length())
    rows = np.repeat(np.arange(n_rows, dtype=np.int64), lens)
    keys = (rows << shift) | rng.integers(0, n_cols, size=total, dtype=np.int64)
    del rows
    keys = np.unique(keys)
    return _from_sorted_keys(f"lognormal_{n_rows}x{n_cols}", n_rows, n_cols, keys, shift, rng, "normal")


def random_csr(n_rows: int, n_cols: int, density: float, seed: int,
               empty_row_frac: float = 0.0, integer_values: bool = False) -> CsrMatrix:
    """Small uniformly random matrix for brute-force tests.  With
    ``integer_values`` every product and sum is exact in float32."""
    rng = np.random.default_rng(seed)
    dense = rng.random((n_rows, n_cols)) < density
    if empty_row_frac > 0:
        dense[rng.random(n_rows) < empty_row_frac, :] = False
    rr, cc = np.nonzero(dense)
    ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(rr, minlength=n_rows), out=ptr[1:])
    nnz = int(ptr[-1])
    if integer_values:
        val = rng.integers(-8, 9, nnz).astype(np.float32)
        val[val == 0] = 1.0
        x = rng.integers(-4, 5, n_cols).astype(np.float32)
    else:
        val = rng.standard_normal(nnz, dtype=np.float32)
        x = rng.uniform(-1.0, 1.0, n_cols).astype(np.float32)
    return CsrMatrix(f"random_{n_rows}x{n_cols}", n_rows, n_cols, ptr.astype(np.int32),
                     cc.astype(np.int32), val, x)


def worked_example_8x8() -> CsrMatrix:
    """The hand-worked 8x8 example: a_ij = 10(i+1) + (j+1) on a fixed pattern,
    x = (1, ..., 8).  One empty row and one empty 4x4 block."""
    pattern = [[0, 2, 5], [], [0, 1, 2, 3, 6], [1], [4, 5, 6, 7], [7], [4, 6], [5]]
    ptr = [0]
    col, val = [], []
    for i, cs in enumerate(pattern):
        for j in cs:
            col.append(j)
            val.append(10.0 * (i + 1) + (j + 1))
        ptr.append(len(col))
    return CsrMatrix("worked8x8", 8, 8, np.array(ptr, dtype=np.int32), np.array(col, dtype=np.int32),
                     np.array(val, dtype=np.float32), np.arange(1, 9, dtype=np.float32))


def widen_to_f64(m: CsrMatrix, seed: int = 64) -> CsrMatrix:
    """The same matrix and vector stored in float64, with seeded random bits below float32's
    last place (each value is scaled by 1 + u * 2**-24, u uniform in [0, 1)), so that a
    path which rounds its values to float32 anywhere is told apart from one that does not."""
    rng = np.random.default_rng(seed)
    val = m.val.astype(np.float64) * (1.0 + rng.random(m.val.shape[0]) * 2.0**-24)
    x = m.x.astype(np.float64) * (1.0 + rng.random(m.x.shape[0]) * 2.0**-24)
    return CsrMatrix(m.name + "_f64", m.n_rows, m.n_cols, m.ptr, m.col, val, x)


CONFIG_NAMES = {
    1: "laplace2d_64",
    2: "stencil27_128",
    3: "rowtemplate_2^20",
    4: "rmat_2^22",
    5: "lognormal_4Mx1M",
}


def make_config(number: int, scale: float = 1.0) -> CsrMatrix:
    """Configuration ``number`` (1..5).  ``scale`` < 1 shrinks the problem:
    grid sides scale with its cube/square root, power-of-two sizes drop whole bits."""
    seed = 8860 + number
    if number == 1:
        return laplacian_2d(max(4, int(round(64 * scale**0.5))), seed)
    if number == 2:
        return stencil_27pt(max(3, int(round(128 * scale ** (1.0 / 3.0)))), seed)
    drop = 0 if scale >= 1.0 else int(round(np.log2(1.0 / scale)))
    if number == 3:
        return row_template(max(8, 20 - drop), n_templates=max(8, 1024 >> (drop // 2)), seed=seed)
    if number == 4:
        return rmat(max(8, 22 - drop), seed=seed)
    if number == 5:
        return lognormal_rect(max(64, int(4_000_000 * scale)), max(64, int(1_000_000 * scale)), seed=seed)
    raise ValueError(f"no configuration {number}")
