"""Pins for the oracle's y = A x (Algorithm 1) against what mathematics fixes:
the hand-worked example, dense brute force, exact integer cases, linearity."""
import json
import os

import numpy as np
import pytest

from workloads import random_csr, worked_example_8x8, make_config

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_8x8.json")


def dense_of(m):
    a = np.zeros((m.n_rows, m.n_cols), dtype=np.float64)
    for i in range(m.n_rows):
        for j in range(m.ptr[i], m.ptr[i + 1]):
            a[i, m.col[j]] = m.val[j]
    return a


def test_worked_example_y(oracle):
    g = json.load(open(GOLDEN))
    m = worked_example_8x8()
    assert [list(m.col[m.ptr[i]:m.ptr[i + 1]]) for i in range(8)] == g["pattern"]
    y, s = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    assert y.tolist() == g["y"]
    assert s.tolist() == g["y"]  # all products are positive


@pytest.mark.parametrize("seed", range(6))
def test_dense_brute_force_exact_integers(oracle, seed):
    m = random_csr(37 + seed, 29 + 3 * seed, 0.2, seed, empty_row_frac=0.2, integer_values=True)
    y, s = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    a = dense_of(m)
    assert np.array_equal(y, a @ m.x.astype(np.float64))
    assert np.array_equal(s, np.abs(a) @ np.abs(m.x.astype(np.float64)))


@pytest.mark.parametrize("seed", range(4))
def test_dense_brute_force_real(oracle, seed):
    m = random_csr(64, 80, 0.15, 100 + seed, empty_row_frac=0.1)
    y, s = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    a = dense_of(m)
    ref = a @ m.x.astype(np.float64)
    assert np.all(np.abs(y - ref) <= 1e-13 * (s + 1e-300))
    assert np.all(y[np.diff(m.ptr) == 0] == 0.0)


def test_transposed_operand_would_fail(oracle):
    """A x and A^T x differ on a non-symmetric matrix: guards against reading x by row."""
    m = random_csr(16, 16, 0.3, 7, integer_values=True)
    y, _ = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
    a = dense_of(m)
    assert not np.array_equal(y, a.T @ m.x.astype(np.float64))


def test_identity_and_scaling(oracle):
    n = 50
    ptr = np.arange(n + 1, dtype=np.int32)
    col = np.arange(n, dtype=np.int32)
    val = np.full(n, 3.0, dtype=np.float32)
    x = np.linspace(-1, 1, n).astype(np.float32)
    y, s = oracle.csr_spmv_f64(ptr, col, val, x)
    assert np.array_equal(y, 3.0 * x.astype(np.float64))
    assert np.array_equal(s, np.abs(3.0 * x.astype(np.float64)))


def test_laplacian_constant_vector(oracle):
    """A noise-free 5-point Laplacian applied to the constant vector gives 4 minus the
    number of neighbours: 0 inside, 1 on edges, 2 at corners."""
    m = make_config(1)
    side = 64
    base = np.where(m.col == np.repeat(np.arange(m.n_rows), np.diff(m.ptr)), 4.0, -1.0).astype(np.float32)
    y, _ = oracle.csr_spmv_f64(m.ptr, m.col, base, np.ones(m.n_cols, dtype=np.float32))
    y = y.reshape(side, side)
    assert np.all(y[1:-1, 1:-1] == 0)
    assert np.all(y[0, 1:-1] == 1) and np.all(y[1:-1, 0] == 1)
    assert y[0, 0] == 2 and y[-1, -1] == 2
    assert m.nnz == 5 * 4096 - 4 * 64
