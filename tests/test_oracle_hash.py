"""Pins for the nonlinear hash (Section 3.2) and the sampled shift: hand-computed values,
the properties the paper's text fixes, and brute force over the sampled rows."""
import numpy as np
import pytest

from workloads import random_csr, make_config


def test_hand_computed_keys(oracle):
    # R = 512 -> b = d = 56.  a = 0: key = 56 * min(n, 8).
    assert oracle.hash_key(0, 0, 512) == 0
    assert oracle.hash_key(3, 0, 512) == 168
    assert oracle.hash_key(8, 0, 512) == 448
    assert oracle.hash_key(100, 0, 512) == 448
    # a = 2 (c = 4): n = 5 -> class 1, (5 mod 4) * 56 >> 2 = 14 -> 70
    assert oracle.hash_key(5, 2, 512) == 70
    assert oracle.hash_key(7, 2, 512) == 98
    assert oracle.hash_key(35, 2, 512) == 490   # class 8, lin 42
    assert oracle.hash_key(36, 2, 512) == 448   # 36 >> 2 = 9, treated as 8; lin 0
    # R = 4 -> b = 1, key = min(n, 3) at a = 0 (the worked example)
    assert [oracle.hash_key(n, 0, 4) for n in range(6)] == [0, 1, 2, 3, 3, 3]
    # tiny R: key never leaves the table
    assert oracle.hash_key(1000, 0, 1) == 0


@pytest.mark.parametrize("R", [1, 4, 9, 64, 512, 4096, 8192, 65536])
@pytest.mark.parametrize("a", [0, 1, 2, 5, 12])
def test_key_properties(oracle, R, a):
    b = max(1, R // 9)
    ns = list(range(0, min(9 << a, 3000) + 40)) + [4095, 4096, 32767, 65535]
    keys = [oracle.hash_key(n, a, R) for n in ns]
    assert all(0 <= k < R for k in keys)                       # stays inside the block's table
    prev = -1
    for n, k in zip(ns, keys):
        cls = min(n >> a, 8)
        if R >= 9 * b + 0 and (8 * b + b - 1) <= R - 1:
            assert k // b == cls                                 # dispersion: one band per class
            assert k - cls * b < b                               # linear part stays inside its band
        if n < (9 << a) and n < 3000:
            assert k >= prev                                     # small rows first, monotone
            prev = k
    # rows with equal n >> a <= 8 share an aggregation class (paper: a = 2 groups 4k..4k+3)
    if (8 * b + b - 1) <= R - 1:
        for n in range(0, 8 << a, max(1, (1 << a))):
            band = {oracle.hash_key(n + i, a, R) // b for i in range(1 << a)}
            assert len(band) == 1


def test_paper_shift_example(oracle):
    """With a = 2 the aggregation puts 4k .. 4k+3 together (Section 3.2, Fig. 4 text)."""
    R, b = 512, 56
    for k in range(9):
        assert {oracle.hash_key(4 * k + i, 2, R) // b for i in range(4)} == {min(k, 8)}
    assert oracle.hash_key(4 * 9, 2, R) // b == 8      # overflow rows count as class 8


def test_strictly_increasing_when_shift_small(oracle):
    # 2^a <= b: distinct n below 9 * 2^a get distinct keys
    for a in (0, 1, 3, 5):
        keys = [oracle.hash_key(n, a, 512) for n in range(9 << a)]
        assert all(x < y for x, y in zip(keys, keys[1:]))


def brute_shift(ptr, col, n_rows, C):
    S = min(n_rows, 4096)
    lens = []
    for k in range(S):
        r = (k * n_rows) // S
        blocks = [int(c) // C for c in col[ptr[r]:ptr[r + 1]]]
        for bn in sorted(set(blocks)):
            lens.append(blocks.count(bn))
    if not lens:
        return 0
    lens = np.array(lens)
    for a in range(13):
        if 16 * np.sum(lens < 9 * 2**a) >= 15 * len(lens):
            return a
    return 12


@pytest.mark.parametrize("seed,C", [(0, 8), (1, 16), (2, 64), (3, 1000)])
def test_sample_shift_brute_force(oracle, seed, C):
    m = random_csr(300, 1000, 0.05 + 0.1 * seed, seed, empty_row_frac=0.1)
    assert oracle.sample_shift(m.ptr, m.col, m.n_rows, C) == brute_shift(m.ptr, m.col, m.n_rows, C)


def test_sample_shift_subsamples_rows(oracle):
    m = make_config(5, scale=0.003)   # 12000 rows > 4096: only every ~3rd row is looked at
    assert m.n_rows > 4096
    assert oracle.sample_shift(m.ptr, m.col, m.n_rows, 256) == brute_shift(m.ptr, m.col, m.n_rows, 256)


@pytest.mark.parametrize("n", [1, 8, 9, 17, 18, 35, 36, 100, 1000])
def test_sample_shift_equal_rows(oracle, n):
    """All rows of length n in one column block: a is the smallest shift with n < 9 * 2^a."""
    rows = 40
    ptr = (np.arange(rows + 1) * n).astype(np.int32)
    col = np.tile(np.arange(n), rows).astype(np.int32)
    expect = next(a for a in range(13) if n < 9 * 2**a)
    assert oracle.sample_shift(ptr, col, rows, 4096) == expect


def test_sample_shift_empty(oracle):
    ptr = np.zeros(11, dtype=np.int32)
    col = np.zeros(1, dtype=np.int32)
    assert oracle.sample_shift(ptr, col, 10, 16) == 0
