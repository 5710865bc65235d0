"""GPU parity of the fp64 variant (hbp_build_f64 / hbp_spmv_f64; Section 3.1 counts 8 bytes per
stored value): same checks as the fp32 tests, on inputs whose values are not representable in
float32, so that a path that narrows anything to fp32 fails.  Layout bit-equal (data as 64-bit
patterns); y and the per-slot partial sums within 168 * 2^-53 * sum_j |a_ij x_j|."""
import os

import numpy as np
import pytest

from test_gpu_parity import H, _mixed_matrix, _with_long_rows, check_against_oracle, to_dev, TOL_F64  # noqa: F401
from workloads import make_config, random_csr, widen_to_f64

pytestmark = pytest.mark.gpu

SMALL = [
    # rows, cols, density, seed, R, C, W, shift
    (40, 40, 0.2, 1, 8, 8, 4, -1),
    (129, 65, 0.5, 4, 32, 16, 3, 2),
    (200, 30, 0.1, 6, 512, 4096, 64, -1),
    (1000, 1000, 0.02, 7, 100, 333, 64, -1),
    (5000, 3000, 0.01, 8, 512, 1024, 32, -1),
    (3000, 9000, 0.05, 9, 4096, 16384, 64, -1),   # the largest block the fp64 variant accepts
    (2500, 700, 0.3, 10, 1, 1, 1, 0),
]


@pytest.mark.parametrize("case", SMALL)
def test_small_random(H, oracle, case):
    nr, nc, dens, seed, R, C, W, shift = case
    m = widen_to_f64(random_csr(nr, nc, dens, seed, empty_row_frac=0.15), seed)
    check_against_oracle(H, oracle, m, rows_per_block=R, cols_per_block=C, group_width=W, hash_shift=shift)


@pytest.mark.parametrize("number,scale,R,C", [(1, 1.0, 512, 4096), (2, 0.02, 512, 16384), (3, 2**-6, 256, 1024),
                                              (4, 2**-7, 512, 2048), (5, 0.01, 2048, 16384)])
def test_configs_reduced(H, oracle, number, scale, R, C):
    check_against_oracle(H, oracle, widen_to_f64(make_config(number, scale)), rows_per_block=R, cols_per_block=C)


@pytest.mark.parametrize("rounds", [2, 4, 8, 9, 16])
@pytest.mark.parametrize("threads", [256, 512, 1024])
def test_kernel_variants(H, oracle, rounds, threads):
    """Every fp64 instantiation of the SpMV-part kernel, on the matrix that reaches all walking
    modes (aligned wide loads, packs of groups, deep batches, whole-wavefront spans)."""
    m = widen_to_f64(_mixed_matrix())
    for q8, workers in ((256, 7), (160, 5)):
        check_against_oracle(H, oracle, m, check_add_sign=False, rows_per_block=1024, cols_per_block=8192,
                             rounds_per_batch=rounds, threads_per_worker=threads, fixed_fraction_q8=q8,
                             num_workers=workers, slot_weight=3)


@pytest.mark.parametrize("heavy", [1, 60, 700])
@pytest.mark.parametrize("rounds,threads", [(4, 512), (8, 1024), (16, 256)])
def test_heavy_groups_shared_by_a_worker(H, oracle, heavy, rounds, threads):
    m = widen_to_f64(_mixed_matrix(seed=7))
    for q8, workers in ((256, 3), (128, 6)):
        check_against_oracle(H, oracle, m, check_add_sign=False, rows_per_block=2048, cols_per_block=8192,
                             rounds_per_batch=rounds, threads_per_worker=threads, fixed_fraction_q8=q8,
                             num_workers=workers, heavy_group_rounds=heavy)


@pytest.mark.parametrize("unit_slots", [64, 5000])
def test_split_row_blocks(H, oracle, unit_slots):
    """Units of a split row block meet in y through fp64 atomic adds."""
    m = widen_to_f64(_mixed_matrix(seed=41))
    for R in (256, 2048):
        info = check_against_oracle(H, oracle, m, rows_per_block=R, cols_per_block=512, combine_unit_slots=unit_slots)
        if unit_slots == 64:
            assert info.split_row_blocks > 0


@pytest.mark.parametrize("seed", range(int(os.environ.get("HBP_RANDOM_CASES", "12"))))
def test_random_parameters(H, oracle, seed):
    rng = np.random.default_rng(2000 + seed)
    n_rows = int(rng.integers(1, 6000))
    n_cols = int(rng.integers(1, 9000))
    density = float(rng.choice([0.002, 0.01, 0.05, 0.2]))
    m = random_csr(n_rows, n_cols, density, 700 + seed, empty_row_frac=float(rng.choice([0.0, 0.3])))
    if seed % 3 == 0:
        m = _with_long_rows(m, rng)
    params = dict(
        rows_per_block=int(rng.choice([1, 7, 64, 512, 2048, 4096])),
        cols_per_block=int(rng.choice([1, 33, 256, 4096, 16384])),
        group_width=int(rng.choice([1, 5, 32, 64])),
        num_workers=int(rng.choice([0, 1, 3, 17, 300])),
        fixed_fraction_q8=int(rng.choice([0, 77, 192, 255, 256])),
        claim_chunk=int(rng.choice([0, 1, 3, 50])),
        threads_per_worker=int(rng.choice([256, 512, 1024])),
        rounds_per_batch=int(rng.choice([2, 4, 8, 9, 16])),
        slot_weight=int(rng.choice([0, 1, 4, 64])),
        group_weight=int(rng.choice([0, 10, 4096])),
        round_weight=int(rng.choice([0, 8, 1024])),
        column_weight=int(rng.choice([0, 0, 50, 100000])),
        combine_unit_slots=int(rng.choice([0, 64, 1000])),
        heavy_group_rounds=int(rng.choice([0, 1, 20, 300])),
        hash_shift=int(rng.choice([-1, 0, 3, 12])),
    )
    if params["rows_per_block"] * params["cols_per_block"] < 64 and n_rows * n_cols > 4_000_000:
        params["rows_per_block"] = 64
    check_against_oracle(H, oracle, widen_to_f64(m, seed), check_add_sign=seed % 3 == 0, **params)


def test_plain_2d_partition(H, oracle):
    check_against_oracle(H, oracle, widen_to_f64(_mixed_matrix(seed=3)), rows_per_block=512, cols_per_block=4096, no_reorder=True)


def test_handles_are_typed_and_limits(H):
    """An fp32 handle is refused by the fp64 calls and the other way round; the fp64 variant's
    block limits are half the fp32 ones in C and R (twice the LDS per element)."""
    import torch
    m = random_csr(50, 60, 0.2, 1)
    ptr, col, val, x = to_dev(m)
    h32 = H.hbp_build(ptr, col, val, m.n_rows, m.n_cols)
    h64 = H.hbp_build_f64(ptr, col, val.double(), m.n_rows, m.n_cols)
    y32 = torch.zeros(m.n_rows, device="cuda")
    y64 = torch.zeros(m.n_rows, device="cuda", dtype=torch.float64)
    try:
        for call in (lambda: H.lib().hbp_spmv(h64, x.data_ptr(), y32.data_ptr(), None),
                     lambda: H.lib().hbp_spmv_f64(h32, x.double().data_ptr(), y64.data_ptr(), None)):
            assert call() == -1
        assert H.hbp_get_info(h32).value_bytes == 4 and H.hbp_get_info(h64).value_bytes == 8
    finally:
        H.hbp_free(h32)
        H.hbp_free(h64)
    for kw in (dict(rows_per_block=4097), dict(cols_per_block=16385)):
        with pytest.raises(H.HbpError) as e:
            H.hbp_build_f64(ptr, col, val.double(), m.n_rows, m.n_cols, **kw)
        assert e.value.status == -1


@pytest.mark.parametrize("kind", [0, 1])
def test_csr_baselines(H, oracle, kind):
    import torch
    for m in (make_config(1), random_csr(300, 200, 0.2, 4, empty_row_frac=0.2)):
        m = widen_to_f64(m)
        ptr, col, val, x = to_dev(m)
        y = torch.full((m.n_rows,), float("nan"), device="cuda", dtype=torch.float64)
        H.hbp_csr_spmv_f64(kind, ptr, col, val, x, y)
        torch.cuda.synchronize()
        y_ref, s_abs = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
        assert np.all(np.abs(y.cpu().numpy() - y_ref) <= TOL_F64 * s_abs)
