"""Full-size parity on the five benchmark configurations, in the launch configuration bench.py
times: block parameters chosen by the library itself.  The C oracle builds the whole layout in
seconds, so every array (the keys and add_sign included) is compared in full, bit for bit, and
every row of y and every partial sum is checked against the fp64 definition."""
import numpy as np
import pytest

from workloads import make_config

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("number", [1, 2, 3, 4, 5])
def test_full_config(oracle, number):
    import paper_2504_08860_amd as H
    from test_gpu_parity import check_against_oracle
    m = make_config(number)
    print(f"[full] config {number}: {m.name} nnz={m.nnz}", flush=True)
    check_against_oracle(H, oracle, m, check_add_sign=True, validate=False)


@pytest.mark.parametrize("number", [2, 5])
def test_full_config_tuned_and_paper_schedule(oracle, number):
    """The comparison legs of bench.py at full size: hand-picked block sizes, and the paper's own schedule."""
    import paper_2504_08860_amd as H
    from paper_2504_08860_amd.presets import tuned_block_sizes
    from test_gpu_parity import check_against_oracle
    m = make_config(number)
    print(f"[full] config {number} legs: {m.name} nnz={m.nnz}", flush=True)
    check_against_oracle(H, oracle, m, check_add_sign=False, validate=False, **tuned_block_sizes(number))
    check_against_oracle(H, oracle, m, check_add_sign=False, validate=False, paper_schedule=True)


@pytest.mark.parametrize("number", [2, 4])
def test_full_config_f64(oracle, number):
    """The fp64 variant at full size, in the launch configuration `bench.py --dtype f64` times:
    the stencil (aligned wide loads) and the R-MAT matrix (competition, heavy groups)."""
    import paper_2504_08860_amd as H
    from test_gpu_parity import check_against_oracle
    from workloads import widen_to_f64
    m = widen_to_f64(make_config(number))
    print(f"[full] config {number} fp64: {m.name} nnz={m.nnz}", flush=True)
    check_against_oracle(H, oracle, m, check_add_sign=False, validate=False)
