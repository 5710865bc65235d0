"""Full-size parity on the five benchmark configurations, with the block parameters the
bench uses.  The C oracle builds the whole layout in seconds, so every array is compared
in full, bit for bit, and every row of y is checked against the fp64 definition."""
import numpy as np
import pytest

from workloads import make_config

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("number", [1, 2, 3, 4, 5])
def test_full_config(oracle, number):
    import paper_2504_08860_amd as H
    from paper_2504_08860_amd.presets import preset
    from test_gpu_parity import check_against_oracle
    m = make_config(number)
    print(f"[full] config {number}: {m.name} nnz={m.nnz}", flush=True)
    check_against_oracle(H, oracle, m, check_add_sign=(number <= 2), validate=False, **preset(number))


@pytest.mark.parametrize("number", [2, 4])
def test_full_config_f64(oracle, number):
    """The fp64 variant at full size, in the launch configuration `bench.py --dtype f64` times:
    the stencil (aligned wide loads) and the R-MAT matrix (competition, heavy groups)."""
    import paper_2504_08860_amd as H
    from paper_2504_08860_amd.presets import preset
    from test_gpu_parity import check_against_oracle
    from workloads import widen_to_f64
    m = widen_to_f64(make_config(number))
    params = preset(number, "f64")
    print(f"[full] config {number} fp64: {m.name} nnz={m.nnz}", flush=True)
    check_against_oracle(H, oracle, m, check_add_sign=False, validate=False, **params)
