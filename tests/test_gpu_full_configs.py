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
