"""Seeded synthetic CSR workloads.

These generators are the only code shared by the CPU oracle's tests and the
HIP path's tests/bench.  They hold none of the method's arithmetic: they only
produce CSR matrices (int32 ``ptr``/``col``, float32 ``val``; ``widen_to_f64`` gives the
float64 variant) and dense vectors
``x`` whose shapes and sparsity structure stand in for the SuiteSparse matrices
of the paper's Table 1, which cannot be obtained here.

Every matrix has strictly ascending, duplicate-free column indices inside each
row, as the data-preparation scan of the paper's Algorithm 2 presumes.
"""
from .generators import (  # noqa: F401
    CsrMatrix,
    CONFIG_NAMES,
    make_config,
    laplacian_2d,
    stencil_27pt,
    row_template,
    rmat,
    lognormal_rect,
    random_csr,
    worked_example_8x8,
    widen_to_f64,
)
