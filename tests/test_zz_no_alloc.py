"""hbp_spmv_static_scratch (the entry point that allocates nothing: partial sums and claim counters in
the library's fixed array) against hbp_spmv, through the C ABI: two calls in a row, the second on a
smaller matrix, plus the size limit."""
import ctypes

import numpy as np
import pytest

from workloads import make_config, random_csr

pytestmark = pytest.mark.gpu

TOL = 1e-5


def _dev(m):
    import torch
    t = lambda a: torch.from_numpy(a).cuda()
    return t(m.ptr), t(m.col), t(m.val), t(m.x)


def test_static_scratch_matches_hbp_spmv(oracle):
    import torch
    import paper_2504_08860_amd as H
    L = H.lib()
    stream = torch.cuda.current_stream().cuda_stream
    # the larger one first (competitive part on, several block columns), then a smaller one: the second
    # call finds the first one's partial sums and counters in the array
    cases = [(make_config(5, 0.02), dict(rows_per_block=512, cols_per_block=2048, fixed_fraction_q8=160, num_workers=48)),
             (random_csr(3000, 2500, 0.01, 5, empty_row_frac=0.2), dict(rows_per_block=64, cols_per_block=256, num_workers=7))]
    first_call = True
    for m, params in cases:
        print(f"[no-alloc] {m.name} nnz={m.nnz} {params}", flush=True)
        ptr, col, val, x = _dev(m)
        h = H.hbp_build(ptr, col, val, m.n_rows, m.n_cols, **params)
        try:
            info = H.hbp_get_info(h)
            assert info.split_row_blocks == 0      # every sum has one order: the two entry points must agree bit for bit
            y_ref = torch.full((m.n_rows,), float("nan"), device="cuda")
            H.hbp_spmv(h, x, y_ref)
            torch.cuda.synchronize()
            for rep in range(2):
                y = torch.full((m.n_rows,), float("nan"), device="cuda")
                # free device memory as the driver sees it (tensors that Python drops meanwhile go back to
                # torch's cache, not to the device, so only an allocation from the device would move it)
                torch.cuda.synchronize()
                free_before = torch.cuda.mem_get_info()[0]
                rc = L.hbp_spmv_static_scratch(ctypes.c_void_p(h), ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(y.data_ptr()),
                                               ctypes.c_void_p(stream))
                assert rc == 0, H.hbp_status_string(rc)
                torch.cuda.synchronize()
                # (the process's very first call makes the runtime load the code object that holds the
                # fixed array, which is when the device gives it its 32 MiB: not an allocation of the call)
                assert first_call or torch.cuda.mem_get_info()[0] == free_before
                first_call = False
                assert torch.equal(y, y_ref), f"{m.name} rep {rep}"
            yo, s_abs = oracle.csr_spmv_f64(m.ptr, m.col, m.val, m.x)
            assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - yo) <= TOL * s_abs)
            # the handle's own entry point still works after the other one has run
            y2 = torch.full((m.n_rows,), float("nan"), device="cuda")
            H.hbp_spmv(h, x, y2)
            torch.cuda.synchronize()
            assert torch.equal(y2, y_ref)
        finally:
            H.hbp_free(h)


def test_static_scratch_limits():
    import torch
    import paper_2504_08860_amd as H
    L = H.lib()
    # more slots than the array holds (8,323,072): refused, nothing launched
    m = make_config(3, 0.5)
    ptr, col, val, x = _dev(m)
    h = H.hbp_build(ptr, col, val, m.n_rows, m.n_cols, cols_per_block=4096)
    try:
        assert H.hbp_get_info(h).slots > 8_323_072
        y = torch.zeros(m.n_rows, device="cuda")
        with pytest.raises(H.HbpError) as e:
            H.hbp_spmv_static_scratch(h, x, y)
        assert e.value.status == -4
        assert L.hbp_spmv_static_scratch(None, None, None, None) == -1
    finally:
        H.hbp_free(h)
