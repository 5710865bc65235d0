// fp64 instantiations of the SpMV kernels (the fp64 variant stores values as Section 3.1's cost
// estimate counts them: 8 bytes each); see hbp_spmv_impl.h.
#include "hbp_spmv_impl.h"

namespace hbp {

int launch_spmv_part_f64(const hbp_handle_s *h, const double *x, double *y, hipStream_t st, SpmvScratch sc)
{
    return launch_part_t<double>(h, x, y, st, sc);
}

int launch_combine_f64(const hbp_handle_s *h, double *y, hipStream_t st, SpmvScratch sc) { return launch_combine_t<double>(h, y, st, sc); }

int launch_csr_f64(int kind, const int32_t *ptr, const int32_t *col, const double *val, const double *x, double *y, int64_t n_rows,
                   hipStream_t st)
{
    return launch_csr_t<double>(kind, ptr, col, val, x, y, n_rows, st);
}

}  // namespace hbp
