// Two-step HBP SpMV (Fig. 1, Algorithm 3, Section 3.3) and the in-repo CSR baselines.
//
// SpMV part: P persistent workgroups ("workers").  The column-major group list is cut into P
// ranges; a worker first runs the fixed groups of its range, then competes for the rest: every
// range has an atomic counter over its competitive groups (the tail of the range, inside one
// block column), and a worker claims groups from the range whose slice of x it has staged in
// LDS: its own first, then the range with the most left (the paper's single ticket lock, split
// per range so that a 128 KB slice is not restaged for every claim).  A wavefront takes one
// group at a time; lane q owns slot q of the group and walks its row round by round.  The
// distance add_sign of Algorithm 3 is not read from memory: in round k the lanes still alive
// are known from a ballot over the lane lengths, and a lane's element is the base of the
// round plus the number of live lanes below it.
//
// Combine part: one workgroup per row block adds the per-slot partial sums of that row
// block's blocks into an LDS copy of the y slice and writes it out, zeros included.
#include "hbp_spmv_impl.h"

namespace hbp {

Layout hbp_view(const hbp_handle_s *h)
{
    Layout L;
    L.R = h->R; L.C = h->C; L.W = h->W;
    L.B = (int32_t)h->B; L.S = (int32_t)h->S; L.G = (int32_t)h->G;
    L.NBR = (int32_t)h->NBR; L.NBC = (int32_t)h->NBC; L.P = h->P;
    const bool paper = h->first_ticket_block >= 0;
    L.competitive = !paper && h->fixed_q8 < 256 ? 1 : 0;
    L.ticket_b0 = paper ? (int32_t)h->first_ticket_block : -1;
    L.n_rows = h->n_rows; L.n_cols = h->n_cols;
    L.blk_bm = h->blk_bm; L.blk_bn = h->blk_bn; L.slot_ptr = h->slot_ptr; L.blk_group_ptr = h->blk_group_ptr;
    L.col_blk_ptr = h->col_blk_ptr; L.stripe_ptr = h->stripe_ptr; L.stripe_blk = h->stripe_blk;
    L.group_ptr = h->group_ptr; L.group_slot = h->group_slot; L.group_rounds = h->group_rounds;
    L.row_local = h->row_local; L.seg_len = h->seg_len; L.col_local = h->col_local; L.data = h->data;
    L.col_group_ptr = h->col_group_ptr; L.comp_lo = h->comp_lo; L.comp_col = h->comp_col;
    L.fixed_start = h->fixed_start; L.fixed_col = h->fixed_col;
    L.unit_ptr = h->unit_ptr; L.unit_stripe = h->unit_stripe; L.unit_k = h->unit_k; L.multi_stripes = h->multi_stripes;
    L.NM = (int32_t)h->NM;
    L.claim = h->claim_chunk * (h->threads / kWave);
    L.SW = h->slot_weight; L.RW = h->round_weight; L.GW = h->group_weight;
    L.steal_min = 2 * h->column_weight;
    L.heavy_rounds = h->heavy_rounds;
    L.long_rounds = long_rounds_of(h->heavy_rounds);
    return L;
}

// Workers the schedule is built for when the caller does not say: as many workgroups as fit
// on the device at once given the LDS a vector segment takes.
int default_workers(int device, int32_t C, int32_t value_bytes, int32_t threads_wanted, int32_t *threads_out, int32_t *workers_out)
{
    hipDeviceProp_t prop;
    HBP_HIP(hipGetDeviceProperties(&prop, device));
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const size_t lds = (size_t)C * (size_t)value_bytes + 64;
    const int threads = threads_wanted ? threads_wanted : (lds > 80 * 1024 ? 1024 : 512);
    int per_cu = (int)((160 * 1024) / lds);
    const int by_threads = 2048 / threads;
    if (per_cu > by_threads) per_cu = by_threads;
    if (per_cu < 1) per_cu = 1;
    *threads_out = threads;
    *workers_out = cus * per_cu;
    return HBP_OK;
}

// fp64 instantiations live in a translation unit of their own (hbp_spmv_f64.hip)
int launch_spmv_part_f64(const hbp_handle_s *h, const double *x, double *y, hipStream_t st, SpmvScratch sc);
int launch_combine_f64(const hbp_handle_s *h, double *y, hipStream_t st, SpmvScratch sc);
int launch_csr_f64(int kind, const int32_t *ptr, const int32_t *col, const double *val, const double *x, double *y, int64_t n_rows,
                   hipStream_t st);

int launch_spmv_part(const hbp_handle_s *h, const void *x, void *y, hipStream_t st, SpmvScratch sc)
{
    if (h->value_bytes == 8) return launch_spmv_part_f64(h, static_cast<const double *>(x), static_cast<double *>(y), st, sc);
    return launch_part_t<float>(h, static_cast<const float *>(x), static_cast<float *>(y), st, sc);
}

int launch_combine(const hbp_handle_s *h, void *y, hipStream_t st, SpmvScratch sc)
{
    if (h->value_bytes == 8) return launch_combine_f64(h, static_cast<double *>(y), st, sc);
    return launch_combine_t<float>(h, static_cast<float *>(y), st, sc);
}

int launch_csr(int kind, int value_bytes, const int32_t *ptr, const int32_t *col, const void *val, const void *x, void *y,
               int64_t n_rows, hipStream_t st)
{
    if (value_bytes == 8)
        return launch_csr_f64(kind, ptr, col, static_cast<const double *>(val), static_cast<const double *>(x),
                              static_cast<double *>(y), n_rows, st);
    return launch_csr_t<float>(kind, ptr, col, static_cast<const float *>(val), static_cast<const float *>(x),
                               static_cast<float *>(y), n_rows, st);
}

}  // namespace hbp
