// Internal declarations shared by the translation units of libhbp (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hbp.h"

namespace hbp {

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kMaxR = 8192;          // rows per block: one block's slots are ordered in 64 KB of LDS
constexpr int kMaxC = 32768;         // columns per block: fp32 vector segment of 128 KB in LDS
constexpr int kMaxC64 = 16384;       // the same 128 KB with fp64 values
constexpr int kMaxR64 = 4096;        // fp64: the combine part keeps four copies of a y slice in LDS
constexpr int64_t kMaxDense = int64_t(1) << 27;  // NBR * NBC table entries
// rows longer than this (and up to heavy_group_rounds) make their group a "long" one
inline int32_t long_rounds_of(int32_t heavy_rounds) { return heavy_rounds / 8 > 0 ? heavy_rounds / 8 : 1; }

// Device-side view of the layout, passed by value to kernels.
struct Layout {
    int32_t R, C, W;
    int32_t B, S, G;
    int32_t NBR, NBC, P;
    int32_t competitive;  // 0 when every group is fixed (nothing to compete for)
    int32_t ticket_b0;    // the paper's schedule: first block behind the single ticket counter; -1: not in use
    int64_t n_rows, n_cols;
    const int32_t *blk_bm, *blk_bn, *slot_ptr, *blk_group_ptr, *col_blk_ptr, *stripe_ptr, *stripe_blk;
    const int32_t *group_ptr, *group_slot, *group_rounds;
    const int32_t *col_group_ptr, *comp_lo, *comp_col, *fixed_start, *fixed_col;  // schedule (Section 3.3)
    const int32_t *unit_ptr, *unit_stripe, *unit_k, *multi_stripes;               // combine work units
    int32_t NM;                                                        // row blocks with several units
    int32_t claim;  // competitive groups a worker claims from a range's counter at a time
    int32_t SW, RW, GW;  // schedule weights of a slot, a round, a group (a nonzero weighs 1)
    int32_t steal_min;   // weight a range's competitive part must have left for another worker to enter it
    int32_t heavy_rounds;  // a group with a longer row is walked by all wavefronts of a worker together
    int32_t long_rounds;   // a group with a longer row (up to heavy_rounds) waits for a wavefront of its own
    const uint16_t *row_local, *seg_len, *col_local;
    const void *data;  // float or double, by the handle's value type
};

}  // namespace hbp

struct hbp_handle_s {
    int device;
    int64_t n_rows, n_cols, nnz;
    int32_t R, C, W, a;
    int64_t NBR, NBC, B, S, G;
    int32_t P, fixed_q8, slot_weight, claim_chunk, threads;
    int32_t unroll;      // rounds taken per batch by the SpMV-part kernel
    double build_ms;
    // device arrays (owned): views into two allocations, arena[0] sized before the matrix is
    // looked at, arena[1] after the segment, group and block counts are known
    void *arena[2];
    int32_t *blk_bm, *blk_bn, *slot_ptr, *blk_group_ptr, *col_blk_ptr, *stripe_ptr, *stripe_blk;
    int32_t *group_ptr, *group_slot;
    int32_t *col_group_ptr, *comp_lo, *comp_col, *fixed_start, *fixed_col;
    int32_t *group_rounds;               // [G+1] prefix sums of the groups' longest rows
    int32_t *unit_ptr, *unit_stripe, *unit_k, *multi_stripes;
    int64_t U, NM;       // combine work units, row blocks cut into several units
    int32_t unit_slots;  // target slots per combine unit
    int32_t heavy_rounds;  // groups with a longer row are shared by a worker's wavefronts
    int32_t group_weight;  // schedule weight of a group as such
    int32_t longest_segment;  // longest row segment of the matrix (0 unless it makes a group long)
    int32_t round_weight;  // schedule weight of a group on top of its nonzeros and slots
    int32_t column_weight;  // schedule weight of entering a block column
    int32_t *col_rank;     // [NBC+1] non-empty block columns before each column
    uint16_t *row_local, *seg_len, *col_local;
    int32_t value_bytes; // 4: fp32 values (data, partial, x, y), 8: fp64
    void *data;
    void *partial;       // [S] per-slot partial sums of the SpMV part
    uint32_t *ticket;    // [P] competitive groups of every worker's range claimed so far, zero between calls
    uint32_t *slot_key;  // [S] key each slot was placed by, or null (HBP_FLAG_KEEP_KEYS)
    int32_t *blk_shift;  // [B] shift a of each block's keys
    int64_t first_ticket_block;  // the paper's schedule (HBP_FLAG_PAPER_SCHEDULE): P F; -1 otherwise
    uint32_t flags;      // HBP_FLAG_* the handle was built with
};

namespace hbp {

// error plumbing -----------------------------------------------------------------------
void set_last_hip_error(hipError_t e);
#define HBP_HIP(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) {                        \
            hbp::set_last_hip_error(e_);               \
            return e_ == hipErrorOutOfMemory ? HBP_ERR_OUT_OF_MEMORY : HBP_ERR_HIP; \
        }                                              \
    } while (0)

// build (hbp_build.hip)
int build_layout(hbp_handle_s *h, const int32_t *csr_ptr, const int32_t *csr_col, const void *csr_val,
                 const hbp_params_t &p, hipStream_t stream);
int build_schedule(hbp_handle_s *h, hipStream_t stream);
int choose_block_parameters(const int32_t *csr_ptr, const int32_t *csr_col, int64_t n_rows, int64_t n_cols, int32_t value_bytes,
                            hbp_params_t &p, hipStream_t stream);
int derive_add_sign(const hbp_handle_s *h, int32_t *d_out, hipStream_t stream);
int hash_keys(const uint32_t *n, int64_t count, int32_t a, int32_t R, uint32_t *keys, hipStream_t stream);
int release_workspace();

// spmv (hbp_spmv.hip)
Layout hbp_view(const hbp_handle_s *h);
int default_workers(int device, int32_t C, int32_t value_bytes, int32_t threads_wanted, int32_t *threads_out, int32_t *workers_out);
// x, y (and val): arrays of the handle's value type (value_bytes for the CSR baselines)
// where one SpMV keeps its per-slot partial sums (S values of the handle's type) and its claim counters (P)
struct SpmvScratch {
    void *partial;
    uint32_t *ticket;
};
int launch_spmv_part(const hbp_handle_s *h, const void *x, void *y, hipStream_t stream, SpmvScratch scratch);
int launch_combine(const hbp_handle_s *h, void *y, hipStream_t stream, SpmvScratch scratch);
int launch_csr(int kind, int value_bytes, const int32_t *ptr, const int32_t *col, const void *val, const void *x, void *y,
               int64_t n_rows, hipStream_t stream);

}  // namespace hbp
