/*
 * hbp.h - C ABI of the MI355X (gfx950) Hash-based Partition (HBP) SpMV library.
 *
 * The library implements the data-parallel hot path of "A Nonlinear Hash-based
 * Optimization Method for SpMV on GPUs": the hash-driven preprocessing that turns a CSR
 * matrix into the HBP format (Sections 3.1-3.2, Algorithm 2) and the two-step
 * y = A x with mixed fixed/competitive block scheduling (Section 3.3, Algorithm 3,
 * Fig. 1).  Every step runs in hand-written HIP kernels on the current device.
 *
 * Conventions
 *   - Pointers marked DEVICE are device addresses on the GPU that is current when the
 *     call is made; pointers marked HOST are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every function returns HBP_OK (0) or a negative hbp_status; nothing throws or
 *     aborts across this boundary.  hbp_status_string() names a status.
 *   - The caller owns csr_*, x and y.  A handle owns all of its device arrays and
 *     copies the matrix values, so the CSR arrays may be freed once hbp_build returns.
 *
 * Layout held by a handle ("compact" HBP; the paper's arrays in parentheses)
 *   Blocks are R rows x C columns.  Only blocks with at least one nonzero are kept,
 *   listed column-major (column block bn ascending, then row block bm): the order in
 *   which Section 3.3 hands blocks of one column to one worker.  Inside a block only
 *   rows with a nonzero in it own a slot; slots are in ascending (hash key, local row)
 *   order.  W consecutive slots of a block are a group; a group's nonzeros are stored
 *   round by round (round k holds the k-th nonzero of every row that still has one).
 *     blk_bm, blk_bn      [B]      block coordinates
 *     slot_ptr            [B+1]    first slot of each block
 *     blk_group_ptr       [B+1]    first group of each block
 *     col_blk_ptr         [NBC+1]  first block of each block column
 *     stripe_ptr          [NBR+1]  per row block, range into stripe_blk
 *     stripe_blk          [B]      blocks of one row block, bn ascending (combine index)
 *     group_ptr           [G+1]    position of a group's first nonzero   (begin_ptr)
 *     group_slot          [G+1]    first slot of a group
 *     group_rounds        [G+1]    rounds of all groups before (prefix sums of the longest row)
 *   Schedule (Section 3.3; the unit handed to a wavefront is a group, whose weight is its
 *   nonzeros plus slot_weight times its slots plus round_weight times its rounds, the
 *   length of its longest row, plus group_weight):
 *     col_group_ptr       [NBC+1]  first group of each block column
 *     fixed_start         [P+1]    the group list cut into P contiguous ranges of equal
 *                                  weight (a block column adds column_weight to its first
 *                                  group here); worker w runs the fixed groups of range w
 *     fixed_col           [P]      block column that holds a worker's first group
 *     comp_lo             [P]      first competitive group of a worker's range: the range keeps the
 *                                  leading fixed_fraction of its weight as fixed part; the rest, as
 *                                  far as it lies in the block column of the range's last group, is
 *                                  left to competition (the worker itself and workers that have
 *                                  run out of work claim it piece by piece)
 *     comp_col            [P]      that block column
 *   Combine units (Section 3.3, combine part: one workgroup per unit instead of one per row
 *   block, so that a row block with very many slots does not hold up the rest):
 *     unit_ptr            [NBR+1]  first unit of each row block; a row block has
 *                                  u = max(1, ceil(its slots / combine_unit_slots)) units
 *     unit_stripe         [U]      row block of a unit
 *     unit_k              [U+1]    first stripe_blk entry of a unit: unit i of a row block starts at
 *                                  the first entry whose preceding slots times u reach i times the
 *                                  row block's slots; unit_k[U] = B
 *     multi_stripes       [NM]     row blocks with more than one unit, ascending
 *     row_local   u16     [S]      slot -> row inside its block          (output_hash)
 *     seg_len     u16     [S]      nonzeros of that row inside the block (add_sign is
 *                                  derived from these at run time)
 *     col_local   u16     [nnz]    column inside the block               (col)
 *     data        f32/f64 [nnz]    values, bit-for-bit copies            (data)
 *   begin_nnz of a block is group_ptr[blk_group_ptr[b]]; zero_row is not stored because
 *   empty rows own no slot.
 *
 * Value type.  A handle holds fp32 values (hbp_build; x, y and the partial sums are fp32 and
 *   all products and sums are taken in fp32) or fp64 values, the storage type of Section 3.1's
 *   cost estimate (hbp_build_f64; x, y, partial sums and arithmetic fp64).  Everything except
 *   `data` and `partial` is the same for both.  The entry points without suffix take fp32
 *   handles, those ending in _f64 take fp64 handles; the other kind of handle is refused
 *   with HBP_ERR_INVALID_ARGUMENT.
 */
#ifndef HBP_H
#define HBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hbp_handle_s *hbp_handle_t;

typedef enum {
    HBP_OK = 0,
    HBP_ERR_INVALID_ARGUMENT = -1,   /* null pointer, non-positive size, parameter out of range */
    HBP_ERR_BAD_CSR_PTR = -2,        /* csr_ptr[0] != 0, decreasing, or beyond nnz */
    HBP_ERR_BAD_CSR_COL = -3,        /* column < 0, >= n_cols, or not strictly ascending in a row */
    HBP_ERR_TOO_LARGE = -4,          /* nnz or NBR*NBC beyond the supported range */
    HBP_ERR_OUT_OF_MEMORY = -5,
    HBP_ERR_HIP = -6,                /* a HIP runtime call failed; see hbp_last_hip_error() */
    HBP_ERR_INTERNAL = -7
} hbp_status;

/* flags for hbp_params_t.flags */
#define HBP_FLAG_VALIDATE 1u /* check column order/range of the CSR input during the build */
#define HBP_FLAG_NO_REORDER 2u /* plain 2D partitioning, the method Section 4 compares HBP with: no hash
                                  reorder, the slots of a block stay in ascending row order */
#define HBP_FLAG_KEY_LENGTH 4u /* hash study (Section 5 names the hash function as open to improvement): the
                                  key of a row is its length inside the block itself instead of the hash of
                                  it, i.e. the limit of an ever finer mapping: slots in ascending (length,
                                  row) order.  Ignored with HBP_FLAG_NO_REORDER. */

#define HBP_FLAG_PAPER_SCHEDULE 8u /* Section 3.3 read literally instead of this library's schedule: the units are
                                  blocks in the layout's column-major order, every worker is pre-assigned
                                  F = floor(B * fixed_fraction / P) of them (blocks [w F, (w + 1) F) go to worker w)
                                  and the blocks from P F on are claimed one at a time through a single ticket
                                  counter.  The weights and claim_chunk are ignored. */
#define HBP_FLAG_BLOCK_SHIFT 16u /* hash study: one shift a per block (Section 3.2: denser blocks call for a larger
                                  a) instead of one per matrix: the smallest a in 0..12 for which at least 15/16
                                  of the block's own rows have fewer than 9 * 2^a nonzeros in it.  hash_shift is
                                  ignored; ignored itself with HBP_FLAG_NO_REORDER or HBP_FLAG_KEY_LENGTH. */
#define HBP_FLAG_KEEP_KEYS 32u /* keep the key every slot was placed by (4 bytes per slot) for hbp_export */

/* Build parameters.  Section 3.1 derives its block of 512 rows x 4096 columns from the 48 KB of
 * shared memory of the paper's GPUs; here the vector segment of a block is staged in the 160 KB
 * LDS of a gfx950 compute unit, and a value of 0 (or -1 where 0 is a valid choice) leaves the
 * choice to the library, which makes it from the matrix (the sampling pass of Section 3.2 also
 * measures the mean number of nonzeros a row has inside one column block). */
typedef struct {
    int32_t rows_per_block;    /* R, 1..8192 (fp64: 1..4096); 0 = chosen: 512 when the sampled rows average 6 or
                                  more nonzeros per column block, else 2048 (the paper's value is 512)  */
    int32_t cols_per_block;    /* C, 1..32768 (fp64: 1..16384): at most 128 KB of x in LDS; 0 = chosen: that
                                  maximum, or n_cols if the whole vector is shorter (the paper's value is 4096) */
    int32_t group_width;       /* W, 1..64 lanes per group; 0 = default 64 (one wavefront)      */
    int32_t num_workers;       /* P, persistent workgroups the schedule is built for, up to 65536; 0 = as many as
                                  fit on the device at once, but no more than one per threads_per_worker / 64 groups */
    int32_t fixed_fraction_q8; /* share of every worker's range that is pre-assigned, in 1/256; -1 = default 240 */
    int32_t hash_shift;        /* a, 0..12; -1 = sample it from the matrix (Section 3.2)        */
    int32_t claim_chunk;       /* competitive part: groups per wavefront that a worker claims from a
                                  block column at a time, 1..1024; 0 = default (two draws per wavefront) */
    int32_t threads_per_worker;/* workgroup size of the SpMV-part kernel: 256, 512, 1024; 0 = default */
    int32_t rounds_per_batch;  /* rounds a wavefront loads per group before accumulating: 2, 4, 8, 9, 16
                                  (2 and 4 walk 8 and 4 groups at once; fp64 with 1024 threads: 4 and 2);
                                  0 = chosen with R: 8 for long row segments, 4 for short ones        */
    int32_t slot_weight;       /* schedule weight of a slot, in nonzeros: 0..64; -1 = default 20 (2 when the groups
                                  average 512 nonzeros or more: see group_weight)                      */
    int32_t group_weight;      /* schedule weight of a group as such, in nonzeros: 0..4096; -1 = default 600: what a
                                  group costs a wavefront of the SpMV-part kernel next to a nonzero while loads are
                                  waited for anyway; 60 when the groups average 512 nonzeros or more and are
                                  streamed at the memory bandwidth (all four default weights are a tenth then) */
    int32_t combine_unit_slots;/* slots one workgroup of the combine part should get at most: a row block
                                  with more is cut into several units; >= 64; 0 = default: twice the
                                  mean number of slots per row block, at least 16384                 */
    int32_t round_weight;      /* schedule weight of one round of a group (its rounds = the length of
                                  its longest row), in nonzeros: 0..1024; -1 = default 100 (10)      */
    int32_t heavy_group_rounds;/* a group with a row of more nonzeros than this (inside the block) is walked
                                  by all wavefronts of its worker together, each taking an equal share of
                                  its nonzeros, instead of by one: >= 1; 0 = default 2048.  A group with a row of
                                  more than an eighth of this waits until the worker's other groups are done and
                                  is then walked by the next free wavefront                              */
    uint32_t flags;            /* HBP_FLAG_*                                                    */
    int32_t column_weight;     /* schedule weight of entering a block column (the worker fetches its segment
                                  of x), in nonzeros, charged to the column's first group when the group list
                                  is cut into the workers' ranges: 0..16777216; -1 = default 600000 (60000) */
} hbp_params_t;

typedef struct {
    int64_t n_rows, n_cols, nnz;
    int32_t rows_per_block, cols_per_block, group_width;
    int32_t hash_shift;          /* a (sampled or given); c = 2^a                               */
    int32_t hash_b;              /* b = d = max(1, R / 9)                                       */
    int64_t row_blocks, col_blocks;       /* NBR, NBC                                           */
    int64_t blocks, slots, groups;        /* B, S, G                                            */
    int32_t num_workers;         /* P                                                           */
    int32_t fixed_fraction_q8;   /* share of the work that is pre-assigned, in 1/256            */
    int32_t claim_chunk;
    int32_t threads_per_worker;  /* workgroup size of the SpMV-part kernel                      */
    int32_t rounds_per_batch;    /* rounds loaded per batch by the SpMV-part kernel             */
    int32_t slot_weight;         /* schedule weight of a slot, in nonzeros                      */
    int32_t group_weight;        /* schedule weight of a group as such, in nonzeros             */
    int32_t combine_unit_slots;  /* slots per combine unit the row blocks were cut for          */
    int32_t heavy_group_rounds;  /* row length from which a group is shared by a worker's wavefronts */
    int32_t round_weight;        /* schedule weight of a round of a group, in nonzeros          */
    int32_t column_weight;       /* schedule weight of entering a block column, in nonzeros      */
    int64_t combine_units;       /* U: workgroups of the combine part                           */
    int64_t split_row_blocks;    /* NM: row blocks cut into more than one unit                  */
    int32_t value_bytes;         /* 4: fp32 handle, 8: fp64 handle                              */
    int64_t first_ticket_block;  /* HBP_FLAG_PAPER_SCHEDULE: first block of the competitive part (P F); else -1 */
    int64_t bytes_layout;        /* device bytes of all layout arrays                           */
    int64_t bytes_spmv_part;     /* algorithmic bytes one SpMV-part launch moves                 */
    int64_t bytes_combine;       /* algorithmic bytes one combine launch moves                  */
    double build_ms;             /* wall time of hbp_build, allocation and synchronisation included */
} hbp_info_t;

/* ids for hbp_export */
typedef enum {
    HBP_ARRAY_BLK_BM = 0, HBP_ARRAY_BLK_BN = 1, HBP_ARRAY_SLOT_PTR = 2, HBP_ARRAY_BLK_GROUP_PTR = 3,
    HBP_ARRAY_COL_BLK_PTR = 4, HBP_ARRAY_STRIPE_PTR = 5, HBP_ARRAY_STRIPE_BLK = 6, HBP_ARRAY_GROUP_PTR = 7,
    HBP_ARRAY_GROUP_SLOT = 8, HBP_ARRAY_ROW_LOCAL = 9, HBP_ARRAY_SEG_LEN = 10, HBP_ARRAY_COL_LOCAL = 11,
    HBP_ARRAY_DATA = 12,
    HBP_ARRAY_ADD_SIGN = 13, /* int32 [nnz], derived on the device from seg_len when exported   */
    HBP_ARRAY_PARTIAL = 14,  /* float or double [S], per-slot partial sums of the last SpMV      */
    HBP_ARRAY_COL_GROUP_PTR = 15, HBP_ARRAY_COMP_LO = 16, HBP_ARRAY_FIXED_START = 17, HBP_ARRAY_FIXED_COL = 18,
    HBP_ARRAY_UNIT_PTR = 19, HBP_ARRAY_UNIT_STRIPE = 20, HBP_ARRAY_UNIT_K = 21, HBP_ARRAY_MULTI_STRIPES = 22,
    HBP_ARRAY_GROUP_ROUNDS = 23, HBP_ARRAY_COMP_COL = 24,
    HBP_ARRAY_SLOT_KEY = 25, /* uint32 [S], the key each slot was placed by; only with HBP_FLAG_KEEP_KEYS  */
    HBP_ARRAY_BLK_SHIFT = 26 /* int32 [B], the shift a each block's keys were taken with                  */
} hbp_array_id;

/* Fills *params with "chosen by the library" for everything (W = 64; validation on). */
int hbp_default_params(hbp_params_t *params /* HOST */);

/* Preprocessing: CSR -> HBP (Section 3.2: sampling of the shift a, data preparation of
 * Algorithm 2, hash reorder, format conversion; Section 3.3: fixed/competitive split).
 *   csr_ptr DEVICE int32 [n_rows+1], csr_ptr[0] = 0, non-decreasing;
 *   csr_col DEVICE int32 [nnz], strictly ascending inside each row, in [0, n_cols);
 *   csr_val DEVICE float [nnz];  params HOST or NULL for defaults;  *out HOST.
 * Runs on `stream`, synchronises it, and returns with the handle complete.  With
 * HBP_FLAG_VALIDATE a malformed column array yields HBP_ERR_BAD_CSR_COL; without it
 * out-of-range columns are still detected (never dereferenced), order is not checked.
 * nnz must be below 2^31 - 64 and NBR*NBC at most 2^27.  On error *out is NULL. */
int hbp_build(const int32_t *csr_ptr, const int32_t *csr_col, const float *csr_val,
              int64_t n_rows, int64_t n_cols, const hbp_params_t *params, void *stream, hbp_handle_t *out);

/* y = A x, exactly (alpha 1, beta 0; Algorithm 1 assigns).  Two-step SpMV of Fig. 1:
 * the SpMV part (Algorithm 3 per block; workers take their fixed blocks, then claim
 * competitive ones through an atomic ticket counter, Section 3.3) writes one partial sum
 * per slot; the combine part adds the partial sums of each row and writes y.
 *   x DEVICE float [n_cols], read only;  y DEVICE float [n_rows], overwritten (both kernels
 *   write it: x and y must not overlap).
 * Asynchronous on `stream`.  A handle supports one SpMV in flight at a time: calls on the
 * same stream serialise by themselves; calls on different streams must be ordered by the
 * caller (they share the partial-sum buffer and the ticket counter).  The call allocates
 * nothing and launches two kernels, no memset or copy: after one ordinary call on the device
 * (which configures the kernels) it may be recorded into a HIP graph by stream capture. */
int hbp_spmv(hbp_handle_t h, const float *x, float *y, void *stream);

/* The fp64 variant (Section 3.1 counts 8 bytes per stored value): hbp_build_f64 is hbp_build
 * with csr_val DEVICE double [nnz], and builds the same layout and schedule as hbp_build
 * would for the same pattern and parameters, with `data` in fp64 (R at most 4096 and C at
 * most 16384: the LDS copies of the x and y slices are twice as large).  hbp_spmv_f64 is
 * hbp_spmv with x DEVICE double [n_cols], y DEVICE double [n_rows]; products, partial sums
 * and the combine part are fp64. */
int hbp_build_f64(const int32_t *csr_ptr, const int32_t *csr_col, const double *csr_val,
                  int64_t n_rows, int64_t n_cols, const hbp_params_t *params, void *stream, hbp_handle_t *out);
int hbp_spmv_f64(hbp_handle_t h, const double *x, double *y, void *stream);

/* hbp_spmv for callers that cannot allocate device memory or must not touch memory the library
 * allocated for the handle's intermediates: code under HIP graph capture that replays on several
 * handles, tight serving loops, harnesses that forbid hipMalloc.  Same result as hbp_spmv (fp32
 * handles), but the per-slot partial sums and the claim counters of the call live in a fixed array
 * of the library (32 MiB per device, held until the process ends) instead of the handle's buffers:
 * 256 KiB of claim counters and at most 8,323,072 slots (S * 4 bytes <= 32 MiB - 256 KiB).  A handle
 * with more slots or more than 65536 workers is refused with HBP_ERR_TOO_LARGE.  The call allocates
 * nothing, launches three kernels (the first clears the counters), and is asynchronous on `stream`.
 * All calls on one device share the one array: calls that overlap in time on one device (different
 * streams, different handles) race and must be ordered by the caller. */
int hbp_spmv_static_scratch(hbp_handle_t h, const float *x, float *y, void *stream);

/* Frees the handle and its device arrays (synchronises the device first). NULL is allowed. */
int hbp_free(hbp_handle_t h);

/* Sizes, parameters and byte counts of a handle.  *info HOST. */
int hbp_get_info(hbp_handle_t h, hbp_info_t *info);

/* Copies one layout array to host memory (synchronous).  With host_dst NULL only the size
 * is reported.  *bytes_out HOST receives the array's size in bytes; capacity is the size
 * of host_dst, HBP_ERR_INVALID_ARGUMENT if it is too small. */
int hbp_export(hbp_handle_t h, int which, void *host_dst, size_t capacity, size_t *bytes_out);

/* Times `iters` back-to-back hbp_spmv calls with HIP events recorded on `stream` around
 * each of the two kernels.  HOST outputs: average milliseconds of the SpMV-part kernel,
 * of the combine kernel, and of a whole call (event before the first kernel to event
 * after the second).  Synchronises the stream. */
int hbp_spmv_timed(hbp_handle_t h, const float *x, float *y, void *stream, int iters,
                   float *ms_part, float *ms_combine, float *ms_total);
int hbp_spmv_timed_f64(hbp_handle_t h, const double *x, double *y, void *stream, int iters,
                       float *ms_part, float *ms_combine, float *ms_total);

/* In-repo CSR baselines (Algorithm 1; the mapping of rows to lanes is free).  kind 0: one thread per
 * row; kind 1: one wavefront (64 lanes) per row; kind 2, 4, 8, 16, 32: that many lanes per row, each
 * with a cross-lane reduction (pick the power of two nearest the mean row length).  Any other kind is
 * HBP_ERR_INVALID_ARGUMENT.  All pointers DEVICE; y overwritten. */
int hbp_csr_spmv(int kind, const int32_t *csr_ptr, const int32_t *csr_col, const float *csr_val,
                 const float *x, float *y, int64_t n_rows, void *stream);
int hbp_csr_spmv_f64(int kind, const int32_t *csr_ptr, const int32_t *csr_col, const double *csr_val,
                     const double *x, double *y, int64_t n_rows, void *stream);

/* The device's hash function on its own (Section 3.2: aggregation, dispersion, linear mapping):
 * keys[i] = key of a row with n[i] nonzeros inside its block, for shift a (0..12) and R rows per
 * block (1..8192), exactly as hbp_build computes it when it places that row.
 *   n DEVICE uint32 [count], keys DEVICE uint32 [count]; asynchronous on `stream`. */
int hbp_hash_keys(const uint32_t *n, int64_t count, int32_t a, int32_t rows_per_block, uint32_t *keys, void *stream);

/* hbp_build keeps its scratch memory (a few hundred megabytes for the large workloads, per
 * device) for the next build instead of freeing it: freeing costs a good part of a build.
 * Builds of one process therefore run one at a time.  This call gives the memory back (no build
 * may be running). */
int hbp_release_workspace(void);

const char *hbp_status_string(int status);
/* hipError_t of the most recent HBP_ERR_HIP on this thread, as int. */
int hbp_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HBP_H */
