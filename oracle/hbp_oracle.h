/*
 * Shared declarations of the CPU oracle (TEST INFRASTRUCTURE ONLY; see hbp_oracle.c).
 *
 * hbp_oracle.c           what the paper defines: Algorithm 1, the hash, the sampled shift, the
 *                        2D partition, Algorithm 2's segments, the hash reorder, the column-major
 *                        fill with add_sign, Algorithm 3's walk, the combine, HBP -> COO.
 * hbp_oracle_schedule.c  what Section 3.3 leaves open and this build (or the reading of the
 *                        paper's own sentence) fills in: who walks which block or group, and
 *                        how the combine part is cut into work units.
 * The second file reads the layout the first one built and never changes it.
 */
#ifndef HBP_ORACLE_H
#define HBP_ORACLE_H

#include <stdint.h>

typedef struct {
    int64_t n_rows, n_cols, nnz;
    int32_t R, C, W, a;
    int64_t NBR, NBC;   /* row blocks, column blocks */
    int64_t B, S, G;    /* non-empty blocks, slots (= segments), groups */
    int64_t P, fixed_q8; /* workers, share of the work that is pre-assigned in 1/256 (Section 3.3) */
    int32_t *blk_bm, *blk_bn;     /* B   : block coordinates, column-major order          */
    int32_t *slot_ptr;            /* B+1 : first slot of each block                        */
    int32_t *blk_group_ptr;       /* B+1 : first group of each block                       */
    int32_t *col_blk_ptr;         /* NBC+1 : first block of each block column              */
    int32_t *stripe_ptr;          /* NBR+1 : per row block, range into stripe_blk          */
    int32_t *stripe_blk;          /* B   : blocks of a row block, bn ascending             */
    int32_t *group_ptr;           /* G+1 : position of a group's first nonzero (begin_ptr) */
    int32_t *group_rounds;        /* G+1 : rounds of all groups before (a group's rounds = its longest row) */
    int32_t *group_slot;          /* G+1 : a group's first slot                            */
    uint16_t *row_local;          /* S   : slot -> row inside its block (output_hash)      */
    uint16_t *seg_len;            /* S   : nonzeros of that row inside the block           */
    uint32_t *slot_key;           /* S   : the key the row was placed by (hash of seg_len; 0 or seg_len in the study modes) */
    int32_t *blk_shift;           /* B   : the shift a the keys of a block were taken with  */
    uint16_t *col_local;          /* nnz : column inside the block's column range          */
    float *data;                  /* nnz (fp32 storage)                                    */
    double *data64;               /* nnz (fp64 storage); exactly one of data / data64 is set */
    int32_t value_bytes;          /* 4 or 8                                                */
    int32_t *add_sign;            /* nnz : distance to the row's next nonzero, -1 at its end */
    /* ---- filled by hbp_oracle_schedule.c ---- */
    int32_t schedule_mode;        /* 0: ranges of equal weight, 1: the paper's equal block counts */
    int64_t first_ticket_block;   /* mode 1: first block of the competitive part (P F); -1 otherwise */
    int32_t *col_group_ptr;       /* NBC+1 : first group of each block column                 */
    int32_t *comp_lo;             /* P   : first competitive group of a worker's range          */
    int32_t *comp_col;            /* P   : block column that holds the range's competitive groups */
    int32_t *fixed_start;         /* P+1 : group ranges of the workers                        */
    int32_t *fixed_col;           /* P   : block column holding a worker's first group        */
    int64_t U, NM;                /* combine units, row blocks cut into more than one unit    */
    int32_t *unit_ptr;            /* NBR+1 : units of each row block                          */
    int32_t *unit_stripe;         /* U   : row block of a unit                                */
    int32_t *unit_k;              /* U+1 : first stripe_blk entry of a unit                   */
    int32_t *multi_stripes;       /* NM  : row blocks with more than one unit, ascending      */
} oracle_hbp;

uint32_t oracle_hash_key(uint32_t n, int32_t a, int32_t R);

#endif
