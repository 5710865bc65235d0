/*
 * CPU oracle for the Hash-based Partition (HBP) SpMV path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, sequential, single-threaded C.  It shares no code, header, table or
 * helper with the HIP library and must never be reached from the product path:
 * only tests, the smoke check and the bench's cpu_baseline leg load it.
 *
 * What it computes, and the passage of the paper each part follows:
 *   - oracle_csr_spmv_f64      y = A x by the plain definition (Algorithm 1), fp64.
 *   - oracle_csr_spmv_f64_d    the same with the matrix and vector stored in fp64.
 *   - oracle_hash_key          the nonlinear hash = aggregation + dispersion + linear
 *                              mapping (Section 3.2; its figure with the formula is not
 *                              available, so the formula below is this build's reading).
 *   - oracle_sample_shift      the sampled shift a (Section 3.2, "most rows map to 0..8").
 *   - oracle_hbp_build         2D partition (Section 3.1), per-(row, column block) segment
 *                              discovery (Algorithm 2), hash reorder, warp-group
 *                              column-major fill with add_sign (Section 3.2, last
 *                              paragraph).  (The block schedule of Section 3.3 and the work
 *                              units of the combine part are in hbp_oracle_schedule.c: the
 *                              paper leaves them open, and nothing in this file depends on
 *                              them.)
 *   - oracle_hbp_spmv          the two-step SpMV through the layout: per-block walk via
 *                              add_sign (Algorithm 3, with the do-while reading of its
 *                              loop) then the combine of partial sums (Fig. 1), fp64.
 *   - oracle_hbp_to_coo        inverse of the format conversion.
 *
 * Values are stored as fp32 (value_bytes 4) or fp64 (value_bytes 8, the storage type of
 * Section 3.1's cost estimate); everything except the data array is the same for both,
 * and all arithmetic is fp64 either way.
 *
 * Layout produced ("compact" mode): only non-empty blocks and, inside a block, only
 * rows with at least one nonzero in it are stored.  Blocks are listed column-major
 * (column block bn ascending, then row block bm), which is the order the schedule of
 * Section 3.3 hands them to workers.  Inside a block, slots list rows in ascending
 * (hash key, local row) order: the deterministic limit of the paper's atomic hash-table
 * insertion.  W consecutive slots of a block form a group; a group's nonzeros are
 * stored round by round (round k = the k-th nonzero of every row that still has one).
 *
 * Parity status: y, segments, permutation, fill and add_sign are pinned by the tests under
 * tests/ (definitions, brute force, round trip, closed forms, a hand-worked 8x8 example).
 * The hash formula itself and the sampling quantile are NOT given by the paper (its figure
 * with the formula is not available): "parity unpinned" against the authors'
 * implementation; they are pinned only to this build's stated reading.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "hbp_oracle.h"

/* ------------------------------------------------------------------ Algorithm 1 */

/* y_ref[i] = sum_j (double)val[j] * (double)x[col[j]] over row i, in CSR order;
 * s_abs[i] = sum_j |val[j] * x[col[j]]| (the scale of the tolerance test). */
void oracle_csr_spmv_f64(const int32_t *ptr, const int32_t *col, const float *val, const float *x,
                         int64_t n_rows, double *y_ref, double *s_abs)
{
    for (int64_t i = 0; i < n_rows; i++) {
        double sum = 0.0, mag = 0.0;
        for (int64_t j = ptr[i]; j < ptr[i + 1]; j++) {
            double p = (double)val[j] * (double)x[col[j]];
            sum += p;
            mag += p < 0 ? -p : p;
        }
        y_ref[i] = sum;
        if (s_abs) s_abs[i] = mag;
    }
}

/* The same for fp64 storage (the paper's storage type, Section 3.1): val and x are doubles.
 * Products and sums are taken in long double (x87 extended, 64-bit significand, on the x86-64
 * hosts this runs on) and rounded to double once at the end, so that the reference is as far
 * above an fp64 path as the fp64 reference is above an fp32 path. */
void oracle_csr_spmv_f64_d(const int32_t *ptr, const int32_t *col, const double *val, const double *x,
                           int64_t n_rows, double *y_ref, double *s_abs)
{
    for (int64_t i = 0; i < n_rows; i++) {
        long double sum = 0.0L, mag = 0.0L;
        for (int64_t j = ptr[i]; j < ptr[i + 1]; j++) {
            long double p = (long double)val[j] * (long double)x[col[j]];
            sum += p;
            mag += p < 0 ? -p : p;
        }
        y_ref[i] = (double)sum;
        if (s_abs) s_abs[i] = (double)mag;
    }
}

/* ------------------------------------------------------------------ Section 3.2: hash */

/* b = d = max(1, floor(R / 9)): nine aggregation classes 0..8 spread over the R table
 * positions of one block ("b and d are fixed by the row-direction partition size"). */
static uint32_t hash_b(int32_t R) { uint32_t b = (uint32_t)R / 9u; return b ? b : 1u; }

/* key(n) for a row with n nonzeros inside the block:
 *   aggregation   agg  = min(n >> a, 8)          rows with similar n share a class; the
 *                                                 few rows above class 8 are treated as 8
 *   dispersion    disp = agg * b                 classes spread over the table
 *   linear map    lin  = ((n mod c) * d) >> a    c = 2^a; fine position inside a class
 *   key = min(disp + lin, R - 1)                 stays inside the block's table        */
uint32_t oracle_hash_key(uint32_t n, int32_t a, int32_t R)
{
    uint32_t b = hash_b(R), d = b, c = 1u << a;
    uint32_t agg = n >> a;
    if (agg > 8u) agg = 8u;
    uint32_t lin = ((n % c) * d) >> a;
    uint32_t key = agg * b + lin;
    if (key > (uint32_t)R - 1u) key = (uint32_t)R - 1u;
    return key;
}

/* keys[i] = oracle_hash_key(n[i], a, R): the same function over a vector of lengths. */
void oracle_hash_keys(const uint32_t *n, int64_t count, int32_t a, int32_t R, uint32_t *keys)
{
    for (int64_t i = 0; i < count; i++) keys[i] = oracle_hash_key(n[i], a, R);
}

/* Walk one row and call back once per segment (maximal run of nonzeros whose columns
 * fall in the same column block), left to right as Algorithm 2 does, with the row-end
 * guard its inner loop lacks. */
typedef void (*seg_fn)(void *ctx, int64_t row, int64_t bn, int64_t j0, int64_t n);
static void for_each_segment(const int32_t *ptr, const int32_t *col, int64_t row, int32_t C, seg_fn fn, void *ctx)
{
    int64_t j = ptr[row], end = ptr[row + 1];
    while (j < end) {
        int64_t bn = col[j] / C, j0 = j;
        while (j < end && col[j] < (bn + 1) * (int64_t)C) j++;
        fn(ctx, row, bn, j0, j - j0);
    }
}

typedef struct { int64_t total; int64_t below[13]; } sample_ctx;
static void sample_seg(void *vctx, int64_t row, int64_t bn, int64_t j0, int64_t n)
{
    (void)row; (void)bn; (void)j0;
    sample_ctx *s = (sample_ctx *)vctx;
    s->total++;
    for (int a = 0; a <= 12; a++)
        if (n < (int64_t)9 << a) s->below[a]++;
}

/* Sampled shift a: look at S = min(n_rows, 4096) evenly spaced rows r_k = floor(k n_rows / S);
 * a is the smallest value in 0..12 for which at least 15/16 of the sampled segments
 * aggregate into 0..8, i.e. have n < 9 * 2^a.  a = 0 when nothing was sampled. */
int32_t oracle_sample_shift(const int32_t *ptr, const int32_t *col, int64_t n_rows, int32_t C)
{
    sample_ctx s;
    memset(&s, 0, sizeof s);
    int64_t S = n_rows < 4096 ? n_rows : 4096;
    for (int64_t k = 0; k < S; k++) for_each_segment(ptr, col, (k * n_rows) / S, C, sample_seg, &s);
    if (s.total == 0) return 0;
    for (int a = 0; a <= 12; a++)
        if (16 * s.below[a] >= 15 * s.total) return a;
    return 12;
}

/* ------------------------------------------------------------------ the layout */


typedef struct { int64_t *cnt; int64_t NBR; int32_t R; } count_ctx;
static void count_seg(void *vctx, int64_t row, int64_t bn, int64_t j0, int64_t n)
{
    (void)j0; (void)n;
    count_ctx *c = (count_ctx *)vctx;
    c->cnt[bn * c->NBR + row / c->R]++;
}

typedef struct { int64_t *cursor; int64_t NBR; int32_t R; int32_t *q, *n, *j; } place_ctx;
static void place_seg(void *vctx, int64_t row, int64_t bn, int64_t j0, int64_t n)
{
    place_ctx *p = (place_ctx *)vctx;
    int64_t pos = p->cursor[bn * p->NBR + row / p->R]++;
    p->q[pos] = (int32_t)(row % p->R);
    p->n[pos] = (int32_t)n;
    p->j[pos] = (int32_t)j0;
}

void oracle_hbp_free(oracle_hbp *h)
{
    if (!h) return;
    free(h->blk_bm); free(h->blk_bn); free(h->slot_ptr); free(h->blk_group_ptr); free(h->col_blk_ptr);
    free(h->stripe_ptr); free(h->stripe_blk); free(h->group_ptr); free(h->group_rounds); free(h->group_slot);
    free(h->row_local); free(h->seg_len); free(h->slot_key); free(h->blk_shift); free(h->col_local); free(h->data); free(h->data64); free(h->add_sign); free(h->col_group_ptr); free(h->comp_lo); free(h->comp_col); free(h->fixed_start); free(h->fixed_col);
    free(h->unit_ptr); free(h->unit_stripe); free(h->unit_k); free(h->multi_stripes);
    free(h);
}

/* Build the compact layout.  hash_shift = -1 samples a; hash_shift = -2 also switches the reorder off (the plain
 * 2D-partitioning method the paper compares with in Section 4: slots of a block in ascending row order);
 * hash_shift = -3 replaces the hash key by the row's length inside the block itself (the limit of an ever finer
 * linear mapping, Section 5's "room for improvement in the hash function": rows of a block in ascending
 * (length, row) order, which no hash of the length can improve on);
 * hash_shift = -4 takes the shift per block instead of per matrix (Section 3.2: "as matrix blocks become denser,
 * the value of a will increase"): a block's a is the smallest value in 0..12 for which at least 15/16 of the
 * block's own segments have n < 9 * 2^a -- the rule of the sampled shift applied to all rows of the block.
 * Returns NULL on invalid parameters (R in 1..65536, C in 1..65535, W >= 1).  The schedule arrays and the
 * combine units are filled in by oracle_hbp_schedule / oracle_hbp_units (hbp_oracle_schedule.c). */
oracle_hbp *oracle_hbp_build(const int32_t *ptr, const int32_t *col, const void *val, int32_t value_bytes, int64_t n_rows, int64_t n_cols,
                             int32_t R, int32_t C, int32_t W, int32_t hash_shift)
{
    if (R < 1 || R > 65536 || C < 1 || C > 65535 || W < 1 || n_rows < 1 || n_cols < 1 || (value_bytes != 4 && value_bytes != 8)) return NULL;
    oracle_hbp *h = (oracle_hbp *)calloc(1, sizeof *h);
    h->n_rows = n_rows; h->n_cols = n_cols; h->nnz = ptr[n_rows];
    h->R = R; h->C = C; h->W = W;
    h->a = hash_shift >= 0 ? hash_shift : oracle_sample_shift(ptr, col, n_rows, C);
    const int plain = hash_shift == -2;  /* plain 2D partition: no reorder, every row gets key 0 */
    const int by_length = hash_shift == -3;  /* key = length of the row inside the block (at most C < 65536) */
    const int per_block = hash_shift == -4;  /* the shift is taken from the block's own segment lengths */
    const int64_t n_keys = by_length ? 65536 : R;
    int32_t a_blk = h->a;                    /* shift of the block being ordered */
#define ORACLE_KEY(n) (plain ? 0u : by_length ? (uint32_t)(n) : oracle_hash_key((uint32_t)(n), a_blk, R))
    int64_t NBR = (n_rows + R - 1) / R, NBC = (n_cols + C - 1) / C;
    h->NBR = NBR; h->NBC = NBC;

    /* pass 1: how many rows of each block hold a nonzero in it */
    int64_t *cnt = (int64_t *)calloc((size_t)(NBR * NBC), sizeof(int64_t));
    count_ctx cc = { cnt, NBR, R };
    for (int64_t r = 0; r < n_rows; r++) for_each_segment(ptr, col, r, C, count_seg, &cc);

    /* non-empty blocks in column-major order, their slot and group ranges */
    int64_t B = 0, S = 0, G = 0;
    for (int64_t d = 0; d < NBR * NBC; d++) if (cnt[d]) { B++; S += cnt[d]; G += (cnt[d] + W - 1) / W; }
    h->B = B; h->S = S; h->G = G;
    h->blk_bm = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B + 1));
    h->blk_bn = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B + 1));
    h->slot_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B + 1));
    h->blk_group_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B + 1));
    h->col_blk_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NBC + 1));
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)(NBR * NBC));
    int64_t *compact_id = (int64_t *)malloc(sizeof(int64_t) * (size_t)(NBR * NBC));
    {
        int64_t b = 0, s = 0, g = 0;
        for (int64_t bn = 0; bn < NBC; bn++) {
            h->col_blk_ptr[bn] = (int32_t)b;
            for (int64_t bm = 0; bm < NBR; bm++) {
                int64_t d = bn * NBR + bm;
                cursor[d] = s;
                compact_id[d] = -1;
                if (!cnt[d]) continue;
                compact_id[d] = b;
                h->blk_bm[b] = (int32_t)bm; h->blk_bn[b] = (int32_t)bn;
                h->slot_ptr[b] = (int32_t)s; h->blk_group_ptr[b] = (int32_t)g;
                s += cnt[d]; g += (cnt[d] + W - 1) / W; b++;
            }
        }
        h->col_blk_ptr[NBC] = (int32_t)b;
        h->slot_ptr[B] = (int32_t)s; h->blk_group_ptr[B] = (int32_t)g;
    }

    /* pass 2: gather each block's rows; visiting rows in ascending order leaves every
     * block's list sorted by local row */
    int32_t *tq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    int32_t *tn = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    int32_t *tj = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    place_ctx pc = { cursor, NBR, R, tq, tn, tj };
    for (int64_t r = 0; r < n_rows; r++) for_each_segment(ptr, col, r, C, place_seg, &pc);

    /* hash reorder: stable counting sort of each block's rows by key */
    h->row_local = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(S + 1));
    h->seg_len = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(S + 1));
    int32_t *slot_j = (int32_t *)malloc(sizeof(int32_t) * (size_t)(S + 1));
    int64_t *table = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_keys + 1));
    h->slot_key = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(S + 1));
    h->blk_shift = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B + 1));
    for (int64_t b = 0; b < B; b++) {
        int64_t s0 = h->slot_ptr[b], s1 = h->slot_ptr[b + 1];
        if (per_block) {   /* smallest a with 16 #{n < 9 2^a} >= 15 #{segments of the block} */
            a_blk = 12;
            for (int a = 0; a <= 12; a++) {
                int64_t below = 0;
                for (int64_t s = s0; s < s1; s++) if (tn[s] < (int64_t)9 << a) below++;
                if (16 * below >= 15 * (s1 - s0)) { a_blk = a; break; }
            }
        }
        h->blk_shift[b] = a_blk;
        int64_t used = 0;  /* keys 0 .. used-1 occur in this block */
        for (int64_t s = s0; s < s1; s++) if ((int64_t)ORACLE_KEY(tn[s]) >= used) used = (int64_t)ORACLE_KEY(tn[s]) + 1;
        memset(table, 0, sizeof(int64_t) * (size_t)(used + 1));
        for (int64_t s = s0; s < s1; s++) table[ORACLE_KEY(tn[s]) + 1]++;
        for (int64_t k = 0; k < used; k++) table[k + 1] += table[k];
        for (int64_t s = s0; s < s1; s++) {   /* ascending local row */
            int64_t slot = s0 + table[ORACLE_KEY(tn[s])]++;
            h->row_local[slot] = (uint16_t)tq[s];
            h->seg_len[slot] = (uint16_t)tn[s];
            h->slot_key[slot] = ORACLE_KEY(tn[s]);
            slot_j[slot] = tj[s];
        }
    }
#undef ORACLE_KEY

    /* format conversion: groups of W slots, round-by-round fill, add_sign */
    h->group_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(G + 1));
    h->group_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)(G + 1));
    h->col_local = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(h->nnz + 1));
    h->value_bytes = value_bytes;
    if (value_bytes == 4) h->data = (float *)malloc(sizeof(float) * (size_t)(h->nnz + 1));
    else h->data64 = (double *)malloc(sizeof(double) * (size_t)(h->nnz + 1));
    h->add_sign = (int32_t *)malloc(sizeof(int32_t) * (size_t)(h->nnz + 1));
    {
        int64_t pos = 0, g = 0;
        for (int64_t b = 0; b < B; b++) {
            int64_t col0 = (int64_t)h->blk_bn[b] * C;
            for (int64_t s0 = h->slot_ptr[b]; s0 < h->slot_ptr[b + 1]; s0 += W, g++) {
                int64_t s1 = s0 + W < h->slot_ptr[b + 1] ? s0 + W : h->slot_ptr[b + 1];
                h->group_ptr[g] = (int32_t)pos; h->group_slot[g] = (int32_t)s0;
                int64_t live = 0;   /* rows of the group that still have nonzeros to store */
                for (int64_t s = s0; s < s1; s++) if (h->seg_len[s] > 0) live++;
                for (int64_t k = 0; live > 0; k++) {
                    for (int64_t s = s0; s < s1; s++) {
                        if (k >= h->seg_len[s]) continue;
                        h->col_local[pos] = (uint16_t)(col[slot_j[s] + k] - col0);
                        if (value_bytes == 4) h->data[pos] = ((const float *)val)[slot_j[s] + k];
                        else h->data64[pos] = ((const double *)val)[slot_j[s] + k];
                        if (k + 1 == h->seg_len[s]) { h->add_sign[pos] = -1; live--; }
                        else h->add_sign[pos] = (int32_t)live;
                        pos++;
                    }
                }
            }
        }
        h->group_ptr[G] = (int32_t)pos; h->group_slot[G] = (int32_t)S;
    }

    /* combine index: for each row block, its non-empty blocks with bn ascending */
    h->stripe_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NBR + 1));
    h->stripe_blk = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B + 1));
    {
        int64_t k = 0;
        for (int64_t bm = 0; bm < NBR; bm++) {
            h->stripe_ptr[bm] = (int32_t)k;
            for (int64_t bn = 0; bn < NBC; bn++)
                if (compact_id[bn * NBR + bm] >= 0) h->stripe_blk[k++] = (int32_t)compact_id[bn * NBR + bm];
        }
        h->stripe_ptr[NBR] = (int32_t)k;
    }

    h->first_ticket_block = -1;
    free(cnt); free(cursor); free(compact_id); free(tq); free(tn); free(tj); free(slot_j); free(table);
    return h;
}

/* dims[0..16] = n_rows n_cols nnz R C W a NBR NBC B S G P fixed_q8 U NM first_ticket_block */
void oracle_hbp_dims(const oracle_hbp *h, int64_t *dims)
{
    int64_t v[17] = { h->n_rows, h->n_cols, h->nnz, h->R, h->C, h->W, h->a, h->NBR, h->NBC, h->B, h->S, h->G, h->P, h->fixed_q8,
                      h->U, h->NM, h->first_ticket_block };
    memcpy(dims, v, sizeof v);
}

/* which: 0 blk_bm 1 blk_bn 2 slot_ptr 3 blk_group_ptr 4 col_blk_ptr 5 stripe_ptr 6 stripe_blk
 *        7 group_ptr 8 group_slot 9 row_local 10 seg_len 11 col_local 12 data 13 add_sign
 *        14 col_group_ptr 15 comp_lo 16 fixed_start 17 fixed_col
 *        18 unit_ptr 19 unit_stripe 20 unit_k 21 multi_stripes 22 group_rounds 23 comp_col
 *        24 slot_key 25 blk_shift.
 * Copies the array into dst and returns its size in bytes (0 for an unknown id). */
int64_t oracle_hbp_copy(const oracle_hbp *h, int32_t which, void *dst)
{
    const void *src = NULL; int64_t bytes = 0;
    switch (which) {
    case 0: src = h->blk_bm; bytes = 4 * h->B; break;
    case 1: src = h->blk_bn; bytes = 4 * h->B; break;
    case 2: src = h->slot_ptr; bytes = 4 * (h->B + 1); break;
    case 3: src = h->blk_group_ptr; bytes = 4 * (h->B + 1); break;
    case 4: src = h->col_blk_ptr; bytes = 4 * (h->NBC + 1); break;
    case 5: src = h->stripe_ptr; bytes = 4 * (h->NBR + 1); break;
    case 6: src = h->stripe_blk; bytes = 4 * h->B; break;
    case 7: src = h->group_ptr; bytes = 4 * (h->G + 1); break;
    case 8: src = h->group_slot; bytes = 4 * (h->G + 1); break;
    case 9: src = h->row_local; bytes = 2 * h->S; break;
    case 10: src = h->seg_len; bytes = 2 * h->S; break;
    case 11: src = h->col_local; bytes = 2 * h->nnz; break;
    case 12: src = h->value_bytes == 4 ? (const void *)h->data : (const void *)h->data64; bytes = h->value_bytes * h->nnz; break;
    case 13: src = h->add_sign; bytes = 4 * h->nnz; break;
    case 14: src = h->col_group_ptr; bytes = 4 * (h->NBC + 1); break;
    case 15: src = h->comp_lo; bytes = 4 * h->P; break;
    case 16: src = h->fixed_start; bytes = 4 * (h->P + 1); break;
    case 17: src = h->fixed_col; bytes = 4 * h->P; break;
    case 18: src = h->unit_ptr; bytes = 4 * (h->NBR + 1); break;
    case 19: src = h->unit_stripe; bytes = 4 * h->U; break;
    case 20: src = h->unit_k; bytes = 4 * (h->U + 1); break;
    case 21: src = h->multi_stripes; bytes = 4 * h->NM; break;
    case 22: src = h->group_rounds; bytes = 4 * (h->G + 1); break;
    case 23: src = h->comp_col; bytes = 4 * h->P; break;
    case 24: src = h->slot_key; bytes = 4 * h->S; break;
    case 25: src = h->blk_shift; bytes = 4 * h->B; break;
    default: return 0;
    }
    if (dst && bytes) memcpy(dst, src, (size_t)bytes);
    return bytes;
}

/* Two-step SpMV through the layout, fp64.  SpMV part (Algorithm 3): the lane of slot s in
 * group g starts at group_ptr[g] + (s - group_slot[g]) (no empty slots in compact mode,
 * so the zero_row correction is 0) and walks its row with add_sign, accumulating then
 * stopping once add_sign is negative.  partial[s] is the block's contribution to row
 * bm*R + row_local[s].  Combine part: partial sums of a row are added with bn ascending.
 * partial_abs (may be NULL): the sum of the absolute products of each slot, the scale of a
 * tolerance test on the partial sums. */
void oracle_hbp_spmv(const oracle_hbp *h, const void *x_any, double *partial, double *y, double *partial_abs)
{
    for (int64_t b = 0; b < h->B; b++) {
        const int64_t x0 = (int64_t)h->blk_bn[b] * h->C;   /* start of the block's vector segment */
        for (int64_t g = h->blk_group_ptr[b]; g < h->blk_group_ptr[b + 1]; g++) {
            for (int64_t s = h->group_slot[g]; s < h->group_slot[g + 1]; s++) {
                int64_t j = h->group_ptr[g] + (s - h->group_slot[g]);
                double sum = 0.0, mag = 0.0;
                int32_t step;
                do {
                    double prod = h->value_bytes == 4 ? (double)h->data[j] * (double)((const float *)x_any)[x0 + h->col_local[j]]
                                                      : h->data64[j] * ((const double *)x_any)[x0 + h->col_local[j]];
                    sum += prod;
                    mag += prod < 0 ? -prod : prod;
                    step = h->add_sign[j];
                    j += step;
                } while (step > 0);
                partial[s] = sum;
                if (partial_abs) partial_abs[s] = mag;
            }
        }
    }
    for (int64_t i = 0; i < h->n_rows; i++) y[i] = 0.0;
    for (int64_t bm = 0; bm < h->NBR; bm++)
        for (int64_t k = h->stripe_ptr[bm]; k < h->stripe_ptr[bm + 1]; k++) {
            int64_t b = h->stripe_blk[k];
            for (int64_t s = h->slot_ptr[b]; s < h->slot_ptr[b + 1]; s++)
                y[bm * h->R + h->row_local[s]] += partial[s];
        }
}

/* Inverse of the conversion: every stored nonzero as (row, global column, value), in
 * storage order. */
void oracle_hbp_to_coo(const oracle_hbp *h, int64_t *rows, int64_t *cols, void *vals)
{
    for (int64_t b = 0; b < h->B; b++)
        for (int64_t g = h->blk_group_ptr[b]; g < h->blk_group_ptr[b + 1]; g++)
            for (int64_t s = h->group_slot[g]; s < h->group_slot[g + 1]; s++) {
                int64_t j = h->group_ptr[g] + (s - h->group_slot[g]);
                for (;;) {
                    rows[j] = (int64_t)h->blk_bm[b] * h->R + h->row_local[s];
                    cols[j] = (int64_t)h->blk_bn[b] * h->C + h->col_local[j];
                    if (h->value_bytes == 4) ((float *)vals)[j] = h->data[j];
                    else ((double *)vals)[j] = h->data64[j];
                    if (h->add_sign[j] < 0) break;
                    j += h->add_sign[j];
                }
            }
}
