/*
 * CPU oracle, second part: the schedule of Section 3.3 and the work units of the combine part.
 * TEST INFRASTRUCTURE ONLY (see hbp_oracle.c).
 *
 * Section 3.3 ("mixed execution allocation") gives the principle only: the blocks are divided
 * into a fixed part, pre-assigned to the warps in equal numbers with blocks of the same column
 * kept together, and a competitive part, claimed one at a time through a ticket lock.  It states
 * neither the ratio nor the number of warps.  Two readings are built here, both from a layout
 * that oracle_hbp_build has finished and that this file only reads:
 *
 *   mode 1, the paper's sentence taken literally: units are blocks, in the layout's column-major
 *           order; F = floor(B * fixed_q8 / (256 * P)) blocks per worker, worker w owns blocks
 *           [w F, (w + 1) F); blocks [P F, B) are the competitive part, claimed in list order,
 *           one ticket per block.
 *   mode 0, this build's own schedule (units are groups, ranges of equal weight, a competitive
 *           tail per range): what the library uses by default.  Its definition follows no
 *           passage of the paper beyond the principle above.
 *
 * y does not depend on either (beyond the order of additions).  "Parity unpinned": the paper
 * prints no schedule to compare with; the tests pin these arrays to their definitions here.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "hbp_oracle.h"

static void free_schedule(oracle_hbp *h)
{
    free(h->group_rounds); free(h->col_group_ptr); free(h->comp_lo); free(h->comp_col); free(h->fixed_start); free(h->fixed_col);
    h->group_rounds = h->col_group_ptr = h->comp_lo = h->comp_col = h->fixed_start = h->fixed_col = NULL;
}

/* Fills group_rounds, col_group_ptr, fixed_start, fixed_col, comp_lo, comp_col (and first_ticket_block).
 * Returns 0, or -1 on invalid parameters. */
int32_t oracle_hbp_schedule(oracle_hbp *h, int64_t num_workers, int32_t fixed_q8, int32_t slot_weight, int32_t round_weight,
                            int32_t group_weight, int32_t column_weight, int32_t mode)
{
    if (!h || num_workers < 1 || fixed_q8 < 0 || fixed_q8 > 256 || slot_weight < 0 || round_weight < 0 || group_weight < 0 ||
        column_weight < 0 || (mode != 0 && mode != 1))
        return -1;
    free_schedule(h);
    const int64_t G = h->G, NBC = h->NBC, B = h->B;
    h->schedule_mode = mode;
    h->first_ticket_block = -1;
    h->P = num_workers; h->fixed_q8 = fixed_q8;

    /* a group's rounds = the length of its longest row: the steps a wavefront takes through it */
    h->group_rounds = (int32_t *)malloc(sizeof(int32_t) * (size_t)(G + 1));
    h->group_rounds[0] = 0;
    for (int64_t g = 0; g < G; g++) {
        int32_t longest = 0;
        for (int64_t q = h->group_slot[g]; q < h->group_slot[g + 1]; q++)
            if (h->seg_len[q] > longest) longest = h->seg_len[q];
        h->group_rounds[g + 1] = h->group_rounds[g] + longest;
    }
    h->col_group_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NBC + 1));
    h->comp_lo = (int32_t *)malloc(sizeof(int32_t) * (size_t)(num_workers + 1));
    h->comp_col = (int32_t *)malloc(sizeof(int32_t) * (size_t)(num_workers + 1));
    h->fixed_start = (int32_t *)malloc(sizeof(int32_t) * (size_t)(num_workers + 1));
    h->fixed_col = (int32_t *)malloc(sizeof(int32_t) * (size_t)(num_workers + 1));
    for (int64_t c = 0; c <= NBC; c++) h->col_group_ptr[c] = h->blk_group_ptr[h->col_blk_ptr[c]];

    if (mode == 1) {
        /* Section 3.3 read literally: equal numbers of blocks, the rest behind one ticket counter.
         * The ranges are handed over in the units the kernels walk (groups): worker w's range is
         * the groups of its F blocks; nothing inside a range is left to competition. */
        const int64_t F = (B * (int64_t)fixed_q8) / (256 * num_workers);
        h->first_ticket_block = num_workers * F;
        for (int64_t w = 0; w <= num_workers; w++) {
            const int64_t b = w * F;   /* <= P F <= B */
            h->fixed_start[w] = h->blk_group_ptr[b];
        }
        for (int64_t w = 0; w < num_workers; w++) {
            const int64_t b = w * F;
            h->fixed_col[w] = b < B ? h->blk_bn[b] : (int32_t)(NBC - 1);   /* column of the range's first block */
            h->comp_lo[w] = h->fixed_start[w + 1];
            int64_t last = (w + 1) * F - 1;                                /* column of its last block */
            h->comp_col[w] = F > 0 ? h->blk_bn[last] : h->fixed_col[w];
        }
        return 0;
    }

    /* Mode 0.  The unit handed to a wavefront is a group; the weight of a group is group_weight plus
     * its nonzeros plus slot_weight times its slots plus round_weight times its rounds, so
     * Wt(g) = group_ptr[g] + slot_weight * group_slot[g] + round_weight * group_rounds[g] + group_weight * g
     * is the weight of all groups before g.
     *   - the group list is cut into P contiguous ranges of equal weight, fixed_start[w] being
     *     the first group of worker w; a worker runs the fixed groups inside its range and then
     *     competes, starting with the column it is on.  For this cut a block column weighs
     *     column_weight on top of its groups (a worker that enters it has to fetch its segment of
     *     the vector), charged to the column's first group: the weight before g is
     *     Wt(g) + column_weight * (number of non-empty block columns that start before g);
     *   - every range keeps the first fixed_q8/256 of its weight as its fixed part and leaves
     *     the rest to competition, as far as that rest lies in the range's last block column (so
     *     that whoever takes it needs one segment of the vector): comp_lo[w] is the range's
     *     first competitive group, comp_col[w] that block column. */
    #define WT(g) ((int64_t)h->group_ptr[g] + (int64_t)slot_weight * (int64_t)h->group_slot[g] + (int64_t)round_weight * (int64_t)h->group_rounds[g] + (int64_t)group_weight * (int64_t)(g))
    {
        /* entered[g]: non-empty block columns whose first group lies before g */
        int64_t *entered = (int64_t *)calloc((size_t)(G + 2), sizeof(int64_t));
        for (int64_t c = 0; c < NBC; c++)
            if (h->col_group_ptr[c + 1] > h->col_group_ptr[c]) entered[h->col_group_ptr[c] + 1]++;
        for (int64_t g = 0; g <= G; g++) entered[g + 1] += entered[g];
        #define WTC(g) (WT(g) + (int64_t)column_weight * entered[g])
        int64_t g = 0, c = 0;
        for (int64_t w = 0; w <= num_workers; w++) {
            while (g < G && WTC(g) * num_workers < w * WTC(G)) g++;
            h->fixed_start[w] = (int32_t)g;
            if (w == num_workers) break;
            while (c + 1 < NBC && h->col_group_ptr[c + 1] <= g) c++;   /* last column starting at or before g */
            h->fixed_col[w] = (int32_t)c;
        }
        #undef WTC
        free(entered);
    }
    for (int64_t w = 0; w < num_workers; w++) {
        int64_t g0 = h->fixed_start[w], g1 = h->fixed_start[w + 1], g = g0, c = h->fixed_col[w];
        while (g < g1 && (WT(g) - WT(g0)) * 256 < (WT(g1) - WT(g0)) * (int64_t)fixed_q8) g++;
        if (g1 > g0) {
            c = 0;
            while (c + 1 < NBC && h->col_group_ptr[c + 1] <= g1 - 1) c++;   /* column of the range's last group */
            if (g < h->col_group_ptr[c]) g = h->col_group_ptr[c];
        }
        h->comp_lo[w] = (int32_t)g;
        h->comp_col[w] = (int32_t)c;
    }
    #undef WT
    return 0;
}

/* Work units of the combine part (Fig. 1 leaves open which partial sums one task adds up).  A row
 * block with many slots is cut into u = ceil(slots / unit_slots) units of consecutive stripe_blk
 * entries; unit i starts at the first entry whose preceding slots, times u, reach i times the row
 * block's slots.  Returns 0, or -1 on invalid parameters. */
int32_t oracle_hbp_units(oracle_hbp *h, int32_t unit_slots)
{
    if (!h || unit_slots < 1) return -1;
    free(h->unit_ptr); free(h->unit_stripe); free(h->unit_k); free(h->multi_stripes);
    const int64_t B = h->B, NBR = h->NBR;
    int64_t *cum = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B + 1));
    cum[0] = 0;
    for (int64_t k = 0; k < B; k++) {
        int64_t b = h->stripe_blk[k];
        cum[k + 1] = cum[k] + (h->slot_ptr[b + 1] - h->slot_ptr[b]);
    }
    h->unit_ptr = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NBR + 1));
    int64_t U = 0, NM = 0;
    for (int64_t bm = 0; bm < NBR; bm++) {
        int64_t slots = cum[h->stripe_ptr[bm + 1]] - cum[h->stripe_ptr[bm]];
        int64_t u = (slots + unit_slots - 1) / unit_slots;
        if (u < 1) u = 1;
        h->unit_ptr[bm] = (int32_t)U;
        U += u;
        if (u > 1) NM++;
    }
    h->unit_ptr[NBR] = (int32_t)U;
    h->U = U; h->NM = NM;
    h->unit_stripe = (int32_t *)malloc(sizeof(int32_t) * (size_t)(U + 1));
    h->unit_k = (int32_t *)malloc(sizeof(int32_t) * (size_t)(U + 1));
    h->multi_stripes = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NM + 1));
    int64_t nm = 0;
    for (int64_t bm = 0; bm < NBR; bm++) {
        int64_t k0 = h->stripe_ptr[bm], k1 = h->stripe_ptr[bm + 1];
        int64_t slots = cum[k1] - cum[k0], u = h->unit_ptr[bm + 1] - h->unit_ptr[bm];
        int64_t k = k0;
        for (int64_t i = 0; i < u; i++) {
            while (k < k1 && (cum[k] - cum[k0]) * u < i * slots) k++;
            h->unit_stripe[h->unit_ptr[bm] + i] = (int32_t)bm;
            h->unit_k[h->unit_ptr[bm] + i] = (int32_t)k;
        }
        if (u > 1) h->multi_stripes[nm++] = (int32_t)bm;
    }
    h->unit_k[U] = (int32_t)B;
    free(cum);
    return 0;
}
