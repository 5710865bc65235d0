// HBP preprocessing on the GPU: CSR -> compact HBP layout (Sections 3.1-3.3 of the paper).
//
// The paper's Algorithm 2 walks one matrix row per thread and inserts rows into a per-block
// hash table with atomics.  Here the same quantities are produced with coalesced passes
// over the CSR arrays and a deterministic placement:
//   1. row-start bits      one bit per nonzero marking the first nonzero of a row
//   2. segment flags       a nonzero starts a segment when it starts a row or its column
//                          block differs from its left neighbour's (Algorithm 2's inner
//                          while loop, evaluated for all nonzeros at once)
//   3. segment records     (first nonzero, row, column block) in CSR order via a scan
//   4. block table         count of segments per (column block, row block); scans give each
//                          non-empty block its slot range, group range and list position
//   5. bucketed scatter    every segment drops (hash key, local row, segment id) into its
//                          block's slot range through an atomic cursor
//   6. block ordering      each block's range is ordered by (key, local row) in LDS; the
//                          pair is unique inside a block, so the result does not depend on
//                          the order in which step 5's atomics were served.  This is the
//                          deterministic limit of the paper's atomic hash-table insertion.
//   7. fill                one wavefront per group writes col/data round by round
//                          (column-major inside the group, Section 3.2 last paragraph)
#include "hbp_internal.h"

#include <chrono>
#include <mutex>
#include <vector>

namespace hbp {
namespace {

constexpr int32_t kErrPtr = 1, kErrCol = 2;  // bits of the device-side error word

__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Exclusive scan of one value per thread over a 256-thread workgroup; *total is the
// workgroup sum.  sh needs 4 entries.
__device__ __forceinline__ uint32_t block_excl_scan_256(uint32_t v, uint32_t *total, uint32_t *sh)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t t = __shfl_up(inc, d);
        if (lane >= d) inc += t;
    }
    if (lane == 63) sh[w] = inc;
    __syncthreads();
    uint32_t woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint32_t s = sh[i];
        if (i < w) woff += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return woff + inc - v;
}

// ------------------------------------------------------------------ device-wide exclusive scan

enum { kOpIdentity = 0, kOpCeilDivW = 1, kOpNonZero = 2 };
template <int OP>
__device__ __forceinline__ uint32_t scan_input(uint32_t v, uint32_t W)
{
    if (OP == kOpCeilDivW) return (v + W - 1) / W;
    if (OP == kOpNonZero) return v ? 1u : 0u;
    return v;
}

constexpr int kScanTile = 2048;  // 256 threads x 8 consecutive items

template <int OP>
__global__ __launch_bounds__(256) void k_scan_reduce(const uint32_t *__restrict__ in, int64_t n, uint32_t W,
                                                     uint32_t *__restrict__ tile_sum)
{
    __shared__ uint32_t sh[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 8;
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; i++)
        if (base + i < n) s += scan_input<OP>(in[base + i], W);
    uint32_t total;
    block_excl_scan_256(s, &total, sh);
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = total;
}

// One workgroup scans the tile sums in place (exclusive) and writes the grand total.
__global__ __launch_bounds__(256) void k_scan_tiles(uint32_t *__restrict__ tile_sum, int64_t n_tiles,
                                                    uint32_t *__restrict__ total_out)
{
    __shared__ uint32_t sh[4];
    uint32_t carry = 0;
    for (int64_t base = 0; base < n_tiles; base += 256) {
        int64_t i = base + threadIdx.x;
        uint32_t v = i < n_tiles ? tile_sum[i] : 0u, total;
        uint32_t ex = block_excl_scan_256(v, &total, sh);
        if (i < n_tiles) tile_sum[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) *total_out = carry;
}

template <int OP>
__global__ __launch_bounds__(256) void k_scan_down(const uint32_t *__restrict__ in, int64_t n, uint32_t W,
                                                   const uint32_t *__restrict__ tile_off, uint32_t *__restrict__ out)
{
    __shared__ uint32_t sh[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * 8;
    uint32_t v[8], s = 0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        v[i] = base + i < n ? scan_input<OP>(in[base + i], W) : 0u;
        s += v[i];
    }
    uint32_t total;
    uint32_t run = tile_off[blockIdx.x] + block_excl_scan_256(s, &total, sh);
#pragma unroll
    for (int i = 0; i < 8; i++) {
        if (base + i < n) out[base + i] = run;
        run += v[i];
    }
}

// out[0..n) = exclusive scan of OP(in), out[n] = total.  `in` and `out` may alias.
// tile_tmp must hold ceil(n / 2048) entries.
template <int OP>
int exclusive_scan(const uint32_t *in, uint32_t *out, int64_t n, uint32_t W, uint32_t *tile_tmp, hipStream_t st)
{
    if (n <= 0) {
        HBP_HIP(hipMemsetAsync(out, 0, sizeof(uint32_t), st));
        return HBP_OK;
    }
    const int64_t tiles = (n + kScanTile - 1) / kScanTile;
    k_scan_reduce<OP><<<dim3((unsigned)tiles), 256, 0, st>>>(in, n, W, tile_tmp);
    k_scan_tiles<<<1, 256, 0, st>>>(tile_tmp, tiles, out + n);
    k_scan_down<OP><<<dim3((unsigned)tiles), 256, 0, st>>>(in, n, W, tile_tmp, out);
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

// ------------------------------------------------------------------ Section 3.2: hash

// key(n) = min(min(n >> a, 8) * b + (((n mod 2^a) * d) >> a), R - 1) with b = d = max(1, R / 9):
// aggregation (shift, rows beyond class 8 count as 8), dispersion (class bands of width b),
// linear mapping (position inside the band).
__device__ __forceinline__ uint32_t hash_key(uint32_t n, uint32_t a, uint32_t b, uint32_t R)
{
    uint32_t agg = n >> a;
    agg = agg > 8u ? 8u : agg;
    uint32_t lin = ((n & ((1u << a) - 1u)) * b) >> a;
    uint32_t key = agg * b + lin;
    return key > R - 1u ? R - 1u : key;
}

// Sampling of the shift a: histogram, over the segments of up to 4096 evenly spaced rows, of
// the smallest a in 0..12 with n < 9 * 2^a.  One wavefront walks one sampled row.  hist[14] also
// counts the sampled segments with at least kLongSegment nonzeros (block sizes are chosen by it).
constexpr int kLongSegment = 6;
__global__ __launch_bounds__(256) void k_sample_hist(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                     int64_t n_rows, int64_t nnz, int32_t C, int32_t S,
                                                     uint32_t *__restrict__ hist)
{
    __shared__ uint32_t sh_hist[15];  // [14]: sampled segments with kLongSegment or more nonzeros
    if (threadIdx.x < 15) sh_hist[threadIdx.x] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
    auto tally = [&](int n) {
        int a = 0;
        while (a < 13 && n >= (9 << a)) a++;
        atomicAdd(&sh_hist[a], 1u);
        if (n >= kLongSegment) atomicAdd(&sh_hist[14], 1u);
    };
    if (k < S) {
        const int64_t r = ((int64_t)k * n_rows) / S;
        int64_t j0 = ptr[r], j1 = ptr[r + 1];
        if (j0 < 0 || j1 > nnz || j1 < j0) j1 = j0;  // malformed ptr is reported by the row-bit pass
        int64_t open = -1;                            // start of the segment whose end is not yet seen
        int bn_left = -1;                             // column block of the nonzero left of this chunk
        // A long row that spans few column blocks (R-MAT has rows of 10^5 nonzeros; walking one
        // chunk by chunk took 0.36 ms): its columns ascend, so its segment in column block bn is
        // [first column >= bn C, first column >= (bn + 1) C), two binary searches per lane.
        if (j1 - j0 > 4096) {
            const int64_t bn_first = col[j0] / C, bn_last = col[j1 - 1] / C;
            if (col[j0] >= 0 && bn_last >= bn_first && bn_last - bn_first < 4096) {
                auto lower_bound = [&](int64_t target) {  // first j in [j0, j1] with col[j] >= target
                    int64_t lo = j0, hi = j1;
                    while (lo < hi) {
                        const int64_t mid = lo + ((hi - lo) >> 1);
                        if ((int64_t)col[mid] >= target) hi = mid; else lo = mid + 1;
                    }
                    return lo;
                };
                for (int64_t bn = bn_first + lane; bn <= bn_last; bn += 64) {
                    const int64_t n = lower_bound((bn + 1) * C) - lower_bound(bn * C);
                    if (n > 0) tally((int)n);
                }
                j1 = j0;  // done: the walk below finds nothing
            }
        }
        // eight chunks of 64 columns are fetched at a time
        constexpr int kAhead = 8;
        for (int64_t base0 = j0; base0 < j1; base0 += 64 * kAhead) {
            int32_t cols[kAhead];
#pragma unroll
            for (int u = 0; u < kAhead; u++) {
                const int64_t j = base0 + 64 * u + lane;
                cols[u] = j < j1 ? col[j] : -1;
            }
#pragma unroll
            for (int u = 0; u < kAhead; u++) {
            const int64_t base = base0 + 64 * u;
            if (base >= j1) break;
            const int64_t j = base + lane;
            const bool valid = j < j1;
            const int bn = valid ? cols[u] / C : -2;
            int bn_prev = __shfl_up(bn, 1);
            if (lane == 0) bn_prev = bn_left;
            const bool start = valid && bn != bn_prev;
            const uint64_t mask = __ballot(start);
            if (mask) {
                const int first = __ffsll((long long)mask) - 1;
                if (open >= 0 && lane == 0) tally((int)(base + first - open));
                if (start) {
                    const uint64_t above = mask & ~((2ull << lane) - 1ull);
                    if (above) tally(__ffsll((long long)above) - 1 - lane);
                }
                open = base + (63 - __clzll((long long)mask));
            }
            bn_left = __shfl(bn, 63);
            }
        }
        if (open >= 0 && lane == 0) tally((int)(j1 - open));
    }
    __syncthreads();
    if (threadIdx.x < 15 && sh_hist[threadIdx.x]) atomicAdd(&hist[threadIdx.x], sh_hist[threadIdx.x]);
}

// a = smallest shift for which at least 15/16 of the sampled segments aggregate into 0..8.
__global__ void k_pick_shift(const uint32_t *__restrict__ hist, int32_t *__restrict__ a_out)
{
    if (threadIdx.x || blockIdx.x) return;
    uint64_t total = 0, below = 0;
    for (int i = 0; i < 14; i++) total += hist[i];
    int a = 0;
    if (total) {
        a = 12;
        for (int i = 0; i <= 12; i++) {
            below += hist[i];
            if (16 * below >= 15 * total) { a = i; break; }
        }
    }
    *a_out = a;
}

// Empty matrix: one empty combine unit per row block (it writes the zeros of y).
__global__ __launch_bounds__(256) void k_iota_units(int32_t *unit_ptr, int32_t *unit_stripe, int32_t *unit_k, int32_t NBR)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i > NBR) return;
    unit_ptr[i] = (int32_t)i;
    unit_k[i] = 0;
    if (i < NBR) unit_stripe[i] = (int32_t)i;
}

__global__ void k_set_i32(int32_t *p, int32_t v)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

// ------------------------------------------------------------------ steps 1-3: segments

__global__ __launch_bounds__(256) void k_row_bits(const int32_t *__restrict__ ptr, int64_t n_rows, int64_t nnz,
                                                  uint32_t *__restrict__ row_bits, int32_t *__restrict__ err)
{
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= n_rows) return;
    const int64_t p0 = ptr[r], p1 = ptr[r + 1];
    if (p0 < 0 || p1 < p0 || p1 > nnz) {
        atomicOr(err, kErrPtr);
        return;
    }
    if (p1 > p0) atomicOr(&row_bits[p0 >> 5], 1u << (p0 & 31));
}

// word_row[w] = the row that holds nonzero 64 w (largest r with ptr[r] <= 64 w); word_row[n_words] = n_rows - 1.
__global__ __launch_bounds__(256) void k_word_rows(const int32_t *__restrict__ ptr, int64_t n_rows, int64_t n_words,
                                                   int32_t *__restrict__ word_row)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w > n_words) return;
    if (w == n_words) { word_row[w] = (int32_t)(n_rows - 1); return; }
    const int64_t j = w * 64;
    int64_t lo = 0, hi = n_rows - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (ptr[mid] <= j) lo = mid; else hi = mid - 1;
    }
    word_row[w] = (int32_t)lo;
}

// A wavefront takes kWordsPerWave words of 64 consecutive nonzeros each, all loads issued before
// the first use: segment-start bits of every word and their count.  (One word per wavefront
// left the kernel waiting on a single load per lane.)  shift_c >= 0: C = 2^shift_c.
constexpr int kWordsPerWave = 4;

__device__ __forceinline__ int32_t block_column(int32_t c, int32_t C, int32_t shift_c)
{
    return shift_c >= 0 ? c >> shift_c : c / C;
}

__global__ __launch_bounds__(256) void k_seg_flags(const int32_t *__restrict__ col, const uint32_t *__restrict__ row_bits,
                                                   int64_t nnz, int64_t n_cols, int32_t C, int32_t shift_c, int64_t n_words,
                                                   int validate, uint64_t *__restrict__ seg_bits,
                                                   uint32_t *__restrict__ seg_cnt, int32_t *__restrict__ err)
{
    const int lane = threadIdx.x & 63;
    const int64_t w0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * kWordsPerWave;
    if (w0 >= n_words) return;
    int32_t c[kWordsPerWave];
    uint32_t bits[kWordsPerWave];
#pragma unroll
    for (int u = 0; u < kWordsPerWave; u++) {
        const int64_t j = (w0 + u) * 64 + lane;
        c[u] = j < nnz ? col[j] : 0;
        bits[u] = j < nnz ? row_bits[j >> 5] : 0u;
    }
    int32_t before = -1;  // the nonzero in front of this wavefront's first
    if (lane == 0 && w0 > 0) before = col[w0 * 64 - 1];
#pragma unroll
    for (int u = 0; u < kWordsPerWave; u++) {
        const int64_t w = w0 + u;
        if (w >= n_words) break;  // wave-uniform
        const int64_t j = w * 64 + lane;
        const bool valid = j < nnz;
        int32_t c_prev = __shfl_up(c[u], 1);
        const int32_t last_of_prev = u > 0 ? __shfl(c[u > 0 ? u - 1 : 0], 63) : before;
        if (lane == 0) c_prev = last_of_prev;
        const bool row_start = valid && ((bits[u] >> (j & 31)) & 1u);
        const bool in_range = c[u] >= 0 && c[u] < n_cols;
        if (valid && !in_range) atomicOr(err, kErrCol);
        if (validate && valid && !row_start && c[u] <= c_prev) atomicOr(err, kErrCol);
        const bool start = valid && (row_start || block_column(c[u], C, shift_c) != block_column(c_prev, C, shift_c));
        const uint64_t mask = __ballot(start);
        if (lane == 0) {
            seg_bits[w] = mask;
            seg_cnt[w] = (uint32_t)__popcll(mask);
        }
    }
}

// Segment list: every set bit of seg_bits becomes a segment (first nonzero, row, block column).
// A wavefront takes kWordsPerWave words; the row of a segment start is found by a binary search
// over the rows its word spans, the searches of the wavefront's words advancing together so that
// their loads overlap.
__global__ __launch_bounds__(256) void k_seg_emit(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                  const uint64_t *__restrict__ seg_bits, const uint32_t *__restrict__ word_off,
                                                  const int32_t *__restrict__ word_row, int64_t nnz, int64_t n_cols,
                                                  int32_t R, int32_t C, int32_t shift_c, int32_t NBR, int64_t n_words,
                                                  int32_t *__restrict__ seg_j, int32_t *__restrict__ seg_row,
                                                  int32_t *__restrict__ seg_bn)
{
    const int lane = threadIdx.x & 63;
    const int64_t w0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * kWordsPerWave;
    if (w0 >= n_words) return;
    uint64_t mask[kWordsPerWave];
    int32_t c[kWordsPerWave], lo[kWordsPerWave], hi[kWordsPerWave];
    uint32_t off[kWordsPerWave];
    bool mine[kWordsPerWave];
#pragma unroll
    for (int u = 0; u < kWordsPerWave; u++) {
        const int64_t w = min(w0 + u, n_words - 1);
        mask[u] = w0 + u < n_words ? seg_bits[w] : 0ull;
        off[u] = word_off[w];
        lo[u] = word_row[w];
        hi[u] = word_row[w + 1];
    }
    if (w0 + kWordsPerWave >= n_words && lane == 0) seg_j[word_off[n_words]] = (int32_t)nnz;  // sentinel: end of the last segment
#pragma unroll
    for (int u = 0; u < kWordsPerWave; u++) {
        mine[u] = (mask[u] >> lane) & 1ull;
        c[u] = mine[u] ? col[(w0 + u) * 64 + lane] : 0;
        if (c[u] < 0 || c[u] >= n_cols) mine[u] = false;  // already reported; never index with it
        if (!mine[u]) hi[u] = lo[u];
    }
    for (;;) {  // largest row with ptr[row] <= j, for all words at once
        bool any = false;
        int32_t mid[kWordsPerWave], p[kWordsPerWave];
#pragma unroll
        for (int u = 0; u < kWordsPerWave; u++) {
            mid[u] = lo[u] + ((hi[u] - lo[u] + 1) >> 1);
            any |= lo[u] < hi[u];
        }
        if (!__ballot(any)) break;
#pragma unroll
        for (int u = 0; u < kWordsPerWave; u++) p[u] = ptr[mid[u]];
#pragma unroll
        for (int u = 0; u < kWordsPerWave; u++) {
            if (lo[u] < hi[u]) {
                if (p[u] <= (w0 + u) * 64 + lane) lo[u] = mid[u]; else hi[u] = mid[u] - 1;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kWordsPerWave; u++) {
        if (!mine[u]) continue;
        const uint32_t s = off[u] + (uint32_t)lanes_below(mask[u]);
        seg_j[s] = (int32_t)((w0 + u) * 64 + lane);
        seg_row[s] = lo[u];
        seg_bn[s] = block_column(c[u], C, shift_c);
    }
}

// ------------------------------------------------------------------ step 4: block table

// Non-empty blocks get their coordinates and ranges; thread d also fills col_blk_ptr[d].
__global__ __launch_bounds__(256) void k_compact_blocks(const uint32_t *__restrict__ dense_cnt, const uint32_t *__restrict__ slot_off,
                                                        const uint32_t *__restrict__ group_off, const uint32_t *__restrict__ blk_id,
                                                        int64_t D, int32_t NBR, int32_t NBC, int32_t *__restrict__ blk_bm,
                                                        int32_t *__restrict__ blk_bn, int32_t *__restrict__ slot_ptr,
                                                        int32_t *__restrict__ blk_group_ptr, int32_t *__restrict__ col_blk_ptr)
{
    const int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (d <= NBC) col_blk_ptr[d] = (int32_t)blk_id[d * NBR];   // blk_id[D] = B closes the last column
    if (d > D) return;
    if (d == D) {
        const uint32_t B = blk_id[D];
        slot_ptr[B] = (int32_t)slot_off[D];
        blk_group_ptr[B] = (int32_t)group_off[D];
        return;
    }
    if (!dense_cnt[d]) return;
    const uint32_t b = blk_id[d];
    blk_bn[b] = (int32_t)(d / NBR);
    blk_bm[b] = (int32_t)(d % NBR);
    slot_ptr[b] = (int32_t)slot_off[d];
    blk_group_ptr[b] = (int32_t)group_off[d];
}

// Combine index: thread bm walks its row of the block table left to right (coalesced over bm).
__global__ __launch_bounds__(256) void k_stripe_count(const uint32_t *__restrict__ dense_cnt, int32_t NBR, int32_t NBC,
                                                      uint32_t *__restrict__ stripe_cnt)
{
    const int64_t bm = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (bm >= NBR) return;
    uint32_t n = 0;
    for (int64_t bn = 0; bn < NBC; bn++) n += dense_cnt[bn * NBR + bm] ? 1u : 0u;
    stripe_cnt[bm] = n;
}

__global__ __launch_bounds__(256) void k_stripe_fill(const uint32_t *__restrict__ dense_cnt, const uint32_t *__restrict__ blk_id,
                                                     const int32_t *__restrict__ stripe_ptr, int32_t NBR, int32_t NBC,
                                                     int32_t *__restrict__ stripe_blk)
{
    const int64_t bm = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (bm >= NBR) return;
    int32_t k = stripe_ptr[bm];
    for (int64_t bn = 0; bn < NBC; bn++) {
        const int64_t d = bn * NBR + bm;
        if (dense_cnt[d]) stripe_blk[k++] = (int32_t)blk_id[d];
    }
}

// ------------------------------------------------------------------ steps 5-6: hash + placement

// Wave-aggregated fetch-add: lanes of the wavefront that target the same counter are served by
// one atomic (neighbouring segments mostly fall into the same block, and same-address atomics
// serialise).  Returns, for an active lane, the value its own atomicAdd(&counters[key], 1) would
// have returned in some serial order.  After a few distinct keys the rest go one by one.
__device__ __forceinline__ uint32_t aggregated_add(uint32_t *counters, int64_t key, bool active)
{
    const int lane = threadIdx.x & 63;
    uint64_t todo = __ballot(active);
    uint32_t result = 0;
    for (int it = 0; todo && it < 8; it++) {
        const int leader = __ffsll((long long)todo) - 1;
        const int64_t k = __shfl(key, leader);
        const uint64_t same = __ballot(active && key == k) & todo;
        uint32_t base = 0;
        if (lane == leader) base = atomicAdd(&counters[k], (uint32_t)__popcll(same));
        base = __shfl(base, leader);
        if ((same >> lane) & 1ull) result = base + (uint32_t)lanes_below(same);
        todo &= ~same;
    }
    if ((todo >> lane) & 1ull) result = atomicAdd(&counters[key], 1u);
    return result;
}

// Tiles for the two passes that touch a per-block counter for every segment.  A workgroup takes
// kTileSegs consecutive segments.  They are in CSR order, so their rows ascend and the tile
// touches the blocks of a few neighbouring row blocks only: (bm_hi - bm_lo + 1) * NBC counters.
// When those fit in LDS the tile counts there (LDS integer atomics are two orders of magnitude
// faster than scattered global ones) and goes to global memory once per counter it has
// touched; otherwise every segment goes to global memory with wave-aggregated atomics.
constexpr int kTileSegs = 2048;      // 256 threads x 8 segments
constexpr int kTileCounters = 8192;  // 32 KB of LDS

struct Tile {
    int64_t base, S;
    int32_t bm_lo, span;  // span = 0: the counters do not fit
};

__device__ __forceinline__ Tile tile_of(const int32_t *__restrict__ seg_row, int64_t S, int32_t R, int32_t NBC)
{
    Tile t;
    t.S = S;
    t.base = (int64_t)blockIdx.x * kTileSegs;
    t.bm_lo = 0;
    t.span = 0;
    if (t.base < S) {
        const int64_t last = min(t.base + kTileSegs, S) - 1;
        t.bm_lo = seg_row[t.base] / R;
        const int64_t span = (int64_t)(seg_row[last] / R - t.bm_lo + 1) * NBC;
        t.span = span <= kTileCounters ? (int32_t)span : 0;
    }
    return t;
}

// Segments per block of the (column block, row block) table.
// The segment count is still on the device (last entry of the scan) and the records of a
// malformed matrix are incomplete, hence S_ptr and err.
__global__ __launch_bounds__(256) void k_count_blocks(const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_bn,
                                                      const uint32_t *__restrict__ S_ptr, const int32_t *__restrict__ err,
                                                      int32_t R, int32_t NBR, int32_t NBC, uint32_t *__restrict__ dense_cnt)
{
    __shared__ uint32_t cnt[kTileCounters];
    if (*err) return;
    const Tile t = tile_of(seg_row, (int64_t)*S_ptr, R, NBC);
    if (t.base >= t.S) return;
    if (t.span == 0) {
        for (int i = 0; i < kTileSegs / 256; i++) {
            const int64_t s = t.base + i * 256 + threadIdx.x;
            const bool active = s < t.S;
            const int64_t d = active ? (int64_t)seg_bn[s] * NBR + seg_row[s] / R : 0;
            aggregated_add(dense_cnt, d, active);
        }
        return;
    }
    for (int i = threadIdx.x; i < t.span; i += 256) cnt[i] = 0u;
    __syncthreads();
    for (int i = 0; i < kTileSegs / 256; i++) {
        const int64_t s = t.base + i * 256 + threadIdx.x;
        if (s < t.S) atomicAdd(&cnt[(seg_row[s] / R - t.bm_lo) * NBC + seg_bn[s]], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < t.span; i += 256) {
        const uint32_t c = cnt[i];
        if (c) atomicAdd(&dense_cnt[(int64_t)(i % NBC) * NBR + t.bm_lo + i / NBC], c);
    }
}

// Bucketed scatter: (length << 16 | local row, first nonzero) of every segment into its block's
// slot range.  The order in which the segments of a block arrive is arbitrary (k_order_block
// computes the keys and sorts them).
__global__ __launch_bounds__(256) void k_bucket(const int32_t *__restrict__ seg_j, const int32_t *__restrict__ seg_row,
                                                const int32_t *__restrict__ seg_bn, int64_t S, int32_t R, int32_t NBR, int32_t NBC,
                                                uint32_t *__restrict__ cursor, uint32_t *__restrict__ bucket_len_row, int32_t *__restrict__ bucket_j)
{
    __shared__ uint32_t cnt[kTileCounters];  // per counter of the tile: segments seen, then their first position
    const Tile t = tile_of(seg_row, S, R, NBC);
    if (t.base >= t.S) return;
    auto emit = [&](int64_t s, int32_t row, uint32_t pos) {
        const int32_t j0 = seg_j[s];
        bucket_len_row[pos] = ((uint32_t)(seg_j[s + 1] - j0) << 16) | (uint32_t)(row % R);  // length <= C <= 32768
        bucket_j[pos] = j0;
    };
    if (t.span == 0) {
        for (int i = 0; i < kTileSegs / 256; i++) {
            const int64_t s = t.base + i * 256 + threadIdx.x;
            const bool active = s < t.S;
            const int32_t row = active ? seg_row[s] : 0;
            const int64_t d = active ? (int64_t)seg_bn[s] * NBR + row / R : 0;
            const uint32_t pos = aggregated_add(cursor, d, active);
            if (active) emit(s, row, pos);
        }
        return;
    }
    for (int i = threadIdx.x; i < t.span; i += 256) cnt[i] = 0u;
    __syncthreads();
    int32_t row[kTileSegs / 256], local[kTileSegs / 256];
    uint32_t rank[kTileSegs / 256];
#pragma unroll
    for (int i = 0; i < kTileSegs / 256; i++) {
        const int64_t s = t.base + i * 256 + threadIdx.x;
        row[i] = 0; local[i] = 0; rank[i] = 0;
        if (s < t.S) {
            row[i] = seg_row[s];
            local[i] = (row[i] / R - t.bm_lo) * NBC + seg_bn[s];
            rank[i] = atomicAdd(&cnt[local[i]], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < t.span; i += 256) {
        const uint32_t c = cnt[i];
        if (c) cnt[i] = atomicAdd(&cursor[(int64_t)(i % NBC) * NBR + t.bm_lo + i / NBC], c);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kTileSegs / 256; i++) {
        const int64_t s = t.base + i * 256 + threadIdx.x;
        if (s < t.S) emit(s, row[i], cnt[local[i]] + rank[i]);
    }
}

// Which blocks a workgroup of k_fill takes.  The kernel gathers from arrays in CSR order (columns,
// values), where the pieces that the blocks of one row block need lie side by side in the same
// 128-byte lines.  Taken in the layout's column-major order every block fetches those lines anew
// (16 times the bytes on a matrix with short row segments).  Here the blocks are taken row block
// by row block (the order of stripe_blk), `parts` workgroups per row block, each taking every
// parts-th block of it; and since consecutive workgroups are dealt round-robin to the 8 XCDs,
// each with its own L2, the workgroups of a row block are numbered so that all of them land on
// one XCD: an XCD runs a few dozen workgroups at a time, which then share the lines of one or a
// few row blocks.
struct StripeWalk {
    int32_t k, k_end, step;  // entries k, k + step, ... below k_end of stripe_blk
};

__device__ __forceinline__ StripeWalk stripe_walk(const int32_t *__restrict__ stripe_ptr, int32_t NBR, int32_t parts)
{
    const int32_t q = (int32_t)(blockIdx.x >> 3), x = (int32_t)(blockIdx.x & 7u);
    const int32_t octet = q / parts, p = q % parts;
    // Which of the octet's eight row blocks goes to XCD x: x xor-ed with every 3-bit field of the
    // octet's number, a bijection inside the octet.  (With bm mod 8 itself a matrix whose density
    // follows the bits of the row index, as R-MAT's does, put 44 % of the work on one XCD.)
    int32_t fold = 0;
    for (int32_t t = octet; t; t >>= 3) fold ^= t & 7;
    const int32_t bm = octet * 8 + (x ^ fold);
    if (bm >= NBR) return {0, 0, 1};
    return {stripe_ptr[bm] + p, stripe_ptr[bm + 1], parts};
}

// Exclusive prefix sums of a[0 .. n) in LDS, in place, by the 256 threads of a workgroup.
// sh_wave: four words of LDS.  Ends with a barrier.
__device__ __forceinline__ void scan_in_lds(uint32_t *a, int n, uint32_t *sh_wave)
{
    const int chunk = (n + 255) / 256, lo = min(n, (int)threadIdx.x * chunk), hi = min(n, lo + chunk);
    uint32_t sum = 0;
    for (int i = lo; i < hi; i++) sum += a[i];
    uint32_t incl = sum;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    if (lane == 63) sh_wave[threadIdx.x >> 6] = incl;
    __syncthreads();
    uint32_t run = incl - sum;
    for (int w = 0; w < (int)(threadIdx.x >> 6); w++) run += sh_wave[w];
    for (int i = lo; i < hi; i++) {
        const uint32_t t = a[i];
        a[i] = run;
        run += t;
    }
    __syncthreads();
}

// One workgroup per non-empty block: compute the keys of its segments, order its slots by (key,
// local row), then write the slot arrays and the nonzero count of each group.
// reorder 0: no key (plain 2D partition), 1: the hash with the matrix's shift, 2: the length
// itself, 3: the hash with a shift of the block's own (Section 3.2: denser blocks call for a
// larger a; a = smallest shift for which at least 15/16 of the block's rows aggregate into 0..8).
// Blocks of more than kSmallBlock slots: the local rows of a block are distinct, so the order by
// row costs nothing: entry (key << 16 | position in the block's bucket) is stored at index `row`
// of an LDS array, which leaves holes for the rows without a segment.  Stable counting passes
// over 4 bits of the key at a time, lowest first, then put the entries in key order and keep the
// row order inside a key; the first pass also closes the holes.  In a pass a wavefront takes 64
// consecutive entries at a time; the lanes that hold the same digit find each other with four
// ballots, which gives an entry its rank among them and the tile its count per digit; a prefix
// sum over (digit, tile) turns the counts into positions.  As many passes as the block's largest
// key has hex digits.  Smaller blocks (the passes would still walk all R rows): a bitonic network
// over (key, row, length, position) words.
__global__ __launch_bounds__(256) void k_order_block(const uint32_t *__restrict__ bucket_len_row, const int32_t *__restrict__ bucket_j,
                                                     const int32_t *__restrict__ slot_ptr, const int32_t *__restrict__ blk_group_ptr,
                                                     int32_t W, uint16_t *__restrict__ row_local, uint16_t *__restrict__ seg_len,
                                                     int32_t *__restrict__ slot_j, uint32_t *__restrict__ group_nnz, uint32_t *__restrict__ group_longest,
                                                     int32_t *__restrict__ group_slot, int32_t *__restrict__ group_blk, uint32_t heavy_rounds,
                                                     uint32_t *__restrict__ longest_all, int32_t reorder, uint32_t R,
                                                     const int32_t *__restrict__ a_ptr, int32_t *__restrict__ blk_shift,
                                                     uint32_t *__restrict__ slot_key)
{
    extern __shared__ __align__(8) uint32_t order_lds[];  // two arrays of cap entries, then 16 counters per tile of 64
    __shared__ uint32_t sh_hist[14];
    __shared__ int32_t sh_shift;
    __shared__ uint32_t sh_max_key, sh_wave[4];
    constexpr uint32_t kHole = 0xffffffffu;
    constexpr int kSmallBlock = 256;  // slots: one entry per thread
    const int cap = (int)((R + 63u) & ~63u);
    uint32_t *from = order_lds, *to = order_lds + cap, *cnt = order_lds + 2 * cap;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x;
    const int s0 = slot_ptr[b], m = slot_ptr[b + 1] - s0;
    const bool small = m <= kSmallBlock;
    if (!small)
        for (int i = threadIdx.x; i < cap; i += 256) from[i] = kHole;
    if (threadIdx.x < 14) sh_hist[threadIdx.x] = 0u;
    if (threadIdx.x == 0) {
        sh_max_key = 0u;
        sh_shift = *a_ptr;
    }
    __syncthreads();
    if (reorder == 3) {
        for (int i = threadIdx.x; i < m; i += 256) {
            const uint32_t n = bucket_len_row[s0 + i] >> 16;
            int a = 0;
            while (a < 13 && n >= (9u << a)) a++;
            atomicAdd(&sh_hist[a], 1u);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t below = 0;
            int a = 12;
            for (int i = 0; i <= 12; i++) {
                below += sh_hist[i];
                if (16ull * below >= 15ull * (uint32_t)m) { a = i; break; }
            }
            sh_shift = a;
        }
        __syncthreads();
    }
    const uint32_t shift_a = (uint32_t)sh_shift, band = R / 9u ? R / 9u : 1u;
    auto key_of = [&](uint32_t n) __attribute__((always_inline)) {
        return reorder == 0 ? 0u : reorder == 2 ? n : hash_key(n, shift_a, band, R);
    };
    if (threadIdx.x == 0) blk_shift[b] = (int32_t)shift_a;
    if (small) {
        uint64_t *wide = reinterpret_cast<uint64_t *>(order_lds);  // 2 cap words: room for cap >= m entries
        int n2 = 1;
        while (n2 < m) n2 <<= 1;
        for (int i = threadIdx.x; i < n2; i += 256) {
            uint64_t e = ~0ull;
            if (i < m) {
                const uint32_t lr = bucket_len_row[s0 + i];
                e = ((uint64_t)key_of(lr >> 16) << 48) | ((uint64_t)(lr & 0xffffu) << 32) | (lr & 0xffff0000u) | (uint32_t)i;
            }
            wide[i] = e;
        }
        __syncthreads();
        for (int k = 2; k <= n2; k <<= 1)
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int t = threadIdx.x; t < n2 / 2; t += 256) {  // pair t: i has bit j clear, its partner has it set
                    const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), p = i | j;
                    const uint64_t x = wide[i], y = wide[p];
                    if ((x > y) == ((i & k) == 0)) { wide[i] = y; wide[p] = x; }
                }
                __syncthreads();
            }
        const int i = threadIdx.x;  // m <= 256: one entry per thread
        uint64_t e = 0;
        if (i < m) e = wide[i];
        __syncthreads();  // `to` may overlap `wide`
        if (i < m) {
            const uint32_t n = (uint32_t)(e >> 16) & 0xffffu;
            row_local[s0 + i] = (uint16_t)((e >> 32) & 0xffffu);
            seg_len[s0 + i] = (uint16_t)n;
            if (slot_key) slot_key[s0 + i] = (uint32_t)(e >> 48);
            slot_j[s0 + i] = bucket_j[s0 + (int32_t)(e & 0xffffu)];  // a gather inside the block's own range
            to[i] = n;
        }
    } else {
        uint32_t most = 0;
        for (int i = threadIdx.x; i < m; i += 256) {
            const uint32_t lr = bucket_len_row[s0 + i];
            const uint32_t key = key_of(lr >> 16);
            from[lr & 0xffffu] = (key << 16) | (uint32_t)i;
            most = max(most, key);
        }
        if (most) atomicMax(&sh_max_key, most);
        __syncthreads();
        const uint32_t max_key = sh_max_key;
        const int passes = max_key ? (35 - __clz(max_key)) / 4 : 1;  // hex digits of the largest key; one pass at least: it closes the holes
        int len = cap;  // entries of `from` (with holes in the first pass)
        for (int pass = 0; pass < passes; pass++) {
            const int tiles = (len + 63) / 64, shift = 16 + 4 * pass;
            for (int i = threadIdx.x; i < 16 * tiles; i += 256) cnt[i] = 0u;
            __syncthreads();
            // the lanes of a tile with the same digit as this lane (its rank among them: the lanes below it)
            auto classify = [&](int tile, uint32_t &e, uint32_t &digit, uint64_t &same) __attribute__((always_inline)) {
                const int i = tile * 64 + lane;
                e = i < len ? from[i] : kHole;
                const bool valid = e != kHole;
                digit = (e >> shift) & 15u;
                same = __ballot(valid);
#pragma unroll
                for (int bit = 0; bit < 4; bit++) {
                    const bool set = (digit >> bit) & 1u;
                    const uint64_t with = __ballot(valid && set);
                    same &= set ? with : ~with;
                }
                return valid;
            };
            // the first kKeep tiles of a wavefront (all of them up to R = 2048) keep their entry,
            // counter and rank in registers for the scatter; tiles beyond are classified again
            constexpr int kKeep = 8;
            uint32_t kept_e[kKeep], kept_at[kKeep];  // kept_at: counter index << 6 | rank
#pragma unroll
            for (int t = 0; t < kKeep; t++) {
                const int tile = wave + 4 * t;
                kept_e[t] = kHole;
                kept_at[t] = 0u;
                if (tile < tiles) {
                    uint32_t digit;
                    uint64_t same;
                    const bool valid = classify(tile, kept_e[t], digit, same);
                    const uint32_t rank = (uint32_t)lanes_below(same);
                    if (valid && rank == 0) cnt[digit * tiles + tile] = (uint32_t)__popcll(same);
                    kept_at[t] = ((digit * (uint32_t)tiles + (uint32_t)tile) << 6) | rank;
                }
            }
            for (int tile = wave + 4 * kKeep; tile < tiles; tile += 4) {
                uint32_t e, digit;
                uint64_t same;
                const bool valid = classify(tile, e, digit, same);
                if (valid && lanes_below(same) == 0) cnt[digit * tiles + tile] = (uint32_t)__popcll(same);
            }
            __syncthreads();
            scan_in_lds(cnt, 16 * tiles, sh_wave);
#pragma unroll
            for (int t = 0; t < kKeep; t++)
                if (kept_e[t] != kHole) to[cnt[kept_at[t] >> 6] + (kept_at[t] & 63u)] = kept_e[t];
            for (int tile = wave + 4 * kKeep; tile < tiles; tile += 4) {
                uint32_t e, digit;
                uint64_t same;
                const bool valid = classify(tile, e, digit, same);
                if (valid) to[cnt[digit * tiles + tile] + (uint32_t)lanes_below(same)] = e;
            }
            __syncthreads();
            uint32_t *t = from; from = to; to = t;
            len = m;
        }
        // `from` holds the m entries in (key, local row) order; `to` is free: the lengths go there
        for (int i = threadIdx.x; i < m; i += 256) {
            const uint32_t e = from[i];
            const int32_t at = s0 + (int32_t)(e & 0xffffu);  // the segment's place in the block's bucket (gathers inside the block's own range)
            const uint32_t lr = bucket_len_row[at];
            row_local[s0 + i] = (uint16_t)(lr & 0xffffu);
            seg_len[s0 + i] = (uint16_t)(lr >> 16);
            if (slot_key) slot_key[s0 + i] = e >> 16;
            slot_j[s0 + i] = bucket_j[at];
            to[i] = lr >> 16;
        }
    }
    __syncthreads();
    // a wavefront per group (W <= 64 slots): nonzeros and longest row by a reduction over the lanes
    const int g0 = blk_group_ptr[b], ng = (m + W - 1) / W;
    for (int gi = wave; gi < ng; gi += 4) {
        const int i = gi * W + lane;
        uint32_t sum = lane < W && i < m ? to[i] : 0u, longest = sum;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) {
            sum += __shfl_xor(sum, d);
            longest = max(longest, __shfl_xor(longest, d));
        }
        if (lane == 0) {
            group_nnz[g0 + gi] = sum;
            group_longest[g0 + gi] = longest;
            if (longest > heavy_rounds) atomicMax(longest_all, longest);  // only that long rows matter to the caller
            group_slot[g0 + gi] = s0 + gi * W;
            group_blk[g0 + gi] = b;
        }
    }
}

// ------------------------------------------------------------------ step 7: fill

// One group, one wavefront.  Round k stores the k-th nonzero of every lane that still has one,
// lanes in slot order; rows keep their CSR (ascending column) order.  col0 is the first column of
// the group's block column.
template <typename T>
__device__ __forceinline__ void fill_group(int32_t g, int32_t col0, int lane, int64_t nnz, const int32_t *__restrict__ csr_col,
                                           const T *__restrict__ csr_val, const int32_t *__restrict__ group_ptr,
                                           const int32_t *__restrict__ group_slot, const uint16_t *__restrict__ seg_len,
                                           const int32_t *__restrict__ slot_j, uint16_t *__restrict__ col_local, T *__restrict__ data)
{
    const int s0 = group_slot[g], cnt = group_slot[g + 1] - s0;
    const int n = lane < cnt ? seg_len[s0 + lane] : 0;
    const int64_t j = lane < cnt ? slot_j[s0 + lane] : 0;
    int64_t base = group_ptr[g];
    // eight rounds at a time: the sixteen loads are independent of each other and of the stores
    constexpr int kRounds = 8, kLongRounds = 32;
    for (int k = 0; __ballot(k < n); k += kRounds) {
        // Few rows left, each with at least kLongRounds more nonzeros: the set of live lanes does
        // not change over these rounds, so round k + u of a live lane lands at base + u * m + its
        // rank, and a lane copies kLongRounds of its row at a time.  (Eight rounds per memory
        // round trip made the longest row of the matrix the critical path of the whole kernel.)
        for (;;) {
            const uint64_t live = __ballot(k < n);
            const int m = __popcll(live);
            if (m == 0 || m > 16 || __ballot(k + kLongRounds <= n) != live) break;
            if (k < n) {
                const int64_t dst0 = base + lanes_below(live);
                int32_t cl[kLongRounds];
                T vl[kLongRounds];
                __builtin_memcpy(cl, csr_col + j + k, sizeof cl);  // unaligned 16-byte loads
                __builtin_memcpy(vl, csr_val + j + k, sizeof vl);
#pragma unroll
                for (int u = 0; u < kLongRounds; u++) {
                    col_local[dst0 + (int64_t)u * m] = (uint16_t)(cl[u] - col0);
                    data[dst0 + (int64_t)u * m] = vl[u];
                }
            }
            base += (int64_t)kLongRounds * m;
            k += kLongRounds;
        }
        if (!__ballot(k < n)) break;
        int32_t c[kRounds];
        T v[kRounds];
        if (k + kRounds <= n) {
            // a full batch: 16-byte loads (the row starts at any multiple of 4 bytes; the copies
            // below are unaligned vector loads).  Lanes read different rows, so a 4-byte load
            // would cost a whole sector of L2 traffic per element.
            __builtin_memcpy(c, csr_col + j + k, sizeof c);
            __builtin_memcpy(v, csr_val + j + k, sizeof v);
        } else {
            // The end of a row: its elements are read four at a time all the same, as long as the
            // four lie inside the arrays (what is read past the row's end is not stored).  Lanes
            // read different rows: an instruction costs a line per lane whatever its width.
#pragma unroll
            for (int u = 0; u < kRounds; u++) {
                c[u] = 0;
                v[u] = T(0);
            }
#pragma unroll
            for (int q = 0; q < kRounds; q += 4) {
                if (k + q < n) {
                    if (j + k + q + 4 <= nnz) {
                        __builtin_memcpy(c + q, csr_col + j + k + q, 4 * sizeof(int32_t));
                        __builtin_memcpy(v + q, csr_val + j + k + q, 4 * sizeof(T));
                    } else {
#pragma unroll
                        for (int u = q; u < q + 4; u++)
                            if (k + u < n) {
                                c[u] = csr_col[j + k + u];
                                v[u] = csr_val[j + k + u];
                            }
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kRounds; u++) {
            const uint64_t live = __ballot(k + u < n);
            if (k + u < n) {
                const int64_t dst = base + lanes_below(live);
                col_local[dst] = (uint16_t)(c[u] - col0);
                data[dst] = v[u];
            }
            base += __popcll(live);
        }
    }
}

// Workgroups take blocks as stripe_walk says, the wavefronts of one taking a block's groups in turn.
template <typename T>
__global__ __launch_bounds__(256) void k_fill(const int32_t *__restrict__ stripe_ptr, const int32_t *__restrict__ stripe_blk,
                                              int32_t NBR, int32_t B, int32_t parts,
                                              const int32_t *__restrict__ csr_col, const T *__restrict__ csr_val,
                                              const int32_t *__restrict__ group_ptr, const int32_t *__restrict__ group_slot,
                                              const int32_t *__restrict__ blk_group_ptr, const int32_t *__restrict__ blk_bn,
                                              const uint16_t *__restrict__ seg_len, const int32_t *__restrict__ slot_j,
                                              int32_t C, int64_t nnz, uint16_t *__restrict__ col_local, T *__restrict__ data)
{
    const int lane = threadIdx.x & 63;
    const StripeWalk walk = stripe_walk(stripe_ptr, NBR, parts);
    for (int32_t entry = walk.k; entry < walk.k_end; entry += walk.step) {
        const int32_t b = stripe_blk[entry];
        const int32_t col0 = blk_bn[b] * C;
        const int32_t g_end = blk_group_ptr[b + 1];
        for (int32_t g = blk_group_ptr[b] + (int32_t)(threadIdx.x >> 6); g < g_end; g += 4)
            fill_group<T>(g, col0, lane, nnz, csr_col, csr_val, group_ptr, group_slot, seg_len, slot_j, col_local, data);
    }
}

// The same with one wavefront per group, in the layout's own order.
template <typename T>
__global__ __launch_bounds__(256) void k_fill_flat(const int32_t *__restrict__ csr_col, const T *__restrict__ csr_val,
                                                   const int32_t *__restrict__ group_ptr, const int32_t *__restrict__ group_slot,
                                                   const int32_t *__restrict__ group_blk, const int32_t *__restrict__ blk_bn,
                                                   const uint16_t *__restrict__ seg_len, const int32_t *__restrict__ slot_j,
                                                   int32_t G, int32_t C, int64_t nnz, uint16_t *__restrict__ col_local, T *__restrict__ data)
{
    const int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= G) return;
    fill_group<T>((int32_t)g, blk_bn[group_blk[g]] * C, (int)(threadIdx.x & 63), nnz, csr_col, csr_val, group_ptr, group_slot, seg_len, slot_j,
                  col_local, data);
}

// add_sign derived from seg_len (Section 3.2: distance to the row's next nonzero = nonzeros
// after it in this round + nonzeros before it in the next round + 1; -1 at the row's end).
__global__ __launch_bounds__(256) void k_add_sign(const int32_t *__restrict__ group_ptr, const int32_t *__restrict__ group_slot,
                                                  const uint16_t *__restrict__ seg_len, int32_t G, int32_t *__restrict__ add_sign)
{
    const int lane = threadIdx.x & 63;
    const int64_t g = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= G) return;
    const int s0 = group_slot[g], cnt = group_slot[g + 1] - s0;
    const int n = lane < cnt ? seg_len[s0 + lane] : 0;
    int64_t base = group_ptr[g];
    const uint64_t above_me = ~((2ull << lane) - 1ull);
    for (int k = 0;; k++) {
        const uint64_t live = __ballot(k < n);
        if (!live) break;
        const uint64_t next = __ballot(k + 1 < n);
        if (k < n) {
            const int64_t dst = base + lanes_below(live);
            add_sign[dst] = k + 1 < n ? __popcll(live & above_me) + lanes_below(next) + 1 : -1;
        }
        base += __popcll(live);
    }
}

// ------------------------------------------------------------------ combine work units
//
// A row block with many slots is cut into u = ceil(slots / unit_slots) units of consecutive
// stripe_blk entries, so that no workgroup of the combine part gets much more than unit_slots
// slots; unit i starts at the first entry whose preceding slots, times u, reach i times the row
// block's slots.

__global__ __launch_bounds__(256) void k_stripe_sizes(const int32_t *__restrict__ stripe_blk, const int32_t *__restrict__ slot_ptr,
                                                      int32_t B, uint32_t *__restrict__ size)
{
    const int64_t k = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= B) return;
    const int32_t b = stripe_blk[k];
    size[k] = (uint32_t)(slot_ptr[b + 1] - slot_ptr[b]);
}

__global__ __launch_bounds__(256) void k_unit_count(const int32_t *__restrict__ stripe_ptr, const uint32_t *__restrict__ cum,
                                                    int32_t NBR, int32_t unit_slots, uint32_t *__restrict__ units)
{
    const int64_t bm = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (bm >= NBR) return;
    const int64_t slots = (int64_t)cum[stripe_ptr[bm + 1]] - (int64_t)cum[stripe_ptr[bm]];
    const int64_t u = (slots + unit_slots - 1) / unit_slots;
    units[bm] = (uint32_t)(u < 1 ? 1 : u);
}

// multi[bm] = 1 when the row block has more than one unit (input of the scan that numbers them)
__global__ __launch_bounds__(256) void k_unit_multi(const uint32_t *__restrict__ units, int32_t NBR, uint32_t *__restrict__ multi)
{
    const int64_t bm = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (bm < NBR) multi[bm] = units[bm] > 1 ? 1u : 0u;
}

__global__ __launch_bounds__(256) void k_unit_fill(const int32_t *__restrict__ stripe_ptr, const uint32_t *__restrict__ cum,
                                                   const int32_t *__restrict__ unit_ptr, const uint32_t *__restrict__ multi_idx,
                                                   int32_t NBR, int32_t B, int32_t *__restrict__ unit_stripe,
                                                   int32_t *__restrict__ unit_k, int32_t *__restrict__ multi_stripes)
{
    const int64_t bm = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (bm >= NBR) return;
    const int32_t k0 = stripe_ptr[bm], k1 = stripe_ptr[bm + 1];
    const int32_t u0 = unit_ptr[bm], u = unit_ptr[bm + 1] - u0;
    const int64_t base = cum[k0], slots = (int64_t)cum[k1] - base;
    for (int32_t i = 0; i < u; i++) {
        int32_t lo = k0, hi = k1;  // smallest k in [k0, k1] with (cum[k] - base) * u >= i * slots
        while (lo < hi) {
            const int32_t mid = lo + ((hi - lo) >> 1);
            if (((int64_t)cum[mid] - base) * u >= (int64_t)i * slots) hi = mid; else lo = mid + 1;
        }
        unit_stripe[u0 + i] = (int32_t)bm;
        unit_k[u0 + i] = lo;
    }
    if (u > 1) multi_stripes[multi_idx[bm]] = (int32_t)bm;
    if (bm == NBR - 1) unit_k[u0 + u] = B;
}

// ------------------------------------------------------------------ Section 3.3: schedule
//
// Weight of a group = GW + its nonzeros + SW times its slots + RW times its rounds (GW =
// group_weight, SW = slot_weight, RW = round_weight: the costs of a group as such, of a row and
// of a round of a group, measured in nonzeros; a group has as many rounds as its longest row
// has nonzeros);
// Wt(g) = group_ptr[g] + SW * group_slot[g] + RW * group_rounds[g] + GW * g is the weight of all
// groups before g.
struct Weights {
    const int32_t *group_ptr, *group_slot, *group_rounds;
    int64_t SW, RW, GW;
    __device__ __forceinline__ int64_t before(int32_t g) const
    {
        return (int64_t)group_ptr[g] + SW * group_slot[g] + RW * group_rounds[g] + GW * g;
    }
};

__global__ __launch_bounds__(256) void k_col_group_ptr(const int32_t *__restrict__ col_blk_ptr, const int32_t *__restrict__ blk_group_ptr,
                                                       int32_t NBC, int32_t *__restrict__ col_group_ptr)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c <= NBC) col_group_ptr[c] = blk_group_ptr[col_blk_ptr[c]];
}

// comp_lo[w]: first group of worker w's range left to competition: the first g in the range whose
// preceding weight inside the range reaches fixed_q8/256 of the range's weight, but not before
// the first group of the block column that holds the range's last group (comp_col[w]), so that
// the competitive groups of a range need one segment of the vector.
__global__ __launch_bounds__(256) void k_comp_lo(const int32_t *__restrict__ col_group_ptr, Weights wt, int32_t NBC, int32_t P,
                                                 int32_t fixed_q8, const int32_t *__restrict__ fixed_start,
                                                 const int32_t *__restrict__ fixed_col, int32_t *__restrict__ comp_lo,
                                                 int32_t *__restrict__ comp_col)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= P) return;
    const int32_t g0 = fixed_start[w], g1 = fixed_start[w + 1];
    const int64_t w0 = wt.before(g0);
    const int64_t need = (wt.before(g1) - w0) * fixed_q8;
    int32_t lo = g0, hi = g1;  // smallest g in [g0, g1] with (Wt(g) - w0) * 256 >= need
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if ((wt.before(mid) - w0) * 256 >= need) hi = mid; else lo = mid + 1;
    }
    int32_t c = fixed_col[w];
    if (g1 > g0) {
        int32_t c_lo = 0, c_hi = NBC - 1;  // largest c with col_group_ptr[c] <= g1 - 1
        while (c_lo < c_hi) {
            const int32_t mid = c_lo + ((c_hi - c_lo + 1) >> 1);
            if (col_group_ptr[mid] <= g1 - 1) c_lo = mid; else c_hi = mid - 1;
        }
        c = c_lo;
        lo = max(lo, col_group_ptr[c]);
    }
    comp_lo[w] = lo;
    comp_col[w] = c;
}

// col_rank[c], c in 0..NBC: block columns before c that hold a group.  One workgroup: every thread
// counts a contiguous piece, the pieces' counts are scanned in LDS, every thread writes its piece.
__global__ __launch_bounds__(256) void k_col_rank(const int32_t *__restrict__ col_group_ptr, int32_t NBC, int32_t *__restrict__ col_rank)
{
    __shared__ int32_t piece_sum[256];
    const int32_t per = (NBC + 255) / 256, c0 = min(NBC, (int32_t)threadIdx.x * per), c1 = min(NBC, c0 + per);
    int32_t mine = 0;
    for (int32_t c = c0; c < c1; c++) mine += col_group_ptr[c + 1] > col_group_ptr[c];
    piece_sum[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t run = 0;
        for (int i = 0; i < 256; i++) { const int32_t v = piece_sum[i]; piece_sum[i] = run; run += v; }
    }
    __syncthreads();
    int32_t run = piece_sum[threadIdx.x];
    for (int32_t c = c0; c < c1; c++) {
        col_rank[c] = run;
        run += col_group_ptr[c + 1] > col_group_ptr[c];
    }
    if (c1 == NBC && c0 < NBC) col_rank[NBC] = run;  // the thread that holds the last column
}

// fixed_start[w]: first g with Wc(g) * P >= w * Wc(G) (P contiguous ranges of equal weight), where
// Wc(g) = Wt(g) + CW * (block columns with a group that start before g): entering a block column
// costs a worker the fetch of its vector segment, charged to the column's first group;
// fixed_col[w]: the last block column that starts at or before that group.
__global__ __launch_bounds__(256) void k_fixed_start(const int32_t *__restrict__ col_group_ptr, Weights wt,
                                                     const int32_t *__restrict__ col_rank, int64_t CW, int32_t NBC, int32_t G,
                                                     int32_t P, int32_t *__restrict__ fixed_start, int32_t *__restrict__ fixed_col)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w > P) return;
    auto before = [&](int32_t g) {
        int64_t v = wt.before(g);
        if (CW) {
            int32_t c_lo = 0, c_hi = NBC;  // first c in 0..NBC with col_group_ptr[c] >= g (col_group_ptr[NBC] = G)
            while (c_lo < c_hi) {
                const int32_t mid = c_lo + ((c_hi - c_lo) >> 1);
                if (col_group_ptr[mid] >= g) c_hi = mid; else c_lo = mid + 1;
            }
            v += CW * col_rank[c_lo];
        }
        return v;
    };
    const int64_t need = w * before(G);
    int32_t lo = 0, hi = G;
    while (lo < hi) {
        const int32_t mid = lo + ((hi - lo) >> 1);
        if (before(mid) * P >= need) hi = mid; else lo = mid + 1;
    }
    fixed_start[w] = lo;
    if (w == P) return;
    int32_t c_lo = 0, c_hi = NBC - 1;  // largest c with col_group_ptr[c] <= lo
    while (c_lo < c_hi) {
        const int32_t mid = c_lo + ((c_hi - c_lo + 1) >> 1);
        if (col_group_ptr[mid] <= lo) c_lo = mid; else c_hi = mid - 1;
    }
    fixed_col[w] = c_lo;
}

// The paper's schedule (Section 3.3 read literally): worker w is pre-assigned the F blocks
// [w F, (w + 1) F) of the column-major block list; handed over as group ranges (the unit the
// kernels walk).  Nothing inside a range is competitive: the blocks from P F on are claimed one at
// a time through a single ticket counter.
__global__ __launch_bounds__(256) void k_paper_schedule(const int32_t *__restrict__ blk_group_ptr, const int32_t *__restrict__ blk_bn,
                                                        int64_t F, int32_t B, int32_t NBC, int32_t P, int32_t *__restrict__ fixed_start,
                                                        int32_t *__restrict__ fixed_col, int32_t *__restrict__ comp_lo,
                                                        int32_t *__restrict__ comp_col)
{
    const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w > P) return;
    const int64_t b = w * F;  // <= P F <= B
    fixed_start[w] = blk_group_ptr[b];
    if (w == P) return;
    const int32_t first_col = b < B ? blk_bn[b] : NBC - 1;
    fixed_col[w] = first_col;
    comp_lo[w] = blk_group_ptr[b + F];
    comp_col[w] = F > 0 ? blk_bn[b + F - 1] : first_col;
}

__global__ __launch_bounds__(256) void k_hash_keys(const uint32_t *__restrict__ n, int64_t count, uint32_t a, uint32_t R,
                                                   uint32_t *__restrict__ keys)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) keys[i] = hash_key(n[i], a, R / 9u ? R / 9u : 1u, R);
}

// Scratch memory of the build, kept between builds: freeing a few hundred megabytes costs a
// quarter of a millisecond per allocation, a good part of a build.  Two slots per device (a
// build has two scratch arenas alive at a time), grown when a build needs more, given back by
// hbp_release_workspace().  The device's lock is held for the whole of build_layout: the builds
// of one process on one device are serialised; builds on different devices are not.
constexpr int kWorkspaceDevices = 64, kWorkspaceSlots = 2;
struct Workspace { void *base = nullptr; size_t bytes = 0; };
Workspace g_workspace[kWorkspaceDevices][kWorkspaceSlots];
std::mutex g_workspace_mutex[kWorkspaceDevices];

std::mutex &workspace_mutex(int device) { return g_workspace_mutex[device >= 0 && device < kWorkspaceDevices ? device : 0]; }

int workspace_get(int device, int slot, size_t bytes, void **out)
{
    if (device < 0 || device >= kWorkspaceDevices) return HBP_ERR_INTERNAL;
    Workspace &w = g_workspace[device][slot];
    if (w.bytes < bytes) {
        if (w.base) (void)hipFree(w.base);
        w.base = nullptr;
        w.bytes = 0;
        const size_t want = bytes + bytes / 8;  // some room, so that similar matrices do not reallocate
        HBP_HIP(hipMalloc(&w.base, want));
        w.bytes = want;
    }
    *out = w.base;
    return HBP_OK;
}

// One device allocation carved into 256-byte aligned arrays: reserve() every array first,
// commit() allocates once and hands out the pointers.  hipMalloc/hipFree calls are a large part
// of the preprocessing time otherwise (each hipFree synchronises the device).  An arena is
// either handed to the caller (the handle's arrays) or lives in a workspace slot.
class Arena {
public:
    explicit Arena(bool owned_by_caller, int device = -1, int workspace_slot = -1)
        : keep_(owned_by_caller), device_(device), slot_(workspace_slot) {}
    ~Arena() { if (free_at_end_ && base_) (void)hipFree(base_); }
    template <typename T>
    void reserve(T **out, int64_t count)
    {
        reserve_bytes((void **)out, (int64_t)sizeof(T) * (count > 0 ? count : 1));
    }
    void reserve_bytes(void **out, int64_t n_bytes)
    {
        const size_t bytes = ((size_t)(n_bytes > 0 ? n_bytes : 1) + 255) & ~(size_t)255;
        slots_.push_back({out, total_});
        total_ += bytes;
    }
    int commit()
    {
        if (keep_) {
            HBP_HIP(hipMalloc(&base_, total_ ? total_ : 256));
        } else if (device_ < 0 || device_ >= kWorkspaceDevices || slot_ < 0 || slot_ >= kWorkspaceSlots) {
            HBP_HIP(hipMalloc(&base_, total_ ? total_ : 256));  // no workspace slot for it: freed when the build ends
            free_at_end_ = true;
        } else {
            const int rc = workspace_get(device_, slot_, total_ ? total_ : 256, &base_);
            if (rc != HBP_OK) return rc;
        }
        for (auto &s : slots_) *s.out = (char *)base_ + s.offset;
        return HBP_OK;
    }
    void *base() const { return base_; }

private:
    struct Slot { void **out; size_t offset; };
    std::vector<Slot> slots_;
    size_t total_ = 0;
    void *base_ = nullptr;
    bool keep_, free_at_end_ = false;
    int device_, slot_;
};

inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

#define HBP_TRY(expr) do { int rc_ = (expr); if (rc_ != HBP_OK) return rc_; } while (0)

}  // namespace

// Parameters left at "choose for me" (Section 3.1 derives its 512 x 4096 from the shared memory of
// the paper's GPUs; here they follow the matrix and the 160 KB of LDS of a gfx950 compute unit):
//   C     the widest segment of x that fits the LDS budget of a worker (32768 fp32 / 16384 fp64
//         values), or the whole vector when it is shorter: every column block less means one
//         partial sum less per row, and the partial sums are the traffic the method adds;
//   R, rounds per batch
//         from the nonzeros the sampled rows have inside one column block (the sampling pass of
//         Section 3.2, which also yields the shift a): when at least half of the sampled segments
//         hold 6 or more nonzeros, the paper's R = 512 and deep batches (8 rounds, one group at a
//         time); otherwise R = 2048 (four times fewer, fuller blocks for the same slots) and 4
//         rounds with four groups in flight.  Both thresholds are measured on MI355X.
// The sampled shift is written back into p.hash_shift, so that the build does not sample again.
int choose_block_parameters(const int32_t *csr_ptr, const int32_t *csr_col, int64_t n_rows, int64_t n_cols, int32_t value_bytes,
                            hbp_params_t &p, hipStream_t st)
{
    const int32_t max_c = value_bytes == 8 ? kMaxC64 : kMaxC;
    if (p.cols_per_block == 0) p.cols_per_block = (int32_t)std::min<int64_t>(max_c, n_cols);
    const bool need_stats = p.rows_per_block == 0 || p.rounds_per_batch == 0;
    if (!need_stats) return HBP_OK;
    if (p.cols_per_block < 1 || p.cols_per_block > max_c) return HBP_ERR_INVALID_ARGUMENT;
    int device = 0;
    HBP_HIP(hipGetDevice(&device));
    std::lock_guard<std::mutex> workspace_lock(workspace_mutex(device));
    int32_t ends[2] = {0, 0};
    HBP_HIP(hipMemcpyAsync(&ends[0], csr_ptr, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&ends[1], csr_ptr + n_rows, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HBP_HIP(hipStreamSynchronize(st));
    if (ends[0] != 0 || ends[1] < 0) return HBP_ERR_BAD_CSR_PTR;
    const int64_t nnz = ends[1];
    uint32_t host[16] = {0};
    int32_t a = 0;
    if (nnz > 0) {
        void *buf = nullptr;
        const int rc = workspace_get(device, 1, 256, &buf);
        if (rc != HBP_OK) return rc;
        uint32_t *hist = static_cast<uint32_t *>(buf);
        int32_t *d_a = reinterpret_cast<int32_t *>(hist + 16);
        HBP_HIP(hipMemsetAsync(hist, 0, 17 * sizeof(uint32_t), st));
        const int32_t S_rows = (int32_t)std::min<int64_t>(n_rows, 4096);
        k_sample_hist<<<blocks_for(S_rows, 4), 256, 0, st>>>(csr_ptr, csr_col, n_rows, nnz, p.cols_per_block, S_rows, hist);
        k_pick_shift<<<1, 64, 0, st>>>(hist, d_a);
        HBP_HIP(hipGetLastError());
        HBP_HIP(hipMemcpyAsync(host, hist, sizeof host, hipMemcpyDeviceToHost, st));
        HBP_HIP(hipMemcpyAsync(&a, d_a, sizeof a, hipMemcpyDeviceToHost, st));
        HBP_HIP(hipStreamSynchronize(st));
    }
    uint64_t segments = 0;
    for (int i = 0; i < 14; i++) segments += host[i];
    const bool long_segments = segments > 0 && 2 * (uint64_t)host[14] >= segments;
    if (p.rows_per_block == 0) p.rows_per_block = long_segments ? 512 : 2048;
    if (p.rounds_per_batch == 0) p.rounds_per_batch = long_segments ? 8 : 4;
    if (p.hash_shift < 0 && nnz > 0) p.hash_shift = a;
    return HBP_OK;
}

static int build_layout_locked(hbp_handle_s *h, const int32_t *csr_ptr, const int32_t *csr_col, const void *csr_val,
                               const hbp_params_t &p, hipStream_t st);

int build_layout(hbp_handle_s *h, const int32_t *csr_ptr, const int32_t *csr_col, const void *csr_val,
                 const hbp_params_t &p, hipStream_t st)
{
    std::lock_guard<std::mutex> workspace_lock(workspace_mutex(h->device));
    const int rc = build_layout_locked(h, csr_ptr, csr_col, csr_val, p, st);
    // A build that gives up may have kernels in flight that still use the shared workspace: they
    // have to finish before the lock is released and the next build takes the workspace over.
    if (rc != HBP_OK) (void)hipStreamSynchronize(st);
    return rc;
}

static int build_layout_locked(hbp_handle_s *h, const int32_t *csr_ptr, const int32_t *csr_col, const void *csr_val,
                               const hbp_params_t &p, hipStream_t st)
{
    const int64_t n_rows = h->n_rows, n_cols = h->n_cols;
    const int32_t R = h->R, C = h->C, W = h->W;
    const int64_t NBR = h->NBR, NBC = h->NBC, D = NBR * NBC;

    // nnz and csr_ptr[0] are needed on the host before anything can be sized
    int32_t ends[2] = {0, 0};
    HBP_HIP(hipMemcpyAsync(&ends[0], csr_ptr, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&ends[1], csr_ptr + n_rows, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HBP_HIP(hipStreamSynchronize(st));
    if (ends[0] != 0 || ends[1] < 0) return HBP_ERR_BAD_CSR_PTR;
    const int64_t nnz = ends[1];
    if (nnz >= (int64_t(1) << 31) - 64) return HBP_ERR_TOO_LARGE;
    h->nnz = nnz;

    // arrays whose size does not depend on the matrix content
    Arena own0(true);
    own0.reserve(&h->col_blk_ptr, NBC + 1);
    own0.reserve(&h->stripe_ptr, NBR + 1);
    own0.reserve(&h->ticket, (int64_t)h->P);
    own0.reserve(&h->comp_lo, (int64_t)h->P);
    own0.reserve(&h->comp_col, (int64_t)h->P);
    own0.reserve(&h->col_group_ptr, NBC + 1);
    own0.reserve(&h->fixed_start, (int64_t)h->P + 1);
    own0.reserve(&h->fixed_col, (int64_t)h->P);
    own0.reserve(&h->unit_ptr, NBR + 1);
    own0.reserve(&h->col_rank, NBC + 1);
    HBP_TRY(own0.commit());
    h->arena[0] = own0.base();
    HBP_HIP(hipMemsetAsync(h->ticket, 0, sizeof(uint32_t) * (size_t)h->P, st));
    HBP_HIP(hipMemsetAsync(h->col_blk_ptr, 0, sizeof(int32_t) * (size_t)(NBC + 1), st));
    HBP_HIP(hipMemsetAsync(h->stripe_ptr, 0, sizeof(int32_t) * (size_t)(NBR + 1), st));
    HBP_HIP(hipMemsetAsync(h->comp_lo, 0, sizeof(int32_t) * (size_t)h->P, st));
    HBP_HIP(hipMemsetAsync(h->comp_col, 0, sizeof(int32_t) * (size_t)h->P, st));
    HBP_HIP(hipMemsetAsync(h->col_group_ptr, 0, sizeof(int32_t) * (size_t)(NBC + 1), st));
    HBP_HIP(hipMemsetAsync(h->fixed_start, 0, sizeof(int32_t) * (size_t)(h->P + 1), st));
    HBP_HIP(hipMemsetAsync(h->fixed_col, 0, sizeof(int32_t) * (size_t)h->P, st));

    if (nnz == 0) {  // empty matrix: no blocks; the combine part alone writes y = 0
        h->B = h->S = h->G = 0;
        h->a = p.hash_shift >= 0 ? p.hash_shift : 0;
        Arena own1(true);
        own1.reserve(&h->blk_bm, 1); own1.reserve(&h->blk_bn, 1); own1.reserve(&h->slot_ptr, 1);
        own1.reserve(&h->blk_group_ptr, 1); own1.reserve(&h->stripe_blk, 1); own1.reserve(&h->group_ptr, 1);
        own1.reserve(&h->group_slot, 1); own1.reserve(&h->group_rounds, 1); own1.reserve(&h->row_local, 1); own1.reserve(&h->seg_len, 1); own1.reserve(&h->blk_shift, 1);
        own1.reserve(&h->col_local, 1); own1.reserve_bytes(&h->data, 8); own1.reserve_bytes(&h->partial, 8);
        own1.reserve(&h->unit_stripe, NBR + 1); own1.reserve(&h->unit_k, NBR + 2); own1.reserve(&h->multi_stripes, 1);
        HBP_TRY(own1.commit());
        h->arena[1] = own1.base();
        h->U = NBR; h->NM = 0;
        if (h->unit_slots == 0) h->unit_slots = 16384;
        k_iota_units<<<blocks_for(NBR + 1, 256), 256, 0, st>>>(h->unit_ptr, h->unit_stripe, h->unit_k, (int32_t)NBR);
        HBP_HIP(hipMemsetAsync(h->slot_ptr, 0, 4, st)); HBP_HIP(hipMemsetAsync(h->blk_group_ptr, 0, 4, st));
        HBP_HIP(hipMemsetAsync(h->group_ptr, 0, 4, st)); HBP_HIP(hipMemsetAsync(h->group_slot, 0, 4, st));
        HBP_HIP(hipMemsetAsync(h->group_rounds, 0, 4, st));
        HBP_HIP(hipStreamSynchronize(st));
        return HBP_OK;
    }

    Arena tmp(false, h->device, 0);
    const int64_t n_words = (nnz + 63) / 64;
    const int64_t scan_n = std::max<int64_t>(std::max<int64_t>(n_words, D), std::max<int64_t>(NBR, nnz / W + D)) + 1;
    uint32_t *row_bits, *seg_cnt, *word_off, *dense_cnt, *slot_off, *group_off, *blk_id, *scan_tmp, *hist, *stripe_cnt;
    uint64_t *seg_bits;
    int32_t *word_row, *seg_j, *seg_row, *seg_bn, *d_a, *d_err;
    tmp.reserve(&row_bits, (nnz + 31) / 32 + 1);
    tmp.reserve(&seg_bits, n_words);
    tmp.reserve(&seg_cnt, n_words);
    tmp.reserve(&word_off, n_words + 1);
    tmp.reserve(&word_row, n_words + 1);
    tmp.reserve(&seg_j, nnz + 1);     // S <= nnz: sized by the bound, no host round trip needed
    tmp.reserve(&seg_row, nnz);
    tmp.reserve(&seg_bn, nnz);
    tmp.reserve(&dense_cnt, D);
    tmp.reserve(&slot_off, D + 1);
    tmp.reserve(&group_off, D + 1);
    tmp.reserve(&blk_id, D + 1);
    tmp.reserve(&stripe_cnt, NBR);
    tmp.reserve(&scan_tmp, scan_n / kScanTile + 2);
    tmp.reserve(&hist, 16);
    tmp.reserve(&d_a, 1);
    tmp.reserve(&d_err, 1);
    HBP_TRY(tmp.commit());
    HBP_HIP(hipMemsetAsync(row_bits, 0, sizeof(uint32_t) * (size_t)((nnz + 31) / 32 + 1), st));
    HBP_HIP(hipMemsetAsync(dense_cnt, 0, sizeof(uint32_t) * (size_t)D, st));
    HBP_HIP(hipMemsetAsync(hist, 0, sizeof(uint32_t) * 16, st));
    HBP_HIP(hipMemsetAsync(d_err, 0, sizeof(int32_t), st));

    // Section 3.2: shift a, sampled or given
    if (p.hash_shift >= 0) {
        k_set_i32<<<1, 64, 0, st>>>(d_a, p.hash_shift);
    } else {
        const int32_t S_rows = (int32_t)std::min<int64_t>(n_rows, 4096);
        k_sample_hist<<<blocks_for(S_rows, 4), 256, 0, st>>>(csr_ptr, csr_col, n_rows, nnz, C, S_rows, hist);
        k_pick_shift<<<1, 64, 0, st>>>(hist, d_a);
    }

    // steps 1-3
    k_row_bits<<<blocks_for(n_rows, 256), 256, 0, st>>>(csr_ptr, n_rows, nnz, row_bits, d_err);
    k_word_rows<<<blocks_for(n_words + 1, 256), 256, 0, st>>>(csr_ptr, n_rows, n_words, word_row);
    int32_t shift_c = -1;  // C = 2^shift_c, or -1
    for (int32_t b = 0; b < 31; b++)
        if (C == (int32_t(1) << b)) shift_c = b;
    k_seg_flags<<<blocks_for(n_words, 4 * kWordsPerWave), 256, 0, st>>>(csr_col, row_bits, nnz, n_cols, C, shift_c, n_words,
                                                                       (p.flags & HBP_FLAG_VALIDATE) ? 1 : 0, seg_bits, seg_cnt, d_err);
    HBP_TRY(exclusive_scan<kOpIdentity>(seg_cnt, word_off, n_words, 1, scan_tmp, st));
    k_seg_emit<<<blocks_for(n_words, 4 * kWordsPerWave), 256, 0, st>>>(csr_ptr, csr_col, seg_bits, word_off, word_row, nnz, n_cols, R, C,
                                                                      shift_c, (int32_t)NBR, n_words, seg_j, seg_row, seg_bn);
    k_count_blocks<<<blocks_for(nnz, kTileSegs), 256, 0, st>>>(seg_row, seg_bn, word_off + n_words, d_err, R, (int32_t)NBR, (int32_t)NBC,
                                                               dense_cnt);
    // step 4: scans over the block table
    HBP_TRY(exclusive_scan<kOpIdentity>(dense_cnt, slot_off, D, 1, scan_tmp, st));
    HBP_TRY(exclusive_scan<kOpCeilDivW>(dense_cnt, group_off, D, (uint32_t)W, scan_tmp, st));
    HBP_TRY(exclusive_scan<kOpNonZero>(dense_cnt, blk_id, D, 1, scan_tmp, st));
    k_stripe_count<<<blocks_for(NBR, 256), 256, 0, st>>>(dense_cnt, (int32_t)NBR, (int32_t)NBC, stripe_cnt);
    HBP_TRY(exclusive_scan<kOpIdentity>(stripe_cnt, (uint32_t *)h->stripe_ptr, NBR, 1, scan_tmp, st));
    HBP_HIP(hipGetLastError());

    // the one host round trip of the build: totals (and the error word)
    uint32_t totals[3];
    int32_t err = 0, a = 0;
    HBP_HIP(hipMemcpyAsync(&totals[0], slot_off + D, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&totals[1], group_off + D, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&totals[2], blk_id + D, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&err, d_err, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&a, d_a, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipStreamSynchronize(st));
    if (err & kErrPtr) return HBP_ERR_BAD_CSR_PTR;
    if (err & kErrCol) return HBP_ERR_BAD_CSR_COL;
    const int64_t S = totals[0], G = totals[1], B = totals[2];
    h->S = S; h->G = G; h->B = B; h->a = a;

    Arena own1(true);
    own1.reserve(&h->blk_bm, B + 1); own1.reserve(&h->blk_bn, B + 1);
    own1.reserve(&h->slot_ptr, B + 1); own1.reserve(&h->blk_group_ptr, B + 1);
    own1.reserve(&h->stripe_blk, B + 1);
    own1.reserve(&h->group_ptr, G + 1); own1.reserve(&h->group_slot, G + 1); own1.reserve(&h->group_rounds, G + 1);
    own1.reserve(&h->row_local, S + 1); own1.reserve(&h->seg_len, S + 1);
    own1.reserve(&h->blk_shift, B + 1);
    if (p.flags & HBP_FLAG_KEEP_KEYS) own1.reserve(&h->slot_key, S + 1);
    // 256 elements of padding: the SpMV part reads whole aligned 256-element chunks
    own1.reserve(&h->col_local, nnz + 256); own1.reserve_bytes(&h->data, (nnz + 256) * h->value_bytes);
    own1.reserve_bytes(&h->partial, (S + 1) * h->value_bytes);
    if (h->unit_slots == 0) {
        // default: only row blocks with more than twice the average number of slots are cut
        const int64_t twice_mean = 2 * ((S + NBR - 1) / NBR);
        h->unit_slots = (int32_t)std::min<int64_t>(std::max<int64_t>(16384, twice_mean), INT32_MAX);
    }
    const int64_t max_units = NBR + S / h->unit_slots + 2;
    own1.reserve(&h->unit_stripe, max_units); own1.reserve(&h->unit_k, max_units + 1);
    own1.reserve(&h->multi_stripes, NBR);
    HBP_TRY(own1.commit());
    h->arena[1] = own1.base();
    Arena tmp2(false, h->device, 1);
    uint32_t *stripe_cum, *unit_cnt, *multi_idx;
    tmp2.reserve(&stripe_cum, B + 1); tmp2.reserve(&unit_cnt, NBR + 1); tmp2.reserve(&multi_idx, NBR + 1);
    uint32_t *bucket_len_row, *group_nnz, *group_longest, *longest_all;
    int32_t *bucket_j;
    int32_t *slot_j, *group_blk;
    tmp2.reserve(&bucket_len_row, S); tmp2.reserve(&bucket_j, S);
    tmp2.reserve(&slot_j, S); tmp2.reserve(&group_nnz, G + 1); tmp2.reserve(&group_longest, G + 1); tmp2.reserve(&longest_all, 1); tmp2.reserve(&group_blk, G + 1);
    HBP_TRY(tmp2.commit());
    HBP_HIP(hipMemsetAsync(longest_all, 0, sizeof(uint32_t), st));

    k_compact_blocks<<<blocks_for(std::max<int64_t>(D, NBC) + 1, 256), 256, 0, st>>>(
        dense_cnt, slot_off, group_off, blk_id, D, (int32_t)NBR, (int32_t)NBC, h->blk_bm, h->blk_bn, h->slot_ptr,
        h->blk_group_ptr, h->col_blk_ptr);
    k_stripe_fill<<<blocks_for(NBR, 256), 256, 0, st>>>(dense_cnt, blk_id, h->stripe_ptr, (int32_t)NBR, (int32_t)NBC,
                                                       h->stripe_blk);
    // combine work units
    k_stripe_sizes<<<blocks_for(B, 256), 256, 0, st>>>(h->stripe_blk, h->slot_ptr, (int32_t)B, stripe_cum);
    HBP_TRY(exclusive_scan<kOpIdentity>(stripe_cum, stripe_cum, B, 1, scan_tmp, st));
    k_unit_count<<<blocks_for(NBR, 256), 256, 0, st>>>(h->stripe_ptr, stripe_cum, (int32_t)NBR, h->unit_slots, unit_cnt);
    k_unit_multi<<<blocks_for(NBR, 256), 256, 0, st>>>(unit_cnt, (int32_t)NBR, multi_idx);
    HBP_TRY(exclusive_scan<kOpIdentity>(unit_cnt, (uint32_t *)h->unit_ptr, NBR, 1, scan_tmp, st));
    HBP_TRY(exclusive_scan<kOpIdentity>(multi_idx, multi_idx, NBR, 1, scan_tmp, st));
    k_unit_fill<<<blocks_for(NBR, 256), 256, 0, st>>>(h->stripe_ptr, stripe_cum, h->unit_ptr, multi_idx, (int32_t)NBR, (int32_t)B,
                                                     h->unit_stripe, h->unit_k, h->multi_stripes);
    // steps 5-6 (slot_off doubles as the per-block cursor from here on)
    const int32_t reorder = (p.flags & HBP_FLAG_NO_REORDER) ? 0 : (p.flags & HBP_FLAG_KEY_LENGTH) ? 2 : (p.flags & HBP_FLAG_BLOCK_SHIFT) ? 3 : 1;
    k_bucket<<<blocks_for(S, kTileSegs), 256, 0, st>>>(seg_j, seg_row, seg_bn, S, R, (int32_t)NBR, (int32_t)NBC, slot_off,
                                                       bucket_len_row, bucket_j);
    // The order in which k_fill takes the blocks (see stripe_walk).  Row block by
    // row block pays where a row segment is a small part of the 128-byte lines it is gathered from
    // (fewer than 4 nonzeros on average) and the blocks are large enough to keep a workgroup busy
    // (256 slots on average); measured: k_fill 2.30 -> 1.10 ms on the 4M x 1M matrix with 2 nonzeros
    // per segment, 0.79 -> 0.37 ms on the 2^20 one with 1.6; with 13 nonzeros per segment (27-point
    // stencil) or 86 slots per block (R-MAT, whose dense row blocks then also wait for a few
    // workgroups) it is slower than the layout's own order with a wavefront per group.
    const bool by_row_block = NBR >= 64 && nnz < 4 * S && S >= 256 * B;
    const int32_t parts = !by_row_block ? 0 : (int32_t)std::min<int64_t>(32, std::max<int64_t>(1, (B + NBR - 1) / NBR));
    const dim3 stripe_grid((unsigned)(8 * ((NBR + 7) / 8) * std::max(parts, 1)));
    const size_t order_cap = ((size_t)R + 63) & ~(size_t)63;
    size_t small_n2 = 1;  // the bitonic network of a small block: 8-byte words, the next power of two above min(R, 256) slots
    while (small_n2 < (size_t)std::min(R, 256)) small_n2 <<= 1;
    const size_t order_lds = std::max(sizeof(uint32_t) * (2 * order_cap + 16 * (order_cap / 64)),  // two entry arrays, 16 counters per tile
                                      sizeof(uint64_t) * small_n2);
    HBP_HIP(hipFuncSetAttribute((const void *)k_order_block, hipFuncAttributeMaxDynamicSharedMemorySize, (int)order_lds));
    k_order_block<<<dim3((unsigned)B), 256, order_lds, st>>>(bucket_len_row, bucket_j, h->slot_ptr, h->blk_group_ptr, W,
                                                            h->row_local, h->seg_len, slot_j, group_nnz, group_longest, h->group_slot,
                                                            group_blk, (uint32_t)long_rounds_of(h->heavy_rounds), longest_all,
                                                            reorder, (uint32_t)R, d_a, h->blk_shift, h->slot_key);
    HBP_TRY(exclusive_scan<kOpIdentity>(group_nnz, (uint32_t *)h->group_ptr, G, 1, scan_tmp, st));
    HBP_TRY(exclusive_scan<kOpIdentity>(group_longest, (uint32_t *)h->group_rounds, G, 1, scan_tmp, st));
    k_set_i32<<<1, 64, 0, st>>>(h->group_slot + G, (int32_t)S);
    // step 7
    // the padding behind the last group is read (and its products dropped) by lanes without an element
    HBP_HIP(hipMemsetAsync(h->col_local + nnz, 0, 256 * sizeof(uint16_t), st));
    HBP_HIP(hipMemsetAsync((char *)h->data + (size_t)nnz * h->value_bytes, 0, 256 * (size_t)h->value_bytes, st));
    if (parts == 0) {
        if (h->value_bytes == 8)
            k_fill_flat<double><<<blocks_for(G, 4), 256, 0, st>>>(csr_col, static_cast<const double *>(csr_val), h->group_ptr, h->group_slot,
                                                                  group_blk, h->blk_bn, h->seg_len, slot_j, (int32_t)G, C, nnz, h->col_local,
                                                                  static_cast<double *>(h->data));
        else
            k_fill_flat<float><<<blocks_for(G, 4), 256, 0, st>>>(csr_col, static_cast<const float *>(csr_val), h->group_ptr, h->group_slot,
                                                                 group_blk, h->blk_bn, h->seg_len, slot_j, (int32_t)G, C, nnz, h->col_local,
                                                                 static_cast<float *>(h->data));
    } else if (h->value_bytes == 8) {
        k_fill<double><<<stripe_grid, 256, 0, st>>>(h->stripe_ptr, h->stripe_blk, (int32_t)NBR, (int32_t)B, parts, csr_col,
                                                    static_cast<const double *>(csr_val), h->group_ptr, h->group_slot, h->blk_group_ptr,
                                                    h->blk_bn, h->seg_len, slot_j, C, nnz, h->col_local, static_cast<double *>(h->data));
    } else {
        k_fill<float><<<stripe_grid, 256, 0, st>>>(h->stripe_ptr, h->stripe_blk, (int32_t)NBR, (int32_t)B, parts, csr_col,
                                                   static_cast<const float *>(csr_val), h->group_ptr, h->group_slot, h->blk_group_ptr,
                                                   h->blk_bn, h->seg_len, slot_j, C, nnz, h->col_local, static_cast<float *>(h->data));
    }
    HBP_HIP(hipGetLastError());
    uint32_t n_units = 0, n_multi = 0, longest = 0;
    HBP_HIP(hipMemcpyAsync(&longest, longest_all, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&n_units, h->unit_ptr + NBR, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipMemcpyAsync(&n_multi, multi_idx + NBR, 4, hipMemcpyDeviceToHost, st));
    HBP_HIP(hipStreamSynchronize(st));
    h->U = n_units; h->NM = n_multi;
    h->longest_segment = (int32_t)longest;  // 0 unless it makes a group long
    return HBP_OK;
}

// Section 3.3: which groups are pre-assigned to which worker and which are left to competition.
int build_schedule(hbp_handle_s *h, hipStream_t st)
{
    h->first_ticket_block = -1;
    if (h->G > 0 && (h->flags & HBP_FLAG_PAPER_SCHEDULE)) {
        const int32_t NBC = (int32_t)h->NBC;
        const int64_t F = (h->B * (int64_t)h->fixed_q8) / (256 * (int64_t)h->P);
        h->first_ticket_block = F * h->P;
        k_col_group_ptr<<<blocks_for(h->NBC + 1, 256), 256, 0, st>>>(h->col_blk_ptr, h->blk_group_ptr, NBC, h->col_group_ptr);
        k_paper_schedule<<<blocks_for((int64_t)h->P + 1, 256), 256, 0, st>>>(h->blk_group_ptr, h->blk_bn, F, (int32_t)h->B, NBC, h->P,
                                                                             h->fixed_start, h->fixed_col, h->comp_lo, h->comp_col);
    } else if (h->G > 0) {
        const int32_t NBC = (int32_t)h->NBC;
        k_col_group_ptr<<<blocks_for(h->NBC + 1, 256), 256, 0, st>>>(h->col_blk_ptr, h->blk_group_ptr, NBC, h->col_group_ptr);
        const Weights wt{h->group_ptr, h->group_slot, h->group_rounds, (int64_t)h->slot_weight, (int64_t)h->round_weight,
                         (int64_t)h->group_weight};
        k_col_rank<<<1, 256, 0, st>>>(h->col_group_ptr, NBC, h->col_rank);
        k_fixed_start<<<blocks_for((int64_t)h->P + 1, 256), 256, 0, st>>>(h->col_group_ptr, wt, h->col_rank, (int64_t)h->column_weight,
                                                                          NBC, (int32_t)h->G, h->P, h->fixed_start, h->fixed_col);
        k_comp_lo<<<blocks_for((int64_t)h->P, 256), 256, 0, st>>>(h->col_group_ptr, wt, NBC, h->P, h->fixed_q8, h->fixed_start,
                                                                  h->fixed_col, h->comp_lo, h->comp_col);
    }
    HBP_HIP(hipGetLastError());
    HBP_HIP(hipStreamSynchronize(st));
    return HBP_OK;
}

int release_workspace()
{
    int rc = HBP_OK;
    for (int device = 0; device < kWorkspaceDevices; device++) {
        std::lock_guard<std::mutex> workspace_lock(workspace_mutex(device));
        for (auto &w : g_workspace[device]) {
            if (w.base && hipFree(w.base) != hipSuccess) rc = HBP_ERR_HIP;
            w.base = nullptr;
            w.bytes = 0;
        }
    }
    return rc;
}

int hash_keys(const uint32_t *n, int64_t count, int32_t a, int32_t R, uint32_t *keys, hipStream_t st)
{
    if (count > 0) k_hash_keys<<<blocks_for(count, 256), 256, 0, st>>>(n, count, (uint32_t)a, (uint32_t)R, keys);
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

int derive_add_sign(const hbp_handle_s *h, int32_t *d_out, hipStream_t st)
{
    if (h->G > 0)
        k_add_sign<<<blocks_for(h->G, 4), 256, 0, st>>>(h->group_ptr, h->group_slot, h->seg_len, (int32_t)h->G, d_out);
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

}  // namespace hbp
