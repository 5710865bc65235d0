// Two-step HBP SpMV (Fig. 1, Algorithm 3, Section 3.3) and the in-repo CSR baselines.
//
// SpMV part: P persistent workgroups ("workers").  A worker first runs its F fixed blocks,
// a contiguous piece of the column-major block list, then claims chunks of the remaining
// (competitive) blocks through an atomic ticket counter until none are left.  Before it
// touches a block column it stages that column's slice of x in LDS; blocks of one column are
// adjacent in the list, so a slice is staged once per run of blocks.  Each wavefront takes
// groups of the run; lane q owns slot q of the group and walks its row round by round.  The
// distance add_sign of Algorithm 3 is not read from memory: in round k the lanes still alive
// are known from a ballot over the lane lengths, and a lane's element is the base of the
// round plus the number of live lanes below it.
//
// Combine part: one workgroup per row block adds the per-slot partial sums of that row
// block's blocks into an LDS copy of the y slice and writes it out, zeros included.
#include "hbp_internal.h"

namespace hbp {
namespace {

__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_spmv_part(Layout L, int32_t P, int32_t F, int32_t chunk,
                                                       const float *__restrict__ x, float *__restrict__ partial,
                                                       uint32_t *__restrict__ ticket)
{
    extern __shared__ float xs[];  // the staged vector segment, C floats
    __shared__ int32_t sh_ticket;
    constexpr int kWaves = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int staged_bn = -1;

    auto run_blocks = [&](int32_t e0, int32_t e1) {  // list entries [e0, e1), uniform over the workgroup
        int32_t b = e0;
        while (b < e1) {
            const int32_t bn = L.blk_bn[b];
            const int32_t be = min(e1, L.col_blk_ptr[bn + 1]);  // end of the run of blocks in column bn
            if (bn != staged_bn) {
                __syncthreads();  // every wavefront is done with the previous slice
                const int64_t c0 = (int64_t)bn * L.C;
                const int32_t width = (int32_t)min((int64_t)L.C, L.n_cols - c0);
                for (int32_t i = threadIdx.x; i < width; i += THREADS) xs[i] = x[c0 + i];
                __syncthreads();
                staged_bn = bn;
            }
            const int32_t g1 = L.blk_group_ptr[be];
            for (int32_t g = L.blk_group_ptr[b] + wave; g < g1; g += kWaves) {
                const int32_t s0 = L.group_slot[g], cnt = L.group_slot[g + 1] - s0;
                const int32_t n = lane < cnt ? L.seg_len[s0 + lane] : 0;
                int64_t base = L.group_ptr[g];
                float acc = 0.f;
                for (int32_t k = 0;; k++) {
                    const uint64_t live = __ballot(k < n);
                    if (!live) break;
                    if (k < n) {
                        const int64_t j = base + lanes_below(live);
                        acc += L.data[j] * xs[L.col_local[j]];
                    }
                    base += __popcll(live);
                }
                if (lane < cnt) partial[s0 + lane] = acc;
            }
            b = be;
        }
    };

    // fixed part: worker w owns list entries [w F, (w+1) F)
    run_blocks((int32_t)blockIdx.x * F, ((int32_t)blockIdx.x + 1) * F);
    // competitive part: tickets hand out chunks of the rest of the list in order
    const int64_t first = (int64_t)P * F;
    for (;;) {
        if (threadIdx.x == 0) sh_ticket = (int32_t)atomicAdd(ticket, 1u);
        __syncthreads();
        const int64_t e0 = first + (int64_t)sh_ticket * chunk;
        __syncthreads();
        if (e0 >= L.B) break;
        run_blocks((int32_t)e0, (int32_t)min((int64_t)L.B, e0 + chunk));
    }
}

// Combine part.  Also re-arms the ticket counter for the next call (the SpMV part of this
// call has finished: same stream).
template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_combine(Layout L, const float *__restrict__ partial, float *__restrict__ y,
                                                     uint32_t *__restrict__ ticket)
{
    extern __shared__ float ys[];  // R floats
    const int32_t bm = blockIdx.x;
    if (bm == 0 && threadIdx.x == 0) *ticket = 0u;
    const int64_t r0 = (int64_t)bm * L.R;
    const int32_t rows = (int32_t)min((int64_t)L.R, L.n_rows - r0);
    for (int32_t i = threadIdx.x; i < rows; i += THREADS) ys[i] = 0.f;
    __syncthreads();
    for (int32_t k = L.stripe_ptr[bm]; k < L.stripe_ptr[bm + 1]; k++) {
        const int32_t b = L.stripe_blk[k];
        const int32_t s1 = L.slot_ptr[b + 1];
        for (int32_t s = L.slot_ptr[b] + threadIdx.x; s < s1; s += THREADS)
            atomicAdd(&ys[L.row_local[s]], partial[s]);  // LDS atomic; a block holds a row at most once
    }
    __syncthreads();
    for (int32_t i = threadIdx.x; i < rows; i += THREADS) y[r0 + i] = ys[i];
}

// ------------------------------------------------------------------ CSR baselines (Algorithm 1)

__global__ __launch_bounds__(256) void k_csr_scalar(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                    const float *__restrict__ val, const float *__restrict__ x,
                                                    float *__restrict__ y, int64_t n_rows)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_rows) return;
    float sum = 0.f;
    for (int32_t j = ptr[i]; j < ptr[i + 1]; j++) sum += val[j] * x[col[j]];
    y[i] = sum;
}

__global__ __launch_bounds__(256) void k_csr_vector(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                    const float *__restrict__ val, const float *__restrict__ x,
                                                    float *__restrict__ y, int64_t n_rows)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n_rows) return;
    float sum = 0.f;
    for (int32_t j = ptr[i] + lane; j < ptr[i + 1]; j += 64) sum += val[j] * x[col[j]];
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d);
    if (lane == 0) y[i] = sum;
}

}  // namespace

Layout hbp_view(const hbp_handle_s *h)
{
    Layout L;
    L.R = h->R; L.C = h->C; L.W = h->W;
    L.B = (int32_t)h->B; L.S = (int32_t)h->S; L.G = (int32_t)h->G;
    L.NBR = (int32_t)h->NBR; L.NBC = (int32_t)h->NBC;
    L.n_rows = h->n_rows; L.n_cols = h->n_cols;
    L.blk_bm = h->blk_bm; L.blk_bn = h->blk_bn; L.slot_ptr = h->slot_ptr; L.blk_group_ptr = h->blk_group_ptr;
    L.col_blk_ptr = h->col_blk_ptr; L.stripe_ptr = h->stripe_ptr; L.stripe_blk = h->stripe_blk;
    L.group_ptr = h->group_ptr; L.group_slot = h->group_slot;
    L.row_local = h->row_local; L.seg_len = h->seg_len; L.col_local = h->col_local; L.data = h->data;
    return L;
}

// Workers the schedule is built for when the caller does not say: as many workgroups as fit
// on the device at once given the LDS a vector segment takes.
int default_workers(int device, int32_t C, int32_t *threads_out, int32_t *workers_out)
{
    hipDeviceProp_t prop;
    HBP_HIP(hipGetDeviceProperties(&prop, device));
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const size_t lds = (size_t)C * sizeof(float) + 64;
    const int threads = lds > 80 * 1024 ? 1024 : 512;
    int per_cu = (int)((160 * 1024) / lds);
    const int by_threads = 2048 / threads;
    if (per_cu > by_threads) per_cu = by_threads;
    if (per_cu < 1) per_cu = 1;
    *threads_out = threads;
    *workers_out = cus * per_cu;
    return HBP_OK;
}

int launch_spmv_part(const hbp_handle_s *h, const float *x, hipStream_t st)
{
    const Layout L = hbp_view(h);
    const size_t lds = (size_t)h->C * sizeof(float);
    if (h->threads == 1024) {
        HBP_HIP(hipFuncSetAttribute((const void *)k_spmv_part<1024>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        k_spmv_part<1024><<<dim3((unsigned)h->P), 1024, lds, st>>>(L, h->P, h->F, h->claim_chunk, x, h->partial, h->ticket);
    } else if (h->threads == 512) {
        HBP_HIP(hipFuncSetAttribute((const void *)k_spmv_part<512>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        k_spmv_part<512><<<dim3((unsigned)h->P), 512, lds, st>>>(L, h->P, h->F, h->claim_chunk, x, h->partial, h->ticket);
    } else {
        HBP_HIP(hipFuncSetAttribute((const void *)k_spmv_part<256>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        k_spmv_part<256><<<dim3((unsigned)h->P), 256, lds, st>>>(L, h->P, h->F, h->claim_chunk, x, h->partial, h->ticket);
    }
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

int launch_combine(const hbp_handle_s *h, float *y, hipStream_t st)
{
    const Layout L = hbp_view(h);
    k_combine<256><<<dim3((unsigned)h->NBR), 256, (size_t)h->R * sizeof(float), st>>>(L, h->partial, y, h->ticket);
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

int launch_csr(int kind, const int32_t *ptr, const int32_t *col, const float *val, const float *x, float *y,
               int64_t n_rows, hipStream_t st)
{
    if (kind == 0)
        k_csr_scalar<<<dim3((unsigned)((n_rows + 255) / 256)), 256, 0, st>>>(ptr, col, val, x, y, n_rows);
    else
        k_csr_vector<<<dim3((unsigned)((n_rows + 3) / 4)), 256, 0, st>>>(ptr, col, val, x, y, n_rows);
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

}  // namespace hbp
