// C ABI of libhbp: argument checking, handle lifetime, export and timing hooks.
#include "hbp_internal.h"

#include <algorithm>
#include <chrono>
#include <cstring>
#include <mutex>
#include <new>

namespace hbp {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace hbp

namespace {

struct DeviceGuard {  // makes the handle's device current for the duration of a call
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int device)
    {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != device && hipSetDevice(device) != hipSuccess) ok = false;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

void free_arrays(hbp_handle_s *h)
{
    for (void *p : h->arena)
        if (p) (void)hipFree(p);
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// hbp_spmv_static_scratch: the per-slot partial sums and the claim counters of one SpMV in a
// fixed array of the library instead of the handle's own buffers.
constexpr size_t kStaticTicketBytes = 65536 * sizeof(uint32_t);     // the largest worker count
constexpr size_t kStaticScratchBytes = size_t(32) << 20;            // 32 MiB per device
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

__global__ __launch_bounds__(256) void k_clear_u32(uint32_t *p, int32_t n)
{
    const int32_t i = (int32_t)(blockIdx.x * 256 + threadIdx.x);
    if (i < n) p[i] = 0u;
}

// Device address of `scratch` on each device, looked up once with that device current (every GPU
// holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_static_scratch_mutex;
void *g_static_scratch[kMaxDevices] = {};

int static_scratch_address(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return HBP_ERR_INVALID_ARGUMENT;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[device]) {
        void *p = nullptr;
        HBP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));  // the caller has made `device` current
        g_static_scratch[device] = p;
    }
    *out = g_static_scratch[device];
    return HBP_OK;
}

}  // namespace

extern "C" {

int hbp_default_params(hbp_params_t *p)
{
    if (!p) return HBP_ERR_INVALID_ARGUMENT;
    p->rows_per_block = 0;
    p->cols_per_block = 0;
    p->group_width = 64;
    p->num_workers = 0;
    p->fixed_fraction_q8 = -1;
    p->hash_shift = -1;
    p->claim_chunk = 0;
    p->threads_per_worker = 0;
    p->rounds_per_batch = 0;
    p->slot_weight = -1;
    p->group_weight = -1;
    p->combine_unit_slots = 0;
    p->round_weight = -1;
    p->column_weight = -1;
    p->heavy_group_rounds = 0;
    p->flags = HBP_FLAG_VALIDATE;
    return HBP_OK;
}

static int build_any(int32_t value_bytes, const int32_t *csr_ptr, const int32_t *csr_col, const void *csr_val, int64_t n_rows,
                     int64_t n_cols, const hbp_params_t *params, void *stream, hbp_handle_t *out)
{
    if (!out) return HBP_ERR_INVALID_ARGUMENT;
    *out = nullptr;
    if (!csr_ptr || !csr_col || !csr_val || n_rows < 1 || n_cols < 1) return HBP_ERR_INVALID_ARGUMENT;
    if (n_rows >= (int64_t(1) << 31) - 1 || n_cols >= (int64_t(1) << 31) - 1) return HBP_ERR_TOO_LARGE;
    hbp_params_t p;
    hbp_default_params(&p);
    if (params) p = *params;
    if (p.group_width == 0) p.group_width = 64;
    if (p.fixed_fraction_q8 < 0) p.fixed_fraction_q8 = 240;
    if (p.heavy_group_rounds == 0) p.heavy_group_rounds = 2048;
    const int32_t max_r = value_bytes == 8 ? hbp::kMaxR64 : hbp::kMaxR, max_c = value_bytes == 8 ? hbp::kMaxC64 : hbp::kMaxC;
    if (p.rows_per_block < 0 || p.cols_per_block < 0 || p.rows_per_block > max_r || p.cols_per_block > max_c) return HBP_ERR_INVALID_ARGUMENT;
    {
        // whatever was left to the library is chosen from the matrix now (one sampling pass)
        const int rc_choice = hbp::choose_block_parameters(csr_ptr, csr_col, n_rows, n_cols, value_bytes, p, (hipStream_t)stream);
        if (rc_choice != HBP_OK) return rc_choice;
    }
    if (p.rows_per_block < 1 || p.rows_per_block > max_r || p.cols_per_block < 1 || p.cols_per_block > max_c ||
        p.group_width < 1 || p.group_width > hbp::kWave || p.num_workers < 0 || p.num_workers > 65536 ||
        p.fixed_fraction_q8 > 256 || p.hash_shift > 12 || p.claim_chunk < 0 || p.claim_chunk > 1024 || p.slot_weight > 64 || p.group_weight > 4096 ||
        (p.combine_unit_slots != 0 && p.combine_unit_slots < 64) || p.round_weight > 1024 || p.column_weight > (1 << 24) || p.heavy_group_rounds < 1 ||
        (p.threads_per_worker != 0 && p.threads_per_worker != 256 && p.threads_per_worker != 512 &&
         p.threads_per_worker != 1024) ||
        (p.rounds_per_batch != 0 && p.rounds_per_batch != 2 && p.rounds_per_batch != 4 && p.rounds_per_batch != 8 &&
         p.rounds_per_batch != 9 && p.rounds_per_batch != 16))
        return HBP_ERR_INVALID_ARGUMENT;

    const auto t0 = std::chrono::steady_clock::now();
    hbp_handle_s *h = new (std::nothrow) hbp_handle_s;
    if (!h) return HBP_ERR_OUT_OF_MEMORY;
    std::memset(h, 0, sizeof *h);
    if (hipGetDevice(&h->device) != hipSuccess) { delete h; return HBP_ERR_HIP; }
    h->n_rows = n_rows; h->n_cols = n_cols;
    h->value_bytes = value_bytes;
    h->flags = p.flags;
    h->first_ticket_block = -1;
    h->R = p.rows_per_block; h->C = p.cols_per_block; h->W = p.group_width;
    h->NBR = (n_rows + h->R - 1) / h->R;
    h->NBC = (n_cols + h->C - 1) / h->C;
    h->claim_chunk = p.claim_chunk;
    if (h->claim_chunk == 0)  // two draws per wavefront; a draw is 8 / 4 / 1 groups for 2 / 4 / more rounds per batch
        h->claim_chunk = p.rounds_per_batch == 2 ? 16 : p.rounds_per_batch == 4 ? 8 : 2;
    int rc = HBP_OK;
    if (h->NBR * h->NBC > hbp::kMaxDense) rc = HBP_ERR_TOO_LARGE;
    int32_t threads = 0, workers = 0;
    if (rc == HBP_OK) rc = hbp::default_workers(h->device, h->C, value_bytes, p.threads_per_worker, &threads, &workers);
    if (rc == HBP_OK) {
        h->threads = threads;
        h->unroll = p.rounds_per_batch ? p.rounds_per_batch : 8;
        h->fixed_q8 = p.fixed_fraction_q8;
        h->unit_slots = p.combine_unit_slots;
        h->heavy_rounds = p.heavy_group_rounds;
        h->P = p.num_workers > 0 ? p.num_workers : workers;
        rc = hbp::build_layout(h, csr_ptr, csr_col, csr_val, p, (hipStream_t)stream);
    }
    if (rc != HBP_OK) {
        (void)hipStreamSynchronize((hipStream_t)stream);
        free_arrays(h);
        delete h;
        return rc;
    }
    {
        // Schedule weights, in units of one nonzero, where the caller left them open.  They are costs of
        // the SpMV-part kernel on MI355X, not properties of a matrix: measured over workers with very
        // different mixes, a group costs a wavefront 18 ns, a round 3 ns, a slot 0.6 ns and entering a
        // block column costs the worker 19 us, next to 0.03 ns per nonzero while the wavefront waits for
        // its loads anyway (groups of a few hundred nonzeros).  Groups of 512 nonzeros and more are
        // streamed at the worker's share of the memory bandwidth instead (0.3 ns per nonzero): the same
        // costs are a tenth as many nonzeros there.
        const bool streamed = h->G > 0 && h->nnz >= 512 * h->G;
        h->slot_weight = p.slot_weight >= 0 ? p.slot_weight : streamed ? 2 : 20;
        h->group_weight = p.group_weight >= 0 ? p.group_weight : streamed ? 60 : 600;
        h->round_weight = p.round_weight >= 0 ? p.round_weight : streamed ? 10 : 100;
        h->column_weight = p.column_weight >= 0 ? p.column_weight : streamed ? 60000 : 600000;
    }
    if (p.num_workers == 0) {
        // device default: no more workers than the groups can keep busy, one group per wavefront
        const int64_t waves = h->threads / hbp::kWave;
        const int64_t useful = std::max<int64_t>(1, (h->G + waves - 1) / waves);
        if (useful < h->P) h->P = (int32_t)useful;
    }
    rc = hbp::build_schedule(h, (hipStream_t)stream);
    if (rc != HBP_OK) {
        free_arrays(h);
        delete h;
        return rc;
    }
    h->build_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
    *out = h;
    return HBP_OK;
}

static int spmv_any(int32_t value_bytes, hbp_handle_t h, const void *x, void *y, void *stream)
{
    if (!h || !x || !y || h->value_bytes != value_bytes) return HBP_ERR_INVALID_ARGUMENT;
    DeviceGuard guard(h->device);
    if (!guard.ok) return HBP_ERR_HIP;
    const hbp::SpmvScratch own{h->partial, h->ticket};
    int rc = hbp::launch_spmv_part(h, x, y, (hipStream_t)stream, own);
    if (rc != HBP_OK) return rc;
    return hbp::launch_combine(h, y, (hipStream_t)stream, own);
}

static int spmv_timed_any(int32_t value_bytes, hbp_handle_t h, const void *x, void *y, void *stream, int iters, float *ms_part,
                          float *ms_combine, float *ms_total)
{
    if (!h || !x || !y || h->value_bytes != value_bytes || iters < 1 || iters > 100000) return HBP_ERR_INVALID_ARGUMENT;
    DeviceGuard guard(h->device);
    if (!guard.ok) return HBP_ERR_HIP;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    double part = 0, comb = 0, total = 0;
    // every HIP call goes through `check`, so that the events are destroyed on every way out
    hipError_t err = hipSuccess;
    auto check = [&](hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; return err == hipSuccess; };
    int rc = HBP_OK;
    const hbp::SpmvScratch own{h->partial, h->ticket};
    for (auto &e : ev)
        if (!check(hipEventCreate(&e))) break;
    for (int i = 0; i < iters && rc == HBP_OK && err == hipSuccess; i++) {
        if (!check(hipEventRecord(ev[0], st))) break;
        rc = hbp::launch_spmv_part(h, x, y, st, own);
        if (!check(hipEventRecord(ev[1], st))) break;
        if (rc == HBP_OK) rc = hbp::launch_combine(h, y, st, own);
        if (!check(hipEventRecord(ev[2], st))) break;
        if (!check(hipEventSynchronize(ev[2])) || rc != HBP_OK) break;
        float a = 0, b = 0, c = 0;
        if (!check(hipEventElapsedTime(&a, ev[0], ev[1])) || !check(hipEventElapsedTime(&b, ev[1], ev[2])) ||
            !check(hipEventElapsedTime(&c, ev[0], ev[2])))
            break;
        part += a; comb += b; total += c;
    }
    if (err != hipSuccess || rc != HBP_OK) (void)hipStreamSynchronize(st);  // nothing of this call is left in flight
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
    if (rc != HBP_OK) return rc;
    HBP_HIP(err);
    if (ms_part) *ms_part = (float)(part / iters);
    if (ms_combine) *ms_combine = (float)(comb / iters);
    if (ms_total) *ms_total = (float)(total / iters);
    return HBP_OK;
}

int hbp_free(hbp_handle_t h)
{
    if (!h) return HBP_OK;
    DeviceGuard guard(h->device);
    (void)hipDeviceSynchronize();
    free_arrays(h);
    delete h;
    return HBP_OK;
}

int hbp_get_info(hbp_handle_t h, hbp_info_t *info)
{
    if (!h || !info) return HBP_ERR_INVALID_ARGUMENT;
    std::memset(info, 0, sizeof *info);
    info->n_rows = h->n_rows; info->n_cols = h->n_cols; info->nnz = h->nnz;
    info->rows_per_block = h->R; info->cols_per_block = h->C; info->group_width = h->W;
    info->hash_shift = h->a;
    info->hash_b = h->R / 9 > 0 ? h->R / 9 : 1;
    info->row_blocks = h->NBR; info->col_blocks = h->NBC;
    info->blocks = h->B; info->slots = h->S; info->groups = h->G;
    info->num_workers = h->P; info->fixed_fraction_q8 = h->fixed_q8; info->claim_chunk = h->claim_chunk;
    info->threads_per_worker = h->threads;
    info->rounds_per_batch = h->unroll;
    info->slot_weight = h->slot_weight;
    info->group_weight = h->group_weight;
    info->combine_unit_slots = h->unit_slots;
    info->round_weight = h->round_weight;
    info->column_weight = h->column_weight;
    info->heavy_group_rounds = h->heavy_rounds;
    info->combine_units = h->U;
    info->split_row_blocks = h->NM;
    info->value_bytes = h->value_bytes;
    info->first_ticket_block = h->first_ticket_block;
    const int64_t blk = 4 * (4 * (h->B + 1) + h->B + (h->NBC + 1) + (h->NBR + 1));
    const int64_t grp = 4 * 2 * (h->G + 1);
    const int64_t vb = h->value_bytes;
    info->bytes_layout = blk + grp + 2 * 2 * h->S + (2 + vb) * h->nnz;
    // SpMV part: col + data per nonzero, seg_len per slot, both group arrays, the block arrays it
    // reads (blk_bn, blk_group_ptr, col_blk_ptr), x once, one partial sum written per slot.
    info->bytes_spmv_part = (2 + vb) * h->nnz + 2 * h->S + grp + 4 * (2 * (h->B + 1) + h->NBC + 1) + vb * h->n_cols + vb * h->S;
    // combine: partial sum + row_local per slot, stripe index and slot_ptr, y written once.
    info->bytes_combine = (2 + vb) * h->S + 4 * ((h->NBR + 1) + 2 * h->B + 1) + vb * h->n_rows;
    info->build_ms = h->build_ms;
    return HBP_OK;
}

int hbp_export(hbp_handle_t h, int which, void *host_dst, size_t capacity, size_t *bytes_out)
{
    if (!h) return HBP_ERR_INVALID_ARGUMENT;
    DeviceGuard guard(h->device);
    if (!guard.ok) return HBP_ERR_HIP;
    const void *src = nullptr;
    size_t bytes = 0;
    switch (which) {
    case HBP_ARRAY_BLK_BM: src = h->blk_bm; bytes = 4 * (size_t)h->B; break;
    case HBP_ARRAY_BLK_BN: src = h->blk_bn; bytes = 4 * (size_t)h->B; break;
    case HBP_ARRAY_SLOT_PTR: src = h->slot_ptr; bytes = 4 * (size_t)(h->B + 1); break;
    case HBP_ARRAY_BLK_GROUP_PTR: src = h->blk_group_ptr; bytes = 4 * (size_t)(h->B + 1); break;
    case HBP_ARRAY_COL_BLK_PTR: src = h->col_blk_ptr; bytes = 4 * (size_t)(h->NBC + 1); break;
    case HBP_ARRAY_STRIPE_PTR: src = h->stripe_ptr; bytes = 4 * (size_t)(h->NBR + 1); break;
    case HBP_ARRAY_STRIPE_BLK: src = h->stripe_blk; bytes = 4 * (size_t)h->B; break;
    case HBP_ARRAY_GROUP_PTR: src = h->group_ptr; bytes = 4 * (size_t)(h->G + 1); break;
    case HBP_ARRAY_GROUP_SLOT: src = h->group_slot; bytes = 4 * (size_t)(h->G + 1); break;
    case HBP_ARRAY_ROW_LOCAL: src = h->row_local; bytes = 2 * (size_t)h->S; break;
    case HBP_ARRAY_SEG_LEN: src = h->seg_len; bytes = 2 * (size_t)h->S; break;
    case HBP_ARRAY_COL_LOCAL: src = h->col_local; bytes = 2 * (size_t)h->nnz; break;
    case HBP_ARRAY_DATA: src = h->data; bytes = (size_t)h->value_bytes * (size_t)h->nnz; break;
    case HBP_ARRAY_ADD_SIGN: bytes = 4 * (size_t)h->nnz; break;
    case HBP_ARRAY_PARTIAL: src = h->partial; bytes = (size_t)h->value_bytes * (size_t)h->S; break;
    case HBP_ARRAY_COL_GROUP_PTR: src = h->col_group_ptr; bytes = 4 * (size_t)(h->NBC + 1); break;
    case HBP_ARRAY_COMP_LO: src = h->comp_lo; bytes = 4 * (size_t)h->P; break;
    case HBP_ARRAY_COMP_COL: src = h->comp_col; bytes = 4 * (size_t)h->P; break;
    case HBP_ARRAY_FIXED_START: src = h->fixed_start; bytes = 4 * (size_t)(h->P + 1); break;
    case HBP_ARRAY_FIXED_COL: src = h->fixed_col; bytes = 4 * (size_t)h->P; break;
    case HBP_ARRAY_UNIT_PTR: src = h->unit_ptr; bytes = 4 * (size_t)(h->NBR + 1); break;
    case HBP_ARRAY_UNIT_STRIPE: src = h->unit_stripe; bytes = 4 * (size_t)h->U; break;
    case HBP_ARRAY_UNIT_K: src = h->unit_k; bytes = 4 * (size_t)(h->U + 1); break;
    case HBP_ARRAY_MULTI_STRIPES: src = h->multi_stripes; bytes = 4 * (size_t)h->NM; break;
    case HBP_ARRAY_GROUP_ROUNDS: src = h->group_rounds; bytes = 4 * (size_t)(h->G + 1); break;
    case HBP_ARRAY_SLOT_KEY:
        if (!h->slot_key) return HBP_ERR_INVALID_ARGUMENT;  // built without HBP_FLAG_KEEP_KEYS
        src = h->slot_key; bytes = 4 * (size_t)h->S; break;
    case HBP_ARRAY_BLK_SHIFT: src = h->blk_shift; bytes = 4 * (size_t)h->B; break;
    default: return HBP_ERR_INVALID_ARGUMENT;
    }
    if (bytes_out) *bytes_out = bytes;
    if (!host_dst) return HBP_OK;
    if (capacity < bytes) return HBP_ERR_INVALID_ARGUMENT;
    if (bytes == 0) return HBP_OK;
    HBP_HIP(hipDeviceSynchronize());
    if (which == HBP_ARRAY_ADD_SIGN) {
        int32_t *tmp = nullptr;
        HBP_HIP(hipMalloc((void **)&tmp, bytes));
        int rc = hbp::derive_add_sign(h, tmp, nullptr);
        hipError_t e = rc == HBP_OK ? hipMemcpy(host_dst, tmp, bytes, hipMemcpyDeviceToHost) : hipSuccess;
        (void)hipFree(tmp);
        if (rc != HBP_OK) return rc;
        HBP_HIP(e);
        return HBP_OK;
    }
    HBP_HIP(hipMemcpy(host_dst, src, bytes, hipMemcpyDeviceToHost));
    return HBP_OK;
}

static int csr_any(int32_t value_bytes, int kind, const int32_t *csr_ptr, const int32_t *csr_col, const void *csr_val, const void *x,
                   void *y, int64_t n_rows, void *stream)
{
    if (!csr_ptr || !csr_col || !csr_val || !x || !y || n_rows < 1 ||
        n_rows >= (int64_t(1) << 31) - 1)
        return HBP_ERR_INVALID_ARGUMENT;
    return hbp::launch_csr(kind, value_bytes, csr_ptr, csr_col, csr_val, x, y, n_rows, (hipStream_t)stream);
}

int hbp_build(const int32_t *csr_ptr, const int32_t *csr_col, const float *csr_val, int64_t n_rows, int64_t n_cols,
              const hbp_params_t *params, void *stream, hbp_handle_t *out)
{
    return build_any(4, csr_ptr, csr_col, csr_val, n_rows, n_cols, params, stream, out);
}

int hbp_build_f64(const int32_t *csr_ptr, const int32_t *csr_col, const double *csr_val, int64_t n_rows, int64_t n_cols,
                  const hbp_params_t *params, void *stream, hbp_handle_t *out)
{
    return build_any(8, csr_ptr, csr_col, csr_val, n_rows, n_cols, params, stream, out);
}

int hbp_spmv(hbp_handle_t h, const float *x, float *y, void *stream) { return spmv_any(4, h, x, y, stream); }

int hbp_spmv_f64(hbp_handle_t h, const double *x, double *y, void *stream) { return spmv_any(8, h, x, y, stream); }

int hbp_spmv_static_scratch(hbp_handle_t h, const float *x, float *y, void *stream)
{
    if (!h || !x || !y || h->value_bytes != 4) return HBP_ERR_INVALID_ARGUMENT;
    // the claim counters take the first 256 KiB, the partial sums (one fp32 value per slot) the rest
    if ((size_t)h->P * sizeof(uint32_t) > kStaticTicketBytes ||
        (size_t)h->S * sizeof(float) > kStaticScratchBytes - kStaticTicketBytes)
        return HBP_ERR_TOO_LARGE;
    DeviceGuard guard(h->device);
    if (!guard.ok) return HBP_ERR_HIP;
    void *base = nullptr;
    int rc = static_scratch_address(h->device, &base);
    if (rc != HBP_OK) return rc;
    const hbp::SpmvScratch fixed{static_cast<unsigned char *>(base) + kStaticTicketBytes, static_cast<uint32_t *>(base)};
    // whatever the last call on this device left in the counters goes (a fill kernel, not a memset
    // node: the call may be recorded into a HIP graph)
    k_clear_u32<<<dim3((unsigned)((h->P + 255) / 256)), 256, 0, (hipStream_t)stream>>>(fixed.ticket, h->P);
    HBP_HIP(hipGetLastError());
    rc = hbp::launch_spmv_part(h, x, y, (hipStream_t)stream, fixed);
    if (rc != HBP_OK) return rc;
    return hbp::launch_combine(h, y, (hipStream_t)stream, fixed);
}

int hbp_spmv_timed(hbp_handle_t h, const float *x, float *y, void *stream, int iters, float *ms_part, float *ms_combine,
                   float *ms_total)
{
    return spmv_timed_any(4, h, x, y, stream, iters, ms_part, ms_combine, ms_total);
}

int hbp_spmv_timed_f64(hbp_handle_t h, const double *x, double *y, void *stream, int iters, float *ms_part, float *ms_combine,
                       float *ms_total)
{
    return spmv_timed_any(8, h, x, y, stream, iters, ms_part, ms_combine, ms_total);
}

int hbp_csr_spmv(int kind, const int32_t *csr_ptr, const int32_t *csr_col, const float *csr_val, const float *x, float *y,
                 int64_t n_rows, void *stream)
{
    return csr_any(4, kind, csr_ptr, csr_col, csr_val, x, y, n_rows, stream);
}

int hbp_csr_spmv_f64(int kind, const int32_t *csr_ptr, const int32_t *csr_col, const double *csr_val, const double *x, double *y,
                     int64_t n_rows, void *stream)
{
    return csr_any(8, kind, csr_ptr, csr_col, csr_val, x, y, n_rows, stream);
}

const char *hbp_status_string(int status)
{
    switch (status) {
    case HBP_OK: return "ok";
    case HBP_ERR_INVALID_ARGUMENT: return "invalid argument";
    case HBP_ERR_BAD_CSR_PTR: return "csr_ptr is not a valid row pointer array";
    case HBP_ERR_BAD_CSR_COL: return "csr_col has an out-of-range or unsorted column index";
    case HBP_ERR_TOO_LARGE: return "matrix or block table too large";
    case HBP_ERR_OUT_OF_MEMORY: return "out of device memory";
    case HBP_ERR_HIP: return "HIP runtime error";
    case HBP_ERR_INTERNAL: return "internal error";
    default: return "unknown status";
    }
}

int hbp_last_hip_error(void) { return hbp::g_last_hip_error; }

int hbp_release_workspace(void) { return hbp::release_workspace(); }

int hbp_hash_keys(const uint32_t *n, int64_t count, int32_t a, int32_t rows_per_block, uint32_t *keys, void *stream)
{
    if (count < 0 || (count > 0 && (!n || !keys)) || a < 0 || a > 12 || rows_per_block < 1 || rows_per_block > hbp::kMaxR)
        return HBP_ERR_INVALID_ARGUMENT;
    return hbp::hash_keys(n, count, a, rows_per_block, keys, (hipStream_t)stream);
}

}  // extern "C"
