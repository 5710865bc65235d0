// Kernels of the two-step HBP SpMV (Fig. 1, Algorithm 3, Section 3.3) and of the in-repo CSR
// baselines (Algorithm 1), as templates over the value type, with their launchers.  Included by
// one translation unit per value type (hbp_spmv.hip: fp32, hbp_spmv_f64.hip: fp64) so that the two
// sets of instantiations compile side by side.
#pragma once

#include "hbp_internal.h"

#include <atomic>
#include <type_traits>

namespace hbp {
namespace {

__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Wave-uniform read of a layout array that no kernel writes while an SpMV runs.  Going through
// the constant address space lets the compiler use a scalar load, whose result lands in an
// SGPR without a wait at the point of issue: this is what keeps the prefetch of the next
// groups' metadata off the critical path.
__device__ __forceinline__ int32_t uniform_load(const int32_t *p, int32_t i)
{
    typedef const int32_t __attribute__((address_space(4))) *const_ptr;
    return ((const_ptr)(uintptr_t)p)[i];
}

// One group, one wavefront.  Lane q owns slot q and has n nonzeros.  Rounds are taken U at a
// time ("a batch"): the U ballots give each round's live lanes, a lane's element in a round
// sits at the round's base plus the number of live lanes below it, all 2U loads are issued,
// then the products are accumulated through the staged vector segment.
// T is the value type, float or double.
template <int U, typename T>
struct Batch {
    uint32_t c[U];
    T v[U];
    int rounds;  // rounds of the batch in which some lane has a nonzero (they are the leading ones)
};

// a * b + c in one instruction (the value of a lane without an element in the round is zeroed
// before it, one select instead of a select between a multiply and an add)
__device__ __forceinline__ float fma_of(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_of(double a, double b, double c) { return __builtin_fma(a, b, c); }

// Issues the loads of rounds k .. k+U-1 and advances base past them.  No load is predicated: a
// lane without an element in a round reads a neighbour's (or the position just behind the
// round: inside the group, or inside the padding behind the last group) and drops the product.
template <int U, typename T>
__device__ __forceinline__ void issue_batch(Batch<U, T> &b, const uint16_t *__restrict__ col_local,
                                            const T *__restrict__ data, uint32_t &base, int32_t n, int32_t k)
{
    b.rounds = 0;
#pragma unroll
    for (int u = 0; u < U; u++) {
        const uint64_t live = __ballot(k + u < n);
        b.c[u] = 0;
        b.v[u] = T(0);
        if (live) {  // wave-uniform: rounds past every row's end issue nothing
            // the round's base stays in the scalar part of the address, the lane's rank among the
            // live lanes is the 32-bit vector part: no 64-bit vector arithmetic per load
            const uint32_t rank = (uint32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(live >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)live, 0u));
            const char *round_col = reinterpret_cast<const char *>(col_local) + ((uint64_t)base << 1);
            const char *round_val = reinterpret_cast<const char *>(data) + (uint64_t)base * sizeof(T);
            b.c[u] = __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(round_col + (rank << 1)));
            b.v[u] = __builtin_nontemporal_load(reinterpret_cast<const T *>(round_val + rank * (uint32_t)sizeof(T)));
            base += (uint32_t)__popcll(live);
            b.rounds = u + 1;
        }
    }
}

// Products of the batch, summed per lane.  QUARTERS: the batch is taken in four quarters and a
// quarter without a nonzero is skipped (deep batches behind a group's first one are mostly
// empty when the rows are only a little longer than the first batch).
template <int U, bool QUARTERS = false, typename T>
__device__ __forceinline__ T consume_batch(const Batch<U, T> &b, const T *xs, int32_t n, int32_t k)
{
    T acc = T(0);
    if constexpr (QUARTERS) {
        constexpr int Q = U / 4;
#pragma unroll
        for (int q0 = 0; q0 < U; q0 += Q) {
            if (q0 < b.rounds) {  // wave-uniform
                T xv[Q];
#pragma unroll
                for (int u = 0; u < Q; u++) xv[u] = xs[b.c[q0 + u]];
#pragma unroll
                for (int u = 0; u < Q; u++) acc = fma_of(k + q0 + u < n ? b.v[q0 + u] : T(0), xv[u], acc);
            }
        }
    } else {
        T xv[U];
#pragma unroll
        for (int u = 0; u < U; u++) xv[u] = xs[b.c[u]];
#pragma unroll
        for (int u = 0; u < U; u++) acc = fma_of(k + u < n ? b.v[u] : T(0), xv[u], acc);
    }
    return acc;
}

// Fast path for a full group whose 64 rows all have the same length n0 >= 4: its nonzeros are
// one contiguous run of 64 n0 elements in which element o belongs to the row of lane o mod 64.
// The run is read in 256-element chunks aligned to 1 KB (fp32 data) / 512 B (columns), four
// consecutive elements per lane with one 16-byte and one 8-byte load.  With d = distance from
// the first chunk's start to the run, lane l's j-th element of every chunk belongs to the row
// of lane (4 l + j - d) mod 64, so a lane keeps four running sums and no shuffle is needed
// until the end, when the four lanes l, l^16, l^32, l^48 that serve the same rows are added.
// Lanes whose four elements lie outside the run load nothing; elements outside the run that
// share a 16-byte quad with it are read but contribute nothing.  Used by the fp32 kernels only:
// with fp64 values the round-by-round walk measured 5 % faster on the 27-point stencil.
template <typename T>
struct Vec4 {
    typedef T type __attribute__((ext_vector_type(4)));
};
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int CH, typename T>
struct WideBatch {
    typename Vec4<T>::type v[CH];
    u32x2 c[CH];
};

// FIRST: the chunks start at the run's first chunk; only that one can hold elements in front of
// the run, so the other chunks are tested against the run's end alone.
template <int CH, bool FIRST = true, typename T>
__device__ __forceinline__ void issue_wide(WideBatch<CH, T> &b, const uint16_t *__restrict__ col_local,
                                           const T *__restrict__ data, uint32_t chunk0, uint32_t i0, uint32_t run_begin,
                                           uint32_t run_end, int lane)
{
#pragma unroll
    for (int u = 0; u < CH; u++) {
        const uint32_t p = chunk0 + 256u * (i0 + u) + 4u * (uint32_t)lane;
        b.v[u] = typename Vec4<T>::type{T(0), T(0), T(0), T(0)};
        b.c[u] = u32x2{0u, 0u};
        if ((!(FIRST && u == 0) || p + 3u >= run_begin) && p < run_end) {  // lanes whose four elements miss the run load nothing
            b.v[u] = __builtin_nontemporal_load(reinterpret_cast<const typename Vec4<T>::type *>(data + p));
            b.c[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(col_local + p));
        }
    }
}

template <int CH, bool FIRST = true, typename T>
__device__ __forceinline__ void consume_wide(const WideBatch<CH, T> &b, const T *xs, uint32_t chunk0, uint32_t i0,
                                             uint32_t run_begin, uint32_t run_end, int lane, T (&acc)[4])
{
    uint32_t c[CH][4];
    bool ok[CH][4];
    T xv[CH][4];
#pragma unroll
    for (int u = 0; u < CH; u++) {
        const uint32_t p = chunk0 + 256u * (i0 + u) + 4u * (uint32_t)lane;
        const uint32_t lo = b.c[u].x, hi = b.c[u].y;
        c[u][0] = lo & 0xffffu; c[u][1] = lo >> 16; c[u][2] = hi & 0xffffu; c[u][3] = hi >> 16;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            ok[u][j] = (!(FIRST && u == 0) || p + j >= run_begin) && p + j < run_end;
            c[u][j] = ok[u][j] ? c[u][j] : 0u;  // never index the segment with a foreign column
        }
    }
#pragma unroll
    for (int u = 0; u < CH; u++)
#pragma unroll
        for (int j = 0; j < 4; j++) xv[u][j] = xs[c[u][j]];
#pragma unroll
    for (int u = 0; u < CH; u++) {
        const T v[4] = {b.v[u].x, b.v[u].y, b.v[u].z, b.v[u].w};
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const T prod = v[j] * xv[u][j];
            acc[j] += ok[u][j] ? prod : T(0);
        }
    }
}

template <int THREADS, int U, int GP, bool HEAVY, typename T>
// (second launch bound: four wavefronts per SIMD, i.e. at most 128 vector registers per lane
// whatever the workgroup size; with more, two 512-thread workers no longer fit a CU together)
__global__ __launch_bounds__(THREADS, 4) void k_spmv_part(Layout L,
                                                       const T *__restrict__ x, T *__restrict__ partial,
                                                       T *__restrict__ y, uint32_t *__restrict__ col_ticket)
{
    const T *__restrict__ const data = static_cast<const T *>(L.data);
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    T *const xs = reinterpret_cast<T *>(dyn_lds);  // the staged vector segment, C values
    __shared__ int32_t sh_next;  // whose range to compete for next, broadcast to the worker
    __shared__ unsigned long long sh_rng;  // groups of the worker still to draw: end << 32 | next
    __shared__ int32_t sh_dry;   // nothing more to claim from the current competitive part
    __shared__ int32_t sh_lock;  // end of the last range reported as used up
    __shared__ int32_t sh_col[3];  // whose competitive part is being claimed, its first group, its end
    __shared__ T sh_hand[THREADS];  // per wavefront: hand-over of span sums to the owning lanes
    constexpr int kHeavyCap = 64;
    __shared__ int32_t sh_heavy[kHeavyCap];  // heavy groups of the current range, left to the whole worker
    __shared__ int32_t sh_heavy_n;
    constexpr int kLongCap = 256;
    __shared__ int32_t sh_long[kLongCap];  // long groups of the current range, each left to the next free wavefront
    __shared__ int32_t sh_long_n, sh_long_next;
    __shared__ int32_t sh_lens[THREADS];  // per wavefront: segment lengths of the heavy group being cut
    __shared__ int32_t sh_cut_k[THREADS / 64 + 1];   // heavy group: first round of every wavefront's share
    __shared__ uint32_t sh_cut_pos[THREADS / 64 + 1];  // and the nonzeros before that round
    constexpr int kWaves = THREADS / 64;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int staged_bn = -1;
    // Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2.  Workers with
    // neighbouring ranges share block columns, hence slices of x: runs of four consecutive
    // workers are placed on one XCD (a slice is then fetched into that L2 once and re-staged from
    // there), successive runs on successive XCDs so that no XCD gets one contiguous part of the
    // matrix.
    const int32_t n_workers = (int32_t)gridDim.x;
    int32_t worker = (int32_t)blockIdx.x;
    if ((n_workers & 31) == 0) {
        const int32_t xcd = worker & 7, i = worker >> 3;
        worker = (((i >> 2) << 3) + xcd) * 4 + (i & 3);
    }

    // Copies the vector segment of block column bn into LDS (no barriers: the caller orders it).
    auto copy_slice = [&](int32_t bn) __attribute__((always_inline)) {
        const int64_t c0 = (int64_t)bn * L.C;
        const int32_t width = (int32_t)min((int64_t)L.C, L.n_cols - c0);
        // 16-byte loads, eight in flight per thread, when the slice is 16-byte aligned
        typedef T vec16 __attribute__((ext_vector_type(16 / sizeof(T))));
        constexpr int32_t kPer = 16 / (int32_t)sizeof(T);
        const T *src = x + c0;
        const int32_t n4 = (reinterpret_cast<uintptr_t>(src) & 15u) == 0 ? width / kPer : 0;
        for (int32_t i0 = 0; i0 < n4; i0 += THREADS * 8) {
            vec16 t[8];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int32_t i = min(i0 + u * THREADS + (int32_t)threadIdx.x, n4 - 1);
                t[u] = reinterpret_cast<const vec16 *>(src)[i];
            }
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int32_t i = i0 + u * THREADS + (int32_t)threadIdx.x;
                if (i < n4) reinterpret_cast<vec16 *>(xs)[i] = t[u];
            }
        }
        for (int32_t i = kPer * n4 + threadIdx.x; i < width; i += THREADS) xs[i] = src[i];
    };

    // The wavefronts of the worker share out the groups [*, g_end) of the current range by
    // drawing packs of GP consecutive groups from an LDS counter (wavefronts do not progress at
    // the same speed, so a static deal would leave the slow ones behind).  Each wavefront keeps
    // three draws in hand and runs them as a two-deep software pipeline: while a pack is
    // walked, the lane lengths of the next one and the slot ranges / first positions of the one
    // after it are already on their way, and the partial sums of the previous one are stored
    // behind the current pack's loads.  GP > 1 is for matrices whose groups hold few nonzeros:
    // the first batches of all GP groups are issued before any is consumed.  A group index at
    // or beyond g_end gives an idle lane set (n = 0, position 0).
    //
    // Draws.  sh_rng holds the worker's current range of groups; a draw takes GP groups off its
    // front with one LDS atomic (draw_issue) whose result is looked at an iteration later
    // (draw_resolve), so that its latency is never waited for.  A draw that finds the range
    // used up, in a worker that competes for some worker's range (Section 3.3), leads to a claim:
    // the first wavefront to report the range that ended at `end` as used up (atomic max on
    // sh_lock; the ends of successive ranges grow) takes that range's next `claim` competitive
    // groups from its counter in global memory and publishes them as the new range;
    // the other wavefronts wait for the range to move (a bounded wait: a wavefront that gives
    // up just stops drawing, the claimed groups are walked by those that go on).  So the
    // wavefronts of a worker pass from fixed to competitive groups and from claim to claim
    // without a barrier.  Once the competitive part has nothing left (or in a worker that does not
    // compete) a used-up range makes the draw, and every later draw of the wavefront in this
    // range, return kNone.
    constexpr int32_t kNone = 0x7fffffff;
    constexpr int kSpinLimit = 1 << 16;
    bool stop = false;  // this wavefront draws no more in the current range
    // does group g + q of the pack (g, its end e) exist?
    auto in_pack = [&](int32_t g, int32_t e, int q) __attribute__((always_inline)) {
        return GP == 1 ? g != kNone : q < e - g;
    };
    auto draw_issue = [&]() __attribute__((always_inline)) {
        unsigned long long old = 0;  // reads as a used-up range
        if (lane == 0 && !stop) old = atomicAdd(&sh_rng, (unsigned long long)GP);
        return old;
    };
    auto draw_resolve = [&](unsigned long long old, int32_t &pack_end) __attribute__((always_inline)) {
        int32_t v = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)old);
        int32_t end = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)(old >> 32));
        int spins = 0;
        while (v >= end) {
            if (stop || __hip_atomic_load(&sh_dry, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) {
                stop = true;
                pack_end = 0;
                return kNone;
            }
            int32_t reported = 0;
            if (lane == 0) reported = atomicMax(&sh_lock, end);
            reported = __builtin_amdgcn_readfirstlane(reported);
            if (reported < end) {
                // first to report this range as used up: claim the next competitive groups
                // (their owner's numbers sit in LDS: this path is rare, registers are not)
                const int32_t claim = L.claim, col_end = sh_col[2];
                uint32_t t = 0;
                if (lane == 0) t = atomicAdd(&col_ticket[sh_col[0]], (uint32_t)claim);
                t = __builtin_amdgcn_readfirstlane(t);
                const int64_t c0 = (int64_t)sh_col[1] + t;
                if (c0 >= col_end) {
                    if (lane == 0) __hip_atomic_store(&sh_dry, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    continue;  // leaves through the test above
                }
                const unsigned long long c1 = (unsigned long long)min(c0 + claim, (int64_t)col_end);
                if (lane == 0) atomicExch(&sh_rng, (c1 << 32) | (unsigned long long)c0);
            } else {
                // another wavefront claims: wait until the range's end moves or the column is dry
                bool moved = false;
                while (spins < kSpinLimit) {
                    const unsigned long long now = __hip_atomic_load(&sh_rng, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    const int dry = __hip_atomic_load(&sh_dry, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    spins++;
                    if ((int32_t)(uint32_t)(now >> 32) != end || dry) { moved = true; break; }
                    __builtin_amdgcn_s_sleep(2);
                }
                if (!moved) stop = true;  // gave up: leaves through the test above
            }
            if (stop) continue;
            unsigned long long again = 0;
            if (lane == 0) again = atomicAdd(&sh_rng, (unsigned long long)GP);
            v = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)again);
            end = __builtin_amdgcn_readfirstlane((int32_t)(uint32_t)(again >> 32));
        }
        pack_end = GP == 1 ? v + 1 : min(v + GP, end);
        return v;
    };
    // Rounds k, k+1, ... of one group until no lane has a nonzero left (lane q has n; `base` is
    // the position of round k), added into acc.
    auto walk_rounds = [&](uint32_t &base, int32_t n, int32_t k, T &acc) __attribute__((always_inline)) {
        for (;;) {
            const uint64_t live = __ballot(k < n);
            if (!live) break;
            const int32_t m = __popcll(live);
            constexpr int UL = 16;
            // (The folded batches below are compiled into the variant for matrices with very long
            // rows only: in the other variants, whose groups rarely get there, their code cost the
            // main path 4-10 % through registers and instruction cache.)
            const bool few = HEAVY ? m <= 32 : (m <= 32 && __ballot(k + 2 * U < n) == live);
            if (!few) {
                // many rows still going: a deep batch of rounds
                Batch<UL, T> deep;
                issue_batch<UL>(deep, L.col_local, data, base, n, k);
                acc += consume_batch<UL, true>(deep, xs, n, k);
                k += UL;
                continue;
            }
            if (HEAVY && __ballot(k + 2 * U < n) != live) {
                // Few rows left and one of them ends soon.  A batch would use m of 64 lanes, so the
                // wavefront is folded: with mm the power of two that holds the m live rows and
                // f = 64 / mm, lane j * mm + c serves the c-th live row in the rounds k + j, k + j + f,
                // k + j + 2f, ...  In that lane order (round, then row) the elements of f consecutive
                // rounds are exactly what one step of a batch reads, so the batch code runs
                // unchanged on the folded lanes' own counts and covers UL * f rounds.
                const int sh = m > 16 ? 5 : m > 8 ? 4 : m > 4 ? 3 : m > 2 ? 2 : m > 1 ? 1 : 0;  // mm = 2^sh
                int32_t *left = reinterpret_cast<int32_t *>(sh_hand + wave * 64);
                left[lane] = 0;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                if (k < n) left[lanes_below(live)] = n - k;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                const int32_t mine = left[lane & ((1 << sh) - 1)], j = lane >> sh;  // rounds left in the row this lane serves
                const int32_t steps = mine > j ? (mine - j + (64 >> sh) - 1) >> (6 - sh) : 0;
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                Batch<UL, T> deep;
                issue_batch<UL>(deep, L.col_local, data, base, steps, 0);
                T *hand = sh_hand + wave * 64;
                hand[lane] = consume_batch<UL, true>(deep, xs, steps, 0);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                if (k < n)
                    for (int32_t t = lanes_below(live); t < 64; t += 1 << sh) acc += hand[t];
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                k += UL << (6 - sh);
                continue;
            }
            // Few rows left, all of them with at least 2U more rounds.  Until the shortest of
            // them ends, the live set is constant and the rounds k .. k_end-1 form one contiguous
            // span in which element o belongs to the (o mod m)-th live row.  The whole wavefront
            // reads the span: lanes 0 .. S-1 (S = largest multiple of m up to 64) take elements
            // lane, lane + S, ..., all for one row each, and the per-lane sums are handed to the
            // owning lanes through LDS.
            int32_t k_end = k < n ? n : 0x7fffffff;
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) k_end = min(k_end, __shfl_xor(k_end, d));
            const uint32_t span = (uint32_t)m * (uint32_t)(k_end - k);
            const uint32_t S = (64u / (uint32_t)m) * (uint32_t)m;
            T sum = T(0);
            if ((uint32_t)lane < S) {
                uint32_t o = (uint32_t)lane;
                for (; o + 3u * S < span; o += 4u * S) {
                    uint32_t c4[4];
                    T v4[4];
#pragma unroll
                    for (int u = 0; u < 4; u++) {
                        c4[u] = __builtin_nontemporal_load(L.col_local + base + o + u * S);
                        v4[u] = __builtin_nontemporal_load(data + base + o + u * S);
                    }
#pragma unroll
                    for (int u = 0; u < 4; u++) sum += v4[u] * xs[c4[u]];
                }
                for (; o < span; o += S) sum += data[base + o] * xs[L.col_local[base + o]];
            }
            T *hand = sh_hand + wave * 64;
            hand[lane] = sum;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            if (k < n)
                for (uint32_t t = (uint32_t)lanes_below(live); t < S; t += (uint32_t)m) acc += hand[t];
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            base += span;
            k = k_end;
        }
    };
    // Runs the groups [g_begin, g_end) of block column bn with all wavefronts of the worker.
    auto run_range = [&](int32_t bn, int32_t g_begin, int32_t g_end, bool compete, int32_t owner) __attribute__((always_inline)) {
        __syncthreads();  // every wavefront has left the previous range (and its slice of x)
        if (threadIdx.x == 0) {
            sh_rng = ((unsigned long long)(uint32_t)g_end << 32) | (uint32_t)g_begin;
            sh_dry = compete ? 0 : 1;
            sh_lock = -1;
            sh_heavy_n = 0;
            sh_long_n = 0;
            sh_long_next = 0;
            sh_col[0] = owner;  // whose competitive groups are claimed from here on
            sh_col[1] = L.comp_lo[owner];
            sh_col[2] = L.fixed_start[owner + 1];
        }
        stop = false;
        __syncthreads();
        int32_t e = 0, e1 = 0, e2 = 0;  // ends of the packs g, g1, g2: group g + q exists if it is below e
        int32_t g = draw_resolve(draw_issue(), e), g1 = draw_resolve(draw_issue(), e1), g2 = kNone;
        unsigned long long raw2 = draw_issue();
        int32_t s0[GP], s1[GP], n[GP], done_slot[GP];
        // The slot ranges and first positions of a pack's groups travel in one vector register per
        // pack: lane l <= GP holds group_slot[first + l], lane 32 + l (l < GP) holds
        // group_ptr[first + l], zero where the pack has no such group; they are read out into
        // scalars where they are used.  (Loaded as scalars and carried three packs deep they did
        // not fit the scalar registers: the spills cost some fifty instructions per pack and made
        // the wavefront wait for each scalar load right where it was issued.)
        auto load_meta = [&](int32_t first, int32_t end) __attribute__((always_inline)) {
            uint32_t m = 0;
            const int32_t l = lane & 31;
            const bool position = lane >= 32;
            if (first != kNone && l <= GP && l < end - first + (position ? 0 : 1))
                m = (uint32_t)(position ? L.group_ptr : L.group_slot)[first + l];
            return m;
        };
        auto meta_slots = [&](uint32_t m, int32_t first, int32_t end, int q, int32_t &from, int32_t &to) __attribute__((always_inline)) {
            const bool there = in_pack(first, end, q);
            from = there ? (int32_t)__builtin_amdgcn_readlane(m, q) : 0;
            to = there ? (int32_t)__builtin_amdgcn_readlane(m, q + 1) : 0;
        };
        auto meta_base = [&](uint32_t m, int32_t first, int32_t end, int q) __attribute__((always_inline)) {
            return in_pack(first, end, q) ? (uint32_t)__builtin_amdgcn_readlane(m, 32 + q) : 0u;
        };
        uint32_t meta = load_meta(g, e), meta_n = load_meta(g1, e1);  // of the packs g and g1
        // Packs of short rows have a path of their own in the fp64 kernels.  (In fp32 it measured
        // 2-3 % slower than the general path: the kernel is bound by the latency of a pack's
        // loads, not by its instructions, and the extra code costs registers.)
        constexpr bool kShortPacks = GP > 1 && sizeof(T) == 8;
        // longest row of the packs g and g1 (wave-uniform; only looked at where kShortPacks)
        int32_t pack_longest = 0, pack_longestn = 0;
        auto longest_in_pack = [&](int32_t first, int32_t end) __attribute__((always_inline)) {
            int32_t most = 0;
            if constexpr (kShortPacks) {
#pragma unroll
                for (int q = 0; q < GP; q++)
                    if (in_pack(first, end, q))
                        most = max(most, uniform_load(L.group_rounds, first + q + 1) - uniform_load(L.group_rounds, first + q));
            }
            return most;
        };
        uint32_t base[GP];  // positions stay 32-bit: nnz < 2^31
        T done_acc[GP];
#pragma unroll
        for (int q = 0; q < GP; q++) {
            done_slot[q] = -1;
            done_acc[q] = T(0);
            meta_slots(meta, g, e, q, s0[q], s1[q]);
            n[q] = s0[q] + lane < s1[q] ? L.seg_len[s0[q] + lane] : 0;
        }
        pack_longest = longest_in_pack(g, e);
        pack_longestn = longest_in_pack(g1, e1);
        // the first packs' metadata is on its way while the slice of x is staged
        if (bn != staged_bn) {
            copy_slice(bn);
            __syncthreads();
            staged_bn = bn;
        }
        for (;;) {
            g2 = draw_resolve(raw2, e2);  // drawn an iteration ago
            if (g == kNone && g1 == kNone && g2 == kNone) break;  // and this wavefront has stopped drawing
            raw2 = draw_issue();
#pragma unroll
            for (int q = 0; q < GP; q++) {
                meta_slots(meta, g, e, q, s0[q], s1[q]);
                base[q] = meta_base(meta, g, e, q);
            }
            // A group with a row of more than heavy_rounds nonzeros would keep this wavefront busy
            // long after the rest of the worker has run dry: it goes on the worker's heavy list and
            // looks empty here (unless the list is full: then this wavefront walks it alone).  A
            // group with a row of more than long_rounds goes on the long list: such groups come in
            // runs (the last groups of a block), a pack would hand several of them to one
            // wavefront to walk one after the other, and they are taken one per wavefront instead
            // once the range's other groups are done.
            if (HEAVY && (!kShortPacks || pack_longest > L.long_rounds)) {
#pragma unroll
                for (int q = 0; q < GP; q++) {
                    if (__ballot(n[q] > L.long_rounds)) {
                        const bool heavy = __ballot(n[q] > L.heavy_rounds) != 0;
                        int32_t idx = 0;
                        if (lane == 0) idx = atomicAdd(heavy ? &sh_heavy_n : &sh_long_n, 1);
                        idx = __builtin_amdgcn_readfirstlane(idx);
                        if (idx < (heavy ? kHeavyCap : kLongCap)) {
                            if (lane == 0) (heavy ? sh_heavy : sh_long)[idx] = g + q;
                            n[q] = 0;
                            s1[q] = s0[q];
                        }
                    }
                }
            }
            int32_t nn[GP], slot[GP];
            const int32_t pack_longestnn = longest_in_pack(g2, e2);
            const uint32_t meta_nn = load_meta(g2, e2);
            T acc[GP];
            // lane lengths of group q of the pack g1
            auto next_lengths = [&](int q) __attribute__((always_inline)) {
                int32_t from, to;
                meta_slots(meta_n, g1, e1, q, from, to);
                return from + lane < to ? (int32_t)L.seg_len[from + lane] : 0;
            };
            bool wide = false;
            if constexpr (GP == 1 && sizeof(T) == 4) {
                const int32_t n0 = __builtin_amdgcn_readfirstlane(n[0]);
                wide = s1[0] - s0[0] == 64 && n0 >= 4 && __ballot(n[0] != n0) == 0;
                if (wide) {
                    // full group, equal rows: aligned wide loads
                    constexpr int CH = 4;
                    const uint32_t chunk0 = base[0] & ~255u, run_end = base[0] + 64u * (uint32_t)n0;
                    const uint32_t n_chunks = (run_end - chunk0 + 255u) >> 8;
                    T a4[4] = {T(0), T(0), T(0), T(0)};
                    WideBatch<CH, T> wb;
                    issue_wide<CH>(wb, L.col_local, data, chunk0, 0, base[0], run_end, lane);
                    if (done_slot[0] >= 0) partial[done_slot[0]] = done_acc[0];
                    nn[0] = next_lengths(0);
                    consume_wide<CH>(wb, xs, chunk0, 0, base[0], run_end, lane, a4);
                    for (uint32_t i0 = CH; i0 < n_chunks; i0 += CH) {
                        issue_wide<CH, false>(wb, L.col_local, data, chunk0, i0, base[0], run_end, lane);
                        consume_wide<CH, false>(wb, xs, chunk0, i0, base[0], run_end, lane, a4);
                    }
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        a4[j] += __shfl_xor(a4[j], 16);
                        a4[j] += __shfl_xor(a4[j], 32);
                    }
                    const int m = lane >> 4;  // this lane reports the m-th of its four rows
                    acc[0] = m == 0 ? a4[0] : m == 1 ? a4[1] : m == 2 ? a4[2] : a4[3];
                    slot[0] = s0[0] + (int32_t)((4u * (uint32_t)(lane & 15) + (uint32_t)m + 256u - (base[0] - chunk0)) & 63u);
                }
            }
            if (kShortPacks && pack_longest <= 2) {
                // Packs of groups whose rows have one or two nonzeros (wave-uniform, known from the
                // groups' longest rows): round 0 of a group is its slots in order, so lane q's first
                // element sits at base + q and no ballot is needed; round 1 holds the second
                // elements of the rows that have one.  Lanes without a slot or a second element read
                // a position inside the group or the padding behind it and drop the product.
                uint32_t c0[GP], c1[GP];
                T v0[GP], v1[GP];
#pragma unroll
                for (int q = 0; q < GP; q++) {
                    c0[q] = __builtin_nontemporal_load(L.col_local + base[q] + lane);
                    v0[q] = __builtin_nontemporal_load(data + base[q] + lane);
                }
                if (pack_longest == 2) {
#pragma unroll
                    for (int q = 0; q < GP; q++) {
                        const uint64_t live = __ballot(n[q] > 1);
                        const uint32_t j = (uint32_t)__builtin_amdgcn_mbcnt_hi(
                            (uint32_t)(live >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)live, base[q] + (uint32_t)(s1[q] - s0[q])));
                        c1[q] = __builtin_nontemporal_load(L.col_local + j);
                        v1[q] = __builtin_nontemporal_load(data + j);
                    }
                }
#pragma unroll
                for (int q = 0; q < GP; q++) {
                    if (done_slot[q] >= 0) partial[done_slot[q]] = done_acc[q];
                    nn[q] = next_lengths(q);
                }
                if (pack_longest == 2) {
                    T x0[GP], x1[GP];
#pragma unroll
                    for (int q = 0; q < GP; q++) { x0[q] = xs[c0[q]]; x1[q] = xs[c1[q]]; }
#pragma unroll
                    for (int q = 0; q < GP; q++) {
                        const T p1 = v1[q] * x1[q];
                        acc[q] = v0[q] * x0[q] + (n[q] > 1 ? p1 : T(0));
                    }
                } else {
                    T x0[GP];
#pragma unroll
                    for (int q = 0; q < GP; q++) x0[q] = xs[c0[q]];
#pragma unroll
                    for (int q = 0; q < GP; q++) acc[q] = v0[q] * x0[q];
                }
#pragma unroll
                for (int q = 0; q < GP; q++) slot[q] = s0[q] + lane < s1[q] ? s0[q] + lane : -1;
            } else if (!wide) {
                // general groups: round by round, U rounds per batch
                Batch<U, T> bt[GP];
#pragma unroll
                for (int q = 0; q < GP; q++) issue_batch<U>(bt[q], L.col_local, data, base[q], n[q], 0);
#pragma unroll
                for (int q = 0; q < GP; q++) {
                    if (done_slot[q] >= 0) partial[done_slot[q]] = done_acc[q];
                    nn[q] = next_lengths(q);
                }
#pragma unroll
                for (int q = 0; q < GP; q++) acc[q] = consume_batch<U>(bt[q], xs, n[q], 0);
#pragma unroll
                for (int q = 0; q < GP; q++) {  // rows longer than U, one group at a time
                    // (the test keeps what the compiler hoists out of the walk's loops, a dozen
                    // values per group, off the path of the groups without such rows)
                    if (__ballot(U < n[q])) walk_rounds(base[q], n[q], U, acc[q]);
                    slot[q] = s0[q] + lane < s1[q] ? s0[q] + lane : -1;
                }
            }
#pragma unroll
            for (int q = 0; q < GP; q++) {
                done_acc[q] = acc[q];
                done_slot[q] = slot[q];
                n[q] = nn[q];
            }
            meta = meta_n;
            meta_n = meta_nn;
            g = g1; g1 = g2;
            e = e1; e1 = e2;
            pack_longest = pack_longestn; pack_longestn = pack_longestnn;
        }
#pragma unroll
        for (int q = 0; q < GP; q++)
            if (done_slot[q] >= 0) partial[done_slot[q]] = done_acc[q];

        // Heavy groups of this range: all wavefronts of the worker walk each of them together.
        // Wavefront w takes the rounds [k_w, k_{w+1}), where k_w is the first round that has
        // w / kWaves of the group's nonzeros before it, and the per-lane sums of the wavefronts
        // are added in LDS in wavefront order.
        if constexpr (!HEAVY) return;
        __syncthreads();
        // Long groups of this range: one wavefront each, whoever is free next.
        const int32_t n_long = min(sh_long_n, kLongCap);
        if (n_long > 0) {
            for (;;) {
                int32_t i = 0;
                if (lane == 0) i = atomicAdd(&sh_long_next, 1);
                i = __builtin_amdgcn_readfirstlane(i);
                if (i >= n_long) break;
                const int32_t gl = sh_long[i];
                const int32_t ls0 = uniform_load(L.group_slot, gl), ls1 = uniform_load(L.group_slot, gl + 1);
                uint32_t pos = (uint32_t)uniform_load(L.group_ptr, gl);
                const int32_t len = ls0 + lane < ls1 ? (int32_t)L.seg_len[ls0 + lane] : 0;
                T sum = T(0);
                walk_rounds(pos, len, 0, sum);
                if (ls0 + lane < ls1) partial[ls0 + lane] = sum;
            }
        }
        const int32_t n_heavy = min(sh_heavy_n, kHeavyCap);
        for (int32_t i = 0; i < n_heavy; i++) {
            const int32_t gh = sh_heavy[i];
            const int32_t hs0 = uniform_load(L.group_slot, gh), hs1 = uniform_load(L.group_slot, gh + 1);
            const uint32_t b0 = (uint32_t)uniform_load(L.group_ptr, gh);
            const uint32_t total = (uint32_t)uniform_load(L.group_ptr, gh + 1) - b0;
            const int32_t len = hs0 + lane < hs1 ? (int32_t)L.seg_len[hs0 + lane] : 0;
            int32_t *lens = sh_lens + wave * 64;
            lens[lane] = len;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // nonzeros of the group in rounds 0 .. k-1; every lane may ask for another k
            auto before = [&](int32_t k) __attribute__((always_inline)) {
                uint32_t sum = 0;
#pragma unroll 16
                for (int t = 0; t < 64; t++) sum += (uint32_t)min(lens[t], k);
                return sum;
            };
            // smallest k with before(k) >= target, by three 64-way splits of (0, 65536]: a segment
            // has fewer than 65536 nonzeros, so before(65536) = total >= target
            const uint32_t target = (uint32_t)(((uint64_t)total * (uint32_t)wave) / (uint32_t)kWaves);
            int32_t cut_k = 0;
            uint32_t cut_pos = 0;
            if (target > 0) {
                int32_t lo = 0;
                auto split = [&](int32_t step) __attribute__((always_inline)) {
                    // candidates lo + step, lo + 2 step, ...: the last one is known to reach the target
                    const uint32_t got = before(lo + (lane + 1) * step);
                    const int first = __builtin_ctzll(__ballot(got >= target));
                    lo += first * step;
                    return (uint32_t)__shfl(got, first);
                };
                split(1024);
                split(16);
                cut_pos = split(1);
                cut_k = lo + 1;
            }
            if (lane == 0) { sh_cut_k[wave] = cut_k; sh_cut_pos[wave] = cut_pos; }
            if (threadIdx.x == 0) sh_cut_k[kWaves] = 0x10000;
            __syncthreads();
            const int32_t k_lo = sh_cut_k[wave], k_hi = sh_cut_k[wave + 1];
            uint32_t pos = b0 + sh_cut_pos[wave];
            T sum = T(0);
            walk_rounds(pos, min(len, k_hi), k_lo, sum);
            sh_hand[threadIdx.x] = sum;
            __syncthreads();
            if (wave == 0 && hs0 + lane < hs1) {
                T total_sum = sh_hand[lane];
#pragma unroll
                for (int w = 1; w < kWaves; w++) total_sum += sh_hand[w * 64 + lane];
                partial[hs0 + lane] = total_sum;
            }
            __syncthreads();  // sh_hand and the cuts are reused by the next heavy group
        }
    };

    // The worker's ranges, one after the other (run_range is expanded once, here):
    //   phase 0, fixed part (Section 3.3): the group list is cut into P contiguous ranges of
    //     equal weight; worker w runs, column by column, the groups of its range below comp_lo[w].
    //     The groups from comp_lo[w] on, all in the last column of the range, are its competitive
    //     part: the worker goes on, without a break, to claim them piece by piece from the range's
    //     counter (the segment of x is staged already), and so may others;
    //   phase 2, competitive part: the counter of a range holds how many of its competitive groups
    //     have been claimed; a worker that has run out of work moves to the range with the most
    //     weight left (and stages the segment of x of that range's last column), until no range
    //     has enough left to be worth entering.  So a range that takes longer than its weight said is finished by the workers
    //     that were faster than theirs;
    //   phase 3 instead of 2, the paper's schedule: one ticket counter over the blocks that were not pre-assigned.
    const bool competitive = L.competitive != 0;
    int32_t col = L.fixed_col[worker];
    int32_t g_next = L.fixed_start[worker];
    const int32_t g_stop = L.fixed_start[worker + 1];
    const int32_t own_lo = L.comp_lo[worker];
    for (int phase = 0;;) {
        int32_t r_bn = 0, r_g0 = 0, r_g1 = 0, r_owner = worker;
        bool r_compete = true;
        if (phase == 0) {
            bool found = false;
            while (g_next < g_stop && !found) {
                const int32_t c_end = L.col_group_ptr[col + 1];
                if (g_next >= c_end) { col++; continue; }  // columns without groups
                const int32_t ge = min(g_stop, c_end), fe = max(g_next, min(ge, own_lo));
                const bool last = ge == g_stop;
                if (g_next < fe || (last && competitive)) {
                    r_bn = col;
                    // (an empty fixed part is handed over as [0, 0): the ends of a worker's
                    // successive ranges must grow, and claimed ranges start at comp_lo)
                    r_g0 = g_next < fe ? g_next : 0;
                    r_g1 = g_next < fe ? fe : 0;
                    r_compete = last && competitive;
                    found = true;
                }
                g_next = ge;
            }
            if (!found) {
                if (L.ticket_b0 >= 0) { phase = 3; continue; }
                if (!competitive) break;
                phase = 2;
                continue;
            }
        } else if (phase == 3) {
            // The paper's own competitive part (Section 3.3, when the handle was built for it): the
            // blocks behind the pre-assigned ones are claimed one at a time through a single ticket
            // counter; whoever holds a ticket fetches that block's segment of x and walks the block.
            if (threadIdx.x == 0) sh_next = (int32_t)atomicAdd(&col_ticket[0], 1u);
            __syncthreads();
            const int64_t b = (int64_t)L.ticket_b0 + (uint32_t)sh_next;
            __syncthreads();  // sh_next is rewritten in the next turn
            if (b >= L.B) break;
            r_bn = L.blk_bn[b];
            r_g0 = L.blk_group_ptr[b];
            r_g1 = L.blk_group_ptr[b + 1];
            r_compete = false;
        } else {
            if (wave == 0) {
                int32_t best = -1;
                uint32_t best_left = 0;
                for (int32_t v0 = 0; v0 < L.P; v0 += 64) {
                    int32_t v = v0 + lane;
                    uint32_t left = 0;
                    if (v < L.P) {
                        // weight of the competitive groups of range v that nobody has claimed; a range
                        // with less left than entering it costs (staging its segment of x, about two
                        // block columns' weight counting the pipeline restart) is left to those who
                        // are there already
                        const int32_t end = L.fixed_start[v + 1];
                        const int64_t total = end - L.comp_lo[v];
                        const int64_t used = (int64_t)__hip_atomic_load(&col_ticket[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (used < total) {
                            const int32_t g = L.comp_lo[v] + (int32_t)used;
                            auto before = [&](int32_t i) {
                                return (int64_t)L.group_ptr[i] + (int64_t)L.SW * L.group_slot[i] + (int64_t)L.RW * L.group_rounds[i] +
                                       (int64_t)L.GW * i;
                            };
                            const int64_t w_left = before(end) - before(g);
                            left = w_left < L.steal_min ? 0u : w_left > 0xffffffffll ? 0xffffffffu : (uint32_t)w_left;
                        }
                    }
#pragma unroll
                    for (int d = 32; d > 0; d >>= 1) {
                        const uint32_t o_left = __shfl_xor(left, d);
                        const int32_t o_v = __shfl_xor(v, d);
                        if (o_left > left || (o_left == left && o_v < v)) { left = o_left; v = o_v; }
                    }
                    if (left > best_left) { best_left = left; best = v; }
                }
                if (lane == 0) sh_next = best;
            }
            __syncthreads();
            r_owner = sh_next;
            __syncthreads();  // sh_next is rewritten in the next turn
            if (r_owner < 0) break;
            r_bn = L.comp_col[r_owner];
        }
        run_range(r_bn, r_g0, r_g1, r_compete, r_owner);
    }
    // Row blocks that the combine part cuts into several units are summed into y with atomic
    // adds: their rows of y start at zero.  (Done last: in front of the first range it delays
    // every worker's start.)
    for (int32_t ms = (int32_t)blockIdx.x; ms < L.NM; ms += n_workers) {
        const int64_t r0 = (int64_t)L.multi_stripes[ms] * L.R;
        const int32_t rows = (int32_t)min((int64_t)L.R, L.n_rows - r0);
        for (int32_t r = threadIdx.x; r < rows; r += THREADS) y[r0 + r] = T(0);
    }
}

// Combine part (Fig. 1): one workgroup per row block adds the partial sums of that row block's
// blocks into LDS copies of its y slice and writes the slice out, zeros included.  The slot
// ranges of up to kPass blocks are fetched in parallel first; then wavefronts take blocks
// round-robin and lanes stride over a block's slots.  With kRing > 0 a wavefront keeps a ring of
// kRing chunks of 64 kChunk slots in flight across its blocks (the kernel is bound by the bytes
// it has in flight); with kRing = 0 it walks block by block, four loads per lane at a time, and
// loads the small blocks of a pass together.
// Every wavefront accumulates into its own copy of the slice with plain LDS read-add-write:
// a block holds a row at most once, so the lanes of one instruction never collide, and a
// wavefront's LDS accesses complete in order.  (LDS float atomics would allow one shared copy
// but run an order of magnitude slower on this hardware.)  The copies are summed on the way out.
// Also re-arms the per-column ticket counters for the next call (the SpMV part of this call
// has finished: same stream).
template <int THREADS, typename T, int kRing, int kChunk>
__global__ __launch_bounds__(THREADS) void k_combine(Layout L, const T *__restrict__ partial, T *__restrict__ y,
                                                     uint32_t *__restrict__ ticket)
{
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    T *const ys_all = reinterpret_cast<T *>(dyn_lds);  // kWaves copies of R values
    constexpr int kPass = 128, kWaves = THREADS / 64;
    __shared__ int32_t range[2 * kPass];
    // One workgroup per combine unit: entries [unit_k[j], unit_k[j + 1]) of stripe_blk, all of row
    // block bm.  A row block with a single unit is stored; the units of a split row block add
    // their sums into y, which the SpMV part has zeroed.
    const int32_t unit = blockIdx.x;
    const int32_t bm = L.unit_stripe[unit];
    const bool split = L.unit_ptr[bm + 1] - L.unit_ptr[bm] > 1;
    for (int64_t i = (int64_t)unit * THREADS + threadIdx.x; i < L.P; i += (int64_t)gridDim.x * THREADS) ticket[i] = 0u;
    const int64_t r0 = (int64_t)bm * L.R;
    const int32_t rows = (int32_t)min((int64_t)L.R, L.n_rows - r0);
    for (int32_t i = threadIdx.x; i < kWaves * L.R; i += THREADS) ys_all[i] = T(0);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    T *ys = ys_all + wave * L.R;
    const int32_t k1 = L.unit_k[unit + 1];
    for (int32_t k0 = L.unit_k[unit]; k0 < k1; k0 += kPass) {
        const int32_t nb = min(kPass, k1 - k0);
        __syncthreads();  // slices zeroed / previous pass done with range[]
        constexpr int kTogether = 4, kFirst = 4;
        int small = 0;  // does the pass hold a block with few slots?
        for (int32_t t = threadIdx.x; t < nb; t += THREADS) {
            const int32_t b = L.stripe_blk[k0 + t];
            const int32_t first = L.slot_ptr[b], end = L.slot_ptr[b + 1];
            range[2 * t] = first;
            range[2 * t + 1] = end;
            small |= end - first <= 64 * kFirst;
        }
        if constexpr (kRing > 0) {
            __syncthreads();
            // A ring of kRing chunks of up to 64 kChunk consecutive slots of one block is kept in
            // flight per wavefront: the chunks of a wavefront's blocks follow each other whatever
            // the blocks' sizes, and a chunk is added (read all, then write all: its slots are
            // distinct rows) while the loads of the next kRing - 1 are on their way.
            int32_t next_block = wave, cur = 0, cur_end = 0;
            int32_t c0[kRing], c1[kRing];
            uint32_t r[kRing][kChunk];
            T p[kRing][kChunk];
            auto issue = [&](int d) __attribute__((always_inline)) {
                while (cur >= cur_end && next_block < nb) {
                    cur = __builtin_amdgcn_readfirstlane(range[2 * next_block]);
                    cur_end = __builtin_amdgcn_readfirstlane(range[2 * next_block + 1]);
                    next_block += kWaves;
                }
                c0[d] = cur;
                c1[d] = min(cur + 64 * kChunk, cur_end);
                cur = c1[d];
#pragma unroll
                for (int u = 0; u < kChunk; u++) {
                    r[d][u] = 0;
                    p[d][u] = T(0);
                    if (c0[d] + 64 * u < c1[d]) {  // wave-uniform; clamped: always a slot of this chunk
                        const int32_t idx = min(c0[d] + lane + 64 * u, c1[d] - 1);
                        r[d][u] = L.row_local[idx];
                        p[d][u] = partial[idx];
                    }
                }
            };
#pragma unroll
            for (int d = 0; d < kRing; d++) issue(d);
            while (c1[0] > c0[0]) {  // chunks are issued in order: when this one is empty, all are
#pragma unroll
                for (int d = 0; d < kRing; d++) {
                    if (c1[d] > c0[d]) {
                        T o[kChunk];
#pragma unroll
                        for (int u = 0; u < kChunk; u++) o[u] = ys[r[d][u]];
#pragma unroll
                        for (int u = 0; u < kChunk; u++)
                            if (c0[d] + lane + 64 * u < c1[d]) ys[r[d][u]] = o[u] + p[d][u];
                    }
                    issue(d);
                }
            }
            continue;
        }
        if (!__syncthreads_or(small)) {
            // only blocks with many slots: wavefronts take them one by one, KU slots per lane in
            // flight (the kernel is bound by the bytes it has in flight); the slots of a step are
            // distinct rows of one block: read all, then write all
            for (int32_t i = wave; i < nb; i += kWaves) {
                const int32_t s0 = range[2 * i], s1 = range[2 * i + 1];
                auto add_block = [&](auto ku) __attribute__((always_inline)) {
                    constexpr int KU = decltype(ku)::value;
                    for (int32_t s = s0 + lane; s < s1; s += 64 * KU) {
                        uint32_t r[KU];
                        T p[KU], o[KU];
#pragma unroll
                        for (int u = 0; u < KU; u++) {
                            const int32_t idx = min(s + 64 * u, s1 - 1);  // clamped: always a slot of this block
                            r[u] = L.row_local[idx];
                            p[u] = partial[idx];
                        }
#pragma unroll
                        for (int u = 0; u < KU; u++) o[u] = ys[r[u]];
#pragma unroll
                        for (int u = 0; u < KU; u++)
                            if (s + 64 * u < s1) ys[r[u]] = o[u] + p[u];
                    }
                };
                add_block(std::integral_constant<int, 4>{});
            }
            continue;
        }
        // A wavefront takes kTogether blocks at a time.  Blocks with few slots are one load deep:
        // taken one by one, a wavefront would sit through a memory latency per block.  So the
        // slots of those of the kTogether blocks that have at most 64 kFirst of them are loaded
        // first; then the blocks are added one after the other (a row occurs once per block but
        // may occur in several blocks), a larger block with KU slots per lane in flight (the
        // kernel is bound by the bytes it has in flight).
        for (int32_t i0 = wave; i0 < nb; i0 += kWaves * kTogether) {
            int32_t b0[kTogether], b1[kTogether];
            uint32_t rf[kTogether][kFirst];
            T pf[kTogether][kFirst];
#pragma unroll
            for (int j = 0; j < kTogether; j++) {
                const int32_t i = i0 + j * kWaves;
                b0[j] = b1[j] = 0;
                if (i < nb) { b0[j] = range[2 * i]; b1[j] = range[2 * i + 1]; }
                const int32_t slots = b1[j] - b0[j];  // 0 for a block that does not exist
#pragma unroll
                for (int u = 0; u < kFirst; u++) {
                    rf[j][u] = 0;
                    pf[j][u] = T(0);
                    if (slots > 64 * u && slots <= 64 * kFirst) {  // wave-uniform; clamped: always a slot of this block
                        const int32_t idx = min(b0[j] + lane + 64 * u, b1[j] - 1);
                        rf[j][u] = L.row_local[idx];
                        pf[j][u] = partial[idx];
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < kTogether; j++) {
                const int32_t s0 = b0[j], s1 = b1[j], slots = s1 - s0;
                if (slots <= 64 * kFirst) {  // wave-uniform
                    if (slots <= 0) continue;
                    // the slots of a step are distinct rows of one block: read all, then write all
                    T o[kFirst];
#pragma unroll
                    for (int u = 0; u < kFirst; u++) o[u] = ys[rf[j][u]];
#pragma unroll
                    for (int u = 0; u < kFirst; u++)
                        if (s0 + lane + 64 * u < s1) ys[rf[j][u]] = o[u] + pf[j][u];
                    continue;
                }
                auto add_block = [&](auto ku) __attribute__((always_inline)) {
                    constexpr int KU = decltype(ku)::value;
                    for (int32_t s = s0 + lane; s < s1; s += 64 * KU) {
                        uint32_t r[KU];
                        T p[KU], o[KU];
#pragma unroll
                        for (int u = 0; u < KU; u++) {
                            const int32_t idx = min(s + 64 * u, s1 - 1);  // clamped: always a slot of this block
                            r[u] = L.row_local[idx];
                            p[u] = partial[idx];
                        }
#pragma unroll
                        for (int u = 0; u < KU; u++) o[u] = ys[r[u]];
#pragma unroll
                        for (int u = 0; u < KU; u++)
                            if (s + 64 * u < s1) ys[r[u]] = o[u] + p[u];
                    }
                };
                add_block(std::integral_constant<int, 4>{});
            }
        }
    }
    __syncthreads();
    for (int32_t i = threadIdx.x; i < rows; i += THREADS) {
        T sum = ys_all[i];
#pragma unroll
        for (int w = 1; w < kWaves; w++) sum += ys_all[w * L.R + i];
        if (split) atomicAdd(&y[r0 + i], sum);
        else y[r0 + i] = sum;
    }
}

// ------------------------------------------------------------------ CSR baselines (Algorithm 1)

template <typename T>
__global__ __launch_bounds__(256) void k_csr_scalar(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                    const T *__restrict__ val, const T *__restrict__ x,
                                                    T *__restrict__ y, int64_t n_rows)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_rows) return;
    T sum = T(0);
    for (int32_t j = ptr[i]; j < ptr[i + 1]; j++) sum += val[j] * x[col[j]];
    y[i] = sum;
}

// LPR lanes per row (a power of two below 64): the mapping between one thread and one wavefront per
// row, for matrices whose rows hold a few to a few dozen nonzeros.
template <int LPR, typename T>
__global__ __launch_bounds__(256) void k_csr_sub(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                 const T *__restrict__ val, const T *__restrict__ x,
                                                 T *__restrict__ y, int64_t n_rows)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t i = t / LPR;
    const int sub = (int)(t % LPR);
    T sum = T(0);
    if (i < n_rows)
        for (int32_t j = ptr[i] + sub; j < ptr[i + 1]; j += LPR) sum += val[j] * x[col[j]];
#pragma unroll
    for (int d = LPR / 2; d > 0; d >>= 1) sum += __shfl_xor(sum, d);  // stays inside the row's LPR lanes
    if (i < n_rows && sub == 0) y[i] = sum;
}

template <typename T>
__global__ __launch_bounds__(256) void k_csr_vector(const int32_t *__restrict__ ptr, const int32_t *__restrict__ col,
                                                    const T *__restrict__ val, const T *__restrict__ x,
                                                    T *__restrict__ y, int64_t n_rows)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n_rows) return;
    T sum = T(0);
    for (int32_t j = ptr[i] + lane; j < ptr[i + 1]; j += 64) sum += val[j] * x[col[j]];
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d);
    if (lane == 0) y[i] = sum;
}

}  // namespace

// Raises a kernel's dynamic-LDS cap on `device` (the attribute is per device).  `done` has a bit
// per device and is only a fast path: the call is idempotent, so two threads that both find the
// bit clear may both make it.
template <typename K>
static int raise_lds_cap(std::atomic<uint64_t> &done, int device, K kernel, int bytes)
{
    const uint64_t bit = device >= 0 && device < 64 ? uint64_t(1) << device : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return HBP_OK;
    HBP_HIP(hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    if (bit) done.fetch_or(bit, std::memory_order_release);
    return HBP_OK;
}

template <int THREADS, int U, int GP, bool HEAVY, typename T>
static int launch_part(const hbp_handle_s *h, const Layout &L, const T *x, T *y, hipStream_t st, SpmvScratch sc)
{
    const size_t lds = (size_t)h->C * sizeof(T);
    static std::atomic<uint64_t> configured{0};  // per instantiation
    const int rc = raise_lds_cap(configured, h->device, k_spmv_part<THREADS, U, GP, HEAVY, T>,
                                 kMaxC * (int)sizeof(float));  // 128 KB: kMaxC floats or kMaxC64 doubles
    if (rc != HBP_OK) return rc;
    k_spmv_part<THREADS, U, GP, HEAVY, T><<<dim3((unsigned)h->P), THREADS, lds, st>>>(L, x, static_cast<T *>(sc.partial), y, sc.ticket);
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

template <int THREADS, bool HEAVY, typename T>
static int launch_part_u(const hbp_handle_s *h, const Layout &L, const T *x, T *y, hipStream_t st, SpmvScratch sc)
{
    // fp64 at 1024 threads (128 registers per lane): half as many groups at once, or the batches spill
    constexpr int kHalf = sizeof(T) == 8 && THREADS == 1024 ? 2 : 1;
    switch (h->unroll) {  // rounds per batch; short batches walk several groups at once
    case 2: return launch_part<THREADS, 2, 8 / kHalf, HEAVY, T>(h, L, x, y, st, sc);
    case 4: return launch_part<THREADS, 4, 4 / kHalf, HEAVY, T>(h, L, x, y, st, sc);
    case 9: return launch_part<THREADS, 9, 1, HEAVY, T>(h, L, x, y, st, sc);
    case 16: return launch_part<THREADS, 16, 1, HEAVY, T>(h, L, x, y, st, sc);
    default: return launch_part<THREADS, 8, 1, HEAVY, T>(h, L, x, y, st, sc);
    }
}

template <typename T>
static int launch_part_t(const hbp_handle_s *h, const T *x, T *y, hipStream_t st, SpmvScratch sc)
{
    const Layout L = hbp_view(h);
    // the kernel that can share heavy groups among a worker's wavefronts only where the matrix has one
    if (h->longest_segment > long_rounds_of(h->heavy_rounds)) {
        if (h->threads == 1024) return launch_part_u<1024, true, T>(h, L, x, y, st, sc);
        if (h->threads == 512) return launch_part_u<512, true, T>(h, L, x, y, st, sc);
        return launch_part_u<256, true, T>(h, L, x, y, st, sc);
    }
    if (h->threads == 1024) return launch_part_u<1024, false, T>(h, L, x, y, st, sc);
    if (h->threads == 512) return launch_part_u<512, false, T>(h, L, x, y, st, sc);
    return launch_part_u<256, false, T>(h, L, x, y, st, sc);
}

template <typename T>
static int launch_combine_t(const hbp_handle_s *h, T *y, hipStream_t st, SpmvScratch sc)
{
    const Layout L = hbp_view(h);
    const T *partial = static_cast<const T *>(sc.partial);
    if (h->R <= 1024) {
        // two copies of a short slice: enough workgroups per CU for the plain block-by-block walk
        k_combine<128, T, 0, 0><<<dim3((unsigned)h->U), 128, 2 * (size_t)h->R * sizeof(T), st>>>(L, partial, y, sc.ticket);
    } else {
        // four copies (up to 128 KB: kMaxR floats or kMaxR64 doubles); a ring of chunks in flight,
        // shorter chunks and more of them where the blocks hold few slots on average
        auto go = [&](auto kr, auto kc, std::atomic<uint64_t> &configured) {
            constexpr int KR = decltype(kr)::value, KC = decltype(kc)::value;
            const int rc = raise_lds_cap(configured, h->device, k_combine<256, T, KR, KC>, 4 * kMaxR * (int)sizeof(float));
            if (rc != HBP_OK) return rc;
            k_combine<256, T, KR, KC><<<dim3((unsigned)h->U), 256, 4 * (size_t)h->R * sizeof(T), st>>>(L, partial, y, sc.ticket);
            return (int)HBP_OK;
        };
        static std::atomic<uint64_t> configured_long{0}, configured_short{0};
        const int rc = h->S < 128 * h->B ? go(std::integral_constant<int, 8>{}, std::integral_constant<int, 2>{}, configured_short)
                                         : go(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{}, configured_long);
        if (rc != HBP_OK) return rc;
    }
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

template <typename T>
static int launch_csr_t(int kind, const int32_t *ptr, const int32_t *col, const T *val, const T *x, T *y, int64_t n_rows,
                        hipStream_t st)
{
    auto sub = [&](auto lanes) {
        constexpr int LPR = decltype(lanes)::value;
        k_csr_sub<LPR, T><<<dim3((unsigned)((n_rows * LPR + 255) / 256)), 256, 0, st>>>(ptr, col, val, x, y, n_rows);
    };
    switch (kind) {
    case 0: k_csr_scalar<T><<<dim3((unsigned)((n_rows + 255) / 256)), 256, 0, st>>>(ptr, col, val, x, y, n_rows); break;
    case 1: k_csr_vector<T><<<dim3((unsigned)((n_rows + 3) / 4)), 256, 0, st>>>(ptr, col, val, x, y, n_rows); break;
    case 2: sub(std::integral_constant<int, 2>{}); break;
    case 4: sub(std::integral_constant<int, 4>{}); break;
    case 8: sub(std::integral_constant<int, 8>{}); break;
    case 16: sub(std::integral_constant<int, 16>{}); break;
    case 32: sub(std::integral_constant<int, 32>{}); break;
    default: return HBP_ERR_INVALID_ARGUMENT;
    }
    HBP_HIP(hipGetLastError());
    return HBP_OK;
}

}  // namespace hbp
