// Shared host/device helpers of the DropIT gfx950 library (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "dropit.h"

namespace dropit {

constexpr int WAVE = 64;

// true iff p is aligned to `a` bytes (a power of two)
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Product of a host shape; returns -1 if any extent is < 1, ndim < 1, or the
// product exceeds 2^31 - 1 (int32 flat indices).
inline int64_t checked_numel(const int64_t *shape, int ndim)
{
    if (shape == nullptr || ndim < 1) return -1;
    int64_t n = 1;
    for (int i = 0; i < ndim; ++i) {
        if (shape[i] < 1) return -1;
        if (n > INT32_MAX / shape[i]) return -1;
        n *= shape[i];
    }
    return n;
}

// Runs `setup` (returns true on success) once for every device this process uses, on the device that
// is current: kernel attributes and occupancy answers belong to a device, not to the process.  Two
// threads may both run it the first time, which is harmless for idempotent set-up.  Devices beyond
// the 64th run it on every call.
template <typename F> inline bool once_per_device(std::atomic<uint64_t> &done, F &&setup)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && (done.load(std::memory_order_acquire) >> dev & 1)) return true;
    if (!setup()) return false;
    if (tracked) done.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    return true;
}

inline dropit_status launch_status()
{
    return hipGetLastError() == hipSuccess ? DROPIT_OK : DROPIT_EHIP;
}

// ---- optional per-kernel timing marks (see dropit_trace_events) ---------
struct TraceState {
    hipEvent_t *events;
    int count, next;
};
TraceState &trace_state();                       // per host thread; defined in compress.hip
inline void trace_mark(hipStream_t stream)
{
    TraceState &t = trace_state();
    if (t.next < t.count) (void)hipEventRecord(t.events[t.next++], stream);
}

// how dropit_compress runs its select: 0 persistent kernel, 1 separate kernels, 2 cooperative launch,
// 3 forced serial redo (see dropit_set_select_mode)
int &select_mode();                              // per host thread; defined in compress.hip

// ---- wave / block primitives (64-wide wavefronts) -----------------------
// The 32-bit scans and sums run on the VALU's data-parallel primitives (row shifts inside
// 16-lane rows, then the two row broadcasts), not on LDS-routed shuffles: a kernel with 16
// wavefronts per compute unit that scans in a loop is otherwise bound by LDS instruction issue.

// inclusive prefix sum across the 64 lanes of a wavefront
__device__ inline uint32_t wave_inclusive_scan(uint32_t v)
{
    // lanes whose source lies outside the row (or whose row is masked off) add the `old` operand, 0
#define DROPIT_DPP_ADD(ctrl, row_mask) \
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), ctrl, row_mask, 0xf, false))
    DROPIT_DPP_ADD(0x111, 0xf);   // row_shr:1
    DROPIT_DPP_ADD(0x112, 0xf);   // row_shr:2
    DROPIT_DPP_ADD(0x114, 0xf);   // row_shr:4
    DROPIT_DPP_ADD(0x118, 0xf);   // row_shr:8   -> inclusive inside each row of 16
    DROPIT_DPP_ADD(0x142, 0xa);   // row_bcast:15 into rows 1 and 3
    DROPIT_DPP_ADD(0x143, 0xc);   // row_bcast:31 into rows 2 and 3
#undef DROPIT_DPP_ADD
    return v;
}

// sum over the 64 lanes, in every lane
__device__ inline uint32_t wave_sum(uint32_t v)
{
    return uint32_t(__builtin_amdgcn_readlane(int(wave_inclusive_scan(v)), WAVE - 1));
}

// generic (slow) form for other types
template <typename T>
__device__ inline T wave_inclusive_scan(T v)
{
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        T up = __shfl_up(v, o, WAVE);
        if (lane >= o) v += up;
    }
    return v;
}

// Exclusive prefix sum over a block of THREADS threads (THREADS % 64 == 0, at most 64 wavefronts).
// `wave_tot` is LDS scratch of THREADS/64 entries.  Returns the exclusive
// prefix of `v`; `total` receives the block sum.  Contains two barriers, so
// every thread of the block must call it.
template <int THREADS>
__device__ inline uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot, uint32_t &total)
{
    constexpr int NW = THREADS / WAVE;
    static_assert(NW <= WAVE, "the wavefront totals are scanned by one wavefront's lanes");
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const uint32_t inc = wave_inclusive_scan(v);
    __syncthreads();                      // protects wave_tot reuse across calls
    if (lane == WAVE - 1) wave_tot[w] = inc;
    __syncthreads();
    // every wavefront scans the totals itself: lane j holds wavefront j's
    const uint32_t t = lane < NW ? wave_tot[lane] : 0u;
    const uint32_t tinc = wave_inclusive_scan(t);
    total = uint32_t(__builtin_amdgcn_readlane(int(tinc), WAVE - 1));
    const uint32_t before = uint32_t(__builtin_amdgcn_readlane(int(tinc), w)) - uint32_t(__builtin_amdgcn_readlane(int(t), w));
    return before + inc - v;
}

// Two independent exclusive block scans sharing their barriers (a[2], b[2] of wave_tot2 rows).
template <int THREADS>
__device__ inline void block_exclusive_scan2(uint32_t va, uint32_t vb, uint32_t *wave_tot2 /*[2][THREADS/64]*/,
                                             uint32_t &ea, uint32_t &eb, uint32_t &ta, uint32_t &tb)
{
    constexpr int NW = THREADS / WAVE;
    static_assert(NW <= WAVE, "the wavefront totals are scanned by one wavefront's lanes");
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const uint32_t ia = wave_inclusive_scan(va), ib = wave_inclusive_scan(vb);
    __syncthreads();
    if (lane == WAVE - 1) {
        wave_tot2[w] = ia;
        wave_tot2[NW + w] = ib;
    }
    __syncthreads();
    const uint32_t xa = lane < NW ? wave_tot2[lane] : 0u, xb = lane < NW ? wave_tot2[NW + lane] : 0u;
    const uint32_t sa = wave_inclusive_scan(xa), sb = wave_inclusive_scan(xb);
    ta = uint32_t(__builtin_amdgcn_readlane(int(sa), WAVE - 1));
    tb = uint32_t(__builtin_amdgcn_readlane(int(sb), WAVE - 1));
    ea = uint32_t(__builtin_amdgcn_readlane(int(sa), w)) - uint32_t(__builtin_amdgcn_readlane(int(xa), w)) + ia - va;
    eb = uint32_t(__builtin_amdgcn_readlane(int(sb), w)) - uint32_t(__builtin_amdgcn_readlane(int(xb), w)) + ib - vb;
}

// ---------------------------------------------------------------------------
// Cooperative lower_bound over a sorted int32 array for two targets at once
// (number of elements < t0 and < t1): THREADS-ary search, both targets share the
// rounds: 3 rounds of one load each over a million elements, 2 over a range of a few thousand.
// All threads of the block must call it (contains barriers).
// The search starts from the ranges [from0, to0) and [from1, to1), which must contain the respective
// answers; the whole array is [0, n) for both.
template <int THREADS>
__device__ inline void block_lower_bound2(const int32_t *__restrict__ idx, int64_t t0, int64_t t1, int64_t from0,
                                          int64_t to0, int64_t from1, int64_t to1, int64_t &r0, int64_t &r1)
{
    int64_t lo[2] = {from0, from1}, hi[2] = {to0, to1};
    const int64_t target[2] = {t0, t1};
    while (hi[0] > lo[0] || hi[1] > lo[1]) {
        int pred[2];
        int64_t step[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int64_t span = hi[q] - lo[q];
            step[q] = (span + THREADS - 1) / THREADS;
            const int64_t pos = lo[q] + int64_t(threadIdx.x) * step[q];
            pred[q] = (pos < hi[q]) && (int64_t(idx[pos]) < target[q]);
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int c = __syncthreads_count(pred[q]);   // probes are monotone: the first c are true
            if (hi[q] > lo[q]) {
                if (c == 0) {
                    hi[q] = lo[q];
                } else {
                    const int64_t nlo = lo[q] + int64_t(c - 1) * step[q] + 1;
                    const int64_t nhi = min(lo[q] + int64_t(c) * step[q], hi[q]);
                    lo[q] = nlo;
                    hi[q] = nhi;
                }
            }
        }
    }
    r0 = lo[0];
    r1 = lo[1];
}

// ---------------------------------------------------------------------------
// Calls place(flat, value) for the pairs of the index-sorted arrays whose flat index lies in
// [first, last), and possibly for some neighbours outside it (place must ignore those).
// Where the pairs of a flat-index range start is first guessed, not searched: min-k keeps a fixed
// fraction of the tensor, so the pair with flat index f sits near position f * k / numel, and if the
// kept elements are spread evenly the guess is off by a few sqrt(k) at most.  The workgroup loads a
// window of pairs around the guesses for both ends (margin `margin` on either side) in ONE round of
// loads, values included, checks with the loaded indices themselves that the window covers the
// range, and hands over what it loaded.  Only if the window does not cover it (density that varies
// along the tensor) or would not fit WN entries per thread does it fall back to the exact search,
// three dependent rounds of loads, and a further round for the pairs.
// between() runs after the window's loads are issued and before any place(): the place for the
// caller's LDS zero fill (a barrier follows it).  All threads of the block must call this.
template <int THREADS, int WN, typename Place, typename Between>
__device__ inline void for_pairs_in_range(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx,
                                          int64_t k, int64_t numel, int64_t first, int64_t last, int64_t margin,
                                          Place &&place, Between &&between)
{
    const int tid = threadIdx.x;
    const int64_t g_lo = static_cast<int64_t>(static_cast<double>(first) * static_cast<double>(k) / static_cast<double>(numel));
    const int64_t g_hi = static_cast<int64_t>(static_cast<double>(last) * static_cast<double>(k) / static_cast<double>(numel));
    const int64_t w_lo = max<int64_t>(g_lo - margin, 0), w_hi = min<int64_t>(g_hi + margin, k);
    const bool window_fits = w_hi - w_lo <= int64_t(WN) * THREADS;
    int32_t wi[WN];
    uint32_t wv[WN];        // a full register each: 16-bit destinations get packed in pairs, and the second load
                            // of a pair then waits for the first
    if (window_fits) {
#pragma unroll
        for (int u = 0; u < WN; ++u) {
            const int64_t j = w_lo + int64_t(u) * THREADS + tid;
            if (j < w_hi) {
                wi[u] = idx[j];
                wv[u] = vals[j];
            }
        }
    }
    between();
    // the window covers the range iff nothing of it can lie before its first or after its last entry
    bool uncovered = !window_fits;
    if (window_fits && tid == 0) {
        if (w_lo > 0 && w_lo < w_hi && int64_t(wi[0]) >= first) uncovered = true;
        if (w_lo > 0 && w_lo >= w_hi) uncovered = first < last;       // empty window in the middle of the array
    }
    if (window_fits && w_hi < k) {
        const int64_t j_last = w_hi - 1;                              // held by thread (j_last - w_lo) % THREADS, slot / THREADS
        if (j_last >= w_lo && (j_last - w_lo) % THREADS == tid) {
            bool short_of_end = false;
#pragma unroll
            for (int u = 0; u < WN; ++u)
                if ((j_last - w_lo) / THREADS == u) short_of_end = int64_t(wi[u]) < last;
            uncovered = uncovered || short_of_end;
        }
    }
    if (__syncthreads_or(uncovered)) {                                // also orders between() before the first place()
        int64_t lo, hi;
        block_lower_bound2<THREADS>(idx, first, last, 0, k, 0, k, lo, hi);
        // eight pairs per thread at a time: their loads are all in flight before the first place()
        constexpr int BATCH = 8;
        for (int64_t j0 = lo + tid; j0 < hi; j0 += int64_t(BATCH) * THREADS) {
            int32_t pi[BATCH];
            uint32_t pv[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int64_t j = j0 + int64_t(u) * THREADS;
                if (j < hi) {
                    pi[u] = idx[j];
                    pv[u] = vals[j];
                }
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u)
                if (j0 + int64_t(u) * THREADS < hi) place(pi[u], pv[u]);
        }
    } else {
#pragma unroll
        for (int u = 0; u < WN; ++u)
            if (w_lo + int64_t(u) * THREADS + tid < w_hi) place(wi[u], wv[u]);
    }
}

}  // namespace dropit
