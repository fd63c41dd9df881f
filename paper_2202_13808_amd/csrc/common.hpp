// Shared host/device helpers of the DropIT gfx950 library (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

__device__ inline uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// inclusive prefix sum across the 64 lanes of a wavefront
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

// Exclusive prefix sum over a block of THREADS threads (THREADS % 64 == 0).
// `wave_tot` is LDS scratch of THREADS/64 entries.  Returns the exclusive
// prefix of `v`; `total` receives the block sum.  Contains two barriers, so
// every thread of the block must call it.
template <int THREADS, typename T>
__device__ inline T block_exclusive_scan(T v, T *wave_tot, T &total)
{
    constexpr int NW = THREADS / WAVE;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = threadIdx.x / WAVE;
    T inc = wave_inclusive_scan(v);
    __syncthreads();                      // protects wave_tot reuse across calls
    if (lane == WAVE - 1) wave_tot[w] = inc;
    __syncthreads();
    T before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        T t = wave_tot[i];
        if (i < w) before += t;
        all += t;
    }
    total = all;
    return before + inc - v;
}

}  // namespace dropit
